"""Host-side checks of the C ABI that need no GPU: the library loads, exports every
symbol the header declares, and rejects bad scalars/pointers before touching HIP."""
import ctypes
import os
import re

import pytest

import paper_2405_07542_amd as ems

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADERS = [os.path.join(ROOT, "include", "ems.h"), os.path.join(ROOT, "include", "ems_measure.h")]


def declared_symbols():
    text = "".join(open(h).read() for h in HEADERS)
    return re.findall(r"EMS_API\s+[\w\s\*]+?\b(ems_\w+)\s*\(", text)


def test_library_exports_every_declared_symbol():
    names = declared_symbols()
    assert {"ems_verify_attention", "ems_greedy_accept", "ems_kv_append", "ems_workspace_bytes",
            "ems_profile_enable", "ems_stream_read_probe", "ems_set_attention_variant"} <= set(names)
    L = ems.lib()
    for n in names:
        assert hasattr(L, n), "libems.so does not export %s" % n
    assert re.match(rb"\d+\.\d+$", L.ems_version())


def test_workspace_sizes_are_host_arithmetic():
    for args in ((64, 384, 32, 128, 2048), (1, 1, 1, 64, 0), (128, 448, 32, 128, 4096), (0, 0, 0, 0, 0)):
        assert ems.ems_workspace_bytes(*args) == ems.ems_attention_workspace_bytes(*args)
    assert ems.ems_attention_workspace_bytes(64, 384, 32, 128, 2048) >= 256
    assert ems.ems_attention_workspace_bytes(1, 1, 1, 64, 0) >= 256
    assert ems.ems_attention_workspace_bytes(128, 448, 32, 128, 4096) <= 160 << 20
    assert ems.ems_accept_workspace_bytes(0, 50272) == 0
    assert ems.ems_accept_workspace_bytes(384, 0) == 0
    assert ems.ems_accept_workspace_bytes(384, 50272) >= 384 * 8


FAKE = 0x1000          # a 16-byte aligned non-NULL address that is never dereferenced on the host


def attention(**over):
    a = dict(q=FAKE, k_new=FAKE, v_new=FAKE, cache=ems.KvCacheStruct(FAKE, FAKE, 4096, 128, 1024),
             cu=FAKE, ks=FAKE, kl=FAKE, out=FAKE, out_dtype=ems.EMS_F16, B=4, T=8, H=32, D=128,
             max_k=4, max_kv_len=100, scale=0.1, dtype=ems.EMS_F16, ws=FAKE, ws_bytes=1 << 30)
    a.update(over)
    cache = a["cache"]
    return ems.lib().ems_verify_attention(
        a["q"], a["k_new"], a["v_new"], ctypes.byref(cache) if cache is not None else None,
        a["cu"], a["ks"], a["kl"], a["out"], a["out_dtype"], a["B"], a["T"], a["H"], a["D"],
        a["max_k"], a["max_kv_len"], a["scale"], a["dtype"], a["ws"], a["ws_bytes"], None)


@pytest.mark.parametrize("over,status,text", [
    (dict(B=0), ems.EMS_ERR_INVALID_ARG, "B"),
    (dict(T=-1), ems.EMS_ERR_INVALID_ARG, "T"),
    (dict(H=0), ems.EMS_ERR_INVALID_ARG, "H"),
    (dict(max_k=-1), ems.EMS_ERR_INVALID_ARG, "max_k"),
    (dict(scale=float("nan")), ems.EMS_ERR_INVALID_ARG, "scale"),
    (dict(dtype=ems.EMS_F32), ems.EMS_ERR_INVALID_ARG, "dtype"),
    (dict(out_dtype=ems.EMS_BF16), ems.EMS_ERR_INVALID_ARG, "out_dtype"),
    (dict(cu=None), ems.EMS_ERR_INVALID_ARG, "cu_seqlens"),
    (dict(q=None), ems.EMS_ERR_INVALID_ARG, "NULL"),
    (dict(out=FAKE + 2), ems.EMS_ERR_INVALID_ARG, "aligned"),
    (dict(cache=None), ems.EMS_ERR_INVALID_ARG, "cache"),
    (dict(cache=ems.KvCacheStruct(FAKE, FAKE, 4100, 128, 1024)), ems.EMS_ERR_INVALID_ARG, "strides"),
    (dict(D=96), ems.EMS_ERR_UNSUPPORTED, "head dim"),
    (dict(max_k=65), ems.EMS_ERR_UNSUPPORTED, "rows per sample"),
    (dict(B=10000), ems.EMS_ERR_UNSUPPORTED, "samples"),
    (dict(max_kv_len=1 << 20), ems.EMS_ERR_UNSUPPORTED, "4 GiB"),
    (dict(ws=None), ems.EMS_ERR_WORKSPACE, "workspace"),
    (dict(ws_bytes=16), ems.EMS_ERR_WORKSPACE, "workspace"),
])
def test_attention_rejects_bad_arguments_on_the_host(over, status, text):
    assert attention(**over) == status
    assert text in ems.lib().ems_last_error_string().decode()


def test_attention_with_no_rows_is_a_noop_without_a_gpu():
    assert attention(T=0, q=None, k_new=None, v_new=None, out=None, ws=None, ws_bytes=0) == ems.EMS_OK


def accept(**over):
    a = dict(logits=None, dtype=ems.EMS_F16, V=0, tgt=FAKE, ids=FAKE, cu=FAKE, B=4, T=8,
             acc=FAKE, acc_cu=FAKE, toks=None, ws=None, ws_bytes=0)
    a.update(over)
    return ems.lib().ems_greedy_accept(a["logits"], a["dtype"], a["V"], a["tgt"], a["ids"], a["cu"],
                                       a["B"], a["T"], a["acc"], a["acc_cu"], a["toks"], a["ws"],
                                       a["ws_bytes"], None)


@pytest.mark.parametrize("over,status", [
    (dict(B=0), ems.EMS_ERR_INVALID_ARG),
    (dict(T=-3), ems.EMS_ERR_INVALID_ARG),
    (dict(V=-1), ems.EMS_ERR_INVALID_ARG),
    (dict(acc=None), ems.EMS_ERR_INVALID_ARG),
    (dict(tgt=None), ems.EMS_ERR_INVALID_ARG),
    (dict(B=9000), ems.EMS_ERR_UNSUPPORTED),
    (dict(T=70000), ems.EMS_ERR_UNSUPPORTED),
    (dict(logits=FAKE, V=0), ems.EMS_ERR_INVALID_ARG),
    (dict(logits=FAKE, V=50272, dtype=7), ems.EMS_ERR_INVALID_ARG),
    (dict(logits=FAKE + 4, V=50272), ems.EMS_ERR_INVALID_ARG),
    (dict(logits=FAKE, V=50272, ws=None), ems.EMS_ERR_WORKSPACE),
    (dict(logits=FAKE, V=50272, ws=FAKE, ws_bytes=8), ems.EMS_ERR_WORKSPACE),
])
def test_accept_rejects_bad_arguments_on_the_host(over, status):
    assert accept(**over) == status
    assert ems.lib().ems_last_error_string()


def append(**over):
    a = dict(n=2, B=4, T=8, H=32, D=128, dtype=ems.EMS_BF16, cu=FAKE, acc=FAKE, ks=FAKE, kl=FAKE,
             out=None, knew=[FAKE, FAKE], vnew=[FAKE, FAKE],
             caches=[ems.KvCacheStruct(FAKE, FAKE, 4096, 128, 64)] * 2)
    a.update(over)
    n = len(a["knew"])
    karr = (ctypes.c_void_p * n)(*a["knew"])
    varr = (ctypes.c_void_p * n)(*a["vnew"])
    carr = (ems.KvCacheStruct * n)(*a["caches"])
    return ems.lib().ems_kv_append(karr, varr, carr, a["n"], a["cu"], a["acc"], a["ks"], a["kl"],
                                   a["out"], a["B"], a["T"], a["H"], a["D"], a["dtype"], None)


@pytest.mark.parametrize("over", [
    dict(n=0), dict(B=0), dict(T=-1), dict(H=0), dict(D=12), dict(D=0), dict(dtype=ems.EMS_F32),
    dict(acc=None), dict(knew=[FAKE, None]), dict(vnew=[FAKE + 8, FAKE]),
    dict(caches=[ems.KvCacheStruct(FAKE, FAKE, 4096, 128, 64), ems.KvCacheStruct(FAKE, FAKE, 64, 128, 64)]),
])
def test_append_rejects_bad_arguments_on_the_host(over):
    assert append(**over) == ems.EMS_ERR_INVALID_ARG
    assert ems.lib().ems_last_error_string()


def test_validate_inputs_rejects_bad_scalars_on_the_host():
    L = ems.lib()
    assert L.ems_validate_inputs(FAKE, FAKE, FAKE, 0, 0, 1, 1, 10, None) == ems.EMS_ERR_INVALID_ARG
    assert L.ems_validate_inputs(None, FAKE, FAKE, 1, 0, 1, 1, 10, None) == ems.EMS_ERR_INVALID_ARG


def test_write_through_and_advance_reject_bad_arguments_on_the_host():
    L = ems.lib()
    assert L.ems_kv_advance(FAKE, FAKE, FAKE, 0, None) == ems.EMS_ERR_INVALID_ARG
    assert L.ems_kv_advance(None, FAKE, FAKE, 4, None) == ems.EMS_ERR_INVALID_ARG
    cache = ems.KvCacheStruct(FAKE, FAKE, 4096, 128, 1024)
    args = [FAKE, FAKE, FAKE, ctypes.byref(cache), FAKE, FAKE, FAKE, FAKE, ems.EMS_F16, 4, 8, 32, 96, 4,
            100, 0.1, ems.EMS_F16, FAKE, 1 << 30, None]
    assert L.ems_verify_attention_write_through(*args) == ems.EMS_ERR_UNSUPPORTED     # D = 96
    args[12] = 128
    args[9] = 0
    assert L.ems_verify_attention_write_through(*args) == ems.EMS_ERR_INVALID_ARG     # B = 0


def test_attention_variant_switch_is_per_thread_host_state():
    import threading
    L = ems.lib()
    seen = {}

    def other_thread():
        seen["before"] = L.ems_get_attention_variant()
        L.ems_set_attention_variant(ems.EMS_ATTN_VALU)
        seen["after"] = L.ems_get_attention_variant()
    t = threading.Thread(target=other_thread)
    t.start()
    t.join()
    assert seen == {"before": ems.EMS_ATTN_MFMA, "after": ems.EMS_ATTN_VALU}
    assert L.ems_get_attention_variant() == ems.EMS_ATTN_MFMA       # this thread's calls are unaffected
    assert L.ems_get_attention_variant() == ems.EMS_ATTN_MFMA
    assert L.ems_set_attention_variant(ems.EMS_ATTN_VALU) == ems.EMS_OK
    assert L.ems_get_attention_variant() == ems.EMS_ATTN_VALU
    assert L.ems_set_attention_variant(5) == ems.EMS_ERR_INVALID_ARG
    assert L.ems_get_attention_variant() == ems.EMS_ATTN_VALU
    assert L.ems_set_attention_variant(ems.EMS_ATTN_MFMA) == ems.EMS_OK


def test_tree_entry_points_reject_bad_arguments_on_the_host():
    L = ems.lib()
    cache = ems.KvCacheStruct(FAKE, FAKE, 4096, 128, 1024)
    args = [FAKE, FAKE, FAKE, ctypes.byref(cache), FAKE, None, FAKE, FAKE, FAKE, ems.EMS_F16, 4, 8, 32, 128,
            4, 100, 0.1, ems.EMS_F16, FAKE, 1 << 30, None]
    assert L.ems_tree_verify_attention(*args) == ems.EMS_ERR_INVALID_ARG          # parent = NULL
    assert b"parent" in L.ems_last_error_string()
    args[5] = FAKE
    args[13] = 96
    assert L.ems_tree_verify_attention(*args) == ems.EMS_ERR_UNSUPPORTED          # D = 96
    args[13] = 128
    args[10] = 0
    assert L.ems_tree_verify_attention(*args) == ems.EMS_ERR_INVALID_ARG          # B = 0
    # accept: parent required with rows; sizes checked as in the plain call
    assert L.ems_tree_accept(None, ems.EMS_F16, 0, FAKE, FAKE, None, FAKE, 4, 8, FAKE, FAKE, None, None,
                             None, 0, None) == ems.EMS_ERR_INVALID_ARG
    assert L.ems_tree_accept(None, ems.EMS_F16, 0, FAKE, FAKE, FAKE, FAKE, 0, 8, FAKE, FAKE, None, None,
                             None, 0, None) == ems.EMS_ERR_INVALID_ARG
    # gathered append
    karr = (ctypes.c_void_p * 1)(FAKE)
    carr = (ems.KvCacheStruct * 1)(cache)
    assert L.ems_kv_append_rows(karr, karr, carr, 1, None, FAKE, FAKE, FAKE, None, 4, 8, 32, 128,
                                ems.EMS_F16, None) == ems.EMS_ERR_INVALID_ARG
    assert L.ems_kv_append_rows(karr, karr, carr, 0, FAKE, FAKE, FAKE, FAKE, None, 4, 8, 32, 128,
                                ems.EMS_F16, None) == ems.EMS_ERR_INVALID_ARG
    assert L.ems_stream_read_probe(None, 4096, FAKE, None) == ems.EMS_ERR_INVALID_ARG
    assert L.ems_stream_read_probe(FAKE, 100, FAKE, None) == ems.EMS_ERR_INVALID_ARG


def test_pack_tokens_rejects_bad_arguments_on_the_host():
    L = ems.lib()
    assert L.ems_pack_tokens(FAKE, FAKE, 0, 4, FAKE, FAKE, None) == ems.EMS_ERR_INVALID_ARG
    assert L.ems_pack_tokens(FAKE, FAKE, 9000, 4, FAKE, FAKE, None) == ems.EMS_ERR_UNSUPPORTED
    assert L.ems_pack_tokens(FAKE, FAKE, 4, -1, FAKE, FAKE, None) == ems.EMS_ERR_INVALID_ARG
    assert L.ems_pack_tokens(FAKE, None, 4, 4, FAKE, FAKE, None) == ems.EMS_ERR_INVALID_ARG
    assert L.ems_pack_tokens(None, FAKE, 4, 4, FAKE, FAKE, None) == ems.EMS_ERR_INVALID_ARG


def test_device_memory_figures_rejects_null_pointers():
    assert ems.lib().ems_device_memory_figures(None, None) == ems.EMS_ERR_INVALID_ARG


def test_the_header_is_plain_c_and_the_library_is_usable_from_c(tmp_path):
    """gcc -std=c11 -pedantic compiles a C program against include/ems.h; the program loads
    libems.so with dlopen and calls host-only paths of the ABI (no Python, no C++, no GPU)."""
    import subprocess
    exe = str(tmp_path / "abi_from_c")
    subprocess.check_call(["gcc", "-std=c11", "-Wall", "-Wextra", "-Werror", "-pedantic", "-D_GNU_SOURCE",
                           "-I", os.path.join(ROOT, "include"), "-o", exe,
                           os.path.join(ROOT, "tests", "c_abi", "abi_from_c.c"), "-ldl"])
    res = subprocess.run([exe, ems.LIB_PATH], capture_output=True, text=True, timeout=120)
    assert res.returncode == 0, (res.returncode, res.stdout, res.stderr)
    assert res.stdout.startswith("ok ")


def test_the_noalloc_buffer_is_a_global_symbol_of_the_device_image(tmp_path):
    """ems_verify_attention_noalloc finds its buffer by name (hipGetSymbolAddress); the runtime
    aborts the process if the device image holds that name only as a local symbol -- which is
    what happens when the static device array is not referred to by host code in a way the
    compiler sees, or carries a `used` attribute.  Compile the API's device side alone and look."""
    import subprocess
    hipcc = "/opt/rocm/bin/hipcc"
    readelf = "/opt/rocm/llvm/bin/llvm-readelf"
    if not (os.path.exists(hipcc) and os.path.exists(readelf)):
        pytest.skip("needs the ROCm compilers")
    obj = str(tmp_path / "api_device.o")
    subprocess.check_call([hipcc, "-O3", "-std=c++17", "--offload-arch=gfx950", "--cuda-device-only", "--no-gpu-bundle-output",
                           "-fPIC", "-fvisibility=hidden", "-c", os.path.join(ROOT, "paper_2405_07542_amd", "csrc", "ems_api.hip"),
                           "-o", obj], stderr=subprocess.DEVNULL)
    table = subprocess.run([readelf, "-s", obj], capture_output=True, text=True, check=True).stdout
    rows = [l.split() for l in table.splitlines() if l.strip().endswith("scratch")]
    assert rows, table
    assert all(r[3] == "OBJECT" and r[4] == "GLOBAL" and int(r[2]) == ems.EMS_NOALLOC_SCRATCH_BYTES for r in rows), rows
