/* The header is plain C and the library can be driven from C without Python or C++:
 * load libems.so, resolve a few entry points by the names the header declares, and call the
 * ones that need no GPU.  Exit code 0 = all as expected. */
#include <dlfcn.h>
#include <stdio.h>
#include <string.h>

#include "ems.h"

typedef const char* (*version_fn)(void);
typedef size_t (*ws_fn)(int, int, int, int, int);
typedef ems_status (*attn_fn)(const void*, const void*, const void*, const ems_kv_cache*, const int32_t*,
                              const int32_t*, const int32_t*, void*, ems_dtype, int, int, int, int, int, int,
                              float, ems_dtype, void*, size_t, void*);
typedef const char* (*err_fn)(void);

int main(int argc, char** argv) {
    if (argc < 2) return 2;
    void* lib = dlopen(argv[1], RTLD_NOW | RTLD_LOCAL);
    if (!lib) { fprintf(stderr, "dlopen: %s\n", dlerror()); return 3; }
    version_fn version;
    ws_fn ws_bytes;
    attn_fn attention;
    err_fn last_error;
    /* (the POSIX way to turn dlsym's object pointer into a function pointer) */
    *(void**)(&version) = dlsym(lib, "ems_version");
    *(void**)(&ws_bytes) = dlsym(lib, "ems_workspace_bytes");
    *(void**)(&attention) = dlsym(lib, "ems_verify_attention");
    *(void**)(&last_error) = dlsym(lib, "ems_last_error_string");
    if (!version || !ws_bytes || !attention || !last_error) return 4;
    if (strcmp(version(), "0.1") != 0) return 5;
    if (ws_bytes(64, 384, 32, 128, 2048) < 256) return 6;
    /* a call with no rows is a no-op that needs no device memory at all */
    ems_kv_cache cache = {(void*)0x1000, (void*)0x1000, 4096, 128, 1024};
    int32_t* fake = (int32_t*)0x1000;
    if (attention(NULL, NULL, NULL, &cache, fake, fake, fake, NULL, EMS_F16, 4, 0, 32, 128, 4, 100, 0.1f, EMS_F16,
                  NULL, 0, NULL) != EMS_OK) return 7;
    /* an unsupported head dim is refused on the host, with a message */
    if (attention(fake, fake, fake, &cache, fake, fake, fake, fake, EMS_F16, 4, 8, 32, 96, 4, 100, 0.1f, EMS_F16,
                  fake, (size_t)1 << 30, NULL) != EMS_ERR_UNSUPPORTED) return 8;
    if (strstr(last_error(), "head dim") == NULL) return 9;
    printf("ok %s\n", version());
    return 0;
}
