/* A C99 client of the library's header: proves that include/fnn.h is plain C and that the
 * entry points can be reached without Python.  Host-only calls (sizes, status strings and
 * argument errors, which are detected before anything is enqueued), so it runs without a GPU.
 * usage: c_abi_check /path/to/libfnn.so */
#include <dlfcn.h>
#include <stdio.h>
#include <string.h>

#include "fnn.h"

#define CHECK(cond)                                              \
    do {                                                         \
        if (!(cond)) {                                           \
            printf("FAILED line %d: %s\n", __LINE__, #cond);     \
            return 1;                                            \
        }                                                        \
    } while (0)

typedef const char* (*status_string_fn)(int32_t);
typedef size_t (*workspace_bytes_fn)(int32_t, int64_t, int64_t, int32_t, int64_t, int32_t);
typedef size_t (*workspace_bytes_opts_fn)(int32_t, int64_t, int64_t, int32_t, int64_t, const fnn_opts*);
typedef int32_t (*nearest_fn)(int32_t, const fnn_map*, const int32_t*, int64_t, const int32_t*, const fnn_map*,
                              const fnn_opts*, int32_t*, float*, void*, size_t, void*);

int main(int argc, char** argv) {
    void* lib;
    status_string_fn status_string;
    workspace_bytes_fn workspace_bytes;
    workspace_bytes_opts_fn workspace_bytes_opts;
    nearest_fn nearest;
    fnn_opts opts;
    fnn_map map;
    size_t plain, wide;

    if (argc < 2) return 2;
    lib = dlopen(argv[1], RTLD_NOW | RTLD_LOCAL);
    if (!lib) {
        printf("dlopen: %s\n", dlerror());
        return 2;
    }
    *(void**)&status_string = dlsym(lib, "fnn_status_string");
    *(void**)&workspace_bytes = dlsym(lib, "fnn_workspace_bytes");
    *(void**)&workspace_bytes_opts = dlsym(lib, "fnn_workspace_bytes_opts");
    *(void**)&nearest = dlsym(lib, "fnn_nearest");
    CHECK(status_string && workspace_bytes && workspace_bytes_opts && nearest);

    CHECK(strcmp(status_string(FNN_OK), "ok") == 0);
    CHECK(strcmp(status_string(FNN_E_WORKSPACE), status_string(FNN_E_HIP)) != 0);

    plain = workspace_bytes(1, 196608, 196608, 24, 3072, FNN_F16);
    CHECK(plain >= (size_t)2 * 196608 * 24 * 2);      /* at least the two prepared maps */
    CHECK(workspace_bytes(0, 196608, 196608, 24, 3072, FNN_F16) == 0);
    CHECK(workspace_bytes(1, 196608, 196608, FNN_MAX_D + 1, 3072, FNN_F16) == 0);

    memset(&opts, 0, sizeof(opts));
    opts.compute = FNN_F16;
    CHECK(workspace_bytes_opts(1, 196608, 196608, 24, 3072, &opts) == plain);
    opts.flags = FNN_FLAG_SPLIT;
    wide = workspace_bytes_opts(1, 196608, 196608, 24, 3072, &opts);
    CHECK(wide > plain);
    opts.flags = FNN_FLAG_SPLIT | FNN_FLAG_L2;
    CHECK(workspace_bytes_opts(1, 196608, 196608, 24, 3072, &opts) == 0);

    /* argument errors come back as codes, before anything touches a device */
    memset(&map, 0, sizeof(map));
    map.data = (const void*)0x1000;
    map.n = 64;
    map.d = 24;
    map.dtype = FNN_F32;
    map.row_stride = 24;
    opts.flags = 0;
    CHECK(nearest(1, NULL, NULL, 64, NULL, &map, &opts, (int32_t*)0x2000, NULL, (void*)0x10000, plain, NULL) == FNN_E_NULL);
    CHECK(nearest(0, &map, NULL, 64, NULL, &map, &opts, (int32_t*)0x2000, NULL, (void*)0x10000, plain, NULL) == FNN_E_SHAPE);
    opts.compute = 9;
    CHECK(nearest(1, &map, NULL, 64, NULL, &map, &opts, (int32_t*)0x2000, NULL, (void*)0x10000, plain, NULL) == FNN_E_DTYPE);
    opts.compute = FNN_F16;
    opts.flags = 1 << 20;
    CHECK(nearest(1, &map, NULL, 64, NULL, &map, &opts, (int32_t*)0x2000, NULL, (void*)0x10000, plain, NULL) == FNN_E_RANGE);
    opts.flags = 0;
    CHECK(nearest(1, &map, NULL, 64, NULL, &map, &opts, (int32_t*)0x2000, NULL, NULL, 0, NULL) == FNN_E_WORKSPACE);
    CHECK(nearest(1, &map, NULL, 0, NULL, &map, &opts, NULL, NULL, NULL, 0, NULL) == FNN_OK); /* nothing to do */

    printf("c abi ok\n");
    dlclose(lib);
    return 0;
}
