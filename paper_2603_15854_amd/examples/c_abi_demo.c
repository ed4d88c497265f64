/*
 * The C ABI used from plain C (no Python, no C++): reads a problem from raw files, uploads it,
 * calls flash_sample() -- the plain entry point of include/flash_sample.h -- and writes the result.
 *
 *   c_abi_demo hidden.bin W.bin temperature.bin B D V seed out.bin
 *
 * hidden.bin: B*D bf16 values, W.bin: V*D bf16 values, temperature.bin: B fp32 values (host byte
 * order, row-major).  out.bin receives B int32 indices followed by B fp32 values.
 * Built by paper_2603_15854_amd/build.py next to the library; tests/test_gpu_zz_c_abi.py runs it.
 */
#include <hip/hip_runtime_api.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

#include "flash_sample.h"

static void* read_file(const char* path, size_t bytes)
{
    FILE* f = fopen(path, "rb");
    if (!f) { fprintf(stderr, "cannot open %s\n", path); exit(2); }
    void* buf = malloc(bytes);
    if (!buf || fread(buf, 1, bytes, f) != bytes) { fprintf(stderr, "short read on %s\n", path); exit(2); }
    fclose(f);
    return buf;
}

static void* upload(const void* host, size_t bytes)
{
    void* dev = NULL;
    if (hipMalloc(&dev, bytes) != hipSuccess || hipMemcpy(dev, host, bytes, hipMemcpyHostToDevice) != hipSuccess) {
        fprintf(stderr, "upload of %zu bytes failed\n", bytes);
        exit(3);
    }
    return dev;
}

int main(int argc, char** argv)
{
    if (argc != 9) {
        fprintf(stderr, "usage: %s hidden.bin W.bin temperature.bin B D V seed out.bin\n", argv[0]);
        return 1;
    }
    const int B = atoi(argv[4]), D = atoi(argv[5]), V = atoi(argv[6]);
    const uint64_t seed = strtoull(argv[7], NULL, 10);
    void* h = read_file(argv[1], (size_t)B * D * 2);
    void* w = read_file(argv[2], (size_t)V * D * 2);
    void* t = read_file(argv[3], (size_t)B * 4);
    void* dh = upload(h, (size_t)B * D * 2);
    void* dw = upload(w, (size_t)V * D * 2);
    void* dt = upload(t, (size_t)B * 4);
    int32_t* didx = NULL;
    float* dval = NULL;
    if (hipMalloc((void**)&didx, (size_t)B * 4) != hipSuccess || hipMalloc((void**)&dval, (size_t)B * 4) != hipSuccess) return 3;

    const fs_status st = flash_sample(dh, dw, B, D, V, (const float*)dt, seed, didx, dval);
    if (st != FS_OK) { fprintf(stderr, "flash_sample: %s\n", fs_status_string(st)); return 4; }
    if (hipDeviceSynchronize() != hipSuccess) return 5;

    int32_t* idx = (int32_t*)malloc((size_t)B * 4);
    float* val = (float*)malloc((size_t)B * 4);
    if (hipMemcpy(idx, didx, (size_t)B * 4, hipMemcpyDeviceToHost) != hipSuccess ||
        hipMemcpy(val, dval, (size_t)B * 4, hipMemcpyDeviceToHost) != hipSuccess) return 5;
    FILE* f = fopen(argv[8], "wb");
    if (!f) return 6;
    fwrite(idx, 4, (size_t)B, f);
    fwrite(val, 4, (size_t)B, f);
    fclose(f);
    printf("sampled %d rows; row 0 -> id %d (score %.6f)\n", B, idx[0], val[0]);
    return 0;
}
