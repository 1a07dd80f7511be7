/*
 * A plain C client of libqsdp: no Python, no C++ runtime of its own. Reads a weight vector and
 * a gradient vector (raw little-endian float32 files of n values each), runs on GPU 0
 *   1. qsdp_quantize_grad (gbits) and qsdp_dequantize of the result to fp32,
 *   2. qsdp_fused_step (wbits, gbits) in place, with the packed codes of the new weights,
 * and writes <prefix>.gcodes, <prefix>.gmeta, <prefix>.ghat, <prefix>.x, <prefix>.wcodes,
 * <prefix>.wmeta as raw files. Exit status 0 on success.
 *
 *   qsdp_client x.f32 g.f32 n wbits gbits bucket lr seed prefix
 *
 * Build (see paper_2302_02390_amd/build.py, build_client):
 *   gcc -std=c11 -D__HIP_PLATFORM_AMD__ -Iinclude -I/opt/rocm/include examples/qsdp_client.c \
 *       -Lpaper_2302_02390_amd -lqsdp -L/opt/rocm/lib -lamdhip64 -o examples/qsdp_client
 */
#include <hip/hip_runtime_api.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "qsdp.h"

#define HIP_OK(call)                                                                   \
    do {                                                                               \
        hipError_t e_ = (call);                                                        \
        if (e_ != hipSuccess) {                                                        \
            fprintf(stderr, "%s: %s\n", #call, hipGetErrorString(e_));                 \
            return 2;                                                                  \
        }                                                                              \
    } while (0)

#define QSDP_DO(call)                                                                  \
    do {                                                                               \
        int s_ = (call);                                                               \
        if (s_ != QSDP_OK) {                                                           \
            fprintf(stderr, "%s: %s\n", #call, qsdp_status_string(s_));                \
            return 3;                                                                  \
        }                                                                              \
    } while (0)

static void* read_file(const char* path, size_t bytes) {
    void* buf = malloc(bytes);
    FILE* f = fopen(path, "rb");
    if (!buf || !f || fread(buf, 1, bytes, f) != bytes) {
        fprintf(stderr, "cannot read %zu bytes from %s\n", bytes, path);
        exit(1);
    }
    fclose(f);
    return buf;
}

static int dump(const char* prefix, const char* suffix, const void* dev, size_t bytes) {
    char path[4096];
    void* host = malloc(bytes);
    if (!host) return 1;
    HIP_OK(hipMemcpy(host, dev, bytes, hipMemcpyDeviceToHost));
    snprintf(path, sizeof path, "%s.%s", prefix, suffix);
    FILE* f = fopen(path, "wb");
    if (!f || fwrite(host, 1, bytes, f) != bytes) {
        fprintf(stderr, "cannot write %s\n", path);
        return 1;
    }
    fclose(f);
    free(host);
    return 0;
}

int main(int argc, char** argv) {
    if (argc != 10) {
        fprintf(stderr, "usage: %s x.f32 g.f32 n wbits gbits bucket lr seed prefix\n", argv[0]);
        return 1;
    }
    const uint64_t n = strtoull(argv[3], NULL, 10);
    const int wbits = atoi(argv[4]), gbits = atoi(argv[5]), bucket = atoi(argv[6]);
    const float lr = strtof(argv[7], NULL);
    const uint64_t seed = strtoull(argv[8], NULL, 10);
    const char* prefix = argv[9];

    const uint64_t gcb = qsdp_codes_bytes(n, gbits, bucket), wcb = qsdp_codes_bytes(n, wbits, bucket);
    const uint64_t mb = qsdp_meta_bytes(n, bucket);
    if (gcb == 0 || wcb == 0 || mb == 0) {
        fprintf(stderr, "invalid n / bits / bucket\n");
        return 1;
    }
    float* hx = read_file(argv[1], n * sizeof(float));
    float* hg = read_file(argv[2], n * sizeof(float));

    float *x, *g, *ghat, *gmeta, *wmeta;
    uint32_t *gcodes, *wcodes;
    uint64_t* nsat;
    hipStream_t stream;
    HIP_OK(hipSetDevice(0));
    HIP_OK(hipStreamCreate(&stream));
    HIP_OK(hipMalloc((void**)&x, n * sizeof(float)));
    HIP_OK(hipMalloc((void**)&g, n * sizeof(float)));
    HIP_OK(hipMalloc((void**)&ghat, n * sizeof(float)));
    HIP_OK(hipMalloc((void**)&gcodes, gcb));
    HIP_OK(hipMalloc((void**)&wcodes, wcb));
    HIP_OK(hipMalloc((void**)&gmeta, mb));
    HIP_OK(hipMalloc((void**)&wmeta, mb));
    HIP_OK(hipMalloc((void**)&nsat, sizeof(uint64_t)));
    HIP_OK(hipMemcpy(x, hx, n * sizeof(float), hipMemcpyHostToDevice));
    HIP_OK(hipMemcpy(g, hg, n * sizeof(float), hipMemcpyHostToDevice));
    HIP_OK(hipMemset(nsat, 0, sizeof(uint64_t)));

    QSDP_DO(qsdp_quantize_grad(g, n, gbits, bucket, seed, 0, gcodes, gmeta, stream));
    QSDP_DO(qsdp_dequantize(gcodes, gmeta, n, gbits, bucket, QSDP_F32, ghat, stream));
    QSDP_DO(qsdp_fused_step(x, g, n, lr, wbits, gbits, bucket, 0.0f, seed, 0, wcodes, wmeta, nsat, stream));
    HIP_OK(hipStreamSynchronize(stream));

    if (dump(prefix, "gcodes", gcodes, gcb) || dump(prefix, "gmeta", gmeta, mb) ||
        dump(prefix, "ghat", ghat, n * sizeof(float)) || dump(prefix, "x", x, n * sizeof(float)) ||
        dump(prefix, "wcodes", wcodes, wcb) || dump(prefix, "wmeta", wmeta, mb))
        return 4;
    printf("qsdp_client: spec %d, n=%llu, W%d G%d, bucket %d: ok\n", qsdp_spec_version(),
           (unsigned long long)n, wbits, gbits, bucket);

    hipFree(x); hipFree(g); hipFree(ghat); hipFree(gcodes); hipFree(wcodes); hipFree(gmeta); hipFree(wmeta);
    hipFree(nsat);
    hipStreamDestroy(stream);
    free(hx);
    free(hg);
    return 0;
}
