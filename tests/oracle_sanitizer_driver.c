/*
 * Calls every entry point of the CPU oracle once per shape on exactly-sized heap buffers, so that
 * an AddressSanitizer / UndefinedBehaviorSanitizer build of the oracle (this file is compiled
 * together with oracle/qsdp_ref.c, see test_oracle_sanitizers.py) reports any access outside a
 * buffer, any overflow of a per-thread bucket array, and any undefined arithmetic. CPU only.
 * Prints "done <number of calls>" and exits 0 when every call returned success.
 */
#include <math.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "qsdp_ref.h"

static unsigned long long state = 88172645463325252ull;

static float unit(void) { /* xorshift: values in [0, 1) */
    state ^= state << 13;
    state ^= state >> 7;
    state ^= state << 17;
    return (float)((state >> 40) & 0xFFFFFFu) * 0x1p-24f;
}

static float* values(uint64_t n, float scale) {
    float* p = (float*)malloc((size_t)n * sizeof(float));
    for (uint64_t i = 0; i < n; ++i) p[i] = (unit() - 0.5f) * scale;
    return p;
}

static int calls = 0;

#define MUST(expr)                                                        \
    do {                                                                  \
        if ((expr) != QSDP_REF_OK) {                                      \
            fprintf(stderr, "failed: %s (n=%llu bucket=%d bits=%d)\n", #expr, (unsigned long long)n, bucket, bits); \
            return 1;                                                     \
        }                                                                 \
        ++calls;                                                          \
    } while (0)

static int one_shape(uint64_t n, int bucket, int bits) {
    const int P = 3;
    uint64_t nb = (n + (uint64_t)bucket - 1) / (uint64_t)bucket;
    size_t cbytes = qsdp_ref_codes_bytes(n, bits, bucket);
    size_t mbytes = qsdp_ref_meta_bytes(n, bucket);
    if (cbytes == 0 || mbytes != nb * 2 * sizeof(float)) return 1;
    float* x = values(n, 0.04f);
    float* g = values(n, 2e-3f);
    float* u = (float*)malloc((size_t)n * sizeof(float));
    for (uint64_t i = 0; i < n; ++i) u[i] = unit();
    uint8_t* bytes = (uint8_t*)malloc((size_t)n);
    uint8_t* bytes2 = (uint8_t*)malloc((size_t)n);
    uint32_t* codes = (uint32_t*)malloc(cbytes);
    uint32_t* peer_codes = (uint32_t*)malloc(cbytes * P);
    float* meta = (float*)malloc(mbytes);
    float* peer_meta = (float*)malloc(mbytes * P);
    float* out = (float*)malloc((size_t)n * sizeof(float));
    uint16_t* out16 = (uint16_t*)malloc((size_t)n * sizeof(uint16_t));
    float* mom = (float*)calloc((size_t)n, sizeof(float));
    float* var = (float*)calloc((size_t)n, sizeof(float));
    float levels[256];
    uint64_t sat = 0;

    MUST(qsdp_ref_quantize_grad_u(g, n, bits, bucket, u, bytes, meta));
    MUST(qsdp_ref_quantize_grad_u_ex(g, n, bits, bucket, u, 4u, bytes, meta));
    MUST(qsdp_ref_quantize_weight_xi(x, n, bits, bucket, 0.0f, 0.25f, bytes, meta, &sat));
    MUST(qsdp_ref_quantize_weight_xi_ex(x, n, bits, bucket, 0x1p-9f, -0.5f, 0u, bytes, meta, &sat));
    qsdp_ref_pack(bytes, n, bits, bucket, codes);
    qsdp_ref_unpack(codes, n, bits, bucket, bytes2);
    calls += 2;
    if (memcmp(bytes, bytes2, (size_t)n) != 0) return 1;
    MUST(qsdp_ref_quantize_grad(g, n, bits, bucket, 7u, 64u, codes, meta));
    MUST(qsdp_ref_quantize_grad_ex(g, n, bits, bucket, 7u, 0u, 1u, codes, meta));
    MUST(qsdp_ref_quantize_weight(x, n, bits, bucket, 0.0f, 7u, codes, meta, &sat));
    MUST(qsdp_ref_quantize_weight_ex(x, n, bits, bucket, 0x1p-8f, 7u, 2u, codes, meta, NULL));
    MUST(qsdp_ref_dequantize(codes, meta, n, bits, bucket, QSDP_REF_F32, out));
    MUST(qsdp_ref_dequantize(codes, meta, n, bits, bucket, QSDP_REF_BF16, out16));
    MUST(qsdp_ref_dequantize(codes, meta, n, bits, bucket, QSDP_REF_F16, out16));
    for (int p = 0; p < P; ++p)
        MUST(qsdp_ref_quantize_grad(g, n, bits, bucket, 100u + (uint64_t)p, 0u, peer_codes + p * (cbytes / 4),
                                    peer_meta + p * (mbytes / 4)));
    MUST(qsdp_ref_dequantize_add(peer_codes, cbytes / 4, peer_meta, mbytes / 4, P, n, bits, bucket, 1.0f / P, out));
    MUST(qsdp_ref_fused_step(x, g, n, 1e-3f, bits, bits, bucket, 0.0f, 3u, 0u, NULL, NULL, NULL));
    MUST(qsdp_ref_fused_step(x, g, n, 1e-3f, bits, 4, bucket, 0x1p-10f, 3u, 8u, codes, meta, &sat));
    MUST(qsdp_ref_fused_step_ex(x, g, n, 1e-3f, bits, 3, bucket, 0.0f, 3u, 0u, 1u | 4u | 8u, codes, meta, &sat));
    MUST(qsdp_ref_fused_step_codes(codes, meta, g, n, 1e-3f, bits, 5, bucket, 0.0f, 4u, 0u, 0u, &sat));
    MUST(qsdp_ref_fused_adamw_step(x, g, mom, var, n, 1e-3f, 0.9f, 0.95f, 1e-8f, 0.01f, 0.1f, 0.05f, bits, 4, bucket,
                                   0.0f, 5u, 0u, 0u, codes, meta, &sat));
    MUST(qsdp_ref_recv_step(x, peer_codes, cbytes / 4, peer_meta, mbytes / 4, P, n, 1.0f / P, 1e-3f, bits, bits, bucket,
                            0.0f, 6u, 0u, codes, meta, &sat));
    MUST(qsdp_ref_recv_step(x, peer_codes, cbytes / 4, peer_meta, mbytes / 4, P, n, 1.0f / P, 1e-3f, bits, bits, bucket,
                            0.0f, 6u, 8u, NULL, NULL, NULL));
    MUST(qsdp_ref_recv_adamw_step(x, mom, var, peer_codes, cbytes / 4, peer_meta, mbytes / 4, P, n, 1.0f / P, 1e-3f, 0.9f,
                                  0.95f, 1e-8f, 0.0f, 0.19f, 0.0975f, bits, bits, bucket, 0.0f, 7u, 8u, codes, meta, &sat));
    MUST(qsdp_ref_levels_uniform(bits, levels));
    MUST(qsdp_ref_fit_levels(x, n, bits, bucket, 0.01f, 0u, levels));
    MUST(qsdp_ref_fit_levels_sequential(x, n, bits, bucket, 0.01f, 2u, levels));
    MUST(qsdp_ref_quantize_levels(x, n, bits, bucket, levels, codes, meta));
    MUST(qsdp_ref_dequantize_levels(codes, meta, n, bits, bucket, levels, QSDP_REF_F32, out));
    MUST(qsdp_ref_dequantize_levels(codes, meta, n, bits, bucket, levels, QSDP_REF_BF16, out16));
    MUST(qsdp_ref_quantize_levels_stochastic(x, n, bits, bucket, levels, 9u, 16u, codes, meta));
    MUST(qsdp_ref_quantize_levels_u(x, n, bits, bucket, levels, u, bytes, meta));

    free(x); free(g); free(u); free(bytes); free(bytes2); free(codes); free(peer_codes); free(meta);
    free(peer_meta); free(out); free(out16); free(mom); free(var);
    return 0;
}

int main(void) {
    uint32_t ctr[4] = {1u, 2u, 3u, 4u}, key[2] = {5u, 6u}, blk[4];
    qsdp_ref_philox4x32_10(ctr, key, blk);
    float acc = qsdp_ref_grad_uniform(1u, ~0ull) + qsdp_ref_weight_shift(~0ull) + qsdp_ref_grad_shift(3u);
    acc += (float)qsdp_ref_f32_to_bf16(1.5f) + (float)qsdp_ref_f32_to_f16(65519.0f) + (float)qsdp_ref_f32_to_f16(1e-8f);
    if (!(acc == acc)) return 1;
    calls += 7;
    const int buckets[] = {32, 96, 8192};
    const int widths[] = {1, 3, 8};
    for (int threads = 1; threads <= 3; threads += 2) {
        qsdp_ref_set_threads(threads);
        for (int b = 0; b < 3; ++b) {
            const int bucket = buckets[b];
            const uint64_t sizes[] = {1u, (uint64_t)bucket - 1u, (uint64_t)bucket, 3u * (uint64_t)bucket + 5u};
            for (int s = 0; s < 4; ++s)
                for (int w = 0; w < 3; ++w)
                    if (one_shape(sizes[s], bucket, widths[w]) != 0) return 1;
        }
    }
    printf("done %d\n", calls);
    return 0;
}
