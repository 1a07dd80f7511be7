/*
 * qsdp_ref.h -- CPU oracle for the QSDP quantization codec and quantized SGD step.
 *
 * TEST INFRASTRUCTURE ONLY. This is a plain, slow, obviously-correct host
 * implementation used to check the GPU library and to report a CPU baseline.
 * Nothing in the product path may include, link or call it. It shares no code
 * with the HIP kernels.
 *
 * Everything is IEEE-754 binary32, round-to-nearest-even, no contraction: an
 * expression written a*b+c is two roundings, fmaf(a,b,c) is one.
 *
 * What each routine follows (paper = "Quantized Distributed Training of Large
 * Models with Convergence Guarantees", arXiv 2302.02390):
 *   - gradient quantizer Q^g : "quantization by flipping a coin" (appendix
 *     definition of Q^g_delta), applied in per-bucket min-max coordinates
 *     (Section 5.1, bucketing paragraph).
 *   - weight quantizer  Q^w : Definition 1 "quantization by random shift",
 *     either on a per-bucket min-max grid or on the explicit grid delta*(Z+xi).
 *   - step              : x_{t+1} = Q^w(x_t - eta * Q^g(g_t)) (Section 3.3,
 *     last display; Section 4.1 iteration).
 * The paper fixes neither a random number generator nor a wire format; those
 * are this project's choices and are documented where they are implemented.
 *
 * Parity pins: every routine here is pinned by tests that do not call it to
 * produce their own expectation (closed forms of Lemma 3 and of the coin-flip
 * lemma, exhaustive enumeration of the randomness, a textbook affine quantizer,
 * a third-party Philox implementation, brute-force bit extraction). No routine
 * is "parity unpinned".
 */
#ifndef QSDP_REF_H
#define QSDP_REF_H
#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum { QSDP_REF_OK = 0, QSDP_REF_EINVAL = -1 };
enum { QSDP_REF_F32 = 0, QSDP_REF_BF16 = 1, QSDP_REF_F16 = 2 };

/* Quantizer variants the paper names as admissible (flags of the *_ex routines):
 *  GRAD_SHIFT  gradients are quantized by random shift too (the appendix observes that the
 *              shift-and-round operator meets the definition of an unbiased gradient quantizer):
 *              one shift xi_g per call (stream 2), no per-element randomness;
 *  NO_SHIFT    xi = 0 (and xi_g = 0): deterministic round-to-nearest;
 *  SYMMETRIC   per-bucket grid over [-a, a], a = max |v| (the symmetric scaling of
 *              Section 3.2) instead of [min, max]; ignored with an explicit delta.
 * For the step routines only (fused_step_ex, fused_adamw_step, recv_step):
 *  KEEP_MASTER the weight partition stays in full precision, as in Algorithm 2 where
 *              WeightUpdate acts on w_p and QuantizeWeights only produces what is transmitted:
 *              x <- y (the updated value itself) while wcodes / wmeta still receive Q^w(y). */
enum {
    QSDP_REF_FLAG_GRAD_SHIFT = 1,
    QSDP_REF_FLAG_NO_SHIFT = 2,
    QSDP_REF_FLAG_SYMMETRIC = 4,
    QSDP_REF_FLAG_ALL = 7, /* the quantizer variants */
    QSDP_REF_FLAG_KEEP_MASTER = 8
};

/* Number of worker threads for the bucket loop (buckets are independent, so the
 * output does not depend on it). Default 1. Returns the value now in force. */
int qsdp_ref_set_threads(int threads);

/* Philox4x32-10 block function (Salmon, Moraes, Dror, Shaw, SC'11). */
void qsdp_ref_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]);

/* The uniform u in [0,1) that decides the rounding of the gradient element whose
 * GLOBAL index is e, and the shift xi in [-1/2,1/2) of a weight quantization. */
float qsdp_ref_grad_uniform(uint64_t seed, uint64_t e);
uint32_t qsdp_ref_grad_uniform16(uint64_t seed, uint64_t e); /* the same as the integer h = u * 2^16 */
float qsdp_ref_weight_shift(uint64_t seed);
float qsdp_ref_grad_shift(uint64_t seed);

/* Sizes of the packed representation. */
size_t qsdp_ref_codes_bytes(uint64_t n, int bits, int bucket);
size_t qsdp_ref_meta_bytes(uint64_t n, int bucket);

/* --- cores with the randomness passed in (one code per byte, not packed) --- */
int qsdp_ref_quantize_grad_u(const float* g, uint64_t n, int bits, int bucket,
                             const float* u /* n uniforms in [0,1) */,
                             uint8_t* codes /* n */, float* meta /* 2*nb */);
int qsdp_ref_quantize_weight_xi(const float* x, uint64_t n, int bits, int bucket,
                                float delta, float xi,
                                uint8_t* codes /* n */, float* meta /* 2*nb */,
                                uint64_t* n_saturated /* nullable, incremented */);
int qsdp_ref_quantize_grad_u_ex(const float* g, uint64_t n, int bits, int bucket, const float* u,
                                uint32_t flags, uint8_t* codes, float* meta);
int qsdp_ref_quantize_weight_xi_ex(const float* x, uint64_t n, int bits, int bucket, float delta,
                                   float xi, uint32_t flags, uint8_t* codes, float* meta,
                                   uint64_t* n_saturated);
void qsdp_ref_pack(const uint8_t* codes, uint64_t n, int bits, int bucket, uint32_t* words);
void qsdp_ref_unpack(const uint32_t* words, uint64_t n, int bits, int bucket, uint8_t* codes);
uint16_t qsdp_ref_f32_to_bf16(float v);
/* binary32 -> IEEE binary16, round to nearest even, subnormals kept, overflow to infinity. */
uint16_t qsdp_ref_f32_to_f16(float v);

/* --- the four operations, same meaning as the library's entry points, on host
 * pointers, synchronous --- */
int qsdp_ref_quantize_grad(const float* g, uint64_t n, int bits, int bucket,
                           uint64_t seed, uint64_t index_offset,
                           uint32_t* codes, float* meta);
int qsdp_ref_quantize_weight(const float* x, uint64_t n, int bits, int bucket,
                             float delta, uint64_t seed,
                             uint32_t* codes, float* meta, uint64_t* n_saturated);
int qsdp_ref_dequantize(const uint32_t* codes, const float* meta, uint64_t n, int bits,
                        int bucket, int out_dtype, void* out);
/* The same three operations with variant flags. */
int qsdp_ref_quantize_grad_ex(const float* g, uint64_t n, int bits, int bucket, uint64_t seed,
                              uint64_t index_offset, uint32_t flags, uint32_t* codes, float* meta);
int qsdp_ref_quantize_weight_ex(const float* x, uint64_t n, int bits, int bucket, float delta,
                                uint64_t seed, uint32_t flags, uint32_t* codes, float* meta,
                                uint64_t* n_saturated);
int qsdp_ref_fused_step_ex(float* x, const float* g, uint64_t n, float lr, int wbits, int gbits,
                           int bucket, float delta, uint64_t seed, uint64_t index_offset,
                           uint32_t flags, uint32_t* wcodes, float* wmeta, uint64_t* n_saturated);

/* Receive side of a quantized gradient exchange (Algorithm 2: every worker's quantized
 * gradient slice arrives, the slices are decoded and summed before the weight update):
 * out[i] = alpha * (((d_0[i] + d_1[i]) + d_2[i]) + ...), d_p = decoded slice of peer p, the
 * sum taken in peer order with one binary32 rounding per addition. Peer p's codes start
 * codes_stride_words words after peer p-1's, its meta meta_stride_floats floats after. */
int qsdp_ref_dequantize_add(const uint32_t* codes, uint64_t codes_stride_words, const float* meta,
                            uint64_t meta_stride_floats, int npeers, uint64_t n, int bits,
                            int bucket, float alpha, float* out);
int qsdp_ref_fused_step(float* x, const float* g, uint64_t n, float lr,
                        int wbits, int gbits, int bucket, float delta,
                        uint64_t seed, uint64_t index_offset,
                        uint32_t* wcodes /* nullable */, float* wmeta /* nullable */,
                        uint64_t* n_saturated /* nullable */);

/* AdamW-flavoured quantized step (the optimizer of the paper's experiments, Appendix A, in
 * place of plain SGD inside the quantized iteration): per bucket ghat = decode(Q^g(g)); then per
 * element, all in binary32 in this order:
 *   m <- fma(beta1, m, (1-beta1)*ghat);  v <- fma(beta2, v, ((1-beta2)*ghat)*ghat);
 *   upd = (m / bias1) / (sqrt(v / bias2) + eps);  y = fma(-lr, fma(weight_decay, x, upd), x);
 * then x <- decode(Q^w(y)). bias1 = 1-beta1^t and bias2 = 1-beta2^t are passed in by the caller.
 * m and v are updated in place. flags, delta, seeds as in qsdp_ref_fused_step_ex. */
int qsdp_ref_fused_adamw_step(float* x, const float* g, float* m, float* v, uint64_t n, float lr,
                              float beta1, float beta2, float eps, float weight_decay, float bias1,
                              float bias2, int wbits, int gbits, int bucket, float delta,
                              uint64_t seed, uint64_t index_offset, uint32_t flags,
                              uint32_t* wcodes, float* wmeta, uint64_t* n_saturated);

/* ---- Learned (non-uniform) quantization levels: Section 5.2, Algorithm 1, Appendix C ----
 * A level table holds 2^bits positions in bucket-normalised coordinates z = (v - lo)/(hi - lo)
 * in [0, 1], ascending. Encoding picks the NEAREST level (ties: the lowest index); decoding is
 * a table lookup: v' = fma(levels[code], hi - lo, lo). meta = {lo, hi - lo}. The wire format
 * of the codes is the one of the uniform quantizers.
 *
 * fit_levels is the level optimisation of Algorithm 1 in its batched form (batch = one bucket,
 * the paper's batch size equals its bucket size): the values of a batch are normalised
 * bucket-wise and assigned to their closest level with the levels frozen; then every level
 * that received c > 0 values takes the c steps q <- q - lr*(q - v) of the algorithm towards
 * the mean m of its values at once: q <- q - (1 - (1-lr)^c) * (q - m). Sums are exact
 * (32.32 fixed point, order independent), the update is evaluated in binary64 and the level
 * is stored in binary32. Batches are visited in order, first `max_batches` only if > 0. */
int qsdp_ref_levels_uniform(int bits, float* levels /* 2^bits */);
int qsdp_ref_quantize_levels(const float* v, uint64_t n, int bits, int bucket, const float* levels,
                             uint32_t* codes, float* meta);
int qsdp_ref_dequantize_levels(const uint32_t* codes, const float* meta, uint64_t n, int bits,
                               int bucket, const float* levels, int out_dtype, void* out);
/* Unbiased (coin-flip) rounding onto the two levels that enclose the normalised value; uniforms
 * from Philox stream 0 as for the gradient quantizer. codes of the _u form are unpacked (u8). */
int qsdp_ref_quantize_levels_stochastic(const float* v, uint64_t n, int bits, int bucket, const float* levels,
                                        uint64_t seed, uint64_t index_offset, uint32_t* codes, float* meta);
int qsdp_ref_quantize_levels_u(const float* v, uint64_t n, int bits, int bucket, const float* levels,
                               const float* u, uint8_t* codes, float* meta);
int qsdp_ref_fit_levels(const float* v, uint64_t n, int bits, int bucket, float lr,
                        uint64_t max_batches, float* levels /* in: start, out: fitted */);
/* Algorithm 1 as printed: one value at a time against the current table, one step of the chosen
 * level per value (no batches; `max_batches` only bounds how many buckets of values are visited). */
int qsdp_ref_fit_levels_sequential(const float* v, uint64_t n, int bits, int bucket, float lr,
                                   uint64_t max_batches, float* levels /* in: start, out: fitted */);

/* The step on weights held as codes: decode (wcodes, wmeta), take the fused step, write the
 * codes and meta of the result back. By definition the composition of the two routines. */
int qsdp_ref_fused_step_codes(uint32_t* wcodes, float* wmeta, const float* g, uint64_t n, float lr,
                              int wbits, int gbits, int bucket, float delta,
                              uint64_t seed, uint64_t index_offset, uint32_t flags,
                              uint64_t* n_saturated);

/* The shard owner's update with P workers (Algorithm 2): decode-and-average the peers'
 * quantized gradient slices, take the SGD step, quantize the new weights with Q^w and decode:
 * ghat = alpha * (((d_0 + d_1) + ...)); y = fma(-lr, ghat, x); x <- decode(Q^w(y)).
 * By definition the composition of qsdp_ref_dequantize_add, the fma and qsdp_ref_quantize_weight_ex
 * + qsdp_ref_dequantize. flags: NO_SHIFT, SYMMETRIC. */
int qsdp_ref_recv_step(float* x, const uint32_t* gcodes, uint64_t codes_stride_words, const float* gmeta,
                       uint64_t meta_stride_floats, int npeers, uint64_t n, float alpha, float lr,
                       int wbits, int gbits, int bucket, float delta, uint64_t seed, uint32_t flags,
                       uint32_t* wcodes, float* wmeta, uint64_t* n_saturated);

/* The same with AdamW (Appendix A) in place of the SGD step: ghat as above, then per element
 * m, v, y as in qsdp_ref_fused_adamw_step, then Q^w(y). flags: NO_SHIFT, SYMMETRIC, KEEP_MASTER. */
int qsdp_ref_recv_adamw_step(float* x, float* mom, float* var, const uint32_t* gcodes,
                             uint64_t codes_stride_words, const float* gmeta, uint64_t meta_stride_floats,
                             int npeers, uint64_t n, float alpha, float lr, float beta1, float beta2, float eps,
                             float weight_decay, float bias1, float bias2, int wbits, int gbits, int bucket,
                             float delta, uint64_t seed, uint32_t flags, uint32_t* wcodes, float* wmeta,
                             uint64_t* n_saturated);

#ifdef __cplusplus
}
#endif
#endif
