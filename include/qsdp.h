/*
 * qsdp.h -- C ABI of the MI355X (gfx950) QSDP quantization codec and fused quantized
 * SGD step.
 *
 * The operations are those of "Quantized Distributed Training of Large Models with
 * Convergence Guarantees" (arXiv 2302.02390):
 *   Q^g  unbiased stochastic ("coin-flip") quantizer of gradients (Section 3.2; appendix
 *        definition "quantization by flipping a coin"), applied per bucket in min-max
 *        coordinates (Section 5.1, bucketing);
 *   Q^w  quantization of weights by random shift (Section 4.1, Definition 1), on a
 *        per-bucket min-max grid or on the explicit grid delta*(Z + xi);
 *   step x_{t+1} = Q^w(x_t - eta * Q^g(g_t)) (Section 3.3, last display).
 *
 * Conventions shared by every entry point
 * ---------------------------------------
 *  - All tensor pointers are DEVICE pointers (HIP global memory of the current device),
 *    16-byte aligned, allocated and owned by the caller. The library allocates no device
 *    memory, keeps no pointer after returning and has no mutable global state.
 *  - `stream` is a hipStream_t passed as void* (NULL = the default stream). Work is
 *    enqueued on it and the call returns without synchronising.
 *  - Return value: QSDP_OK, or a negative error. On error nothing has been launched.
 *  - n >= 1 elements; bits in [1,8]; bucket a multiple of 32 in [32, 8192]. The vector is
 *    cut into buckets of `bucket` consecutive elements; the last one may be short.
 *  - Inputs must be finite. Non-finite inputs give unspecified codes but no fault.
 *
 * Random numbers (the paper leaves the generator open): Philox4x32-10, key =
 * (seed low 32 bits, seed high 32 bits), counter = (c low, c high, stream, 0).
 *   stream 0, gradient rounding: the element with GLOBAL index e = index_offset + i uses
 *     block c = e/8 and the 16-bit half (e%8) of its four words (word (e%8)/2, low half
 *     first): an integer h in [0, 2^16). index_offset must be a multiple of 8. Quantizing a
 *     bucket-aligned shard with its global offset gives the bytes the whole vector gives.
 *   stream 1, weight shift: c = 0, xi = (word0 >> 8) * 2^-24 - 1/2 in [-1/2, 1/2); one
 *     draw per call whatever the shard (Definition 1 shifts the whole vector by one scalar).
 *
 * Packed representation (the paper leaves the layout open)
 * ---------------------------------------------------------
 *  codes: bucket j owns the 32-bit words [j*bucket*bits/32, (j+1)*bucket*bits/32). Within
 *         a bucket, element i occupies bits [i*bits, (i+1)*bits) of a little-endian bit
 *         stream (stream bit p = bit p%32 of word p/32). Slots past the end of a short
 *         last bucket are written as 0.
 *  meta:  float[2*nb]: {base_j, scale_j}; the decoded value of code c is
 *         fma(c, scale_j, base_j). For Q^w the shift is folded into base_j.
 *
 * Arithmetic is IEEE binary32, round to nearest even, in a fixed operation order, so that
 * the output is a pure function of the arguments (bit-reproducible, no atomics on data).
 */
#ifndef QSDP_H
#define QSDP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    QSDP_OK = 0,
    QSDP_EINVAL = -1,  /* bad n / bits / bucket / delta / lr / dtype / index_offset / NULL */
    QSDP_EALIGN = -2,  /* a pointer is not 16-byte aligned */
    QSDP_ELAUNCH = -3  /* the HIP runtime refused the launch */
};

/* Formats of decoded output (all three) and of 16-bit gradient input (QSDP_BF16, QSDP_F16).
 * QSDP_F16 is IEEE binary16, the half precision of the paper's mixed-precision setting. */
typedef enum { QSDP_F32 = 0, QSDP_BF16 = 1, QSDP_F16 = 2 } qsdp_dtype;

/* Version of the arithmetic/wire specification implemented (3: 16-bit uniforms, 8 per Philox
 * block; coin flips decided in integers with the fraction rounded to 16 bits to nearest). */
uint32_t qsdp_spec_version(void);

/* Bytes of the packed codes / of the meta-data for n elements: nb*bucket*bits/8 and
 * nb*2*sizeof(float), nb = ceil(n/bucket). 0 if the arguments are invalid. Host only. */
size_t qsdp_codes_bytes(uint64_t n, int bits, int bucket);
size_t qsdp_meta_bytes(uint64_t n, int bucket);

/* Human-readable text for a status code (static storage). */
const char* qsdp_status_string(int status);

/*
 * Q^g: bucketed unbiased stochastic quantization (coin-flip definition; Section 5.1).
 * Per bucket: lo = min, hi = max, scale = (hi-lo)/L, L = 2^bits-1; the position t = (g-lo)*(L/(hi-lo))
 * is taken in units of 2^-16 of a cell, rounded to nearest: ti = min(floor(fma(g-lo, 2^16*L/(hi-lo), 1/2)),
 * L*2^16); code = floor((ti + h)/2^16), i.e. floor(t)+1 for (ti mod 2^16) of the 2^16 values of h,
 * floor(t) otherwise; meta = {lo, scale}. A constant bucket (or one whose range is so small that
 * 2^16*L/(hi-lo) overflows) gets scale 0 and codes 0.
 *   g      in   device float[n]
 *   codes  out  device uint32[qsdp_codes_bytes/4]
 *   meta   out  device float[2*nb]
 */
int qsdp_quantize_grad(const float* g, uint64_t n, int bits, int bucket,
                       uint64_t seed, uint64_t index_offset,
                       uint32_t* codes, float* meta, void* stream);

/*
 * Q^w: quantization by random shift (Definition 1).
 *   delta == 0: per-bucket grid lo + scale*(Z + xi), scale = (hi-lo)/L;
 *               code = clamp(round((x-lo)/scale - xi), 0, L); meta = {lo + xi*scale, scale}.
 *   delta  > 0: the grid delta*(Z + xi) of Definition 1; lattice coordinate
 *               k = round(x/delta - xi); a bucket stores k - k0 (k0 = coordinate of its
 *               minimum) in `bits` bits; meta = {(k0+xi)*delta, delta}. Coordinates more
 *               than L above k0 are clamped to L and counted in *n_saturated.
 *   n_saturated  in/out, nullable, device uint64: incremented (atomically) by the number of
 *               clamped elements; the caller zeroes it.
 */
int qsdp_quantize_weight(const float* x, uint64_t n, int bits, int bucket,
                         float delta, uint64_t seed,
                         uint32_t* codes, float* meta,
                         uint64_t* n_saturated, void* stream);

/*
 * Decoding (the inverse map of Section 4.1: lattice coordinate back to a value, shift
 * included; what a worker does with a gathered quantized layer in Algorithm 2):
 * out[i] = fma(code_i, scale_j, base_j),
 * stored as float (QSDP_F32) or rounded to nearest-even bfloat16 (QSDP_BF16) or IEEE binary16
 * (QSDP_F16: subnormal results kept, magnitudes beyond 65504 + half an ulp become infinity); the
 * same three formats hold for every decoding entry point below. Serves both quantizers. Elements
 * past n are not written.
 *   out  out  device float[n] or uint16[n]
 */
int qsdp_dequantize(const uint32_t* codes, const float* meta, uint64_t n, int bits,
                    int bucket, qsdp_dtype out_dtype, void* out, void* stream);

/*
 * Decoding of a gathered layer (Algorithm 2: after the all-gather of the quantized weight
 * shards a worker holds one slot per peer and decodes the whole layer, twice per micro-batch;
 * the highest-volume call of the scheme): peer p's slot holds the packed codes and meta of
 * elements [p*shard, min((p+1)*shard, n)) of the layer, quantized on their own by
 * qsdp_quantize_weight (or a fused step); `shard` is a multiple of `bucket`, so the buckets are
 * those of the unsharded layer, and npeers = ceil(n / shard). One launch writes
 * out[0..n) = what qsdp_dequantize gives slot by slot. Peer p's codes start
 * p * codes_stride_bytes after `codes`, its meta p * meta_stride_bytes after `meta` (strides:
 * multiples of 16, at least the size of a full shard's codes / meta; a receive buffer whose
 * slots hold codes followed by meta is addressed with equal strides). shard < 2^37,
 * npeers <= 65535.
 *   out  out  device float[n] or uint16[n]
 */
int qsdp_dequantize_gathered(const uint32_t* codes, uint64_t codes_stride_bytes,
                             const float* meta, uint64_t meta_stride_bytes, int npeers,
                             uint64_t n, uint64_t shard, int bits, int bucket,
                             qsdp_dtype out_dtype, void* out, void* stream);

/*
 * Decode-and-sum, the receive side of a quantized gradient exchange (Algorithm 2: the
 * quantized gradient slices of all workers reach the owner of a shard, which decodes and adds
 * them before the weight update; codes with different per-bucket scales cannot be added in
 * flight): out[i] = alpha * (((d_0[i] + d_1[i]) + d_2[i]) + ...), d_p = decoded slice of peer p
 * (as qsdp_dequantize would give), summed in peer order with one rounding per addition; pass
 * alpha = 1/npeers for the average. Peer p's packed codes start p * codes_stride_bytes after
 * `codes`, its meta p * meta_stride_bytes after `meta` (a receive buffer with one slot per
 * peer); strides are multiples of 4 and at least the size of one slice.
 *   out  out  device float[n]
 */
int qsdp_dequantize_add(const uint32_t* codes, uint64_t codes_stride_bytes,
                        const float* meta, uint64_t meta_stride_bytes, int npeers,
                        uint64_t n, int bits, int bucket, float alpha,
                        float* out, void* stream);

/*
 * Fused quantized SGD step, in place: x <- Q^w(x - lr * Q^g(g)) (Section 3.3 / 4.1), one
 * pass over HBM (read x, read g, write x). Per bucket: Q^g of g with `gbits`, decoded in
 * registers; y = fma(-lr, ghat, x); Q^w of y with `wbits` (delta as in
 * qsdp_quantize_weight), decoded into x. The same seed drives both random streams.
 *   x        in/out device float[n]
 *   g        in     device float[n]
 *   wcodes   out, nullable: packed Q^w codes of the new x (what the next weight gather
 *            would transmit); wmeta must be given iff wcodes is.
 *   n_saturated as in qsdp_quantize_weight.
 */
int qsdp_fused_step(float* x, const float* g, uint64_t n, float lr,
                    int wbits, int gbits, int bucket, float delta,
                    uint64_t seed, uint64_t index_offset,
                    uint32_t* wcodes, float* wmeta,
                    uint64_t* n_saturated, void* stream);

/*
 * The shard owner's step with P workers (Algorithm 2: the quantized gradient slices of all
 * workers reach the owner of a shard, which averages them, updates its weights and quantizes
 * them for the next weight gather), fused into one pass: read x and the P code slices, write x
 * (and the packed Q^w codes): 8 + P * gbits/8 (+ wbits/8) bytes per parameter instead of the
 * 16 + P * gbits/8 of qsdp_dequantize_add followed by a separate update.
 *   ghat = alpha * (((d_0 + d_1) + d_2) + ...)   as qsdp_dequantize_add computes it
 *   y = fma(-lr, ghat, x);   x <- decode(Q^w(y)) as in qsdp_fused_step (delta, seed, wcodes,
 *   wmeta, n_saturated as there). No Q^g is applied: the slices were quantized by their senders.
 * gcodes / gmeta and their strides as in qsdp_dequantize_add, except that the code stride is a
 * multiple of 16 bytes; flags: QSDP_FLAG_NO_SHIFT, QSDP_FLAG_SYMMETRIC, QSDP_FLAG_KEEP_MASTER.
 */
int qsdp_recv_step(float* x, const uint32_t* gcodes, uint64_t gcodes_stride_bytes,
                   const float* gmeta, uint64_t gmeta_stride_bytes, int npeers, uint64_t n,
                   float alpha, float lr, int wbits, int gbits, int bucket, float delta,
                   uint64_t seed, uint32_t flags, uint32_t* wcodes, float* wmeta,
                   uint64_t* n_saturated, void* stream);

/*
 * The same with AdamW (Appendix A) in place of the SGD update, which is what the paper's
 * experiments run on every shard: ghat as in qsdp_recv_step, then per element m, v, u, y as in
 * qsdp_fused_adamw_step (defined below), then Q^w(y). Reads x, m, v and the P code slices,
 * writes x, m, v (and the packed codes): 24 + P * gbits/8 (+ wbits/8) bytes per parameter.
 * With QSDP_FLAG_KEEP_MASTER this is Algorithm 2's weight update as written: AdamW on the
 * full-precision partition, the codes being what the next weight gather transmits.
 */
int qsdp_recv_adamw_step(float* x, float* m, float* v, const uint32_t* gcodes,
                         uint64_t gcodes_stride_bytes, const float* gmeta,
                         uint64_t gmeta_stride_bytes, int npeers, uint64_t n, float alpha,
                         float lr, float beta1, float beta2, float eps, float weight_decay,
                         float bias1, float bias2, int wbits, int gbits, int bucket, float delta,
                         uint64_t seed, uint32_t flags, uint32_t* wcodes, float* wmeta,
                         uint64_t* n_saturated, void* stream);

/*
 * Quantizer variants the paper names as admissible, selected by `flags` (0 = the default
 * operators above; meta-data and wire format are unchanged, so qsdp_dequantize serves all):
 *   QSDP_FLAG_GRAD_SHIFT  gradients are quantized by random shift as well (the appendix notes
 *                         that the shift-and-round operator is an unbiased quantizer in the
 *                         sense required of Q^g): one shift xi_g per call from Philox stream 2,
 *                         code = clamp(round((g-lo)/scale - xi_g), 0, L), meta = {lo + xi_g*scale,
 *                         scale}; nothing is drawn per element, index_offset has no effect.
 *   QSDP_FLAG_NO_SHIFT    xi = 0 and xi_g = 0: deterministic round-to-nearest (biased).
 *   QSDP_FLAG_SYMMETRIC   per-bucket grid over [-a, a], a = max |v| (the symmetric scaling of
 *                         Section 3.2) instead of [min, max]; no effect with delta > 0.
 * For the entry points that update a weight partition in place (qsdp_fused_step_ex,
 * qsdp_fused_adamw_step, qsdp_recv_step, qsdp_recv_adamw_step) there is also
 *   QSDP_FLAG_KEEP_MASTER the partition stays in full precision, as in Algorithm 2 where the
 *                         weight update acts on w_p and the weight quantizer only produces what is
 *                         transmitted: x receives the updated value y itself instead of
 *                         decode(Q^w(y)); wcodes / wmeta / n_saturated are unchanged.
 * Other bits, and bits an entry point has no use for, are rejected with QSDP_EINVAL.
 */
enum {
    QSDP_FLAG_GRAD_SHIFT = 1, QSDP_FLAG_NO_SHIFT = 2, QSDP_FLAG_SYMMETRIC = 4,
    QSDP_FLAG_ALL = 7, /* the quantizer variants */
    QSDP_FLAG_KEEP_MASTER = 8
};

int qsdp_quantize_grad_ex(const float* g, uint64_t n, int bits, int bucket,
                          uint64_t seed, uint64_t index_offset, uint32_t flags,
                          uint32_t* codes, float* meta, void* stream);
int qsdp_quantize_weight_ex(const float* x, uint64_t n, int bits, int bucket,
                            float delta, uint64_t seed, uint32_t flags,
                            uint32_t* codes, float* meta,
                            uint64_t* n_saturated, void* stream);
/* (thin forward of qsdp_fused_step_opts) */
int qsdp_fused_step_ex(float* x, const float* g, uint64_t n, float lr,
                       int wbits, int gbits, int bucket, float delta,
                       uint64_t seed, uint64_t index_offset, uint32_t flags,
                       uint32_t* wcodes, float* wmeta,
                       uint64_t* n_saturated, void* stream);

/*
 * Gradients that arrive in a 16-bit format: the paper's system receives half-precision
 * gradients and converts them to full precision before quantizing (Section 6, experimental
 * setup). Here the kernels widen each value to binary32 on load, which is exact for both
 * formats, so the result equals the fp32 entry point called on the converted gradient, without
 * the conversion pass and with 2 bytes of gradient traffic per parameter instead of 4.
 *   g        in  device uint16[n] bit patterns of g_dtype, 16-byte aligned
 *   g_dtype      QSDP_F16 (IEEE binary16, the paper's) or QSDP_BF16; anything else: QSDP_EINVAL
 * Everything else as in qsdp_quantize_grad_ex / qsdp_fused_step_ex.
 */
int qsdp_quantize_grad_g16(const void* g, qsdp_dtype g_dtype, uint64_t n, int bits, int bucket,
                           uint64_t seed, uint64_t index_offset, uint32_t flags,
                           uint32_t* codes, float* meta, void* stream);
/* (thin forward of qsdp_fused_step_opts) */
int qsdp_fused_step_g16(float* x, const void* g, qsdp_dtype g_dtype, uint64_t n, float lr,
                        int wbits, int gbits, int bucket, float delta,
                        uint64_t seed, uint64_t index_offset, uint32_t flags,
                        uint32_t* wcodes, float* wmeta,
                        uint64_t* n_saturated, void* stream);

/*
 * The fused step in a mixed-precision training loop: the gradient may arrive in 16 bits (as in
 * the *_g16 calls; g_dtype QSDP_F32, QSDP_F16 or QSDP_BF16 says what g points to), and the new
 * quantized weights Q^w(y), which x receives in fp32 (unless QSDP_FLAG_KEEP_MASTER keeps y
 * there), can be written once more in 16 bits for the next forward pass:
 *   x16        out, nullable  device uint16[n], 16-byte aligned: decode(Q^w(y)) rounded to x16_dtype
 *                             (nearest even), i.e. what qsdp_dequantize gives for the emitted codes
 *   x16_dtype                 QSDP_BF16 or QSDP_F16 (ignored when x16 is NULL)
 * 2 more bytes written per parameter instead of a separate conversion or decoding pass.
 * Everything else as in qsdp_fused_step_ex.
 */
/* (thin forward of qsdp_fused_step_opts) */
int qsdp_fused_step_mp(float* x, const void* g, qsdp_dtype g_dtype, uint64_t n, float lr,
                       int wbits, int gbits, int bucket, float delta,
                       uint64_t seed, uint64_t index_offset, uint32_t flags,
                       uint32_t* wcodes, float* wmeta, void* x16, qsdp_dtype x16_dtype,
                       uint64_t* n_saturated, void* stream);

/* qsdp_fused_adamw_step in the same mixed-precision form (gradient format g_dtype, optional 16-bit
 * copy x16 of the new quantized weights): the training step of the paper's experiments on one worker. */
/* (thin forward of qsdp_fused_adamw_step_opts) */
int qsdp_fused_adamw_step_mp(float* x, const void* g, qsdp_dtype g_dtype, float* m, float* v,
                             uint64_t n, float lr, float beta1, float beta2, float eps,
                             float weight_decay, float bias1, float bias2,
                             int wbits, int gbits, int bucket, float delta,
                             uint64_t seed, uint64_t index_offset, uint32_t flags,
                             uint32_t* wcodes, float* wmeta, void* x16, qsdp_dtype x16_dtype,
                             uint64_t* n_saturated, void* stream);

/*
 * qsdp_fused_step_ex with the seed advanced from device memory, for callers that capture the
 * step in a HIP graph: kernel arguments are frozen at capture, so a replayed step would draw the
 * same random numbers again; here the seed in force is seed + *seed_dev (mod 2^64), read when the
 * kernel starts, and other work in the same graph (any kernel that increments *seed_dev) moves it
 * on between replays. seed_dev: device uint64, 8-byte aligned. Equal to qsdp_fused_step_ex called
 * with that sum.
 */
/* (thin forward of qsdp_fused_step_opts) */
int qsdp_fused_step_dseed(float* x, const float* g, uint64_t n, float lr,
                          int wbits, int gbits, int bucket, float delta,
                          uint64_t seed, const uint64_t* seed_dev, uint64_t index_offset,
                          uint32_t flags, uint32_t* wcodes, float* wmeta,
                          uint64_t* n_saturated, void* stream);

/*
 * The quantized step with AdamW (the optimizer of the paper's experiments, Appendix A: betas
 * 0.9 / 0.95, eps 1e-8) between the two quantizers in place of the plain SGD update, one pass
 * over HBM: read x, g, m, v; write x, m, v (28 bytes per parameter). Per bucket
 * ghat = decode(Q^g(g)), then per element, in binary32 and in this order:
 *   m <- fma(beta1, m, (1-beta1)*ghat);   v <- fma(beta2, v, ((1-beta2)*ghat)*ghat);
 *   u = (m / bias1) / (sqrt(v / bias2) + eps);   y = fma(-lr, fma(weight_decay, x, u), x);
 * then x <- decode(Q^w(y)). bias1 = 1 - beta1^t and bias2 = 1 - beta2^t (t = step number from
 * 1) are computed by the caller. 0 <= beta < 1, eps > 0, bias > 0.
 *   m, v  in/out  device float[n], the moment estimates (start at 0)
 * flags as in the *_ex entry points; the other arguments as in qsdp_fused_step.
 */
/* (thin forward of qsdp_fused_adamw_step_opts) */
int qsdp_fused_adamw_step(float* x, const float* g, float* m, float* v, uint64_t n, float lr,
                          float beta1, float beta2, float eps, float weight_decay,
                          float bias1, float bias2,
                          int wbits, int gbits, int bucket, float delta,
                          uint64_t seed, uint64_t index_offset, uint32_t flags,
                          uint32_t* wcodes, float* wmeta,
                          uint64_t* n_saturated, void* stream);

/*
 * The same step with the weights RESIDENT AS CODES: every iterate of the quantized iteration
 * lies on its bucket grids (Section 4.1: the iterates live in the lattice domain), so
 * (wcodes, wmeta) hold x_t exactly and the fp32 copy is redundant. The call decodes x_t in
 * registers, takes the step and writes the codes and meta of x_{t+1} back in place:
 * 4 + 2*wbits/8 bytes of HBM traffic per parameter instead of 12. Bit-identical to
 * qsdp_dequantize followed by qsdp_fused_step_ex with code output and the same flags.
 *   wcodes, wmeta  in/out  packed Q^w representation of x (as written by qsdp_quantize_weight
 *                  or a fused step with the same wbits and bucket)
 */
int qsdp_fused_step_codes(uint32_t* wcodes, float* wmeta, const float* g, uint64_t n, float lr,
                          int wbits, int gbits, int bucket, float delta,
                          uint64_t seed, uint64_t index_offset, uint32_t flags,
                          uint64_t* n_saturated, void* stream);

/*
 * qsdp_fused_adamw_step on code-resident weights: x_t is decoded from (wcodes, wmeta) in
 * registers as in qsdp_fused_step_codes, the AdamW update uses the fp32 moments m, v (read and
 * written), and the codes and meta of x_{t+1} = Q^w(y) overwrite the inputs. Bit-identical to
 * qsdp_dequantize followed by qsdp_fused_adamw_step with code output. flags: the quantizer
 * variants only (there is no fp32 copy of x to keep).
 */
int qsdp_fused_adamw_step_codes(uint32_t* wcodes, float* wmeta, const float* g, float* m, float* v,
                                uint64_t n, float lr, float beta1, float beta2, float eps,
                                float weight_decay, float bias1, float bias2,
                                int wbits, int gbits, int bucket, float delta,
                                uint64_t seed, uint64_t index_offset, uint32_t flags,
                                uint64_t* n_saturated, void* stream);

/*
 * Learned (non-uniform) quantization levels: Section 5.2, Algorithm 1, Appendix C.
 * A level table is 2^bits floats in bucket-normalised coordinates z = (v-lo)/(hi-lo) in
 * [0,1], ascending (DEVICE memory, 4-byte aligned; the library does not validate its contents;
 * unsorted levels give unspecified codes but no fault). Per bucket meta = {lo, hi-lo}.
 *   qsdp_levels_uniform     host only: fills a HOST array with k/(2^bits-1), the usual start.
 *   qsdp_quantize_levels    code = index of the NEAREST level to z (ties and equal levels: the
 *                           lowest index); deterministic. Wire format as for the other codes.
 *   qsdp_quantize_levels_stochastic  the unbiased counterpart for gradients (the coin-flip
 *                           definition of the appendix applied between the two levels that
 *                           enclose z): with i the largest index such that levels[i] <= z,
 *                           code = i + [2^16 - (h + 1/2) < p * 2^16], p = (z - levels[i]) /
 *                           (levels[i+1] - levels[i]), h the 16-bit rounding uniform of
 *                           qsdp_quantize_grad (same seed / index_offset rules): up for the
 *                           round(p * 2^16) largest values of h; z below the first level gives 0, at or above the last
 *                           2^bits-1, so the mean of the decoded value equals the input exactly
 *                           when the table starts at 0 and ends at 1.
 *   qsdp_dequantize_levels  out = fma(levels[code], hi-lo, lo), fp32 or bf16.
 *   qsdp_fit_levels         the level optimisation of Algorithm 1 in batched form, batch = one
 *                           bucket, visited in order (the first max_batches only, if > 0): the
 *                           values of a batch are normalised and assigned to their nearest
 *                           level with the levels frozen; every level that received c > 0
 *                           values takes its c steps of rate lr towards the mean m of those
 *                           values at once: q <- q - (1-(1-lr)^c)(q-m). Sums are exact (32.32
 *                           fixed point), the update is evaluated in binary64: the result is
 *                           reproducible bit for bit. Runs as ONE workgroup (each batch starts
 *                           from the levels the previous one left); it is a rare, offline-like
 *                           call (the paper runs it a few times per training), not a hot path.
 *                           0 < lr < 1. `levels` is read as the start and overwritten.
 */
int qsdp_levels_uniform(int bits, float* levels);
int qsdp_quantize_levels(const float* v, uint64_t n, int bits, int bucket, const float* levels,
                         uint32_t* codes, float* meta, void* stream);
int qsdp_quantize_levels_stochastic(const float* v, uint64_t n, int bits, int bucket,
                                    const float* levels, uint64_t seed, uint64_t index_offset,
                                    uint32_t* codes, float* meta, void* stream);
int qsdp_dequantize_levels(const uint32_t* codes, const float* meta, uint64_t n, int bits,
                           int bucket, const float* levels, qsdp_dtype out_dtype,
                           void* out, void* stream);
int qsdp_fit_levels(const float* v, uint64_t n, int bits, int bucket, float lr,
                    uint64_t max_batches, float* levels, void* stream);
/* qsdp_dequantize_gathered for slots that were encoded with qsdp_quantize_levels (all slots with
 * the same level table): out = what qsdp_dequantize_levels gives slot by slot. */
int qsdp_dequantize_levels_gathered(const uint32_t* codes, uint64_t codes_stride_bytes,
                                    const float* meta, uint64_t meta_stride_bytes, int npeers,
                                    uint64_t n, uint64_t shard, int bits, int bucket,
                                    const float* levels, qsdp_dtype out_dtype, void* out,
                                    void* stream);

/*
 * Multi-tensor ("segmented") variants: in the paper's system every layer is compressed on
 * its own (Section 5.1), i.e. bucketing restarts at each tensor.
 * These calls do that for many tensors laid back to back in one flat buffer with ONE kernel
 * launch, which matters when a model has hundreds of small tensors.
 *
 * A qsdp_segment describes one tensor: `n` elements at element offset `offset` of the flat
 * x / g buffers; its buckets carry the numbers first_bucket .. first_bucket + ceil(n/bucket)-1.
 * Packed codes and meta-data are indexed by bucket number exactly as in the single-tensor
 * calls (every bucket padded to `bucket` slots), so tensor t's codes start at word
 * first_bucket_t * bucket * bits / 32 and its meta at float 2 * first_bucket_t. The rounding
 * uniform of an element depends on index_offset + its position in the flat buffer, so the
 * result equals calling the single-tensor entry point on each tensor with
 * index_offset + offset_t.
 *
 * qsdp_segments_build (host only) fills a HOST table from tensor sizes, packing the tensors
 * contiguously (offset_t = sum of earlier sizes), and returns the total number of buckets, or 0
 * if a size is 0 or a size other than the last is not a multiple of 8 (offsets must keep 16-byte
 * alignment and Philox-block alignment). The caller copies the table to device memory and
 * passes that DEVICE pointer (8-byte aligned) with the same nseg / total_buckets / bucket. The
 * library does not validate the device table's contents.
 */
typedef struct qsdp_segment {
    uint64_t offset;
    uint64_t n;
    uint64_t first_bucket;
} qsdp_segment;

uint64_t qsdp_segments_build(const uint64_t* sizes, uint32_t nseg, int bucket, qsdp_segment* table);
/* The segmented entry points take a DEVICE copy of a table that qsdp_segments_build wrote, unchanged
 * (offsets multiples of 8, ascending first_bucket, total_buckets its return value). They check only the
 * pointer and the counts; a table with other contents leads to misaligned or out-of-range accesses. */

/*
 * ONE options block for every form of the fused step. The step of Section 3.3,
 * x <- Q^w(x - lr * Q^g(g)) (qsdp_fused_step_opts), or the same with AdamW between the quantizers
 * (qsdp_fused_adamw_step_opts, arithmetic as documented at qsdp_fused_adamw_step), with every
 * optional part named in the block: zero-initialise it, set `size`, fill in what is wanted.
 * opt == NULL means no options (the plain qsdp_fused_step). The entry points
 * qsdp_fused_step, _ex, _g16, _mp, _dseed, _segmented, _segmented_mp and qsdp_fused_adamw_step,
 * _mp, _segmented are thin forwards of these two calls that fill the block from their argument
 * lists; they stay for source compatibility and add nothing.
 *   size            sizeof(qsdp_step_options); anything else: QSDP_EINVAL
 *   flags           QSDP_FLAG_* (quantizer variants and KEEP_MASTER)
 *   g_dtype         what g points to: QSDP_F32 (0, float[n]), QSDP_BF16 or QSDP_F16 (uint16[n],
 *                   widened exactly on load)
 *   x16, x16_dtype  optional second copy of the new quantized weights in QSDP_BF16 / QSDP_F16
 *   segments, nseg, total_buckets   optional multi-tensor table (device memory, see above): the
 *                   buffers hold the tensors back to back, bucketing restarts per tensor, `n` is ignored
 *   seed_increment  optional device uint64 (8-byte aligned): the seed in force is seed +
 *                   *seed_increment, read when the kernel starts (for replayed HIP graphs)
 *   wcodes, wmeta   optional output (both or neither): packed codes and meta of the new weights
 *   n_saturated     optional in/out device uint64, incremented by the clamped elements (delta > 0)
 *   m, v, beta1, beta2, eps, weight_decay, bias1, bias2   AdamW only: moments (in/out, fp32) and
 *                   scalars; ignored by qsdp_fused_step_opts
 */
typedef struct qsdp_step_options {
    uint32_t size;
    uint32_t flags;
    qsdp_dtype g_dtype;
    qsdp_dtype x16_dtype;
    void* x16;
    const qsdp_segment* segments;
    uint32_t nseg;
    uint32_t reserved;
    uint64_t total_buckets;
    const uint64_t* seed_increment;
    uint32_t* wcodes;
    float* wmeta;
    uint64_t* n_saturated;
    float* m;
    float* v;
    float beta1, beta2, eps, weight_decay, bias1, bias2;
} qsdp_step_options;

int qsdp_fused_step_opts(float* x, const void* g, uint64_t n, float lr,
                         int wbits, int gbits, int bucket, float delta,
                         uint64_t seed, uint64_t index_offset,
                         const qsdp_step_options* opt, void* stream);
int qsdp_fused_adamw_step_opts(float* x, const void* g, uint64_t n, float lr,
                               int wbits, int gbits, int bucket, float delta,
                               uint64_t seed, uint64_t index_offset,
                               const qsdp_step_options* opt, void* stream);

int qsdp_quantize_grad_segmented(const float* g, const qsdp_segment* table, uint32_t nseg,
                                 uint64_t total_buckets, int bits, int bucket,
                                 uint64_t seed, uint64_t index_offset,
                                 uint32_t* codes, float* meta, void* stream);

int qsdp_quantize_weight_segmented(const float* x, const qsdp_segment* table, uint32_t nseg,
                                   uint64_t total_buckets, int bits, int bucket,
                                   float delta, uint64_t seed,
                                   uint32_t* codes, float* meta,
                                   uint64_t* n_saturated, void* stream);

/* (thin forward of qsdp_fused_step_opts) */
int qsdp_fused_step_segmented(float* x, const float* g, const qsdp_segment* table, uint32_t nseg,
                              uint64_t total_buckets, float lr,
                              int wbits, int gbits, int bucket, float delta,
                              uint64_t seed, uint64_t index_offset,
                              uint32_t* wcodes, float* wmeta,
                              uint64_t* n_saturated, void* stream);

/*
 * Decoding of a multi-tensor code buffer (what a worker does with a gathered set of quantized
 * layers, Algorithm 2, in one launch): tensor t's elements are decoded from the codes and meta
 * of its buckets, as qsdp_dequantize would from word first_bucket_t * bucket * bits / 32, into
 * out[offset_t .. offset_t + n_t). Padding slots are skipped. total_buckets * bucket < 2^37.
 *   out  out  device float[] or uint16[] covering every tensor's range of the flat buffer
 */
int qsdp_dequantize_segmented(const uint32_t* codes, const float* meta, const qsdp_segment* table,
                              uint32_t nseg, uint64_t total_buckets, int bits, int bucket,
                              qsdp_dtype out_dtype, void* out, void* stream);

/*
 * The receive-side steps for a partition that holds many tensors, each bucketed on its own
 * (Section 5.1): x (and m, v) are the flat buffers the segment table describes; the peers'
 * gradient codes and meta, like wcodes / wmeta, are indexed by bucket number as in the other
 * segmented calls (peer k's slot starts k * stride after gcodes / gmeta and holds
 * total_buckets * bucket code slots). Equal to qsdp_recv_step / qsdp_recv_adamw_step tensor by
 * tensor; n_saturated accumulates over all tensors. qsdp_fused_adamw_step_segmented and
 * qsdp_fused_step_codes_segmented are the multi-tensor forms of those two single-worker steps
 * (gradient uniforms follow index_offset + the position in the flat buffer, as in
 * qsdp_fused_step_segmented).
 */
/* (thin forward of qsdp_fused_adamw_step_opts) */
int qsdp_fused_adamw_step_segmented(float* x, const float* g, float* m, float* v,
                                    const qsdp_segment* table, uint32_t nseg,
                                    uint64_t total_buckets, float lr, float beta1, float beta2,
                                    float eps, float weight_decay, float bias1, float bias2,
                                    int wbits, int gbits, int bucket, float delta, uint64_t seed,
                                    uint64_t index_offset, uint32_t flags, uint32_t* wcodes,
                                    float* wmeta, uint64_t* n_saturated, void* stream);
int qsdp_fused_step_codes_segmented(uint32_t* wcodes, float* wmeta, const float* g,
                                    const qsdp_segment* table, uint32_t nseg,
                                    uint64_t total_buckets, float lr, int wbits, int gbits,
                                    int bucket, float delta, uint64_t seed, uint64_t index_offset,
                                    uint32_t flags, uint64_t* n_saturated, void* stream);
/* qsdp_fused_step_mp for many tensors in one launch (flags as in qsdp_fused_step_ex; x16, like x and g,
 * is indexed by the position in the flat buffer). */
/* (thin forward of qsdp_fused_step_opts) */
int qsdp_fused_step_segmented_mp(float* x, const void* g, qsdp_dtype g_dtype,
                                 const qsdp_segment* table, uint32_t nseg, uint64_t total_buckets,
                                 float lr, int wbits, int gbits, int bucket, float delta,
                                 uint64_t seed, uint64_t index_offset, uint32_t flags,
                                 uint32_t* wcodes, float* wmeta, void* x16, qsdp_dtype x16_dtype,
                                 uint64_t* n_saturated, void* stream);
/* The level fit of many tensors side by side (the paper fits every large layer on its own,
 * Appendix C): tensor t of the table is fitted exactly as qsdp_fit_levels would fit it alone
 * (at most max_batches of its buckets, if > 0), starting from and overwriting
 * levels[t * 2^bits .. (t+1) * 2^bits); one workgroup per tensor, all in one launch. */
int qsdp_fit_levels_segmented(const float* v, const qsdp_segment* table, uint32_t nseg, int bits,
                              int bucket, float lr, uint64_t max_batches, float* levels,
                              void* stream);
/* Learned levels with ONE TABLE PER TENSOR (Section 5.2 fits the levels of every layer, and of its
 * weights and gradients, separately; Appendix C leaves small layers on the uniform table): `levels`
 * holds nseg tables of 2^bits floats back to back, tensor t's at levels + t * 2^bits, the layout
 * qsdp_fit_levels_segmented writes. Equal, tensor by tensor, to qsdp_quantize_levels (stochastic =
 * 0) or qsdp_quantize_levels_stochastic (stochastic = 1, uniforms from index_offset + the position
 * in the flat buffer) and to qsdp_dequantize_levels with that tensor's table. */
int qsdp_quantize_levels_segmented(const float* v, const qsdp_segment* table, uint32_t nseg,
                                   uint64_t total_buckets, int bits, int bucket,
                                   const float* levels, int stochastic, uint64_t seed,
                                   uint64_t index_offset, uint32_t* codes, float* meta,
                                   void* stream);
int qsdp_dequantize_levels_segmented(const uint32_t* codes, const float* meta,
                                     const qsdp_segment* table, uint32_t nseg,
                                     uint64_t total_buckets, int bits, int bucket,
                                     const float* levels, qsdp_dtype out_dtype, void* out,
                                     void* stream);
int qsdp_recv_step_segmented(float* x, const qsdp_segment* table, uint32_t nseg,
                             uint64_t total_buckets, const uint32_t* gcodes,
                             uint64_t gcodes_stride_bytes, const float* gmeta,
                             uint64_t gmeta_stride_bytes, int npeers, float alpha, float lr,
                             int wbits, int gbits, int bucket, float delta, uint64_t seed,
                             uint32_t flags, uint32_t* wcodes, float* wmeta,
                             uint64_t* n_saturated, void* stream);
int qsdp_recv_adamw_step_segmented(float* x, float* m, float* v, const qsdp_segment* table,
                                   uint32_t nseg, uint64_t total_buckets, const uint32_t* gcodes,
                                   uint64_t gcodes_stride_bytes, const float* gmeta,
                                   uint64_t gmeta_stride_bytes, int npeers, float alpha, float lr,
                                   float beta1, float beta2, float eps, float weight_decay,
                                   float bias1, float bias2, int wbits, int gbits, int bucket,
                                   float delta, uint64_t seed, uint32_t flags, uint32_t* wcodes,
                                   float* wmeta, uint64_t* n_saturated, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* QSDP_H */
