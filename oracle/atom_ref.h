/*
 * atom_ref.h -- CPU oracle for the Atom W4A4 hot path (arxiv 2310.19102).
 *
 * TEST INFRASTRUCTURE ONLY.  This is a plain, slow, single-threaded C
 * implementation of what the GPU library computes.  It shares no code with
 * the HIP path and nothing in the product may call it: only the tests, the
 * smoke check and the benchmark's CPU-baseline leg do.
 *
 * Every function takes HOST pointers.  Matrices are row-major.  fp16 values
 * travel as raw uint16_t bit patterns (IEEE binary16).
 *
 * Notation (Section 4.1-4.2 of the paper): K input channels, O outlier
 * channels kept in INT8 and placed last by the reorder index, K4 = K - O
 * normal channels in INT4, group size Gs (128 in the paper), G = K / Gs
 * groups of which the first G4 = K4 / Gs are INT4 and the rest INT8.
 *
 * Arithmetic contract (the readings of the paper taken here):
 *   - symmetric quantisation, Section 2:  s = 2*max|X| / (2^n - 1) * c,
 *     Xq = clamp(round(X / s), -2^(n-1), 2^(n-1) - 1); evaluated in fp32 as
 *     ((2*amax)*c)/(2^n-1); "round" is round-half-to-even; the scale is then
 *     rounded to fp16 (the 16-bit scale per group of the effective-bit
 *     footnote in Section 4.2, saturated at 65504) and the codes are produced
 *     by an IEEE fp32 division by that STORED scale.  A zero scale gives zero
 *     codes.
 *   - RMSNorm in fp32 (Section 4.5 fuses the layer norm of Llama into the
 *     quantisation operator); the sum of squares follows one fixed tree
 *     (see atom_ref_sumsq) so that it has exactly one correct value.
 *   - GEMM, Section 4.2 steps 1-3: per group an exact int32 partial, then
 *     acc = fma(float(P), float(sa)*float(sw), acc) over ascending groups in
 *     fp32, result rounded to fp16.
 */
#ifndef ATOM_REF_H
#define ATOM_REF_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* IEEE binary16 <-> binary32, round-half-to-even on narrowing. */
float    atom_ref_f16_to_f32(uint16_t h);
uint16_t atom_ref_f32_to_f16(float f);

/* Sum of squares of one row of K fp16 values by the canonical tree:
 * vectors of 8 consecutive channels are squared and added pairwise
 * ((0+1)+(2+3))+((4+5)+(6+7)); vector v goes to accumulator v mod 64 in
 * increasing v; the 64 accumulators are folded with strides 1,2,4,...,32. */
float atom_ref_sumsq(const uint16_t *x_f16, int32_t K);

/* One row of RMSNorm (Section 4.5): r = 1/sqrt(S/K + eps),
 * y[k] = (x[k]*r)*gamma[k], all fp32.  gamma == NULL means y = x. */
void atom_ref_rmsnorm_row(const uint16_t *x_f16, const uint16_t *gamma_f16,
                          float eps, int32_t K, float *y_out);

/* Fused front end (Sections 4.1-4.3): optional RMSNorm, reorder
 * yr[j] = y[idx[j]], per-group symmetric quantisation.
 *   x_f16   [M, ldx]  fp16, K valid columns
 *   gamma   [K] fp16 in ORIGINAL channel order, or NULL (no norm)
 *   idx     [K] permutation; the last O entries are the outlier channels
 *   q4      [M, K4/2] bytes: low nibble = even column, high nibble = odd
 *   q8      [M, O]    int8
 *   scale   [M, G]    fp16
 * Returns 0, or -1 on bad shapes. */
int atom_ref_quantize_act(const uint16_t *x_f16, int64_t M, int64_t ldx,
                          const uint16_t *gamma_f16, float eps,
                          const int32_t *idx, int32_t K, int32_t Gs, int32_t O,
                          float clip, uint8_t *q4, int8_t *q8, uint16_t *scale);

/* The same front end behind a residual add (Sections 4.1 and 4.3 fuse the
 * reorder and the dynamic quantisation into the operator before them; in a
 * Llama block the operator before the norm is the residual add):
 *   h = fp16(x + res)  (sum formed in fp32, rounded once to fp16),
 *   sum_out [M, ldo] = h  (the new residual stream; may alias x or res),
 *   then atom_ref_quantize_act on h. */
int atom_ref_add_quantize_act(const uint16_t *x_f16, const uint16_t *res_f16,
                              int64_t M, int64_t ldx, int64_t ldr,
                              uint16_t *sum_out_f16, int64_t ldo,
                              const uint16_t *gamma_f16, float eps,
                              const int32_t *idx, int32_t K, int32_t Gs,
                              int32_t O, float clip, uint8_t *q4, int8_t *q8,
                              uint16_t *scale);

/* The front end behind the activation function of the MLP (Sections 4.1, 4.3
 * and 4.5: the quantisation of the down projection's input is fused into the
 * operator before it, which in a Llama block is silu(gate) * up):
 *   y = (g * sigma(g)) * u in fp32, sigma(g) = 1/(1 + exp(-g)), never stored,
 *   then reorder and group quantisation as in atom_ref_quantize_act (no norm).
 * exp is the fixed sequence of IEEE operations of atom_ref_expf, so y has one
 * correct value.  gate [M, ldg], up [M, ldu] fp16. */
float atom_ref_expf(float x);
float atom_ref_silu_mul(uint16_t gate_f16, uint16_t up_f16);
int atom_ref_swiglu_quantize_act(const uint16_t *gate_f16, const uint16_t *up_f16,
                                 int64_t M, int64_t ldg, int64_t ldu,
                                 const int32_t *idx, int32_t K, int32_t Gs,
                                 int32_t O, float clip, uint8_t *q4, int8_t *q8,
                                 uint16_t *scale);

/* Offline weight path (Section 4.1 reorder, Section 5.1 clip): same as the
 * front end without the norm; round-to-nearest only (no GPTQ). */
int atom_ref_quantize_weight(const uint16_t *w_f16, int64_t N, int64_t ldw,
                             const int32_t *idx, int32_t K, int32_t Gs,
                             int32_t O, float clip, uint8_t *q4, int8_t *q8,
                             uint16_t *scale);

/* Mixed-precision group GEMM (Section 4.2, Figure "fused GEMM operator").
 *   y_f16     [M, ldy] fp16 out
 *   partials  NULL or [M, N, G] int32 (per-group integer sums)
 *   acc_f32   NULL or [M, N] fp32 accumulators before the fp16 rounding */
int atom_ref_w4a4_gemm(const uint8_t *a_q4, const int8_t *a_q8,
                       const uint16_t *a_scale, int64_t M,
                       const uint8_t *w_q4, const int8_t *w_q8,
                       const uint16_t *w_scale, int64_t N,
                       int32_t K, int32_t Gs, int32_t O,
                       uint16_t *y_f16, int64_t ldy,
                       int32_t *partials, float *acc_f32);

/* The same four with the width n of the normal channels as a parameter: 4, or 3
 * for the W3A3 configuration of the accuracy evaluation (Section 5.2).  Section
 * 2's equations with n = 3: s = 2*amax*c / 7, codes clamped to [-4, 3]; the
 * codes still travel sign-extended in 4-bit containers (same q4 layout), the
 * outlier channels stay at 8 bits, and the GEMM is unchanged. */
int atom_ref_quantize_act_n(const uint16_t *x_f16, int64_t M, int64_t ldx,
                            const uint16_t *gamma_f16, float eps,
                            const int32_t *idx, int32_t K, int32_t Gs, int32_t O,
                            int32_t bits, float clip, uint8_t *q4, int8_t *q8,
                            uint16_t *scale);
int atom_ref_add_quantize_act_n(const uint16_t *x_f16, const uint16_t *res_f16,
                                int64_t M, int64_t ldx, int64_t ldr,
                                uint16_t *sum_out_f16, int64_t ldo,
                                const uint16_t *gamma_f16, float eps,
                                const int32_t *idx, int32_t K, int32_t Gs,
                                int32_t O, int32_t bits, float clip, uint8_t *q4,
                                int8_t *q8, uint16_t *scale);
int atom_ref_swiglu_quantize_act_n(const uint16_t *gate_f16, const uint16_t *up_f16,
                                   int64_t M, int64_t ldg, int64_t ldu,
                                   const int32_t *idx, int32_t K, int32_t Gs,
                                   int32_t O, int32_t bits, float clip, uint8_t *q4,
                                   int8_t *q8, uint16_t *scale);

/* ---- INT4 KV cache (Section 4.4; asymmetric equations of Section 2) ---------
 * One row = the D values of one token of one attention head (the paper's
 * granularity), n = 4 bits:
 *   s = fp16(((max - min) * clip) / 15)  (stored, saturated at 65504),
 *   z = clamp(round(-min / s), -32768, 32767)  (stored, int16),
 *   code = clamp(round(x / s) + z, 0, 15), round = half to even, IEEE fp32
 *   division by the STORED scale; s == 0 (constant row) gives z = 0, codes 0.
 * Codes are packed two per byte, even d in the low nibble.
 * Dequantisation: (code - z) * s in fp32. */
int atom_ref_kv_quantize(const uint16_t *x_f16, int64_t R, int64_t ldx, int32_t D,
                         float clip, uint8_t *q /* [R, D/2] */,
                         uint16_t *scale_f16 /* [R] */, int16_t *zero /* [R] */);
float atom_ref_kv_dequant(uint8_t code, uint16_t scale_f16, int16_t zero);

/* Decode-stage attention over the INT4 cache (Sections 4.4 and 4.5: the cache is
 * loaded in low precision and dequantised inside the attention operator).
 *   q        [B, H, D] fp16, one query token per sequence
 *   kq, vq   [B, Hkv, Tmax, D/2] codes; ks, vs [B, Hkv, Tmax] fp16 scales;
 *            kz, vz [B, Hkv, Tmax] int16 zero points; query head h reads
 *            cache head h / (H / Hkv)
 *   seq_len  [B] tokens in the cache of each sequence (<= Tmax)
 *   out[b,h,:] = fp16( sum_t softmax_t(sm_scale * q . k_t) * v_t ), all sums in
 *   double; an empty cache gives zeros. */
int atom_ref_decode_attention_kv4(const uint16_t *q_f16, int32_t B, int32_t H,
                                  int32_t Hkv, int32_t D, int32_t Tmax,
                                  const int32_t *seq_len, const uint8_t *kq,
                                  const uint16_t *ks, const int16_t *kz,
                                  const uint8_t *vq, const uint16_t *vs,
                                  const int16_t *vz, float sm_scale,
                                  uint16_t *out_f16);

/* ---- MX (microscaling) variant of the path.  The paper evaluates its recipe
 * with FP4 codes and names the MX formats, whose group scaling is applied by
 * the hardware (last paragraph of the accuracy evaluation, Section 5.2).  The
 * reading taken: the reorder and the mixed precision stay; a block of 32
 * reordered channels shares one power-of-two scale (E8M0 byte, 2^(byte-127));
 * normal channels are FP4 E2M1 (magnitudes 0 .5 1 1.5 2 3 4 6, sign in bit 3),
 * the O outlier channels FP8 E4M3 (bias 7, no infinity, largest 448), as the
 * MX specification the paper cites defines them:
 *   byte  = clamp(floor(log2(amax * clip)) - emax, -127, 127) + 127,
 *           emax = 2 (E2M1) or 8 (E4M3); an all-zero block gives byte 0
 *   code  = nearest representable of y / 2^(byte-127), ties to the even
 *           mantissa, magnitudes beyond the largest saturate to it
 * Layout: q4 [rows, K4/2] two codes per byte, even channel in the low nibble;
 * q8 [rows, O] bytes; e8 [rows, K/32] bytes, FP4 blocks first.
 * GEMM: Y[m,n] = fp16( sum_b 2^(ea[m,b]+ew[n,b]-254) * sum_{k in b} a*w ), all
 * sums in double. */
float   atom_ref_e2m1_to_f32(uint8_t code);
float   atom_ref_e4m3_to_f32(uint8_t code);
uint8_t atom_ref_f32_to_e2m1(float v);
uint8_t atom_ref_f32_to_e4m3(float v);
uint8_t atom_ref_mx_scale_byte(float clipped_amax, int emax);
/* gamma == NULL: no norm (weights, or activations behind an activation function) */
int atom_ref_mx_quantize_act(const uint16_t *x_f16, int64_t M, int64_t ldx,
                             const uint16_t *gamma_f16, float eps,
                             const int32_t *idx, int32_t K, int32_t O, float clip,
                             uint8_t *q4, uint8_t *q8, uint8_t *e8);
int atom_ref_mx_gemm(const uint8_t *a_q4, const uint8_t *a_q8, const uint8_t *a_e8,
                     int64_t M, const uint8_t *w_q4, const uint8_t *w_q8,
                     const uint8_t *w_e8, int64_t N, int32_t K, int32_t O,
                     uint16_t *y_f16, int64_t ldy);

/* ---- Offline calibration (Section 5.1): per-channel square sum of the
 * calibration activations x [T, ldx] fp16, exact (an integer count of 2^-48,
 * independent of the order of the additions; reported as the nearest double),
 * and the reorder index: channels in ascending order of (exact square sum,
 * channel number), so that the O channels with the highest square sums come
 * last. */
int atom_ref_calibrate_reorder(const uint16_t *x_f16, int64_t T, int64_t ldx, int32_t K,
                               double *stat /* [K] */, int32_t *idx /* [K] */);

#ifdef __cplusplus
}
#endif
#endif
