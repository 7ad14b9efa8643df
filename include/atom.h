/*
 * atom.h -- C ABI of the MI355X (gfx950) implementation of the Atom W4A4
 * hot path (arxiv 2310.19102): fused activation front end, one-time weight
 * quantisation, and the mixed-precision group-quantised GEMM.
 *
 * Conventions common to every entry point
 *   - Every data pointer is a DEVICE pointer unless it says "host".
 *   - The caller owns every buffer.  Except where stated the library
 *     allocates nothing; the only state it keeps between calls is the
 *     one-time, per-process and per-device kernel attribute set-up (the opt-in
 *     for more than 64 KB of LDS), held in atomics: calls may come from
 *     several host threads.
 *   - Calls are asynchronous on `stream` (a hipStream_t passed as void*;
 *     NULL = the default stream).  Outputs are valid once the stream has
 *     reached the end of the call.
 *   - Nothing throws or aborts.  Every failure is a return code decided on the
 *     host before any kernel is launched (except ATOM_ERR_HIP, which reports
 *     the launch error).  M == 0 or N == 0 returns ATOM_OK without a launch.
 *   - Matrices are row-major.  fp16 = IEEE binary16.
 *   - Contents the host cannot see are not validated: a reorder index that is
 *     not a permutation of 0..K-1 (checked only `< K` by the kernels, so it
 *     cannot fault, but the result is meaningless) and non-finite inputs are
 *     the caller's responsibility.  atom_check_reorder_idx is the host guard.
 *
 * Notation (Sections 4.1-4.2): K input channels; the last O = n_outlier
 * reordered channels are the outliers kept in INT8; K4 = K - O normal channels
 * in INT4; group size Gs; G = K / Gs groups, the first G4 = K4 / Gs of them
 * INT4.  Supported: Gs = 128, O a positive multiple of 128 with O < K,
 * bits 4 / 8, K <= 32768; and bits 3 / 8, the W3A3 configuration of the
 * accuracy evaluation (Section 5.2): the normal channels are quantised with
 * n = 3 in the equations of Section 2 (s = 2 amax c / 7, codes in [-4, 3]) and
 * still travel one code per nibble, sign-extended, so the layouts below and
 * the GEMM are the same for both widths.
 *
 * Quantised layouts (what parity is judged on)
 *   q4    [rows, K4/2] bytes; byte b of a row holds reordered channel 2b in
 *         its low nibble and 2b+1 in its high nibble, two's complement
 *   q8    [rows, O]    int8, reordered channels K4 .. K-1
 *   scale [rows, G]    fp16, group g of the row; the INT8 groups come last
 */
#ifndef ATOM_H
#define ATOM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    ATOM_OK              = 0,
    ATOM_ERR_NULL        = 1,  /* a required pointer is NULL                   */
    ATOM_ERR_SHAPE       = 2,  /* negative size, ld too small, K % Gs != 0 ... */
    ATOM_ERR_UNSUPPORTED = 3,  /* a group size, bit width, K or shape the entry point does not take */
    ATOM_ERR_ALIGN       = 4,  /* a pointer or leading dimension is misaligned */
    ATOM_ERR_WORKSPACE   = 5,  /* workspace missing or too small               */
    ATOM_ERR_HIP         = 6   /* the HIP runtime refused the launch           */
} atom_status;

/* The quantisation set-up of Section 5.1: { K, 128, 128, 4, 8 }. */
typedef struct {
    int32_t K;             /* input channels of the linear layer            */
    int32_t group_size;    /* Gs, Section 4.2: 128; 64 and 256 (the variation
                              of Section 5.4.1) on the front-end entry points
                              and atom_w4a4_gemm, on plain kernels; all other
                              entry points: ATOM_ERR_UNSUPPORTED            */
    int32_t n_outlier;     /* O, Section 4.1                                */
    int32_t bits_normal;   /* 4, or 3 (W3A3, Section 5.2)                   */
    int32_t bits_outlier;  /* 8                                             */
} atom_desc;

/*
 * Fused activation front end (Section 4.3 dynamic quantisation fused into the
 * preceding operator, Section 4.1 reorder, Section 4.5 workflow):
 *   y  = gamma ? RMSNorm(x) * gamma : x            (fp32, never stored)
 *   yr[m, j] = y[m, reorder_idx[j]]
 *   per group: s = fp16(((2*max|yr|)*clip)/(2^n - 1)),  q = clamp(rne(yr/s))
 * following the symmetric equations of Section 2.
 *
 *   x_f16        [M, ldx] fp16, ldx >= K, 16-byte aligned rows (ldx % 8 == 0)
 *   gamma_f16    [K] fp16 in ORIGINAL channel order, or NULL for no norm
 *   eps          RMSNorm epsilon
 *   reorder_idx  [K] int32: output column j reads input column idx[j]; or
 *                NULL when x already is in reordered channel order (Section
 *                4.1: the reorder fused into the operator that produced x,
 *                see atom_permute_rows): same result as the identity index,
 *                without the gather.  Every front-end entry point (this one,
 *                atom_add_quantize_act, atom_swiglu_quantize_act,
 *                atom_quantize_weight, atom_decode_linear) takes NULL so.
 *   clip         clip factor c (0.9 for activations in Section 5.1)
 *   q4, q8, scale_f16   outputs in the layouts above; q4 and q8 16-byte
 *                       aligned, scale_f16 2-byte aligned
 */
atom_status atom_quantize_act(const void *x_f16, int64_t M, int64_t ldx,
                              const void *gamma_f16, float eps,
                              const int32_t *reorder_idx, const atom_desc *d,
                              float clip, void *q4, void *q8, void *scale_f16,
                              void *stream);

/*
 * The same front end behind the residual add of a transformer block (Sections
 * 4.1 and 4.3: reorder and dynamic quantisation are fused into the operator
 * before them; Section 4.5 workflow):
 *   h = fp16(x + residual)          (correctly rounded fp16 sum)
 *   sum_out_f16 = h                 (the new residual stream)
 *   then atom_quantize_act on h.
 *
 *   residual_f16 [M, ldr] fp16, ldr >= K, ldr % 8 == 0, 16-byte aligned
 *   sum_out_f16  [M, ldo] fp16, ldo >= K, ldo % 8 == 0, 16-byte aligned; may be
 *                the same buffer as x_f16 or residual_f16 (same ld), must not
 *                overlap them otherwise
 *   other arguments, alignment and errors as atom_quantize_act
 */
atom_status atom_add_quantize_act(const void *x_f16, const void *residual_f16,
                                  int64_t M, int64_t ldx, int64_t ldr,
                                  void *sum_out_f16, int64_t ldo,
                                  const void *gamma_f16, float eps,
                                  const int32_t *reorder_idx,
                                  const atom_desc *d, float clip, void *q4,
                                  void *q8, void *scale_f16, void *stream);

/*
 * The front end behind the activation function of the MLP (Sections 4.1, 4.3
 * and 4.5: the quantisation of the down projection's input is fused into the
 * operator before it, silu(gate) * up in a Llama block):
 *   y = (g * sigma(g)) * u in fp32, sigma(g) = 1 / (1 + exp(-g)), never stored,
 *   then reorder and group quantisation as in atom_quantize_act (no norm).
 * exp is evaluated by a fixed sequence of IEEE fp32 operations (round x*log2(e),
 * two-part ln2 reduction, degree-7 Taylor polynomial, exponent-field scaling,
 * argument clamped to [-87, 87]), so codes and scales have one correct value.
 *
 *   gate_f16 [M, ldg], up_f16 [M, ldu] fp16; K = d->K columns each (the
 *   intermediate size); ldg, ldu >= K and % 8 == 0, rows 16-byte aligned.  The
 *   two may be the halves of one [M, 2K] matrix (up_f16 = gate_f16 + K).
 *   other arguments, alignment and errors as atom_quantize_act
 */
atom_status atom_swiglu_quantize_act(const void *gate_f16, const void *up_f16,
                                     int64_t M, int64_t ldg, int64_t ldu,
                                     const int32_t *reorder_idx,
                                     const atom_desc *d, float clip, void *q4,
                                     void *q8, void *scale_f16, void *stream);

/*
 * One-time weight path (Section 4.1: weights are reordered offline with the
 * activations' index; Section 5.1: clip 0.85): reorder + round-to-nearest
 * group quantisation of W[N, K] (nn.Linear layout).  No norm, no GPTQ.
 * Arguments as atom_quantize_act.
 */
atom_status atom_quantize_weight(const void *w_f16, int64_t N, int64_t ldw,
                                 const int32_t *reorder_idx,
                                 const atom_desc *d, float clip, void *q4,
                                 void *q8, void *scale_f16, void *stream);

/*
 * Mixed-precision group GEMM (Section 4.2, fused GEMM operator, steps 1-3):
 *   P[m, n, g] = sum over the 128 channels of group g of aq * wq   (int32)
 *   Y[m, n]    = fp16( sum_g float(P[m, n, g]) * a_scale[m, g] * w_scale[n, g] )
 * accumulated in fp32: one fused multiply-add per group, over ascending g
 * within a contiguous run of groups.  Large launches take all of K as one run;
 * launches of few rows or few tiles split K into 2, 4 or 8 contiguous runs
 * that are added in run order.  The order depends on the shape only, so
 * results are deterministic; they differ from a single ascending chain by
 * fp32 rounding (inside 1e-3 of the result's range).  The integer sums P are
 * exact in every case.
 *
 *   a_q4 / a_q8 / a_scale   activation codes and scales for M rows
 *   w_q4 / w_q8 / w_scale   weight codes and scales for N rows
 *   y_f16         [M, ldy] fp16 out, ldy >= N
 *   partials_dbg  NULL, or [M, N, G] int32: every per-group integer sum is
 *                 also written (a slow path meant for verification)
 *   workspace     device scratch of at least
 *                 atom_w4a4_gemm_workspace_bytes(M, N, d) bytes, 256-byte
 *                 aligned; may be NULL when that size is 0
 * Code pointers must be 16-byte aligned, scale pointers 2-byte aligned.
 * ATOM_ERR_UNSUPPORTED when a code or scale array of either operand reaches
 * 4 GiB (rows * K4 / 2, rows * O or rows * G >= 2^32: the kernels use 32-bit
 * offsets) or the launch would have more than 2^31 - 1 tiles.
 */
atom_status atom_w4a4_gemm(const void *a_q4, const void *a_q8,
                           const void *a_scale, int64_t M, const void *w_q4,
                           const void *w_q8, const void *w_scale, int64_t N,
                           const atom_desc *d, void *y_f16, int64_t ldy,
                           int32_t *partials_dbg, void *workspace,
                           size_t workspace_bytes, void *stream);

/*
 * Decode-sized group GEMM (M <= 256) on weight codes re-tiled for it (Section 3:
 * at these sizes a dense layer is bound by reading its weights; Section 4.2
 * for the arithmetic).  atom_tile_weight_decode rewrites the canonical code
 * arrays once, offline, into blocks of 16 rows x one group x 64 lanes x 16
 * bytes, so that every load instruction of the kernel reads whole 128-byte
 * lines (the canonical rows, (K - O)/2 bytes long, start in the middle of
 * lines); rows past N are zeros.  Scales stay canonical.  Same arithmetic and
 * the same sum over groups as atom_w4a4_gemm at these sizes: bit-identical Y.
 *
 *   atom_tile_weight_decode_bytes(N, d, which)   size of the tiled INT4
 *                 (which = 0) or INT8 (which = 1) array: ceil(N/16)*16 rows
 *   w_q4_tiled / w_q8_tiled   16-byte aligned device arrays of those sizes
 * atom_w4a4_gemm_decode_tiled: ATOM_ERR_UNSUPPORTED unless M <= 256,
 * n_outlier = 128, K/128 even and at least 8, and the arrays stay
 * below 4 GiB; both scale arrays 8-byte aligned (ATOM_ERR_ALIGN).
 */
size_t atom_tile_weight_decode_bytes(int64_t N, const atom_desc *d, int which);
atom_status atom_tile_weight_decode(const void *w_q4, const void *w_q8, int64_t N,
                                    const atom_desc *d, void *w_q4_tiled,
                                    size_t q4_bytes, void *w_q8_tiled,
                                    size_t q8_bytes, void *stream);
atom_status atom_w4a4_gemm_decode_tiled(const void *a_q4, const void *a_q8,
                                        const void *a_scale, int64_t M,
                                        const void *w_q4_tiled,
                                        const void *w_q8_tiled,
                                        const void *w_scale, int64_t N,
                                        const atom_desc *d, void *y_f16,
                                        int64_t ldy, void *stream);

/*
 * Offline helper of the fused reorder (Section 4.1: the reorder index is known
 * after calibration, so the operator that PRODUCES an activation can emit it
 * in reordered order at no run-time cost):  out[r, :] = in[row_idx[r], :] over
 * fp16 matrices.  Applied once to the rows of the producing weight (e.g. the
 * gate and up projections, with the down projection's index: their output
 * columns, and so silu(gate) * up, then arrive reordered) or to gamma as a
 * [K, 1] matrix; the consuming front end is then called with a NULL index.
 * A GEMM with permuted weight rows computes the same values in permuted
 * columns, so the codes are those of the gathering front end bit for bit
 * (without RMSNorm; with it, the sum of squares runs over the permuted order).
 *
 *   in_f16  [rows_in, ld_in] fp16;  out_f16 [rows_out, ld_out] fp16, not in place
 *   row_idx [rows_out] int32 on the device, values in [0, rows_in) (others are
 *           clamped into the array)
 */
atom_status atom_permute_rows(const void *in_f16, int64_t rows_in, int64_t cols,
                              int64_t ld_in, const int32_t *row_idx,
                              int64_t rows_out, void *out_f16, int64_t ld_out,
                              void *stream);

/*
 * One launch for a whole linear layer at decode-sized batches (Section 3:
 * small-batch dense layers are bound by reading the weights; Sections 4.1 and
 * 4.2): the front end of atom_quantize_act (RMSNorm when gamma is given,
 * reorder, dynamic group quantisation) runs in the prologue of the
 * weight-streaming group GEMM, so the codes never travel through HBM.
 * Codes and scales are those of atom_quantize_act bit for bit; Y is that of
 * atom_w4a4_gemm on them up to the order of the fp32 sum over groups (eight
 * contiguous runs of groups, added in run order; the same tree atom_w4a4_gemm
 * uses at these sizes when its scale arrays are 8-byte aligned).
 *
 *   x_f16 [M, ldx], gamma_f16, eps, reorder_idx, clip   as atom_quantize_act
 *   w_q4 / w_q8 / w_scale   canonical weight codes and scales for N rows
 *   y_f16 [M, ldy] fp16 out, ldy >= N
 *   dbg_q4 / dbg_q8 / dbg_scale   all NULL, or device arrays as the outputs of
 *                 atom_quantize_act for M rows: the codes and scales the
 *                 kernel computed are also written (verification)
 * ATOM_ERR_UNSUPPORTED unless 1 <= M <= 16 (M = 0 is a no-op), K <= 12288,
 * 2^-20 <= clip <= 1 and atom_decode_linear_lds_bytes(M, d, norm, index) <=
 * 163840 (the codes of all M rows and, with an index, the staged row live in
 * one workgroup's LDS).  Every workgroup quantises the M rows itself, one after
 * the other (atom_decode_linear_coop does it once per launch instead).
 * Alignment as atom_quantize_act and atom_w4a4_gemm; debug arrays 4-byte.
 */
atom_status atom_decode_linear(const void *x_f16, int64_t M, int64_t ldx,
                               const void *gamma_f16, float eps,
                               const int32_t *reorder_idx, const atom_desc *d,
                               float clip, const void *w_q4, const void *w_q8,
                               const void *w_scale, int64_t N, void *y_f16,
                               int64_t ldy, void *dbg_q4, void *dbg_q8,
                               void *dbg_scale, void *stream);

/*
 * The same linear layer in one launch with the front end done once (Sections
 * 3, 4.1, 4.2, 4.5): the first M workgroups of the launch quantise one row of
 * x each into a_q4 / a_q8 / a_scale (the outputs of atom_quantize_act, bit
 * for bit) and count themselves in; all other workgroups are those of
 * atom_w4a4_gemm at this size: they request their weights, wait until M rows
 * are counted, and fetch the codes, so the front end runs while the weights
 * travel from HBM.  Y is bit-identical to atom_quantize_act followed by
 * atom_w4a4_gemm (the same kernel routine, the same sum over groups).
 *
 *   a_q4 [M, (K-O)/2], a_q8 [M, O], a_scale [M, K/Gs]   outputs (device), also
 *                 the kernel's own channel between its workgroups: each
 *                 128-byte aligned, and nothing else that the call reads may
 *                 lie in the same 128-byte lines (the consumers rely on
 *                 finding none of these lines in a cache before the rows are
 *                 counted)
 *   sync_words    atom_decode_linear_coop_sync_bytes() bytes of device memory,
 *                 128-byte aligned, that hold zeros before the first call
 *                 (hipMemset once) and are used by no other call at the same
 *                 time; a call leaves them zero again, so calls in stream
 *                 order, and replays of a captured graph, need no clearing in
 *                 between.  The second 32-bit word stays zero unless a workgroup
 *                 waited for the rows longer than 2^18 polls (it then goes on
 *                 with whatever the arrays hold; the kernel always ends):
 *                 nonzero means Y of some call was wrong, e.g. because the
 *                 words were not zero at its start.
 * ATOM_ERR_UNSUPPORTED unless 1 <= M <= 16 (M = 0 is a no-op), K <= 12288,
 * n_outlier = 128, K/128 even and at least 8, 2^-20 <= clip <= 1 and the arrays
 * below 4 GiB.  Alignment otherwise as atom_quantize_act and atom_w4a4_gemm,
 * w_scale 8-byte aligned.
 */
size_t atom_decode_linear_coop_sync_bytes(void);
atom_status atom_decode_linear_coop(const void *x_f16, int64_t M, int64_t ldx,
                                    const void *gamma_f16, float eps,
                                    const int32_t *reorder_idx,
                                    const atom_desc *d, float clip,
                                    const void *w_q4, const void *w_q8,
                                    const void *w_scale, int64_t N, void *y_f16,
                                    int64_t ldy, void *a_q4, void *a_q8,
                                    void *a_scale, void *sync_words,
                                    void *stream);

/* LDS bytes per workgroup atom_decode_linear needs (0 for a bad descriptor). */
size_t atom_decode_linear_lds_bytes(int64_t M, const atom_desc *d, int with_norm,
                                    int with_index);

/* Scratch the GEMM needs for these sizes (0 when it needs none). */
size_t atom_w4a4_gemm_workspace_bytes(int64_t M, int64_t N,
                                      const atom_desc *d);

/*
 * The same GEMM on weights in an opaque tiled layout (Section 4.1: the weights
 * are prepared once, offline; Section 4.2 for the arithmetic, which is that of
 * atom_w4a4_gemm).  atom_pack_weight turns canonical (w_q4, w_q8, w_scale) into
 * the layout the compute-bound kernel streams without any address arithmetic:
 * tiles of 64 rows, group by group, every INT4 code re-encoded as the FP6
 * (E3M2) number of the same integer value -- every integer in [-8, 8] is one,
 * so nothing is re-quantised -- which lets the group sums run on the FP6
 * matrix instruction at twice the INT8 rate; its fp32 accumulation of these
 * integers is exact, so P[m, n, g] is the same integer as above.  INT8 groups
 * and scales are carried as they are.  The packed bytes are a bijection of the
 * canonical arrays (plus zero rows up to a multiple of 64); the canonical
 * layouts stay what parity is judged on.
 *
 *   atom_pack_weight_bytes(N, d)   size of the packed buffer (0 on bad d or N)
 *   w_packed      device, 256-byte aligned, packed_bytes >= that size
 * atom_w4a4_gemm_packed: activations canonical as atom_quantize_act writes
 * them; they are re-tiled into `workspace` first (one extra launch), which must
 * hold atom_w4a4_gemm_packed_workspace_bytes(M, N, d) bytes, 256-byte aligned.
 * Y is accumulated over ascending g in one chain of fused multiply-adds, the
 * INT8 groups last: the definition's order.  partials_dbg as in atom_w4a4_gemm.
 * Any M is accepted; the kernel is meant for M > 64.
 * Errors: as atom_w4a4_gemm, and ATOM_ERR_UNSUPPORTED beyond 65535 * 64 rows
 * of either operand; ATOM_ERR_WORKSPACE when w_packed or workspace is too small.
 */
size_t atom_pack_weight_bytes(int64_t N, const atom_desc *d);
atom_status atom_pack_weight(const void *w_q4, const void *w_q8,
                             const void *w_scale, int64_t N, const atom_desc *d,
                             void *w_packed, size_t packed_bytes, void *stream);
size_t atom_w4a4_gemm_packed_workspace_bytes(int64_t M, int64_t N,
                                             const atom_desc *d);
/*
 * The two halves of atom_w4a4_gemm_packed as calls of their own, for a caller
 * that keeps the tiled activations (several GEMMs on one input: Q, K and V),
 * or wants to time the stages apart: atom_pack_act re-tiles the canonical
 * activation arrays of M rows into a_packed (atom_pack_weight_bytes(M, d)
 * bytes, 256-byte aligned; the same layout as the weights'), and
 * atom_w4a4_gemm_prepacked is the GEMM on two tiled operands.  Errors as
 * atom_pack_weight / atom_w4a4_gemm_packed.
 */
atom_status atom_pack_act(const void *a_q4, const void *a_q8,
                          const void *a_scale, int64_t M, const atom_desc *d,
                          void *a_packed, size_t packed_bytes, void *stream);
atom_status atom_w4a4_gemm_prepacked(const void *a_packed, int64_t M,
                                     const void *w_packed, int64_t N,
                                     const atom_desc *d, void *y_f16,
                                     int64_t ldy, int32_t *partials_dbg,
                                     void *stream);
atom_status atom_w4a4_gemm_packed(const void *a_q4, const void *a_q8,
                                  const void *a_scale, int64_t M,
                                  const void *w_packed, int64_t N,
                                  const atom_desc *d, void *y_f16, int64_t ldy,
                                  int32_t *partials_dbg, void *workspace,
                                  size_t workspace_bytes, void *stream);

/*
 * The front ends writing the tiled activations directly (Sections 4.1 - 4.3:
 * everything between the producing operator and the GEMM in one kernel): the
 * result in a_packed is byte for byte what atom_quantize_act (or
 * atom_add_quantize_act, atom_swiglu_quantize_act) followed by atom_pack_act
 * leaves there, without the canonical arrays and without the re-tiling pass;
 * atom_w4a4_gemm_prepacked takes it.  Arguments as the canonical entry points
 * (reorder_idx may be NULL likewise); a_packed: atom_pack_weight_bytes(M, d)
 * bytes, 256-byte aligned.
 * ATOM_ERR_UNSUPPORTED unless group_size = 128, 2^-20 <= clip <= 1 and the
 * row's staging fits the LDS (4 K bytes with an index, K / 2 with RMSNorm,
 * 3 (K - O) / 4 + O for the packed row: K <= 28672 with an index and RMSNorm,
 * every K without an index); ATOM_ERR_WORKSPACE when packed_bytes is too small.
 */
atom_status atom_quantize_act_packed(const void *x_f16, int64_t M, int64_t ldx,
                                     const void *gamma_f16, float eps,
                                     const int32_t *reorder_idx,
                                     const atom_desc *d, float clip,
                                     void *a_packed, size_t packed_bytes,
                                     void *stream);
atom_status atom_add_quantize_act_packed(const void *x_f16, const void *residual_f16,
                                         int64_t M, int64_t ldx, int64_t ldr,
                                         void *sum_out_f16, int64_t ldo,
                                         const void *gamma_f16, float eps,
                                         const int32_t *reorder_idx,
                                         const atom_desc *d, float clip,
                                         void *a_packed, size_t packed_bytes,
                                         void *stream);
atom_status atom_swiglu_quantize_act_packed(const void *gate_f16, const void *up_f16,
                                            int64_t M, int64_t ldg, int64_t ldu,
                                            const int32_t *reorder_idx,
                                            const atom_desc *d, float clip,
                                            void *a_packed, size_t packed_bytes,
                                            void *stream);

/*
 * KV-cache quantisation (Section 2, asymmetric uniform quantisation; Section
 * 4.4: one scale and zero point per attention head, 4 bits; Section 4.5: fused
 * into the operator that produces K and V, here a kernel of its own that the
 * producer's epilogue calls on its output rows).  Row r holds the D values of
 * one head of one token:
 *   s    = fp16( ((max - min) * clip) / 15 )   IEEE fp32, round to nearest even,
 *                                              saturated at 65504
 *   z    = rne(-min / s) clamped to int16       (IEEE fp32 division by the stored s)
 *   code = clamp(rne(x / s) + z, 0, 15)         dequantised value (code - z) * s
 * A row with s == 0 (constant row, or a range below fp16's smallest value)
 * stores codes 0 and z = 0.  Results are bit-exact.
 *
 *   x_f16     [R, ldx] fp16, device; ldx >= D, ldx % 8 == 0, 16-byte aligned
 *   D         64 or 128
 *   clip      the clipping factor c of Section 4.2 applied to the range (1 = none)
 *   pos       NULL: row r is written to row r of the outputs (prefill: a whole
 *             cache at once).  Otherwise device int32 [R / rows_per_seq]: row r
 *             is written to row r * Tmax + pos[r / rows_per_seq] (decode: the new
 *             token of every sequence, rows ordered (sequence, head), appended
 *             in place to a cache laid out [B, Hkv, Tmax]; rows_per_seq = Hkv).
 *             A position outside [0, Tmax) writes nothing.
 *   q         [rows, D/2] bytes, two codes per byte, even d in the low nibble;
 *             4-byte aligned.  scale_f16 [rows] fp16, zero_i16 [rows] int16.
 * Errors: ATOM_ERR_NULL, ATOM_ERR_SHAPE (R < 0, ldx < D, with pos:
 * rows_per_seq <= 0, R % rows_per_seq != 0 or Tmax <= 0), ATOM_ERR_UNSUPPORTED
 * (D), ATOM_ERR_ALIGN.  R == 0 returns ATOM_OK without a launch.
 */
atom_status atom_kv_quantize(const void *x_f16, int64_t R, int64_t ldx,
                             int32_t D, float clip, const int32_t *pos,
                             int32_t rows_per_seq, int64_t Tmax, void *q,
                             void *scale_f16, void *zero_i16, void *stream);

/*
 * The K rows and the V rows of one step in one launch (Section 4.5: the
 * quantisation of K and V sits behind the one operator that produces both):
 * exactly atom_kv_quantize(k_f16, ..., k_q, k_scale, k_zero) followed by
 * atom_kv_quantize(v_f16, ..., v_q, v_scale, v_zero), with R, ldx, D, clip,
 * pos, rows_per_seq and Tmax shared.  Arguments, layouts, results and errors
 * as there, for either tensor; the six outputs must not overlap.
 */
atom_status atom_kv_quantize_pair(const void *k_f16, const void *v_f16, int64_t R,
                                  int64_t ldx, int32_t D, float clip,
                                  const int32_t *pos, int32_t rows_per_seq,
                                  int64_t Tmax, void *k_q, void *k_scale_f16,
                                  void *k_zero_i16, void *v_q, void *v_scale_f16,
                                  void *v_zero_i16, void *stream);

/*
 * Decode-stage self-attention of one new token per sequence over the INT4 KV
 * cache (Section 4.4: the cache is loaded in 4 bits and dequantised inside the
 * attention operator, whose arithmetic stays in floating point; Section 4.5):
 *   K[t, :] = (k_codes[t, :] - k_zero[t]) * k_scale[t], V likewise
 *   out[b, h, :] = softmax_t( sm_scale * q[b, h, :] . K[b, kv(h), t, :] ) V[b, kv(h)]
 * over t < seq_len[b]; kv(h) = h / (H / Hkv) (grouped-query attention when
 * Hkv < H).  fp32 arithmetic, fp16 output; seq_len[b] == 0 gives zeros.
 * With 2 to 16 query heads per cache head the two contractions run on the
 * fp16 matrix cores with fp32 accumulation (the codes are exact in fp16, the
 * softmax weights travel as fp16 hi + lo, 22 bits); the results agree with
 * the fp32 path within the 1e-3 the tests allow.
 *
 *   q_f16    [B, H, D] fp16, device, 16-byte aligned; D = 128
 *   seq_len  device int32 [B]; values are clamped to [0, Tmax] by the kernel
 *   k_codes, v_codes [B, Hkv, Tmax, D/2] bytes (16-byte aligned);
 *   k_scale, v_scale [B, Hkv, Tmax] fp16; k_zero, v_zero [B, Hkv, Tmax] int16,
 *   as atom_kv_quantize writes them
 *   out_f16  [B, H, D] fp16
 *   workspace  device scratch of at least
 *            atom_decode_attention_kv4_workspace_bytes(B, H, Hkv, D, Tmax) bytes, 16-byte
 *            aligned (may be NULL when that is 0): when B * H alone cannot fill
 *            the GPU the token range is split over several workgroups whose
 *            partial (max, sum, accumulator) triples meet in a second kernel.
 *            Contents need no initialisation and are dead after the call.
 * Errors: ATOM_ERR_NULL, ATOM_ERR_SHAPE (negative sizes, H % Hkv != 0),
 * ATOM_ERR_UNSUPPORTED (D != 128, Tmax > 2^25), ATOM_ERR_ALIGN, ATOM_ERR_WORKSPACE.
 * B == 0 returns ATOM_OK.
 */
atom_status atom_decode_attention_kv4(const void *q_f16, int32_t B, int32_t H,
                                      int32_t Hkv, int32_t D, int64_t Tmax,
                                      const int32_t *seq_len,
                                      const void *k_codes, const void *k_scale,
                                      const void *k_zero, const void *v_codes,
                                      const void *v_scale, const void *v_zero,
                                      float sm_scale, void *out_f16,
                                      void *workspace, size_t workspace_bytes,
                                      void *stream);

/*
 * atom_decode_attention_kv4 for callers that cannot allocate device memory and
 * have no workspace to hand over (code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc): the same kernels, with the partials
 * of a split launch in a scratch array of atom_static_scratch_bytes() = 4 MiB
 * that is part of the library's device image (each GPU the library runs on
 * holds its own copy until the process ends).  The call allocates nothing; the
 * array's address is looked up on the first call on a device.  Arguments,
 * results and errors as atom_decode_attention_kv4 without the workspace; sizes
 * whose partials exceed the array return ATOM_ERR_WORKSPACE
 * (atom_decode_attention_kv4_workspace_bytes tells).  The scratch needs no
 * initialisation and is dead after the call, but every call on a GPU uses the
 * same array: calls that may overlap on one GPU (different streams) race.
 */
atom_status atom_decode_attention_kv4_static(const void *q_f16, int32_t B,
                                             int32_t H, int32_t Hkv, int32_t D,
                                             int64_t Tmax, const int32_t *seq_len,
                                             const void *k_codes,
                                             const void *k_scale,
                                             const void *k_zero,
                                             const void *v_codes,
                                             const void *v_scale,
                                             const void *v_zero, float sm_scale,
                                             void *out_f16, void *stream);
size_t atom_static_scratch_bytes(void);

/* Scratch atom_decode_attention_kv4 needs for these sizes (0 when none). */
size_t atom_decode_attention_kv4_workspace_bytes(int32_t B, int32_t H,
                                                 int32_t Hkv, int32_t D,
                                                 int64_t Tmax);

/*
 * MX variant of the path.  The paper also runs its recipe with FP4 codes and
 * names the MX formats, whose group scaling new hardware applies by itself and
 * which it expects to remove the group-dequantisation overhead of the fused
 * GEMM (Section 5.2, FP4 paragraph; overhead: Section 5.4.2).  On gfx950 that
 * hardware is the scaled FP8/FP6/FP4 MFMA.  Reading taken here: reorder and
 * mixed precision stay as they are; a block of 32 reordered channels shares one
 * power-of-two scale (E8M0 byte, 2^(byte - 127)); the K4 = K - O normal
 * channels are FP4 E2M1 (magnitudes 0 .5 1 1.5 2 3 4 6, sign in bit 3), the O
 * outlier channels FP8 E4M3 (bias 7, largest 448, no infinity):
 *   byte = clamp(floor(log2(amax * clip)) - emax, -127, 127) + 127, emax = 2
 *          (E2M1) or 8 (E4M3); an all-zero block gives byte 0
 *   code = nearest representable of y / 2^(byte - 127), ties to the even
 *          mantissa, larger magnitudes saturate
 * Results are bit-exact.  d->group_size must be 32, bits 4 / 8; K and O
 * multiples of 128, 0 < O < K, K <= 32768.
 *
 *   x_f16, gamma_f16, eps, reorder_idx, clip: as atom_quantize_act
 * Layout (step-major, so that the GEMM streams whole cache lines): with M the
 * number of rows of the call,
 *   q4 [K4/128, M, 64] bytes: 128 reordered channels of a row per 64 bytes, two
 *      FP4 codes per byte, even channel in the low nibble
 *   q8 [O/64, M, 64] bytes: 64 outlier channels of a row, one FP8 code each
 *   e8 [K/128, M, 4] bytes: the four scale bytes of 128 channels of a row, FP4
 *      blocks first
 *   (q4, q8 16-byte aligned, e8 4-byte aligned).  The arrays of one call belong
 *   to that call's M rows as a whole; a GEMM takes them as produced.
 * Errors as atom_quantize_act.
 */
atom_status atom_mx_quantize_act(const void *x_f16, int64_t M, int64_t ldx,
                                 const void *gamma_f16, float eps,
                                 const int32_t *reorder_idx, const atom_desc *d,
                                 float clip, void *q4, void *q8, void *e8,
                                 void *stream);

/* Weights of the MX variant: reorder + quantisation of W[N, K], no norm. */
atom_status atom_mx_quantize_weight(const void *w_f16, int64_t N, int64_t ldw,
                                    const int32_t *reorder_idx,
                                    const atom_desc *d, float clip, void *q4,
                                    void *q8, void *e8, void *stream);

/*
 * GEMM of the MX variant:
 *   Y[m, n] = fp16( sum_b 2^(ea[m,b] + ew[n,b] - 254) * sum_{k in block b} a[m,k] * w[n,k] )
 * over all K/32 blocks, the block scaling applied by the matrix instruction
 * itself, fp32 accumulation inside it (the order of its additions is the
 * hardware's; the result is within the library's 1e-3 tolerance of the exact
 * sum).  Operands as atom_mx_quantize_act / _weight produce them; Y [M, ldy]
 * fp16, ldy >= N.  No workspace.
 * Errors: ATOM_ERR_NULL, ATOM_ERR_SHAPE, ATOM_ERR_UNSUPPORTED, ATOM_ERR_ALIGN.
 */
atom_status atom_mx_gemm(const void *a_q4, const void *a_q8, const void *a_e8,
                         int64_t M, const void *w_q4, const void *w_q8,
                         const void *w_e8, int64_t N, const atom_desc *d,
                         void *y_f16, int64_t ldy, void *stream);

/*
 * Offline calibration (Section 5.1: the channels with the highest square sums
 * over the calibration activations are the outliers; activations and weights
 * are reordered by their indices).  From calibration activations X [T, ldx]
 * fp16 (device; T rows of K channels, e.g. the inputs a layer saw on the
 * calibration sentences):
 *   stat[k] = sum_t X[t, k]^2, exact: every square is a multiple of 2^-48
 *             below 2^32, so the sum is an integer of at most 112 bits in any
 *             order of the additions; reported as the nearest double (ties to
 *             even); Inf and NaN count as magnitude 2^16
 *   idx     = the channels in ascending order of (exact stat, channel number): a
 *             permutation whose last O entries are the O channels with the
 *             highest square sums, for every O; equal channels keep their order
 * idx is what atom_quantize_act / atom_quantize_weight (and the MX variants)
 * take as reorder_idx.  Results are bit-exact.  T == 0 gives the identity.
 *
 *   workspace  device scratch of atom_calibrate_reorder_workspace_bytes(T, K)
 *              bytes, 16-byte aligned; its last K doubles hold stat afterwards
 *   idx_out    device int32 [K]
 * Errors: ATOM_ERR_NULL, ATOM_ERR_SHAPE (T < 0, K <= 0, ldx < K),
 * ATOM_ERR_UNSUPPORTED (K > 32768), ATOM_ERR_ALIGN, ATOM_ERR_WORKSPACE.
 */
atom_status atom_calibrate_reorder(const void *x_f16, int64_t T, int64_t ldx,
                                   int32_t K, void *workspace,
                                   size_t workspace_bytes, int32_t *idx_out,
                                   void *stream);
size_t atom_calibrate_reorder_workspace_bytes(int64_t T, int32_t K);

/*
 * Measurement helper, not a step of the method (the roofline of Section 3 is
 * priced against the matrix units' peak; this quotes what the device sustains):
 * launches a kernel that issues nothing but independent matrix instructions,
 * 4 * iters per wavefront on 4096 wavefronts -- kind 0: INT8 32x32x32 (the
 * canonical GEMM kernels and the outlier group), kind 1: FP6 32x32x64 (the
 * INT4 groups of the packed GEMM) -- and returns the number of integer /
 * floating-point operations of the launch (2 per multiply-add); time the
 * launch on `stream` and divide.  scratch4: 4 writable device bytes.  *status
 * (may be NULL) receives ATOM_ERR_SHAPE (kind, iters <= 0), ATOM_ERR_NULL,
 * ATOM_ERR_ALIGN or ATOM_ERR_HIP, and the return value is then 0.
 */
double atom_mfma_rate_probe(int32_t kind, int32_t iters, void *scratch4,
                            void *stream, atom_status *status);

/* Host helper: ATOM_OK iff idx_host[0..K) is a permutation of 0..K-1. */
atom_status atom_check_reorder_idx(const int32_t *idx_host, int32_t K);

/* Static, NUL-terminated description of a status code. */
const char *atom_status_string(int status);   /* any int: values that are no atom_status give "unknown status" */

#ifdef __cplusplus
}
#endif
#endif
