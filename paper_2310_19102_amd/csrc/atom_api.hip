// C-ABI shim: argument validation on the host, then one kernel launch per call.
// Nothing here allocates, synchronises or keeps state.

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <new>

#include "atom.h"
#include "atom_internal.h"

namespace {

inline bool aligned(const void *p, uintptr_t a)
{
    return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0;
}

// other_groups: the entry point also takes the group sizes 64 and 256 (the front ends and
// atom_w4a4_gemm); everything else is built around the group of 128
atom_status check_desc(const atom_desc *d, bool other_groups = false)
{
    if (!d) return ATOM_ERR_NULL;
    if (d->K <= 0 || d->group_size <= 0 || d->n_outlier < 0) return ATOM_ERR_SHAPE;
    const bool gs_ok = d->group_size == atom_internal::kGroup ||
                       (other_groups && (d->group_size == 64 || d->group_size == 256));
    if (!gs_ok || (d->bits_normal != 4 && d->bits_normal != 3) || d->bits_outlier != 8)
        return ATOM_ERR_UNSUPPORTED;
    if (d->K % d->group_size || d->n_outlier % d->group_size) return ATOM_ERR_SHAPE;
    if (d->n_outlier >= d->K) return ATOM_ERR_SHAPE;
    if (d->n_outlier == 0) return ATOM_ERR_UNSUPPORTED;
    if (d->K > atom_internal::kMaxK) return ATOM_ERR_UNSUPPORTED;
    return ATOM_OK;
}

atom_status quantize_common(const void *x, int64_t rows, int64_t ld, int pre, const void *res,
                            int64_t ldr, void *sum_out, int64_t ldo, const void *gamma, float eps,
                            const int32_t *idx, const atom_desc *d, float clip, void *q4,
                            void *q8, void *scale, void *stream)
{
    atom_status st = check_desc(d, true);
    if (st != ATOM_OK) return st;
    if (rows < 0 || ld < d->K) return ATOM_ERR_SHAPE;
    if (pre != 0 && ldr < d->K) return ATOM_ERR_SHAPE;
    if (pre == 1 && ldo < d->K) return ATOM_ERR_SHAPE;
    if (rows == 0) return ATOM_OK;
    if (!x || !q4 || !q8 || !scale) return ATOM_ERR_NULL;     // idx may be null: identity order
    if (pre != 0 && !res) return ATOM_ERR_NULL;
    if (pre == 1 && !sum_out) return ATOM_ERR_NULL;
    if (!aligned(x, 16) || (ld % 8) || !aligned(idx, 16) || !aligned(q4, 16) || !aligned(q8, 16) ||
        !aligned(scale, 2) || (gamma && !aligned(gamma, 16)))
        return ATOM_ERR_ALIGN;
    if (pre != 0 && (!aligned(res, 16) || (ldr % 8))) return ATOM_ERR_ALIGN;
    if (pre == 1 && (!aligned(sum_out, 16) || (ldo % 8))) return ATOM_ERR_ALIGN;
    hipError_t err = atom_internal::launch_quantize_rows(x, rows, ld, pre, res, ldr, sum_out, ldo,
                                                         gamma, eps, idx, d->K, d->n_outlier,
                                                         d->bits_normal, clip,
                                                         q4, q8, scale,
                                                         static_cast<hipStream_t>(stream), d->group_size);
    return err == hipSuccess ? ATOM_OK : ATOM_ERR_HIP;
}

atom_status quantize_packed_common(const void *x, int64_t rows, int64_t ld, int pre, const void *res, int64_t ldr,
                                   void *sum_out, int64_t ldo, const void *gamma, float eps, const int32_t *idx,
                                   const atom_desc *d, float clip, void *out, size_t out_bytes, void *stream)
{
    atom_status st = check_desc(d);
    if (st != ATOM_OK) return st;
    if (rows < 0 || ld < d->K) return ATOM_ERR_SHAPE;
    if (pre != 0 && ldr < d->K) return ATOM_ERR_SHAPE;
    if (pre == 1 && ldo < d->K) return ATOM_ERR_SHAPE;
    if (rows == 0) return ATOM_OK;
    if (!x || !out) return ATOM_ERR_NULL;
    if (pre != 0 && !res) return ATOM_ERR_NULL;
    if (pre == 1 && !sum_out) return ATOM_ERR_NULL;
    if (!aligned(x, 16) || (ld % 8) || !aligned(idx, 16) || !aligned(out, 256) || (gamma && !aligned(gamma, 16)))
        return ATOM_ERR_ALIGN;
    if (pre != 0 && (!aligned(res, 16) || (ldr % 8))) return ATOM_ERR_ALIGN;
    if (pre == 1 && (!aligned(sum_out, 16) || (ldo % 8))) return ATOM_ERR_ALIGN;
    if (!(clip >= 9.5367431640625e-07f && clip <= 1.0f)) return ATOM_ERR_UNSUPPORTED;
    if (atom_internal::quantize_packed_lds_bytes(d->K, d->n_outlier, gamma != nullptr, idx == nullptr) > 160 * 1024)
        return ATOM_ERR_UNSUPPORTED;
    if ((rows + 63) / 64 > 65535) return ATOM_ERR_UNSUPPORTED;       // what the packed GEMM takes
    if (out_bytes < atom_internal::f6_packed_bytes(rows, d->K, d->n_outlier)) return ATOM_ERR_WORKSPACE;
    hipError_t err = atom_internal::launch_quantize_rows_packed(x, rows, ld, pre, res, ldr, sum_out, ldo, gamma, eps, idx,
                                                                d->K, d->n_outlier, d->bits_normal, clip, out,
                                                                static_cast<hipStream_t>(stream));
    return err == hipSuccess ? ATOM_OK : ATOM_ERR_HIP;
}

}  // namespace

extern "C" {
atom_status atom_quantize_act_packed(const void *x_f16, int64_t M, int64_t ldx, const void *gamma_f16, float eps,
                                     const int32_t *reorder_idx, const atom_desc *d, float clip, void *a_packed,
                                     size_t packed_bytes, void *stream)
{
    return quantize_packed_common(x_f16, M, ldx, 0, nullptr, 0, nullptr, 0, gamma_f16, eps, reorder_idx, d, clip,
                                  a_packed, packed_bytes, stream);
}

atom_status atom_add_quantize_act_packed(const void *x_f16, const void *residual_f16, int64_t M, int64_t ldx,
                                         int64_t ldr, void *sum_out_f16, int64_t ldo, const void *gamma_f16, float eps,
                                         const int32_t *reorder_idx, const atom_desc *d, float clip, void *a_packed,
                                         size_t packed_bytes, void *stream)
{
    return quantize_packed_common(x_f16, M, ldx, 1, residual_f16, ldr, sum_out_f16, ldo, gamma_f16, eps, reorder_idx, d,
                                  clip, a_packed, packed_bytes, stream);
}

atom_status atom_swiglu_quantize_act_packed(const void *gate_f16, const void *up_f16, int64_t M, int64_t ldg,
                                            int64_t ldu, const int32_t *reorder_idx, const atom_desc *d, float clip,
                                            void *a_packed, size_t packed_bytes, void *stream)
{
    return quantize_packed_common(gate_f16, M, ldg, 2, up_f16, ldu, nullptr, 0, nullptr, 0.0f, reorder_idx, d, clip,
                                  a_packed, packed_bytes, stream);
}


atom_status atom_quantize_act(const void *x_f16, int64_t M, int64_t ldx, const void *gamma_f16,
                              float eps, const int32_t *reorder_idx, const atom_desc *d,
                              float clip, void *q4, void *q8, void *scale_f16, void *stream)
{
    return quantize_common(x_f16, M, ldx, 0, nullptr, 0, nullptr, 0, gamma_f16, eps, reorder_idx, d, clip, q4, q8, scale_f16,
                           stream);
}

atom_status atom_add_quantize_act(const void *x_f16, const void *residual_f16, int64_t M,
                                  int64_t ldx, int64_t ldr, void *sum_out_f16, int64_t ldo,
                                  const void *gamma_f16, float eps, const int32_t *reorder_idx,
                                  const atom_desc *d, float clip, void *q4, void *q8,
                                  void *scale_f16, void *stream)
{
    return quantize_common(x_f16, M, ldx, 1, residual_f16, ldr, sum_out_f16, ldo, gamma_f16, eps,
                           reorder_idx, d, clip, q4, q8, scale_f16, stream);
}

atom_status atom_swiglu_quantize_act(const void *gate_f16, const void *up_f16, int64_t M,
                                     int64_t ldg, int64_t ldu, const int32_t *reorder_idx,
                                     const atom_desc *d, float clip, void *q4, void *q8,
                                     void *scale_f16, void *stream)
{
    return quantize_common(gate_f16, M, ldg, 2, up_f16, ldu, nullptr, 0, nullptr, 0.0f, reorder_idx,
                           d, clip, q4, q8, scale_f16, stream);
}

atom_status atom_quantize_weight(const void *w_f16, int64_t N, int64_t ldw,
                                 const int32_t *reorder_idx, const atom_desc *d, float clip,
                                 void *q4, void *q8, void *scale_f16, void *stream)
{
    return quantize_common(w_f16, N, ldw, 0, nullptr, 0, nullptr, 0, nullptr, 0.0f, reorder_idx, d, clip, q4, q8, scale_f16,
                           stream);
}

size_t atom_w4a4_gemm_workspace_bytes(int64_t M, int64_t N, const atom_desc *d)
{
    if (check_desc(d, true) != ATOM_OK || M <= 0 || N <= 0) return 0;
    return atom_internal::gemm_workspace_bytes(M, N, d->K, d->n_outlier);
}

atom_status atom_w4a4_gemm(const void *a_q4, const void *a_q8, const void *a_scale, int64_t M,
                           const void *w_q4, const void *w_q8, const void *w_scale, int64_t N,
                           const atom_desc *d, void *y_f16, int64_t ldy, int32_t *partials_dbg,
                           void *workspace, size_t workspace_bytes, void *stream)
{
    atom_status st = check_desc(d, true);
    if (st != ATOM_OK) return st;
    if (M < 0 || N < 0 || ldy < N) return ATOM_ERR_SHAPE;
    if (M == 0 || N == 0) return ATOM_OK;
    if (!a_q4 || !a_q8 || !a_scale || !w_q4 || !w_q8 || !w_scale || !y_f16) return ATOM_ERR_NULL;
    if (!aligned(a_q4, 16) || !aligned(a_q8, 16) || !aligned(a_scale, 2) || !aligned(w_q4, 16) ||
        !aligned(w_q8, 16) || !aligned(w_scale, 2) || !aligned(y_f16, 2) ||
        (partials_dbg && !aligned(partials_dbg, 4)))
        return ATOM_ERR_ALIGN;
    // the tiled kernels address the code and scale arrays with 32-bit offsets and number their
    // tiles in 32 bits
    {
        const uint64_t lim = 1ull << 32, K4h = (uint64_t)(d->K - d->n_outlier) / 2, O = (uint64_t)d->n_outlier,
                       G = (uint64_t)(d->K / d->group_size);
        const uint64_t rows = (uint64_t)(M > N ? M : N);
        if (rows * K4h >= lim || rows * O >= lim || rows * G >= lim) return ATOM_ERR_UNSUPPORTED;
        if (((uint64_t)M + 63) / 64 * (((uint64_t)N + 31) / 32) > 0x7fffffffull) return ATOM_ERR_UNSUPPORTED;
    }
    const size_t need = atom_internal::gemm_workspace_bytes(M, N, d->K, d->n_outlier);
    if (need) {
        if (!workspace || workspace_bytes < need) return ATOM_ERR_WORKSPACE;
        if (!aligned(workspace, 256)) return ATOM_ERR_ALIGN;
    }
    atom_internal::GemmArgs g;
    g.a_q4 = static_cast<const uint8_t *>(a_q4);
    g.a_q8 = static_cast<const int8_t *>(a_q8);
    g.a_scale = static_cast<const uint16_t *>(a_scale);
    g.M = M;
    g.w_q4 = static_cast<const uint8_t *>(w_q4);
    g.w_q8 = static_cast<const int8_t *>(w_q8);
    g.w_scale = static_cast<const uint16_t *>(w_scale);
    g.N = N;
    g.K = d->K;
    g.O = d->n_outlier;
    g.y = static_cast<uint16_t *>(y_f16);
    g.ldy = ldy;
    g.partials = partials_dbg;
    g.workspace = workspace;
    g.workspace_bytes = workspace_bytes;
    if (d->group_size != atom_internal::kGroup) {
        if ((M + 63) / 64 > 65535) return ATOM_ERR_UNSUPPORTED;         // grid rows of the plain kernel
        hipError_t e2 = atom_internal::launch_w4a4_gemm_gs(g, d->group_size, static_cast<hipStream_t>(stream));
        return e2 == hipSuccess ? ATOM_OK : ATOM_ERR_HIP;
    }
    hipError_t err = atom_internal::launch_w4a4_gemm(g, static_cast<hipStream_t>(stream));
    return err == hipSuccess ? ATOM_OK : ATOM_ERR_HIP;
}

atom_status atom_permute_rows(const void *in_f16, int64_t rows_in, int64_t cols, int64_t ld_in,
                              const int32_t *row_idx, int64_t rows_out, void *out_f16, int64_t ld_out,
                              void *stream)
{
    if (rows_in <= 0 || rows_out < 0 || cols < 0 || ld_in < cols || ld_out < cols) return ATOM_ERR_SHAPE;
    if (rows_out == 0 || cols == 0) return ATOM_OK;
    if (!in_f16 || !row_idx || !out_f16) return ATOM_ERR_NULL;
    if (!aligned(in_f16, 2) || !aligned(out_f16, 2) || !aligned(row_idx, 4)) return ATOM_ERR_ALIGN;
    if (in_f16 == out_f16) return ATOM_ERR_UNSUPPORTED;           // not in place
    if (rows_out > 0x7fffffff) return ATOM_ERR_UNSUPPORTED;
    hipError_t err = atom_internal::launch_permute_rows(in_f16, rows_in, rows_out, cols, ld_in, row_idx, out_f16,
                                                        ld_out, static_cast<hipStream_t>(stream));
    return err == hipSuccess ? ATOM_OK : ATOM_ERR_HIP;
}

size_t atom_decode_linear_lds_bytes(int64_t M, const atom_desc *d, int with_norm, int with_index)
{
    if (check_desc(d) != ATOM_OK || M <= 0 || M > 16) return 0;
    return atom_internal::decode_linear_lds_bytes((int)M, d->K, d->n_outlier, with_norm != 0, with_index == 0);
}

atom_status atom_decode_linear(const void *x_f16, int64_t M, int64_t ldx, const void *gamma_f16,
                               float eps, const int32_t *reorder_idx, const atom_desc *d, float clip,
                               const void *w_q4, const void *w_q8, const void *w_scale, int64_t N,
                               void *y_f16, int64_t ldy, void *dbg_q4, void *dbg_q8, void *dbg_scale,
                               void *stream)
{
    atom_status st = check_desc(d);
    if (st != ATOM_OK) return st;
    if (M < 0 || N < 0 || ldx < d->K || ldy < N) return ATOM_ERR_SHAPE;
    if (M == 0 || N == 0) return ATOM_OK;
    if (M > 16 || d->K > 12288 || !(clip >= 9.5367431640625e-07f && clip <= 1.0f)) return ATOM_ERR_UNSUPPORTED;
    if (atom_internal::decode_linear_lds_bytes((int)M, d->K, d->n_outlier, gamma_f16 != nullptr, reorder_idx == nullptr) > 160 * 1024)
        return ATOM_ERR_UNSUPPORTED;
    if (!x_f16 || !w_q4 || !w_q8 || !w_scale || !y_f16) return ATOM_ERR_NULL;       // reorder_idx may be null
    const int ndbg = (dbg_q4 != nullptr) + (dbg_q8 != nullptr) + (dbg_scale != nullptr);
    if (ndbg != 0 && ndbg != 3) return ATOM_ERR_NULL;
    if (!aligned(x_f16, 16) || (ldx % 8) || !aligned(reorder_idx, 16) || (gamma_f16 && !aligned(gamma_f16, 16)) ||
        !aligned(w_q4, 16) || !aligned(w_q8, 16) || !aligned(w_scale, 2) || !aligned(y_f16, 2) ||
        (ndbg && (!aligned(dbg_q4, 4) || !aligned(dbg_q8, 4) || !aligned(dbg_scale, 2))))
        return ATOM_ERR_ALIGN;
    hipError_t err = atom_internal::launch_decode_linear(x_f16, (int)M, ldx, gamma_f16, eps, reorder_idx, d->K,
                                                         d->n_outlier, d->bits_normal, clip, w_q4, w_q8, w_scale,
                                                         N, y_f16, ldy, dbg_q4, dbg_q8, dbg_scale,
                                                         static_cast<hipStream_t>(stream));
    return err == hipSuccess ? ATOM_OK : ATOM_ERR_HIP;
}

size_t atom_decode_linear_coop_sync_bytes(void) { return atom_internal::decode_linear_coop_sync_bytes(); }

atom_status atom_decode_linear_coop(const void *x_f16, int64_t M, int64_t ldx, const void *gamma_f16,
                                    float eps, const int32_t *reorder_idx, const atom_desc *d, float clip,
                                    const void *w_q4, const void *w_q8, const void *w_scale, int64_t N,
                                    void *y_f16, int64_t ldy, void *a_q4, void *a_q8, void *a_scale,
                                    void *sync_words, void *stream)
{
    atom_status st = check_desc(d);
    if (st != ATOM_OK) return st;
    if (M < 0 || N < 0 || ldx < d->K || ldy < N) return ATOM_ERR_SHAPE;
    if (M == 0 || N == 0) return ATOM_OK;
    if (!x_f16 || !w_q4 || !w_q8 || !w_scale || !y_f16 || !a_q4 || !a_q8 || !a_scale || !sync_words)
        return ATOM_ERR_NULL;                                                        // reorder_idx may be null
    if (!aligned(x_f16, 16) || (ldx % 8) || !aligned(reorder_idx, 16) || (gamma_f16 && !aligned(gamma_f16, 16)) ||
        !aligned(w_q4, 16) || !aligned(w_q8, 16) || !aligned(w_scale, 8) || !aligned(y_f16, 2) ||
        !aligned(a_q4, 128) || !aligned(a_q8, 128) || !aligned(a_scale, 128) || !aligned(sync_words, 128))
        return ATOM_ERR_ALIGN;
    if (M > 16 || !(clip >= 9.5367431640625e-07f && clip <= 1.0f) ||
        !atom_internal::decode_linear_coop_supported((int)M, d->K, d->n_outlier, a_scale, w_scale, N))
        return ATOM_ERR_UNSUPPORTED;
    hipError_t err = atom_internal::launch_decode_linear_coop(x_f16, (int)M, ldx, gamma_f16, eps, reorder_idx, d->K,
                                                              d->n_outlier, d->bits_normal, clip, w_q4, w_q8,
                                                              w_scale, N, y_f16, ldy, a_q4, a_q8, a_scale,
                                                              sync_words, static_cast<hipStream_t>(stream));
    return err == hipSuccess ? ATOM_OK : ATOM_ERR_HIP;
}

size_t atom_tile_weight_decode_bytes(int64_t N, const atom_desc *d, int which)
{
    if (check_desc(d) != ATOM_OK || N <= 0 || (which != 0 && which != 1)) return 0;
    const size_t rows = (size_t)((N + 15) / 16) * 16;
    return rows * (which == 0 ? (size_t)(d->K - d->n_outlier) / 2 : (size_t)d->n_outlier);
}

atom_status atom_tile_weight_decode(const void *w_q4, const void *w_q8, int64_t N, const atom_desc *d,
                                    void *w_q4_tiled, size_t q4_bytes, void *w_q8_tiled, size_t q8_bytes,
                                    void *stream)
{
    atom_status st = check_desc(d);
    if (st != ATOM_OK) return st;
    if (N < 0) return ATOM_ERR_SHAPE;
    if (N == 0) return ATOM_OK;
    if (!w_q4 || !w_q8 || !w_q4_tiled || !w_q8_tiled) return ATOM_ERR_NULL;
    if (!aligned(w_q4, 16) || !aligned(w_q8, 16) || !aligned(w_q4_tiled, 16) || !aligned(w_q8_tiled, 16))
        return ATOM_ERR_ALIGN;
    if (q4_bytes < atom_tile_weight_decode_bytes(N, d, 0) || q8_bytes < atom_tile_weight_decode_bytes(N, d, 1))
        return ATOM_ERR_WORKSPACE;
    if ((N + 15) / 16 > 0x7fffffff) return ATOM_ERR_UNSUPPORTED;
    hipError_t err = atom_internal::launch_tile_weight_decode(w_q4, w_q8, N, d->K, d->n_outlier, w_q4_tiled,
                                                              w_q8_tiled, static_cast<hipStream_t>(stream));
    return err == hipSuccess ? ATOM_OK : ATOM_ERR_HIP;
}

atom_status atom_w4a4_gemm_decode_tiled(const void *a_q4, const void *a_q8, const void *a_scale, int64_t M,
                                        const void *w_q4_tiled, const void *w_q8_tiled, const void *w_scale,
                                        int64_t N, const atom_desc *d, void *y_f16, int64_t ldy, void *stream)
{
    atom_status st = check_desc(d);
    if (st != ATOM_OK) return st;
    if (M < 0 || N < 0 || ldy < N) return ATOM_ERR_SHAPE;
    if (M == 0 || N == 0) return ATOM_OK;
    if (!a_q4 || !a_q8 || !a_scale || !w_q4_tiled || !w_q8_tiled || !w_scale || !y_f16) return ATOM_ERR_NULL;
    if (!aligned(a_q4, 16) || !aligned(a_q8, 16) || !aligned(a_scale, 8) || !aligned(w_q4_tiled, 16) ||
        !aligned(w_q8_tiled, 16) || !aligned(w_scale, 8) || !aligned(y_f16, 2))
        return ATOM_ERR_ALIGN;
    atom_internal::GemmArgs g;
    g.a_q4 = static_cast<const uint8_t *>(a_q4);
    g.a_q8 = static_cast<const int8_t *>(a_q8);
    g.a_scale = static_cast<const uint16_t *>(a_scale);
    g.M = M;
    g.w_q4 = static_cast<const uint8_t *>(w_q4_tiled);
    g.w_q8 = static_cast<const int8_t *>(w_q8_tiled);
    g.w_scale = static_cast<const uint16_t *>(w_scale);
    g.N = N;
    g.K = d->K;
    g.O = d->n_outlier;
    g.y = static_cast<uint16_t *>(y_f16);
    g.ldy = ldy;
    g.partials = nullptr;
    g.workspace = nullptr;
    g.workspace_bytes = 0;
    if (!atom_internal::decode_tiled_supported(g)) return ATOM_ERR_UNSUPPORTED;
    hipError_t err = atom_internal::launch_w4a4_gemm_decode_tiled(g, static_cast<hipStream_t>(stream));
    return err == hipSuccess ? ATOM_OK : ATOM_ERR_HIP;
}

size_t atom_pack_weight_bytes(int64_t N, const atom_desc *d)
{
    if (check_desc(d) != ATOM_OK || N <= 0) return 0;
    return atom_internal::f6_packed_bytes(N, d->K, d->n_outlier);
}

atom_status atom_pack_weight(const void *w_q4, const void *w_q8, const void *w_scale, int64_t N,
                             const atom_desc *d, void *w_packed, size_t packed_bytes, void *stream)
{
    atom_status st = check_desc(d);
    if (st != ATOM_OK) return st;
    if (N < 0) return ATOM_ERR_SHAPE;
    if (N == 0) return ATOM_OK;
    if (!w_q4 || !w_q8 || !w_scale || !w_packed) return ATOM_ERR_NULL;
    if (!aligned(w_q4, 16) || !aligned(w_q8, 16) || !aligned(w_scale, 2) || !aligned(w_packed, 256))
        return ATOM_ERR_ALIGN;
    if ((N + 63) / 64 > 65535) return ATOM_ERR_UNSUPPORTED;          // one grid row per 64 rows
    if (packed_bytes < atom_internal::f6_packed_bytes(N, d->K, d->n_outlier)) return ATOM_ERR_WORKSPACE;
    hipError_t err = atom_internal::launch_f6_pack(w_q4, w_q8, w_scale, N, d->K, d->n_outlier, w_packed,
                                                   static_cast<hipStream_t>(stream));
    return err == hipSuccess ? ATOM_OK : ATOM_ERR_HIP;
}

atom_status atom_pack_act(const void *a_q4, const void *a_q8, const void *a_scale, int64_t M,
                          const atom_desc *d, void *a_packed, size_t packed_bytes, void *stream)
{
    return atom_pack_weight(a_q4, a_q8, a_scale, M, d, a_packed, packed_bytes, stream);
}

atom_status atom_w4a4_gemm_prepacked(const void *a_packed, int64_t M, const void *w_packed, int64_t N,
                                     const atom_desc *d, void *y_f16, int64_t ldy, int32_t *partials_dbg,
                                     void *stream)
{
    atom_status st = check_desc(d);
    if (st != ATOM_OK) return st;
    if (M < 0 || N < 0 || ldy < N) return ATOM_ERR_SHAPE;
    if (M == 0 || N == 0) return ATOM_OK;
    if (!a_packed || !w_packed || !y_f16) return ATOM_ERR_NULL;
    if (!aligned(a_packed, 256) || !aligned(w_packed, 256) || !aligned(y_f16, 2) ||
        (partials_dbg && !aligned(partials_dbg, 4)))
        return ATOM_ERR_ALIGN;
    const int64_t mu = (M + 63) / 64, nu = (N + 63) / 64;
    if (mu > 65535 || mu * ((nu + 1) / 2) > 0x7fffffffLL) return ATOM_ERR_UNSUPPORTED;
    hipError_t err = atom_internal::launch_f6_gemm(a_packed, M, w_packed, N, d->K, d->n_outlier, y_f16, ldy,
                                                   partials_dbg, static_cast<hipStream_t>(stream));
    return err == hipSuccess ? ATOM_OK : ATOM_ERR_HIP;
}

size_t atom_w4a4_gemm_packed_workspace_bytes(int64_t M, int64_t N, const atom_desc *d)
{
    (void)N;
    if (check_desc(d) != ATOM_OK || M <= 0) return 0;
    return atom_internal::f6_packed_bytes(M, d->K, d->n_outlier);
}

atom_status atom_w4a4_gemm_packed(const void *a_q4, const void *a_q8, const void *a_scale, int64_t M,
                                  const void *w_packed, int64_t N, const atom_desc *d, void *y_f16,
                                  int64_t ldy, int32_t *partials_dbg, void *workspace,
                                  size_t workspace_bytes, void *stream)
{
    atom_status st = check_desc(d);
    if (st != ATOM_OK) return st;
    if (M < 0 || N < 0 || ldy < N) return ATOM_ERR_SHAPE;
    if (M == 0 || N == 0) return ATOM_OK;
    if (!a_q4 || !a_q8 || !a_scale || !w_packed || !y_f16) return ATOM_ERR_NULL;
    if (!aligned(a_q4, 16) || !aligned(a_q8, 16) || !aligned(a_scale, 2) || !aligned(w_packed, 256) ||
        !aligned(y_f16, 2) || (partials_dbg && !aligned(partials_dbg, 4)))
        return ATOM_ERR_ALIGN;
    const int64_t mu = (M + 63) / 64, nu = (N + 63) / 64;
    if (mu > 65535 || mu * ((nu + 1) / 2) > 0x7fffffffLL) return ATOM_ERR_UNSUPPORTED;
    const size_t need = atom_internal::f6_packed_bytes(M, d->K, d->n_outlier);
    if (!workspace || workspace_bytes < need) return ATOM_ERR_WORKSPACE;
    if (!aligned(workspace, 256)) return ATOM_ERR_ALIGN;
    st = atom_pack_act(a_q4, a_q8, a_scale, M, d, workspace, workspace_bytes, stream);
    if (st != ATOM_OK) return st;
    return atom_w4a4_gemm_prepacked(workspace, M, w_packed, N, d, y_f16, ldy, partials_dbg, stream);
}

atom_status atom_kv_quantize(const void *x_f16, int64_t R, int64_t ldx, int32_t D, float clip,
                             const int32_t *pos, int32_t rows_per_seq, int64_t Tmax, void *q,
                             void *scale_f16, void *zero_i16, void *stream)
{
    if (D != 64 && D != 128) return D > 0 && D % 2 == 0 ? ATOM_ERR_UNSUPPORTED : ATOM_ERR_SHAPE;
    if (R < 0 || ldx < D) return ATOM_ERR_SHAPE;
    if (pos && (rows_per_seq <= 0 || R % rows_per_seq || Tmax <= 0)) return ATOM_ERR_SHAPE;
    if (R == 0) return ATOM_OK;
    if (!x_f16 || !q || !scale_f16 || !zero_i16) return ATOM_ERR_NULL;
    if (!aligned(x_f16, 16) || (ldx % 8) || !aligned(q, 4) || !aligned(scale_f16, 2) ||
        !aligned(zero_i16, 2) || (pos && !aligned(pos, 4)))
        return ATOM_ERR_ALIGN;
    if (R * (D / 8) / 256 + 1 > 0x7fffffffLL) return ATOM_ERR_UNSUPPORTED;
    hipError_t err = atom_internal::launch_kv_quantize(x_f16, R, ldx, D, clip, pos, rows_per_seq,
                                                       Tmax, q, scale_f16, zero_i16,
                                                       static_cast<hipStream_t>(stream));
    return err == hipSuccess ? ATOM_OK : ATOM_ERR_HIP;
}

atom_status atom_kv_quantize_pair(const void *k_f16, const void *v_f16, int64_t R, int64_t ldx,
                                  int32_t D, float clip, const int32_t *pos, int32_t rows_per_seq,
                                  int64_t Tmax, void *k_q, void *k_scale_f16, void *k_zero_i16,
                                  void *v_q, void *v_scale_f16, void *v_zero_i16, void *stream)
{
    if (D != 64 && D != 128) return D > 0 && D % 2 == 0 ? ATOM_ERR_UNSUPPORTED : ATOM_ERR_SHAPE;
    if (R < 0 || ldx < D) return ATOM_ERR_SHAPE;
    if (pos && (rows_per_seq <= 0 || R % rows_per_seq || Tmax <= 0)) return ATOM_ERR_SHAPE;
    if (R == 0) return ATOM_OK;
    if (!k_f16 || !k_q || !k_scale_f16 || !k_zero_i16 || !v_f16 || !v_q || !v_scale_f16 || !v_zero_i16)
        return ATOM_ERR_NULL;
    if (!aligned(k_f16, 16) || !aligned(v_f16, 16) || (ldx % 8) || !aligned(k_q, 4) || !aligned(v_q, 4) ||
        !aligned(k_scale_f16, 2) || !aligned(v_scale_f16, 2) || !aligned(k_zero_i16, 2) ||
        !aligned(v_zero_i16, 2) || (pos && !aligned(pos, 4)))
        return ATOM_ERR_ALIGN;
    if (R * (D / 8) / 256 + 1 > 0x7fffffffLL) return ATOM_ERR_UNSUPPORTED;
    hipError_t err = atom_internal::launch_kv_quantize(k_f16, R, ldx, D, clip, pos, rows_per_seq, Tmax,
                                                       k_q, k_scale_f16, k_zero_i16,
                                                       static_cast<hipStream_t>(stream), v_f16, v_q,
                                                       v_scale_f16, v_zero_i16);
    return err == hipSuccess ? ATOM_OK : ATOM_ERR_HIP;
}

atom_status atom_decode_attention_kv4(const void *q_f16, int32_t B, int32_t H, int32_t Hkv,
                                      int32_t D, int64_t Tmax, const int32_t *seq_len,
                                      const void *k_codes, const void *k_scale, const void *k_zero,
                                      const void *v_codes, const void *v_scale, const void *v_zero,
                                      float sm_scale, void *out_f16, void *workspace,
                                      size_t workspace_bytes, void *stream)
{
    if (B < 0 || H <= 0 || Hkv <= 0 || H % Hkv || D <= 0 || Tmax < 0 || Tmax > 0x7fffffffLL)
        return ATOM_ERR_SHAPE;
    if (D != 128) return ATOM_ERR_UNSUPPORTED;
    if ((int64_t)B * H > 0x7fffffffLL) return ATOM_ERR_UNSUPPORTED;
    if (Tmax > (1LL << 25)) return ATOM_ERR_UNSUPPORTED;      // 32-bit byte offsets inside a cache head
    if (B == 0) return ATOM_OK;
    if (!q_f16 || !seq_len || !out_f16) return ATOM_ERR_NULL;
    if (Tmax > 0 && (!k_codes || !k_scale || !k_zero || !v_codes || !v_scale || !v_zero))
        return ATOM_ERR_NULL;
    if (!aligned(q_f16, 16) || !aligned(seq_len, 4) || !aligned(out_f16, 2) ||
        !aligned(k_codes, 16) || !aligned(v_codes, 16) || !aligned(k_scale, 2) ||
        !aligned(v_scale, 2) || !aligned(k_zero, 2) || !aligned(v_zero, 2))
        return ATOM_ERR_ALIGN;
    const size_t need = atom_internal::decode_attention_workspace_bytes(B, H, Hkv, Tmax);
    if (need) {
        if (!workspace || workspace_bytes < need) return ATOM_ERR_WORKSPACE;
        if (!aligned(workspace, 16)) return ATOM_ERR_ALIGN;
    }
    hipError_t err = atom_internal::launch_decode_attention_kv4(
        q_f16, B, H, Hkv, Tmax, seq_len, k_codes, k_scale, k_zero, v_codes, v_scale, v_zero,
        sm_scale, out_f16, workspace, static_cast<hipStream_t>(stream));
    return err == hipSuccess ? ATOM_OK : ATOM_ERR_HIP;
}

size_t atom_static_scratch_bytes(void) { return atom_internal::static_scratch_bytes(); }

atom_status atom_decode_attention_kv4_static(const void *q_f16, int32_t B, int32_t H, int32_t Hkv,
                                             int32_t D, int64_t Tmax, const int32_t *seq_len,
                                             const void *k_codes, const void *k_scale,
                                             const void *k_zero, const void *v_codes,
                                             const void *v_scale, const void *v_zero, float sm_scale,
                                             void *out_f16, void *stream)
{
    if (B < 0 || H <= 0 || Hkv <= 0 || H % Hkv || D <= 0 || Tmax < 0 || Tmax > 0x7fffffffLL)
        return ATOM_ERR_SHAPE;
    if (D != 128) return ATOM_ERR_UNSUPPORTED;
    if ((int64_t)B * H > 0x7fffffffLL || Tmax > (1LL << 25)) return ATOM_ERR_UNSUPPORTED;
    if (B == 0) return ATOM_OK;
    // the partials of a split launch must fit the library's own scratch array
    const size_t need = atom_internal::decode_attention_workspace_bytes(B, H, Hkv, Tmax);
    if (need > atom_internal::static_scratch_bytes()) return ATOM_ERR_WORKSPACE;
    void *ws = nullptr;
    if (atom_internal::static_scratch(&ws) != hipSuccess) return ATOM_ERR_HIP;
    return atom_decode_attention_kv4(q_f16, B, H, Hkv, D, Tmax, seq_len, k_codes, k_scale, k_zero, v_codes,
                                     v_scale, v_zero, sm_scale, out_f16, ws,
                                     atom_internal::static_scratch_bytes(), stream);
}

size_t atom_decode_attention_kv4_workspace_bytes(int32_t B, int32_t H, int32_t Hkv, int32_t D,
                                                 int64_t Tmax)
{
    if (B <= 0 || H <= 0 || Hkv <= 0 || H % Hkv || D != 128 || Tmax <= 0 || Tmax > 0x7fffffffLL)
        return 0;
    return atom_internal::decode_attention_workspace_bytes(B, H, Hkv, Tmax);
}

}  // extern "C"

namespace {

atom_status check_desc_mx(const atom_desc *d)
{
    if (!d) return ATOM_ERR_NULL;
    if (d->K <= 0 || d->group_size <= 0 || d->n_outlier < 0) return ATOM_ERR_SHAPE;
    if (d->group_size != 32 || d->bits_normal != 4 || d->bits_outlier != 8) return ATOM_ERR_UNSUPPORTED;
    if (d->K % 128 || d->n_outlier % 128 || d->n_outlier >= d->K) return ATOM_ERR_SHAPE;
    if (d->n_outlier == 0 || d->K > atom_internal::kMaxK) return ATOM_ERR_UNSUPPORTED;
    return ATOM_OK;
}

atom_status mx_quantize_common(const void *x, int64_t rows, int64_t ld, const void *gamma, float eps,
                               const int32_t *idx, const atom_desc *d, float clip, void *q4, void *q8,
                               void *e8, void *stream)
{
    atom_status st = check_desc_mx(d);
    if (st != ATOM_OK) return st;
    if (rows < 0 || ld < d->K) return ATOM_ERR_SHAPE;
    if (rows == 0) return ATOM_OK;
    if (!x || !idx || !q4 || !q8 || !e8) return ATOM_ERR_NULL;
    if (!aligned(x, 16) || (ld % 8) || !aligned(idx, 16) || !aligned(q4, 16) || !aligned(q8, 16) ||
        !aligned(e8, 4) || (gamma && !aligned(gamma, 16)))
        return ATOM_ERR_ALIGN;
    hipError_t err = atom_internal::launch_quantize_rows_mx(x, rows, ld, gamma, eps, idx, d->K,
                                                            d->n_outlier, clip, q4, q8, e8,
                                                            static_cast<hipStream_t>(stream));
    return err == hipSuccess ? ATOM_OK : ATOM_ERR_HIP;
}

}  // namespace

extern "C" {

atom_status atom_mx_quantize_act(const void *x_f16, int64_t M, int64_t ldx, const void *gamma_f16,
                                 float eps, const int32_t *reorder_idx, const atom_desc *d, float clip,
                                 void *q4, void *q8, void *e8, void *stream)
{
    return mx_quantize_common(x_f16, M, ldx, gamma_f16, eps, reorder_idx, d, clip, q4, q8, e8, stream);
}

atom_status atom_mx_quantize_weight(const void *w_f16, int64_t N, int64_t ldw,
                                    const int32_t *reorder_idx, const atom_desc *d, float clip,
                                    void *q4, void *q8, void *e8, void *stream)
{
    return mx_quantize_common(w_f16, N, ldw, nullptr, 0.0f, reorder_idx, d, clip, q4, q8, e8, stream);
}

atom_status atom_mx_gemm(const void *a_q4, const void *a_q8, const void *a_e8, int64_t M,
                         const void *w_q4, const void *w_q8, const void *w_e8, int64_t N,
                         const atom_desc *d, void *y_f16, int64_t ldy, void *stream)
{
    atom_status st = check_desc_mx(d);
    if (st != ATOM_OK) return st;
    if (M < 0 || N < 0 || ldy < N) return ATOM_ERR_SHAPE;
    if (M == 0 || N == 0) return ATOM_OK;
    if (!a_q4 || !a_q8 || !a_e8 || !w_q4 || !w_q8 || !w_e8 || !y_f16) return ATOM_ERR_NULL;
    if (!aligned(a_q4, 16) || !aligned(a_q8, 16) || !aligned(a_e8, 4) || !aligned(w_q4, 16) ||
        !aligned(w_q8, 16) || !aligned(w_e8, 4) || !aligned(y_f16, 2))
        return ATOM_ERR_ALIGN;
    if (M >= (int64_t)1 << 26 || N >= (int64_t)1 << 26) return ATOM_ERR_UNSUPPORTED;   // 32-bit row offsets
    const int64_t tiles = ((M + 255) / 256) * ((N + 255) / 256);
    if (tiles > 0x7fffffffLL) return ATOM_ERR_UNSUPPORTED;
    hipError_t err = atom_internal::launch_mx_gemm(a_q4, a_q8, a_e8, M, w_q4, w_q8, w_e8, N, d->K,
                                                   d->n_outlier, y_f16, ldy,
                                                   static_cast<hipStream_t>(stream));
    return err == hipSuccess ? ATOM_OK : ATOM_ERR_HIP;
}

}  // extern "C"

extern "C" {

size_t atom_calibrate_reorder_workspace_bytes(int64_t T, int32_t K)
{
    if (T < 0 || K <= 0 || K > atom_internal::kMaxK) return 0;
    return atom_internal::calibrate_workspace_bytes(T, K);
}

atom_status atom_calibrate_reorder(const void *x_f16, int64_t T, int64_t ldx, int32_t K,
                                   void *workspace, size_t workspace_bytes, int32_t *idx_out,
                                   void *stream)
{
    if (T < 0 || K <= 0 || ldx < K) return ATOM_ERR_SHAPE;
    if (K > atom_internal::kMaxK || (T + 255) / 256 > 65535) return ATOM_ERR_UNSUPPORTED;
    if (!idx_out || !workspace || (T > 0 && !x_f16)) return ATOM_ERR_NULL;
    if (!aligned(x_f16, 2) || !aligned(workspace, 16) || !aligned(idx_out, 4)) return ATOM_ERR_ALIGN;
    if (workspace_bytes < atom_internal::calibrate_workspace_bytes(T, K)) return ATOM_ERR_WORKSPACE;
    hipError_t err = atom_internal::launch_calibrate_reorder(x_f16, T, ldx, K, workspace, idx_out,
                                                             static_cast<hipStream_t>(stream));
    return err == hipSuccess ? ATOM_OK : ATOM_ERR_HIP;
}

}  // extern "C"

extern "C" {

double atom_mfma_rate_probe(int32_t kind, int32_t iters, void *scratch4, void *stream, atom_status *status)
{
    atom_status st = ATOM_OK;
    double ops = 0.0;
    if ((kind != 0 && kind != 1) || iters <= 0) st = ATOM_ERR_SHAPE;
    else if (!scratch4) st = ATOM_ERR_NULL;
    else if (!aligned(scratch4, 4)) st = ATOM_ERR_ALIGN;
    else {
        st = atom_internal::launch_mfma_rate_probe(kind, iters, scratch4, static_cast<hipStream_t>(stream)) == hipSuccess
                 ? ATOM_OK : ATOM_ERR_HIP;
        if (st == ATOM_OK) ops = atom_internal::mfma_rate_probe_ops(kind, iters);
    }
    if (status) *status = st;
    return ops;
}

atom_status atom_check_reorder_idx(const int32_t *idx_host, int32_t K)
{
    if (!idx_host) return ATOM_ERR_NULL;
    if (K <= 0) return ATOM_ERR_SHAPE;
    unsigned char *seen = new (std::nothrow) unsigned char[(size_t)K]();
    if (!seen) return ATOM_ERR_WORKSPACE;
    atom_status st = ATOM_OK;
    for (int32_t j = 0; j < K && st == ATOM_OK; ++j) {
        const int32_t v = idx_host[j];
        if (v < 0 || v >= K || seen[(size_t)v]) st = ATOM_ERR_SHAPE;
        else seen[(size_t)v] = 1;
    }
    delete[] seen;
    return st;
}

const char *atom_status_string(int status)
{
    switch (status) {
    case ATOM_OK:              return "ok";
    case ATOM_ERR_NULL:        return "a required pointer is NULL";
    case ATOM_ERR_SHAPE:       return "invalid shape, leading dimension or reorder index";
    case ATOM_ERR_UNSUPPORTED: return "unsupported group size, bit-width or K";
    case ATOM_ERR_ALIGN:       return "misaligned pointer or leading dimension";
    case ATOM_ERR_WORKSPACE:   return "workspace missing or too small";
    case ATOM_ERR_HIP:         return "HIP launch failed";
    }
    return "unknown status";
}

}  // extern "C"
