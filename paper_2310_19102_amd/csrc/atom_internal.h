// Internal launch interface between the C-ABI shim and the kernel files.
#ifndef ATOM_INTERNAL_H
#define ATOM_INTERNAL_H

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace atom_internal {

constexpr int kGroup    = 128;     // channels per quantisation group
constexpr int kMaxK     = 32768;   // a staged fp32 row must fit the 160 KB LDS

size_t quantize_lds_bytes(int K, bool norm);

// One row per workgroup: optional RMSNorm, reorder gather, group quantisation.
// pre: 0 = the rows of x as they are; 1 = x + res rounded to fp16, written to sum_out;
// 2 = silu(x) * res in fp32 (x = gate rows, res = up rows; no norm).
// nbits: width of the normal channels, 4 or 3 (either way one code per nibble).
hipError_t launch_quantize_rows(const void *x, int64_t rows, int64_t ld, int pre, const void *res,
                                int64_t ldr, void *sum_out, int64_t ldo, const void *gamma,
                                float eps, const int32_t *idx, int K, int O, int nbits, float clip,
                                void *q4, void *q8, void *scale, hipStream_t stream, int group_size = 128);

struct GemmArgs {
    const uint8_t *a_q4; const int8_t *a_q8; const uint16_t *a_scale; int64_t M;
    const uint8_t *w_q4; const int8_t *w_q8; const uint16_t *w_scale; int64_t N;
    int K, O;
    uint16_t *y; int64_t ldy;
    int32_t *partials;          // NULL or [M, N, G]
    void *workspace; size_t workspace_bytes;
};

size_t     gemm_workspace_bytes(int64_t M, int64_t N, int K, int O);
hipError_t launch_w4a4_gemm(const GemmArgs &a, hipStream_t stream);
// Group sizes 64 and 256 (atom_gemm_gs.hip): one plain kernel, a single ascending chain of groups.
hipError_t launch_w4a4_gemm_gs(const GemmArgs &a, int group_size, hipStream_t stream);

// Decode-sized GEMM (M <= 64) on weight codes re-tiled into whole 128-byte lines per load
// (atom_gemm_decode.hip); w_q4 / w_q8 of the arguments are the tiled arrays, scales canonical.
bool       decode_tiled_supported(const GemmArgs &a);
hipError_t launch_w4a4_gemm_decode_tiled(const GemmArgs &a, hipStream_t stream);
hipError_t launch_tile_weight_decode(const void *q4, const void *q8, int64_t N, int K, int O, void *t4, void *t8,
                                     hipStream_t stream);

// Group GEMM on pre-tiled operands, INT4 groups carried in FP6 (atom_gemm_f6.hip): bytes of the
// tiled image of `rows` rows, the packing kernel (canonical q4 / q8 / scale -> image), the GEMM.
size_t     f6_packed_bytes(int64_t rows, int K, int O);
hipError_t launch_f6_pack(const void *q4, const void *q8, const void *scale, int64_t rows, int K, int O,
                          void *out, hipStream_t stream);
hipError_t launch_f6_gemm(const void *a_pk, int64_t M, const void *w_pk, int64_t N, int K, int O, void *y,
                          int64_t ldy, int32_t *partials, hipStream_t stream);

// Measurement helper (atom_probe.hip): a loop of MFMAs only; kind 0 = INT8 32x32x32, 1 = FP6 32x32x64.
double     mfma_rate_probe_ops(int kind, int iters);
hipError_t launch_mfma_rate_probe(int kind, int iters, void *out, hipStream_t stream);

// MX variant: front end (FP4 / FP8 codes, E8M0 scale byte per 32 channels) and GEMM on the
// scaled FP8/FP6/FP4 MFMA.
// The front end writing the packed GEMM's unit images directly (atom_quantize_packed.hip); pre as
// launch_quantize_rows.
size_t quantize_packed_lds_bytes(int K, int O, bool norm, bool ident);
hipError_t launch_quantize_rows_packed(const void *x, int64_t rows, int64_t ld, int pre, const void *res, int64_t ldr,
                                       void *sum_out, int64_t ldo, const void *gamma, float eps, const int32_t *idx,
                                       int K, int O, int nbits, float clip, void *out, hipStream_t stream);

// out[r, :] = in[row_idx[r], :] over fp16 matrices (offline helper of the fused reorder).
hipError_t launch_permute_rows(const void *in, int64_t rows_in, int64_t rows_out, int64_t cols, int64_t ld_in,
                               const int32_t *row_idx, void *out, int64_t ld_out, hipStream_t stream);

// One-launch decode linear (atom_decode_fused.hip): front end in the prologue of the
// weight-streaming GEMM, M <= 16.
size_t decode_linear_lds_bytes(int M, int K, int O, bool norm, bool ident);
hipError_t launch_decode_linear(const void *x, int M, int64_t ldx, const void *gamma, float eps,
                                const int32_t *idx, int K, int O, int nbits, float clip,
                                const void *w_q4, const void *w_q8, const void *w_scale, int64_t N,
                                void *y, int64_t ldy, void *dbg_q4, void *dbg_q8, void *dbg_scale,
                                hipStream_t stream);

// The one-launch decode linear with the front end done once by the first M workgroups (see
// atom_decode_fused.hip); a_q4 / a_q8 / a_scale are outputs, sync decode_linear_coop_sync_bytes()
// zeroed bytes.
size_t     decode_linear_coop_sync_bytes();
bool       decode_linear_coop_supported(int M, int K, int O, const void *a_scale, const void *w_scale, int64_t N);
hipError_t launch_decode_linear_coop(const void *x, int M, int64_t ldx, const void *gamma, float eps,
                                     const int32_t *idx, int K, int O, int nbits, float clip,
                                     const void *w_q4, const void *w_q8, const void *w_scale, int64_t N,
                                     void *y, int64_t ldy, void *a_q4, void *a_q8, void *a_scale, void *sync,
                                     hipStream_t stream);

hipError_t launch_quantize_rows_mx(const void *x, int64_t rows, int64_t ld, const void *gamma,
                                   float eps, const int32_t *idx, int K, int O, float clip, void *q4,
                                   void *q8, void *e8, hipStream_t stream);
hipError_t launch_mx_gemm(const void *a_q4, const void *a_q8, const void *a_e8, int64_t M,
                          const void *w_q4, const void *w_q8, const void *w_e8, int64_t N, int K,
                          int O, void *y, int64_t ldy, hipStream_t stream);

// Offline calibration: per-channel square sums and the reorder index.
size_t     calibrate_workspace_bytes(int64_t T, int K);
hipError_t launch_calibrate_reorder(const void *x, int64_t T, int64_t ldx, int K, void *workspace,
                                    int32_t *idx, hipStream_t stream);

// KV cache: asymmetric INT4 rows of D = 64 or 128 values; decode attention over the cache.
hipError_t launch_kv_quantize(const void *x, int64_t R, int64_t ldx, int D, float clip,
                              const int32_t *pos, int32_t rows_per_seq, int64_t Tmax, void *q,
                              void *scale, void *zero, hipStream_t stream,
                              // optional second tensor and cache, same rows and positions
                              const void *x2 = nullptr, void *q2 = nullptr, void *scale2 = nullptr,
                              void *zero2 = nullptr);
hipError_t launch_decode_attention_kv4(const void *q, int B, int H, int Hkv, int64_t Tmax,
                                       const int32_t *seq_len, const void *kq, const void *ks,
                                       const void *kz, const void *vq, const void *vs,
                                       const void *vz, float sm_scale, void *out, void *workspace,
                                       hipStream_t stream);
size_t     decode_attention_workspace_bytes(int B, int H, int Hkv, int64_t Tmax);
// The library's own per-GPU scratch array (for the entry point that allocates nothing): its size,
// and its device address on the current device (looked up on the first call per device).
size_t     static_scratch_bytes();
hipError_t static_scratch(void **ptr);

}  // namespace atom_internal
#endif
