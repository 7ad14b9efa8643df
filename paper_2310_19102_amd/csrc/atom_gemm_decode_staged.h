// The decode-sized group GEMM for one block of activation rows (M <= 16), as a routine: the
// stand-alone kernel (atom_gemm_decode.hip) and the one-launch decode linear
// (atom_decode_fused.hip) both run it, so their sums agree by construction.
#ifndef ATOM_GEMM_DECODE_STAGED_H
#define ATOM_GEMM_DECODE_STAGED_H

#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include <stdint.h>

#include <type_traits>

#include "atom_gemm_common.h"

namespace atom_decode_staged {

using namespace atom_gemm;

typedef unsigned v4u __attribute__((ext_vector_type(4)));

constexpr int NW = 8;                     // wavefronts per workgroup = K-slices
constexpr int NT = NW * 64;
constexpr int TN = 16;                    // output channels per workgroup
constexpr int kStageRow   = 272;          // a staged row: 256 bytes and 16 that spread the rows over the banks
constexpr int kStageWave  = 16 * kStageRow;        // per wavefront
constexpr int kStageBytes = NW * kStageWave;       // LDS of a workgroup

__device__ __forceinline__ v4i widen_lo(const uint4 &w)
{
    v4u t = {(w.x << 4) & 0xF0F0F0F0u, (w.y << 4) & 0xF0F0F0F0u, (w.z << 4) & 0xF0F0F0F0u,
             (w.w << 4) & 0xF0F0F0F0u};
    return __builtin_bit_cast(v4i, t);
}
__device__ __forceinline__ v4i widen_hi(const uint4 &w)
{
    v4u t = {w.x & 0xF0F0F0F0u, w.y & 0xF0F0F0F0u, w.z & 0xF0F0F0F0u, w.w & 0xF0F0F0F0u};
    return __builtin_bit_cast(v4i, t);
}

typedef _Float16 v4h16 __attribute__((ext_vector_type(4)));
typedef float    v4f32 __attribute__((ext_vector_type(4)));

// Scale operand of group D of a batch: the fp16 number in k-slot 0 (lanes 0-15 hold k-slots 0-3;
// the pieces of the other lanes were zeroed), zeros in slots 1-3.
template <int D>
__device__ __forceinline__ v4h16 scale_operand(const uint2 &piece)
{
    const uint32_t r = D < 2 ? piece.x : piece.y;
    return __builtin_bit_cast(v4h16, make_uint2((D & 1) ? r >> 16 : r & 0xffffu, 0u));
}

// The (up to) four scales of the batch that starts at group gb of scale row `row_off` (in elements).
// A8: one aligned 8-byte piece.  Otherwise the row starts on an even element and the batch on a
// multiple of four: two 4-byte loads, the second held inside the row where the batch is the last
// block of two groups.
template <bool A8>
__device__ __forceinline__ uint2 load_scales(const uint16_t *base, uint32_t row_off, int gb, int G)
{
    if constexpr (A8) return *reinterpret_cast<const uint2 *>(base + (row_off + (uint32_t)gb));
    const int g2 = gb + 2 <= G - 2 ? gb + 2 : G - 2;
    return make_uint2(*reinterpret_cast<const uint32_t *>(base + (row_off + (uint32_t)gb)),
                      *reinterpret_cast<const uint32_t *>(base + (row_off + (uint32_t)g2)));
}

// Which variant of the common decoding case a problem is (host side).
// 3: G a multiple of four, scale rows 8-byte aligned; 1: G = 4 j + 2, scale rows 4-byte aligned; 0: neither.
// In both cases: exactly one INT8 group that is the last group of the last wavefront's run (G >= 8),
// M <= max_rows (the kernels take blocks of 64 rows; more than 256 rows are the tiled kernels' business),
// 32-bit offsets.
constexpr int kDecodeMaxRows = 256;       // four blocks of 64 rows
inline int common_tail(const GemmParams &p, int max_rows = kDecodeMaxRows)
{
    const int G = p.K >> 7;
    const uintptr_t al = reinterpret_cast<uintptr_t>(p.a_scale) | reinterpret_cast<uintptr_t>(p.w_scale);
    if (!(p.M <= max_rows && p.O == 128 && G >= NW && (uint64_t)(p.N + TN) * (uint64_t)(p.K >> 1) < (1ull << 32) &&
          (uint64_t)p.N * (uint64_t)G < (1ull << 31)))
        return 0;
    if (G % 4 == 0 && (al & 7) == 0) return 3;
    if (G % 4 == 2 && (al & 3) == 0) return 1;
    return 0;
}

struct NoWait {
    __device__ __forceinline__ void early() const {}
    __device__ __forceinline__ void wait() const {}
    __device__ __forceinline__ void passed() const {}
};

// The routine.  Cases: M <= 16, O = 128 (one INT8 group, the last group of K), 32-bit offsets, and
// either G a multiple of four with 8-byte aligned scale rows (TAIL = 3) or G = 4 j + 2 with 4-byte
// aligned ones (TAIL = 1); weight codes canonical or re-tiled (TILED).  Arithmetic and order of the
// sums are those of w4a4_gemm_decode16_kernel (atom_gemm_decode.hip, whose header explains them:
// eight K-slices of four-group blocks, scale products on an fp16 MFMA, an accumulator that holds
// 256 x the sum, the batch with the INT8 group as code of its own).
// What it adds: an MFMA operand is 16 rows whatever M is, as many bytes returned to registers as
// the weights.  Here a wavefront copies the M real rows of its batch's activation codes (256
// bytes per row: four groups) into a region of LDS of its own, four rows per load instruction (SI
// instructions), and reads its operand from there; rows >= M of the operand repeat row 0.  No
// barrier: LDS instructions of one wavefront execute in order.
//
// `block`: which 16 output channels; `stage`: kStageBytes of LDS, 16-byte aligned.
// LATE: the activation codes and scales are not ready when the workgroup starts (another workgroup
// of the same launch writes them): sync.early() runs (a first look whose answer returns before
// the weights: loads return in order), the weights are requested, then sync.wait() runs once
// per wavefront (it must end with whatever makes the other workgroup's stores visible), then the
// activations are requested, then sync.passed() runs (the wavefront will not wait again).
template <int SI, bool TILED, int TAIL, bool LATE, class Wait>
__device__ __forceinline__
void decode_staged_body(const GemmParams &p, int block, unsigned char *stage, Wait sync)
{
    constexpr int ROWB = kStageRow, WREG = kStageWave;

    const int tid  = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int col = lane & 15, kc = lane >> 4;

    const int K4 = p.K - 128, G = p.K >> 7;
    const int M = (int)p.M;
    const int64_t n0 = (int64_t)block * TN;
    constexpr bool A8 = TAIL == 3;
    const int nblk    = (G + 3) >> 2;
    const int g_begin = 4 * (int)((int64_t)wave * nblk / NW);
    const int g_end   = min(G, 4 * (int)((int64_t)(wave + 1) * nblk / NW));

    int64_t wr = n0 + col;                                // clamped: columns >= N are computed and never stored
    wr = wr < p.N ? wr : p.N - 1;
    constexpr uint32_t GSTEP = TILED ? 1024u : 64u;
    const uint32_t w4o = TILED ? (uint32_t)block * (uint32_t)((G - 1) * 1024) + lane * 16 : (uint32_t)(wr * (K4 >> 1)) + kc * 16;
    const uint32_t w8o = TILED ? (uint32_t)block * 2048u + lane * 16 : (uint32_t)(wr * 128) + kc * 16;
    const uint8_t *w8b = reinterpret_cast<const uint8_t *>(p.w_q8), *a8b = reinterpret_cast<const uint8_t *>(p.a_q8);
    // staging: instruction i moves rows 4 i .. 4 i + 3, lane -> row 4 i + kc, 16-byte chunk `col` of
    // the row's 256 bytes; rows >= M repeat row M - 1
    uint32_t srow[SI];
#pragma unroll
    for (int i = 0; i < SI; ++i) srow[i] = (uint32_t)(4 * i + kc < M ? 4 * i + kc : M - 1) * (uint32_t)(K4 >> 1);
    unsigned char *mine = stage + wave * WREG;
    unsigned char *st_w = mine + kc * ROWB + col * 16;                        // + 4 i ROWB
    const uint32_t ar = col < M ? col : 0;                                    // operand row of this lane
    const unsigned char *st_r = mine + ar * ROWB + kc * 16;                   // + 64 d
    const uint32_t a8o = ar * 128u + kc * 16;
    const uint32_t wso = (uint32_t)wr * (uint32_t)G, aso = ar * (uint32_t)G;

    float acc[4] = {0.0f, 0.0f, 0.0f, 0.0f};
    bool  waited = false;                     // LATE: the wait comes once, with the wavefront's first batch
    const v4i   zi = {0, 0, 0, 0};
    const v4f32 zf = {0.0f, 0.0f, 0.0f, 0.0f};

    auto batch = [&](int gb, auto has8_c) __attribute__((always_inline)) {
        constexpr bool HAS8 = decltype(has8_c)::value;
        // Every load of the batch is issued before the first is used.  The activation rows come first
        // (they go through LDS and must not wait for the weights: loads return in order), then the
        // scales, then the weights; with LATE the weights and their scales, then the wait for the
        // activations, then those.
        // (named registers, not an array: the array stayed in scratch memory)
        uint4 st0, st1, st2, st3;
        constexpr int NG4 = HAS8 ? TAIL : 4;                                  // INT4 groups of the batch
        const uint32_t ch = col < 4 * NG4 ? col : 4 * NG4 - 1;               // their 64-byte pieces: 4 NG4 chunks of a row
        auto stage_load = [&](int i) __attribute__((always_inline)) {
            return *reinterpret_cast<const uint4 *>(p.a_q4 + (srow[i] + (uint32_t)gb * 64u + ch * 16u));
        };
        uint2 avs, wvs;
        uint4 wq[4], wx, a8[2];
        auto load_activations = [&]() __attribute__((always_inline)) {
            st0 = stage_load(0);
            if constexpr (SI > 1) st1 = stage_load(1);
            if constexpr (SI > 2) { st2 = stage_load(2); st3 = stage_load(3); }
            avs = load_scales<A8>(p.a_scale, aso, gb, G);
            if constexpr (HAS8) {
                a8[0] = *reinterpret_cast<const uint4 *>(a8b + a8o);
                a8[1] = *reinterpret_cast<const uint4 *>(a8b + (a8o + 64u));
            }
        };
        auto load_weights = [&]() __attribute__((always_inline)) {
            wvs = load_scales<A8>(p.w_scale, wso, gb, G);
#pragma unroll
            for (int d = 0; d < NG4; ++d) wq[d] = *reinterpret_cast<const uint4 *>(p.w_q4 + (w4o + (uint32_t)(gb + d) * GSTEP));
            if constexpr (HAS8) {
                wq[TAIL] = *reinterpret_cast<const uint4 *>(w8b + w8o);
                wx       = *reinterpret_cast<const uint4 *>(w8b + (w8o + GSTEP));
            }
        };
        if constexpr (LATE) {
            if (!waited) sync.early();
            load_weights();
            if (!waited) sync.wait();
            load_activations();
            if (!waited) { sync.passed(); waited = true; }
        } else {
            load_activations();
            load_weights();
        }
        // (the fence keeps the loads here: left alone the compiler spreads them between the MFMAs
        // to save registers, which turns one memory round trip per batch into several)
        __builtin_amdgcn_sched_barrier(0);
        *reinterpret_cast<uint4 *>(st_w) = st0;
        if constexpr (SI > 1) *reinterpret_cast<uint4 *>(st_w + 4 * ROWB) = st1;
        if constexpr (SI > 2) { *reinterpret_cast<uint4 *>(st_w + 8 * ROWB) = st2; *reinterpret_cast<uint4 *>(st_w + 12 * ROWB) = st3; }
        uint4 aq[4];
#pragma unroll
        for (int d = 0; d < NG4; ++d) aq[d] = *reinterpret_cast<const uint4 *>(st_r + 64 * d);
        if (kc != 0) { avs = make_uint2(0, 0); wvs = make_uint2(0, 0); }     // k-slots 4 .. 15 of the scale MFMA stay empty

        auto scales = [&](auto dc) __attribute__((always_inline)) -> v4f32 {
            constexpr int D = decltype(dc)::value;
            return __builtin_amdgcn_mfma_f32_16x16x16f16(scale_operand<D>(avs), scale_operand<D>(wvs), zf, 0, 0, 0);
        };
        auto int4_group = [&](const uint4 &w, const uint4 &a, auto dc) __attribute__((always_inline)) {
            v4i c = __builtin_amdgcn_mfma_i32_16x16x64_i8(widen_lo(a), widen_lo(w), zi, 0, 0, 0);
            c = __builtin_amdgcn_mfma_i32_16x16x64_i8(widen_hi(a), widen_hi(w), c, 0, 0, 0);
            const v4f32 sc = scales(dc);
#pragma unroll
            for (int e = 0; e < 4; ++e) acc[e] = fmaf((float)c[e], sc[e], acc[e]);
        };
        int4_group(wq[0], aq[0], std::integral_constant<int, 0>());
        if constexpr (NG4 > 1) int4_group(wq[1], aq[1], std::integral_constant<int, 1>());
        if constexpr (NG4 > 2) int4_group(wq[2], aq[2], std::integral_constant<int, 2>());
        if constexpr (NG4 > 3) int4_group(wq[3], aq[3], std::integral_constant<int, 3>());
        if constexpr (HAS8) {
            v4i c = __builtin_amdgcn_mfma_i32_16x16x64_i8(__builtin_bit_cast(v4i, a8[0]), __builtin_bit_cast(v4i, wq[TAIL]), zi, 0, 0, 0);
            c = __builtin_amdgcn_mfma_i32_16x16x64_i8(__builtin_bit_cast(v4i, a8[1]), __builtin_bit_cast(v4i, wx), c, 0, 0, 0);
            const v4f32 sc = scales(std::integral_constant<int, TAIL>());
#pragma unroll
            for (int e = 0; e < 4; ++e) acc[e] = fmaf((float)c[e], 256.0f * sc[e], acc[e]);   // the accumulator holds 256 x the sum
        }
    };

    const int g_plain = wave == NW - 1 ? g_end - (TAIL + 1) : g_end;
    for (int gb = g_begin; gb < g_plain; gb += 4) batch(gb, std::false_type());
    if (wave == NW - 1) batch(G - (TAIL + 1), std::true_type());

    // the eight K-slices meet in LDS (each wavefront's region, its operand reads are complete) and
    // are added in slice order
    float *red = reinterpret_cast<float *>(mine);
#pragma unroll
    for (int e = 0; e < 4; ++e) red[e * 64 + lane] = acc[e] * (1.0f / 256.0f);
    __syncthreads();
    if (tid < 256) {
        const int l = tid & 63, e = tid >> 6;
        float s = 0.0f;
#pragma unroll
        for (int w = 0; w < NW; ++w) s += reinterpret_cast<const float *>(stage + w * WREG)[e * 64 + l];
        const int64_t m = 4 * (l >> 4) + e;
        const int64_t n = n0 + (l & 15);
        if (m < p.M && n < p.N) p.y[m * p.ldy + n] = __half_as_ushort(__float2half_rn(s));
    }
}


}  // namespace atom_decode_staged
#endif
