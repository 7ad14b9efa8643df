// Weight-streaming variant of the group GEMM for decode-sized M (M <= 64).
//
// Same arithmetic as atom_gemm.hip (Section 4.2 of the paper, steps 1-3), except
// that the per-group terms of one output are summed in a fixed tree (eight K-slices,
// each in ascending group order, then slices 0..7) instead of one ascending chain.
//
// At these sizes the kernel is bound by reading the packed weights once from HBM
// (Section 3 of the paper: small-batch dense layers are memory-bound), so the
// layout of the work follows the weight bytes:
//   * a workgroup (8 wavefronts) owns 16 output channels = 16 weight rows, all of K;
//     N/16 workgroups keep every CU busy even at N = 4096;
//   * wavefront w owns a contiguous run of groups of those rows (split-K inside the
//     workgroup); it fetches its weight bytes with one 128-bit load per lane and
//     group (16 rows x 64 bytes per instruction, four groups in flight) and never
//     shares them, so no LDS staging and no barrier sits on the streaming path;
//   * the activation codes (M x K/2 bytes, L2-resident) are fetched per wavefront
//     in the same MFMA register layout; rows >= M are zeros;
//   * the contraction is the INT8 MFMA 16x16x64: one 128-channel INT4 group is two
//     MFMAs (even-position and odd-position codes after the nibble widening), an
//     INT8 group is two MFMAs of 64 channels;
//   * each wavefront dequantises its own groups into fp32 (convert, scale product,
//     fused multiply-add), the eight partial tiles meet in LDS once, at the end.
//
// MFMA 16x16x64 i8 layout: lane l supplies row (l & 15) of its operand and the
// 16 bytes of K-chunk (l >> 4); the result has column (l & 15) in lane l and rows
// 4*(l >> 4) + e in register e = 0..3.  Activations are the row operand.

#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include <stdint.h>

#include "atom_gemm_common.h"

namespace {

using namespace atom_gemm;

typedef unsigned v4u __attribute__((ext_vector_type(4)));

constexpr int NW = 8;                     // wavefronts per workgroup = K-slices
constexpr int NT = NW * 64;
constexpr int TN = 16;                    // output channels per workgroup

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

// RB: 16-row blocks of activations (M <= 16 * RB)
// VS: the wavefronts' runs are whole blocks of four groups (G even), so the four scales of a
//     batch are one 8-byte load per row (instead of four 2-byte loads that several wavefronts
//     request from the same lines); needs 4-byte aligned scale arrays
// Q4: with VS, G is a multiple of four and the scale arrays are 8-byte aligned: every block is a
//     whole one, its scales an aligned piece, and scale number d of the piece belongs to slot d
// ONE8: there is exactly one INT8 group (O = 128, the set-up of the paper), the last group of the
//     last wavefront's run.  The second 64 bytes of its rows then have registers of their own, and
//     the slots hold one 16-byte piece each: 24 registers less per row block, which is what lets two
//     workgroups share a CU once every load of a batch is in flight at the same time.
// TILED (with ONE8): the weight codes were re-tiled for this kernel (tile_weight_kernel below):
//     block of 16 rows, group, lane -> 16 bytes, so one load instruction of a wavefront reads 1 KB
//     of consecutive bytes (eight whole 128-byte lines) instead of sixteen 64-byte pieces.
template <int RB, bool VS, bool ONE8 = false, bool Q4 = false, bool TILED = false>
__global__ __launch_bounds__(NT, (ONE8 && RB == 1 && Q4) ? 6 : 1)    // six wavefronts per SIMD = three workgroups per CU: 80 registers
void w4a4_gemm_decode_kernel(const GemmParams p)
{
    __shared__ float red[NW][RB][4][64];   // [slice][row block][register][lane]
    // groups whose loads are in flight together per wavefront (register budget)
    constexpr int DEPTH = (RB >= 4 && !ONE8) ? 2 : 4;

    const int tid  = threadIdx.x;
    const int lane = tid & 63;
    // (told to be the same in every lane: the INT4 / INT8 decisions below then are scalar branches;
    // as lane-dependent ones they became exec-masked regions, and the compiler waited for the loads
    // of a slot at the end of its region before it issued the next slot's: four memory round trips
    // per wavefront instead of one)
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int col = lane & 15, kc = lane >> 4;

    const int K4 = p.K - p.O, G = p.K >> 7, G4 = K4 >> 7;
    const int64_t n0 = (int64_t)blockIdx.x * TN;

    // this wavefront's run of groups
    // (VS: in whole blocks of four groups, so that a batch's four scales are one 8-byte piece of
    // a scale row that starts on a multiple of four; the last block of K may be a partial one)
    const int nblk    = VS ? (G + 3) >> 2 : G;
    const int g_begin = (VS ? 4 : 1) * (int)((int64_t)wave * nblk / NW);
    const int g_end   = min(G, (VS ? 4 : 1) * (int)((int64_t)(wave + 1) * nblk / NW));

    // weight row of this lane (clamped: rows >= N are computed and never stored)
    int64_t wr = n0 + col;
    wr = wr < p.N ? wr : p.N - 1;
    const uint8_t  *w4 = p.w_q4 + wr * (K4 >> 1) + kc * 16;
    const int8_t   *w8 = p.w_q8 + wr * p.O + kc * 16;
    const uint16_t *ws = p.w_scale + wr * G;
    // activation rows of this lane as the MFMA row operand (row = col index here)
    const uint8_t *a4[RB];
    const int8_t  *a8[RB];
    bool a_ok[RB];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
        const int64_t m = 16 * rb + col;
        a_ok[rb] = m < p.M;
        const int64_t mc = a_ok[rb] ? m : 0;
        a4[rb] = p.a_q4 + mc * (K4 >> 1) + kc * 16;
        a8[rb] = p.a_q8 + mc * p.O + kc * 16;
    }
    // ONE8 addresses every load as scalar base + 32-bit byte offset (arrays below 4 GiB: host),
    // one register per stream instead of a 64-bit pointer per load
    static_assert(!TILED || ONE8, "the tiled layout is read by the one-INT8-group variants");
    constexpr uint32_t GSTEP = TILED ? 1024u : 64u;      // from one group's piece to the next, and to the second half of the INT8 group
    const uint32_t w4o = TILED ? (uint32_t)blockIdx.x * (uint32_t)(G4 * 1024) + lane * 16 : (uint32_t)(wr * (K4 >> 1)) + kc * 16;
    const uint32_t w8o = TILED ? (uint32_t)blockIdx.x * 2048u + lane * 16 : (uint32_t)(wr * p.O) + kc * 16;
    uint32_t a4o[RB], a8o[RB];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
        const int64_t mc = a_ok[rb] ? 16 * rb + col : 0;
        a4o[rb] = (uint32_t)(mc * (K4 >> 1)) + kc * 16;
        a8o[rb] = (uint32_t)(mc * p.O) + kc * 16;
    }
    const uint8_t *w8b = reinterpret_cast<const uint8_t *>(p.w_q8), *a8b = reinterpret_cast<const uint8_t *>(p.a_q8);
    // rows of the result held by this lane: 16*rb + 4*kc + e
    float acc[RB][4];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb)
#pragma unroll
        for (int e = 0; e < 4; ++e) acc[rb][e] = 0.0f;

    const v4i zi = {0, 0, 0, 0};
    const uint4 z4 = make_uint4(0, 0, 0, 0);

    // Groups are processed in batches of DEPTH.  Every load of a batch (weight codes,
    // weight scales, activation codes, activation scales) is issued before the first is
    // used, so a wavefront pays the memory latency once per batch, not once per group.
    for (int gb = g_begin; gb < g_end; gb += DEPTH) {
        constexpr int HALVES = ONE8 ? 1 : 2;
        uint4    wq[DEPTH][HALVES];       // [group][half]: an INT4 group uses half 0 only
        uint4    aq[DEPTH][RB][HALVES];
        uint4    wx, ax[RB];              // ONE8: the second half of the INT8 group (untouched elsewhere)
        uint16_t wsc[DEPTH];
        uint16_t asc[DEPTH][RB][4];
        uint2    wvs, avs[RB][4];         // VS: the four scales of the batch stay packed until they are used
#pragma unroll
        for (int d = 0; d < DEPTH; ++d) {
            const int  g    = gb + d;
            const bool live = g < g_end;
            const int  gc   = live ? g : g_end - 1;         // dead slots re-read the last group
            const bool is4  = gc < G4;
            // (an INT4 slot leaves its second half alone: writing zeros there made the compiler wait
            // for every load in flight, since one of an earlier batch might still target the register)
            if constexpr (ONE8) {         // one load per slot: array and offset are scalar selects
                wq[d][0] = *reinterpret_cast<const uint4 *>((is4 ? p.w_q4 : w8b) + (is4 ? w4o + (uint32_t)gc * GSTEP : w8o));
            } else if (is4) {
                wq[d][0] = *reinterpret_cast<const uint4 *>(w4 + (size_t)gc * 64);
            } else {
                wq[d][0] = *reinterpret_cast<const uint4 *>(w8 + (size_t)(gc - G4) * 128);
                wq[d][1] = *reinterpret_cast<const uint4 *>(w8 + (size_t)(gc - G4) * 128 + 64);
            }
            if constexpr (!VS) wsc[d] = ws[gc];
#pragma unroll
            for (int rb = 0; rb < RB; ++rb) {
                // rows >= M load row 0 (no lane-dependent branch around a load) and are zeroed below
                if constexpr (ONE8) {
                    aq[d][rb][0] = *reinterpret_cast<const uint4 *>((is4 ? p.a_q4 : a8b) + (is4 ? a4o[rb] + (uint32_t)gc * 64u : a8o[rb]));
                } else if (is4) {
                    aq[d][rb][0] = *reinterpret_cast<const uint4 *>(a4[rb] + (size_t)gc * 64);
                } else {
                    aq[d][rb][0] = *reinterpret_cast<const uint4 *>(a8[rb] + (size_t)(gc - G4) * 128);
                    aq[d][rb][1] = *reinterpret_cast<const uint4 *>(a8[rb] + (size_t)(gc - G4) * 128 + 64);
                }
                if constexpr (!VS) {
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const int64_t m = 16 * rb + 4 * kc + e;
                        asc[d][rb][e] = m < p.M ? p.a_scale[m * G + gc] : (uint16_t)0;
                    }
                }
            }
        }
        if constexpr (ONE8) {
            // Unconditional (a branch around these loads made the compiler wait for them inside it):
            // a batch without the INT8 group reads the first piece of its first group once more.
            const bool has8 = g_end > G4 && gb + DEPTH >= g_end;
            const int  g0   = gb < G4 ? gb : G4 - 1;
            wx = *reinterpret_cast<const uint4 *>((has8 ? w8b : p.w_q4) + (has8 ? w8o + GSTEP : w4o + (uint32_t)g0 * GSTEP));
#pragma unroll
            for (int rb = 0; rb < RB; ++rb)
                ax[rb] = *reinterpret_cast<const uint4 *>((has8 ? a8b : p.a_q4) + (has8 ? a8o[rb] + 64u : a4o[rb] + (uint32_t)g0 * 64u));
        }
        if constexpr (VS) {
            static_assert(!VS || DEPTH == 4, "a batch is four groups");
            // (32-bit element offsets on the scalar bases: M * G and N * G are far below 2^31)
            // Q4: one aligned 8-byte piece.  Otherwise a row of scales starts on an even element
            // (G even) and its four-blocks on 4-byte boundaries: two 4-byte loads, the second one
            // held inside the row where the last block of K has two groups only (its slots are dead).
            const int g2 = gb + 2 <= G - 2 ? gb + 2 : G - 2;
            // (scalar base + 32-bit byte offset per lane, like the codes)
            auto load4 = [&](const uint16_t *base, uint32_t row) {
                const uint8_t *sb  = reinterpret_cast<const uint8_t *>(base);
                const uint32_t off = row * (uint32_t)(2 * G);
                if constexpr (Q4) return *reinterpret_cast<const uint2 *>(base + (row * (uint32_t)G + (uint32_t)gb));
                else return make_uint2(*reinterpret_cast<const uint32_t *>(sb + 2 * gb + off),
                                       *reinterpret_cast<const uint32_t *>(sb + 2 * g2 + off));
            };
            wvs = load4(p.w_scale, (uint32_t)wr);
#pragma unroll
            for (int rb = 0; rb < RB; ++rb)
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int64_t m = 16 * rb + 4 * kc + e;
                    // rows >= M: row 0 is read (no lane-dependent branch around a load), zeros are used
                    uint2 av = load4(p.a_scale, (uint32_t)(m < p.M ? m : 0));
                    if (m >= p.M) av = make_uint2(0, 0);
                    avs[rb][e] = av;
                }
        }
#pragma unroll
        for (int d = 0; d < DEPTH; ++d) {
            const int g = gb + d;
            if (g >= g_end) break;
            const bool is4 = g < G4;
            v4i b0, b1;
            if (is4) { b0 = widen_lo(wq[d][0]); b1 = widen_hi(wq[d][0]); }
            else     { b0 = __builtin_bit_cast(v4i, wq[d][0]); b1 = __builtin_bit_cast(v4i, ONE8 ? wx : wq[d][HALVES - 1]); }
            // 2^-8 of the nibble widening folded into the weight scale (exact)
            // scale number d of a packed four
            const int sidx = d;
            auto unpack = [&](const uint2 &v) { return (uint16_t)((sidx < 2 ? v.x : v.y) >> (16 * (sidx & 1))); };
            const float wsf = half_bits_to_float(VS ? unpack(wvs) : wsc[d]) * (is4 ? (1.0f / 256.0f) : 1.0f);
#pragma unroll
            for (int rb = 0; rb < RB; ++rb) {
                v4i x0, x1;
                if (is4) { x0 = widen_lo(aq[d][rb][0]); x1 = widen_hi(aq[d][rb][0]); }
                else     { x0 = __builtin_bit_cast(v4i, aq[d][rb][0]); x1 = __builtin_bit_cast(v4i, ONE8 ? ax[rb] : aq[d][rb][HALVES - 1]); }
                if (!a_ok[rb]) { x0 = zi; x1 = zi; }
                v4i c = __builtin_amdgcn_mfma_i32_16x16x64_i8(x0, b0, zi, 0, 0, 0);
                c = __builtin_amdgcn_mfma_i32_16x16x64_i8(x1, b1, c, 0, 0, 0);
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    acc[rb][e] = fmaf((float)c[e], half_bits_to_float(VS ? unpack(avs[rb][e]) : asc[d][rb][e]) * wsf, acc[rb][e]);
            }
        }
    }

    // the eight K-slices meet in LDS and are added in slice order
#pragma unroll
    for (int rb = 0; rb < RB; ++rb)
#pragma unroll
        for (int e = 0; e < 4; ++e) red[wave][rb][e][lane] = acc[rb][e];
    __syncthreads();
    for (int idx = tid; idx < RB * 4 * 64; idx += NT) {
        const int l = idx & 63, e = (idx >> 6) & 3, rb = idx >> 8;
        float s = 0.0f;
#pragma unroll
        for (int w = 0; w < NW; ++w) s += red[w][rb][e][l];
        const int64_t m = 16 * rb + 4 * (l >> 4) + e;
        const int64_t n = n0 + (l & 15);
        if (m < p.M && n < p.N) p.y[m * p.ldy + n] = __half_as_ushort(__float2half_rn(s));
    }
}

// Re-tiling of the canonical weight codes for the TILED variants: one workgroup per block of 16
// rows; rows past N are zeros.
__global__ __launch_bounds__(256)
void tile_weight_kernel(const uint8_t *__restrict__ q4, const int8_t *__restrict__ q8, int64_t N, int K4h, int O,
                        uint8_t *__restrict__ t4, uint8_t *__restrict__ t8)
{
    const int64_t blk = blockIdx.x;
    const int G4 = K4h >> 6, G8 = O >> 7;
    // INT4: piece p = (group, lane) -> row blk*16 + (lane & 15), bytes [64 g + 16 (lane >> 4), +16)
    for (int p = threadIdx.x; p < G4 * 64; p += 256) {
        const int g = p >> 6, l = p & 63;
        const int64_t row = blk * 16 + (l & 15);
        uint4 v = make_uint4(0, 0, 0, 0);
        if (row < N) v = *reinterpret_cast<const uint4 *>(q4 + row * K4h + g * 64 + (l >> 4) * 16);
        *reinterpret_cast<uint4 *>(t4 + (blk * G4 + g) * 1024 + l * 16) = v;
    }
    // INT8: piece (group, half, lane) -> row, bytes [128 g + 64 half + 16 (lane >> 4), +16)
    for (int p = threadIdx.x; p < G8 * 128; p += 256) {
        const int g = p >> 7, h = (p >> 6) & 1, l = p & 63;
        const int64_t row = blk * 16 + (l & 15);
        uint4 v = make_uint4(0, 0, 0, 0);
        if (row < N) v = *reinterpret_cast<const uint4 *>(q8 + row * O + g * 128 + h * 64 + (l >> 4) * 16);
        *reinterpret_cast<uint4 *>(t8 + ((blk * G8 + g) * 2 + h) * 1024 + l * 16) = v;
    }
}

}  // namespace

namespace atom_gemm {

hipError_t launch_tile_weight(const void *q4, const void *q8, int64_t N, int K, int O, void *t4, void *t8,
                              hipStream_t stream)
{
    hipLaunchKernelGGL(tile_weight_kernel, dim3((unsigned)((N + TN - 1) / TN)), dim3(256), 0, stream,
                       (const uint8_t *)q4, (const int8_t *)q8, N, (K - O) >> 1, O, (uint8_t *)t4, (uint8_t *)t8);
    return hipGetLastError();
}

// What the tiled variants need: one INT8 group that is the last group of the last wavefront's run,
// whole blocks of four groups with 8-byte aligned scale rows, M <= 64.
bool decode_tiled_supported(const GemmParams &p)
{
    const int G = p.K >> 7;
    return p.M <= 64 && p.O == 128 && G >= NW && G % 4 == 0 &&
           ((reinterpret_cast<uintptr_t>(p.a_scale) | reinterpret_cast<uintptr_t>(p.w_scale)) & 7) == 0 &&
           (uint64_t)(p.N + TN) * (uint64_t)(p.K >> 1) < (1ull << 32) && (uint64_t)p.N * (uint64_t)G < (1ull << 31);
}

hipError_t launch_decode_tiled(const GemmParams &p, hipStream_t stream)
{
    const unsigned blocks = (unsigned)((p.N + TN - 1) / TN);
    if (p.M <= 16)      hipLaunchKernelGGL((w4a4_gemm_decode_kernel<1, true, true, true, true>), dim3(blocks), dim3(NT), 0, stream, p);
    else if (p.M <= 32) hipLaunchKernelGGL((w4a4_gemm_decode_kernel<2, true, true, true, true>), dim3(blocks), dim3(NT), 0, stream, p);
    else                hipLaunchKernelGGL((w4a4_gemm_decode_kernel<4, true, true, true, true>), dim3(blocks), dim3(NT), 0, stream, p);
    return hipGetLastError();
}

hipError_t launch_decode(const GemmParams &p, hipStream_t stream)
{
    const unsigned blocks = (unsigned)((p.N + TN - 1) / TN);
    // vector scale loads: G even (a scale row then starts on a 4-byte boundary), both scale arrays
    // 4-byte aligned
    const int  G  = p.K >> 7;
    const bool vs = G % 2 == 0 && G >= 4 && ((reinterpret_cast<uintptr_t>(p.a_scale) | reinterpret_cast<uintptr_t>(p.w_scale)) & 3) == 0 &&
                    (uint64_t)p.N * (uint64_t)G < (1ull << 31);          // 32-bit scale offsets
    // exactly one INT8 group, and it is the last group of the last wavefront's run (G >= 8)
    const bool one8 = p.O == 128 && G >= NW && (uint64_t)p.N * (uint64_t)(p.K >> 1) < (1ull << 32);   // 32-bit byte offsets
    const bool q4 = G % 4 == 0 && ((reinterpret_cast<uintptr_t>(p.a_scale) | reinterpret_cast<uintptr_t>(p.w_scale)) & 7) == 0;
    if (p.M <= 16 && vs && one8) {
        if (q4) hipLaunchKernelGGL((w4a4_gemm_decode_kernel<1, true, true, true>), dim3(blocks), dim3(NT), 0, stream, p);
        else    hipLaunchKernelGGL((w4a4_gemm_decode_kernel<1, true, true>), dim3(blocks), dim3(NT), 0, stream, p);
    } else if (p.M <= 32 && vs && one8) {
        if (q4) hipLaunchKernelGGL((w4a4_gemm_decode_kernel<2, true, true, true>), dim3(blocks), dim3(NT), 0, stream, p);
        else    hipLaunchKernelGGL((w4a4_gemm_decode_kernel<2, true, true>), dim3(blocks), dim3(NT), 0, stream, p);
    } else if (vs && one8) {
        if (q4) hipLaunchKernelGGL((w4a4_gemm_decode_kernel<4, true, true, true>), dim3(blocks), dim3(NT), 0, stream, p);
        else    hipLaunchKernelGGL((w4a4_gemm_decode_kernel<4, true, true>), dim3(blocks), dim3(NT), 0, stream, p);
    } else if (p.M <= 16) {
        if (vs) hipLaunchKernelGGL((w4a4_gemm_decode_kernel<1, true>), dim3(blocks), dim3(NT), 0, stream, p);
        else    hipLaunchKernelGGL((w4a4_gemm_decode_kernel<1, false>), dim3(blocks), dim3(NT), 0, stream, p);
    } else if (p.M <= 32) {
        if (vs) hipLaunchKernelGGL((w4a4_gemm_decode_kernel<2, true>), dim3(blocks), dim3(NT), 0, stream, p);
        else    hipLaunchKernelGGL((w4a4_gemm_decode_kernel<2, false>), dim3(blocks), dim3(NT), 0, stream, p);
    } else {
        hipLaunchKernelGGL((w4a4_gemm_decode_kernel<4, false>), dim3(blocks), dim3(NT), 0, stream, p);
    }
    return hipGetLastError();
}

}  // namespace atom_gemm
