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
//     in the same MFMA register layout (at M <= 16 in the common case: the real rows
//     only, through a copy in LDS); rows >= M are zeros or never stored;
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

#include <type_traits>

#include "atom_gemm_common.h"
#include "atom_gemm_decode_staged.h"
#include "atom_launch.h"

namespace {

using namespace atom_gemm;

using namespace atom_decode_staged;        // NW, NT, TN and the helpers shared with the one-launch decode linear

// The general kernel.
// RB: 16-row blocks of activations (M <= 16 * RB)
// VS: the wavefronts' runs are whole blocks of four groups (G even), so the four scales of a
//     batch are one 8-byte load per row (instead of four 2-byte loads that several wavefronts
//     request from the same lines); needs 4-byte aligned scale arrays
// ONE8: there is exactly one INT8 group (O = 128, the set-up of the paper), the last group of the
//     last wavefront's run.  The second 64 bytes of its rows then have registers of their own, and
//     the slots hold one 16-byte piece each.
// The common decoding case (ONE8, G a multiple of four, 8-byte aligned scale rows) has kernels of
// its own below; this one takes everything else.
template <int RB, bool VS, bool ONE8 = false>
__global__ __launch_bounds__(NT, 1)
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
    constexpr uint32_t GSTEP = 64u;                      // from one group's piece to the next, and to the second half of the INT8 group
    const uint32_t w4o = (uint32_t)(wr * (K4 >> 1)) + kc * 16;
    const uint32_t w8o = (uint32_t)(wr * p.O) + kc * 16;
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
            // A row of scales starts on an even element (G even) and its four-blocks on 4-byte
            // boundaries: two 4-byte loads, the second one held inside the row where the last block
            // of K has two groups only (its slots are dead).
            const int g2 = gb + 2 <= G - 2 ? gb + 2 : G - 2;
            // (scalar base + 32-bit byte offset per lane, like the codes)
            auto load4 = [&](const uint16_t *base, uint32_t row) {
                const uint8_t *sb  = reinterpret_cast<const uint8_t *>(base);
                const uint32_t off = row * (uint32_t)(2 * G);
                return make_uint2(*reinterpret_cast<const uint32_t *>(sb + 2 * gb + off),
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

// The cases decoding runs in, written out on their own: RB blocks of 16 activation rows per
// workgroup (blockIdx.y says which 16 RB rows: up to four sets of workgroups, 256 rows), O = 128 (one INT8 group, the last group of K), 32-bit offsets, and either G a
// multiple of four with 8-byte aligned scale rows (TAIL = 3: the last block of four is three INT4
// groups and the INT8 group; the four scales of a batch are one 8-byte load) or G = 4 j + 2 with
// 4-byte aligned scale rows (TAIL = 1: the last block is one INT4 group and the INT8 group; two
// 4-byte loads).  Same sums in the same order as w4a4_gemm_decode_kernel<RB, true,
// true> (eight K-slices of whole four-group blocks, ascending inside a slice, slices added
// 0..7), so the two agree bit for bit.  What differs is the vector work per weight byte and the
// bytes the vector memory path returns to registers (64 per clock and CU), which set the pace here:
//   * a batch is four INT4 groups; the batch that holds the INT8 group (the last block of K, in
//     the last wavefront) is code of its own: no per-slot case analysis, no second half of an INT8 group
//     loaded where there is none;
//   * rows >= M are not zeroed in the operand: an MFMA row depends on its own operand row only, and
//     those rows are never stored;
//   * the accumulator holds 256 x the sum (the nibble widening's factor stays in; the INT8 group's
//     scale products are multiplied by 256 instead, an exact scaling): one multiplication per
//     wavefront at the end instead of one per group;
//   * the scale products of a group and row block are one fp16 MFMA (activation scales of the
//     operand rows against the weight scales of the columns, both in k-slot 0: the result has the
//     layout of the integer tile; a product of two fp16 numbers is exact in fp32), so a lane loads
//     one 8-byte piece of activation scales per batch and row block, not four;
//   * CB blocks of 16 output channels per workgroup share the activation operand: what a
//     workgroup reads of the activations does not depend on how many channels it covers, and with
//     32 rows and more these reads, all of them hits in the L2, are most of what the L2 delivers
//     (about 8 TB/s to all CUs together in these kernels, whatever the shape).  The rows come as
//     whole rows (a load instruction brings four rows of 256 contiguous bytes) and reach the
//     operand layout through a region of LDS of the wavefront's own, like the rows of the staged
//     kernel, one row block at a time.
template <int RB, int CB, bool TILED, int TAIL>
__global__ __launch_bounds__(NT, RB * CB <= 2 ? 4 : 2)     // 128 registers do for two row blocks of one channel block
void w4a4_gemm_decode16_kernel(const GemmParams p)
{
    // per wavefront: 16 staged rows of activation codes (one row block at a time), later its partial sums
    constexpr int WREG = CB * RB * 1024 > kStageWave ? CB * RB * 1024 : kStageWave;
    __shared__ __align__(16) unsigned char stage[NW * WREG];

    const int tid  = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int col = lane & 15, kc = lane >> 4;

    const int K4 = p.K - 128, G = p.K >> 7;
    // blockIdx.y: which 16 RB rows of the activations (one block for M <= 64, up to four for 256 rows)
    const int row0 = (int)blockIdx.y * (16 * RB);
    const int M = min((int)p.M - row0, 16 * RB);          // rows of this workgroup
    const int64_t n0 = (int64_t)blockIdx.x * (TN * CB);
    constexpr bool A8 = TAIL == 3;
    const int nblk    = (G + 3) >> 2;
    const int g_begin = 4 * (int)((int64_t)wave * nblk / NW);
    const int g_end   = min(G, 4 * (int)((int64_t)(wave + 1) * nblk / NW));

    constexpr uint32_t GSTEP = TILED ? 1024u : 64u;
    const uint32_t nb16 = (uint32_t)((p.N + TN - 1) / TN);
    uint32_t w4o[CB], w8o[CB], wso[CB];
#pragma unroll
    for (int cb = 0; cb < CB; ++cb) {
        int64_t wr = n0 + TN * cb + col;                  // clamped: columns >= N are computed and never stored
        wr = wr < p.N ? wr : p.N - 1;
        uint32_t b16 = (uint32_t)blockIdx.x * CB + cb;    // block of 16 channels in the tiled arrays, clamped likewise
        b16 = b16 < nb16 ? b16 : nb16 - 1;
        w4o[cb] = TILED ? b16 * (uint32_t)((G - 1) * 1024) + lane * 16 : (uint32_t)(wr * (K4 >> 1)) + kc * 16;
        w8o[cb] = TILED ? b16 * 2048u + lane * 16 : (uint32_t)(wr * 128) + kc * 16;
        wso[cb] = (uint32_t)wr * (uint32_t)G;
    }
    const uint8_t *w8b = reinterpret_cast<const uint8_t *>(p.w_q8), *a8b = reinterpret_cast<const uint8_t *>(p.a_q8);
    // operand row 16 rb + col of this lane (rows >= M read row 0): INT8 codes and scales
    uint32_t a8o[RB], aso[RB];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
        const uint32_t ar = row0 + (16 * rb + col < M ? 16 * rb + col : 0);
        a8o[rb] = ar * 128u + kc * 16;
        aso[rb] = ar * (uint32_t)G;
    }
    // staging of the INT4 activation codes: instruction (rb, i) moves rows 16 rb + 4 i .. + 3, lane -> row
    // 16 rb + 4 i + kc, 16-byte chunk `col` of the row's 256 bytes (four groups); rows >= M repeat row M - 1
    uint32_t srow[RB][4];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int r = 16 * rb + 4 * i + kc;
            srow[rb][i] = (uint32_t)(row0 + (r < M ? r : M - 1)) * (uint32_t)(K4 >> 1) + col * 16;
        }
    unsigned char *mine = stage + wave * WREG;
    unsigned char *st_w = mine + kc * kStageRow + col * 16;                    // + 4 i kStageRow
    const unsigned char *st_r = mine + col * kStageRow + kc * 16;              // + 64 d

    float acc[CB][RB][4];
#pragma unroll
    for (int cb = 0; cb < CB; ++cb)
#pragma unroll
        for (int rb = 0; rb < RB; ++rb)
#pragma unroll
            for (int e = 0; e < 4; ++e) acc[cb][rb][e] = 0.0f;
    const v4i   zi = {0, 0, 0, 0};
    const v4f32 zf = {0.0f, 0.0f, 0.0f, 0.0f};

    auto batch = [&](int gb, auto has8_c) __attribute__((always_inline)) {
        constexpr bool HAS8 = decltype(has8_c)::value;
        // Every load of the batch is issued before the first is used, the activation rows first: they
        // come from the L2, the weights from HBM, and loads return in order.  In the batch with the
        // INT8 group the chunks of a row past the INT4 groups repeat the last one.
        constexpr int NG4 = HAS8 ? TAIL : 4;               // INT4 groups of the batch
        // (named registers, not an array: the array stayed in scratch memory)
        uint4 s00, s01, s02, s03, s10, s11, s12, s13, s20, s21, s22, s23, s30, s31, s32, s33;
        const uint32_t back = HAS8 && col >= 4 * NG4 ? (uint32_t)(col - (4 * NG4 - 1)) * 16u : 0u;
        auto stage_load = [&](int rb, int i) __attribute__((always_inline)) {
            return *reinterpret_cast<const uint4 *>(p.a_q4 + (srow[rb][i] + (uint32_t)gb * 64u - back));
        };
        s00 = stage_load(0, 0); s01 = stage_load(0, 1); s02 = stage_load(0, 2); s03 = stage_load(0, 3);
        s10 = stage_load(1, 0); s11 = stage_load(1, 1); s12 = stage_load(1, 2); s13 = stage_load(1, 3);
        if constexpr (RB > 2) {
            s20 = stage_load(2, 0); s21 = stage_load(2, 1); s22 = stage_load(2, 2); s23 = stage_load(2, 3);
            s30 = stage_load(3, 0); s31 = stage_load(3, 1); s32 = stage_load(3, 2); s33 = stage_load(3, 3);
        }
        uint2 avs[RB];
#pragma unroll
        for (int rb = 0; rb < RB; ++rb) avs[rb] = load_scales<A8>(p.a_scale, aso[rb], gb, G);
        uint4 a8lo[RB], a8hi[RB];
        if constexpr (HAS8) {
#pragma unroll
            for (int rb = 0; rb < RB; ++rb) {
                a8lo[rb] = *reinterpret_cast<const uint4 *>(a8b + a8o[rb]);
                a8hi[rb] = *reinterpret_cast<const uint4 *>(a8b + (a8o[rb] + 64u));
            }
        }
        // (keeps the activation rows ahead of the weights in the order of the requests)
        __builtin_amdgcn_sched_barrier(0);
        uint2 wvs[CB];
        uint4 wq[CB][4], wx[CB];
#pragma unroll
        for (int cb = 0; cb < CB; ++cb) {
            wvs[cb] = load_scales<A8>(p.w_scale, wso[cb], gb, G);
#pragma unroll
            for (int d = 0; d < NG4; ++d) wq[cb][d] = *reinterpret_cast<const uint4 *>(p.w_q4 + (w4o[cb] + (uint32_t)(gb + d) * GSTEP));
            if constexpr (HAS8) {
                wq[cb][TAIL] = *reinterpret_cast<const uint4 *>(w8b + w8o[cb]);
                wx[cb]       = *reinterpret_cast<const uint4 *>(w8b + (w8o[cb] + GSTEP));
            }
        }
        // (the fence keeps the loads here: left alone the compiler spreads them between the MFMAs
        // to save registers, which turns one memory round trip per batch into several)
        __builtin_amdgcn_sched_barrier(0);
        // one row block at a time through the wavefront's region (LDS instructions of a wavefront
        // execute in order: the next block's writes come after this block's reads)
        uint4 aq[RB][4];
        auto through_lds = [&](auto rbc, const uint4 &r0, const uint4 &r1, const uint4 &r2, const uint4 &r3) __attribute__((always_inline)) {
            constexpr int rb = decltype(rbc)::value;
            *reinterpret_cast<uint4 *>(st_w)                  = r0;
            *reinterpret_cast<uint4 *>(st_w + 4 * kStageRow)  = r1;
            *reinterpret_cast<uint4 *>(st_w + 8 * kStageRow)  = r2;
            *reinterpret_cast<uint4 *>(st_w + 12 * kStageRow) = r3;
#pragma unroll
            for (int d = 0; d < NG4; ++d) aq[rb][d] = *reinterpret_cast<const uint4 *>(st_r + 64 * d);
        };
        through_lds(std::integral_constant<int, 0>(), s00, s01, s02, s03);
        through_lds(std::integral_constant<int, 1>(), s10, s11, s12, s13);
        if constexpr (RB > 2) {
            through_lds(std::integral_constant<int, 2>(), s20, s21, s22, s23);
            through_lds(std::integral_constant<int, 3>(), s30, s31, s32, s33);
        }
        if (kc != 0) {                                    // k-slots 4 .. 15 of the scale MFMA stay empty
#pragma unroll
            for (int rb = 0; rb < RB; ++rb) avs[rb] = make_uint2(0, 0);
        }
        // (what needs the weights stays behind what does not)
        __builtin_amdgcn_sched_barrier(0);
        if (kc != 0) {
#pragma unroll
            for (int cb = 0; cb < CB; ++cb) wvs[cb] = make_uint2(0, 0);
        }

        auto int4_group = [&](auto dc) __attribute__((always_inline)) {
            constexpr int D = decltype(dc)::value;
            v4i b0[CB], b1[CB];
#pragma unroll
            for (int cb = 0; cb < CB; ++cb) { b0[cb] = widen_lo(wq[cb][D]); b1[cb] = widen_hi(wq[cb][D]); }
#pragma unroll
            for (int rb = 0; rb < RB; ++rb) {
                const v4i x0 = widen_lo(aq[rb][D]), x1 = widen_hi(aq[rb][D]);
#pragma unroll
                for (int cb = 0; cb < CB; ++cb) {
                    v4i c = __builtin_amdgcn_mfma_i32_16x16x64_i8(x0, b0[cb], zi, 0, 0, 0);
                    c = __builtin_amdgcn_mfma_i32_16x16x64_i8(x1, b1[cb], c, 0, 0, 0);
                    const v4f32 sc = __builtin_amdgcn_mfma_f32_16x16x16f16(scale_operand<D>(avs[rb]), scale_operand<D>(wvs[cb]), zf, 0, 0, 0);
#pragma unroll
                    for (int e = 0; e < 4; ++e) acc[cb][rb][e] = fmaf((float)c[e], sc[e], acc[cb][rb][e]);
                }
            }
        };
        int4_group(std::integral_constant<int, 0>());
        if constexpr (NG4 > 1) int4_group(std::integral_constant<int, 1>());
        if constexpr (NG4 > 2) int4_group(std::integral_constant<int, 2>());
        if constexpr (NG4 > 3) int4_group(std::integral_constant<int, 3>());
        if constexpr (HAS8) {
#pragma unroll
            for (int rb = 0; rb < RB; ++rb)
#pragma unroll
                for (int cb = 0; cb < CB; ++cb) {
                    v4i c = __builtin_amdgcn_mfma_i32_16x16x64_i8(__builtin_bit_cast(v4i, a8lo[rb]), __builtin_bit_cast(v4i, wq[cb][TAIL]), zi, 0, 0, 0);
                    c = __builtin_amdgcn_mfma_i32_16x16x64_i8(__builtin_bit_cast(v4i, a8hi[rb]), __builtin_bit_cast(v4i, wx[cb]), c, 0, 0, 0);
                    const v4f32 sc = __builtin_amdgcn_mfma_f32_16x16x16f16(scale_operand<TAIL>(avs[rb]), scale_operand<TAIL>(wvs[cb]), zf, 0, 0, 0);
#pragma unroll
                    for (int e = 0; e < 4; ++e) acc[cb][rb][e] = fmaf((float)c[e], 256.0f * sc[e], acc[cb][rb][e]);
                }
        }
    };

    const int g_plain = wave == NW - 1 ? g_end - (TAIL + 1) : g_end;
    for (int gb = g_begin; gb < g_plain; gb += 4) batch(gb, std::false_type());
    if (wave == NW - 1) batch(G - (TAIL + 1), std::true_type());

    // the eight K-slices meet in LDS (each wavefront's region, its operand reads are complete) and
    // are added in slice order
    float *red = reinterpret_cast<float *>(mine);        // [channel block][row block][register][lane]
#pragma unroll
    for (int cb = 0; cb < CB; ++cb)
#pragma unroll
        for (int rb = 0; rb < RB; ++rb)
#pragma unroll
            for (int e = 0; e < 4; ++e) red[((cb * RB + rb) * 4 + e) * 64 + lane] = acc[cb][rb][e] * (1.0f / 256.0f);
    __syncthreads();
    for (int idx = tid; idx < CB * RB * 4 * 64; idx += NT) {
        const int l = idx & 63, e = (idx >> 6) & 3, rb = (idx >> 8) % RB, cb = (idx >> 8) / RB;
        float s = 0.0f;
#pragma unroll
        for (int w = 0; w < NW; ++w) s += reinterpret_cast<const float *>(stage + w * WREG)[idx];
        const int m = 16 * rb + 4 * (l >> 4) + e;
        const int64_t n = n0 + TN * cb + (l & 15);
        if (m < M && n < p.N) p.y[(int64_t)(row0 + m) * p.ldy + n] = __half_as_ushort(__float2half_rn(s));
    }
}

// One block of activation rows (M <= 16): decode_staged_body of atom_gemm_decode_staged.h.
template <int SI, bool TILED, int TAIL>
__global__ __launch_bounds__(NT, 6)
void w4a4_gemm_decode_staged_kernel(const GemmParams p)
{
    __shared__ __align__(16) unsigned char stage[kStageBytes];
    decode_staged_body<SI, TILED, TAIL, false>(p, (int)blockIdx.x, stage, NoWait());
}

// The kernels of the common case: M <= 16 staged, else blocks of 16 rows.
template <bool TILED, int TAIL>
void launch_common(const GemmParams &p, unsigned blocks, hipStream_t stream)
{
    if (p.M <= 4)       hipLaunchKernelGGL((w4a4_gemm_decode_staged_kernel<1, TILED, TAIL>), dim3(blocks), dim3(NT), 0, stream, p);
    else if (p.M <= 8)  hipLaunchKernelGGL((w4a4_gemm_decode_staged_kernel<2, TILED, TAIL>), dim3(blocks), dim3(NT), 0, stream, p);
    else if (p.M <= 16) hipLaunchKernelGGL((w4a4_gemm_decode_staged_kernel<4, TILED, TAIL>), dim3(blocks), dim3(NT), 0, stream, p);
    else if (p.M <= 32) hipLaunchKernelGGL((w4a4_gemm_decode16_kernel<2, 1, TILED, TAIL>), dim3(blocks), dim3(NT), 0, stream, p);
    // Four row blocks (and with more than 64 rows further sets of workgroups for rows 64 and up: the
    // weights of a channel block are then read again, out of the caches): two channel
    // blocks per workgroup once there is more than one workgroup per CU otherwise.  M = 64, K = 4096,
    // weights from HBM: N = 4096 6.6 us with one, 8.2 us with two; N = 5120 10.9 / 8.3; N = 8192 11.5 /
    // 9.1; N = 11008 16.2 / 15.3; N = 22016 30.8 / 23.7.
    else {
        const unsigned yb = (unsigned)((p.M + 63) / 64);
        if ((int64_t)blocks * yb <= atom_launch::compute_units())
            hipLaunchKernelGGL((w4a4_gemm_decode16_kernel<4, 1, TILED, TAIL>), dim3(blocks, yb), dim3(NT), 0, stream, p);
        else
            hipLaunchKernelGGL((w4a4_gemm_decode16_kernel<4, 2, TILED, TAIL>), dim3((blocks + 1) / 2, yb), dim3(NT), 0, stream, p);
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

// What the kernels that read tiled weights need: the common case (see common_tail).
bool decode_tiled_supported(const GemmParams &p) { return common_tail(p) != 0; }

int decode_rounds(const GemmParams &p)
{
    const int64_t cus = atom_launch::compute_units();
    const int64_t blocks = (p.N + TN - 1) / TN, yb = (p.M + 63) / 64;
    const int64_t wgs = blocks * yb <= cus ? blocks * yb : (blocks + 1) / 2 * yb;     // as launch_common picks them
    return (int)((wgs + cus - 1) / cus);
}

hipError_t launch_decode_tiled(const GemmParams &p, hipStream_t stream)
{
    const unsigned blocks = (unsigned)((p.N + TN - 1) / TN);
    if (common_tail(p) == 3) launch_common<true, 3>(p, blocks, stream);
    else                     launch_common<true, 1>(p, blocks, stream);
    return hipGetLastError();
}

hipError_t launch_decode(const GemmParams &p, hipStream_t stream)
{
    const unsigned blocks = (unsigned)((p.N + TN - 1) / TN);
    const int tail = common_tail(p);
    if (tail == 3) { launch_common<false, 3>(p, blocks, stream); return hipGetLastError(); }
    if (tail == 1) { launch_common<false, 1>(p, blocks, stream); return hipGetLastError(); }
    // The general kernel.  Vector scale loads: G even (a scale row then starts on a 4-byte boundary),
    // both scale arrays 4-byte aligned
    const int  G  = p.K >> 7;
    const bool vs = G % 2 == 0 && G >= 4 && ((reinterpret_cast<uintptr_t>(p.a_scale) | reinterpret_cast<uintptr_t>(p.w_scale)) & 3) == 0 &&
                    (uint64_t)p.N * (uint64_t)G < (1ull << 31);          // 32-bit scale offsets
    // exactly one INT8 group, and it is the last group of the last wavefront's run (G >= 8)
    const bool one8 = p.O == 128 && G >= NW && (uint64_t)p.N * (uint64_t)(p.K >> 1) < (1ull << 32);   // 32-bit byte offsets
    if (p.M <= 16 && vs && one8) {
        hipLaunchKernelGGL((w4a4_gemm_decode_kernel<1, true, true>), dim3(blocks), dim3(NT), 0, stream, p);
    } else if (p.M <= 32 && vs && one8) {
        hipLaunchKernelGGL((w4a4_gemm_decode_kernel<2, true, true>), dim3(blocks), dim3(NT), 0, stream, p);
    } else if (vs && one8) {
        hipLaunchKernelGGL((w4a4_gemm_decode_kernel<4, true, true>), dim3(blocks), dim3(NT), 0, stream, p);
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
