// Big-tile variant of the group GEMM for compute-bound sizes (M > 64).
// Same arithmetic as atom_gemm.hip (Section 4.2 of the paper, steps 1-3); what
// differs is the schedule, built on three measurements on gfx950:
//   (1) vector instructions placed between the MFMAs of ONE wavefront are almost
//       free (the matrix pipe runs 32 cycles per 32x32x32 MFMA), whereas a
//       wavefront that issues MFMAs back to back starves the other wavefront of
//       its SIMD of vector issue slots, so overlap has to be built inside each
//       wavefront's own instruction stream;
//   (2) the per-group dequantise-accumulate costs about as many vector cycles as
//       the group's integer MFMAs cost matrix cycles;
//   (3) pulling operand fragments per wavefront straight from L1 saturates the
//       texture path, so operands are shared through LDS.
//
// Workgroup tile 256 x 128 (eight wavefronts) or 128 x 128 (four), wavefront tile
// 64 x 64 (four 32x32 sub-tiles), two LDS stages, one barrier per K-step.  A K-step moves 64 bytes per operand
// row HBM -> registers -> LDS (an INT4 group, widened to 128 INT8 bytes on the
// way; an INT8 group is two half-steps).  Inside a step the hot loop is one
// branch-free basic block in which the four MFMAs of sub-tile t+1 and the fp16
// MFMA that produces the tile of scale products are interleaved with the
// convert + fused-multiply-add of sub-tile t and with the widening and LDS
// writes of the NEXT step's operands.
//
// The 32x32 tile of scale products a_scale[m,g] * w_scale[n,g] is one fp16 MFMA
// (rank-1, single non-zero k; the product of two fp16 values is exact in its
// fp32 accumulator), so the epilogue is one convert and one fused multiply-add
// per element.  INT4 steps carry the 2^8 of the nibble widening in the
// accumulators; they are rescaled once, before the first INT8 step.

#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include <stdint.h>

#include <type_traits>

#include "atom_gemm_common.h"

namespace {

using namespace atom_gemm;

typedef float    v16f __attribute__((ext_vector_type(16)));
typedef _Float16 v4h  __attribute__((ext_vector_type(4)));
typedef unsigned v2u  __attribute__((ext_vector_type(2)));

// BM x BN: workgroup tile; (BM/64) x (BN/64) wavefronts, at least two per SIMD resident
template <int BM, int BN, bool DBG>
__global__ __launch_bounds__((BM / 64) * (BN / 64) * 64, 2)
void w4a4_gemm_big_kernel(const GemmParams p)
{
    constexpr int WM = BM / 64;                         // wavefronts down M
    constexpr int NT = WM * (BN / 64) * 64;
    constexpr int RPT = NT / 4;                         // tile rows covered by one loader pass
    constexpr int CH = (BM + BN) / RPT;                 // 16-byte chunks per thread per K-step
    constexpr int CHA = BM / RPT;                       // of which activation rows
    constexpr int STAGE = (BM + BN) * 128 + NT * 4;     // codes + one scale slot per thread
    static_assert(BM % RPT == 0 && BN % RPT == 0 && RPT % 8 == 0, "loader layout");
    static_assert(BM + BN <= NT, "one scale per thread");

    extern __shared__ __align__(16) unsigned char smem[];

    const int tid  = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wm = wave % WM, wn = wave / WM;
    const int r = lane & 31, h = lane >> 5;

    const int K4 = p.K - p.O, G = p.K >> 7, G4 = K4 >> 7, G8 = p.O >> 7;
    const int U  = G4 + 2 * G8;                         // K-steps of 64 bytes per row

    const int MB      = (int)((p.M + BM - 1) / BM);
    const int logical = xcd_contiguous_block_id();
    const int64_t m0  = (int64_t)(logical % MB) * BM;
    const int64_t n0  = (int64_t)(logical / MB) * BN;

    // ---- loader: thread -> (tile row, 16-byte chunk).  Pass i covers rows wrow + i*RPT of
    // the stacked tile (BM activation rows, then BN weight rows).  Rows clamp to the last
    // valid row (such tile rows are computed and never stored).  32-bit offsets: arrays
    // < 4 GiB.
    const int wrow = tid >> 2, wc = tid & 3;
    uint32_t o4[CH];
#pragma unroll
    for (int i = 0; i < CH; ++i) {
        int64_t row = i < CHA ? m0 + wrow + i * RPT : n0 + wrow + (i - CHA) * RPT;
        const int64_t last = i < CHA ? p.M - 1 : p.N - 1;
        row = row < last ? row : last;
        o4[i] = (uint32_t)(row * (K4 >> 1)) + wc * 16;
    }
    // the one scale this thread stages per group: element offset, or none
    const uint16_t *sbase = tid < BM ? p.a_scale : p.w_scale;
    uint32_t soff = 0;
    bool has_scale = false;
    if (tid < BM) {
        has_scale = m0 + tid < p.M;
        soff = (uint32_t)((has_scale ? m0 + tid : 0) * G);
    } else if (tid < BM + BN) {
        has_scale = n0 + (tid - BM) < p.N;
        soff = (uint32_t)((has_scale ? n0 + (tid - BM) : 0) * G);
    }
    const int w4lo = lds_off(wrow, wc * 2);             // widened INT4: even-position codes
    const int w4hi = lds_off(wrow, wc * 2 + 1);         //               odd-position codes
    const int w8   = lds_off(wrow, wc);                 // INT8 half-step: straight copy, chunks 0..3

    uint4    pre[CH];
    uint32_t sc = 0;

    auto prefetch = [&](int u, auto is8) {
        if (decltype(is8)::value) {
            // INT8 steps are few: their row offsets are recomputed instead of kept in VGPRs
            const uint32_t col = (uint32_t)(u - G4) * 64 + wc * 16;   // g8*128 + half*64 + chunk
            const uint32_t h4 = (uint32_t)(K4 >> 1), o = (uint32_t)p.O;
#pragma unroll
            for (int i = 0; i < CH; ++i) {
                const uint32_t row = (o4[i] - wc * 16) / h4;
                const uint8_t *src = reinterpret_cast<const uint8_t *>(i < CHA ? p.a_q8 : p.w_q8);
                pre[i] = *reinterpret_cast<const uint4 *>(src + (size_t)(row * o + col));
            }
            sc = sbase[(size_t)(soff + (uint32_t)(G4 + ((u - G4) >> 1)))];
        } else {
            const uint32_t col = (uint32_t)u * 64;
#pragma unroll
            for (int i = 0; i < CH; ++i)
                pre[i] = *reinterpret_cast<const uint4 *>((i < CHA ? p.a_q4 : p.w_q4) + (size_t)(o4[i] + col));
            sc = sbase[(size_t)(soff + (uint32_t)u)];
        }
    };
    // registers -> LDS stage S; the scale goes in as raw fp16 bits (an MFMA operand)
    auto stage_to_lds = [&](auto is8, auto stage_c) {
        unsigned char *base = smem + decltype(stage_c)::value * STAGE;
        if (decltype(is8)::value) {
#pragma unroll
            for (int i = 0; i < CH; ++i)
                *reinterpret_cast<uint4 *>(base + w8 + i * RPT * 128) = pre[i];
        } else {
#pragma unroll
            for (int i = 0; i < CH; ++i) {
                const uint4 w = pre[i];
                uint4 lo, hi;
                lo.x = (w.x << 4) & 0xF0F0F0F0u; hi.x = w.x & 0xF0F0F0F0u;
                lo.y = (w.y << 4) & 0xF0F0F0F0u; hi.y = w.y & 0xF0F0F0F0u;
                lo.z = (w.z << 4) & 0xF0F0F0F0u; hi.z = w.z & 0xF0F0F0F0u;
                lo.w = (w.w << 4) & 0xF0F0F0F0u; hi.w = w.w & 0xF0F0F0F0u;
                *reinterpret_cast<uint4 *>(base + w4lo + i * RPT * 128) = lo;
                *reinterpret_cast<uint4 *>(base + w4hi + i * RPT * 128) = hi;
            }
        }
        // threads beyond the tile rows write a slot nobody reads: no branch in the hot loop
        reinterpret_cast<uint32_t *>(base + (BM + BN) * 128)[tid] = has_scale ? sc : 0u;
    };

    // ---- fragment addresses: loop invariant; stage and sub-tile offsets are immediates ---
    int a_addr[4], b_addr[4];
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
        a_addr[kk] = lds_off(wm * 64 + r, 2 * kk + h);
        b_addr[kk] = lds_off(BM + wn * 64 + r, 2 * kk + h);
    }
    const int sa_addr = (BM + BN) * 128 + (wm * 64 + r) * 4;
    const int sb_addr = (BM + BN) * 128 + (BM + wn * 64 + r) * 4;

    float acc[4][16];
#pragma unroll
    for (int t = 0; t < 4; ++t)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[t][e] = 0.0f;

    const v16i zi = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
    const v16f zf = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};

    auto scale_tile = [&](uint32_t abits, uint32_t bbits) {
        const v2u ta = {abits, 0u}, tb = {bbits, 0u};
        return __builtin_amdgcn_mfma_f32_32x32x8f16(__builtin_bit_cast(v4h, ta),
                                                    __builtin_bit_cast(v4h, tb), zf, 0, 0, 0);
    };
    // steps 2 and 3 for one 32x32 sub-tile (i, j) of K-step u
    auto epilogue = [&](int u, int i, int j, const v16i &c, const v16f &ss) {
        float *a_ = acc[i * 2 + j];
#pragma unroll
        for (int e = 0; e < 16; ++e) a_[e] = fmaf((float)c[e], ss[e], a_[e]);
        if (DBG) {
            const int g = u < G4 ? u : G4 + ((u - G4) >> 1);
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int64_t m = m0 + wm * 64 + 32 * i + 8 * (e >> 2) + 4 * h + (e & 3);
                const int64_t n = n0 + wn * 64 + 32 * j + r;
                if (m < p.M && n < p.N) {
                    int32_t *dst = p.partials + (m * p.N + n) * G + g;
                    if (u < G4)                   *dst = c[e] >> 8;
                    else if (((u - G4) & 1) == 0) *dst = c[e];
                    else                          *dst += c[e];     // second half of an INT8 group
                }
            }
        }
    };

    // One K-step.  NKK: MFMAs per sub-tile (4 for a widened INT4 group, 2 for an INT8
    // half-step).  NEXT: kind of step u+1, whose operands go registers -> LDS here
    // (0 = none, 1 = INT4, 2 = INT8).  PF: kind of step u+2, whose global loads are
    // issued here.  S: LDS stage of this step.  Everything is a compile-time choice so
    // the step is ONE basic block: branches would let the compiler sink the dequantise
    // work below them, away from the MFMAs it is meant to overlap with.
    auto step = [&](int u, auto nkk_c, auto next_c, auto pf_c, auto stage_c) {
        constexpr int NKK = decltype(nkk_c)::value, NEXT = decltype(next_c)::value;
        constexpr int PF = decltype(pf_c)::value;
        constexpr int S = decltype(stage_c)::value;
        const unsigned char *base = smem + S * STAGE;
        v4i a[2][NKK], b[2][NKK];
        auto load_frag = [&](v4i (&f)[NKK], const int (&addr)[4], int blk) {
#pragma unroll
            for (int kk = 0; kk < NKK; ++kk)
                f[kk] = *reinterpret_cast<const v4i *>(base + addr[kk] + blk * 32 * 128);
        };
        load_frag(a[0], a_addr, 0);
        load_frag(b[0], b_addr, 0);
        uint32_t sa[2], sb[2];
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            sa[i] = *reinterpret_cast<const uint32_t *>(base + sa_addr + i * 32 * 4);
            const uint32_t wb = *reinterpret_cast<const uint32_t *>(base + sb_addr + i * 32 * 4);
            sb[i] = h == 0 ? wb : 0u;      // zero on one side keeps k-slots 4..7 empty
        }
        auto mma = [&](int i, int j) {
            v16i c = zi;
#pragma unroll
            for (int kk = 0; kk < NKK; ++kk)
                c = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[i][kk], b[j][kk], c, 0, 0, 0);
            return c;
        };

        // block 1: MFMAs of sub-tile (0,0); vector side: the next step's operands go
        // registers -> LDS.  b[1] is fetched at the end.
        v16i c00 = mma(0, 0);
        if (NEXT) {
            stage_to_lds(std::integral_constant<bool, NEXT == 2>{}, std::integral_constant<int, 1 - S>{});
        }
        load_frag(b[1], b_addr, 1);
#pragma unroll
        for (int k = 0; k < NKK; ++k) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x002, 10, 0);
            __builtin_amdgcn_sched_group_barrier(0x200, 2, 0);
        }
        __builtin_amdgcn_sched_barrier(0);
        // block 2: scale tile of (0,0) and MFMAs of (0,1); vector side: dequantise (0,0):
        // the converts come first, so the scale tile is ready when the multiply-adds start.
        v16f s00 = scale_tile(sa[0], sb[0]);
        v16i c01 = mma(0, 1);
        epilogue(u, 0, 0, c00, s00);
        load_frag(a[1], a_addr, 1);            // a[0] is dead after the MFMAs above
#pragma unroll
        for (int k = 0; k < NKK + 1; ++k) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x002, 7, 0);
        }
        __builtin_amdgcn_sched_barrier(0);
        v16f s01 = scale_tile(sa[0], sb[1]);
        v16i c11 = mma(1, 1);
        epilogue(u, 0, 1, c01, s01);
#pragma unroll
        for (int k = 0; k < NKK + 1; ++k) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x002, 7, 0);
        }
        __builtin_amdgcn_sched_barrier(0);
        v16f s11 = scale_tile(sa[1], sb[1]);
        v16i c10 = mma(1, 0);
        epilogue(u, 1, 1, c11, s11);
#pragma unroll
        for (int k = 0; k < NKK + 1; ++k) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x002, 7, 0);
        }
        __builtin_amdgcn_sched_barrier(0);
        // tail: global loads for step u+2 go out while the last sub-tile is dequantised
        v16f s10 = scale_tile(sa[1], sb[0]);
        if (PF == 1) prefetch(u + 2, std::false_type{});
        if (PF == 2) prefetch(u + 2, std::true_type{});
        epilogue(u, 1, 0, c10, s10);
        __syncthreads();
    };

    // prologue: step 0 into stage 0, step 1 into registers (there is always an INT4
    // group and an INT8 group: G4 >= 1, G8 >= 1, so U >= 3)
    prefetch(0, std::false_type{});
    stage_to_lds(std::false_type{}, std::integral_constant<int, 0>{});
    if (G4 > 1) prefetch(1, std::false_type{});
    else        prefetch(1, std::true_type{});
    __syncthreads();

    using C0 = std::integral_constant<int, 0>;
    using C1 = std::integral_constant<int, 1>;
    using C2 = std::integral_constant<int, 2>;
    using C4 = std::integral_constant<int, 4>;

    // any step, by run-time dispatch to its compile-time variant (used off the hot loop)
    auto any_step = [&](int u) {
        const int next = u + 1 >= U ? 0 : (u + 1 < G4 ? 1 : 2);
        const int pf   = u + 2 >= U ? 0 : (u + 2 < G4 ? 1 : 2);
        const int s1   = u & 1;
        if (u < G4) {
            // next is 1 or 2 and pf is 1 or 2 here (G8 >= 1 gives at least two INT8 half-steps)
            if (next == 1) {
                if (pf == 1) { if (s1) step(u, C4{}, C1{}, C1{}, C1{}); else step(u, C4{}, C1{}, C1{}, C0{}); }
                else         { if (s1) step(u, C4{}, C1{}, C2{}, C1{}); else step(u, C4{}, C1{}, C2{}, C0{}); }
            } else {
                if (s1) step(u, C4{}, C2{}, C2{}, C1{}); else step(u, C4{}, C2{}, C2{}, C0{});
            }
        } else {
            if (next == 0)    { if (s1) step(u, C2{}, C0{}, C0{}, C1{}); else step(u, C2{}, C0{}, C0{}, C0{}); }
            else if (pf == 0) { if (s1) step(u, C2{}, C2{}, C0{}, C1{}); else step(u, C2{}, C2{}, C0{}, C0{}); }
            else              { if (s1) step(u, C2{}, C2{}, C2{}, C1{}); else step(u, C2{}, C2{}, C2{}, C0{}); }
        }
    };

    int u = 0;
    for (; u + 3 < G4; u += 2) {                        // hot loop: steps u+1, u+2, u+3 are INT4
        step(u, C4{}, C1{}, C1{}, C0{});
        step(u + 1, C4{}, C1{}, C1{}, C1{});
    }
    for (; u < G4; ++u) any_step(u);                    // the last one to three INT4 steps
    // leave the 2^8 of the nibble widening behind before the INT8 steps
#pragma unroll
    for (int t = 0; t < 4; ++t)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[t][e] *= (1.0f / 256.0f);
    for (; u < U; ++u) any_step(u);

    // ---- store: the 64x64 fp16 tile of a wavefront goes through LDS so that global
    // memory sees whole 128-byte rows (a lane holds one column: storing from the MFMA
    // layout directly would write 2 bytes per lane).  The last step ended with a barrier,
    // so the stages are free; each wavefront uses a private region, row stride 144 bytes.
    constexpr int OSTRIDE = 144;
    static_assert((NT / 64) * 64 * OSTRIDE <= 2 * STAGE, "output staging fits the operand stages");
    unsigned char *ot = smem + wave * (64 * OSTRIDE);
#pragma unroll
    for (int t = 0; t < 4; ++t)
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            const int row = 32 * (t >> 1) + 8 * (e >> 2) + 4 * h + (e & 3);
            const int col = 32 * (t & 1) + r;
            *reinterpret_cast<uint16_t *>(ot + row * OSTRIDE + col * 2) =
                __half_as_ushort(__float2half_rn(acc[t][e]));
        }
    __syncthreads();
    const int64_t mw = m0 + wm * 64, nw = n0 + wn * 64;
    const bool vec_ok = ((reinterpret_cast<uintptr_t>(p.y) | (uintptr_t)(p.ldy * 2)) & 15) == 0;
#pragma unroll
    for (int it = 0; it < 8; ++it) {
        const int row = it * 8 + (lane >> 3), ch = lane & 7;
        const int64_t m = mw + row, n = nw + ch * 8;
        if (m >= p.M || n >= p.N) continue;
        const uint4 v = *reinterpret_cast<const uint4 *>(ot + row * OSTRIDE + ch * 16);
        uint16_t *dst = p.y + m * p.ldy + n;
        if (vec_ok && n + 8 <= p.N) {
            *reinterpret_cast<uint4 *>(dst) = v;
        } else {
            const uint16_t *hv = reinterpret_cast<const uint16_t *>(&v);
#pragma unroll
            for (int k = 0; k < 8; ++k)
                if (n + k < p.N) dst[k] = hv[k];
        }
    }
}

template <int BM, int BN, bool DBG>
hipError_t launch_cfg(const GemmParams &p, hipStream_t stream)
{
    constexpr int NT = (BM / 64) * (BN / 64) * 64;
    constexpr int LDS = 2 * ((BM + BN) * 128 + NT * 4);
    const int64_t MB = (p.M + BM - 1) / BM, NB = (p.N + BN - 1) / BN;
    auto kern = &w4a4_gemm_big_kernel<BM, BN, DBG>;
    static bool configured = false;   // one attribute call per kernel variant and process
    if (!configured) {
        hipError_t err = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                             hipFuncAttributeMaxDynamicSharedMemorySize, LDS);
        if (err != hipSuccess) return err;
        configured = true;
    }
    hipLaunchKernelGGL(kern, dim3((unsigned)(MB * NB)), dim3(NT), LDS, stream, p);
    return hipGetLastError();
}

}  // namespace

namespace atom_gemm {

hipError_t launch_big(const GemmParams &p, hipStream_t stream)
{
    if (p.partials) return launch_cfg<128, 128, true>(p, stream);
    // The 256 x 128 tile does a third less loader work per MFMA; the 128 x 128 tile is
    // for shapes whose 256 x 128 tiles would leave compute units idle (one 512-thread
    // workgroup per CU; two of the 256-thread ones).
    const int64_t big_tiles = ((p.M + 255) / 256) * ((p.N + 127) / 128);
    if (big_tiles < 512) return launch_cfg<128, 128, false>(p, stream);
    return launch_cfg<256, 128, false>(p, stream);
}

}  // namespace atom_gemm
