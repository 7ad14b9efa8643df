// Ping-pong variant of the group GEMM for compute-bound sizes (M >= 128).
// Same arithmetic as atom_gemm.hip (Section 4.2 of the paper, steps 1-3); what
// differs is the schedule, built around the fact that on gfx950 the per-group
// dequantise-accumulate (vector ALU) costs about as many cycles as the group's
// integer MFMAs (matrix pipe):
//
//   * Workgroup tile 256 x 128, eight wavefronts of 64 x 64 (four 32x32
//     sub-tiles), two wavefronts per SIMD.  The wavefronts form two sets, one
//     per SIMD each.  Both sets run the same loop (phase M: fragments + MFMAs of
//     K-step u; barrier; phase V: vector work of step u + this thread's loads
//     for a later step; barrier) but set Y runs it one barrier later, so while
//     one set keeps the matrix pipe of a SIMD busy the other keeps its vector
//     ALU busy, instead of both doing the same thing one after the other.
//   * Every K-step moves 64 bytes per operand row HBM -> registers -> LDS: an
//     INT4 group is one step (widened to 128 INT8 bytes on the way), an INT8
//     group two half-steps of 64 channels (the other 64 bytes of the LDS row are
//     zero) whose two integer sums are scaled and added one after the other.
//   * The 32x32 tile of scale products a_scale[m,g] * w_scale[n,g] comes from
//     one fp16 MFMA (a rank-1 product with a single non-zero k; the product of
//     two fp16 values is exact in its fp32 accumulator), so the epilogue is one
//     convert and one fused multiply-add per element.  INT4 steps carry the 2^8
//     of the nibble widening in the accumulators; they are rescaled once, when
//     the first INT8 step arrives.

#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include <stdint.h>

#include <type_traits>

#include "atom_gemm_common.h"

namespace {

using namespace atom_gemm;

typedef float    v16f __attribute__((ext_vector_type(16)));
typedef _Float16 v8h  __attribute__((ext_vector_type(8)));
typedef unsigned v4u  __attribute__((ext_vector_type(4)));

constexpr int BM = 256, BN = 128;          // workgroup tile
constexpr int NT = 512;                    // 8 wavefronts
constexpr int CA = BM * 4 / NT;            // 16-byte chunks per thread per K-step, activations
constexpr int CB = BN * 4 / NT;            // same, weights
constexpr int STAGE = (BM + BN) * 128 + (BM + BN) * 4;
static_assert(CA == 2 && CB == 1, "loader layout");
static_assert(BM + BN <= NT, "one scale per thread");

template <bool DBG>
__global__ __launch_bounds__(NT)
void w4a4_gemm_pp_kernel(const GemmParams p)
{
    extern __shared__ __align__(16) unsigned char smem[];

    const int tid  = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wm   = wave & 3;                                      // 4 wavefronts down M
    const int set  = __builtin_amdgcn_readfirstlane(wave >> 2);     // = position along N
    const int wn   = set;

    const int K4 = p.K - p.O, G = p.K >> 7, G4 = K4 >> 7, G8 = p.O >> 7;
    const int U  = G4 + 2 * G8;                         // K-steps of 64 bytes per row

    const int MB      = (int)((p.M + BM - 1) / BM);
    const int logical = xcd_contiguous_block_id();
    const int64_t m0  = (int64_t)(logical % MB) * BM;
    const int64_t n0  = (int64_t)(logical / MB) * BN;

    // ---- loader set-up: thread -> (tile row, 16-byte chunk) ----------------------
    // rows clamp to the last valid row: out-of-range tile rows are computed and discarded
    uint32_t oa4[CA], oa8[CA], ob4, ob8;
#pragma unroll
    for (int i = 0; i < CA; ++i) {
        int64_t r = m0 + (tid >> 2) + i * (NT / 4);
        r = r < p.M ? r : p.M - 1;
        oa4[i] = (uint32_t)(r * (K4 >> 1)) + (tid & 3) * 16;
        oa8[i] = (uint32_t)(r * p.O) + (tid & 3) * 16;
    }
    {
        int64_t r = n0 + (tid >> 2);
        r = r < p.N ? r : p.N - 1;
        ob4 = (uint32_t)(r * (K4 >> 1)) + (tid & 3) * 16;
        ob8 = (uint32_t)(r * p.O) + (tid & 3) * 16;
    }
    const uint16_t *sptr = nullptr;                     // the one scale this thread stages
    if (tid < BM) {
        if (m0 + tid < p.M) sptr = p.a_scale + (m0 + tid) * G;
    } else if (tid < BM + BN) {
        if (n0 + (tid - BM) < p.N) sptr = p.w_scale + (n0 + (tid - BM)) * G;
    }
    const int wrow   = tid >> 2;                        // tile row of chunk 0 (chunk i: + i*128)
    const int w4lo   = lds_off(wrow, (tid & 3) * 2);    // widened INT4: even-position codes
    const int w4hi   = lds_off(wrow, (tid & 3) * 2 + 1);
    const int w8     = lds_off(wrow, tid & 3);          // INT8 half-step: straight copy
    const int w8z    = lds_off(wrow, 4 + (tid & 3));    // ... and its zero padding

    uint4    pre[CA + CB];
    uint16_t sc = 0;

    auto prefetch = [&](int u) {
        if (u < G4) {
            const uint32_t col = (uint32_t)u * 64;
#pragma unroll
            for (int i = 0; i < CA; ++i)
                pre[i] = *reinterpret_cast<const uint4 *>(p.a_q4 + oa4[i] + col);
            pre[CA] = *reinterpret_cast<const uint4 *>(p.w_q4 + ob4 + col);
            sc = sptr ? sptr[u] : (uint16_t)0;
        } else {
            const uint32_t col = (uint32_t)(u - G4) * 64;           // g8*128 + half*64
#pragma unroll
            for (int i = 0; i < CA; ++i)
                pre[i] = *reinterpret_cast<const uint4 *>(p.a_q8 + oa8[i] + col);
            pre[CA] = *reinterpret_cast<const uint4 *>(p.w_q8 + ob8 + col);
            sc = sptr ? sptr[G4 + ((u - G4) >> 1)] : (uint16_t)0;
        }
    };

    auto stage_to_lds = [&](int u) {
        unsigned char *base = smem + (u & 1) * STAGE;
        if (u < G4) {
#pragma unroll
            for (int i = 0; i < CA + CB; ++i) {
                const uint4 w = pre[i];
                uint4 lo, hi;
                lo.x = (w.x << 4) & 0xF0F0F0F0u; hi.x = w.x & 0xF0F0F0F0u;
                lo.y = (w.y << 4) & 0xF0F0F0F0u; hi.y = w.y & 0xF0F0F0F0u;
                lo.z = (w.z << 4) & 0xF0F0F0F0u; hi.z = w.z & 0xF0F0F0F0u;
                lo.w = (w.w << 4) & 0xF0F0F0F0u; hi.w = w.w & 0xF0F0F0F0u;
                *reinterpret_cast<uint4 *>(base + w4lo + i * (NT / 4) * 128) = lo;
                *reinterpret_cast<uint4 *>(base + w4hi + i * (NT / 4) * 128) = hi;
            }
        } else {
            // 64 INT8 channels in chunks 0..3, zeros in chunks 4..7
#pragma unroll
            for (int i = 0; i < CA + CB; ++i) {
                *reinterpret_cast<uint4 *>(base + w8 + i * (NT / 4) * 128) = pre[i];
                *reinterpret_cast<uint4 *>(base + w8z + i * (NT / 4) * 128) = make_uint4(0, 0, 0, 0);
            }
        }
        if (tid < BM + BN)
            reinterpret_cast<uint32_t *>(base + (BM + BN) * 128)[tid] = (uint32_t)sc;
    };

    // ---- fragment addresses (loop invariant; stage and sub-tile offsets are immediates) ---
    const int ra = wm * 64 + (lane & 31);               // activation tile row of sub-tile i=0
    const int rb = BM + wn * 64 + (lane & 31);          // weight tile row of sub-tile j=0
    int a_addr[4], b_addr[4];
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
        a_addr[kk] = lds_off(ra, 2 * kk + (lane >> 5));
        b_addr[kk] = lds_off(rb, 2 * kk + (lane >> 5));
    }

    float acc[4][16];
#pragma unroll
    for (int t = 0; t < 4; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[t][r] = 0.0f;
    v16i c[4];                                          // integer tiles, phase M -> phase V
    v16f ss[4];                                         // scale-product tiles, phase M -> phase V

    // phase M: fragments from LDS, integer MFMAs, then the scale-product MFMAs
    auto phase_m = [&](auto stage_c) {
        constexpr int S = decltype(stage_c)::value;
        const unsigned char *base = smem + S * STAGE;
        const uint32_t *sS = reinterpret_cast<const uint32_t *>(base + (BM + BN) * 128);
        const v16i zi = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
        for (int t = 0; t < 4; ++t) c[t] = zi;
        v4i a[2][4], b[2][4];
#pragma unroll
        for (int kk = 0; kk < 4; ++kk)
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                a[i][kk] = *reinterpret_cast<const v4i *>(base + a_addr[kk] + i * 32 * 128);
                b[i][kk] = *reinterpret_cast<const v4i *>(base + b_addr[kk] + i * 32 * 128);
            }
#pragma unroll
        for (int kk = 0; kk < 4; ++kk)
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j)
                    c[i * 2 + j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[i][kk], b[j][kk],
                                                                          c[i * 2 + j], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
        v8h sa[2], sb[2];
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const uint32_t abits = sS[wm * 64 + 32 * i + (lane & 31)];
            const uint32_t bbits = sS[BM + wn * 64 + 32 * i + (lane & 31)];
            const v4u ta = {lane < 32 ? abits : 0u, 0u, 0u, 0u};
            const v4u tb = {lane < 32 ? bbits : 0u, 0u, 0u, 0u};
            sa[i] = __builtin_bit_cast(v8h, ta);
            sb[i] = __builtin_bit_cast(v8h, tb);
        }
        const v16f zf = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j)
                ss[i * 2 + j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(sa[i], sb[j], zf, 0, 0, 0);
    };

    // phase V: dequantise the integer tiles of step u and add them (steps 2 and 3)
    auto phase_v = [&](int u) {
        if (u == G4) {
            // first INT8 step: leave the 2^8 of the nibble widening behind
#pragma unroll
            for (int t = 0; t < 4; ++t)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[t][r] *= (1.0f / 256.0f);
        }
#pragma unroll
        for (int t = 0; t < 4; ++t)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[t][r] = fmaf((float)c[t][r], ss[t][r], acc[t][r]);
        if (DBG) {
            const int g = u < G4 ? u : G4 + ((u - G4) >> 1);
#pragma unroll
            for (int t = 0; t < 4; ++t)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int64_t m = m0 + wm * 64 + 32 * (t >> 1) + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
                    const int64_t n = n0 + wn * 64 + 32 * (t & 1) + (lane & 31);
                    if (m < p.M && n < p.N) {
                        int32_t *dst = p.partials + (m * p.N + n) * G + g;
                        if (u < G4)                   *dst = c[t][r] >> 8;
                        else if (((u - G4) & 1) == 0) *dst = c[t][r];
                        else                          *dst += c[t][r];   // second half of an INT8 group
                    }
                }
        }
    };

    // phase L: this thread's share of the next tile it owes goes to LDS, and the global
    // loads of the tile after that are issued.  Set X runs one tile ahead of its own
    // phase M, set Y two tiles ahead (it runs one barrier later and both sets' shares of
    // a tile must be in LDS before set X reads it).
    int t_next = 1;
    auto phase_l = [&]() {
        if (t_next < U) {
            stage_to_lds(t_next);
            if (t_next + 1 < U) prefetch(t_next + 1);
        }
        ++t_next;
    };

    auto step = [&](int u, auto stage_c) {
        phase_m(stage_c);
        __syncthreads();
        phase_v(u);
        phase_l();
        __syncthreads();
    };

    prefetch(0);
    stage_to_lds(0);
    if (U > 1) prefetch(1);
    if (set != 0) phase_l();
    __syncthreads();
    if (set != 0) __syncthreads();                      // set Y starts one barrier later
    for (int u = 0; u < U; u += 2) {
        step(u, std::integral_constant<int, 0>{});
        if (u + 1 < U) step(u + 1, std::integral_constant<int, 1>{});
    }
    if (set == 0) __syncthreads();                      // ... and set X waits for it at the end

#pragma unroll
    for (int t = 0; t < 4; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int64_t m = m0 + wm * 64 + 32 * (t >> 1) + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
            const int64_t n = n0 + wn * 64 + 32 * (t & 1) + (lane & 31);
            if (m < p.M && n < p.N)
                p.y[m * p.ldy + n] = __half_as_ushort(__float2half_rn(acc[t][r]));
        }
}

template <bool DBG>
hipError_t launch_pp(const GemmParams &p, hipStream_t stream)
{
    constexpr int LDS = 2 * STAGE;
    const int64_t MB = (p.M + BM - 1) / BM, NB = (p.N + BN - 1) / BN;
    auto kern = &w4a4_gemm_pp_kernel<DBG>;
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
    return p.partials ? launch_pp<true>(p, stream) : launch_pp<false>(p, stream);
}

}  // namespace atom_gemm
