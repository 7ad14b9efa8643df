// Mixed-precision group-quantised GEMM (Section 4.2 of the paper, steps 1-3)
// for gfx950: nibble-packed INT4 codes stream from HBM with 128-bit loads, are
// widened to INT8 on their way into LDS, are contracted on the INT8 MFMA with
// int32 accumulation one 128-channel group at a time, and every group's
// integer tile is rescaled by a_scale[m,g] * w_scale[n,g] into fp32 VGPR
// accumulators (ascending g, fused multiply-add), stored as fp16.
//
// Widening trick: for a packed dword w (eight codes), (w << 4) & 0xF0F0F0F0
// holds the four even-position codes and w & 0xF0F0F0F0 the four odd-position
// codes, each as the signed byte 16*code.  Both operands are widened the same
// way, so a group's integer sum comes out as 256*P: exact in int32
// (|256 P| <= 2^21) and in fp32, and the factor 2^-8 is folded into the weight
// scale.  The order of the 128 channels inside a group is irrelevant to an
// exact integer sum, so the even/odd split never has to be undone.
//
// MFMA 32x32x32 i8 register layout used here: lane l supplies row (l & 31) of
// its operand and 16 consecutive bytes of the K chunk (l >> 5); the result
// tile has column (l & 31) in lane l and rows 8*(r>>2) + 4*(l>>5) + (r&3) in
// accumulator register r = 0..15.  Activations are the row operand, weights
// the column operand, so a lane owns one output channel n and 16 tokens m.

#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include <stdint.h>

#include "atom_internal.h"

#include "atom_gemm_common.h"

namespace {

using namespace atom_gemm;

template <int BM, int BN, int WM, int WN, bool DBG>
__global__ __launch_bounds__((BM / WM) * (BN / WN) * 64)
void w4a4_gemm_kernel(const GemmParams p)
{
    constexpr int NW = (BM / WM) * (BN / WN);
    constexpr int NT = NW * 64;
    constexpr int TM = WM / 32, TN = WN / 32;
    constexpr int A4 = BM * 4 / NT, B4 = BN * 4 / NT;   // 16-byte chunks per thread, INT4 group
    constexpr int A8 = BM * 8 / NT, B8 = BN * 8 / NT;   // same, INT8 group
    constexpr int SC = (BM + BN + NT - 1) / NT;         // scales per thread
    constexpr int STAGE = (BM + BN) * 128 + (BM + BN) * 4;
    static_assert(BM * 4 % NT == 0 && BN * 4 % NT == 0, "tile/threads mismatch");
    static_assert(A4 >= 1 && B4 >= 1, "tile too small for the thread count");

    extern __shared__ __align__(16) unsigned char smem[];

    const int tid  = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wm   = wave / (BN / WN);
    const int wn   = wave % (BN / WN);

    const int K4 = p.K - p.O, G = p.K >> 7, G4 = K4 >> 7;
    const int64_t a4s = K4 >> 1, o8s = p.O;

    // XCD-aware block order: hardware deals consecutive workgroup ids round-robin
    // to the 8 XCDs; give every XCD a contiguous run of tiles that walk down M
    // inside one band of N, so a weight tile is reused out of that XCD's L2.
    const int MB = (int)((p.M + BM - 1) / BM);
    int logical;
    {
        const int nb = gridDim.x, b = blockIdx.x;
        const int per = nb >> 3, rem = nb & 7, xcd = b & 7;
        logical = xcd * per + (xcd < rem ? xcd : rem) + (b >> 3);
    }
    const int64_t m0 = (int64_t)(logical % MB) * BM;
    const int64_t n0 = (int64_t)(logical / MB) * BN;

    uint4    pre[A8 + B8];
    uint16_t sc[SC];

    auto prefetch = [&](int g) {
        if (g < G4) {
#pragma unroll
            for (int i = 0; i < A4; ++i) {
                int64_t r = m0 + (tid >> 2) + i * (NT / 4);
                r = r < p.M ? r : p.M - 1;
                pre[i] = *reinterpret_cast<const uint4 *>(p.a_q4 + r * a4s + g * 64 + (tid & 3) * 16);
            }
#pragma unroll
            for (int i = 0; i < B4; ++i) {
                int64_t r = n0 + (tid >> 2) + i * (NT / 4);
                r = r < p.N ? r : p.N - 1;
                pre[A8 + i] = *reinterpret_cast<const uint4 *>(p.w_q4 + r * a4s + g * 64 + (tid & 3) * 16);
            }
        } else {
            const int g8 = g - G4;
#pragma unroll
            for (int i = 0; i < A8; ++i) {
                int64_t r = m0 + (tid >> 3) + i * (NT / 8);
                r = r < p.M ? r : p.M - 1;
                pre[i] = *reinterpret_cast<const uint4 *>(p.a_q8 + r * o8s + g8 * 128 + (tid & 7) * 16);
            }
#pragma unroll
            for (int i = 0; i < B8; ++i) {
                int64_t r = n0 + (tid >> 3) + i * (NT / 8);
                r = r < p.N ? r : p.N - 1;
                pre[A8 + i] = *reinterpret_cast<const uint4 *>(p.w_q8 + r * o8s + g8 * 128 + (tid & 7) * 16);
            }
        }
#pragma unroll
        for (int i = 0; i < SC; ++i) {
            const int t = tid + i * NT;
            uint16_t v = 0;
            if (t < BM) {
                if (m0 + t < p.M) v = p.a_scale[(m0 + t) * G + g];
            } else if (t < BM + BN) {
                if (n0 + (t - BM) < p.N) v = p.w_scale[(n0 + (t - BM)) * G + g];
            }
            sc[i] = v;
        }
    };

    auto stage_to_lds = [&](int g, int stage) {
        unsigned char *sA = smem + stage * STAGE;
        unsigned char *sB = sA + BM * 128;
        float *sS = reinterpret_cast<float *>(sB + BN * 128);
        if (g < G4) {
            const int c2 = (tid & 3) * 2;
            auto widen = [&](const uint4 &w, unsigned char *base, int row) {
                uint4 lo, hi;
                lo.x = (w.x << 4) & 0xF0F0F0F0u; hi.x = w.x & 0xF0F0F0F0u;
                lo.y = (w.y << 4) & 0xF0F0F0F0u; hi.y = w.y & 0xF0F0F0F0u;
                lo.z = (w.z << 4) & 0xF0F0F0F0u; hi.z = w.z & 0xF0F0F0F0u;
                lo.w = (w.w << 4) & 0xF0F0F0F0u; hi.w = w.w & 0xF0F0F0F0u;
                *reinterpret_cast<uint4 *>(base + lds_off(row, c2))     = lo;
                *reinterpret_cast<uint4 *>(base + lds_off(row, c2 + 1)) = hi;
            };
#pragma unroll
            for (int i = 0; i < A4; ++i) widen(pre[i], sA, (tid >> 2) + i * (NT / 4));
#pragma unroll
            for (int i = 0; i < B4; ++i) widen(pre[A8 + i], sB, (tid >> 2) + i * (NT / 4));
        } else {
#pragma unroll
            for (int i = 0; i < A8; ++i) {
                const int row = (tid >> 3) + i * (NT / 8);
                *reinterpret_cast<uint4 *>(sA + lds_off(row, tid & 7)) = pre[i];
            }
#pragma unroll
            for (int i = 0; i < B8; ++i) {
                const int row = (tid >> 3) + i * (NT / 8);
                *reinterpret_cast<uint4 *>(sB + lds_off(row, tid & 7)) = pre[A8 + i];
            }
        }
#pragma unroll
        for (int i = 0; i < SC; ++i) {
            const int t = tid + i * NT;
            if (t < BM + BN) sS[t] = half_bits_to_float(sc[i]);
        }
    };

    float acc[TM][TN][16];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

    prefetch(0);
    for (int g = 0; g < G; ++g) {
        const int stage = g & 1;
        stage_to_lds(g, stage);
        __syncthreads();
        if (g + 1 < G) prefetch(g + 1);

        const unsigned char *sA = smem + stage * STAGE;
        const unsigned char *sB = sA + BM * 128;
        const float *sS = reinterpret_cast<const float *>(sB + BN * 128);

        // step 1: integer tile of this group on the matrix cores
        v16i c[TM][TN];
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) c[i][j][r] = 0;
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            v4i a[TM], b[TN];
            const int chunk = 2 * kk + (lane >> 5);
#pragma unroll
            for (int i = 0; i < TM; ++i)
                a[i] = *reinterpret_cast<const v4i *>(sA + lds_off(wm * WM + 32 * i + (lane & 31), chunk));
#pragma unroll
            for (int j = 0; j < TN; ++j)
                b[j] = *reinterpret_cast<const v4i *>(sB + lds_off(wn * WN + 32 * j + (lane & 31), chunk));
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    c[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[i], b[j], c[i][j], 0, 0, 0);
        }

        // steps 2 and 3: dequantise the group's tile and add it in fp32
        const bool  is4  = g < G4;
        const float fold = is4 ? (1.0f / 256.0f) : 1.0f;
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const float wsn = sS[BM + wn * WN + 32 * j + (lane & 31)] * fold;
#pragma unroll
            for (int i = 0; i < TM; ++i) {
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int   ml = wm * WM + 32 * i + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
                    const float ss = sS[ml] * wsn;
                    acc[i][j][r] = fmaf((float)c[i][j][r], ss, acc[i][j][r]);
                    if (DBG) {
                        const int64_t m = m0 + ml, n = n0 + wn * WN + 32 * j + (lane & 31);
                        if (m < p.M && n < p.N)
                            p.partials[(m * p.N + n) * G + g] = is4 ? (c[i][j][r] >> 8) : c[i][j][r];
                    }
                }
            }
        }
    }

#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int64_t m = m0 + wm * WM + 32 * i + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
                const int64_t n = n0 + wn * WN + 32 * j + (lane & 31);
                if (m < p.M && n < p.N)
                    p.y[m * p.ldy + n] = __half_as_ushort(__float2half_rn(acc[i][j][r]));
            }
}

template <int BM, int BN, int WM, int WN, bool DBG>
hipError_t launch_tile(const GemmParams &p, hipStream_t stream)
{
    constexpr int NT = (BM / WM) * (BN / WN) * 64;
    constexpr int LDS = 2 * ((BM + BN) * 128 + (BM + BN) * 4);
    const int64_t MB = (p.M + BM - 1) / BM, NB = (p.N + BN - 1) / BN;
    auto kern = &w4a4_gemm_kernel<BM, BN, WM, WN, DBG>;
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

template <bool DBG>
hipError_t dispatch(const GemmParams &p, hipStream_t stream)
{
    // M <= 64 streams the weights; but from 33 rows on, with many output channels, the big-tile
    // kernel is the faster one (measured at K = 4096: M = 64, N = 11008 42.8 us against 27.1 us,
    // N = 22016 82.6 against 32.5; at N = 4096 the streaming kernel wins, 15.6 against 26.4)
    if (!DBG && p.M <= 64 && !(p.M > 32 && p.N >= 8192)) return launch_decode(p, stream);
    if (!DBG && p.M <= 64) return launch_big(p, stream);
    if (p.M <= 32) return launch_tile<32, 64, 32, 32, DBG>(p, stream);
    if (p.M <= 64) return launch_tile<64, 64, 32, 32, DBG>(p, stream);
    return launch_big(p, stream);
}

}  // namespace

namespace atom_internal {

size_t gemm_workspace_bytes(int64_t, int64_t, int, int) { return 0; }

hipError_t launch_w4a4_gemm(const GemmArgs &a, hipStream_t stream)
{
    GemmParams p;
    p.a_q4 = a.a_q4; p.a_q8 = a.a_q8; p.a_scale = a.a_scale;
    p.w_q4 = a.w_q4; p.w_q8 = a.w_q8; p.w_scale = a.w_scale;
    p.y = a.y; p.partials = a.partials;
    p.M = a.M; p.N = a.N; p.ldy = a.ldy; p.K = a.K; p.O = a.O;
    return a.partials ? dispatch<true>(p, stream) : dispatch<false>(p, stream);
}

}  // namespace atom_internal
