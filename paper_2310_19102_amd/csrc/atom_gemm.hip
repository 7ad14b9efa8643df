// Mixed-precision group-quantised GEMM (Section 4.2 of the paper, steps 1-3)
// for gfx950: nibble-packed INT4 codes stream from HBM with 128-bit loads, are
// widened to INT8 (this file: after the LDS fragment read; the big-tile kernel: on
// their way into LDS), are contracted on the INT8 MFMA with
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
#include "atom_launch.h"

namespace {

using namespace atom_gemm;

// KS wavefront sets per workgroup: set s runs the whole pipeline on its own pair of LDS stages
// over its own contiguous share of the groups; the sets' fp32 tiles meet in LDS at the end and
// set 0 adds them in set order (a fixed tree).  For launches of few tiles, where the time is the
// latency of one set's chain of K-steps and most of the chip would otherwise idle.
// 16 packed bytes -> 16 int8 values 16 * code: the low nibbles, the high nibbles
typedef unsigned v4u __attribute__((ext_vector_type(4)));
__device__ __forceinline__ v4i nibbles_lo(v4u w) { return __builtin_bit_cast(v4i, (w << 4) & 0xF0F0F0F0u); }
__device__ __forceinline__ v4i nibbles_hi(v4u w) { return __builtin_bit_cast(v4i, w & 0xF0F0F0F0u); }

template <int BM, int BN, int WM, int WN, bool DBG, int KS = 1>
__global__ __launch_bounds__((BM / WM) * (BN / WN) * 64 * KS)
void w4a4_gemm_kernel(const GemmParams p)
{
    constexpr int NW = (BM / WM) * (BN / WN);
    constexpr int NT = NW * 64;                          // threads of one set
    static_assert(!DBG || KS == 1, "the partial-sum dump runs one set");
    constexpr int TM = WM / 32, TN = WN / 32;
    constexpr int A4 = BM * 4 / NT, B4 = BN * 4 / NT;   // 16-byte chunks per thread, INT4 group
    constexpr int A8 = BM * 8 / NT, B8 = BN * 8 / NT;   // same, INT8 group
    constexpr int SC = (BM + BN + NT - 1) / NT;         // scales per thread
    constexpr int STAGE = (BM + BN) * 128 + (BM + BN) * 4;
    static_assert(BM * 4 % NT == 0 && BN * 4 % NT == 0, "tile/threads mismatch");
    static_assert(A4 >= 1 && B4 >= 1, "tile too small for the thread count");

    extern __shared__ __align__(16) unsigned char smem_all[];

    const int set  = KS == 1 ? 0 : __builtin_amdgcn_readfirstlane((int)threadIdx.x / NT);
    const int tid  = KS == 1 ? (int)threadIdx.x : (int)threadIdx.x - set * NT;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    unsigned char *smem = smem_all + set * (2 * STAGE);
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

    // the operands of one group on their way from global memory to LDS
    // (first-class vector values: nothing here may end up in scratch)
    struct Pre { v4u a[A8], b[B8]; uint16_t sc[SC]; };

    // Row pointers of the INT4 loads and of the scale loads, computed once: left inside the
    // loop, their 64-bit multiplies were most of a trip's vector instructions.  (The INT8
    // groups are the last trip or two of the last set: their addresses are made on the spot.)
    const uint8_t *a4p[A4], *w4p[B4];
#pragma unroll
    for (int i = 0; i < A4; ++i) {
        int64_t r = m0 + (tid >> 2) + i * (NT / 4);
        r = r < p.M ? r : p.M - 1;
        a4p[i] = p.a_q4 + r * a4s + (tid & 3) * 16;
    }
#pragma unroll
    for (int i = 0; i < B4; ++i) {
        int64_t r = n0 + (tid >> 2) + i * (NT / 4);
        r = r < p.N ? r : p.N - 1;
        w4p[i] = p.w_q4 + r * a4s + (tid & 3) * 16;
    }
    // thread t < BM stages the scale of activation row t, thread BM + t that of weight row t;
    // rows past the end read the last row (their results are never stored), other threads
    // read a value nobody uses: no load sits behind a lane-dependent branch
    const uint16_t *scp[SC];
#pragma unroll
    for (int i = 0; i < SC; ++i) {
        const int t = tid + i * NT;
        int64_t ra = m0 + (t < BM ? t : 0), rw = n0 + (t >= BM && t < BM + BN ? t - BM : 0);
        ra = ra < p.M ? ra : p.M - 1;
        rw = rw < p.N ? rw : p.N - 1;
        scp[i] = t >= BM && t < BM + BN ? p.w_scale + rw * G : p.a_scale + ra * G;
    }

    auto prefetch = [&](int g, Pre &pre) {
        v4u (&preA)[A8] = pre.a; v4u (&preB)[B8] = pre.b; uint16_t (&sc)[SC] = pre.sc;
        if (g < G4) {
#pragma unroll
            for (int i = 0; i < A4; ++i) preA[i] = *reinterpret_cast<const v4u *>(a4p[i] + g * 64);
#pragma unroll
            for (int i = 0; i < B4; ++i) preB[i] = *reinterpret_cast<const v4u *>(w4p[i] + g * 64);
        } else {
            const int g8 = g - G4;
#pragma unroll
            for (int i = 0; i < A8; ++i) {
                int64_t r = m0 + (tid >> 3) + i * (NT / 8);
                r = r < p.M ? r : p.M - 1;
                preA[i] = *reinterpret_cast<const v4u *>(p.a_q8 + r * o8s + g8 * 128 + (tid & 7) * 16);
            }
#pragma unroll
            for (int i = 0; i < B8; ++i) {
                int64_t r = n0 + (tid >> 3) + i * (NT / 8);
                r = r < p.N ? r : p.N - 1;
                preB[i] = *reinterpret_cast<const v4u *>(p.w_q8 + r * o8s + g8 * 128 + (tid & 7) * 16);
            }
        }
#pragma unroll
        for (int i = 0; i < SC; ++i) sc[i] = scp[i][g];
    };

    auto stage_to_lds = [&](int g, int stage, const Pre &pre) {
        const v4u (&preA)[A8] = pre.a; const v4u (&preB)[B8] = pre.b; const uint16_t (&sc)[SC] = pre.sc;
        unsigned char *sA = smem + stage * STAGE;
        unsigned char *sB = sA + BM * 128;
        float *sS = reinterpret_cast<float *>(sB + BN * 128);
        if (g < G4) {
            // an INT4 group stays packed in LDS (pieces 0..3 of the row's slot; LDS writes run
            // at a third of the read rate): the nibbles are widened after the fragment read
#pragma unroll
            for (int i = 0; i < A4; ++i)
                *reinterpret_cast<v4u *>(sA + lds_off((tid >> 2) + i * (NT / 4), tid & 3)) = preA[i];
#pragma unroll
            for (int i = 0; i < B4; ++i)
                *reinterpret_cast<v4u *>(sB + lds_off((tid >> 2) + i * (NT / 4), tid & 3)) = preB[i];
        } else {
#pragma unroll
            for (int i = 0; i < A8; ++i) {
                const int row = (tid >> 3) + i * (NT / 8);
                *reinterpret_cast<v4u *>(sA + lds_off(row, tid & 7)) = preA[i];
            }
#pragma unroll
            for (int i = 0; i < B8; ++i) {
                const int row = (tid >> 3) + i * (NT / 8);
                *reinterpret_cast<v4u *>(sB + lds_off(row, tid & 7)) = preB[i];
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

    // this set's groups; every set makes the same number of trips (and barriers), a set whose
    // share is one group shorter idles through the last one
    const int g_begin = (int)((int64_t)set * G / KS), g_end = (int)((int64_t)(set + 1) * G / KS);
    const int trips   = (G + KS - 1) / KS;
    // Two groups are in flight in registers: the loads issued in trip `it` are consumed at the
    // start of trip it + 2 (with one group of slack a trip lasted as long as a memory round trip).
    Pre pre0, pre1;
    if (g_begin < g_end) prefetch(g_begin, pre0);
    if (g_begin + 1 < g_end) prefetch(g_begin + 1, pre1);
    auto trip = [&](int it, Pre &pre) {
        const int g = g_begin + it;
        const int stage = it & 1;
        const bool live = g < g_end;
        if (live) stage_to_lds(g, stage, pre);
        __syncthreads();
        if (!live) return;
        if (g + 2 < g_end) prefetch(g + 2, pre);

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
        if (g < G4) {
            // A lane reads packed piece 2*kp + (lane >> 5) of its rows once and feeds two MFMAs
            // from it: the low nibbles of its 32 channels, then the high ones (as 16 * code; both
            // operands deal the group's channels to the four MFMAs the same way, and an exact
            // integer sum does not depend on the order).
#pragma unroll
            for (int kp = 0; kp < 2; ++kp) {
                const int piece = 2 * kp + (lane >> 5);
                v4i alo[TM], ahi[TM], blo[TN], bhi[TN];
#pragma unroll
                for (int i = 0; i < TM; ++i) {
                    const v4u r = *reinterpret_cast<const v4u *>(sA + lds_off(wm * WM + 32 * i + (lane & 31), piece));
                    alo[i] = nibbles_lo(r); ahi[i] = nibbles_hi(r);
                }
#pragma unroll
                for (int j = 0; j < TN; ++j) {
                    const v4u r = *reinterpret_cast<const v4u *>(sB + lds_off(wn * WN + 32 * j + (lane & 31), piece));
                    blo[j] = nibbles_lo(r); bhi[j] = nibbles_hi(r);
                }
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int j = 0; j < TN; ++j) {
                        c[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(alo[i], blo[j], c[i][j], 0, 0, 0);
                        c[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(ahi[i], bhi[j], c[i][j], 0, 0, 0);
                    }
            }
        } else {
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
    };
    for (int it = 0; it < trips; it += 2) {
        trip(it, pre0);
        if (it + 1 < trips) trip(it + 1, pre1);
    }

    if constexpr (KS > 1) {
        // sets 1 .. KS-1 hand their tiles over (value v of thread t at [v][t]: conflict-free)
        float *red = reinterpret_cast<float *>(smem_all);
        __syncthreads();                                  // every set is done with its stages
        if (set > 0) {
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
#pragma unroll
                    for (int r = 0; r < 16; ++r)
                        red[(((set - 1) * TM * TN + i * TN + j) * 16 + r) * NT + tid] = acc[i][j][r];
        }
        __syncthreads();
        if (set > 0) return;
        for (int s2 = 0; s2 < KS - 1; ++s2)
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
#pragma unroll
                    for (int r = 0; r < 16; ++r)
                        acc[i][j][r] += red[((s2 * TM * TN + i * TN + j) * 16 + r) * NT + tid];
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

template <int BM, int BN, int WM, int WN, bool DBG, int KS = 1>
hipError_t launch_tile(const GemmParams &p, hipStream_t stream)
{
    constexpr int NT = (BM / WM) * (BN / WN) * 64 * KS;
    constexpr int LDS = KS * 2 * ((BM + BN) * 128 + (BM + BN) * 4);
    static_assert(NT <= 1024 && LDS <= 160 * 1024, "workgroup limits");
    static_assert((KS - 1) * (NT / KS) * (WM / 32) * (WN / 32) * 16 * 4 <= LDS, "the sets' tiles fit the stages");
    const int64_t MB = (p.M + BM - 1) / BM, NB = (p.N + BN - 1) / BN;
    auto kern = &w4a4_gemm_kernel<BM, BN, WM, WN, DBG, KS>;
    static atom_launch::LdsOptIn opt_in;   // one attribute call per kernel variant and device
    hipError_t err = atom_launch::ensure_dynamic_lds(opt_in, reinterpret_cast<const void *>(kern), LDS);
    if (err != hipSuccess) return err;
    hipLaunchKernelGGL(kern, dim3((unsigned)(MB * NB)), dim3(NT), LDS, stream, p);
    return hipGetLastError();
}

template <bool DBG>
hipError_t dispatch(const GemmParams &p, hipStream_t stream)
{
    // M <= 64 streams the weights.  Outside the common decoding case (one INT8 group, whole blocks
    // of four groups or two left over, aligned scales: decode_tiled_supported), where the general
    // streaming kernel runs, a tiled kernel is the faster one from 33 rows on (four row blocks,
    // one workgroup per CU) and more than 4096 output channels (more than one round of
    // workgroups).  Measured with the weights coming from HBM, K = 4096, M = 64: N = 5120 18.3 us
    // general streaming kernel against 15.1 us tiled, N = 8192 19.1 against 15.5, N = 11008 27.5
    // against 19.7 (the kernels of the common case: 8.3, 9.1 and 15.3 us).
    if (!DBG && p.M <= 64 && (decode_tiled_supported(p) || !(p.M > 32 && p.N > 4096))) return launch_decode(p, stream);
    // 65 to 256 rows of the common case: the same streaming kernels on blocks of 64 rows, as long as
    // their workgroups pass in at most three rounds (weights from HBM, K = 4096, against the tiled
    // kernels below: M = 128: N = 4096 8.1 / 14.2 us, N = 8192 15.1 / 18.3, N = 12288 21.6 / 26.3, but
    // N = 16384 29.0 / 27.6; M = 192: N = 8192 21.0 / 24.2; M = 256: N = 4096 14.0 / 17.2, but N = 8192
    // 27.3 / 25.3; K = 11008, N = 4096: M = 128 19.8 / 34.3, M = 256 35.6 / 46.7)
    if (!DBG && p.M <= 256 && decode_tiled_supported(p) && decode_rounds(p) <= 3) return launch_decode(p, stream);
    // Launches of few tiles are bound by the latency of one tile's chain of K-steps: 64 x 64
    // tiles put every compute unit to work and four (or two) wavefront sets per workgroup split
    // that chain (M = 256, N = K = 4096: 25.7 us on 128 x 128 tiles with two sets).
    if constexpr (!DBG) {
        const int64_t t64 = ((p.M + 63) / 64) * ((p.N + 63) / 64);
        if (t64 <= 128) return launch_tile<64, 32, 32, 32, false, 4>(p, stream);    // twice the tiles
        if (t64 <= 256) return launch_tile<64, 64, 32, 32, false, 4>(p, stream);
        if (t64 <= 512) return launch_tile<64, 64, 32, 32, false, 2>(p, stream);
    }
    if (!DBG && p.M <= 64) return launch_big(p, stream);
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

static GemmParams params_of(const GemmArgs &a)
{
    GemmParams p;
    p.a_q4 = a.a_q4; p.a_q8 = a.a_q8; p.a_scale = a.a_scale;
    p.w_q4 = a.w_q4; p.w_q8 = a.w_q8; p.w_scale = a.w_scale;
    p.y = a.y; p.partials = nullptr;
    p.M = a.M; p.N = a.N; p.ldy = a.ldy; p.K = a.K; p.O = a.O;
    return p;
}

bool decode_tiled_supported(const GemmArgs &a) { return atom_gemm::decode_tiled_supported(params_of(a)); }

hipError_t launch_w4a4_gemm_decode_tiled(const GemmArgs &a, hipStream_t stream)
{
    return atom_gemm::launch_decode_tiled(params_of(a), stream);
}

hipError_t launch_tile_weight_decode(const void *q4, const void *q8, int64_t N, int K, int O, void *t4, void *t8,
                                     hipStream_t stream)
{
    return atom_gemm::launch_tile_weight(q4, q8, N, K, O, t4, t8, stream);
}

}  // namespace atom_internal
