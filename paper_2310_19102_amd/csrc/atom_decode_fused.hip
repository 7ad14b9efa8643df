// One-launch linear layer for decode-sized batches (M <= 16): the activation front end
// (RMSNorm, reorder, dynamic group quantisation: Sections 4.1 and 4.2 of the paper) runs in
// the prologue of the weight-streaming group GEMM (Section 4.2 steps 1-3; Section 3 of the
// paper: small-batch dense layers are bound by reading the weights).
//
// Every workgroup owns 16 output channels and all of K, as in the stand-alone decode GEMM,
// and needs the quantised codes of all M rows.  M is tiny, so each workgroup quantises the
// rows itself, into LDS, with the row routine of the stand-alone front end (bit-identical
// codes and scales), while the first batch of its weight loads is in flight.  Every CU repeats
// that work (M K elements at some 20 vector operations each, one to two microseconds per row of
// 4096 channels), which is why the kernel pays only for the smallest batches:
//   1. the workgroup walks the M rows through the front-end routine (with the reorder index, or
//      without its gather when x already is in reordered order); codes and scales land in LDS in
//      the canonical layout ([M][K4/2] nibbles, [M][O] bytes, [M][G] fp16);
//   2. right after the loads of the first row of x, every wavefront issues the loads of the first
//      groups of its K-slice (loads return in order: issued earlier, they would hold the front
//      end back until the weights have arrived from HBM);
//   3. each wavefront multiplies its K-slice (INT8 MFMA 16x16x64 on nibbles widened to the
//      high half of a byte, the 2^-8 folded into the weight scale), dequantises per group
//      with fused multiply-adds in fp32, ascending groups;
//   4. the eight slices meet in LDS and are added in slice order; fp16 store.
// The sum over groups is the same tree as the stand-alone decode kernel's (eight K-slices in
// blocks of four groups when G is even and at least 4, else by single groups).
//
// MFMA 16x16x64 i8 layout: lane l supplies row (l & 15) of its operand and the 16 bytes of
// K-chunk (l >> 4); the result has column (l & 15) in lane l and rows 4*(l >> 4) + e in
// register e = 0..3.  Activations are the row operand.

#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include <stdint.h>

#include "atom_gemm_common.h"
#include "atom_internal.h"
#include "atom_launch.h"
#include "atom_quantize_rows.h"

namespace {

using namespace atom_gemm;
using namespace atom_quantize_rows;

typedef unsigned v4u __attribute__((ext_vector_type(4)));

constexpr int NW = 8;                     // wavefronts per workgroup = K-slices
constexpr int NT = NW * 64;
constexpr int TN = 16;                    // output channels per workgroup

struct FusedParams {
    const __half *x; int64_t ldx; int M;
    const __half *gamma; float eps; const int32_t *idx;
    int K, O, nbits; float clip;
    const uint8_t *w_q4; const int8_t *w_q8; const uint16_t *w_scale; int64_t N;
    uint16_t *y; int64_t ldy;
    uint8_t *dbg_q4; int8_t *dbg_q8; uint16_t *dbg_scale;     // the activation codes, or null
    unsigned lds_front;                                        // bytes of the front end's staging area
};

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

// NORM: RMSNorm in the front end.  NS: register sets of the front end (K <= 4096 * NS).
// DEPTH: groups whose weight loads are in flight together per wavefront.
// IDENT: no reorder index (x already is in reordered order): the row routine without its gather.
template <bool NORM, int NS, int DEPTH, bool IDENT>
__global__ __launch_bounds__(NT)
void decode_linear_kernel(const FusedParams p)
{
    extern __shared__ __align__(16) unsigned char smem[];
    const int K = p.K, O = p.O, K4 = K - O, G = K >> 7, G4 = K4 >> 7, M = p.M;
    // LDS: [front-end staging | a4 [M][K4/2] | a8 [M][O] | a_scale [M][G]]; the staging area
    // (at least 8 KB) holds the slices' partial tiles at the end
    float    *front = reinterpret_cast<float *>(smem);
    uint8_t  *a4 = smem + p.lds_front;
    int8_t   *a8 = reinterpret_cast<int8_t *>(a4 + (size_t)M * (K4 >> 1));
    uint16_t *as = reinterpret_cast<uint16_t *>(a8 + (size_t)M * O);

    const int tid  = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int col = lane & 15, kc = lane >> 4;
    const int64_t n0 = (int64_t)blockIdx.x * TN;

    // this wavefront's run of groups
    const bool blocks4 = G % 2 == 0 && G >= 4;
    const int nblk    = blocks4 ? (G + 3) >> 2 : G;
    const int g_begin = (blocks4 ? 4 : 1) * (int)((int64_t)wave * nblk / NW);
    const int g_end   = min(G, (blocks4 ? 4 : 1) * (int)((int64_t)(wave + 1) * nblk / NW));

    // weight row of this lane (clamped: rows >= N are computed and never stored)
    int64_t wr = n0 + col;
    wr = wr < p.N ? wr : p.N - 1;
    const uint8_t  *w4 = p.w_q4 + wr * (K4 >> 1) + kc * 16;
    const int8_t   *w8 = p.w_q8 + wr * O + kc * 16;
    const uint16_t *ws = p.w_scale + wr * G;

    uint4    wq[DEPTH][2];                // [slot][half]: an INT4 group uses half 0 only
    uint16_t wsc[DEPTH];
    auto load_weights = [&](int gb) {
#pragma unroll
        for (int d = 0; d < DEPTH; ++d) {
            const int g  = gb + d;
            const int gc = g < g_end ? g : (g_end > g_begin ? g_end - 1 : 0);     // dead slots re-read the last group
            if (gc < G4) {
                wq[d][0] = *reinterpret_cast<const uint4 *>(w4 + (size_t)gc * 64);
            } else {
                wq[d][0] = *reinterpret_cast<const uint4 *>(w8 + (size_t)(gc - G4) * 128);
                wq[d][1] = *reinterpret_cast<const uint4 *>(w8 + (size_t)(gc - G4) * 128 + 64);
            }
            wsc[d] = ws[gc];
        }
    };

    // ---- the front end, all rows, into LDS ---------------------------------------------------
    // The first weight loads are issued from inside the routine, right after the loads of its
    // first row: loads return in order, and the routine must not wait for the weights.
    quantize_rows_fast_body<NORM, NS, NT, kPlain, IDENT>(front, 0, 1, p.x, M, p.ldx, nullptr, 0, nullptr, 0,
                                                         p.gamma, p.eps, p.idx, K, O, p.nbits, p.clip, a4, a8,
                                                         reinterpret_cast<__half *>(as),
                                                         [&]() { load_weights(g_begin); });
    if (IDENT && !NORM) __syncthreads();       // (that variant of the routine has no barrier of its own)
    // every code and scale is in LDS
    if (p.dbg_q4 && blockIdx.x == 0) {
        for (int i = tid; i < M * (K4 >> 1) / 4; i += NT)
            reinterpret_cast<uint32_t *>(p.dbg_q4)[i] = reinterpret_cast<const uint32_t *>(a4)[i];
        for (int i = tid; i < M * O / 4; i += NT)
            reinterpret_cast<uint32_t *>(p.dbg_q8)[i] = reinterpret_cast<const uint32_t *>(a8)[i];
        for (int i = tid; i < M * G; i += NT) p.dbg_scale[i] = as[i];
    }

    // ---- this wavefront's K-slice -------------------------------------------------------------
    const bool a_ok = col < M;
    const int  mrow = a_ok ? col : 0;
    const uint8_t *a4r = a4 + (size_t)mrow * (K4 >> 1) + kc * 16;
    const int8_t  *a8r = a8 + (size_t)mrow * O + kc * 16;
    float acc[4] = {0.0f, 0.0f, 0.0f, 0.0f};
    const v4i zi = {0, 0, 0, 0};

    for (int gb = g_begin; gb < g_end; gb += DEPTH) {
        if (gb != g_begin) load_weights(gb);
#pragma unroll
        for (int d = 0; d < DEPTH; ++d) {
            const int g = gb + d;
            if (g >= g_end) break;
            const bool is4 = g < G4;
            v4i b0, b1, x0, x1;
            if (is4) {
                const uint4 av = *reinterpret_cast<const uint4 *>(a4r + (size_t)g * 64);
                b0 = widen_lo(wq[d][0]); b1 = widen_hi(wq[d][0]);
                x0 = widen_lo(av);       x1 = widen_hi(av);
            } else {
                b0 = __builtin_bit_cast(v4i, wq[d][0]);
                b1 = __builtin_bit_cast(v4i, wq[d][1]);
                x0 = *reinterpret_cast<const v4i *>(a8r + (size_t)(g - G4) * 128);
                x1 = *reinterpret_cast<const v4i *>(a8r + (size_t)(g - G4) * 128 + 64);
            }
            if (!a_ok) { x0 = zi; x1 = zi; }
            // 2^-8 of the nibble widening (both operands) folded into the weight scale (exact)
            const float wsf = half_bits_to_float(wsc[d]) * (is4 ? (1.0f / 256.0f) : 1.0f);
            v4i c = __builtin_amdgcn_mfma_i32_16x16x64_i8(x0, b0, zi, 0, 0, 0);
            c = __builtin_amdgcn_mfma_i32_16x16x64_i8(x1, b1, c, 0, 0, 0);
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int m = 4 * kc + e;
                const float sa = m < M ? half_bits_to_float(as[m * G + g]) : 0.0f;
                acc[e] = fmaf((float)c[e], sa * wsf, acc[e]);
            }
        }
    }

    // ---- the eight K-slices meet in LDS and are added in slice order --------------------------
    float (*red)[4][64] = reinterpret_cast<float (*)[4][64]>(front);
#pragma unroll
    for (int e = 0; e < 4; ++e) red[wave][e][lane] = acc[e];
    __syncthreads();
    if (tid < 4 * 64) {
        const int l = tid & 63, e = tid >> 6;
        float s = 0.0f;
#pragma unroll
        for (int w = 0; w < NW; ++w) s += red[w][e][l];
        const int     m = 4 * (l >> 4) + e;
        const int64_t n = n0 + (l & 15);
        if (m < M && n < p.N) p.y[(int64_t)m * p.ldy + n] = __half_as_ushort(__float2half_rn(s));
    }
}

unsigned front_bytes(int K, bool norm, bool ident)
{
    const unsigned need = 4u * (unsigned)((ident ? 0 : K) + (norm ? K / 8 : 0));
    const unsigned red  = NW * 4 * 64 * 4;
    return ((need > red ? need : red) + 15u) & ~15u;
}

template <bool NORM, int NS, int DEPTH, bool IDENT>
hipError_t launch_cfg(const FusedParams &p, size_t lds, hipStream_t stream)
{
    auto kern = &decode_linear_kernel<NORM, NS, DEPTH, IDENT>;
    static atom_launch::LdsOptIn opt_in;
    hipError_t err = atom_launch::ensure_dynamic_lds(opt_in, reinterpret_cast<const void *>(kern), lds);
    if (err != hipSuccess) return err;
    hipLaunchKernelGGL(kern, dim3((unsigned)((p.N + TN - 1) / TN)), dim3(NT), lds, stream, p);
    return hipGetLastError();
}

template <bool NORM, int NS>
hipError_t launch_depth(const FusedParams &p, size_t lds, hipStream_t stream)
{
    // the longest run of groups of a wavefront: one batch of four where that is all there is
    const int G = p.K >> 7;
    const bool blocks4 = G % 2 == 0 && G >= 4;
    const int nblk = blocks4 ? (G + 3) >> 2 : G;
    const int run = (blocks4 ? 4 : 1) * ((nblk + NW - 1) / NW);
    if (p.idx) return run <= 4 ? launch_cfg<NORM, NS, 4, false>(p, lds, stream) : launch_cfg<NORM, NS, 8, false>(p, lds, stream);
    return run <= 4 ? launch_cfg<NORM, NS, 4, true>(p, lds, stream) : launch_cfg<NORM, NS, 8, true>(p, lds, stream);
}

}  // namespace

namespace atom_internal {

size_t decode_linear_lds_bytes(int M, int K, int O, bool norm, bool ident)
{
    return (size_t)front_bytes(K, norm, ident) + (size_t)M * ((size_t)(K - O) / 2 + (size_t)O + 2 * (size_t)(K / 128));
}

hipError_t launch_decode_linear(const void *x, int M, int64_t ldx, const void *gamma, float eps,
                                const int32_t *idx, int K, int O, int nbits, float clip,
                                const void *w_q4, const void *w_q8, const void *w_scale, int64_t N,
                                void *y, int64_t ldy, void *dbg_q4, void *dbg_q8, void *dbg_scale,
                                hipStream_t stream)
{
    const bool norm = gamma != nullptr;
    FusedParams p;
    p.x = static_cast<const __half *>(x); p.ldx = ldx; p.M = M;
    p.gamma = static_cast<const __half *>(gamma); p.eps = eps; p.idx = idx;
    p.K = K; p.O = O; p.nbits = nbits; p.clip = clip;
    p.w_q4 = static_cast<const uint8_t *>(w_q4); p.w_q8 = static_cast<const int8_t *>(w_q8);
    p.w_scale = static_cast<const uint16_t *>(w_scale); p.N = N;
    p.y = static_cast<uint16_t *>(y); p.ldy = ldy;
    p.dbg_q4 = static_cast<uint8_t *>(dbg_q4); p.dbg_q8 = static_cast<int8_t *>(dbg_q8);
    p.dbg_scale = static_cast<uint16_t *>(dbg_scale);
    p.lds_front = front_bytes(K, norm, idx == nullptr);
    const size_t lds = decode_linear_lds_bytes(M, K, O, norm, idx == nullptr);
    if (K <= 4096) return norm ? launch_depth<true, 1>(p, lds, stream) : launch_depth<false, 1>(p, lds, stream);
    if (K <= 8192) return norm ? launch_depth<true, 2>(p, lds, stream) : launch_depth<false, 2>(p, lds, stream);
    return norm ? launch_depth<true, 3>(p, lds, stream) : launch_depth<false, 3>(p, lds, stream);
}

}  // namespace atom_internal
