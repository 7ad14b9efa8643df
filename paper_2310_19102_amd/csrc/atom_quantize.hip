// Fused activation front end and one-time weight quantisation for gfx950.
//
// One workgroup (4 wavefronts) per row:
//   1. the row is read once from HBM with 128-bit loads and staged in LDS as
//      fp32, in ORIGINAL channel order; with RMSNorm every 8-channel vector also
//      leaves its sum of squares in LDS;
//   2. every wavefront folds the vector sums in the fixed order that gives the
//      sum of squares exactly one correct fp32 value (vector v -> lane v mod 64
//      in increasing v, then an xor butterfly with strides 1..32), derives
//      r = 1/sqrt(S/K + eps) and rescales its share of the staged row by
//      r and gamma;
//   3. the reorder (Section 4.1 of the paper) is an LDS gather: lane l of a
//      16-lane row owns 8 consecutive REORDERED channels, so one 16-lane DPP row
//      holds one group of 128 and the group's amax is a 4-step row reduction;
//   4. scale (Section 2 symmetric equations, fp32, stored as fp16), IEEE
//      division by the stored scale, round-half-to-even, clamp, pack: a lane
//      emits one dword of eight INT4 codes or eight INT8 bytes, coalesced.
//
// Compile WITHOUT fast-math: the fp32 division, sqrt and the absence of
// fused multiply-adds are part of the bit-exact contract with the CPU oracle.

#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include <stdint.h>

#include "atom_internal.h"
#include "atom_launch.h"
#include "atom_quantize_rows.h"

namespace {

using namespace atom_quantize_rows;

constexpr int kThreads = 256;

// PRE = kAdd: x is first added to a residual row and the sum (fp16) is written out; x, res
// and sum_out may alias each other (every element is read and written by the same thread).
// PRE = kSwiglu: the row is silu(x) * res.
template <bool NORM, int PRE, bool MX = false>
__global__ __launch_bounds__(kThreads)
void quantize_rows_kernel(const __half *x, int64_t rows, int64_t ld,
                          const __half *res, int64_t ldr, __half *sum_out, int64_t ldo,
                          const __half *__restrict__ gamma, float eps,
                          const int32_t *__restrict__ idx, int K, int O, int nbits, float clip,
                          uint8_t *__restrict__ q4, int8_t *__restrict__ q8,
                          __half *__restrict__ scale, int gl)
{
    // gl: lanes per group = group size / 8 (8, 16 or 32; Section 5.4.1 of the paper varies the
    // group size); the MX variant passes 16 (its sweep of 128 channels holds four MX blocks)
    extern __shared__ __align__(16) float lds[];
    float *ybuf = lds;            // [K]   staged row, original channel order
    float *qbuf = lds + K;        // [K/8] per-vector sums of squares (NORM only)

    const int tid  = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // the same in every lane: group decisions become scalar
    const int V    = K >> 3;      // 8-channel vectors per row
    const int K4   = K - O;
    const int gs   = 8 * gl;      // group size
    const int glsh = 31 - __builtin_clz((unsigned)gl);
    const int G    = K / gs;
    const int G4   = K4 / gs;
    const int gpw  = 64 / gl;     // groups per wavefront sweep

    for (int64_t row = blockIdx.x; row < rows; row += gridDim.x) {
        const __half *xr = x + row * ld;

        // ---- 1. stage the row ------------------------------------------------
        for (int v = tid; v < V; v += kThreads) {
            uint4 raw = *reinterpret_cast<const uint4 *>(xr + 8 * v);
            if (PRE == kAdd) {
                raw = add_halves(raw, *reinterpret_cast<const uint4 *>(res + row * ldr + 8 * v));
                *reinterpret_cast<uint4 *>(sum_out + row * ldo + 8 * v) = raw;
            }
            float f[8];
            halves_to_floats(raw, f);
            if (PRE == kSwiglu) {
                float u[8];
                halves_to_floats(*reinterpret_cast<const uint4 *>(res + row * ldr + 8 * v), u);
#pragma unroll
                for (int e = 0; e < 8; ++e) f[e] = silu_mul(f[e], u[e]);
            }
            *reinterpret_cast<float4 *>(ybuf + 8 * v)     = make_float4(f[0], f[1], f[2], f[3]);
            *reinterpret_cast<float4 *>(ybuf + 8 * v + 4) = make_float4(f[4], f[5], f[6], f[7]);
            if (NORM) {
                float s0 = f[0] * f[0], s1 = f[1] * f[1], s2 = f[2] * f[2], s3 = f[3] * f[3];
                float s4 = f[4] * f[4], s5 = f[5] * f[5], s6 = f[6] * f[6], s7 = f[7] * f[7];
                qbuf[v] = ((s0 + s1) + (s2 + s3)) + ((s4 + s5) + (s6 + s7));
            }
        }
        __syncthreads();

        // ---- 2. RMSNorm ------------------------------------------------------
        if (NORM) {
            float L = 0.0f;
            for (int v = lane; v < V; v += 64) L = L + qbuf[v];
#pragma unroll
            for (int d = 1; d < 64; d <<= 1) L = L + __shfl_xor(L, d, 64);
            const float mean = L / (float)K;
            const float r    = 1.0f / sqrtf(mean + eps);
            // each thread rescales exactly the vectors it staged itself
            for (int v = tid; v < V; v += kThreads) {
                uint4 graw = *reinterpret_cast<const uint4 *>(gamma + 8 * v);
                float g[8];
                halves_to_floats(graw, g);
                float4 lo = *reinterpret_cast<float4 *>(ybuf + 8 * v);
                float4 hi = *reinterpret_cast<float4 *>(ybuf + 8 * v + 4);
                lo.x = (lo.x * r) * g[0]; lo.y = (lo.y * r) * g[1];
                lo.z = (lo.z * r) * g[2]; lo.w = (lo.w * r) * g[3];
                hi.x = (hi.x * r) * g[4]; hi.y = (hi.y * r) * g[5];
                hi.z = (hi.z * r) * g[6]; hi.w = (hi.w * r) * g[7];
                *reinterpret_cast<float4 *>(ybuf + 8 * v)     = lo;
                *reinterpret_cast<float4 *>(ybuf + 8 * v + 4) = hi;
            }
            __syncthreads();
        }

        // ---- 3./4. reorder, group amax, scale, quantise, pack ----------------
        // A wavefront sweep covers 64 / gl groups: gl consecutive lanes <-> group.
        for (int g = gpw * wave + (lane >> glsh); g < ((G + gpw - 1) & ~(gpw - 1)); g += gpw * (kThreads / 64)) {
            const bool live = g < G;          // ragged last sweep: whole groups of lanes idle
            const int  gg   = live ? g : G - 1;
            const int  j0   = gg * gs + (lane & (gl - 1)) * 8;
            int id[8];
            if (idx) {
                const int4 i0 = *reinterpret_cast<const int4 *>(idx + j0);
                const int4 i1 = *reinterpret_cast<const int4 *>(idx + j0 + 4);
                id[0] = i0.x; id[1] = i0.y; id[2] = i0.z; id[3] = i0.w;
                id[4] = i1.x; id[5] = i1.y; id[6] = i1.z; id[7] = i1.w;
            } else {           // no index: the row already is in reordered order
#pragma unroll
                for (int e = 0; e < 8; ++e) id[e] = j0 + e;
            }
            float y[8];
            float amax = 0.0f;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                y[e] = ybuf[min((unsigned)id[e], (unsigned)(K - 1))];
                amax = fmaxf(amax, fabsf(y[e]));
            }
            const bool  is4   = gg < G4;
            if constexpr (MX) {
                // MX variant: the 16 lanes hold four blocks of 32 channels (4 lanes each);
                // one power-of-two scale per block, FP4 E2M1 or FP8 E4M3 elements
                amax = fmaxf(amax, __shfl_xor(amax, 1, 64));
                amax = fmaxf(amax, __shfl_xor(amax, 2, 64));
                const float a = amax * clip;
                int byte = 0;
                if (a > 0.0f) {
                    int E = (__builtin_amdgcn_frexp_expf(a) - 1) - (is4 ? 2 : 8);   // floor(log2 a) - emax
                    E = E < -127 ? -127 : (E > 127 ? 127 : E);
                    byte = E + 127;
                }
                uint32_t w0 = 0, w1 = 0;
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const float    v    = __builtin_amdgcn_ldexpf(y[e], 127 - byte);   // exact
                    const uint32_t sign = __float_as_uint(v) >> 31;
                    const float    m    = fabsf(v);
                    if (is4) {
                        const uint32_t c = (uint32_t)(m > 0.25f) + (m >= 0.75f) + (m > 1.25f) + (m >= 1.75f) +
                                           (m > 2.5f) + (m >= 3.5f) + (m > 5.0f);
                        w0 |= (c | (sign << 3)) << (4 * e);
                    } else {
                        const float    t = fminf(m, 448.0f);
                        const uint32_t u = __float_as_uint(t);
                        // below 2^-6: multiples of 2^-9; above: round the mantissa to 3 bits, ties to even
                        const uint32_t c = t < 0.015625f ? (uint32_t)rintf(t * 512.0f)
                                                         : ((u + 0x7FFFFu + ((u >> 20) & 1u)) >> 20) - 960u;
                        const uint32_t b = c | (sign << 7);
                        if (e < 4) w0 |= b << (8 * e);
                        else       w1 |= b << (8 * (e - 4));
                    }
                }
                if (live) {
                    // step-major layout: 64 bytes (128 FP4 or 64 FP8 channels) of every row
                    // are contiguous per K step, scales as one dword per row and 128 channels
                    if (is4)
                        *reinterpret_cast<uint32_t *>(q4 + ((int64_t)(j0 >> 7) * rows + row) * 64 + ((j0 & 127) >> 1)) = w0;
                    else
                        *reinterpret_cast<uint2 *>(q8 + ((int64_t)((j0 - K4) >> 6) * rows + row) * 64 + ((j0 - K4) & 63)) =
                            make_uint2(w0, w1);
                    if ((lane & 3) == 0)
                        reinterpret_cast<uint8_t *>(scale)[((int64_t)(j0 >> 7) * rows + row) * 4 + ((j0 >> 5) & 3)] =
                            (uint8_t)byte;
                }
                continue;
            }
            for (int d = 1; d < gl; d <<= 1) amax = fmaxf(amax, __shfl_xor(amax, d, 64));   // max is exact in any order

            // normal channels: n = nbits (4, or 3 with the codes still in nibbles), outliers n = 8
            const float denom = is4 ? (nbits == 3 ? 7.0f : 15.0f) : 255.0f;
            const float qmin  = is4 ? (nbits == 3 ? -4.0f : -8.0f) : -128.0f;
            const float qmax  = is4 ? (nbits == 3 ? 3.0f : 7.0f) : 127.0f;
            const float s32   = ((2.0f * amax) * clip) / denom;
            const __half sh   = (s32 > 65504.0f) ? __ushort_as_half((unsigned short)0x7bffu)
                                                 : __float2half_rn(s32);
            const float s     = __half2float(sh);
            int q[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                float t = rintf(y[e] / s);
                t = fminf(fmaxf(t, qmin), qmax);
                q[e] = (s != 0.0f) ? (int)t : 0;
            }
            if (live) {
                if (is4) {
                    uint32_t w = 0;
#pragma unroll
                    for (int e = 0; e < 8; ++e) w |= (uint32_t)(q[e] & 0xF) << (4 * e);
                    *reinterpret_cast<uint32_t *>(q4 + row * (int64_t)(K4 >> 1) + (j0 >> 1)) = w;
                } else {
                    uint32_t w0 = 0, w1 = 0;
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        w0 |= (uint32_t)(q[e] & 0xFF) << (8 * e);
                        w1 |= (uint32_t)(q[e + 4] & 0xFF) << (8 * e);
                    }
                    *reinterpret_cast<uint2 *>(q8 + row * (int64_t)O + (j0 - K4)) = make_uint2(w0, w1);
                }
                if ((lane & (gl - 1)) == 0) scale[row * (int64_t)G + gg] = sh;
            }
        }
        __syncthreads();   // ybuf is rewritten by the next row
    }
}


template <bool NORM, int NS, int NT, int PRE, bool IDENT>
__global__ __launch_bounds__(NT)
void quantize_rows_fast_kernel(const __half *x, int64_t rows, int64_t ld,
                               const __half *res, int64_t ldr, __half *sum_out, int64_t ldo,
                               const __half *__restrict__ gamma, float eps,
                               const int32_t *__restrict__ idx, int K, int O, int nbits, float clip,
                               uint8_t *__restrict__ q4, int8_t *__restrict__ q8,
                               __half *__restrict__ scale)
{
    extern __shared__ __align__(16) float lds[];
    quantize_rows_fast_body<NORM, NS, NT, PRE, IDENT>(lds, blockIdx.x, gridDim.x, x, rows, ld, res, ldr, sum_out, ldo,
                                               gamma, eps, idx, K, O, nbits, clip, q4, q8, scale);
}

// out[r, :] = in[row_idx[r], :]: the offline helper that fuses a reorder into the operator
// producing the activations (its weight rows are permuted once); one workgroup per row
__global__ __launch_bounds__(256)
void permute_rows_kernel(const uint16_t *in, int64_t rows_in, int64_t cols, int64_t ld_in,
                         const int32_t *__restrict__ row_idx, uint16_t *__restrict__ out, int64_t ld_out)
{
    const int64_t r = blockIdx.x;
    int64_t src = row_idx[r];
    src = src < 0 ? 0 : (src >= rows_in ? rows_in - 1 : src);    // a bad index cannot leave the array
    for (int64_t c = threadIdx.x; c < cols; c += 256) out[r * ld_out + c] = in[src * ld_in + c];
}

}  // namespace

namespace atom_internal {

size_t quantize_lds_bytes(int K, bool norm)
{
    return sizeof(float) * (size_t)(K + (norm ? K / 8 : 0));
}

struct QuantArgs {
    const void *x; int64_t rows, ld;
    int pre;                                                       // kPlain, kAdd or kSwiglu
    const void *res; int64_t ldr; void *sum_out; int64_t ldo;     // second input row / fp16 sum out
    const void *gamma; float eps; const int32_t *idx; int K, O, nbits; float clip;
    void *q4, *q8, *scale;
    int gs;                                                        // group size: 128, or 64 / 256 (plain kernel)
};

template <bool NORM, int NS, int NT, int PRE, bool IDENT = false>
hipError_t launch_fast(const QuantArgs &a, size_t lds, hipStream_t stream)
{
    auto kern = &quantize_rows_fast_kernel<NORM, NS, NT, PRE, IDENT>;
    static atom_launch::LdsOptIn opt_in;   // the opt-in for more than 64 KB of dynamic LDS
    hipError_t err = atom_launch::ensure_dynamic_lds(opt_in, reinterpret_cast<const void *>(kern), lds);
    if (err != hipSuccess) return err;
    // workgroups resident per CU (LDS- and wave-limited), then rows dealt evenly over one
    // wave of them
    const int cus = atom_launch::compute_units();
    int64_t per_cu = (int64_t)(160 * 1024) / (int64_t)(lds > 0 ? lds : 1);
    const int64_t by_waves = 2048 / NT;                 // 32 wavefronts per CU
    per_cu = per_cu < 1 ? 1 : (per_cu > by_waves ? by_waves : per_cu);
    const int64_t slots = (int64_t)cus * per_cu;
    const int64_t rows_per_wg = (a.rows + slots - 1) / slots;
    const int64_t grid = (a.rows + rows_per_wg - 1) / rows_per_wg;
    hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(NT), lds, stream, (const __half *)a.x,
                       a.rows, a.ld, (const __half *)a.res, a.ldr, (__half *)a.sum_out, a.ldo,
                       (const __half *)a.gamma, a.eps, a.idx, a.K, a.O, a.nbits, a.clip, (uint8_t *)a.q4,
                       (int8_t *)a.q8, (__half *)a.scale);
    return hipGetLastError();
}

template <bool NORM, int PRE>
hipError_t launch_plain(const QuantArgs &a, size_t lds, hipStream_t stream)
{
    auto kern = &quantize_rows_kernel<NORM, PRE>;
    const int grid = (int)(a.rows < (int64_t)1 << 20 ? a.rows : (int64_t)1 << 20);
    // the opt-in for more than 64 KB of dynamic LDS is raised only when a call needs more
    static atom_launch::LdsOptIn opt_in;
    hipError_t err = atom_launch::ensure_dynamic_lds(opt_in, reinterpret_cast<const void *>(kern), lds);
    if (err != hipSuccess) return err;
    hipLaunchKernelGGL(kern, dim3(grid), dim3(kThreads), lds, stream, (const __half *)a.x, a.rows,
                       a.ld, (const __half *)a.res, a.ldr, (__half *)a.sum_out, a.ldo,
                       (const __half *)a.gamma, a.eps, a.idx, a.K, a.O, a.nbits, a.clip, (uint8_t *)a.q4,
                       (int8_t *)a.q8, (__half *)a.scale, a.gs / 8);
    return hipGetLastError();
}

template <bool NORM, int PRE>
hipError_t dispatch_quantize(const QuantArgs &a, hipStream_t stream)
{
    const bool sane_clip = a.clip >= 9.5367431640625e-07f && a.clip <= 1.0f && a.gs == 128;   // what the fast kernels take
    if (!a.idx && a.K <= 32768 && sane_clip) {
        // no index: the row already is in reordered order; nothing is staged in LDS but the
        // sums of squares, so the register sets alone bound the threads per row
        const size_t lq = NORM ? sizeof(float) * (size_t)(a.K / 8) : 0;
        if (a.K <= 2048)  return launch_fast<NORM, 1, 256, PRE, true>(a, lq, stream);
        if (a.K <= 4096)  return launch_fast<NORM, 2, 256, PRE, true>(a, lq, stream);
        if (a.K <= 8192)  return launch_fast<NORM, 2, 512, PRE, true>(a, lq, stream);
        if (a.K <= 12288) return launch_fast<NORM, 3, 512, PRE, true>(a, lq, stream);
        if (a.K <= 16384) return launch_fast<NORM, 4, 512, PRE, true>(a, lq, stream);
        if (a.K <= 24576) return launch_fast<NORM, 3, 1024, PRE, true>(a, lq, stream);
        return launch_fast<NORM, 4, 1024, PRE, true>(a, lq, stream);
    }
    const size_t lds = quantize_lds_bytes(a.K, NORM);
    // The fast kernel keeps ceil(K / (8 * threads)) gather-offset sets in registers and
    // relies on a sane clip; rows of 8192 channels and more are spread over 512 threads,
    // rows beyond 16384 channels over 1024 (one workgroup per CU: the staged row fills
    // most of the LDS).
    if (a.K <= 32768 && sane_clip) {
        if (a.K <= 2048)  return launch_fast<NORM, 1, 256, PRE>(a, lds, stream);
        if (a.K <= 4096)  return launch_fast<NORM, 2, 256, PRE>(a, lds, stream);
        if (a.K < 8192)   return launch_fast<NORM, 4, 256, PRE>(a, lds, stream);
        if (a.K <= 8192)  return launch_fast<NORM, 2, 512, PRE>(a, lds, stream);
        if (a.K <= 12288) return launch_fast<NORM, 3, 512, PRE>(a, lds, stream);
        if (a.K <= 16384) return launch_fast<NORM, 4, 512, PRE>(a, lds, stream);
        if (a.K <= 24576) return launch_fast<NORM, 3, 1024, PRE>(a, lds, stream);
        return launch_fast<NORM, 4, 1024, PRE>(a, lds, stream);
    }
    return launch_plain<NORM, PRE>(a, lds, stream);
}

// MX variant of the front end (FP4 / FP8 elements, one E8M0 scale byte per 32 channels in e8).
hipError_t launch_quantize_rows_mx(const void *x, int64_t rows, int64_t ld, const void *gamma,
                                   float eps, const int32_t *idx, int K, int O, float clip, void *q4,
                                   void *q8, void *e8, hipStream_t stream)
{
    const bool   norm = gamma != nullptr;
    const size_t lds  = quantize_lds_bytes(K, norm);
    auto kern = norm ? &quantize_rows_kernel<true, kPlain, true> : &quantize_rows_kernel<false, kPlain, true>;
    static atom_launch::LdsOptIn opt_in[2];
    hipError_t err = atom_launch::ensure_dynamic_lds(opt_in[norm], reinterpret_cast<const void *>(kern), lds);
    if (err != hipSuccess) return err;
    const int grid = (int)(rows < (int64_t)1 << 20 ? rows : (int64_t)1 << 20);
    hipLaunchKernelGGL(kern, dim3(grid), dim3(kThreads), lds, stream, (const __half *)x, rows, ld,
                       (const __half *)nullptr, (int64_t)0, (__half *)nullptr, (int64_t)0,
                       (const __half *)gamma, eps, idx, K, O, 4, clip, (uint8_t *)q4, (int8_t *)q8,
                       (__half *)e8, 16);
    return hipGetLastError();
}

hipError_t launch_quantize_rows(const void *x, int64_t rows, int64_t ld, int pre, const void *res,
                                int64_t ldr, void *sum_out, int64_t ldo, const void *gamma,
                                float eps, const int32_t *idx, int K, int O, int nbits, float clip,
                                void *q4, void *q8, void *scale, hipStream_t stream, int group_size)
{
    const QuantArgs a = {x, rows, ld, pre, res, ldr, sum_out, ldo, gamma, eps, idx, K, O, nbits, clip, q4, q8, scale,
                         group_size};
    const bool norm = gamma != nullptr;
    if (pre == kSwiglu) return dispatch_quantize<false, kSwiglu>(a, stream);   // no norm behind an activation
    if (pre == kAdd)
        return norm ? dispatch_quantize<true, kAdd>(a, stream) : dispatch_quantize<false, kAdd>(a, stream);
    return norm ? dispatch_quantize<true, kPlain>(a, stream) : dispatch_quantize<false, kPlain>(a, stream);
}

hipError_t launch_permute_rows(const void *in, int64_t rows_in, int64_t rows_out, int64_t cols, int64_t ld_in,
                               const int32_t *row_idx, void *out, int64_t ld_out, hipStream_t stream)
{
    hipLaunchKernelGGL(permute_rows_kernel, dim3((unsigned)rows_out), dim3(256), 0, stream,
                       (const uint16_t *)in, rows_in, cols, ld_in, row_idx, (uint16_t *)out, ld_out);
    return hipGetLastError();
}

}  // namespace atom_internal
