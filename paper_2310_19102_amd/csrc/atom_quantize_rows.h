// Row routine of the activation front end, shared by the stand-alone front-end kernels and
// by the decode kernel that runs the front end in its prologue: RMSNorm, reorder (Section 4.1
// of the paper), dynamic group quantisation (Section 4.2, Section 2 symmetric equations).
//
// Compile WITHOUT fast-math: the fp32 division, sqrt and the absence of fused multiply-adds
// are part of the bit-exact contract with the CPU oracle.
#pragma once

#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include <stdint.h>

namespace atom_quantize_rows {

__device__ __forceinline__ void halves_to_floats(const uint4 &raw, float *f)
{
    const __half2 *h = reinterpret_cast<const __half2 *>(&raw);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        float2 t = __half22float2(h[i]);
        f[2 * i]     = t.x;
        f[2 * i + 1] = t.y;
    }
}

// h = fp16(a + b) per element: the sum of two fp16 values formed in fp32 and rounded once
// (where the fp32 sum is inexact the addends are more than 2^13 apart, nowhere near an
// fp16 rounding tie, so this is the correctly rounded fp16 sum)
__device__ __forceinline__ uint4 add_halves(const uint4 &a, const uint4 &b)
{
    float fa[8], fb[8];
    halves_to_floats(a, fa);
    halves_to_floats(b, fb);
    uint4 out;
    uint32_t *o = reinterpret_cast<uint32_t *>(&out);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const uint32_t lo = __half_as_ushort(__float2half_rn(fa[2 * i] + fb[2 * i]));
        const uint32_t hi = __half_as_ushort(__float2half_rn(fa[2 * i + 1] + fb[2 * i + 1]));
        o[i] = lo | (hi << 16);
    }
    return out;
}

// exp(x) on [-87, 87] from IEEE operations only (one value on every machine, the CPU
// oracle's included): n = round(x*log2(e)); r = x - n*ln2 with ln2 split in two, the first
// part short enough for n*ln2_hi to be exact; e^r by its Taylor polynomial of degree 7 in
// Horner form; 2^n through the exponent field.
__device__ __forceinline__ float exp_ieee(float x)
{
    x = x < -87.0f ? -87.0f : x;
    x = x > 87.0f ? 87.0f : x;
    const float n = rintf(x * 1.44269502162933349609375f);
    float r = fmaf(n, -0.693145751953125f, x);
    r = fmaf(n, -1.428606765330187045037746429443359375e-06f, r);
    float p = 1.0f / 5040.0f;
    p = fmaf(p, r, 1.0f / 720.0f);
    p = fmaf(p, r, 1.0f / 120.0f);
    p = fmaf(p, r, 1.0f / 24.0f);
    p = fmaf(p, r, 1.0f / 6.0f);
    p = fmaf(p, r, 0.5f);
    p = fmaf(p, r, 1.0f);
    p = fmaf(p, r, 1.0f);
    return p * __int_as_float(((int)n + 127) << 23);
}

// silu(g) * u in fp32: sigma = 1/(1 + exp(-g)) with an IEEE division, then (g*sigma)*u
__device__ __forceinline__ float silu_mul(float g, float u)
{
    const float sigma = 1.0f / (1.0f + exp_ieee(-g));
    return (g * sigma) * u;
}

// what happens to a row before it is normalised and quantised
constexpr int kPlain = 0;    // nothing
constexpr int kAdd = 1;      // x + res, rounded to fp16 and written to sum_out
constexpr int kSwiglu = 2;   // silu(x) * res in fp32 (x = gate row, res = up row), not stored

// max over the 16 lanes of a DPP row (xor butterfly; max is exact in any order)
__device__ __forceinline__ float row16_max(float v)
{
#pragma unroll
    for (int d = 1; d < 16; d <<= 1) v = fmaxf(v, __shfl_xor(v, d, 64));
    return v;
}

// max over the 16 lanes of a DPP row by rotations (max is exact in any order); one
// v_max_f32 with a DPP operand per step, no LDS crossbar traffic
__device__ __forceinline__ float row16_max_dpp(float v)
{
#define ATOM_ROW_ROR(n)                                                                          \
    v = fmaxf(v, __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(                          \
                     0, __builtin_bit_cast(int, v), 0x120 | (n), 0xF, 0xF, false)))
    ATOM_ROW_ROR(8);
    ATOM_ROW_ROR(4);
    ATOM_ROW_ROR(2);
    ATOM_ROW_ROR(1);
#undef ATOM_ROW_ROR
    return v;
}

// Scale of a group from its maximum (Section 2 symmetric equations, fp32, stored as fp16) and the
// codes of this lane's eight values: IEEE division by the stored scale through the shared
// reciprocal refinement described below, round-half-to-even, clamp.  Returns the stored scale,
// s = its fp32 value.  The codes stay floats (whole numbers): what packs them needs no integers
// (pack_nibbles8 below, the conversion to FP6).
__device__ __forceinline__ __half quantise_lane8(const float (&y)[8], float amax, bool is4, int nbits, float clip,
                                                 float (&q)[8], float &s)
{
    // normal channels: n = nbits (4, or 3 with the codes still in nibbles), outliers n = 8
    const float denom = is4 ? (nbits == 3 ? 7.0f : 15.0f) : 255.0f;
    const float qmin  = is4 ? (nbits == 3 ? -4.0f : -8.0f) : -128.0f;
    const float qmax  = is4 ? (nbits == 3 ? 3.0f : 7.0f) : 127.0f;
    const float s32   = ((2.0f * amax) * clip) / denom;
    const __half sh   = (s32 > 65504.0f) ? __ushort_as_half((unsigned short)0x7bffu)
                                         : __float2half_rn(s32);
    s = __half2float(sh);
    const float r0    = __builtin_amdgcn_rcpf(s);
    const float e0    = fmaf(-s, r0, 1.0f);
    const float r1    = fmaf(e0, r0, r0);
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        float qf = y[e] * r1;
        float t  = fmaf(-s, qf, y[e]);
        qf = fmaf(t, r1, qf);
        t  = fmaf(-s, qf, y[e]);
        qf = fmaf(t, r1, qf);
        qf = rintf(qf);
        q[e] = __builtin_amdgcn_fmed3f(qf, qmin, qmax);      // (finite: the same as min(max(qf, qmin), qmax))
    }
    return sh;
}

// Eight codes in [-8, 7], given as floats, to eight two's-complement nibbles, code 0 lowest.
// c0 + 16 c1 + 256 c2 + 4096 c3 is a whole number below 2^16 in magnitude, exact in fp32; with 8
// added to every code (0x8888 to the sum) the digits are the offset-binary nibbles and no digit
// borrows from the next; flipping the top bit of each nibble turns offset binary into two's
// complement.  Eleven instructions instead of a conversion, a mask, a shift and an or per code.
__device__ __forceinline__ uint32_t pack_nibbles8(const float (&c)[8])
{
    const float lo = fmaf(c[3], 4096.0f, fmaf(c[2], 256.0f, fmaf(c[1], 16.0f, c[0])));
    const float hi = fmaf(c[7], 4096.0f, fmaf(c[6], 256.0f, fmaf(c[5], 16.0f, c[4])));
    const uint32_t a = (uint32_t)((int)lo + 0x8888);                       // in [0, 0xffff]
    const uint32_t b = ((uint32_t)(int)hi << 16) + 0x88880000u;
    return (a | b) ^ 0x88888888u;
}

// Same result as the plain front-end kernel (compiler-generated IEEE division), bit for bit, for
// K <= 8 * NT * NS and clip >= 2^-20
// (NT threads per row),
// with the per-element work cut down:
//   * a workgroup walks several rows; the gather offsets of the reorder (they are the same
//     for every row) and gamma stay in registers, and the next row's global loads are in
//     flight while this row is quantised;
//   * the IEEE division by the group's scale shares the reciprocal refinement across the
//     group: r = rcp(s), r += r*(1 - s*r), then per element q = y*r and two residual
//     corrections q += r*(y - s*q).  This is instruction for instruction what the
//     compiler emits for y / s when v_div_scale does not rescale, which it does not for
//     the quotients that matter here: s comes from the group's own maximum, so
//     |y| / s <= (2^n - 1)/(2 clip) * (1 + 2^-11) and s >= 2^-24; quotients below 2^-100
//     round to code 0 either way.  A zero scale (all-zero group) yields zero codes;
//   * the group maximum is a DPP rotation reduction.
// The rows row_first, row_first + row_step, ... < rows are handled by the calling workgroup
// (NT threads, all of them call); lds holds K + (NORM ? K / 8 : 0) floats.  q4, q8 and scale
// are the canonical arrays (row strides (K - O) / 2, O and K / 128) and may live in LDS.
// IDENT: the row already is in reordered channel order (the producer emitted it so, Section 4.1
// of the paper: the reorder fused into the prior operator): thread t's vector t + NT*i is its own
// share of group (t + NT*i) / 16, nothing is staged or gathered, idx is not read and lds holds
// the K / 8 sums of squares only (NORM) or nothing.
struct NoHook { __device__ __forceinline__ void operator()() const {} };

// after_first_fetch is called once, right after the global loads of the first row are issued (a
// caller with loads of its own that may take longer to return issues them there).
// PACKED: the codes and scales do not go to the canonical arrays but straight into the unit images
// the packed GEMM reads (units of 64 rows; per unit one image per group: INT4 codes as FP6 E3M2 in
// three 16-byte chunks per row and half at 2048 c + 1024 h + 16 r, scales as 8-byte entries at
// 6144 + 8 r; INT8: chunk c of row r at 128 r + 16 ((c ^ r ^ (r/8 % 2)) % 8), scales at 8192 + 8 r).
// A row's packed bytes are first collected in LDS (pk_lds: 3 K4 / 4 + O bytes, in the order group,
// half, chunk), then copied out as whole 16-byte chunks.
typedef _Float16 pk_v32h __attribute__((ext_vector_type(32)));
typedef unsigned pk_v6u  __attribute__((ext_vector_type(6)));
constexpr int kImg4 = 6656, kImg8 = 8704, kSc4 = 6144, kSc8 = 8192;

template <bool NORM, int NS, int NT, int PRE, bool IDENT = false, bool PACKED = false, class Hook = NoHook>
__device__ __forceinline__
void quantize_rows_fast_body(float *lds, int64_t row_first, int64_t row_step,
                             const __half *x, int64_t rows, int64_t ld,
                             const __half *res, int64_t ldr, __half *sum_out, int64_t ldo,
                             const __half *__restrict__ gamma, float eps,
                             const int32_t *__restrict__ idx, int K, int O, int nbits, float clip,
                             uint8_t *q4, int8_t *q8, __half *scale, Hook after_first_fetch = Hook(),
                             uint8_t *pk_out = nullptr, uint8_t *pk_lds = nullptr)
{
    float *ybuf = lds;                        // [K]   staged row, original channel order (not IDENT)
    float *qbuf = lds + (IDENT ? 0 : K);      // [K/8] per-vector sums of squares (NORM only)

    const int tid  = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // the same in every lane: group decisions become scalar
    const int V    = K >> 3;
    const int K4   = K - O;
    const int G    = K >> 7;
    const int G4   = K4 >> 7;

    // gather offsets (bytes into ybuf) of this lane's 8 channels in each of its groups
    // (with 1024 threads two 16-bit channel numbers share a register)
    constexpr bool OPACK = NT >= 1024;
    uint32_t off[IDENT ? 1 : NS][OPACK ? 4 : 8];
#pragma unroll
    for (int j = 0; j < (IDENT ? 0 : NS); ++j) {
        const int g  = 4 * wave + (lane >> 4) + (NT / 16) * j;
        const int gg = g < G ? g : G - 1;
        const int j0 = gg * 128 + (lane & 15) * 8;
        const int4 i0 = *reinterpret_cast<const int4 *>(idx + j0);
        const int4 i1 = *reinterpret_cast<const int4 *>(idx + j0 + 4);
        const int id[8] = {i0.x, i0.y, i0.z, i0.w, i1.x, i1.y, i1.z, i1.w};
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const uint32_t c = min((unsigned)id[e], (unsigned)(K - 1));
            if (!OPACK)          off[j][e] = 4u * c;
            else if (e % 2 == 0) off[j][e / 2] = c;
            else                 off[j][e / 2] |= c << 16;
        }
    }
    // gamma stays in registers too, except with 1024 threads (128 registers per lane):
    // there each row re-reads it through the cache
    constexpr bool GREG = NT < 1024;
    uint4 graw[NORM && GREG ? NS : 1];
    if (NORM && GREG) {
#pragma unroll
        for (int i = 0; i < NS; ++i) {
            const int v = tid + NT * i;
            graw[i] = v < V ? *reinterpret_cast<const uint4 *>(gamma + 8 * v) : make_uint4(0, 0, 0, 0);
        }
    }

    uint4 raw[NS];
    uint4 rres[PRE != kPlain ? NS : 1];
    auto fetch_row = [&](int64_t row) {
        const __half *xr = x + row * ld;
#pragma unroll
        for (int i = 0; i < NS; ++i) {
            const int v = tid + NT * i;
            raw[i] = v < V ? *reinterpret_cast<const uint4 *>(xr + 8 * v) : make_uint4(0, 0, 0, 0);
            if (PRE != kPlain)
                rres[i] = v < V ? *reinterpret_cast<const uint4 *>(res + row * ldr + 8 * v)
                                : make_uint4(0, 0, 0, 0);
        }
    };
    int64_t row = row_first;
    if (row < rows) fetch_row(row);
    after_first_fetch();

    for (; row < rows; row += row_step) {
        float yv[IDENT ? NS : 1][8];          // IDENT: the row, normalised, stays in registers
        // ---- 0. residual add; the sum is the new residual stream and the row quantised below
        if (PRE == kAdd) {
#pragma unroll
            for (int i = 0; i < NS; ++i) {
                const int v = tid + NT * i;
                if (v < V) {
                    raw[i] = add_halves(raw[i], rres[i]);
                    *reinterpret_cast<uint4 *>(sum_out + row * ldo + 8 * v) = raw[i];
                }
            }
        }
        // ---- 1./2. stage the row (after RMSNorm, if any) in LDS, original channel order
        float r = 1.0f;
        if (NORM) {
#pragma unroll
            for (int i = 0; i < NS; ++i) {
                const int v = tid + NT * i;
                if (v < V) {
                    float f[8];
                    halves_to_floats(raw[i], f);
                    float s0 = f[0] * f[0], s1 = f[1] * f[1], s2 = f[2] * f[2], s3 = f[3] * f[3];
                    float s4 = f[4] * f[4], s5 = f[5] * f[5], s6 = f[6] * f[6], s7 = f[7] * f[7];
                    qbuf[v] = ((s0 + s1) + (s2 + s3)) + ((s4 + s5) + (s6 + s7));
                }
            }
            __syncthreads();
            float L = 0.0f;
            for (int v = lane; v < V; v += 64) L = L + qbuf[v];
#pragma unroll
            for (int d = 1; d < 64; d <<= 1) L = L + __shfl_xor(L, d, 64);
            const float mean = L / (float)K;
            r = 1.0f / sqrtf(mean + eps);
        }
#pragma unroll
        for (int i = 0; i < NS; ++i) {
            const int v = tid + NT * i;
            if (v < V) {
                float f[8];
                halves_to_floats(raw[i], f);
                if (PRE == kSwiglu) {
                    float u[8];
                    halves_to_floats(rres[i], u);
#pragma unroll
                    for (int e = 0; e < 8; ++e) f[e] = silu_mul(f[e], u[e]);
                }
                if (NORM) {
                    float g[8];
                    halves_to_floats(GREG ? graw[i] : *reinterpret_cast<const uint4 *>(gamma + 8 * v), g);
#pragma unroll
                    for (int e = 0; e < 8; ++e) f[e] = (f[e] * r) * g[e];
                }
                if constexpr (IDENT) {
#pragma unroll
                    for (int e = 0; e < 8; ++e) yv[i][e] = f[e];
                } else {
                    *reinterpret_cast<float4 *>(ybuf + 8 * v)     = make_float4(f[0], f[1], f[2], f[3]);
                    *reinterpret_cast<float4 *>(ybuf + 8 * v + 4) = make_float4(f[4], f[5], f[6], f[7]);
                }
            } else if constexpr (IDENT) {
#pragma unroll
                for (int e = 0; e < 8; ++e) yv[i][e] = 0.0f;
            }
        }
        // the next row's loads fly while this one is quantised
        if (row + row_step < rows) fetch_row(row + row_step);
        if (!IDENT) __syncthreads();

        // ---- 3./4. reorder, group amax, scale, quantise, pack ----------------
#pragma unroll
        for (int j = 0; j < NS; ++j) {
            const int  g    = 4 * wave + (lane >> 4) + (NT / 16) * j;
            const bool live = g < G;          // ragged last sweep: whole 16-lane rows idle
            const int  gg   = live ? g : G - 1;
            const int  j0   = gg * 128 + (lane & 15) * 8;
            float y[8];
            float amax = 0.0f;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                if constexpr (IDENT) {
                    y[e] = yv[j][e];
                } else {
                    uint32_t o = off[j][OPACK ? e / 2 : e];
                    if (OPACK) {
                        // unpacked here, per row: hoisted out of the row loop the unpacked
                        // offsets would take the registers the packing saves
                        asm volatile("" : "+v"(o));
                        o = e % 2 ? (o >> 16) << 2 : (o & 0xffffu) << 2;
                    }
                    y[e] = *reinterpret_cast<const float *>(reinterpret_cast<const unsigned char *>(ybuf) + o);
                }
                amax = fmaxf(amax, fabsf(y[e]));
            }
            amax = row16_max_dpp(amax);

            const bool  is4   = gg < G4;
            float q[8];
            float s;
            const __half sh = quantise_lane8(y, amax, is4, nbits, clip, q, s);
            const bool nz = s != 0.0f;
            if constexpr (PACKED) {
                if (live) {
                    const int pos = lane & 15;                      // 8 channels at 8 * pos of the group
                    const int64_t unit = row >> 6;
                    const int     r    = (int)(row & 63);
                    uint8_t *ubase = pk_out + unit * ((int64_t)G4 * kImg4 + (int64_t)(G - G4) * kImg8);
                    if (is4) {
                        // the E3M2 number of each code (a plain conversion: every code is representable);
                        // eight codes = 48 bits, at byte 6 (pos % 4) of the 24 bytes of their 32-channel block
                        pk_v32h h;
#pragma unroll
                        // (+ 0.0f: a code that was rounded up to zero is -0.0f, and FP6 has a sign bit)
                        for (int e = 0; e < 32; ++e) h[e] = e < 8 ? (_Float16)((nz ? q[e & 7] : 0.0f) + 0.0f) : (_Float16)0.0f;
                        const pk_v6u f6 = __builtin_amdgcn_cvt_scalef32_pk32_bf6_f16(h, 1.0f);
                        const int blk = pos >> 2;                   // block b: half b % 2, first or second MFMA b / 2
                        uint16_t *dst = reinterpret_cast<uint16_t *>(pk_lds + 96 * gg + 48 * (blk & 1) + 24 * (blk >> 1) + 6 * (pos & 3));
                        dst[0] = (uint16_t)f6[0];
                        dst[1] = (uint16_t)(f6[0] >> 16);
                        dst[2] = (uint16_t)f6[1];
                        if (pos == 0)
                            *reinterpret_cast<uint2 *>(ubase + (int64_t)gg * kImg4 + kSc4 + 8 * r) = make_uint2(__half_as_ushort(sh), 0u);
                    } else {
                        uint32_t w0 = 0, w1 = 0;
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            w0 |= (uint32_t)((int)q[e] & 0xFF) << (8 * e);
                            w1 |= (uint32_t)((int)q[e + 4] & 0xFF) << (8 * e);
                        }
                        *reinterpret_cast<uint2 *>(pk_lds + 3 * (K4 >> 2) + (j0 - K4)) = make_uint2(nz ? w0 : 0u, nz ? w1 : 0u);
                        if (pos == 0)
                            *reinterpret_cast<uint2 *>(ubase + (int64_t)G4 * kImg4 + (int64_t)(gg - G4) * kImg8 + kSc8 + 8 * r) =
                                make_uint2(__half_as_ushort(sh), 0u);
                    }
                }
            } else if (live) {
                if (is4) {
                    const uint32_t w = pack_nibbles8(q);
                    *reinterpret_cast<uint32_t *>(q4 + row * (int64_t)(K4 >> 1) + (j0 >> 1)) = nz ? w : 0u;
                } else {
                    uint32_t w0 = 0, w1 = 0;
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        w0 |= (uint32_t)((int)q[e] & 0xFF) << (8 * e);
                        w1 |= (uint32_t)((int)q[e + 4] & 0xFF) << (8 * e);
                    }
                    *reinterpret_cast<uint2 *>(q8 + row * (int64_t)O + (j0 - K4)) =
                        make_uint2(nz ? w0 : 0u, nz ? w1 : 0u);
                }
                if ((lane & 15) == 0) scale[row * (int64_t)G + gg] = sh;
            }
        }
        if (!IDENT || NORM || PACKED) __syncthreads();   // ybuf and qbuf are rewritten by the next row
        if constexpr (PACKED) {
            // the row's packed bytes, 16 at a time: chunk j of the INT4 part is (group j / 6, half
            // (j % 6) / 3, chunk j % 3); chunk j of the INT8 part is (group j / 8, source chunk j % 8)
            const int64_t unit = row >> 6;
            const int     r    = (int)(row & 63);
            uint8_t *ubase = pk_out + unit * ((int64_t)G4 * kImg4 + (int64_t)(G - G4) * kImg8);
            const int n4 = 6 * G4, n8 = O >> 4;
            for (int j = tid; j < n4 + n8; j += NT) {
                const uint4 v = *reinterpret_cast<const uint4 *>(pk_lds + 16 * j);
                uint8_t *dst;
                if (j < n4) {
                    const int gq = j / 6, hc = j - 6 * gq, hh = hc >= 3 ? 1 : 0, c = hc - 3 * hh;
                    dst = ubase + (int64_t)gq * kImg4 + 2048 * c + 1024 * hh + 16 * r;
                } else {
                    const int j8 = j - n4, g8 = j8 >> 3, c = j8 & 7;
                    dst = ubase + (int64_t)G4 * kImg4 + (int64_t)g8 * kImg8 + 128 * r + 16 * ((c ^ r ^ ((r >> 3) & 1)) & 7);
                }
                *reinterpret_cast<uint4 *>(dst) = v;
            }
            if (IDENT && !NORM) __syncthreads();     // (no other barrier stands before the next row's writes to pk_lds)
        }
    }
}

}  // namespace atom_quantize_rows
