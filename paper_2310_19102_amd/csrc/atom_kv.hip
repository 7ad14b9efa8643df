// INT4 KV cache for gfx950: asymmetric per-head quantisation (Section 2 of the paper,
// asymmetric equations; Section 4.4: granularity of one attention head) and decode-stage
// attention that reads the cache in 4 bits and dequantises inside the operator
// (Sections 4.4 and 4.5).
//
// Cache layout (one K cache and one V cache, same shape):
//   codes [B, Hkv, Tmax, D/2] bytes, two codes per byte, even d in the low nibble
//   scale [B, Hkv, Tmax] fp16,  zero [B, Hkv, Tmax] int16
// i.e. 64 + 4 bytes per token and head at D = 128: 4.25 bits per element.

#include <hip/hip_runtime.h>
#include <type_traits>
#include <hip/hip_fp16.h>
#include <stdint.h>

#include <atomic>

#include "atom_internal.h"

namespace {

typedef _Float16 h2 __attribute__((ext_vector_type(2)));

// ---------------------------------------------------------------- quantise rows

// max / min over the LPR (8 or 16) lanes that share a row; LPR lanes are consecutive and
// aligned, so rotations inside the 16-lane DPP row stay inside the row for LPR = 16, and an
// xor butterfly is used for LPR = 8
template <int LPR>
__device__ __forceinline__ void row_minmax(float &mx, float &mn)
{
    if constexpr (LPR == 16) {            // DPP rotations of the 16-lane row: vector-ALU speed, no LDS crossbar
#define ATOM_ROW_ROR(n)                                                                              \
        mx = fmaxf(mx, __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(                        \
                           0, __builtin_bit_cast(int, mx), 0x120 | (n), 0xF, 0xF, false)));          \
        mn = fminf(mn, __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(                        \
                           0, __builtin_bit_cast(int, mn), 0x120 | (n), 0xF, 0xF, false)))
        ATOM_ROW_ROR(8);
        ATOM_ROW_ROR(4);
        ATOM_ROW_ROR(2);
        ATOM_ROW_ROR(1);
#undef ATOM_ROW_ROR
    } else {
#pragma unroll
        for (int d = 1; d < LPR; d <<= 1) {
            mx = fmaxf(mx, __shfl_xor(mx, d, 64));
            mn = fminf(mn, __shfl_xor(mn, d, 64));
        }
    }
}

// One row of D = 8 * LPR values per LPR lanes, 64 / LPR rows per wavefront.
//   s = fp16(((max - min) * clip) / 15), z = clamp(rne(-min / s)), code = clamp(rne(x/s) + z, 0, 15)
// with correctly rounded fp32 quotients by the stored scale; a zero scale gives zero codes and z = 0.
// Output row index: r (pos == nullptr), or r * Tmax + pos[r / rows_per_seq] (append one
// token per sequence: row r = (sequence, head)); rows whose position is outside
// [0, Tmax) write nothing.
// kRows: rows per lane group, i.e. loads in flight per lane: 4 for bulk quantisation, 1 for the
// append of a few hundred rows (there four rows per lane group only quarter the grid)
template <int LPR, int kRows>
__global__ __launch_bounds__(256)
void kv_quantize_kernel(const __half *__restrict__ x0, int64_t R, int64_t ldx, float clip,
                        const int32_t *__restrict__ pos, int32_t rows_per_seq, int64_t Tmax,
                        uint8_t *__restrict__ q0, __half *__restrict__ scale0,
                        int16_t *__restrict__ zero0, const __half *__restrict__ x1,
                        uint8_t *__restrict__ q1, __half *__restrict__ scale1,
                        int16_t *__restrict__ zero1)
{
    constexpr int D = 8 * LPR;
    // grid.y = 2: the same rows of a second tensor into a second cache (K and V of one append)
    const bool second = blockIdx.y != 0;
    const __half *__restrict__ x     = second ? x1 : x0;
    uint8_t      *__restrict__ q     = second ? q1 : q0;
    __half       *__restrict__ scale = second ? scale1 : scale0;
    int16_t      *__restrict__ zero  = second ? zero1 : zero0;
    const int64_t r0 = ((int64_t)blockIdx.x * 256 + threadIdx.x) / LPR;
    const int64_t stride = (int64_t)gridDim.x * (256 / LPR);
    const int     j = threadIdx.x % LPR;
    uint4 raws[kRows];
#pragma unroll
    for (int u = 0; u < kRows; ++u) {
        const int64_t ru = r0 + u * stride;
        const int64_t rr = ru < R ? ru : R - 1;          // idle lanes repeat the last row
        raws[u] = *reinterpret_cast<const uint4 *>(x + rr * ldx + 8 * j);
    }
#pragma unroll
    for (int u = 0; u < kRows; ++u) {
    const int64_t r = r0 + u * stride;
    const bool live = r < R;
    const uint4 raw = raws[u];
    const __half2 *hp = reinterpret_cast<const __half2 *>(&raw);
    float f[8];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const float2 t = __half22float2(hp[i]);
        f[2 * i] = t.x;
        f[2 * i + 1] = t.y;
    }
    float mx = f[0], mn = f[0];
#pragma unroll
    for (int i = 1; i < 8; ++i) {
        mx = fmaxf(mx, f[i]);
        mn = fminf(mn, f[i]);
    }
    row_minmax<LPR>(mx, mn);
    const float  s32 = ((mx - mn) * clip) / 15.0f;
    const __half sh  = (s32 > 65504.0f) ? __ushort_as_half((unsigned short)0x7bffu) : __float2half_rn(s32);
    const float  s   = __half2float(sh);
    int z = 0;
    uint32_t w = 0;
    if (s != 0.0f) {
        // Nine quotients by the same divisor: one refined reciprocal, then two residual
        // corrections per quotient (q += (y - s q) / s, the residual exact in an fma) give the
        // correctly rounded y / s that the IEEE division sequence gives, at a third of its
        // instructions.  y and s are fp16 numbers (s >= 2^-24, |y| <= 65504): no quotient,
        // reciprocal or residual leaves the fp32 range.
        const float r0 = __builtin_amdgcn_rcpf(s);
        const float r1 = fmaf(fmaf(-s, r0, 1.0f), r0, r0);
        auto div_s = [&](float y) {
            float qf = y * r1;
            qf = fmaf(fmaf(-s, qf, y), r1, qf);
            qf = fmaf(fmaf(-s, qf, y), r1, qf);
            return qf;
        };
        float zf = rintf(div_s(-mn));
        zf = fminf(fmaxf(zf, -32768.0f), 32767.0f);
        z = (int)zf;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            float t = rintf(div_s(f[i]));
            t = fminf(fmaxf(t, -100000.0f), 100000.0f);
            int c = (int)t + z;
            c = c < 0 ? 0 : (c > 15 ? 15 : c);
            w |= (uint32_t)c << (4 * i);
        }
    }
    if (live) {
        int64_t orow = r;
        bool    keep = true;
        if (pos) {                                       // a position outside the cache is dropped
            const int64_t p = pos[r / rows_per_seq];
            keep = p >= 0 && p < Tmax;
            orow = r * Tmax + p;
        }
        if (keep) {
            *reinterpret_cast<uint32_t *>(q + orow * (D / 2) + 4 * j) = w;
            if (j == 0) {
                scale[orow] = sh;
                zero[orow]  = (int16_t)z;
            }
        }
    }
    }   // rows of this lane group
}

// ---------------------------------------------------------------- decode attention

// sum / max over the 16 lanes of a DPP row by rotations
__device__ __forceinline__ float row16_sum(float v)
{
#define ATOM_ROW_ROR(n)                                                                          \
    v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v),   \
                                                               0x120 | (n), 0xF, 0xF, false))
    ATOM_ROW_ROR(8);
    ATOM_ROW_ROR(4);
    ATOM_ROW_ROR(2);
    ATOM_ROW_ROR(1);
#undef ATOM_ROW_ROR
    return v;
}
__device__ __forceinline__ float row16_max(float v)
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

// The eight codes of a dword (code n in bits 4n..4n+3) as four fp16 pairs with two shifts:
// a code placed in mantissa bits 6..9 under the exponent of 16 reads as 16 + c, one placed
// in bits 2..5 under the exponent of 256 reads as 256 + c, both exactly.
//   pr[0] = (16 + n1, 16 + n5)   pr[1] = (256 + n0, 256 + n4)      from w << 2
//   pr[2] = (16 + n3, 16 + n7)   pr[3] = (256 + n2, 256 + n6)      from w >> 6
// The offsets are subtracted once per sum by the caller.
constexpr int   kNib[4] = {1, 0, 3, 2};                  // low-half code of pair k
constexpr float kOff[4] = {16.0f, 256.0f, 16.0f, 256.0f};

__device__ __forceinline__ uint32_t and_or(uint32_t a, uint32_t mask, uint32_t magic)
{
    uint32_t r;
    asm("v_and_or_b32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "s"(mask), "v"(magic));
    return r;
}

// All eight as 16 + c, pr[k] = (16 + n_k, 16 + n_(k+4)), with four shifts: for sums whose
// result may be small against the offsets' total (the value side of attention).
__device__ __forceinline__ void unpack8_16(uint32_t w, uint32_t (&pr)[4])
{
    pr[0] = and_or(w << 6, 0x03C003C0u, 0x4C004C00u);
    pr[1] = and_or(w << 2, 0x03C003C0u, 0x4C004C00u);
    pr[2] = and_or(w >> 2, 0x03C003C0u, 0x4C004C00u);
    pr[3] = and_or(w >> 6, 0x03C003C0u, 0x4C004C00u);
}

__device__ __forceinline__ void unpack8(uint32_t w, uint32_t (&pr)[4])
{
    const uint32_t a = w << 2, b = w >> 6;
    pr[0] = and_or(a, 0x03C003C0u, 0x4C004C00u);
    pr[1] = and_or(a, 0x003C003Cu, 0x5C005C00u);
    pr[2] = and_or(b, 0x03C003C0u, 0x4C004C00u);
    pr[3] = and_or(b, 0x003C003Cu, 0x5C005C00u);
}

// max over the lanes l, l ^ 16, l ^ 32, l ^ 48 with the lane-half swaps of gfx950 (vector ALU
// speed; a ds_bpermute pair per exchange would sit on the critical path of every step).  A swap
// exchanges the upper half (32) or the odd rows (16) of its first register with the lower half
// or the even rows of its second; fed two copies of v, the two results hold, lane by lane, v of
// the lane itself and of its partner.  This compiler folds max(first result, second result)
// into the first result, so the second one passes through an empty asm statement (no
// instruction; it only hides where the value came from), and `zero`, a 0 the compiler cannot
// see, keeps the two inputs distinct values.
__device__ __forceinline__ float max_across_chunks(float v, unsigned zero)
{
    typedef unsigned v2ui __attribute__((ext_vector_type(2)));
    unsigned u = __builtin_bit_cast(unsigned, v);
    v2ui r = __builtin_amdgcn_permlane32_swap(u, u | zero, false, false);
    unsigned other = r[1];
    asm volatile("" : "+v"(other));
    u = __builtin_bit_cast(unsigned, fmaxf(__builtin_bit_cast(float, r[0]), __builtin_bit_cast(float, other)));
    r = __builtin_amdgcn_permlane16_swap(u, u | zero, false, false);
    other = r[1];
    asm volatile("" : "+v"(other));
    return fmaxf(__builtin_bit_cast(float, r[0]), __builtin_bit_cast(float, other));
}

// the same exchange for a sum: v(l) + v(l ^ 16), then that + its l ^ 32 partner (the order of
// the two ds_bpermute exchanges it replaces: float addition commutes, the result is bit-identical)
__device__ __forceinline__ float sum_across_chunks(float v, unsigned zero)
{
    typedef unsigned v2ui __attribute__((ext_vector_type(2)));
    unsigned u = __builtin_bit_cast(unsigned, v);
    v2ui r = __builtin_amdgcn_permlane16_swap(u, u | zero, false, false);
    unsigned other = r[1];
    asm volatile("" : "+v"(other));
    u = __builtin_bit_cast(unsigned, __builtin_bit_cast(float, r[0]) + __builtin_bit_cast(float, other));
    r = __builtin_amdgcn_permlane32_swap(u, u | zero, false, false);
    other = r[1];
    asm volatile("" : "+v"(other));
    return __builtin_bit_cast(float, r[0]) + __builtin_bit_cast(float, other);
}

// value i (0..31) of the 32 fp16 numbers held by four 16-byte registers (i known at compile time)
__device__ __forceinline__ float half_of(const uint4 (&raw)[4], int i)
{
    const uint4 &v = raw[i >> 3];
    const uint32_t w = ((i >> 1) & 3) == 0 ? v.x : ((i >> 1) & 3) == 1 ? v.y : ((i >> 1) & 3) == 2 ? v.z : v.w;
    return __half2float(__ushort_as_half((unsigned short)((i & 1) ? w >> 16 : w & 0xFFFFu)));
}

constexpr int kTile  = 16;                // tokens per wavefront step
constexpr int kTokens = 64;                // tokens per wavefront group: four steps, one per ring slot

// One workgroup per (sequence, query head) and split of the token range, head dimension 128.
// A wavefront owns every kWaves-th group of 64 tokens and walks it in four steps of 16 tokens:
// lane l holds token (l & 15) and the 32 head dimensions of chunk (l >> 4), i.e. 16 bytes of
// that token's K row and 16 bytes of its V row (a wavefront load is 1 KB of contiguous cache).
//   scores  : the codes become fp16 offset + c, two at a time (unpack8), and meet the
//             matching pairs of q in v_dot2_f32_f16 (fp32 accumulate); the offsets and the
//             zero point leave as sum(offset * q) + z * sum(q) per chunk (offsets of 16 and
//             256 keep the cancellation in fp32 harmless); the four chunks of a token are
//             added across lanes; then * scale * sm_scale.
//   softmax : online, per wavefront (running max m and sum l); the accumulators are rescaled
//             only when the maximum moves.
//   values  : acc[d] += w * (16 + code[d]) with w = p * v_scale (unpack8_16), the fp16 codes
//             read by mixed-precision fmas; the 16 and the zero points leave once per group
//             of 64 tokens through the sums of w and w * z; the 16 tokens of the lanes meet
//             once, at the end; the wavefronts merge through LDS.
//   loads   : the codes of the next group (four steps ahead) are in flight while a step is
//             computed.  Scales and zero points are read once per group, lane l taking
//             token l of the 64, one full cache line per array, and reach the lane that
//             needs them through ds_bpermute: 2-byte loads per step would have several
//             wavefronts wait on the same line, which stalls the vector cache.
template <int kWaves>                     // wavefronts per workgroup: 4, or 16 when B * H alone is a thin grid
__global__ __launch_bounds__(kWaves * 64)
void decode_attention_kv4_kernel(const __half *__restrict__ q, int H, int Hkv, int64_t Tmax,
                                 const int32_t *__restrict__ seq_len,
                                 const uint8_t *__restrict__ kq, const __half *__restrict__ ks,
                                 const int16_t *__restrict__ kz, const uint8_t *__restrict__ vq,
                                 const __half *__restrict__ vs, const int16_t *__restrict__ vz,
                                 float sm_scale, __half *__restrict__ out, int groups_per_split,
                                 float *__restrict__ part)
{
    constexpr int D = 128;
    __shared__ float s_acc[kWaves][D];
    __shared__ float s_m[kWaves], s_l[kWaves];

    const int b = blockIdx.x / H, h = blockIdx.x % H;
    const int kvh = h / (H / Hkv);
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int tl = lane & 15, c = lane >> 4;
    int T = seq_len[b];
    T = T < 0 ? 0 : (T > Tmax ? (int)Tmax : T);          // never read past the cache
    const int64_t base = ((int64_t)b * Hkv + kvh) * Tmax;
    const uint8_t *kb = kq + base * (D / 2), *vb = vq + base * (D / 2);
    const __half  *ksb = ks + base, *vsb = vs + base;
    const int16_t *kzb = kz + base, *vzb = vz + base;

    // this workgroup's share of the groups (all of them when the grid has one split)
    const int g_first = blockIdx.y * groups_per_split;
    const int g_end   = min((T + kTokens - 1) / kTokens, g_first + groups_per_split);
    int  G     = g_first + wave;
    const bool alive = G < g_end;                        // then T >= 1: clamped addresses are valid
    const int  t_last = min(T, g_end * kTokens) - 1;     // loads never leave this split's tokens

    struct Stage { uint4 k, v; };
    Stage st[4];
    uint32_t kmeta = 0, vmeta = 0;        // scale bits | zero << 16 of token `lane` of the group
    auto fetch = [&](Stage &s_, int tile) {
        int t = tile * kTile + tl;
        t = t <= t_last ? t : t_last;     // masked tokens and steps past the end repeat the last token
        const uint32_t off = (uint32_t)t * (D / 2) + 16u * c;
        s_.k = *reinterpret_cast<const uint4 *>(kb + off);
        s_.v = *reinterpret_cast<const uint4 *>(vb + off);
    };
    auto fetch_meta = [&](int g, uint32_t &km, uint32_t &vm) {
        int t = g * kTokens + lane;
        t = t <= t_last ? t : t_last;
        km = (uint32_t)__half_as_ushort(ksb[(uint32_t)t]) | ((uint32_t)(uint16_t)kzb[(uint32_t)t] << 16);
        vm = (uint32_t)__half_as_ushort(vsb[(uint32_t)t]) | ((uint32_t)(uint16_t)vzb[(uint32_t)t] << 16);
    };
    if (alive) {                          // the first loads leave before q is read
        fetch_meta(G, kmeta, vmeta);
#pragma unroll
        for (int i = 0; i < 4; ++i) fetch(st[i], 4 * G + i);
    }

    // this lane's 32 query values as 16 pairs in the order unpack8 delivers the codes of a
    // dword (dword j holds d = 32c + 8j + 0..7), and the sums that take the offsets back out
    h2 qp[16];
    float qsum = 0.0f, qoff = 0.0f;       // sum(q), sum(offset(d) * q)
    {
        const __half *qv = q + ((int64_t)b * H + h) * D + 32 * c;
        uint4 qraw[4];                    // 64 bytes as four loads (32 two-byte loads cost a microsecond of prologue)
#pragma unroll
        for (int j = 0; j < 4; ++j) qraw[j] = *reinterpret_cast<const uint4 *>(qv + 8 * j);
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const float lo = half_of(qraw, 8 * j + kNib[k]), hi = half_of(qraw, 8 * j + kNib[k] + 4);
                qp[4 * j + k] = h2{(_Float16)lo, (_Float16)hi};
                qsum += lo + hi;
                qoff += kOff[k] * (lo + hi);
            }
    }

    unsigned c_zero = 0u;                 // a zero the compiler cannot see (sum_across_chunks)
    asm volatile("" : "+s"(c_zero));
    float acc[32];                        // acc[8j + 2k + half] <-> d = 32c + 8j + k + 4 half
#pragma unroll
    for (int i = 0; i < 32; ++i) acc[i] = 0.0f;
    float wsum = 0.0f, zacc = 0.0f;       // sums of w = p * v_scale and of w * v_zero since the last flush
    float m_run = -INFINITY, l_run = 0.0f;

    auto consume = [&](const Stage &s_, int tile, int slot) {
        // this token's scale and zero point sit in lane 16 * slot + tl
        const int src = (16 * slot + tl) << 2;
        const uint32_t km = (uint32_t)__builtin_amdgcn_ds_bpermute(src, (int)kmeta);
        const uint32_t vm = (uint32_t)__builtin_amdgcn_ds_bpermute(src, (int)vmeta);

        // ---- scores
        const uint32_t kw[4] = {s_.k.x, s_.k.y, s_.k.z, s_.k.w};
        float dot = 0.0f;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            uint32_t pr[4];
            unpack8(kw[j], pr);
#pragma unroll
            for (int k = 0; k < 4; ++k)
                dot = __builtin_amdgcn_fdot2(__builtin_bit_cast(h2, pr[k]), qp[4 * j + k], dot, false);
        }
        const float k_s = __half2float(__ushort_as_half((unsigned short)(km & 0xFFFFu)));
        const float k_z = (float)(int16_t)(km >> 16);
        const float part_ = sum_across_chunks(dot - fmaf(k_z, qsum, qoff), c_zero);
        const bool valid = tile * kTile + tl < T;
        const float score = valid ? part_ * (k_s * sm_scale) : -INFINITY;

        // ---- online softmax (every lane of the wavefront ends up with the same m and l)
        const float m_new = fmaxf(m_run, row16_max(score));
        if (m_new > m_run) {                              // rare after the first few steps
            const float alpha = __expf(m_run - m_new);    // 0 on the first step
            l_run *= alpha;
            wsum *= alpha;
            zacc *= alpha;
#pragma unroll
            for (int i = 0; i < 32; ++i) acc[i] *= alpha;
            m_run = m_new;
        }
        const float p = __expf(score - m_run);
        l_run += row16_sum(p);

        // ---- values: the fp16 halves go straight into mixed-precision fmas
        const float v_s = __half2float(__ushort_as_half((unsigned short)(vm & 0xFFFFu)));
        const float v_z = (float)(int16_t)(vm >> 16);
        const float wgt = p * v_s;
        wsum += wgt;
        zacc = fmaf(wgt, v_z, zacc);
        const uint32_t vw[4] = {s_.v.x, s_.v.y, s_.v.z, s_.v.w};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            uint32_t pr[4];
            unpack8_16(vw[j], pr);
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const h2 cv = __builtin_bit_cast(h2, pr[k]);
                acc[8 * j + 2 * k]     = fmaf(wgt, (float)cv[0], acc[8 * j + 2 * k]);
                acc[8 * j + 2 * k + 1] = fmaf(wgt, (float)cv[1], acc[8 * j + 2 * k + 1]);
            }
        }
    };

    if (alive) {
        while (G < g_end) {
            const int Gn = G + kWaves;                    // past the end: clamped, unused loads
            uint32_t nk, nv;
            fetch_meta(Gn, nk, nv);
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int tile = 4 * G + i;
                if (tile * kTile < T) consume(st[i], tile, i);
                fetch(st[i], 4 * Gn + i);                 // the slot's next use is four steps away
            }
            // the offsets of this group's four steps leave the accumulators now, not at the end:
            // left in, their sum grows with the sequence and its rounding would show in
            // outputs that are small against it
            const float off = fmaf(16.0f, wsum, zacc);
#pragma unroll
            for (int i = 0; i < 32; ++i) acc[i] -= off;
            wsum = 0.0f;
            zacc = 0.0f;
            kmeta = nk;
            vmeta = nv;
            G = Gn;
        }
    }

    // ---- the 16 tokens of the lanes meet; lane (0, c) then holds chunk c of this wavefront
#pragma unroll
    for (int i = 0; i < 32; ++i) acc[i] = row16_sum(acc[i]);
    if (tl == 0) {
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int k = 0; k < 4; ++k)
#pragma unroll
                for (int hf = 0; hf < 2; ++hf)
                    s_acc[wave][32 * c + 8 * j + k + 4 * hf] = acc[8 * j + 2 * k + hf];
    }
    if (lane == 0) {
        s_m[wave] = m_run;
        s_l[wave] = l_run;
    }
    __syncthreads();

    // ---- merge the wavefronts: out = sum_w e^(m_w - M) acc_w / sum_w e^(m_w - M) l_w
    if (tid < D) {
        float M = s_m[0];
#pragma unroll
        for (int w = 1; w < kWaves; ++w) M = fmaxf(M, s_m[w]);
        float num = 0.0f, den = 0.0f;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) {
            const float e = s_m[w] == -INFINITY ? 0.0f : __expf(s_m[w] - M);
            num += e * s_acc[w][tid];
            den += e * s_l[w];
        }
        if (part == nullptr) {
            out[((int64_t)b * H + h) * D + tid] = __float2half_rn(den > 0.0f ? num / den : 0.0f);
        } else {                                          // one partial (M, den, num[D]) per split
            float *dst = part + ((int64_t)blockIdx.x * gridDim.y + blockIdx.y) * (D + 2);
            dst[2 + tid] = num;
            if (tid == 0) {
                dst[0] = M;
                dst[1] = den;
            }
        }
    }
}

// ---------------------------------------------------------------- grouped-query variant

typedef _Float16 v8h __attribute__((ext_vector_type(8)));
typedef _Float16 v4h __attribute__((ext_vector_type(4)));
typedef float    v4f __attribute__((ext_vector_type(4)));
typedef unsigned v4u __attribute__((ext_vector_type(4)));
typedef unsigned v2u __attribute__((ext_vector_type(2)));

__device__ __forceinline__ v4h pair_operand(uint32_t lo, uint32_t hi)
{
    const v2u t = {lo, hi};
    return __builtin_bit_cast(v4h, t);
}

__device__ __forceinline__ v8h quad_operand(uint32_t a, uint32_t b, uint32_t c, uint32_t d)
{
    const v4u t = {a, b, c, d};
    return __builtin_bit_cast(v8h, t);
}

// unpack8_16 in plain C: these values feed MFMAs, and the wait states an MFMA needs after the
// instruction that wrote its operand are only inserted for instructions the compiler can see
// (mask and magic arrive in registers whose contents the compiler cannot see: with literal
// constants it emits an and and an or, with register operands the fused v_and_or_b32)
__device__ __forceinline__ void unpack8_16_mfma(uint32_t w, uint32_t mask, uint32_t magic, uint32_t (&pr)[4])
{
    pr[0] = ((w << 6) & mask) | magic;
    pr[1] = ((w << 2) & mask) | magic;
    pr[2] = ((w >> 2) & mask) | magic;
    pr[3] = ((w >> 6) & mask) | magic;
}

constexpr int kGqaWaves    = 4;
constexpr int kGqaMaxHeads = 16;          // query heads per cache head served by one MFMA column block
constexpr int kGqaHeadPitch = 4 * 33 + 1; // floats per head in the merge area (32 + 1 per chunk, + 1)

// One workgroup per (sequence, CACHE head) and split of the token range: the Gq = H / Hkv
// query heads that share a cache head (2 <= Gq <= 16) share every load and every unpacked
// code, and both contractions run on the fp16 MFMA 16x16x32 (lane l supplies row or column
// l & 15 and the eight k of chunk l >> 4; the result has column l & 15 in lane l and rows
// 4 (l >> 4) + e in register e).  A wavefront owns every fourth group of 64 tokens and walks
// it in four steps of 16 tokens, as in the per-head kernel.
//   scores  : S[t, h] = sum_d (16 + code[t, d]) q[h, d]: the row operand is the K codes as
//             fp16 16 + c (lane = token l & 15, 32 head dimensions of chunk l >> 4, four
//             MFMAs), the column operand q in the same order of d (registers, loaded once);
//             the result leaves head h = l & 15 and tokens 4 (l >> 4) + e in lane l, and
//             score = k_scale sm_scale (S - (16 + k_zero) sum_d q).
//   softmax : online per head; the four lanes of a head agree on the maximum, each keeps
//             the partial sums of its own tokens; accumulators are rescaled when the
//             maximum moves.
//   values  : out^T[d, h] = sum_t (16 + code[t, d]) w[t, h]: the weights are already laid
//             out as the column operand (tokens 4 (l >> 4) + i of head l & 15); the row
//             operand wants four TOKENS of one d per lane, so the V codes are loaded four
//             bytes per lane and token (lane = d group l & 15 of 8 head dimensions, tokens
//             4 (l >> 4) + i), transposed as bytes in registers and unpacked two tokens at a
//             time; tile j of the eight result tiles holds d = 8 (row) + j, so lane l ends
//             with d = 32 (l >> 4) + 8 e + j of head l & 15.
//             The weights must fit fp16 whatever the scales are:
//             w = p * v_scale * 2^15 / R, R the largest v_scale this wavefront has met so far
//             (fixed per group of 64 tokens; when a new group raises it, the accumulators are
//             rescaled, as for the running maximum of the scores): at most 2^15, and a normal
//             fp16 number down to 2^-29 of that.  One fp16 number per weight is not enough (its rounding alone shows
//             as 1e-2 of the small outputs of a head): w travels as fp16 hi + fp16 lo, one
//             16x16x16 MFMA for each against the same value operand.
//             The 16 and the zero point leave BEFORE the contraction: (16 + code) - (16 + zero)
//             is exact in fp16 (one packed subtraction per pair of codes), so the sums carry
//             no offset that a long context would have to cancel.  Zero points beyond +-1000
//             (rows whose values all sit far on one side of zero) are taken out up to that
//             bound, the rest leaves through sum_t w * rest as in the per-head kernel.
//   scales  : lane l reads the scale and zero point of token l of the group (one cache line
//             per array), turns them into four floats and parks them in LDS, where the step
//             reads the four tokens it needs as broadcast 16-byte reads.
__global__ __launch_bounds__(kGqaWaves * 64)               // (capped at 168 registers it spills and runs slower)
void decode_attention_kv4_gqa_kernel(const __half *__restrict__ q, int H, int Hkv, int64_t Tmax,
                                     const int32_t *__restrict__ seq_len,
                                     const uint8_t *__restrict__ kq, const __half *__restrict__ ks,
                                     const int16_t *__restrict__ kz, const uint8_t *__restrict__ vq,
                                     const __half *__restrict__ vs, const int16_t *__restrict__ vz,
                                     float sm_scale, __half *__restrict__ out, int groups_per_split,
                                     float *__restrict__ part)
{
    constexpr int D = 128;
    constexpr int kWaves = kGqaWaves;
    __shared__ float4 s_meta[kWaves][kTokens];
    __shared__ float  s_rest[kWaves][kTokens];
    __shared__ float  s_m[kWaves][kGqaMaxHeads], s_l[kWaves][kGqaMaxHeads];
    extern __shared__ __align__(16) float s_acc[];        // [kWaves][Gq][kGqaHeadPitch]

    const int Gq = H / Hkv;
    const int b = blockIdx.x / Hkv, kvh = blockIdx.x % Hkv;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int x = lane & 15, c = lane >> 4;
    int T = seq_len[b];
    T = T < 0 ? 0 : (T > Tmax ? (int)Tmax : T);
    const int64_t base = ((int64_t)b * Hkv + kvh) * Tmax;
    const uint8_t *kb = kq + base * (D / 2), *vb = vq + base * (D / 2);
    const __half  *ksb = ks + base, *vsb = vs + base;
    const int16_t *kzb = kz + base, *vzb = vz + base;

    const int g_first = blockIdx.y * groups_per_split;
    const int g_end   = min((T + kTokens - 1) / kTokens, g_first + groups_per_split);
    int  G     = g_first + wave;
    const bool alive = G < g_end;                        // then T >= 1: clamped addresses are valid
    const int  t_last = min(T, g_end * kTokens) - 1;     // loads never leave this split's tokens

    struct Stage { uint4 k; uint32_t v0, v1, v2, v3; };
    Stage st[4];
    const float k_mul = sm_scale * 1.44269504088896340736f;   // scores in units of log2: exp2 below
    // byte offsets inside this cache head: a tile is 16 rows of 64 bytes; rows past t_last
    // (masked tokens, steps past the end) read row t_last instead
    const uint32_t k_lane = 64u * x + 16u * c, k_last = 64u * (uint32_t)max(t_last, 0) + 16u * c;
    const uint32_t v_lane = 64u * (4u * c) + 4u * x, v_last = 64u * (uint32_t)max(t_last, 0) + 4u * x;
    auto fetch = [&](Stage &s_, int tile) {
        const uint32_t t0 = (uint32_t)tile * (kTile * 64u);
        s_.k  = *reinterpret_cast<const uint4 *>(kb + min(t0 + k_lane, k_last));
        s_.v0 = *reinterpret_cast<const uint32_t *>(vb + min(t0 + v_lane, v_last));
        s_.v1 = *reinterpret_cast<const uint32_t *>(vb + min(t0 + v_lane + 64u, v_last));
        s_.v2 = *reinterpret_cast<const uint32_t *>(vb + min(t0 + v_lane + 128u, v_last));
        s_.v3 = *reinterpret_cast<const uint32_t *>(vb + min(t0 + v_lane + 192u, v_last));
    };
    // scales and zero points of token `lane` of group g, raw
    struct Meta { __half ks, vs; int16_t kz, vz; };
    auto fetch_meta = [&](int g) {
        int t = g * kTokens + lane;
        t = t <= t_last ? t : t_last;
        return Meta{ksb[(uint32_t)t], vsb[(uint32_t)t], kzb[(uint32_t)t], vzb[(uint32_t)t]};
    };
    v4f acc[8];                           // acc[j][e] <-> out[head x][d = 32c + 8e + j], in units of R / 2^15
#pragma unroll
    for (int j = 0; j < 8; ++j) acc[j] = v4f{0.0f, 0.0f, 0.0f, 0.0f};
    float m_run = -INFINITY, l_run = 0.0f, off_run = 0.0f;    // l and off: this lane's tokens only
    float R = 0.0f;                       // largest v_scale met so far (the same in every lane)
    unsigned c_zero = 0u;
    asm volatile("" : "+s"(c_zero));
    bool  has_rest = false;               // some zero point of the current group was clamped
    // ... as (k_scale sm_scale log2 e, 16 + k_zero, v_scale * 2^15 / R, 16 + v_zero clamped to
    // +-1000) into LDS, what the clamp cut off beside it
    auto install_meta = [&](const Meta &mt) {
        const float v_s = __half2float(mt.vs);
        const float Rn  = fmaxf(R, max_across_chunks(row16_max(v_s), c_zero));
        if (Rn > R) {                     // the same decision in every lane; rare after the first groups
            const float down = R / Rn;    // 0 the first time
            off_run *= down;
#pragma unroll
            for (int j = 0; j < 8; ++j) acc[j] *= down;
            R = Rn;
        }
        const float rinv  = R > 0.0f ? 32768.0f / R : 0.0f;
        const float v_off = 16.0f + (float)mt.vz;
        const float v_cut = fminf(fmaxf(v_off, -1000.0f), 1000.0f);
        s_meta[wave][lane] = make_float4(__half2float(mt.ks) * k_mul, 16.0f + (float)mt.kz, v_s * rinv, v_cut);
        s_rest[wave][lane] = v_off - v_cut;
        has_rest = __ballot(v_off != v_cut) != 0;
    };
    if (alive) {                          // the first loads leave before q is read
        install_meta(fetch_meta(G));
#pragma unroll
        for (int i = 0; i < 4; ++i) fetch(st[i], 4 * G + i);
    }

    // q of head x as the column operand: MFMA j of a step contracts, for chunk c, the head
    // dimensions 32c + 8j + {0, 4, 1, 5, 2, 6, 3, 7} (the order unpack8_16 delivers)
    v8h qb[4];
    float qsum = 0.0f;
    {
        const bool live = x < Gq;
        const __half *qv = q + ((int64_t)b * H + (int64_t)kvh * Gq + (live ? x : 0)) * D + 32 * c;
        uint4 qraw[4];                    // 64 bytes as four loads
#pragma unroll
        for (int j = 0; j < 4; ++j) qraw[j] = *reinterpret_cast<const uint4 *>(qv + 8 * j);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            float e[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) e[i] = live ? half_of(qraw, 8 * j + (i >> 1) + 4 * (i & 1)) : 0.0f;
            qb[j] = v8h{(_Float16)e[0], (_Float16)e[1], (_Float16)e[2], (_Float16)e[3],
                        (_Float16)e[4], (_Float16)e[5], (_Float16)e[6], (_Float16)e[7]};
            qsum += ((e[0] + e[1]) + (e[2] + e[3])) + ((e[4] + e[5]) + (e[6] + e[7]));
        }
        qsum += __shfl_xor(qsum, 16, 64);
        qsum += __shfl_xor(qsum, 32, 64);
    }

    uint32_t c_mask = 0x03C003C0u, c_magic = 0x4C004C00u;
    asm volatile("" : "+s"(c_mask));
    asm volatile("" : "+v"(c_magic));

    // `masked_c`: the group holds the end of the sequence, some tokens of the step may lie beyond it
    auto consume = [&](const Stage &s_, int tile, int slot, auto masked_c) __attribute__((always_inline)) {
        // ---- scores
        const uint32_t kw[4] = {s_.k.x, s_.k.y, s_.k.z, s_.k.w};
        v4f sa = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            uint32_t pr[4];
            unpack8_16_mfma(kw[j], c_mask, c_magic, pr);
            sa = __builtin_amdgcn_mfma_f32_16x16x32_f16(quad_operand(pr[0], pr[1], pr[2], pr[3]), qb[j], sa, 0, 0, 0);
        }
        float4 mt[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) mt[e] = s_meta[wave][16 * slot + 4 * c + e];
        float sc[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) sc[e] = mt[e].x * fmaf(-mt[e].y, qsum, sa[e]);
        if constexpr (decltype(masked_c)::value) {
#pragma unroll
            for (int e = 0; e < 4; ++e)
                if (tile * kTile + 4 * c + e >= T) sc[e] = -INFINITY;
        }
        // ---- online softmax per head: the four lanes of a head take the same decisions
        float mx = fmaxf(fmaxf(sc[0], sc[1]), fmaxf(sc[2], sc[3]));
        const float m_new = fmaxf(m_run, max_across_chunks(mx, c_zero));
        if (m_new > m_run) {
            const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);   // 0 on the first step
            l_run *= alpha;
            off_run *= alpha;
#pragma unroll
            for (int j = 0; j < 8; ++j) acc[j] *= alpha;
            m_run = m_new;
        }
        // w = hi + lo: hi by the packed conversion (which truncates: any rounding will do, lo
        // takes what hi leaves), two tokens per instruction
        float w[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const float p = __builtin_amdgcn_exp2f(sc[e] - m_run);
            l_run += p;
            w[e] = p * mt[e].z;
        }
        const h2 hi01 = __builtin_bit_cast(h2, __builtin_amdgcn_cvt_pkrtz(w[0], w[1]));
        const h2 hi23 = __builtin_bit_cast(h2, __builtin_amdgcn_cvt_pkrtz(w[2], w[3]));
        const h2 lo01 = __builtin_bit_cast(h2, __builtin_amdgcn_cvt_pkrtz(w[0] - (float)hi01[0], w[1] - (float)hi01[1]));
        const h2 lo23 = __builtin_bit_cast(h2, __builtin_amdgcn_cvt_pkrtz(w[2] - (float)hi23[0], w[3] - (float)hi23[1]));
        if (has_rest) {                   // rare: the part of a zero point the operands cannot carry
            const float *rs = &s_rest[wave][16 * slot + 4 * c];   // (hi + lo is w to 2^-22)
#pragma unroll
            for (int e = 0; e < 4; ++e) off_run = fmaf(w[e], rs[e], off_run);
        }
        const v4h pb_hi = {hi01[0], hi01[1], hi23[0], hi23[1]}, pb_lo = {lo01[0], lo01[1], lo23[0], lo23[1]};
        // (16 + zero) of tokens (0, 1) and (2, 3) of this lane as fp16 pairs
        const h2 z01 = {(_Float16)mt[0].w, (_Float16)mt[1].w}, z23 = {(_Float16)mt[2].w, (_Float16)mt[3].w};

        // ---- values: byte transpose (token i of this lane = dword v_i), then two tokens per unpack
        const uint32_t w0 = s_.v0, w1 = s_.v1, w2 = s_.v2, w3 = s_.v3;
        // v_perm_b32 picks each result byte out of eight: 0-3 the second operand's, 4-7 the first's
        constexpr uint32_t kZipLo = 0x05010400u;          // [b.0 a.0 b.1 a.1] of perm(a, b)
        constexpr uint32_t kZipHi = 0x07030602u;          // [b.2 a.2 b.3 a.3]
        // L01 = [t0.b0 t1.b0 t0.b1 t1.b1], H01 = [t0.b2 t1.b2 t0.b3 t1.b3] (byte 0 first)
        const uint32_t L01 = __builtin_amdgcn_perm(w1, w0, kZipLo), H01 = __builtin_amdgcn_perm(w1, w0, kZipHi);
        const uint32_t L23 = __builtin_amdgcn_perm(w3, w2, kZipLo), H23 = __builtin_amdgcn_perm(w3, w2, kZipHi);
        // Y_b = [t0.b t2.b t1.b t3.b]: the codes of tokens 0 and 1 sit 16 bits apart, as do 2 and 3
        uint32_t Y[4];
        Y[0] = __builtin_amdgcn_perm(L23, L01, kZipLo);
        Y[1] = __builtin_amdgcn_perm(L23, L01, kZipHi);
        Y[2] = __builtin_amdgcn_perm(H23, H01, kZipLo);
        Y[3] = __builtin_amdgcn_perm(H23, H01, kZipHi);
#pragma unroll
        for (int bt = 0; bt < 4; ++bt) {
            uint32_t pr[4];               // (t0,t1).lo  (t0,t1).hi  (t2,t3).lo  (t2,t3).hi of byte bt
            unpack8_16_mfma(Y[bt], c_mask, c_magic, pr);
            const uint32_t e01 = __builtin_bit_cast(uint32_t, __builtin_bit_cast(h2, pr[0]) - z01);
            const uint32_t o01 = __builtin_bit_cast(uint32_t, __builtin_bit_cast(h2, pr[1]) - z01);
            const uint32_t e23 = __builtin_bit_cast(uint32_t, __builtin_bit_cast(h2, pr[2]) - z23);
            const uint32_t o23 = __builtin_bit_cast(uint32_t, __builtin_bit_cast(h2, pr[3]) - z23);
            const v4h ve = pair_operand(e01, e23), vo = pair_operand(o01, o23);     // even / odd d of byte bt
            acc[2 * bt]     = __builtin_amdgcn_mfma_f32_16x16x16f16(ve, pb_hi, acc[2 * bt], 0, 0, 0);
            acc[2 * bt]     = __builtin_amdgcn_mfma_f32_16x16x16f16(ve, pb_lo, acc[2 * bt], 0, 0, 0);
            acc[2 * bt + 1] = __builtin_amdgcn_mfma_f32_16x16x16f16(vo, pb_hi, acc[2 * bt + 1], 0, 0, 0);
            acc[2 * bt + 1] = __builtin_amdgcn_mfma_f32_16x16x16f16(vo, pb_lo, acc[2 * bt + 1], 0, 0, 0);
        }
    };

    if (alive) {
        while (G < g_end) {
            const int Gn = G + kWaves;                    // past the end: clamped, unused loads
            const Meta meta_next = fetch_meta(Gn);
            if ((G + 1) * kTokens <= T) {                 // every token of the group is inside the sequence
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    consume(st[i], 4 * G + i, i, std::false_type{});
                    fetch(st[i], 4 * Gn + i);             // the slot's next use is four steps away
                }
            } else {
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int tile = 4 * G + i;
                    if (tile * kTile < T) consume(st[i], tile, i, std::true_type{});
                    fetch(st[i], 4 * Gn + i);
                }
            }
            if (has_rest) {                               // what the operands could not carry of the zero points
                float off = off_run;
                off += __shfl_xor(off, 16, 64);
                off += __shfl_xor(off, 32, 64);
#pragma unroll
                for (int j = 0; j < 8; ++j) acc[j] -= off;
                off_run = 0.0f;
            }
            install_meta(meta_next);                      // every read of this group's entries is done
            G = Gn;
        }
    }

    // ---- the wavefronts merge through LDS: out = sum_w e^(m_w - M) acc_w / sum_w e^(m_w - M) l_w
    l_run += __shfl_xor(l_run, 16, 64);
    l_run += __shfl_xor(l_run, 32, 64);
    if (x < Gq) {
        float *dst = s_acc + ((size_t)wave * Gq + x) * kGqaHeadPitch + 33 * c;
#pragma unroll
        for (int j = 0; j < 8; ++j)
#pragma unroll
            for (int e = 0; e < 4; ++e) dst[8 * e + j] = acc[j][e] * (R * (1.0f / 32768.0f));
        if (c == 0) {
            s_m[wave][x] = m_run;
            s_l[wave][x] = l_run;
        }
    }
    __syncthreads();
    for (int idx = tid; idx < Gq * D; idx += kWaves * 64) {
        const int hh = idx >> 7, d = idx & (D - 1);
        float M = s_m[0][hh];
#pragma unroll
        for (int w = 1; w < kWaves; ++w) M = fmaxf(M, s_m[w][hh]);
        float num = 0.0f, den = 0.0f;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) {
            const float e = s_m[w][hh] == -INFINITY ? 0.0f : __builtin_amdgcn_exp2f(s_m[w][hh] - M);
            num += e * s_acc[((size_t)w * Gq + hh) * kGqaHeadPitch + 33 * (d >> 5) + (d & 31)];
            den += e * s_l[w][hh];
        }
        const int64_t head = (int64_t)b * H + (int64_t)kvh * Gq + hh;
        if (part == nullptr) {
            out[head * D + d] = __float2half_rn(den > 0.0f ? num / den : 0.0f);
        } else {                          // partials in natural-log units, as the merge kernel reads them
            float *dst = part + (head * gridDim.y + blockIdx.y) * (D + 2);
            dst[2 + d] = num;
            if (d == 0) {
                dst[0] = M * 0.69314718055994530942f;
                dst[1] = den;
            }
        }
    }
}

// Second pass of a split launch: the partials of one (sequence, head) merge as the
// wavefronts did, out = sum_s e^(M_s - M) num_s / sum_s e^(M_s - M) den_s.  At most 64 splits:
// lane s of the first wavefront takes split s, so the maxima are one load per lane and the
// weights e^(M_s - M) are computed once; then thread d sums its column over the splits with
// independent loads (a loop that waits for each split's maximum in turn costs the memory
// latency 2 S times).
__global__ __launch_bounds__(128)
void decode_attention_merge_kernel(const float *__restrict__ part, int S, __half *__restrict__ out)
{
    constexpr int D = 128;
    __shared__ float s_e[64];
    __shared__ float s_den;
    const float *src = part + (int64_t)blockIdx.x * S * (D + 2);
    const int tid = threadIdx.x;
    if (tid < 64) {
        const float ms = tid < S ? src[tid * (D + 2)] : -INFINITY;
        const float dn = tid < S ? src[tid * (D + 2) + 1] : 0.0f;
        float M = row16_max(ms);
        M = fmaxf(M, __shfl_xor(M, 16, 64));
        M = fmaxf(M, __shfl_xor(M, 32, 64));
        const float e = ms == -INFINITY ? 0.0f : __expf(ms - M);
        float den = row16_sum(e * dn);
        den += __shfl_xor(den, 16, 64);
        den += __shfl_xor(den, 32, 64);
        s_e[tid] = e;
        if (tid == 0) s_den = den;
    }
    __syncthreads();
    float num = 0.0f;
#pragma unroll 8
    for (int s = 0; s < S; ++s) num = fmaf(s_e[s], src[s * (D + 2) + 2 + tid], num);
    const float den = s_den;
    out[(int64_t)blockIdx.x * D + tid] = __float2half_rn(den > 0.0f ? num / den : 0.0f);
}

}  // namespace

namespace atom_internal {

hipError_t launch_kv_quantize(const void *x, int64_t R, int64_t ldx, int D, float clip,
                              const int32_t *pos, int32_t rows_per_seq, int64_t Tmax, void *q,
                              void *scale, void *zero, hipStream_t stream, const void *x2, void *q2,
                              void *scale2, void *zero2)
{
    const int     lpr  = D / 8;
    const bool    bulk = R >= 65536;                    // four rows per lane group
    const int64_t per  = (bulk ? 4 : 1) * (256 / lpr);  // rows per workgroup
    const int64_t grid = (R + per - 1) / per;
#define ATOM_KVQ_LAUNCH(LPR, ROWS)                                                                    \
    hipLaunchKernelGGL((kv_quantize_kernel<LPR, ROWS>), dim3((unsigned)grid, x2 ? 2 : 1), dim3(256),  \
                       0, stream, (const __half *)x, R, ldx, clip, pos, rows_per_seq, Tmax,           \
                       (uint8_t *)q, (__half *)scale, (int16_t *)zero, (const __half *)x2,            \
                       (uint8_t *)q2, (__half *)scale2, (int16_t *)zero2)
    if (D == 128) { if (bulk) ATOM_KVQ_LAUNCH(16, 4); else ATOM_KVQ_LAUNCH(16, 1); }
    else          { if (bulk) ATOM_KVQ_LAUNCH(8, 4);  else ATOM_KVQ_LAUNCH(8, 1); }
#undef ATOM_KVQ_LAUNCH
    return hipGetLastError();
}

// Shape of the launch.  B * H workgroups of four wavefronts fill the GPU from about five per
// compute unit; a grid of at most 384 workgroups first gets 16 wavefronts per workgroup (the token range is
// shared inside the workgroup, which merges through LDS: no second kernel), and below 256
// workgroups the token range is also split over several workgroups whose partials meet in
// decode_attention_merge_kernel.  Never less than one 64-token group per wavefront and split.
//
// With 2 to 16 query heads per cache head the grouped-query kernel runs instead: one workgroup of
// four wavefronts per (sequence, cache head), the token range split until about 512 workgroups
// exist.
struct AttentionShape { int waves, splits; bool gqa; };
AttentionShape decode_attention_shape(int B, int H, int Hkv, int64_t Tmax)
{
    const int64_t groups = (Tmax + kTokens - 1) / kTokens;
    const int     Gq     = H / Hkv;
    if (Gq >= 2 && Gq <= kGqaMaxHeads) {
        const int64_t bk = (int64_t)B * Hkv;
        // about 512 workgroups (two per CU, one round); measured against 768 to 4096: more splits only add
        // prologues, epilogues and merge work
        int64_t want = 512 / bk, cap = groups / kGqaWaves;    // no split from 257 workgroups on
        if (want > cap) want = cap;
        if (want > 64) want = 64;
        if (want < 1) want = 1;
        // every split a whole number of rounds of the four wavefronts
        const int64_t per = ((groups + want - 1) / want + kGqaWaves - 1) / kGqaWaves * kGqaWaves;
        return {kGqaWaves, (int)((groups + per - 1) / per), true};
    }
    const int64_t bh     = (int64_t)B * H;
    if (bh > 384 || groups < 16) {
        int64_t want = (1280 + bh - 1) / bh, cap = groups / 4;
        if (want > cap) want = cap;
        if (want > 64) want = 64;
        return {4, want < 1 ? 1 : (int)want, false};
    }
    int64_t want = (256 + bh - 1) / bh, cap = groups / 16;     // 256 x 16 wavefronts = four per SIMD
    if (want > cap) want = cap;
    if (want > 64) want = 64;
    return {16, want < 1 ? 1 : (int)want, false};
}

size_t decode_attention_workspace_bytes(int B, int H, int Hkv, int64_t Tmax)
{
    const int S = decode_attention_shape(B, H, Hkv, Tmax).splits;
    return S > 1 ? (size_t)B * H * S * (128 + 2) * sizeof(float) : 0;
}

hipError_t launch_decode_attention_kv4(const void *q, int B, int H, int Hkv, int64_t Tmax,
                                       const int32_t *seq_len, const void *kq, const void *ks,
                                       const void *kz, const void *vq, const void *vs,
                                       const void *vz, float sm_scale, void *out, void *workspace,
                                       hipStream_t stream)
{
    const AttentionShape sh = decode_attention_shape(B, H, Hkv, Tmax);
    const int S      = sh.splits;
    const int groups = (int)((Tmax + kTokens - 1) / kTokens);
    int tps = S > 1 ? (groups + S - 1) / S : (groups > 0 ? groups : 1);
    if (sh.gqa) tps = (tps + kGqaWaves - 1) / kGqaWaves * kGqaWaves;   // whole rounds of the wavefronts
    float *part = S > 1 ? (float *)workspace : nullptr;
    if (sh.gqa) {
        const size_t lds = (size_t)kGqaWaves * (H / Hkv) * kGqaHeadPitch * sizeof(float);   // <= 34 KB
        hipLaunchKernelGGL(decode_attention_kv4_gqa_kernel, dim3((unsigned)(B * Hkv), (unsigned)S),
                           dim3(kGqaWaves * 64), lds, stream, (const __half *)q, H, Hkv, Tmax, seq_len,
                           (const uint8_t *)kq, (const __half *)ks, (const int16_t *)kz, (const uint8_t *)vq,
                           (const __half *)vs, (const int16_t *)vz, sm_scale, (__half *)out, tps, part);
    } else if (sh.waves == 4)
        hipLaunchKernelGGL(decode_attention_kv4_kernel<4>, dim3((unsigned)(B * H), (unsigned)S), dim3(256),
                           0, stream, (const __half *)q, H, Hkv, Tmax, seq_len, (const uint8_t *)kq,
                           (const __half *)ks, (const int16_t *)kz, (const uint8_t *)vq,
                           (const __half *)vs, (const int16_t *)vz, sm_scale, (__half *)out, tps, part);
    else
        hipLaunchKernelGGL(decode_attention_kv4_kernel<16>, dim3((unsigned)(B * H), (unsigned)S),
                           dim3(1024), 0, stream, (const __half *)q, H, Hkv, Tmax, seq_len,
                           (const uint8_t *)kq, (const __half *)ks, (const int16_t *)kz,
                           (const uint8_t *)vq, (const __half *)vs, (const int16_t *)vz, sm_scale,
                           (__half *)out, tps, part);
    hipError_t err = hipGetLastError();
    if (err != hipSuccess || S == 1) return err;
    hipLaunchKernelGGL(decode_attention_merge_kernel, dim3((unsigned)(B * H)), dim3(128), 0, stream,
                       (const float *)part, S, (__half *)out);
    return hipGetLastError();
}

// Scratch for callers that cannot allocate: one array per GPU, in the library's own device
// image, held until the process ends.  Host code never passes the array's name to a kernel (there
// it is only a handle for the symbol): the device address is looked up once per device with that
// device current, and only that pointer is used afterwards.
namespace {
constexpr size_t kStaticScratchBytes = (size_t)4 << 20;
__device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
constexpr int kMaxDevices = 64;
std::atomic<void *> scratch_ptr[kMaxDevices];
}  // namespace

size_t static_scratch_bytes() { return kStaticScratchBytes; }

hipError_t static_scratch(void **ptr)
{
    int dev = -1;
    hipError_t err = hipGetDevice(&dev);
    if (err != hipSuccess) return err;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    void *p = scratch_ptr[dev].load(std::memory_order_acquire);
    if (!p) {
        err = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (err != hipSuccess) return err;
        if (!p) return hipErrorInvalidSymbol;
        scratch_ptr[dev].store(p, std::memory_order_release);
    }
    *ptr = p;
    return hipSuccess;
}

}  // namespace atom_internal
