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
#include <hip/hip_fp16.h>
#include <stdint.h>

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
#pragma unroll
    for (int d = 1; d < LPR; d <<= 1) {
        mx = fmaxf(mx, __shfl_xor(mx, d, 64));
        mn = fminf(mn, __shfl_xor(mn, d, 64));
    }
}

// One row of D = 8 * LPR values per LPR lanes, 64 / LPR rows per wavefront.
//   s = fp16(((max - min) * clip) / 15), z = clamp(rne(-min / s)), code = clamp(rne(x/s) + z, 0, 15)
// with IEEE fp32 divisions by the stored scale; a zero scale gives zero codes and z = 0.
// Output row index: r (pos == nullptr), or r * Tmax + pos[r / rows_per_seq] (append one
// token per sequence: row r = (sequence, head)); rows whose position is outside
// [0, Tmax) write nothing.
template <int LPR>
__global__ __launch_bounds__(256)
void kv_quantize_kernel(const __half *__restrict__ x, int64_t R, int64_t ldx, float clip,
                        const int32_t *__restrict__ pos, int32_t rows_per_seq, int64_t Tmax,
                        uint8_t *__restrict__ q, __half *__restrict__ scale,
                        int16_t *__restrict__ zero)
{
    constexpr int D = 8 * LPR;
    const int64_t r = ((int64_t)blockIdx.x * 256 + threadIdx.x) / LPR;
    const int     j = threadIdx.x % LPR;
    const bool live = r < R;
    const int64_t rr = live ? r : R - 1;                 // idle lanes repeat the last row
    const uint4 raw = *reinterpret_cast<const uint4 *>(x + rr * ldx + 8 * j);
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
        float zf = rintf(-mn / s);
        zf = fminf(fmaxf(zf, -32768.0f), 32767.0f);
        z = (int)zf;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            float t = rintf(f[i] / s);
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

constexpr int kWaves = 4;                 // wavefronts per workgroup, each walks every 4th tile
constexpr int kTile  = 16;                // tokens per wavefront step

// One workgroup per (sequence, query head), head dimension 128.  A wavefront step covers 16
// tokens: lane l holds token (l & 15) and the 32 head dimensions of chunk (l >> 4), i.e.
// 16 bytes of that token's K row and 16 bytes of its V row (a wavefront load is 1 KB of
// contiguous cache).
//   scores  : the codes become fp16 16 + c, two at a time: a code placed in mantissa bits
//             6..9 under the exponent of 16 (0x4C00) adds exactly c; they meet the matching
//             pairs of q in v_dot2_f32_f16 (fp32 accumulate); the 16 and the zero point
//             leave as (16 + z) * sum(q) per chunk (a small offset keeps the cancellation
//             in fp32 harmless); the four
//             chunks of a token are added across lanes; then * scale * sm_scale.
//   softmax : online, per wavefront (running max m and sum l).
//   values  : acc[d] += (p * v_scale) * code[d] per lane, the zero points as one running
//             sum of (p * v_scale) * z; the 16 tokens of the lanes meet once, at the end;
//             the four wavefronts merge through LDS.
// The next step's loads are issued before the current one is used.
__global__ __launch_bounds__(kWaves * 64)
void decode_attention_kv4_kernel(const __half *__restrict__ q, int H, int Hkv, int64_t Tmax,
                                 const int32_t *__restrict__ seq_len,
                                 const uint8_t *__restrict__ kq, const __half *__restrict__ ks,
                                 const int16_t *__restrict__ kz, const uint8_t *__restrict__ vq,
                                 const __half *__restrict__ vs, const int16_t *__restrict__ vz,
                                 float sm_scale, __half *__restrict__ out, int tiles_per_split,
                                 float *__restrict__ part)
{
    constexpr int D = 128;
    __shared__ float s_acc[kWaves][D];
    __shared__ float s_m[kWaves], s_l[kWaves];

    const int b = blockIdx.x / H, h = blockIdx.x % H;
    const int kvh = h / (H / Hkv);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int tl = lane & 15, c = lane >> 4;
    int T = seq_len[b];
    T = T < 0 ? 0 : (T > Tmax ? (int)Tmax : T);          // never read past the cache
    const int64_t base = ((int64_t)b * Hkv + kvh) * Tmax;

    // this lane's 32 query values as 16 pairs in the order the codes come out of a dword:
    // dword j holds d = 32c + 8j + 0..7; one masked shift picks nibbles (i, i + 4)
    h2 qp[16];
    float qsum = 0.0f;
    {
        const __half *qv = q + ((int64_t)b * H + h) * D + 32 * c;
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const __half a = qv[8 * j + i], bb = qv[8 * j + i + 4];
                qp[4 * j + i] = h2{(_Float16)__half2float(a), (_Float16)__half2float(bb)};
                qsum += __half2float(a) + __half2float(bb);
            }
    }

    float acc[32];
#pragma unroll
    for (int i = 0; i < 32; ++i) acc[i] = 0.0f;
    float zacc = 0.0f;                    // running sum of (p * v_scale) * v_zero
    float m_run = -INFINITY, l_run = 0.0f;

    // this workgroup's share of the steps (all of them when the grid has one split)
    const int tile0  = blockIdx.y * tiles_per_split;
    const int ntiles = min((T + kTile - 1) / kTile, tile0 + tiles_per_split);
    uint4 kraw, vraw;
    uint32_t kmeta, vmeta;                // scale bits | zero << 16
    auto fetch = [&](int tile) {
        int t = tile * kTile + tl;
        t = t < T ? t : T - 1;            // masked tokens repeat the last valid one
        const int64_t row = base + t;
        kraw = *reinterpret_cast<const uint4 *>(kq + row * (D / 2) + 16 * c);
        vraw = *reinterpret_cast<const uint4 *>(vq + row * (D / 2) + 16 * c);
        kmeta = (uint32_t)__half_as_ushort(ks[row]) | ((uint32_t)(uint16_t)kz[row] << 16);
        vmeta = (uint32_t)__half_as_ushort(vs[row]) | ((uint32_t)(uint16_t)vz[row] << 16);
    };
    if (tile0 + wave < ntiles) fetch(tile0 + wave);
    for (int tile = tile0 + wave; tile < ntiles; tile += kWaves) {
        const uint4 kc = kraw, vc = vraw;
        const uint32_t km = kmeta, vm = vmeta;
        if (tile + kWaves < ntiles) fetch(tile + kWaves);

        // ---- scores
        const uint32_t kw[4] = {kc.x, kc.y, kc.z, kc.w};
        float dot = 0.0f;
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                // nibbles (i, i + 4) moved to mantissa bits 6..9 of the two halves
                const uint32_t sh   = i < 2 ? kw[j] << (6 - 4 * i) : kw[j] >> (4 * i - 6);
                const uint32_t pair = (sh & 0x03C003C0u) | 0x4C004C00u;
                dot = __builtin_amdgcn_fdot2(__builtin_bit_cast(h2, pair), qp[4 * j + i], dot, false);
            }
        const float k_s = __half2float(__ushort_as_half((unsigned short)(km & 0xFFFFu)));
        const float k_z = (float)(int16_t)(km >> 16);
        float part = dot - (16.0f + k_z) * qsum;
        part += __shfl_xor(part, 16, 64);
        part += __shfl_xor(part, 32, 64);
        const bool valid = tile * kTile + tl < T;
        const float score = valid ? part * (k_s * sm_scale) : -INFINITY;

        // ---- online softmax (every lane of the wavefront ends up with the same m and l)
        const float m_new = fmaxf(m_run, row16_max(score));
        if (m_new > m_run) {                              // rare after the first few steps
            const float alpha = __expf(m_run - m_new);    // 0 on the first step
            l_run *= alpha;
            zacc *= alpha;
#pragma unroll
            for (int i = 0; i < 32; ++i) acc[i] *= alpha;
            m_run = m_new;
        }
        const float p = __expf(score - m_run);
        l_run += row16_sum(p);

        // ---- values
        const float v_s = __half2float(__ushort_as_half((unsigned short)(vm & 0xFFFFu)));
        const float v_z = (float)(int16_t)(vm >> 16);
        const float wgt = p * v_s;
        zacc = fmaf(wgt, v_z, zacc);
        const uint32_t vw[4] = {vc.x, vc.y, vc.z, vc.w};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const uint32_t lo = vw[j] & 0x0F0F0F0Fu, hi = (vw[j] >> 4) & 0x0F0F0F0Fu;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                // byte i of lo is code 2i, byte i of hi is code 2i + 1
                const float c0 = (float)((lo >> (8 * i)) & 0xFFu), c1 = (float)((hi >> (8 * i)) & 0xFFu);
                acc[8 * j + 2 * i]     = fmaf(wgt, c0, acc[8 * j + 2 * i]);
                acc[8 * j + 2 * i + 1] = fmaf(wgt, c1, acc[8 * j + 2 * i + 1]);
            }
        }
    }

    // ---- the 16 tokens of the lanes meet; lane (0, c) then holds chunk c of this wavefront
    zacc = row16_sum(zacc);
#pragma unroll
    for (int i = 0; i < 32; ++i) acc[i] = row16_sum(acc[i]) - zacc;
    if (tl == 0) {
#pragma unroll
        for (int i = 0; i < 32; ++i) s_acc[wave][32 * c + i] = acc[i];
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

// Second pass of a split launch: the partials of one (sequence, head) merge as the
// wavefronts did, out = sum_s e^(M_s - M) num_s / sum_s e^(M_s - M) den_s.
__global__ __launch_bounds__(128)
void decode_attention_merge_kernel(const float *__restrict__ part, int S, __half *__restrict__ out)
{
    constexpr int D = 128;
    const float *src = part + (int64_t)blockIdx.x * S * (D + 2);
    float M = -INFINITY;
    for (int s = 0; s < S; ++s) M = fmaxf(M, src[s * (D + 2)]);
    float num = 0.0f, den = 0.0f;
    for (int s = 0; s < S; ++s) {
        const float ms = src[s * (D + 2)];
        const float e  = ms == -INFINITY ? 0.0f : __expf(ms - M);
        num += e * src[s * (D + 2) + 2 + threadIdx.x];
        den += e * src[s * (D + 2) + 1];
    }
    out[(int64_t)blockIdx.x * D + threadIdx.x] = __float2half_rn(den > 0.0f ? num / den : 0.0f);
}

}  // namespace

namespace atom_internal {

hipError_t launch_kv_quantize(const void *x, int64_t R, int64_t ldx, int D, float clip,
                              const int32_t *pos, int32_t rows_per_seq, int64_t Tmax, void *q,
                              void *scale, void *zero, hipStream_t stream)
{
    const int     lpr  = D / 8;
    const int64_t grid = (R * lpr + 255) / 256;
    if (D == 128)
        hipLaunchKernelGGL(kv_quantize_kernel<16>, dim3((unsigned)grid), dim3(256), 0, stream,
                           (const __half *)x, R, ldx, clip, pos, rows_per_seq, Tmax, (uint8_t *)q,
                           (__half *)scale, (int16_t *)zero);
    else
        hipLaunchKernelGGL(kv_quantize_kernel<8>, dim3((unsigned)grid), dim3(256), 0, stream,
                           (const __half *)x, R, ldx, clip, pos, rows_per_seq, Tmax, (uint8_t *)q,
                           (__half *)scale, (int16_t *)zero);
    return hipGetLastError();
}

// Splits of the token range per (sequence, head): enough workgroups to keep about five per
// compute unit resident, never less than 16 steps (256 tokens) per split.
int decode_attention_splits(int B, int H, int64_t Tmax)
{
    const int64_t tiles = (Tmax + kTile - 1) / kTile;
    const int64_t bh    = (int64_t)B * H;
    int64_t want = (1280 + bh - 1) / bh;
    int64_t cap  = tiles / 16;
    if (want > cap) want = cap;
    if (want > 64) want = 64;
    return want < 1 ? 1 : (int)want;
}

size_t decode_attention_workspace_bytes(int B, int H, int64_t Tmax)
{
    const int S = decode_attention_splits(B, H, Tmax);
    return S > 1 ? (size_t)B * H * S * (128 + 2) * sizeof(float) : 0;
}

hipError_t launch_decode_attention_kv4(const void *q, int B, int H, int Hkv, int64_t Tmax,
                                       const int32_t *seq_len, const void *kq, const void *ks,
                                       const void *kz, const void *vq, const void *vs,
                                       const void *vz, float sm_scale, void *out, void *workspace,
                                       hipStream_t stream)
{
    const int S     = decode_attention_splits(B, H, Tmax);
    const int tiles = (int)((Tmax + kTile - 1) / kTile);
    const int tps   = S > 1 ? (tiles + S - 1) / S : (tiles > 0 ? tiles : 1);
    float *part = S > 1 ? (float *)workspace : nullptr;
    hipLaunchKernelGGL(decode_attention_kv4_kernel, dim3((unsigned)(B * H), (unsigned)S),
                       dim3(kWaves * 64), 0, stream, (const __half *)q, H, Hkv, Tmax, seq_len,
                       (const uint8_t *)kq, (const __half *)ks, (const int16_t *)kz,
                       (const uint8_t *)vq, (const __half *)vs, (const int16_t *)vz, sm_scale,
                       (__half *)out, tps, part);
    hipError_t err = hipGetLastError();
    if (err != hipSuccess || S == 1) return err;
    hipLaunchKernelGGL(decode_attention_merge_kernel, dim3((unsigned)(B * H)), dim3(128), 0, stream,
                       (const float *)part, S, (__half *)out);
    return hipGetLastError();
}

}  // namespace atom_internal
