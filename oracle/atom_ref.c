/*
 * atom_ref.c -- CPU oracle for the Atom W4A4 hot path (arxiv 2310.19102).
 *
 * TEST INFRASTRUCTURE ONLY: plain single-threaded C, host pointers, no
 * intrinsics, no blocking, no fusion.  The product never calls this file.
 * Build with:  gcc -O2 -ffp-contract=off -shared -fPIC atom_ref.c -lm
 * (-ffp-contract=off keeps every fp32 multiply and add separately rounded;
 * the only fused multiply-add is the explicit fmaf in the GEMM epilogue).
 */
#include "atom_ref.h"

#include <math.h>
#include <stdlib.h>
#include <string.h>

/* ---------------------------------------------------------------- fp16 -- */

float atom_ref_f16_to_f32(uint16_t h)
{
    uint32_t sign = (uint32_t)(h >> 15) << 31;
    int32_t  e    = (h >> 10) & 0x1f;
    uint32_t m    = h & 0x3ffu;
    uint32_t bits;
    if (e == 0) {
        if (m == 0) {
            bits = sign;                          /* signed zero */
        } else {                                  /* subnormal: m * 2^-24 */
            int shift = 0;
            while ((m & 0x400u) == 0) { m <<= 1; ++shift; }
            m &= 0x3ffu;
            bits = sign | ((uint32_t)(127 - 15 - shift + 1) << 23) | (m << 13);
        }
    } else if (e == 31) {
        bits = sign | 0x7f800000u | (m << 13);    /* inf / nan */
    } else {
        bits = sign | ((uint32_t)(e - 15 + 127) << 23) | (m << 13);
    }
    float f;
    memcpy(&f, &bits, sizeof f);
    return f;
}

uint16_t atom_ref_f32_to_f16(float f)
{
    uint32_t bits;
    memcpy(&bits, &f, sizeof bits);
    uint16_t sign = (uint16_t)((bits >> 16) & 0x8000u);
    uint32_t a = bits & 0x7fffffffu;              /* |f| */
    if (a >= 0x7f800000u)                         /* inf or nan */
        return (uint16_t)(sign | 0x7c00u | ((a > 0x7f800000u) ? 0x200u : 0u));
    if (a >= 0x477ff000u)                         /* >= 65520 rounds to inf */
        return (uint16_t)(sign | 0x7c00u);
    if (a < 0x33000000u)                          /* < 2^-25 rounds to zero */
        return sign;
    int32_t  e = (int32_t)(a >> 23) - 127;        /* unbiased exponent */
    uint32_t m = (a & 0x7fffffu) | 0x800000u;     /* 24-bit significand */
    int drop;                                     /* low bits to discard */
    uint32_t base;
    if (e >= -14) { drop = 13;           base = (uint32_t)(e + 15 - 1) << 10; }
    else          { drop = 13 + (-14 - e); base = 0; }
    /* keep (24 - drop) bits; for normals the kept leading 1 adds to base */
    uint32_t kept = m >> drop;
    uint32_t rem  = m & ((1u << drop) - 1u);
    uint32_t half = 1u << (drop - 1);
    if (rem > half || (rem == half && (kept & 1u))) ++kept;
    return (uint16_t)(sign | (base + kept));      /* carries roll exponents */
}

/* fp32 -> fp16 for group scales: finite inputs, overflow saturates at the
 * largest finite fp16 (65504) instead of becoming infinity. */
static uint16_t scale_to_f16(float s32)
{
    uint16_t h = atom_ref_f32_to_f16(s32);
    if ((h & 0x7fffu) >= 0x7c00u) h = (uint16_t)((h & 0x8000u) | 0x7bffu);
    return h;
}

/* ------------------------------------------------------------- RMSNorm -- */

float atom_ref_sumsq(const uint16_t *x, int32_t K)
{
    float L[64];
    for (int l = 0; l < 64; ++l) L[l] = 0.0f;
    int32_t V = (K + 7) / 8;
    for (int32_t v = 0; v < V; ++v) {
        float sq[8];
        for (int i = 0; i < 8; ++i) {
            int32_t k = 8 * v + i;
            float xf = (k < K) ? atom_ref_f16_to_f32(x[k]) : 0.0f;
            sq[i] = xf * xf;                      /* exact: 11-bit x 11-bit */
        }
        float q = ((sq[0] + sq[1]) + (sq[2] + sq[3])) +
                  ((sq[4] + sq[5]) + (sq[6] + sq[7]));
        L[v % 64] = L[v % 64] + q;
    }
    for (int d = 1; d < 64; d *= 2)
        for (int l = 0; l + d < 64; l += 2 * d)
            L[l] = L[l] + L[l + d];
    return L[0];
}

void atom_ref_rmsnorm_row(const uint16_t *x, const uint16_t *gamma, float eps,
                          int32_t K, float *y)
{
    if (gamma == NULL) {
        for (int32_t k = 0; k < K; ++k) y[k] = atom_ref_f16_to_f32(x[k]);
        return;
    }
    float S    = atom_ref_sumsq(x, K);
    float mean = S / (float)K;
    float r    = 1.0f / sqrtf(mean + eps);
    for (int32_t k = 0; k < K; ++k) {
        float xf = atom_ref_f16_to_f32(x[k]);
        float t  = xf * r;
        y[k] = t * atom_ref_f16_to_f32(gamma[k]);
    }
}

/* ------------------------------------------------- group quantisation -- */

static int shapes_ok(int32_t K, int32_t Gs, int32_t O)
{
    if (K <= 0 || Gs <= 0 || O < 0) return 0;
    if (Gs % 2) return 0;                         /* two INT4 per byte */
    if (K % Gs || O % Gs || O >= K) return 0;
    return 1;
}

/* Quantise one row whose fp32 values y[] are in ORIGINAL channel order.
 * `bits` is the width n of the normal channels (4, or 3 for the W3A3 runs of
 * the accuracy evaluation, Section 5.2); the codes of either width travel in
 * 4-bit containers, sign-extended.  The outlier channels stay at 8 bits. */
static void quantize_row(const float *y, const int32_t *idx, int32_t K,
                         int32_t Gs, int32_t O, int32_t bits, float clip, uint8_t *q4,
                         int8_t *q8, uint16_t *scale)
{
    int32_t K4 = K - O, G = K / Gs, G4 = K4 / Gs;
    for (int32_t g = 0; g < G; ++g) {
        int   n    = (g < G4) ? bits : 8;         /* bit-width of the group */
        int   qmin = -(1 << (n - 1)), qmax = (1 << (n - 1)) - 1;
        float amax = 0.0f;
        for (int32_t t = 0; t < Gs; ++t) {
            float a = fabsf(y[idx[g * Gs + t]]);
            if (a > amax) amax = a;
        }
        float s32 = ((2.0f * amax) * clip) / (float)((1 << n) - 1);
        uint16_t sh = scale_to_f16(s32);
        float s = atom_ref_f16_to_f32(sh);
        scale[g] = sh;
        for (int32_t t = 0; t < Gs; ++t) {
            int32_t j = g * Gs + t;
            int q = 0;
            if (s != 0.0f) {
                float v = nearbyintf(y[idx[j]] / s);   /* ties to even */
                if (v < (float)qmin) v = (float)qmin;
                if (v > (float)qmax) v = (float)qmax;
                q = (int)v;
            }
            if (g < G4) {
                uint8_t nib = (uint8_t)(q & 0xf);
                if (j % 2 == 0) q4[j / 2] = nib;
                else            q4[j / 2] = (uint8_t)(q4[j / 2] | (nib << 4));
            } else {
                q8[j - K4] = (int8_t)q;
            }
        }
    }
}

int atom_ref_quantize_act(const uint16_t *x, int64_t M, int64_t ldx,
                          const uint16_t *gamma, float eps, const int32_t *idx,
                          int32_t K, int32_t Gs, int32_t O, float clip,
                          uint8_t *q4, int8_t *q8, uint16_t *scale)
{
    return atom_ref_quantize_act_n(x, M, ldx, gamma, eps, idx, K, Gs, O, 4, clip, q4, q8, scale);
}

int atom_ref_quantize_act_n(const uint16_t *x, int64_t M, int64_t ldx,
                            const uint16_t *gamma, float eps, const int32_t *idx,
                            int32_t K, int32_t Gs, int32_t O, int32_t bits, float clip,
                            uint8_t *q4, int8_t *q8, uint16_t *scale)
{
    if (!shapes_ok(K, Gs, O) || ldx < K || M < 0 || (bits != 3 && bits != 4)) return -1;
    int32_t K4 = K - O, G = K / Gs;
    float *y = (float *)malloc(sizeof(float) * (size_t)K);
    if (!y) return -1;
    for (int64_t m = 0; m < M; ++m) {
        atom_ref_rmsnorm_row(x + m * ldx, gamma, eps, K, y);
        quantize_row(y, idx, K, Gs, O, bits, clip, q4 + m * (K4 / 2), q8 + m * O,
                     scale + m * G);
    }
    free(y);
    return 0;
}

/* Residual add fused in front of the front end: h = fp16(x + res), the sum of
 * the two fp16 values formed in fp32 and rounded once to fp16 (when the fp32
 * sum is inexact the addends are more than 2^13 apart, which is nowhere near
 * an fp16 rounding tie, so this is the correctly rounded fp16 sum). */
int atom_ref_add_quantize_act(const uint16_t *x, const uint16_t *res, int64_t M,
                              int64_t ldx, int64_t ldr, uint16_t *sum_out,
                              int64_t ldo, const uint16_t *gamma, float eps,
                              const int32_t *idx, int32_t K, int32_t Gs,
                              int32_t O, float clip, uint8_t *q4, int8_t *q8,
                              uint16_t *scale)
{
    return atom_ref_add_quantize_act_n(x, res, M, ldx, ldr, sum_out, ldo, gamma, eps, idx, K, Gs, O,
                                       4, clip, q4, q8, scale);
}

int atom_ref_add_quantize_act_n(const uint16_t *x, const uint16_t *res, int64_t M,
                                int64_t ldx, int64_t ldr, uint16_t *sum_out,
                                int64_t ldo, const uint16_t *gamma, float eps,
                                const int32_t *idx, int32_t K, int32_t Gs,
                                int32_t O, int32_t bits, float clip, uint8_t *q4, int8_t *q8,
                                uint16_t *scale)
{
    if (!shapes_ok(K, Gs, O) || ldx < K || ldr < K || ldo < K || M < 0 || (bits != 3 && bits != 4)) return -1;
    int32_t K4 = K - O, G = K / Gs;
    float    *y = (float *)malloc(sizeof(float) * (size_t)K);
    uint16_t *h = (uint16_t *)malloc(sizeof(uint16_t) * (size_t)K);
    if (!y || !h) { free(y); free(h); return -1; }
    for (int64_t m = 0; m < M; ++m) {
        for (int32_t k = 0; k < K; ++k) {
            float a = atom_ref_f16_to_f32(x[m * ldx + k]);
            float b = atom_ref_f16_to_f32(res[m * ldr + k]);
            h[k] = atom_ref_f32_to_f16(a + b);
        }
        for (int32_t k = 0; k < K; ++k) sum_out[m * ldo + k] = h[k];
        atom_ref_rmsnorm_row(h, gamma, eps, K, y);
        quantize_row(y, idx, K, Gs, O, bits, clip, q4 + m * (K4 / 2), q8 + m * O,
                     scale + m * G);
    }
    free(y);
    free(h);
    return 0;
}

/* ------------------------------------------------------- SwiGLU in front -- */

/* exp(x) for x in [-87, 87], from IEEE operations only, so that it has one
 * value on every machine: n = round(x*log2(e)); r = x - n*ln2 with ln2 split
 * in two (the first part has 12 trailing zero bits, so n*ln2_hi is exact);
 * e^r by its Taylor polynomial of degree 7 in Horner form with fused
 * multiply-adds (|r| <= 0.347: truncation 1.3e-8 relative); the result is
 * scaled by 2^n through the exponent field (n in [-126, 126]). */
float atom_ref_expf(float x)
{
    if (x < -87.0f) x = -87.0f;
    if (x > 87.0f) x = 87.0f;
    float n = nearbyintf(x * 1.44269502162933349609375f);
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
    union { uint32_t u; float f; } two_n;
    two_n.u = (uint32_t)((int32_t)n + 127) << 23;
    return p * two_n.f;
}

/* silu(g) * u in fp32: sigma = 1 / (1 + exp(-g)) with the exp above and an
 * IEEE division, then (g * sigma) * u, two fp32 multiplies in this order. */
float atom_ref_silu_mul(uint16_t gate_f16, uint16_t up_f16)
{
    float g = atom_ref_f16_to_f32(gate_f16), u = atom_ref_f16_to_f32(up_f16);
    float e = atom_ref_expf(-g);
    float sigma = 1.0f / (1.0f + e);
    return (g * sigma) * u;
}

int atom_ref_swiglu_quantize_act(const uint16_t *gate, const uint16_t *up,
                                 int64_t M, int64_t ldg, int64_t ldu,
                                 const int32_t *idx, int32_t K, int32_t Gs,
                                 int32_t O, float clip, uint8_t *q4, int8_t *q8,
                                 uint16_t *scale)
{
    return atom_ref_swiglu_quantize_act_n(gate, up, M, ldg, ldu, idx, K, Gs, O, 4, clip, q4, q8, scale);
}

int atom_ref_swiglu_quantize_act_n(const uint16_t *gate, const uint16_t *up,
                                   int64_t M, int64_t ldg, int64_t ldu,
                                   const int32_t *idx, int32_t K, int32_t Gs,
                                   int32_t O, int32_t bits, float clip, uint8_t *q4, int8_t *q8,
                                   uint16_t *scale)
{
    if (!shapes_ok(K, Gs, O) || ldg < K || ldu < K || M < 0 || (bits != 3 && bits != 4)) return -1;
    int32_t K4 = K - O, G = K / Gs;
    float *y = (float *)malloc(sizeof(float) * (size_t)K);
    if (!y) return -1;
    for (int64_t m = 0; m < M; ++m) {
        for (int32_t k = 0; k < K; ++k)
            y[k] = atom_ref_silu_mul(gate[m * ldg + k], up[m * ldu + k]);
        quantize_row(y, idx, K, Gs, O, bits, clip, q4 + m * (K4 / 2), q8 + m * O,
                     scale + m * G);
    }
    free(y);
    return 0;
}

int atom_ref_quantize_weight(const uint16_t *w, int64_t N, int64_t ldw,
                             const int32_t *idx, int32_t K, int32_t Gs,
                             int32_t O, float clip, uint8_t *q4, int8_t *q8,
                             uint16_t *scale)
{
    return atom_ref_quantize_act(w, N, ldw, NULL, 0.0f, idx, K, Gs, O, clip,
                                 q4, q8, scale);
}

/* ----------------------------------------------------------------- GEMM -- */

/* Codes of one operand as int8 [rows, K]: sign-extended nibbles, then the
 * INT8 block, i.e. the reordered channel order j = 0..K-1. */
static int8_t *unpack_codes(const uint8_t *q4, const int8_t *q8, int64_t rows,
                            int32_t K, int32_t O)
{
    int32_t K4 = K - O;
    int8_t *c = (int8_t *)malloc((size_t)rows * (size_t)K + 1);
    if (!c) return NULL;
    for (int64_t r = 0; r < rows; ++r) {
        for (int32_t j = 0; j < K4; ++j) {
            uint8_t b   = q4[r * (K4 / 2) + j / 2];
            int     nib = (j % 2 == 0) ? (b & 0xf) : (b >> 4);
            c[r * K + j] = (int8_t)((nib >= 8) ? nib - 16 : nib);
        }
        for (int32_t j = K4; j < K; ++j) c[r * K + j] = q8[r * O + (j - K4)];
    }
    return c;
}

int atom_ref_w4a4_gemm(const uint8_t *a_q4, const int8_t *a_q8,
                       const uint16_t *a_scale, int64_t M,
                       const uint8_t *w_q4, const int8_t *w_q8,
                       const uint16_t *w_scale, int64_t N, int32_t K,
                       int32_t Gs, int32_t O, uint16_t *y, int64_t ldy,
                       int32_t *partials, float *acc_f32)
{
    if (!shapes_ok(K, Gs, O) || ldy < N || M < 0 || N < 0) return -1;
    int32_t G = K / Gs;
    int8_t *a = unpack_codes(a_q4, a_q8, M, K, O);
    int8_t *w = unpack_codes(w_q4, w_q8, N, K, O);
    if (!a || !w) { free(a); free(w); return -1; }
    for (int64_t m = 0; m < M; ++m) {
        for (int64_t n = 0; n < N; ++n) {
            float acc = 0.0f;
            for (int32_t g = 0; g < G; ++g) {
                const int8_t *ar = a + m * K + g * Gs;
                const int8_t *wr = w + n * K + g * Gs;
                int32_t P = 0;                              /* step 1 */
                for (int32_t t = 0; t < Gs; ++t)
                    P += (int32_t)ar[t] * (int32_t)wr[t];
                float ss = atom_ref_f16_to_f32(a_scale[m * G + g]) *
                           atom_ref_f16_to_f32(w_scale[n * G + g]);
                acc = fmaf((float)P, ss, acc);              /* steps 2, 3 */
                if (partials) partials[(m * N + n) * G + g] = P;
            }
            if (acc_f32) acc_f32[m * N + n] = acc;
            y[m * ldy + n] = atom_ref_f32_to_f16(acc);
        }
    }
    free(a);
    free(w);
    return 0;
}

/* ------------------------------------------------------------- KV cache -- */

int atom_ref_kv_quantize(const uint16_t *x, int64_t R, int64_t ldx, int32_t D,
                         float clip, uint8_t *q, uint16_t *scale, int16_t *zero)
{
    if (D <= 0 || D % 2 || ldx < D || R < 0) return -1;
    for (int64_t r = 0; r < R; ++r) {
        const uint16_t *row = x + r * ldx;
        float mx = atom_ref_f16_to_f32(row[0]), mn = mx;
        for (int32_t d = 1; d < D; ++d) {
            float v = atom_ref_f16_to_f32(row[d]);
            if (v > mx) mx = v;
            if (v < mn) mn = v;
        }
        float    s32 = ((mx - mn) * clip) / 15.0f;
        uint16_t sh  = scale_to_f16(s32);
        float    s   = atom_ref_f16_to_f32(sh);
        int32_t  z   = 0;
        if (s != 0.0f) {
            float zf = nearbyintf(-mn / s);
            if (zf < -32768.0f) zf = -32768.0f;
            if (zf > 32767.0f) zf = 32767.0f;
            z = (int32_t)zf;
        }
        scale[r] = sh;
        zero[r]  = (int16_t)z;
        for (int32_t d = 0; d < D; d += 2) {
            int c[2];
            for (int k = 0; k < 2; ++k) {
                int code = 0;
                if (s != 0.0f) {
                    /* round(x/s) is an integer below 2^24 in magnitude whenever it
                     * matters; clamp it first so that the integer sum cannot overflow */
                    float t = nearbyintf(atom_ref_f16_to_f32(row[d + k]) / s);
                    if (t < -100000.0f) t = -100000.0f;
                    if (t > 100000.0f) t = 100000.0f;
                    code = (int)t + z;
                    if (code < 0) code = 0;
                    if (code > 15) code = 15;
                }
                c[k] = code;
            }
            q[r * (D / 2) + d / 2] = (uint8_t)(c[0] | (c[1] << 4));
        }
    }
    return 0;
}

float atom_ref_kv_dequant(uint8_t code, uint16_t scale_f16, int16_t zero)
{
    return (float)((int)code - (int)zero) * atom_ref_f16_to_f32(scale_f16);
}

int atom_ref_decode_attention_kv4(const uint16_t *q, int32_t B, int32_t H,
                                  int32_t Hkv, int32_t D, int32_t Tmax,
                                  const int32_t *seq_len, const uint8_t *kq,
                                  const uint16_t *ks, const int16_t *kz,
                                  const uint8_t *vq, const uint16_t *vs,
                                  const int16_t *vz, float sm_scale,
                                  uint16_t *out)
{
    if (B < 0 || H <= 0 || Hkv <= 0 || H % Hkv || D <= 0 || D % 2 || Tmax < 0) return -1;
    double *score = (double *)malloc(sizeof(double) * (size_t)(Tmax > 0 ? Tmax : 1));
    double *acc   = (double *)malloc(sizeof(double) * (size_t)D);
    if (!score || !acc) { free(score); free(acc); return -1; }
    for (int32_t b = 0; b < B; ++b) {
        int32_t T = seq_len[b];
        if (T < 0 || T > Tmax) { free(score); free(acc); return -1; }
        for (int32_t h = 0; h < H; ++h) {
            const int32_t   kvh  = h / (H / Hkv);
            const int64_t   base = ((int64_t)b * Hkv + kvh) * Tmax;
            const uint16_t *qv   = q + ((int64_t)b * H + h) * D;
            uint16_t       *o    = out + ((int64_t)b * H + h) * D;
            double m = 0.0;
            for (int32_t t = 0; t < T; ++t) {
                double dot = 0.0;
                for (int32_t d = 0; d < D; ++d) {
                    uint8_t byte = kq[(base + t) * (D / 2) + d / 2];
                    uint8_t code = (d % 2 == 0) ? (byte & 0xf) : (byte >> 4);
                    dot += (double)atom_ref_f16_to_f32(qv[d]) *
                           (double)atom_ref_kv_dequant(code, ks[base + t], kz[base + t]);
                }
                score[t] = dot * (double)sm_scale;
                if (t == 0 || score[t] > m) m = score[t];
            }
            double l = 0.0;
            for (int32_t d = 0; d < D; ++d) acc[d] = 0.0;
            for (int32_t t = 0; t < T; ++t) {
                double p = exp(score[t] - m);
                l += p;
                for (int32_t d = 0; d < D; ++d) {
                    uint8_t byte = vq[(base + t) * (D / 2) + d / 2];
                    uint8_t code = (d % 2 == 0) ? (byte & 0xf) : (byte >> 4);
                    acc[d] += p * (double)atom_ref_kv_dequant(code, vs[base + t], vz[base + t]);
                }
            }
            for (int32_t d = 0; d < D; ++d)
                o[d] = atom_ref_f32_to_f16(T > 0 ? (float)(acc[d] / l) : 0.0f);
        }
    }
    free(score);
    free(acc);
    return 0;
}

/* ------------------------------------------- MX (microscaling) variant -- */
/* Section 5.2 / 6 of the paper evaluates the same recipe with FP4 codes and
 * names the MX formats, whose group scaling new hardware applies by itself.
 * Formats as the MX specification the paper cites defines them: a block of 32
 * elements shares one E8M0 scale 2^(byte - 127); the elements are FP4 E2M1
 * (normal channels) or FP8 E4M3 (outlier channels). */

static const float kE2M1[8] = {0.0f, 0.5f, 1.0f, 1.5f, 2.0f, 3.0f, 4.0f, 6.0f};

float atom_ref_e2m1_to_f32(uint8_t code)
{
    float v = kE2M1[code & 7];
    return (code & 8) ? -v : v;
}

float atom_ref_e4m3_to_f32(uint8_t code)
{
    int   s = code >> 7, e = (code >> 3) & 15, m = code & 7;
    float v;
    if (e == 15 && m == 7) return NAN;               /* the format has no infinity */
    if (e == 0) v = ldexpf((float)m, -9);            /* subnormal: m/8 * 2^-6 */
    else        v = ldexpf(1.0f + (float)m / 8.0f, e - 7);
    return s ? -v : v;
}

/* Nearest representable magnitude among codes 0..last, ties to the even code
 * (= even mantissa), magnitudes beyond the largest one saturate to it. */
static uint8_t nearest_code(float a, int last, float (*decode)(uint8_t))
{
    int best = 0;
    double bestd = fabs((double)a - (double)decode(0));
    for (int c = 1; c <= last; ++c) {
        double d = fabs((double)a - (double)decode((uint8_t)c));
        if (d < bestd || (d == bestd && (c % 2 == 0))) { best = c; bestd = d; }
    }
    return (uint8_t)best;
}

uint8_t atom_ref_f32_to_e2m1(float v)
{
    uint8_t c = nearest_code(fabsf(v), 7, atom_ref_e2m1_to_f32);
    return (uint8_t)(c | (signbit(v) ? 8 : 0));
}

uint8_t atom_ref_f32_to_e4m3(float v)
{
    uint8_t c = nearest_code(fabsf(v), 0x7e, atom_ref_e4m3_to_f32);
    return (uint8_t)(c | (signbit(v) ? 0x80 : 0));
}

/* E8M0 byte of a block whose clipped absolute maximum is a: the exponent of
 * the largest power of two not above a, minus the element format's largest
 * exponent emax (2 for E2M1, 8 for E4M3), clamped to [-127, 127]. */
uint8_t atom_ref_mx_scale_byte(float a, int emax)
{
    if (!(a > 0.0f)) return 0;
    int e;
    (void)frexpf(a, &e);                             /* a = f * 2^e, f in [0.5, 1) */
    int E = (e - 1) - emax;
    if (E < -127) E = -127;
    if (E > 127) E = 127;
    return (uint8_t)(E + 127);
}

/* One row, fp32 values y[] in ORIGINAL channel order. */
static void mx_quantize_row(const float *y, const int32_t *idx, int32_t K, int32_t O,
                            float clip, uint8_t *q4, uint8_t *q8, uint8_t *e8)
{
    int32_t K4 = K - O;
    for (int32_t b = 0; b < K / 32; ++b) {
        int   fp4  = (b * 32 < K4);
        float amax = 0.0f;
        for (int32_t t = 0; t < 32; ++t) {
            float a = fabsf(y[idx[b * 32 + t]]);
            if (a > amax) amax = a;
        }
        uint8_t byte = atom_ref_mx_scale_byte(amax * clip, fp4 ? 2 : 8);
        e8[b] = byte;
        for (int32_t t = 0; t < 32; ++t) {
            int32_t j = b * 32 + t;
            float   v = ldexpf(y[idx[j]], 127 - (int)byte);   /* y / 2^(byte-127), exact */
            if (fp4) {
                uint8_t c = atom_ref_f32_to_e2m1(v);
                if (j % 2 == 0) q4[j / 2] = c;
                else            q4[j / 2] = (uint8_t)(q4[j / 2] | (c << 4));
            } else {
                q8[j - K4] = atom_ref_f32_to_e4m3(v);
            }
        }
    }
}

static int mx_shapes_ok(int32_t K, int32_t O)
{
    return K > 0 && O >= 0 && O < K && K % 32 == 0 && O % 32 == 0;
}

int atom_ref_mx_quantize_act(const uint16_t *x, int64_t M, int64_t ldx,
                             const uint16_t *gamma, float eps, const int32_t *idx,
                             int32_t K, int32_t O, float clip, uint8_t *q4,
                             uint8_t *q8, uint8_t *e8)
{
    if (!mx_shapes_ok(K, O) || ldx < K || M < 0) return -1;
    float *y = (float *)malloc(sizeof(float) * (size_t)K);
    if (!y) return -1;
    for (int64_t m = 0; m < M; ++m) {
        atom_ref_rmsnorm_row(x + m * ldx, gamma, eps, K, y);
        mx_quantize_row(y, idx, K, O, clip, q4 + m * ((K - O) / 2), q8 + m * O,
                        e8 + m * (K / 32));
    }
    free(y);
    return 0;
}

int atom_ref_mx_gemm(const uint8_t *a_q4, const uint8_t *a_q8, const uint8_t *a_e8,
                     int64_t M, const uint8_t *w_q4, const uint8_t *w_q8,
                     const uint8_t *w_e8, int64_t N, int32_t K, int32_t O,
                     uint16_t *y, int64_t ldy)
{
    if (!mx_shapes_ok(K, O) || M < 0 || N < 0 || ldy < N) return -1;
    int32_t K4 = K - O, NB = K / 32;
    /* decode both operands once */
    float *a = (float *)malloc(sizeof(float) * (size_t)(M > 0 ? M : 1) * (size_t)K);
    float *w = (float *)malloc(sizeof(float) * (size_t)(N > 0 ? N : 1) * (size_t)K);
    if (!a || !w) { free(a); free(w); return -1; }
    for (int pass = 0; pass < 2; ++pass) {
        int64_t        R  = pass ? N : M;
        const uint8_t *q4 = pass ? w_q4 : a_q4, *q8 = pass ? w_q8 : a_q8;
        float         *d  = pass ? w : a;
        for (int64_t r = 0; r < R; ++r)
            for (int32_t k = 0; k < K; ++k) {
                if (k < K4) {
                    uint8_t byte = q4[r * (K4 / 2) + k / 2];
                    d[r * K + k] = atom_ref_e2m1_to_f32((k % 2) ? (byte >> 4) : (byte & 0xf));
                } else {
                    d[r * K + k] = atom_ref_e4m3_to_f32(q8[r * O + (k - K4)]);
                }
            }
    }
    for (int64_t m = 0; m < M; ++m)
        for (int64_t n = 0; n < N; ++n) {
            double acc = 0.0;
            for (int32_t b = 0; b < NB; ++b) {
                double p = 0.0;
                for (int32_t t = 0; t < 32; ++t)
                    p += (double)a[m * K + b * 32 + t] * (double)w[n * K + b * 32 + t];
                acc += ldexp(p, (int)a_e8[m * NB + b] - 127 + (int)w_e8[n * NB + b] - 127);
            }
            y[m * ldy + n] = atom_ref_f32_to_f16((float)acc);
        }
    free(a);
    free(w);
    return 0;
}

/* ------------------------------------------------ offline calibration -- */
/* Section 5.1: the outlier channels are the ones with the highest square sum
 * over the calibration activations; activations and weights are reordered by
 * their indices.  Statistic of channel k: sum_t x[t,k]^2, EXACTLY: the square
 * of an fp16 value is an integer multiple of 2^-48 below 2^32, so the sum is
 * an integer of at most 112 bits whatever the order of the additions.  It is
 * reported as the nearest double (one rounding, ties to even); channels are
 * ranked by the exact integers.  Inf and NaN count as magnitude 2^16.
 * Index: channels in ascending order of (statistic, channel number): the O
 * largest come last for every O, and equal channels keep their order. */
static unsigned __int128 square_units(uint16_t h)     /* x^2 in units of 2^-48 */
{
    unsigned e = (h >> 10) & 31u, f = h & 1023u;
    uint64_t m;
    int      E;                                         /* |x| = m * 2^E */
    if (e == 0) { m = f; E = -24; }
    else if (e == 31) { m = 1024; E = 6; }
    else { m = 1024 + f; E = (int)e - 25; }
    return (unsigned __int128)(m * m) << (2 * E + 48);
}

int atom_ref_calibrate_reorder(const uint16_t *x, int64_t T, int64_t ldx, int32_t K,
                               double *stat, int32_t *idx)
{
    if (T < 0 || K <= 0 || ldx < K) return -1;
    unsigned __int128 *exact = (unsigned __int128 *)malloc((size_t)K * sizeof(unsigned __int128));
    if (!exact) return -1;
    for (int32_t k = 0; k < K; ++k) {
        unsigned __int128 s = 0;
        for (int64_t t = 0; t < T; ++t) s += square_units(x[t * ldx + k]);
        exact[k] = s;
        stat[k] = ldexp((double)s, -48);                /* integer -> double rounds to nearest even */
    }
    for (int32_t i = 0; i < K; ++i) {
        int32_t rank = 0;
        for (int32_t j = 0; j < K; ++j)
            if (exact[j] < exact[i] || (exact[j] == exact[i] && j < i)) ++rank;
        idx[rank] = i;
    }
    free(exact);
    return 0;
}
