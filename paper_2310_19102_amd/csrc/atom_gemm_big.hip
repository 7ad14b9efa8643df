// Big-tile variant of the group GEMM for compute-bound sizes (M > 64).
// Same arithmetic as atom_gemm.hip (Section 4.2 of the paper, steps 1-3); what
// differs is the schedule, built on measurements on gfx950:
//   (1) a wavefront keeps issuing vector instructions while its own MFMA runs (32 cycles
//       per 32x32x32 INT8 MFMA), and with two wavefronts per SIMD a stream of "one MFMA,
//       eight vector instructions" runs at the vector-ALU rate with the matrix pipe
//       about 75% busy, provided no slot of that stream waits on memory;
//   (2) the per-group dequantise-accumulate (one convert and one fused multiply-add per
//       output element) costs more vector cycles than the group's integer MFMAs cost
//       matrix cycles, so the vector ALU, not the matrix pipe, bounds this kernel;
//   (3) pulling operand fragments per wavefront straight from L1 saturates the
//       texture path, so operands are shared through LDS.
//
// Workgroup tile 256 x 128 (eight wavefronts) or 128 x 128 (four), wavefront tile
// 64 x 64 (four 32x32 sub-tiles), two LDS stages, one barrier per K-step.  A K-step
// moves 64 bytes per operand row HBM -> registers -> LDS, where they take 128 bytes: an
// INT4 group is widened to INT8 on the way; an INT8 group is two half-steps whose bytes
// are interleaved with zeros, so that every step has the same shape and ONE branch-free
// step body serves the whole K loop (a second, slower body for the few odd steps cost
// a fifth of the run time when it existed).  A step is twenty "slots" of one MFMA each,
// fenced so that the compiler keeps their order; the vector and memory work of a slot
// never consumes what the same slot produced (see `step`).
//
// The 32x32 tile of scale products a_scale[m,g] * w_scale[n,g] is one fp16 MFMA
// (rank-1, single non-zero k; the product of two fp16 values is exact in its
// fp32 accumulator), so the dequantisation is one convert and one fused multiply-add
// per element.  INT4 steps carry the 2^8 of the nibble widening in the
// accumulators; they are rescaled once, before the first INT8 step.

#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include <stdint.h>

#include <type_traits>

#include "atom_gemm_common.h"
#include "atom_launch.h"

namespace {

using namespace atom_gemm;

typedef float    v16f __attribute__((ext_vector_type(16)));
typedef _Float16 v4h  __attribute__((ext_vector_type(4)));
typedef unsigned v2u  __attribute__((ext_vector_type(2)));

// BM x BN: workgroup tile; KS sets of (BM/64) x (BN/64) wavefronts, at least two
// wavefronts per SIMD resident.  With KS = 2 the K-steps are split between two wavefront
// sets that run side by side on their own LDS stages and add their fp32 tiles once at
// the end (set 0 + set 1, a fixed order): for grids of at most one tile per CU, where a
// single set would leave every SIMD with one wavefront and nothing to overlap its MFMAs
// with.
template <int BM, int BN, int KS, bool DBG>
__global__ __launch_bounds__((BM / 64) * (BN / 64) * 64 * KS, 2)
void w4a4_gemm_big_kernel(const GemmParams p)
{
    constexpr int WM = BM / 64;                         // wavefronts down M
    constexpr int NT = WM * (BN / 64) * 64;             // threads of one set
    constexpr int RPT = NT / 4;                         // tile rows covered by one loader pass
    constexpr int CH = (BM + BN) / RPT;                 // 16-byte chunks per thread per K-step
    constexpr int CHA = BM / RPT;                       // of which activation rows
    constexpr int STAGE = (BM + BN) * 128 + NT * 4;     // codes + one scale slot per thread
    static_assert(BM % RPT == 0 && BN % RPT == 0 && RPT % 8 == 0, "loader layout");
    static_assert(BM + BN <= NT, "one scale per thread");

    extern __shared__ __align__(16) unsigned char smem_all[];

    // K-slice of this set: the same for a whole wavefront, and the compiler is told so
    const int ks   = KS == 1 ? 0 : __builtin_amdgcn_readfirstlane((int)threadIdx.x / NT);
    const int tid  = KS == 1 ? (int)threadIdx.x : (int)threadIdx.x % NT;   // thread within the set
    unsigned char *smem = smem_all;                     // the set's offset is folded into the per-thread LDS addresses
    const int set_off = ks * (2 * STAGE);
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wm = wave % WM, wn = wave / WM;
    const int r = lane & 31, h = lane >> 5;

    const int K4 = p.K - p.O, G = p.K >> 7, G4 = K4 >> 7;
    const int U  = G4 + 2 * (G - G4);                   // K-steps: one per INT4 group, two per INT8 group
    // this set's steps [ub, ue); with two sets the first takes the larger half
    const int ub = ks == 0 ? 0 : (U + 1) / 2;
    const int ue = KS == 1 ? U : (ks == 0 ? (U + 1) / 2 : U);

    const int MB      = (int)((p.M + BM - 1) / BM);
    const int logical = xcd_contiguous_block_id();
    const int64_t m0  = (int64_t)(logical % MB) * BM;
    const int64_t n0  = (int64_t)(logical / MB) * BN;

    // ---- loader: thread -> (tile row, 16-byte chunk).  Pass i covers rows wrow + i*RPT of
    // the stacked tile (BM activation rows, then BN weight rows).  Rows clamp to the last
    // valid row (such tile rows are computed and never stored).  32-bit offsets: arrays
    // < 4 GiB.
    const int wrow = tid >> 2, wc = tid & 3;
    uint32_t o4[CH], o8[CH];                           // row offsets into the INT4 / INT8 arrays
#pragma unroll
    for (int i = 0; i < CH; ++i) {
        int64_t row = i < CHA ? m0 + wrow + i * RPT : n0 + wrow + (i - CHA) * RPT;
        const int64_t last = i < CHA ? p.M - 1 : p.N - 1;
        row = row < last ? row : last;
        o4[i] = (uint32_t)(row * (K4 >> 1)) + wc * 16;
        o8[i] = (uint32_t)(row * p.O) + wc * 16;
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
    const int w4lo = set_off + lds_off(wrow, wc * 2);       // widened INT4: even-position codes
    const int w4hi = set_off + lds_off(wrow, wc * 2 + 1);   //               odd-position codes
    const int sc_slot = set_off + (BM + BN) * 128 + tid * 4;

    uint4    pre[CH];
    uint32_t sc = 0;

    // Loader items.  Chunk i of step v travels global -> registers (fetch_chunk) a whole
    // K-step before it travels registers -> LDS (stage_chunk); the step's scale likewise.
    // The kind of step v (INT4 group, or half of an INT8 group) only changes scalar
    // operands: base pointer, column, shift and masks.
    auto group_of = [&](int v) { return v < G4 ? v : G4 + ((v - G4) >> 1); };
    // `int4_c`: the caller knows at compile time that step v is an INT4 group
    auto fetch_chunk = [&](int i, int v, auto int4_c) __attribute__((always_inline)) {
        const bool is8 = decltype(int4_c)::value ? false : v >= G4;
        const uint8_t *base = i < CHA ? (is8 ? reinterpret_cast<const uint8_t *>(p.a_q8) : p.a_q4)
                                      : (is8 ? reinterpret_cast<const uint8_t *>(p.w_q8) : p.w_q4);
        const uint32_t col = (uint32_t)(is8 ? v - G4 : v) * 64;
        pre[i] = *reinterpret_cast<const uint4 *>(base + (size_t)((is8 ? o8[i] : o4[i]) + col));
    };
    auto fetch_scale = [&](int v, auto int4_c) __attribute__((always_inline)) {
        sc = sbase[(size_t)(soff + (uint32_t)(decltype(int4_c)::value ? v : group_of(v)))];
    };
    // INT4: even-position codes (x16) to chunk 2*wc, odd-position codes (x16) to chunk
    // 2*wc+1.  INT8 half-step: the 16 codes as they are to chunk 2*wc, zeros to 2*wc+1.
    auto stage_chunk = [&](int i, int v, unsigned char *base, auto int4_c) __attribute__((always_inline)) {
        const bool is8 = decltype(int4_c)::value ? false : v >= G4;
        const uint32_t sh = is8 ? 0u : 4u, mlo = is8 ? 0xFFFFFFFFu : 0xF0F0F0F0u, mhi = is8 ? 0u : 0xF0F0F0F0u;
        const uint4 w = pre[i];
        uint4 lo, hi;
        lo.x = (w.x << sh) & mlo; hi.x = w.x & mhi;
        lo.y = (w.y << sh) & mlo; hi.y = w.y & mhi;
        lo.z = (w.z << sh) & mlo; hi.z = w.z & mhi;
        lo.w = (w.w << sh) & mlo; hi.w = w.w & mhi;
        *reinterpret_cast<uint4 *>(base + w4lo + i * RPT * 128) = lo;
        *reinterpret_cast<uint4 *>(base + w4hi + i * RPT * 128) = hi;
    };
    // the scale goes in as raw fp16 bits (an MFMA operand); threads beyond the tile rows
    // write a slot nobody reads: no branch in the hot loop
    auto stage_scale = [&](unsigned char *base) __attribute__((always_inline)) {
        *reinterpret_cast<uint32_t *>(base + sc_slot) = has_scale ? sc : 0u;
    };

    // ---- fragment addresses within a stage: loop invariant ------------------------------
    int a_addr[4], b_addr[4];
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
        a_addr[kk] = set_off + lds_off(wm * 64 + r, 2 * kk + h);
        b_addr[kk] = set_off + lds_off(BM + wn * 64 + r, 2 * kk + h);
    }
    const int sa_addr = set_off + (BM + BN) * 128 + (wm * 64 + r) * 4;
    const int sb_addr = set_off + (BM + BN) * 128 + (BM + wn * 64 + r) * 4;

    float acc[4][16];
#pragma unroll
    for (int t = 0; t < 4; ++t)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[t][e] = 0.0f;

    const v16i zi = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
    const v16f zf = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};

    auto scale_tile = [&](uint32_t abits, uint32_t bbits) __attribute__((always_inline)) {
        const v2u ta = {abits, 0u}, tb = {bbits, 0u};
        return __builtin_amdgcn_mfma_f32_32x32x8f16(__builtin_bit_cast(v4h, ta),
                                                    __builtin_bit_cast(v4h, tb), zf, 0, 0, 0);
    };
    // steps 2 and 3 for elements e0 .. e0+ne-1 of the 32x32 sub-tile (i, j) of K-step u
    auto epilogue = [&](int u, int i, int j, const v16i &c, const v16f &ss, int e0, int ne) __attribute__((always_inline)) {
        float *a_ = acc[i * 2 + j];
#pragma unroll
        for (int e = e0; e < e0 + ne; ++e) a_[e] = fmaf((float)c[e], ss[e], a_[e]);
        if (DBG && u >= 0) {
#pragma unroll
            for (int e = e0; e < e0 + ne; ++e) {
                const int64_t m = m0 + wm * 64 + 32 * i + 8 * (e >> 2) + 4 * h + (e & 3);
                const int64_t n = n0 + wn * 64 + 32 * j + r;
                if (m < p.M && n < p.N) {
                    int32_t *dst = p.partials + (m * p.N + n) * G + group_of(u);
                    if (u < G4)                   *dst = c[e] >> 8;
                    else if (((u - G4) & 1) == 0) *dst = c[e];
                    else                          *dst += c[e];     // second half of an INT8 group
                }
            }
        }
    };

    // ---- K-step pipeline -------------------------------------------------------------
    // Carried from step to step: the first operand fragments and the scale bits of the
    // coming step (fetched from LDS in the last block of the step before, behind its
    // barrier, so no LDS latency is exposed at the start of a step), and the integer tile
    // and scale tile of the last sub-tile of the step before, whose dequantisation
    // overlaps the first MFMAs of this step.
    v4i fa0[4], fb0[4];
    uint32_t sa[2], sb[2];
    v16i c_pend = zi;
    v16f s_pend = zf;
    int  u_pend = -1;                                   // K-step of the pending tile (debug dump)

    auto load_first = [&](const unsigned char *base) __attribute__((always_inline)) {
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            fa0[kk] = *reinterpret_cast<const v4i *>(base + a_addr[kk]);
            fb0[kk] = *reinterpret_cast<const v4i *>(base + b_addr[kk]);
        }
    };
    auto load_scales = [&](const unsigned char *base) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            sa[i] = *reinterpret_cast<const uint32_t *>(base + sa_addr + i * 32 * 4);
            const uint32_t wb = *reinterpret_cast<const uint32_t *>(base + sb_addr + i * 32 * 4);
            sb[i] = h == 0 ? wb : 0u;      // zero on one side keeps k-slots 4..7 empty
        }
    };

    // One K-step; the same code for every step.  The operands of step u+1 go into the
    // other LDS stage here and the global loads of step u+2 are issued here; past the end
    // of this set's K range the last step's data is fetched and staged again (in bounds,
    // never read).
    // INT4: steps u+1 and u+2 are known to be INT4 groups (saves the scalar selects).
    //
    // A step is four blocks, one per 32x32 sub-tile in the order (0,0) (0,1) (1,1) (1,0); a
    // block is five slots of one MFMA each: the sub-tile's four integer MFMAs, then the
    // fp16 MFMA of its scale tile.  Beside its MFMA a slot holds
    //   first slot of blocks 0-2 : loader item (chunk t of step u+1 registers -> LDS, then
    //                              the global load of chunk t of step u+2 into the same
    //                              registers: a whole step of slack for HBM latency)
    //   slots 1-4 of every block : a quarter of the dequantisation of the sub-tile of the
    //                              block before (of the last sub-tile of the step before,
    //                              in block 0), whose integer and scale tiles are complete
    //   blocks 0, 1              : LDS reads of this step's second fragments b1, a1
    //   block 3                  : LDS reads of the next step's first fragments and scales
    // LDS hazards, with the single barrier before block 3: step u+1's operands are written
    // in blocks 0-2 of step u and read after the barrier; the stage they overwrite held
    // step u-1's, whose last reads (block 1 of step u-1) were complete at that step's
    // barrier.
    auto step = [&](int u, auto int4_c) __attribute__((always_inline)) {
        constexpr bool INT4 = decltype(int4_c)::value;
        const unsigned char *base = smem + (u & 1) * STAGE;
        unsigned char *nbase = smem + ((u + 1) & 1) * STAGE;
        const int v1 = INT4 || u + 1 < ue ? u + 1 : ue - 1;
        const int v2 = INT4 || u + 2 < ue ? u + 2 : ue - 1;
        v4i a1[4], b1[4];
        uint32_t nsa[2] = {0u, 0u}, nsb[2] = {0u, 0u};  // this step's scale bits stay live to its last slot
        v16i c_prev = c_pend;
        v16f s_prev = s_pend;
        int  u_prev = u_pend;
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            const int ti = t >> 1, tj = (t == 1 || t == 2) ? 1 : 0;       // this block's sub-tile
            const int pi = ((t + 3) & 3) >> 1, pj = (((t + 3) & 3) == 1 || ((t + 3) & 3) == 2) ? 1 : 0;
            const v4i *A = ti ? a1 : fa0;
            const v4i *B = tj ? b1 : fb0;
            v16i c = zi;
            v16f s = zf;
#pragma unroll
            for (int kk = 0; kk < 5; ++kk) {
                if (kk < 4) c = __builtin_amdgcn_mfma_i32_32x32x32_i8(A[kk], B[kk], c, 0, 0, 0);
                else        s = scale_tile(sa[ti], sb[tj]);
                // loader item
                const int item = kk == 0 && t < 3 ? t : (CH == 4 && t == 2 && kk == 2 ? 3 : -1);
                if (item >= 0 && item < CH) {
                    stage_chunk(item, v1, nbase, int4_c);
                    fetch_chunk(item, v2, int4_c);
                    if (item == CH - 1) {
                        stage_scale(nbase);
                        fetch_scale(v2, int4_c);
                    }
                }
                // second fragments of this step
                if (t == 0 && kk < 4) b1[kk] = *reinterpret_cast<const v4i *>(base + b_addr[kk] + 32 * 128);
                if (t == 1 && kk < 4) a1[kk] = *reinterpret_cast<const v4i *>(base + a_addr[kk] + 32 * 128);
                // a quarter of the dequantisation of the block before
                if (kk >= 1) epilogue(t == 0 ? u_prev : u, pi, pj, c_prev, s_prev, 4 * (kk - 1), 4);
                // first fragments and scale bits of the next step (behind the barrier)
                if (t == 3 && kk >= 1) {
                    if (kk <= 2) {
                        fa0[2 * kk - 2] = *reinterpret_cast<const v4i *>(nbase + a_addr[2 * kk - 2]);
                        fa0[2 * kk - 1] = *reinterpret_cast<const v4i *>(nbase + a_addr[2 * kk - 1]);
                        if (kk == 2) {
#pragma unroll
                            for (int i = 0; i < 2; ++i) {
                                nsa[i] = *reinterpret_cast<const uint32_t *>(nbase + sa_addr + i * 32 * 4);
                                nsb[i] = *reinterpret_cast<const uint32_t *>(nbase + sb_addr + i * 32 * 4);
                            }
                        }
                    } else {
                        // fb0 of this step was last used by the MFMA of slot 2 * kk - 5
                        fb0[2 * kk - 6] = *reinterpret_cast<const v4i *>(nbase + b_addr[2 * kk - 6]);
                        fb0[2 * kk - 5] = *reinterpret_cast<const v4i *>(nbase + b_addr[2 * kk - 5]);
                        if (kk == 4) {                  // zero on one side keeps k-slots 4..7 empty
                            nsb[0] = h == 0 ? nsb[0] : 0u;
                            nsb[1] = h == 0 ? nsb[1] : 0u;
                        }
                    }
                }
                __builtin_amdgcn_sched_barrier(0);
            }
            if (t == 2) {
                __syncthreads();
                __builtin_amdgcn_sched_barrier(0);
            }
            c_prev = c; s_prev = s; u_prev = u;
        }
        c_pend = c_prev; s_pend = s_prev; u_pend = u;
        sa[0] = nsa[0]; sa[1] = nsa[1]; sb[0] = nsb[0]; sb[1] = nsb[1];
    };
    // dequantise the pending sub-tile now (before the accumulators are rescaled or stored)
    auto flush_pending = [&]() __attribute__((always_inline)) {
        epilogue(u_pend, 1, 0, c_pend, s_pend, 0, 16);
        c_pend = zi; s_pend = zf; u_pend = -1;
    };

    // prologue: the first step into stage 0, the second into registers (a set has at
    // least two steps: there is always an INT4 group and an INT8 group, so U >= 3)
    const int ub1 = ub + 1 < ue ? ub + 1 : ue - 1;
#pragma unroll
    for (int i = 0; i < CH; ++i) fetch_chunk(i, ub, std::false_type{});
    fetch_scale(ub, std::false_type{});
#pragma unroll
    for (int i = 0; i < CH; ++i) stage_chunk(i, ub, smem + (ub & 1) * STAGE, std::false_type{});
    stage_scale(smem + (ub & 1) * STAGE);
#pragma unroll
    for (int i = 0; i < CH; ++i) fetch_chunk(i, ub1, std::false_type{});
    fetch_scale(ub1, std::false_type{});
    __syncthreads();
    load_first(smem + (ub & 1) * STAGE);
    load_scales(smem + (ub & 1) * STAGE);

    const int e4 = ue < G4 ? ue : G4;                   // end of this set's INT4 steps
    int u = ub;
    for (; u + 2 < e4; ++u) step(u, std::true_type{});  // INT4 groups followed by two more
    for (; u < e4; ++u) step(u, std::false_type{});     // the last two INT4 groups
    // leave the 2^8 of the nibble widening behind before the INT8 steps
    flush_pending();
#pragma unroll
    for (int t = 0; t < 4; ++t)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[t][e] *= (1.0f / 256.0f);
    for (; u < ue; ++u) step(u, std::false_type{});     // the INT8 groups, two half-steps each
    flush_pending();
    // every set passes the same number of barriers: the second one may have a step less
    if (KS == 2 && ks == 1 && (U & 1)) __syncthreads();
    __syncthreads();                                    // every fragment read is done: LDS is free

    // ---- two sets: set 1 hands its fp32 tile over through LDS, set 0 adds it to its own
    constexpr int XCH = KS == 2 ? (NT / 64) * 64 * 64 * 4 : 0;          // bytes of the exchange area
    if (KS == 2) {
        float *xch = reinterpret_cast<float *>(smem_all) + wave * (64 * 64);
        if (ks == 1) {
#pragma unroll
            for (int t = 0; t < 4; ++t)
#pragma unroll
                for (int e = 0; e < 16; ++e) xch[(t * 16 + e) * 64 + lane] = acc[t][e];
        }
        __syncthreads();
        if (ks == 0) {
#pragma unroll
            for (int t = 0; t < 4; ++t)
#pragma unroll
                for (int e = 0; e < 16; ++e) acc[t][e] = acc[t][e] + xch[(t * 16 + e) * 64 + lane];
        }
    }

    // ---- store: the 64x64 fp16 tile of a wavefront goes through LDS so that global
    // memory sees whole 128-byte rows (a lane holds one column: storing from the MFMA
    // layout directly would write 2 bytes per lane).  The stages are free; each wavefront
    // uses a private region behind the exchange area, row stride 144 bytes.
    constexpr int OSTRIDE = 144;
    static_assert(XCH + (NT / 64) * 64 * OSTRIDE <= KS * 2 * STAGE, "output staging fits the operand stages");
    unsigned char *ot = smem_all + XCH + wave * (64 * OSTRIDE);
    if (ks == 0) {
#pragma unroll
        for (int t = 0; t < 4; ++t)
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int row = 32 * (t >> 1) + 8 * (e >> 2) + 4 * h + (e & 3);
                const int col = 32 * (t & 1) + r;
                *reinterpret_cast<uint16_t *>(ot + row * OSTRIDE + col * 2) =
                    __half_as_ushort(__float2half_rn(acc[t][e]));
            }
    }
    __syncthreads();
    if (ks != 0) return;
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

template <int BM, int BN, int KS, bool DBG>
hipError_t launch_cfg(const GemmParams &p, hipStream_t stream)
{
    constexpr int NT = (BM / 64) * (BN / 64) * 64;
    constexpr int LDS = KS * 2 * ((BM + BN) * 128 + NT * 4);
    const int64_t MB = (p.M + BM - 1) / BM, NB = (p.N + BN - 1) / BN;
    auto kern = &w4a4_gemm_big_kernel<BM, BN, KS, DBG>;
    static atom_launch::LdsOptIn opt_in;   // one attribute call per kernel variant and device
    hipError_t err = atom_launch::ensure_dynamic_lds(opt_in, reinterpret_cast<const void *>(kern), LDS);
    if (err != hipSuccess) return err;
    hipLaunchKernelGGL(kern, dim3((unsigned)(MB * NB)), dim3(NT * KS), LDS, stream, p);
    return hipGetLastError();
}

}  // namespace

namespace atom_gemm {

hipError_t launch_big(const GemmParams &p, hipStream_t stream)
{
    if (p.partials) return launch_cfg<128, 128, 1, true>(p, stream);
    // The 256 x 128 tile does a third less loader work per MFMA; the 128 x 128 tile is
    // for shapes whose 256 x 128 tiles would leave compute units idle (one 512-thread
    // workgroup per CU; two of the 256-thread ones); with at most one 128 x 128 tile per
    // CU (256 CUs) two wavefront sets split K inside the workgroup.
    const int64_t big_tiles = ((p.M + 255) / 256) * ((p.N + 127) / 128);
    const int64_t tiles128  = ((p.M + 127) / 128) * ((p.N + 127) / 128);
    if (big_tiles >= 512) return launch_cfg<256, 128, 1, false>(p, stream);
    if (tiles128 <= 256)  return launch_cfg<128, 128, 2, false>(p, stream);
    return launch_cfg<128, 128, 1, false>(p, stream);
}

}  // namespace atom_gemm
