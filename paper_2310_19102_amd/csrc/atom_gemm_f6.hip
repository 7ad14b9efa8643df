// Group GEMM on pre-tiled operands with the INT4 groups carried in FP6 (Section 4.2 of the
// paper, steps 1-3; the arithmetic is that of atom_gemm.hip).
//
// gfx950 has no INT4 matrix instruction, and on the INT8 one a 4-bit code costs as much as an
// 8-bit code.  It does have v_mfma_f32_32x32x64_f8f6f4, which runs FP6 operands at twice the INT8
// rate, and the E3M2 variant of FP6 represents every integer in [-8, 8] exactly.  An INT4 code is
// therefore re-encoded (not re-quantised) as the E3M2 number of the same value; the products of a
// group are integers of at most 7 bits, their sum over the 128 channels of a group is below 2^14,
// and the instruction's fp32 accumulation of such values is exact (checked on the hardware against
// integer sums, with accumulator inputs up to 2^23).  So the fp32 result tile IS the group's
// integer partial sum P[m, n, g], and step 2 needs no integer-to-float conversion: one fused
// multiply-add per element and group against the tile of scale products.  The 128 outlier channels
// stay INT8 on the INT8 MFMA.
//
// Operands come in an opaque tiled layout (pack_rows_kernel below writes it, from the canonical
// q4 / q8 / scale arrays; weights once, offline; activations per call into the workspace).  A
// "unit" is 64 rows; for every unit the images of its groups follow each other, each image being
// byte for byte what one LDS stage holds for that unit and group, so the K loop's loader is a
// linear copy global -> LDS by global_load_lds_dwordx4 (no registers, no address arithmetic, whole
// cache lines).
//   INT4 group image, 6656 bytes: lane (row r, half g) of the two FP6 MFMAs of a group holds the
//     channels 32 g .. 32 g + 31 (first MFMA) and 64 + 32 g .. 64 + 32 g + 31 (second) of its row:
//     2 x 24 = 48 bytes of FP6, stored as three 16-byte chunks c = 0, 1, 2 at
//     2048 c + 1024 g + 16 r, so that one 128-bit fragment read of a wavefront is one contiguous
//     kilobyte (bank-conflict free) and every address of a step is the lane's base plus an
//     immediate; the fp16 scale of row r, zero-extended to 64 bits (the operand of the fp16 MFMA
//     that forms the scale products: the scale in its first element, zeros behind), at 6144 + 8 r.
//   INT8 group image, 8704 bytes: 16-byte chunk c of row r at 128 r + 16 ((c ^ r ^ (r/8 % 2)) % 8),
//     scale at 8192 + 8 r.
// Rows past the end of the matrix hold zero codes and zero scales.
//
// Kernel: 256 x 128 (or 128 x 128, 64 x 128) tile, wavefront tile 64 x 64 = four 32 x 32 sub-tiles,
// NST LDS stages.  Per INT4 group and sub-tile: two FP6 MFMAs (64 channels each) and one fp16 MFMA
// that forms the 32 x 32 tile of scale products a_scale[m] * w_scale[n] (rank 1, exact in fp32),
// then 16 fused multiply-adds per lane.  Groups are added in ascending order, the INT8 group(s)
// last, each by one fmaf: the accumulation chain of the definition.
//
// PERSIST (256-row tiles, one INT8 group, at least as many tiles as CUs): one workgroup per CU walks
// its share of the tiles, and the stream of requests never stops at a tile's end.  The K loop's last
// two steps, which have nothing of their own tile left to ask for, request groups 0 and 1 of the
// next tile into the stages they have just freed; the INT8 group sits in the other two stages,
// which afterwards hold the output staging areas and then, behind one barrier, the next tile's
// groups 2 and 3.  The next tile starts with its first group long in LDS: no burst of four groups'
// requests, no round trip to memory, no wait for another workgroup to be launched.  Same sums in
// the same order as the one-tile kernel.  The waits count instructions (vmcnt returns in order),
// so what lies between the requests of a tile's groups 3 and 4 is kept at exactly eight
// vector-memory instructions: the eight 16-byte stores of the tile before, or eight dummy
// requests (first tile; a wavefront whose part of the tile is cut by M or N stores first,
// conditionally, and waits for all of it).

#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include <stdint.h>

#include <type_traits>

#include "atom_gemm_common.h"
#include "atom_internal.h"
#include "atom_launch.h"

namespace {

using namespace atom_gemm;

typedef int      v8i  __attribute__((ext_vector_type(8)));
typedef int      v12i __attribute__((ext_vector_type(12)));
typedef unsigned v6u  __attribute__((ext_vector_type(6)));
typedef unsigned v2u  __attribute__((ext_vector_type(2)));
typedef unsigned v4u  __attribute__((ext_vector_type(4)));
typedef float    v16f __attribute__((ext_vector_type(16)));
typedef _Float16 v32h __attribute__((ext_vector_type(32)));
typedef _Float16 v4h  __attribute__((ext_vector_type(4)));

constexpr int IMG4 = 6656;                // bytes of an INT4 group image of one unit
constexpr int IMG8 = 8704;                // bytes of an INT8 group image of one unit
constexpr int kU8  = 9216;                // pitch of the INT8 images in LDS where they are fetched during the K loop
constexpr int SC4  = 6144;                // offset of the scales inside an INT4 image
constexpr int SC8  = 8192;

__host__ __device__ constexpr int round_kb(int x) { return (x + 1023) / 1024 * 1024; }

// ------------------------------------------------------------------------------------------
// Packing: canonical rows -> unit images.  One thread per 16-byte destination chunk.
// ------------------------------------------------------------------------------------------
struct PackParams {
    const uint8_t *q4; const int8_t *q8; const uint16_t *scale;
    uint8_t *out;
    int64_t rows;                         // valid rows
    int     units, G4, G8, O;
    int64_t ustride;                      // bytes per unit = G4 * IMG4 + G8 * IMG8
};

__global__ __launch_bounds__(256)
void pack_rows_kernel(const PackParams p)
{
    const int     G    = p.G4 + p.G8;
    const int64_t K4h  = (int64_t)p.G4 * 64;          // bytes of a canonical q4 row
    const int     unit = blockIdx.y;
    const int     g    = blockIdx.x;                   // group; INT4 groups first
    uint8_t *img = p.out + (int64_t)unit * p.ustride + (g < p.G4 ? (int64_t)g * IMG4 : (int64_t)p.G4 * IMG4 + (int64_t)(g - p.G4) * IMG8);
    const int t = threadIdx.x;
    if (g < p.G4) {
        // thread t < 128: row t % 64, half t / 64; its 48 bytes are pieces `half` and `half + 2` of
        // the group (a piece = 32 consecutive channels = 16 canonical bytes = 24 bytes of FP6)
        if (t >= 128) return;
        const int row = t & 63, half = t >> 6;
        const int64_t m = (int64_t)unit * 64 + row;
        uint32_t out[12] = {0u, 0u, 0u, 0u, 0u, 0u, 0u, 0u, 0u, 0u, 0u, 0u};
        uint32_t sbits = 0;
        if (m < p.rows) {
#pragma unroll
            for (int s = 0; s < 2; ++s) {
                const v4u w = *reinterpret_cast<const v4u *>(p.q4 + m * K4h + (int64_t)g * 64 + (half + 2 * s) * 16);
                v32h h;
#pragma unroll
                for (int d = 0; d < 4; ++d)
#pragma unroll
                    for (int k = 0; k < 8; ++k)
                        h[8 * d + k] = (_Float16)(((int)(w[d] << (28 - 4 * k))) >> 28);   // sign-extended nibble k
                // the E3M2 number of each code (scale 1: a plain conversion; every code is representable)
                const v6u packed = __builtin_amdgcn_cvt_scalef32_pk32_bf6_f16(h, 1.0f);
#pragma unroll
                for (int d = 0; d < 6; ++d) out[6 * s + d] = packed[d];
            }
            sbits = p.scale[m * G + g];
        }
#pragma unroll
        for (int c = 0; c < 3; ++c)
            *reinterpret_cast<v4u *>(img + 2048 * c + 1024 * half + 16 * row) = v4u{out[4 * c], out[4 * c + 1], out[4 * c + 2], out[4 * c + 3]};
        if (half == 0) *reinterpret_cast<v2u *>(img + SC4 + 8 * row) = v2u{sbits, 0u};
    } else {
        // two chunks per thread: chunk ids t and t + 256 of the 512; row id / 8, slot id % 8
#pragma unroll
        for (int half = 0; half < 2; ++half) {
            const int id = t + 256 * half, row = id >> 3, slot = id & 7;
            const int chunk = (slot ^ row ^ ((row >> 3) & 1)) & 7;
            const int64_t m = (int64_t)unit * 64 + row;
            v4u w = {0u, 0u, 0u, 0u};
            uint32_t sbits = 0;
            if (m < p.rows) {
                w = *reinterpret_cast<const v4u *>(p.q8 + m * p.O + (int64_t)(g - p.G4) * 128 + chunk * 16);
                sbits = p.scale[m * G + g];
            }
            *reinterpret_cast<v4u *>(img + 16 * id) = w;
            if (slot == 0) *reinterpret_cast<v2u *>(img + SC8 + 8 * row) = v2u{sbits, 0u};
        }
    }
}

// ------------------------------------------------------------------------------------------
// The GEMM
// ------------------------------------------------------------------------------------------
struct F6Params {
    const uint8_t *a_pk, *w_pk;           // unit images of the activations / weights
    uint16_t *y; int32_t *partials;
    int64_t M, N, ldy;
    int     a_units, w_units, G4, G8;
    int64_t ustride;
};

__device__ __forceinline__ void dma16(uint32_t lds, uint32_t voff, const uint8_t *sbase)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :: "s"(lds), "v"(voff), "s"(sbase) : "memory", "m0");
}

// s_waitcnt immediate: vmcnt(n), lgkmcnt(0), expcnt untouched
__host__ __device__ constexpr int wait_imm(int n) { return (n & 15) | (7 << 4) | (0 << 8) | ((n >> 4) << 14); }

// A lane's operands of the two MFMAs of a group, as the three 128-bit fragment reads deliver them:
// registers 0-5 feed the first MFMA (channels 0-63 of the group), registers 6-11 the second.
template <int S>
__device__ __forceinline__ v16f mfma_f6(const v12i &a, const v12i &b, v16f c)
{
    // cbsz = blgp = 3: both operands E3M2 (six registers each); scale bytes 127 = 2^0
    const v8i a8 = __builtin_shufflevector(a, a, 6 * S, 6 * S + 1, 6 * S + 2, 6 * S + 3, 6 * S + 4, 6 * S + 5, -1, -1);
    const v8i b8 = __builtin_shufflevector(b, b, 6 * S, 6 * S + 1, 6 * S + 2, 6 * S + 3, 6 * S + 4, 6 * S + 5, -1, -1);
    return __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a8, b8, c, 3, 3, 0, 0x7f7f7f7f, 0, 0x7f7f7f7f);
}

// Order control.  MFMAs and fused multiply-adds have no side effects, so instruction selection
// is free to let them drift towards their consumers, which bunches each MFMA with the
// multiply-adds that wait for it.  An empty volatile asm that takes a value as an in/out operand
// is ordered with the other volatile statements and with the scheduling fences: whatever produces
// the value stays above it, whatever consumes it stays below.
#define ATOM_F6_PIN(x) asm volatile("" : "+v"(x))
#define ATOM_F6_SLOT_END()                         \
    do {                                           \
        asm volatile("" ::: "memory");             \
        __builtin_amdgcn_sched_barrier(0);         \
    } while (0)

template <int WM>
struct F6Geom {
    static constexpr int NWAVE = WM * 2;
    static constexpr int NT    = NWAVE * 64;
    static constexpr int NST   = WM == 4 ? 4 : 3;                 // LDS stages
    static constexpr int APART = round_kb(WM * IMG4);              // activation units of a stage (padded to whole DMA instructions)
    static constexpr int STAGE = APART + round_kb(2 * IMG4);
    static constexpr int NA    = APART / 1024, NI = STAGE / 1024; // DMA instructions per stage: NA for activations
    static constexpr int LPW   = (NI + NWAVE - 1) / NWAVE;        // at most, per wavefront
    static constexpr int APART8 = round_kb(WM * IMG8);
    static constexpr int STAGE8 = APART8 + round_kb(2 * IMG8);
    static constexpr int NA8   = APART8 / 1024, NI8 = STAGE8 / 1024;
    static constexpr int LPW8  = (NI8 + NWAVE - 1) / NWAVE;
    static constexpr int OSTRIDE = 144;                            // output staging: bytes per row of a wavefront's 64 x 64 fp16 tile
    static constexpr int OUT   = NWAVE * 64 * OSTRIDE;
    static constexpr int SPARE = NST * STAGE;                      // a kilobyte that is written and never read
    static constexpr int LDS0  = NST * STAGE + 1024 > STAGE8 ? NST * STAGE + 1024 : STAGE8;
    static constexpr int LDS   = LDS0 > OUT ? LDS0 : OUT;
};

template <int WM, bool DBG, bool PERSIST = false>
__global__ __launch_bounds__(WM * 128, 2)
void w4a4_gemm_f6_kernel(const F6Params p)
{
    using Gm = F6Geom<WM>;
    constexpr int NWAVE = Gm::NWAVE, NST = Gm::NST, STAGE = Gm::STAGE, APART = Gm::APART;
    constexpr int NA = Gm::NA, NI = Gm::NI, LPW = Gm::LPW;

    extern __shared__ __align__(16) unsigned char smem[];

    const int tid  = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave % WM, wn = wave / WM;
    const int r = lane & 31, g = lane >> 5;

    const int G4 = p.G4;
    // tile of this workgroup: M-tiles fastest, in bands of up to eight M-tiles so that the tiles an
    // XCD works on at one time share both activation and weight units in its L2
    const int TM = (p.a_units + WM - 1) / WM, TN = (p.w_units + 1) / 2;
    // PERSIST: a workgroup walks tiles logical, logical + lstep, ... < lend of its XCD's contiguous share
    int logical, lstep = 1, lend;
    if constexpr (PERSIST) {
        const int ntiles = TM * TN, nb = gridDim.x, xcd = blockIdx.x & 7;
        const int per = ntiles >> 3, rem = ntiles & 7;
        const int start = xcd * per + (xcd < rem ? xcd : rem);
        logical = start + (int)(blockIdx.x >> 3);
        lstep   = (nb - xcd + 7) >> 3;
        lend    = start + per + (xcd < rem ? 1 : 0);
    } else {
        logical = xcd_contiguous_block_id();
        lend    = logical + 1;
    }
    constexpr int LPWc = Gm::LPW;
    struct Tile {
        int a_valid, w_valid;
        const uint8_t *a_tile, *w_tile;
        int64_t m_w, n_w;
        uint32_t voff[LPWc];
    };
    // (the lane number as the per-tile code sees it: made opaque once per tile, so that what is
    // derived from it is recomputed there and does not hold registers through the K loop)
    int lane_t = lane;
    auto tile_of = [&](int lt) __attribute__((always_inline)) -> Tile {
        Tile t;
        const int band = 8 * TN, b = lt / band, rem = lt - b * band;
        const int hgt = TM - 8 * b < 8 ? TM - 8 * b : 8;          // M-tiles in this band
        const int tm = 8 * b + rem % hgt, tn = rem / hgt;
        const int au0 = tm * WM, wu0 = tn * 2;
        t.a_valid = p.a_units - au0 < WM ? p.a_units - au0 : WM;
        t.w_valid = p.w_units - wu0 < 2 ? p.w_units - wu0 : 2;
        t.a_tile = p.a_pk + (int64_t)au0 * p.ustride;
        t.w_tile = p.w_pk + (int64_t)wu0 * p.ustride;
        t.m_w = (int64_t)au0 * 64 + wm * 64;
        t.n_w = (int64_t)wu0 * 64 + wn * 64;
#pragma unroll
        for (int k = 0; k < LPW; ++k) {
            const int j0 = wave + NWAVE * k, j = j0 < NI ? j0 : wave;
            const bool isa = j < NA;
            int q = 64 * (isa ? j : j - NA) + lane_t;             // 16-byte chunk within the part
            const int nq = (isa ? WM : 2) * (IMG4 / 16);
            q = q < nq ? q : nq - 1;
            int unit = q / (IMG4 / 16);
            const int off = q - unit * (IMG4 / 16);
            const int valid = isa ? t.a_valid : t.w_valid;
            unit = unit < valid ? unit : valid - 1;               // ragged tiles repeat their last unit
            t.voff[k] = (uint32_t)unit * (uint32_t)p.ustride + 16u * off;
        }
        return t;
    };
    Tile T = tile_of(logical), Tn = T;
    uint32_t more_mask = 0;

    // ---- loader: DMA instruction j of a stage fills LDS bytes [1024 j, 1024 j + 1024) of the
    // stage; j < NA: activation units, else weight units.  Wavefront w issues j = w, w + NWAVE, ...
    // Lanes past the end of a part repeat its last chunk (they land in the padding).
    // Every wavefront issues LPW instructions per stage, so that the waits below are the same
    // immediate in every wavefront and no branch sits inside a K-step: a wavefront without an
    // LPW-th block repeats its first block into a spare kilobyte that nobody reads.
    const uint32_t vzero = 0;
    const uint32_t lds0 = (uint32_t)reinterpret_cast<uintptr_t>(smem), spare = lds0 + Gm::SPARE;
    // instruction k of the request of group v into stage `stage`
    auto request_one = [&](int k, int v, int stage) __attribute__((always_inline)) {
        const int j0 = wave + NWAVE * k, j = j0 < NI ? j0 : wave;
        // (selected with a mask, not with ?: -- the compiler turns that into a branch)
        const uint32_t mk = NWAVE * (k + 1) <= NI ? ~0u : 0u - (uint32_t)(j0 < NI);
        const uint32_t dst = spare + ((lds0 + stage * STAGE + 1024 * j - spare) & mk);
        dma16(dst, T.voff[k], (j < NA ? T.a_tile : T.w_tile) + (int64_t)v * IMG4);
    };
    // the same for group v of the workgroup's next tile (nothing real when there is none: the
    // current tile's bytes go to the spare kilobyte)
    auto request_next = [&](int k, int v, int stage) __attribute__((always_inline)) {
        const int j0 = wave + NWAVE * k, j = j0 < NI ? j0 : wave;
        const uint32_t mk = (NWAVE * (k + 1) <= NI ? ~0u : 0u - (uint32_t)(j0 < NI)) & more_mask;
        const uint32_t dst = spare + ((lds0 + stage * STAGE + 1024 * j - spare) & mk);
        dma16(dst, Tn.voff[k], (j < NA ? Tn.a_tile : Tn.w_tile) + (int64_t)v * IMG4);
    };
    // Past the last INT4 group the same number of instructions is issued, so that the count a wait
    // refers to never changes: every lane reads the tile's first 16 bytes (one cache line per
    // instruction) into the spare kilobyte.
    auto request_dummy = [&]() __attribute__((always_inline)) { dma16(spare, vzero, T.a_tile); };
    // Instruction k of the request of the first INT8 group, activation part (NA8 instructions) or
    // weight part, into stage `stage`: issued in place of the dummies of two of the last steps,
    // whose stages are free by then, so that the group has landed when the K loop ends.
    // (Here an image starts on a multiple of kU8 = 9 KB of the stage and is moved by nine
    // instructions of its own, so that everything but the lane's chunk is the same in all lanes.)
    auto request_int8 = [&](int k, int stage, bool act) __attribute__((always_inline)) {
        const int j = wave + NWAVE * k;
        const bool real = j < 9 * (act ? WM : 2);
        const int unit = j / 9, jin = j - 9 * unit;               // (uniform)
        const int valid = act ? T.a_valid : T.w_valid;
        const int src_unit = unit < valid ? unit : valid - 1;     // ragged tiles repeat their last unit
        int chunk = 64 * jin + lane_t;                            // 16-byte chunk of the image; its last instruction is half empty
        chunk = chunk < IMG8 / 16 ? chunk : IMG8 / 16 - 1;
        const uint32_t vo = (uint32_t)src_unit * (uint32_t)p.ustride + 16u * chunk;
        const uint32_t dst = real ? lds0 + stage * STAGE + unit * kU8 + 1024 * jin : spare;
        dma16(dst, vo, (act ? T.a_tile : T.w_tile) + (int64_t)G4 * IMG4);
    };

    // ---- fragment addresses: one register per operand (and one per operand for the scales) holds
    // the lane's address inside the stage of the coming group; everything a step reads is that
    // plus an immediate.  The registers move on by one stage per step.
    const uint32_t lane_off = lds0 + 1024 * g + 16 * r;
    const uint32_t a_off = wm * IMG4 + lane_off, b_off = APART + wn * IMG4 + lane_off;
    const uint32_t sa_off = lds0 + wm * IMG4 + SC4 + 8 * r, sb_off = lds0 + APART + wn * IMG4 + SC4 + 8 * r;

    // the 48 bytes of sub-tile row (column) block i of a unit: the operands of its two MFMAs
    // (addresses are 32-bit LDS addresses, the workgroup's base included)
    typedef __attribute__((address_space(3))) const v4i *lds_v4i;
    typedef __attribute__((address_space(3))) const v2u *lds_v2u;
    auto read_pair = [&](uint32_t addr, int i) __attribute__((always_inline)) -> v12i {
        const v4i c0 = *(lds_v4i)(uintptr_t)(addr + 512 * i);
        const v4i c1 = *(lds_v4i)(uintptr_t)(addr + 512 * i + 2048);
        const v4i c2 = *(lds_v4i)(uintptr_t)(addr + 512 * i + 4096);
        const v8i lo = __builtin_shufflevector(c0, c1, 0, 1, 2, 3, 4, 5, 6, 7);
        const v8i hi = __builtin_shufflevector(c2, c2, 0, 1, 2, 3, -1, -1, -1, -1);
        return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7, 8, 9, 10, 11);
    };
    // scale operand of rows 32 i + r: {fp16 bits, 0, 0, 0}
    auto read_scale = [&](uint32_t addr, int i) __attribute__((always_inline)) -> v2u {
        return *(lds_v2u)(uintptr_t)(addr + 256 * i);
    };

    v16f acc[4];
    const v16f zf = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};

    auto scale_tile = [&](v2u ta, v2u tb) __attribute__((always_inline)) -> v16f {
        return __builtin_amdgcn_mfma_f32_32x32x8f16(__builtin_bit_cast(v4h, ta), __builtin_bit_cast(v4h, tb), zf, 0, 0, 0);
    };
    // steps 2 and 3 for elements e0 .. e1-1 of sub-tile (i, j) of group grp
    auto dequant = [&](int grp, int i, int j, const v16f &c, const v16f &s, int e0, int e1) __attribute__((always_inline)) {
#pragma unroll
        for (int e = e0; e < e1; ++e) acc[2 * i + j][e] = fmaf(c[e], s[e], acc[2 * i + j][e]);
        if (DBG && grp >= 0) {
#pragma unroll
            for (int e = e0; e < e1; ++e) {
                const int64_t m = T.m_w + 32 * i + 8 * (e >> 2) + 4 * g + (e & 3), n = T.n_w + 32 * j + r;
                if (m < p.M && n < p.N) p.partials[(m * p.N + n) * (p.G4 + p.G8) + grp] = (int32_t)c[e];
            }
        }
    };

    // PERSIST: extra vector-memory instructions that stand between the requests of groups 3 and 4
    // of a tile: the eight stores of the tile before (the first tile: eight dummy requests)
    constexpr int XTRA = PERSIST ? 8 : 0;
    int base = 0;                               // stage of the current tile's group 0
    bool first = true;
    v12i af0, bf0;
    v2u sa[2], sb[2];
    v16f c_pend, s_pend;
    int  u_pend;
    int cur;
    uint32_t a_cur, b_cur;
    for (;;) {
    if constexpr (PERSIST) {
        int tz = 0;
        asm volatile("" : "+s"(tz));
        lane_t = lane + tz;
        const int nlogical = logical + lstep;
        const bool more = nlogical < lend;
        more_mask = more ? ~0u : 0u;
        Tn = tile_of(more ? nlogical : logical);
    }
    // ---- prologue: the first NST groups are requested (a later tile of a persistent workgroup: they
    // were, by the tile before), the first one has landed
    if (first) {
#pragma unroll
        for (int v = 0; v < NST; ++v) {
            if (v < G4) {
#pragma unroll
                for (int k = 0; k < LPW; ++k) request_one(k, v, v);
            } else {
#pragma unroll
                for (int k = 0; k < LPW; ++k) request_dummy();
            }
        }
#pragma unroll
        for (int k = 0; k < XTRA; ++k) request_dummy();
        first = false;
    }
    __builtin_amdgcn_s_waitcnt(wait_imm((NST - 1) * LPW + XTRA));
    __syncthreads();
#pragma unroll
    for (int t = 0; t < 4; ++t) acc[t] = zf;
    cur = base; a_cur = a_off + base * STAGE; b_cur = b_off + base * STAGE;
    // carried from step to step: the fragments of sub-tile row 0 / column 0 and the scale operands of
    // the coming step, and the integer and scale tiles of the last sub-tile of the step before
    af0 = read_pair(a_cur, 0); bf0 = read_pair(b_cur, 0);
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        sa[i] = read_scale(sa_off + base * STAGE, i);
        sb[i] = read_scale(sb_off + base * STAGE, i);
        sb[i][0] = g == 0 ? sb[i][0] : 0u;     // zero on one side keeps k-slots 4..7 of the fp16 MFMA empty
    }
    c_pend = zf; s_pend = zf;
    u_pend = -1;

    // One K-step = one INT4 group.  Twelve slots of one MFMA each, fenced so that the compiler keeps
    // their order.  Sub-tiles in the order (0,0) (1,0) (0,1) (1,1): column fragments 0 are free after
    // the second sub-tile and row fragments 0 after the third, and are refilled from the next stage.
    // Of the three slots of a sub-tile the first carries the step's memory instructions and address
    // updates, the other two eight fused multiply-adds each of the sub-tile before (its last MFMA
    // is two slots back by then): the vector ALU has about as much to do as the matrix pipe, and an
    // in-order wavefront that meets more than 32 cycles of vector work between two MFMAs holds
    // the matrix pipe up.  The barrier comes after the third slot: group u+1 has landed (each
    // wavefront waited for its own share before it) and every read of stage u is complete (issued
    // in the first slot), so from there on stage u is refilled with group u + NST, spread over
    // three slots: issued in one burst the requests fill the address queue and hold up MFMAs.
    // A step has no branch (one inside it lets the compiler sink MFMAs past the barrier): MODE says
    // at compile time what the step requests: 0 group u + NST, 1 nothing (dummies), 2 / 3 the
    // activation / weight part of the first INT8 group, 4 / 5 group 0 / 1 of the next tile; LOOSE
    // how many vector-memory instructions beside the requests of two groups may be outstanding at
    // the step's wait (the first three steps of a tile of a persistent workgroup: the eight that
    // stand between groups 3 and 4).
    auto step = [&](int u, auto mode_c, auto loose_c) __attribute__((always_inline)) {
        constexpr int MODE = decltype(mode_c)::value;
        constexpr int LOOSE = decltype(loose_c)::value;
        const int nxt = cur + 1 == NST ? 0 : cur + 1;
        // lane addresses in the next stage (they become the current ones of the next step)
        const uint32_t a_nxt = a_off + nxt * STAGE, b_nxt = b_off + nxt * STAGE;
        const uint32_t sa_nxt = sa_off + nxt * STAGE, sb_nxt = sb_off + nxt * STAGE;
        v12i af1, bf1;
        v16f c0, c1, c2, c3, s0, s1, s2, s3;
        v2u nsa[2], nsb[2];
        int kreq = 0;                           // DMA instructions of this step issued so far
        auto dma_slot = [&](int n) __attribute__((always_inline)) {
#pragma unroll
            for (int q = 0; q < n; ++q, ++kreq) {
                if (kreq < LPW) {
                    if constexpr (MODE == 0)      request_one(kreq, u + NST, cur);
                    else if constexpr (MODE == 2) request_int8(kreq, cur, true);
                    else if constexpr (MODE == 3) request_int8(kreq, cur, false);
                    else if constexpr (MODE == 4) request_next(kreq, 0, cur);
                    else if constexpr (MODE == 5) request_next(kreq, 1, cur);
                    else                          request_dummy();
                }
            }
        };
        constexpr int PER = (LPW + 2) / 3;      // per slot, over the three memory slots behind the barrier
        // slot 0
        ATOM_F6_PIN(af0);
        c0 = mfma_f6<0>(af0, bf0, zf);
        ATOM_F6_PIN(c0);
        af1 = read_pair(a_cur, 1);
        bf1 = read_pair(b_cur, 1);
        ATOM_F6_SLOT_END();
        // slot 1
        ATOM_F6_PIN(sa[0]);
        s0 = scale_tile(sa[0], sb[0]);
        ATOM_F6_PIN(s0);
        dequant(u_pend, 1, 1, c_pend, s_pend, 0, 8);
        ATOM_F6_PIN(acc[3]);
        ATOM_F6_SLOT_END();
        // slot 2
        c0 = mfma_f6<1>(af0, bf0, c0);
        ATOM_F6_PIN(c0);
        dequant(u_pend, 1, 1, c_pend, s_pend, 8, 16);
        ATOM_F6_PIN(acc[3]);
        ATOM_F6_SLOT_END();
        __builtin_amdgcn_s_waitcnt(wait_imm((NST - 2) * LPW + LOOSE));
        __syncthreads();
        __builtin_amdgcn_sched_barrier(0);
        // slot 3
        ATOM_F6_PIN(af1);
        ATOM_F6_PIN(bf0);
        c1 = mfma_f6<0>(af1, bf0, zf);
        ATOM_F6_PIN(c1);
        dma_slot(PER);
        ATOM_F6_SLOT_END();
        // slot 4
        ATOM_F6_PIN(sa[1]);
        s1 = scale_tile(sa[1], sb[0]);
        ATOM_F6_PIN(s1);
        dequant(u, 0, 0, c0, s0, 0, 8);
        ATOM_F6_PIN(acc[0]);
        ATOM_F6_SLOT_END();
        // slot 5
        c1 = mfma_f6<1>(af1, bf0, c1);
        ATOM_F6_PIN(c1);
        dequant(u, 0, 0, c0, s0, 8, 16);
        ATOM_F6_PIN(acc[0]);
        ATOM_F6_SLOT_END();
        // slot 6
        ATOM_F6_PIN(bf1);
        c2 = mfma_f6<0>(af0, bf1, zf);
        ATOM_F6_PIN(c2);
        bf0 = read_pair(b_nxt, 0);
        dma_slot(PER);
        ATOM_F6_SLOT_END();
        // slot 7
        ATOM_F6_PIN(sb[1]);
        s2 = scale_tile(sa[0], sb[1]);
        ATOM_F6_PIN(s2);
        dequant(u, 1, 0, c1, s1, 0, 8);
        ATOM_F6_PIN(acc[2]);
        ATOM_F6_SLOT_END();
        // slot 8
        c2 = mfma_f6<1>(af0, bf1, c2);
        ATOM_F6_PIN(c2);
        dequant(u, 1, 0, c1, s1, 8, 16);
        ATOM_F6_PIN(acc[2]);
        ATOM_F6_SLOT_END();
        // slot 9
        ATOM_F6_PIN(af1);
        c3 = mfma_f6<0>(af1, bf1, zf);
        ATOM_F6_PIN(c3);
        af0 = read_pair(a_nxt, 0);
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            nsa[i] = read_scale(sa_nxt, i);
            nsb[i] = read_scale(sb_nxt, i);
        }
        dma_slot(LPW);                          // whatever is left
        ATOM_F6_SLOT_END();
        // slot 10
        ATOM_F6_PIN(sa[1]);
        s3 = scale_tile(sa[1], sb[1]);
        ATOM_F6_PIN(s3);
        dequant(u, 0, 1, c2, s2, 0, 8);
        ATOM_F6_PIN(acc[1]);
        ATOM_F6_SLOT_END();
        // slot 11
        c3 = mfma_f6<1>(af1, bf1, c3);
        ATOM_F6_PIN(c3);
        dequant(u, 0, 1, c2, s2, 8, 16);
        ATOM_F6_PIN(acc[1]);
        ATOM_F6_PIN(nsa[0]); ATOM_F6_PIN(nsa[1]); ATOM_F6_PIN(nsb[0]); ATOM_F6_PIN(nsb[1]);   // (keeps the wait for these reads down here)
        sa[0] = nsa[0]; sa[1] = nsa[1];
        sb[0] = nsb[0]; sb[1] = nsb[1];
        sb[0][0] = g == 0 ? sb[0][0] : 0u; sb[1][0] = g == 0 ? sb[1][0] : 0u;
        ATOM_F6_SLOT_END();
        c_pend = c3; s_pend = s3; u_pend = u;
        cur = nxt; a_cur = a_nxt; b_cur = b_nxt;
    };
    // The last NST steps have nothing of the K loop left to request.  Two of them fetch the first
    // INT8 group instead (its two parts fit a stage each), which then costs no round trip of its own.
    static_assert(9 * WM <= LPW * NWAVE && 9 * 2 <= LPW * NWAVE && WM * kU8 <= STAGE && 2 * kU8 <= STAGE, "a part per step and stage");
    const bool pre8 = p.G8 >= 1 && G4 >= NST;
    int stage8a = 0, stage8w = 0;
    {
        using std::integral_constant;
        int u = 0;
        if constexpr (PERSIST) {                // (G4 >= NST + 3: the launcher sees to it)
            for (; u < 3; ++u) step(u, integral_constant<int, 0>{}, integral_constant<int, XTRA>{});
        }
        for (; u + NST < G4; ++u) step(u, integral_constant<int, 0>{}, integral_constant<int, 0>{});
        if (pre8) {
            stage8a = cur; step(u++, integral_constant<int, 2>{}, integral_constant<int, 0>{});
            stage8w = cur; step(u++, integral_constant<int, 3>{}, integral_constant<int, 0>{});
        }
        if constexpr (PERSIST) {
            step(u++, integral_constant<int, 4>{}, integral_constant<int, 0>{});
            step(u++, integral_constant<int, 5>{}, integral_constant<int, 0>{});
        } else {
            for (; u < G4; ++u) step(u, integral_constant<int, 1>{}, integral_constant<int, 0>{});
        }
    }
    dequant(u_pend, 1, 1, c_pend, s_pend, 0, 16);

    // ---- the INT8 groups: INT8 MFMA, int32 tile converted to fp32, the same dequantisation
    {
        constexpr int NA8 = Gm::NA8, NI8 = Gm::NI8, LPW8 = Gm::LPW8, APART8 = Gm::APART8;
        uint32_t voff8[LPW8];
#pragma unroll
        for (int k = 0; k < LPW8; ++k) {
            const int j = wave + NWAVE * k;
            const bool isa = j < NA8;
            int q = 64 * (isa ? j : j - NA8) + lane_t;
            const int nq = (isa ? WM : 2) * (IMG8 / 16);
            q = q < nq ? q : nq - 1;
            int unit = q / (IMG8 / 16);
            const int off = q - unit * (IMG8 / 16);
            const int valid = isa ? T.a_valid : T.w_valid;
            unit = unit < valid ? unit : valid - 1;
            voff8[k] = (uint32_t)unit * (uint32_t)p.ustride + 16u * off;
        }
        int ck[4];                                                 // byte offset of chunk 2 kk + g of row r
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) ck[kk] = 128 * (lane_t & 31) + 16 * (((2 * kk + (lane_t >> 5)) ^ (lane_t & 31) ^ (((lane_t & 31) >> 3) & 1)) & 7);
        // the requests of the K loop's last steps (PERSIST: all but the next tile's two groups)
        __builtin_amdgcn_s_waitcnt(wait_imm(PERSIST ? 2 * LPW : 0));
        for (int g8 = 0; g8 < p.G8; ++g8) {
            const bool here = pre8 && g8 == 0;                     // requested during the K loop, in two stages
            const int a_unit8 = here ? stage8a * STAGE + wm * kU8 : wm * IMG8;
            const int b_unit8 = here ? stage8w * STAGE + wn * kU8 : APART8 + wn * IMG8;
            __syncthreads();                                       // every read of the LDS contents so far is done
            if (!here) {
                const uint8_t *ab = T.a_tile + (int64_t)G4 * IMG4 + (int64_t)g8 * IMG8;
                const uint8_t *wb = T.w_tile + (int64_t)G4 * IMG4 + (int64_t)g8 * IMG8;
#pragma unroll
                for (int k = 0; k < LPW8; ++k) {
                    const int j = wave + NWAVE * k;
                    if (j < NI8) dma16(lds0 + 1024 * j, voff8[k], j < NA8 ? ab : wb);
                }
                __builtin_amdgcn_s_waitcnt(wait_imm(0));
                __syncthreads();
            }
            v2u qa[2], qb[2];
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                qa[i] = *reinterpret_cast<const v2u *>(smem + a_unit8 + SC8 + 8 * r + 256 * i);
                qb[i] = *reinterpret_cast<const v2u *>(smem + b_unit8 + SC8 + 8 * r + 256 * i);
                qb[i][0] = g == 0 ? qb[i][0] : 0u;
            }
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j) {
                    v16i ci = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
                    for (int kk = 0; kk < 4; ++kk) {
                        const v4i a = *reinterpret_cast<const v4i *>(smem + a_unit8 + ck[kk] + 4096 * i);
                        const v4i b = *reinterpret_cast<const v4i *>(smem + b_unit8 + ck[kk] + 4096 * j);
                        ci = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, ci, 0, 0, 0);
                    }
                    const v16f s = scale_tile(qa[i], qb[j]);
                    v16f cf;
#pragma unroll
                    for (int e = 0; e < 16; ++e) cf[e] = (float)ci[e];
                    dequant(G4 + g8, i, j, cf, s, 0, 16);
                }
        }
    }
    __syncthreads();                                               // LDS is free (PERSIST: but for the two stages of the next tile)

    // ---- store: the 64 x 64 fp16 tile of a wavefront goes through LDS so that global memory sees
    // whole 128-byte rows (a lane holds one column of the MFMA layout).  PERSIST: the staging areas lie
    // in the two stages the INT8 group was in.
    constexpr int OSTRIDE = Gm::OSTRIDE;
    static_assert(!PERSIST || (NWAVE / 2) * 64 * OSTRIDE <= STAGE, "four staging areas per stage");
    unsigned char *ot = PERSIST ? smem + (wave < NWAVE / 2 ? stage8a : stage8w) * STAGE + (wave % (NWAVE / 2)) * (64 * OSTRIDE)
                                : smem + wave * (64 * OSTRIDE);
#pragma unroll
    for (int t = 0; t < 4; ++t)
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            const int row = 32 * (t >> 1) + 8 * (e >> 2) + 4 * g + (e & 3);
            const int col = 32 * (t & 1) + r;
            *reinterpret_cast<uint16_t *>(ot + row * OSTRIDE + col * 2) = __half_as_ushort(__float2half_rn(acc[t][e]));
        }
    const bool vec_ok = ((reinterpret_cast<uintptr_t>(p.y) | (uintptr_t)(p.ldy * 2)) & 15) == 0;
    if constexpr (!PERSIST) {
        __builtin_amdgcn_s_waitcnt(wait_imm(0));                   // the wavefront reads only what it wrote itself
#pragma unroll
        for (int it = 0; it < 8; ++it) {
            const int row = it * 8 + (lane >> 3), ch = lane & 7;
            const int64_t m = T.m_w + row, n = T.n_w + ch * 8;
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
        break;
    } else {
        __builtin_amdgcn_s_waitcnt(wait_imm(63));                  // (LDS only: the wavefront reads what it wrote itself)
        uint4 ov[8];
#pragma unroll
        for (int it = 0; it < 8; ++it) ov[it] = *reinterpret_cast<const uint4 *>(ot + (it * 8 + (lane >> 3)) * OSTRIDE + (lane & 7) * 16);
        __builtin_amdgcn_s_waitcnt(wait_imm(63));
        __syncthreads();                                           // every staging area is read: the two stages are free
        const bool full = vec_ok && T.m_w + 64 <= p.M && T.n_w + 64 <= p.N;    // (the same in all lanes of a wavefront)
        auto store_rows = [&](auto full_c) __attribute__((always_inline)) {
#pragma unroll
            for (int it = 0; it < 8; ++it) {
                const int row = it * 8 + (lane >> 3), ch = lane & 7;
                const int64_t m = T.m_w + row, n = T.n_w + ch * 8;
                uint16_t *dst = p.y + m * p.ldy + n;
                if constexpr (decltype(full_c)::value) {
                    *reinterpret_cast<uint4 *>(dst) = ov[it];
                } else if (m < p.M && n < p.N) {
                    if (vec_ok && n + 8 <= p.N) {
                        *reinterpret_cast<uint4 *>(dst) = ov[it];
                    } else {
                        const uint16_t *hv = reinterpret_cast<const uint16_t *>(&ov[it]);
#pragma unroll
                        for (int k = 0; k < 8; ++k)
                            if (n + k < p.N) dst[k] = hv[k];
                    }
                }
            }
        };
        // The next tile's groups 2 and 3, then exactly eight more vector-memory instructions: the K
        // loop's first waits count on them.  A wavefront whose part of the tile is cut by M or N
        // stores first, waits for everything, and issues eight dummy requests in their place.
        if (!full) {
            store_rows(std::false_type());
            __builtin_amdgcn_s_waitcnt(wait_imm(0));
        }
#pragma unroll
        for (int k = 0; k < LPW; ++k) request_next(k, 2, stage8a);
#pragma unroll
        for (int k = 0; k < LPW; ++k) request_next(k, 3, stage8w);
        if (full) {
            store_rows(std::true_type());
        } else {
#pragma unroll
            for (int k = 0; k < XTRA; ++k) request_dummy();
        }
        if (more_mask == 0) {
            // (the last requests went to the spare kilobyte: they have landed before the workgroup's LDS is given up)
            __builtin_amdgcn_s_waitcnt(wait_imm(0));
            break;
        }
        logical += lstep;
        T = Tn;
        base = (base + G4 - 2) % NST;
    }
    }
}

template <int WM, bool DBG, bool PERSIST = false>
hipError_t launch_f6_cfg(const F6Params &p, hipStream_t stream)
{
    using Gm = F6Geom<WM>;
    static_assert(Gm::LDS <= 160 * 1024, "LDS of a compute unit");
    static_assert(Gm::LPW * (Gm::NST - 1) <= 63, "vmcnt is a 6-bit counter");
    const int64_t TM = (p.a_units + WM - 1) / WM, TN = (p.w_units + 1) / 2;
    auto kern = &w4a4_gemm_f6_kernel<WM, DBG, PERSIST>;
    static atom_launch::LdsOptIn opt_in;   // one attribute call per kernel variant and device
    hipError_t err = atom_launch::ensure_dynamic_lds(opt_in, reinterpret_cast<const void *>(kern), Gm::LDS);
    if (err != hipSuccess) return err;
    const int64_t grid = PERSIST ? (int64_t)atom_launch::compute_units() : TM * TN;
    hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(Gm::NT), Gm::LDS, stream, p);
    return hipGetLastError();
}

}  // namespace

namespace atom_internal {

size_t f6_packed_bytes(int64_t rows, int K, int O)
{
    const int64_t units = (rows + 63) / 64;
    const int G4 = (K - O) >> 7, G8 = O >> 7;
    return (size_t)(units * ((int64_t)G4 * IMG4 + (int64_t)G8 * IMG8));
}

hipError_t launch_f6_pack(const void *q4, const void *q8, const void *scale, int64_t rows, int K, int O,
                          void *out, hipStream_t stream)
{
    PackParams p;
    p.q4 = static_cast<const uint8_t *>(q4); p.q8 = static_cast<const int8_t *>(q8);
    p.scale = static_cast<const uint16_t *>(scale);
    p.out = static_cast<uint8_t *>(out);
    p.rows = rows;
    p.units = (int)((rows + 63) / 64);
    p.G4 = (K - O) >> 7; p.G8 = O >> 7; p.O = O;
    p.ustride = (int64_t)p.G4 * IMG4 + (int64_t)p.G8 * IMG8;
    hipLaunchKernelGGL(pack_rows_kernel, dim3((unsigned)(p.G4 + p.G8), (unsigned)p.units), dim3(256), 0, stream, p);
    return hipGetLastError();
}

hipError_t launch_f6_gemm(const void *a_pk, int64_t M, const void *w_pk, int64_t N, int K, int O, void *y,
                          int64_t ldy, int32_t *partials, hipStream_t stream)
{
    F6Params p;
    p.a_pk = static_cast<const uint8_t *>(a_pk); p.w_pk = static_cast<const uint8_t *>(w_pk);
    p.y = static_cast<uint16_t *>(y); p.partials = partials;
    p.M = M; p.N = N; p.ldy = ldy;
    p.a_units = (int)((M + 63) / 64); p.w_units = (int)((N + 63) / 64);
    p.G4 = (K - O) >> 7; p.G8 = O >> 7;
    p.ustride = (int64_t)p.G4 * IMG4 + (int64_t)p.G8 * IMG8;
    // 256-row tiles halve the weight traffic per row but want at least four rounds of tiles over the
    // 256 compute units (measured: M = 4096 shapes of 1024 tiles and more are 5-7 % faster with
    // them, M = 1024 shapes 4-15 % slower); 128-row tiles run two workgroups per compute unit,
    // which hides one's prologue, barriers and store behind the other's K loop
    const int64_t tiles256 = ((M + 255) / 256) * ((N + 127) / 128);
    // (the dump of the integer sums runs the same tile shape as the plain call)
    if (M > 128 && tiles256 >= 1024) {
        if (partials) return launch_f6_cfg<4, true>(p, stream);
        // one workgroup per CU that walks the tiles (see PERSIST in the file header): M = 4096, K = 8192:
        // N = 57344 1649 -> 1587 us, N = 10240 322 -> 314 us; K = 28672, N = 8192 787 us either way
        if (p.G8 == 1 && p.G4 >= F6Geom<4>::NST + 3 && tiles256 >= atom_launch::compute_units())
            return launch_f6_cfg<4, false, true>(p, stream);
        return launch_f6_cfg<4, false>(p, stream);
    }
    if (M > 64) return partials ? launch_f6_cfg<2, true>(p, stream) : launch_f6_cfg<2, false>(p, stream);
    return partials ? launch_f6_cfg<1, true>(p, stream) : launch_f6_cfg<1, false>(p, stream);
}

}  // namespace atom_internal
