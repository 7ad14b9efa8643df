// GEMM of the MX variant for gfx950: both operands hold FP4 E2M1 codes (normal channels) and
// FP8 E4M3 codes (outlier channels, last) with one E8M0 scale byte per block of 32 channels.
// The paper (Section 5.2, FP4 paragraph) expects hardware group scaling to take the
// dequantisation out of the kernel; on gfx950 that is v_mfma_scale_f32_32x32x64_f8f6f4, which
// multiplies each lane's 32 elements by 2^(scale byte - 127) inside the matrix core.  The
// K loop below is therefore nothing but operand movement and MFMAs.
//
// Operand layout of the instruction (checked on the hardware against a CPU sum):
//   A 32 x 64: lane l holds row l % 32; FP4: its 16 bytes are elements 32g .. 32g+31 of the
//     K = 64 step, g = l / 32, even element in the low nibble; FP8: its 32 bytes are elements
//     16g .. 16g+15 and 32+16g .. 32+16g+15.  B likewise with columns for rows.
//   scale: byte `op_sel` of the scale register of lane (row, g) is the scale of elements
//     32g .. 32g+31 of the row: for FP4 the lane's own 16 bytes, for FP8 the low (g = 0) or
//     high (g = 1) 16 bytes of both lanes of the row.  Either way an MX block of 32
//     consecutive channels has one scale.
//   C 32 x 32: lane l holds column l % 32, rows 8 (v / 4) + 4 (l / 32) + v % 4, v = 0..15.

#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include <stdint.h>

#include <type_traits>

#include "atom_gemm_common.h"
#include "atom_internal.h"
#include "atom_launch.h"

namespace {

typedef int   v4i  __attribute__((ext_vector_type(4)));
typedef int   v8i  __attribute__((ext_vector_type(8)));
typedef float v16f __attribute__((ext_vector_type(16)));

constexpr int BM = 256, BN = 256;         // workgroup tile
constexpr int NT = 256;                   // 4 wavefronts, 2 x 2, each 128 x 128 (4 x 4 MFMA tiles)
constexpr int ROWB = 64;                  // bytes per tile row and K step: 128 FP4 or 64 FP8 channels
constexpr int CODES = (BM + BN) * ROWB;   // 32 KB of codes per stage
constexpr int STAGE = CODES + (BM + BN) * 4;   // + one scale dword per row
constexpr int NLD = CODES / 16 / NT;      // 16-byte chunks per thread and step (8)
constexpr int EPI_PITCH = 272;            // bytes per output row of a wavefront's LDS region
constexpr int EPI_WAVE  = 64 * EPI_PITCH; // 64 rows per pass
constexpr int LDS_BYTES = 4 * EPI_WAVE > 2 * STAGE ? 4 * EPI_WAVE : 2 * STAGE;

struct MxParams {
    const uint8_t *a_q4, *a_q8, *a_e8;
    const uint8_t *w_q4, *w_q8, *w_e8;
    uint16_t *y;
    int64_t M, N, ldy;
    int K, O;
};

// 16-byte chunk `chunk` (0..3) of tile row `row`: rows r, r+4, r+8, r+12 would share a bank
// group (4 rows of 64 bytes span the 64 banks once), so the chunk index is rotated by row / 4;
// a fragment read (16 consecutive rows, one chunk index) and the loader's writes (4 rows x 4
// chunks per 16 lanes) then touch 16 different bank groups.
__device__ __forceinline__ int mx_lds_off(int row, int chunk)
{
    return row * ROWB + (((chunk + (row >> 2)) & 3) << 4);
}

template <int FMT, int OPSEL>
__device__ __forceinline__ v16f mfma_mx(v8i a, v8i b, v16f c, int sa, int sb)
{
    return __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a, b, c, FMT, FMT, OPSEL, sa, OPSEL, sb);
}

__device__ __forceinline__ v8i widen(v4i lo)
{
    return __builtin_shufflevector(lo, lo, 0, 1, 2, 3, -1, -1, -1, -1);
}
__device__ __forceinline__ v8i join(v4i lo, v4i hi)
{
    return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
}

// One K step per iteration: 64 bytes of every tile row, i.e. 64 FP8 channels (one MFMA per tile
// pair; these outlier steps come first) or 128 FP4 channels (two MFMA sub-steps).  The accumulator
// tiles of a wavefront live in the accumulation registers, everything else in the architectural
// ones.  The operands go from global memory straight into LDS
// (global_load_lds_dwordx4: lane i's 16 bytes land at the LDS address in M0 plus 16 i), so no
// wavefront spends issue slots on staging registers and ds_write.  Four stages: while step u
// is multiplied, tile u+1 has landed or is landing, tile u+2 is on its way and tile u+3 is
// requested.  A wavefront
// instruction fills one kilobyte = 16 tile rows; lane l supplies the chunk that the rotated
// layout wants at its position: row l / 4 of the 16, chunk ((l % 4) - (l / 16)) % 4.
// The loads are inline assembly, the compiler does not count them: the waits on vmcnt before
// the barriers below are written by hand (ten loads per wavefront and tile, two tiles may
// stay in flight).
constexpr int DMA_STAGES = 4;

__device__ __forceinline__ void dma16(uint32_t lds, uint32_t voff, const uint8_t *sbase)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :: "s"(lds), "v"(voff), "s"(sbase) : "memory", "m0");
}
__device__ __forceinline__ void dma4(uint32_t lds, uint32_t voff, const uint8_t *sbase)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dword %1, %2"
                 :: "s"(lds), "v"(voff), "s"(sbase) : "memory", "m0");
}

// Geometry for WT x WT MFMA tiles per wavefront (2 x 2 wavefronts): WT = 4 is the 256 x 256
// workgroup tile, WT = 2 a 128 x 128 tile for grids that would leave most of the GPU idle
// with the large one (its 64 accumulator registers let two workgroups share a CU).
template <int WT>
struct DmaGeom {
    static constexpr int TB     = 64 * WT;                 // tile rows = tile columns
    static constexpr int CODES  = 2 * TB * ROWB;           // bytes of codes per stage
    static constexpr int STAGE  = CODES + 2 * 256 * 4;     // + 256 A and 256 B scale dwords (rows past TB unused)
    static constexpr int NBLK   = 2 * TB / 16 / 4;         // kilobyte blocks per wavefront and stage
    static constexpr int PITCH  = 64 * WT + 16;            // output row of a wavefront in LDS, bytes
    static constexpr int EPIW   = 64 * PITCH;              // 64 rows per pass
    static constexpr int LDS    = DMA_STAGES * STAGE > 4 * EPIW ? DMA_STAGES * STAGE : 4 * EPIW;
    static constexpr int LOADS  = NBLK + 2;                // DMA instructions per wavefront and tile
    // s_waitcnt: vmcnt(2 * LOADS) (two tiles may stay in flight), lgkmcnt(0), expcnt untouched
    static constexpr int LANDED = ((2 * LOADS) & 15) | (7 << 4) | (((2 * LOADS) >> 4) << 14);
};

template <int WT>
__global__ __launch_bounds__(NT) __attribute__((amdgpu_waves_per_eu(1, WT == 4 ? 1 : 2)))
void mx_gemm_dma_kernel(MxParams p)
{
    using Gm = DmaGeom<WT>;
    constexpr int TB = Gm::TB, CODES_ = Gm::CODES, STAGE_ = Gm::STAGE, NBLK = Gm::NBLK;
    extern __shared__ __align__(16) uint8_t smem[];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave >> 1, wn = wave & 1;
    const int lr = lane & 31, g = lane >> 5;

    const int tiles_m = (int)((p.M + TB - 1) / TB);
    const int bid = atom_gemm::xcd_contiguous_block_id();
    const int64_t m0 = (int64_t)(bid % tiles_m) * TB, n0 = (int64_t)(bid / tiles_m) * TB;

    const int K4 = p.K - p.O;
    const int S4 = K4 >> 7, S8 = p.O >> 6, S = S4 + S8;

    // ---- loader: wavefront w fills the kilobyte blocks NBLK w .. NBLK w + NBLK - 1 of a stage
    // (the first half of the blocks are the A rows: wavefronts 0, 1 load A, wavefronts 2, 3
    // load B) and 64 of the A and 64 of the B scale dwords
    const bool loadsA = wave < 2;
    uint32_t goff[NBLK];
#pragma unroll
    for (int j = 0; j < NBLK; ++j) {
        const int trow = 16 * (NBLK * wave + j) + (lane >> 2);           // row of the 2 TB-row stage
        int64_t r = loadsA ? m0 + trow : n0 + (trow - TB);
        const int64_t last = (loadsA ? p.M : p.N) - 1;
        r = r < last ? r : last;                                         // ragged tiles repeat the last row
        goff[j] = (uint32_t)r * ROWB + 16u * (((lane & 3) - (lane >> 4)) & 3);
    }
    const uint32_t sca = (uint32_t)(m0 + 64 * wave + lane < p.M ? m0 + 64 * wave + lane : p.M - 1) * 4u;
    const uint32_t scb = (uint32_t)(n0 + 64 * wave + lane < p.N ? n0 + 64 * wave + lane : p.N - 1) * 4u;
    const uint32_t lds0 = (uint32_t)reinterpret_cast<uintptr_t>(smem);
    // steps 0 .. S8-1 are the FP8 (outlier) steps, the FP4 steps follow
    auto request = [&](int u, int buf) __attribute__((always_inline)) {
        const bool    f8 = u < S8;
        const int64_t sl = f8 ? u : u - S8;                        // slab index inside q8 or q4
        const int64_t d  = f8 ? S4 + (u >> 1) : u - S8;            // slab index inside e8
        const uint8_t *src = loadsA ? (f8 ? p.a_q8 : p.a_q4) + sl * p.M * ROWB
                                    : (f8 ? p.w_q8 : p.w_q4) + sl * p.N * ROWB;
        const uint32_t st = lds0 + buf * STAGE_;
#pragma unroll
        for (int j = 0; j < NBLK; ++j) dma16(st + 1024 * (NBLK * wave + j), goff[j], src);
        dma4(st + CODES_ + 256 * wave, sca, p.a_e8 + d * p.M * 4);
        dma4(st + CODES_ + 1024 + 256 * wave, scb, p.w_e8 + d * p.N * 4);
    };
    // all but the two newest tiles' loads of this wavefront have landed, and its own LDS reads are done
#define ATOM_MX_LANDED() __builtin_amdgcn_s_waitcnt(Gm::LANDED)

    v16f acc[WT][WT];
#pragma unroll
    for (int s = 0; s < WT; ++s)
#pragma unroll
        for (int t = 0; t < WT; ++t)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[s][t][v] = 0.0f;

    const int a_base = mx_lds_off(32 * WT * wm + lr, g);
    const int b_base = mx_lds_off(TB + 32 * WT * wn + lr, g);
    const int sa_off = CODES_ + 4 * (32 * WT * wm + lr), sb_off = CODES_ + 1024 + 4 * (32 * WT * wn + lr);
    int sa[WT], sb[WT];
    auto read_scales = [&](const uint8_t *buf) __attribute__((always_inline)) {
#pragma unroll
        for (int s = 0; s < WT; ++s) {
            sa[s] = (int)(*reinterpret_cast<const uint32_t *>(buf + sa_off + 128 * s) >> (8 * g));
            sb[s] = (int)(*reinterpret_cast<const uint32_t *>(buf + sb_off + 128 * s) >> (8 * g));
        }
    };
    auto mma = [&](auto fmt, auto opsel, const v8i (&af)[WT], const v8i (&bf)[WT], const int (&sa_)[WT],
                   const int (&sb_)[WT]) __attribute__((always_inline)) {
#pragma unroll
        for (int s = 0; s < WT; ++s)
#pragma unroll
            for (int t = 0; t < WT; ++t)
                acc[s][t] = mfma_mx<decltype(fmt)::value, decltype(opsel)::value>(af[s], bf[t], acc[s][t],
                                                                                  sa_[s], sb_[t]);
    };
    using fp4 = std::integral_constant<int, 4>;
    using fp8 = std::integral_constant<int, 0>;
    using b0  = std::integral_constant<int, 0>;
    using b2  = std::integral_constant<int, 2>;

    // stage indices of tiles u, u+1, u+2, u+3
    int cur = 0, nxt = 1, nx2 = 2, nx3 = 3;
    request(0, 0);
    request(min(1, S - 1), 1);
    request(min(2, S - 1), 2);
    ATOM_MX_LANDED();
    __syncthreads();

    // ---- FP8 steps first, in pairs
    auto load8 = [&](const uint8_t *buf, v8i (&af8)[WT], v8i (&bf8)[WT]) __attribute__((always_inline)) {
#pragma unroll
        for (int s = 0; s < WT; ++s) {
            af8[s] = join(*reinterpret_cast<const v4i *>(buf + (a_base + 2048 * s)),
                          *reinterpret_cast<const v4i *>(buf + ((a_base ^ 32) + 2048 * s)));
            bf8[s] = join(*reinterpret_cast<const v4i *>(buf + (b_base + 2048 * s)),
                          *reinterpret_cast<const v4i *>(buf + ((b_base ^ 32) + 2048 * s)));
        }
    };
#define ATOM_MX_ROTATE()                                                                         \
    do {                                                                                         \
        const int t_ = cur;                                                                      \
        cur = nxt;                                                                               \
        nxt = nx2;                                                                               \
        nx2 = nx3;                                                                               \
        nx3 = t_;                                                                                \
    } while (0)
#define ATOM_MX_FP8_STEP(u, OPSEL)                                                               \
    do {                                                                                         \
        request(min((u) + 3, S - 1), nx3);                                                       \
        v8i af8[WT], bf8[WT];                                                                    \
        load8(smem + cur * STAGE_, af8, bf8);                                                    \
        read_scales(smem + cur * STAGE_);                                                        \
        mma(fp8{}, OPSEL{}, af8, bf8, sa, sb);                                                   \
        ATOM_MX_LANDED();                                                                        \
        __syncthreads();                                                                         \
        ATOM_MX_ROTATE();                                                                        \
    } while (0)
    int u = 0;
    for (; u < S8; u += 2) {
        ATOM_MX_FP8_STEP(u, b0);
        ATOM_MX_FP8_STEP(u + 1, b2);
    }
#undef ATOM_MX_FP8_STEP

    // ---- FP4 steps, software-pipelined: the second sub-step's fragments are read under the first
    // sub-step's MFMAs, the next step's first fragments and scales under the second's
    v8i af[WT], bf[WT];
#pragma unroll
    for (int s = 0; s < WT; ++s) {
        af[s] = widen(*reinterpret_cast<const v4i *>(smem + cur * STAGE_ + (a_base + 2048 * s)));
        bf[s] = widen(*reinterpret_cast<const v4i *>(smem + cur * STAGE_ + (b_base + 2048 * s)));
    }
    read_scales(smem + cur * STAGE_);
    for (; u < S; ++u) {
        const uint8_t *buf = smem + cur * STAGE_, *nbuf = smem + nxt * STAGE_;
        request(min(u + 3, S - 1), nx3);
        v8i ag[WT], bg[WT];
#pragma unroll
        for (int s = 0; s < WT; ++s) {
            ag[s] = widen(*reinterpret_cast<const v4i *>(buf + ((a_base ^ 32) + 2048 * s)));
            bg[s] = widen(*reinterpret_cast<const v4i *>(buf + ((b_base ^ 32) + 2048 * s)));
        }
        mma(fp4{}, b0{}, af, bf, sa, sb);
        // the reads go out under the first MFMAs, the remaining MFMAs cover them
#pragma unroll
        for (int i = 0; i < 2 * WT; ++i) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
        }
        if (WT * WT > 2 * WT) __builtin_amdgcn_sched_group_barrier(0x008, WT * WT - 2 * WT, 0);
        ATOM_MX_LANDED();                 // tile u+1 is in its stage ...
        __syncthreads();                  // ... for every wavefront; stage u has been read
        __builtin_amdgcn_sched_barrier(0);
        int sc[WT], sd[WT];
#pragma unroll
        for (int s = 0; s < WT; ++s) {
            sc[s] = sa[s];
            sd[s] = sb[s];
            af[s] = widen(*reinterpret_cast<const v4i *>(nbuf + (a_base + 2048 * s)));
            bf[s] = widen(*reinterpret_cast<const v4i *>(nbuf + (b_base + 2048 * s)));
        }
        read_scales(nbuf);
        mma(fp4{}, b2{}, ag, bg, sc, sd);
#pragma unroll
        for (int i = 0; i < 2 * WT; ++i) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 1);
            __builtin_amdgcn_sched_group_barrier(0x100, 2, 1);
        }
        if (WT * WT > 2 * WT) __builtin_amdgcn_sched_group_barrier(0x008, WT * WT - 2 * WT, 1);
        __builtin_amdgcn_sched_barrier(0);
        ATOM_MX_ROTATE();
    }
#undef ATOM_MX_ROTATE
#undef ATOM_MX_LANDED

    // ---- store: through LDS, so that global memory sees 16-byte row pieces; the last (repeated)
    // requests must have landed before the stages are reused
    __builtin_amdgcn_s_waitcnt(0x0F70);                            // vmcnt(0)
    const int64_t wrow = m0 + 32 * WT * wm, wcol = n0 + 32 * WT * wn;
    const bool whole = wrow + 32 * WT <= p.M && wcol + 32 * WT <= p.N && (p.ldy & 7) == 0 &&
                       (reinterpret_cast<uintptr_t>(p.y) & 15) == 0;
    __syncthreads();
    if (whole) {
        // passes of 64 rows; a row of the wavefront's block is 64 WT bytes = 4 WT lanes of 16 bytes
        uint8_t *reg = smem + wave * Gm::EPIW;
        constexpr int LPR = 4 * WT;                                // lanes per output row
#pragma unroll
        for (int pass = 0; pass < WT / 2; ++pass) {
#pragma unroll
            for (int sh = 0; sh < 2; ++sh)
#pragma unroll
                for (int t = 0; t < WT; ++t)
#pragma unroll
                    for (int v = 0; v < 16; ++v) {
                        const int r = 32 * sh + 8 * (v >> 2) + 4 * g + (v & 3);
                        *reinterpret_cast<uint16_t *>(reg + r * Gm::PITCH + 2 * (32 * t + lr)) =
                            __half_as_ushort(__float2half_rn(acc[2 * pass + sh][t][v]));
                    }
#pragma unroll
            for (int i = 0; i < 64 * LPR / 64; ++i) {
                const int r = (64 / LPR) * i + lane / LPR;
                const v4i d = *reinterpret_cast<const v4i *>(reg + r * Gm::PITCH + 16 * (lane % LPR));
                *reinterpret_cast<v4i *>(p.y + (wrow + 64 * pass + r) * p.ldy + wcol + 8 * (lane % LPR)) = d;
            }
        }
    } else {
        const int64_t row0 = wrow + 4 * g, col0 = wcol + lr;
        uint16_t *yp = p.y + row0 * p.ldy + col0;
#pragma unroll
        for (int s = 0; s < WT; ++s)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int dr = 32 * s + 8 * (v >> 2) + (v & 3);
                if (row0 + dr < p.M) {
                    uint16_t *yr = yp + (int64_t)dr * p.ldy;
#pragma unroll
                    for (int t = 0; t < WT; ++t)
                        if (col0 + 32 * t < p.N) yr[32 * t] = __half_as_ushort(__float2half_rn(acc[s][t][v]));
                }
            }
    }
}

}  // namespace

namespace atom_internal {

hipError_t launch_mx_gemm(const void *a_q4, const void *a_q8, const void *a_e8, int64_t M,
                          const void *w_q4, const void *w_q8, const void *w_e8, int64_t N, int K,
                          int O, void *y, int64_t ldy, hipStream_t stream)
{
    MxParams p;
    p.a_q4 = (const uint8_t *)a_q4; p.a_q8 = (const uint8_t *)a_q8; p.a_e8 = (const uint8_t *)a_e8;
    p.w_q4 = (const uint8_t *)w_q4; p.w_q8 = (const uint8_t *)w_q8; p.w_e8 = (const uint8_t *)w_e8;
    p.y = (uint16_t *)y; p.M = M; p.N = N; p.ldy = ldy; p.K = K; p.O = O;
    const int64_t tiles = ((M + BM - 1) / BM) * ((N + BN - 1) / BN);
    if (tiles >= 192) {
        static atom_launch::LdsOptIn opt_in;
        hipError_t err = atom_launch::ensure_dynamic_lds(opt_in, reinterpret_cast<const void *>(&mx_gemm_dma_kernel<4>), DmaGeom<4>::LDS);
        if (err != hipSuccess) return err;
        hipLaunchKernelGGL(mx_gemm_dma_kernel<4>, dim3((unsigned)tiles), dim3(NT), DmaGeom<4>::LDS, stream, p);
    } else {
        // fewer 256 x 256 tiles than would occupy three quarters of the CUs: 128 x 128 tiles, two
        // workgroups per CU (measured on M = 1024, K = 11008, N = 4096: 82 -> 40 us)
        const int64_t small = ((M + 127) / 128) * ((N + 127) / 128);
        static atom_launch::LdsOptIn opt_in;
        hipError_t err = atom_launch::ensure_dynamic_lds(opt_in, reinterpret_cast<const void *>(&mx_gemm_dma_kernel<2>), DmaGeom<2>::LDS);
        if (err != hipSuccess) return err;
        hipLaunchKernelGGL(mx_gemm_dma_kernel<2>, dim3((unsigned)small), dim3(NT), DmaGeom<2>::LDS, stream, p);
    }
    return hipGetLastError();
}

}  // namespace atom_internal
