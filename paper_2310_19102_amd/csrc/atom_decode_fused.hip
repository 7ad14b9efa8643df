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
//
// A second kernel (decode_linear_coop_kernel, further down) does the front end once per launch
// instead of once per workgroup, for the price of a wait between workgroups.

#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include <stdint.h>

#include "atom_gemm_common.h"
#include "atom_gemm_decode_staged.h"
#include "atom_internal.h"
#include "atom_launch.h"
#include "atom_quantize_rows.h"

namespace {

using namespace atom_gemm;
using namespace atom_quantize_rows;

using namespace atom_decode_staged;      // NW, NT, TN, widen_lo / widen_hi, decode_staged_body

struct FusedParams {
    const __half *x; int64_t ldx; int M;
    const __half *gamma; float eps; const int32_t *idx;
    int K, O, nbits; float clip;
    const uint8_t *w_q4; const int8_t *w_q8; const uint16_t *w_scale; int64_t N;
    uint16_t *y; int64_t ldy;
    uint8_t *dbg_q4; int8_t *dbg_q8; uint16_t *dbg_scale;     // the activation codes, or null
    unsigned lds_front;                                        // bytes of the front end's staging area
};

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

// ------------------------------------------------------------------------------------------
// The same linear layer with the front end done once.  The first M workgroups of the launch
// quantise one row each into global arrays (the outputs of the stand-alone front end) and
// count themselves in; every other workgroup is a workgroup of the stand-alone decode GEMM that
// requests its weights first, waits until the count says M, and then fetches the codes: the
// front end runs while the weights travel from HBM.  Workgroups are dispatched in index order, so
// the M producers are running (or done) before any consumer waits for them, and they wait for
// nobody.  A consumer's wait is bounded (kSpinLimit polls): if it runs out, a word is set that
// the caller can read, and the kernel still ends.
//
// The words of `sync` (32-bit; each counter in a 128-byte line of its own):
//   [0]                 rows ready
//   [1]                 a wait ran out (never cleared here)
//   [32]                buckets complete
//   [64 + 32 b]         consumers of bucket b (workgroup c belongs to bucket c % 32) past their wait
// A consumer counts itself into its bucket when it is past its wait (the value comes back while
// it computes), with an increment that wraps to zero at the bucket's size; whoever completes a
// bucket counts the bucket the same way, whoever completes the buckets zeroes the rows: by then
// every consumer is past its wait, and the next launch finds zeros.  (One counter for all
// consumers would do, but read-modify-writes of one address are served one after the other.)
//
// What it costs: the chain front end -> release -> poll -> fetch of the codes from memory is
// about as long as the gap between two launches in a stream, so inside a HIP graph the kernel
// ties with the two launches (and loses where N / 16 workgroups need a second round, which can
// only start when the first, waiting, round is through); called eagerly, where the host's launch
// cost sets the pace, one launch is what counts.
// ------------------------------------------------------------------------------------------
constexpr uint32_t kSpinLimit = 1u << 18;
constexpr int kBuckets = 32;
constexpr int kSyncWords = 64 + 32 * kBuckets;

struct CoopParams {
    const __half *x; int64_t ldx;
    const __half *gamma; float eps; const int32_t *idx; int nbits; float clip;
    GemmParams g;                 // a_q4 / a_q8 / a_scale: written by the producers, read by the consumers
    uint32_t *sync;
    int variant;                  // 2 * log2(staging instructions) + (last block of K has two groups)
};

// One wavefront of a consumer workgroup (the last: it always has groups to work on) polls the
// count in memory and passes the news on through a word in LDS; the others poll that word.
// No cache is invalidated: a load of the consumer misses in its CU's vector cache (invalidated at
// the start of a kernel, and the workgroup has not read the arrays before) and in its XCD's L2
// (likewise, and nobody on any XCD reads the arrays before the count is complete: they share no
// 128-byte line with anything else the kernel reads), so it is served from memory, where the
// producers' release has put their rows.  An L2 invalidation per waiting wavefront, which an
// acquire at agent scope amounts to, took 0.1 us per workgroup.
struct WaitForRows {
    uint32_t *sync; uint32_t rows; uint32_t *lds_flag; bool poller; uint32_t bucket, members; uint32_t *before_me;
    uint32_t *first_look;
    // A plain load of the count, requested before the weights so that its answer is there before
    // theirs.  It may be served by the XCD's L2 and may therefore be old, but the count only grows
    // during a launch and no L2 holds a value of an earlier launch: "all rows" is always true.  A
    // workgroup that starts after the rows are done (the second round and later of a large N) then
    // goes on without a round trip to memory.
    // (every wavefront takes it, with no branch around the load: behind a branch the compiler waits
    // for the answer before it goes on)
    __device__ __forceinline__ void early() const
    {
        *first_look = __hip_atomic_load(sync, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
    }
    __device__ __forceinline__ void wait() const
    {
        if (poller) {
            uint32_t polls = 0;
            while (*first_look < rows && __hip_atomic_load(sync, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < rows) {
                if (++polls > kSpinLimit) {
                    __hip_atomic_store(sync + 1, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    break;
                }
                __builtin_amdgcn_s_sleep(4);
            }
            __hip_atomic_store(lds_flag, 1u, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_WORKGROUP);
        } else {
            while (__hip_atomic_load(lds_flag, __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_WORKGROUP) == 0u)
                __builtin_amdgcn_s_sleep(2);
        }
        // (keeps the compiler from moving the loads of the codes above the wait)
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
    }
    // the polling wavefront counts the workgroup into its bucket (it is the last to leave the wait);
    // issued behind the loads of the codes, so that its return does not hold theirs up
    __device__ __forceinline__ void passed() const
    {
        // (a wrapping increment: the counter is back at zero with its last member.  Also, the
        // compiler rewrites a fetch-and-add of a uniform address into a form that needs the answer
        // on the spot; this one it leaves alone)
        if (poller && (threadIdx.x & 63) == 0)
            *before_me = __builtin_amdgcn_atomic_inc32(sync + 64 + 32 * bucket, members - 1u, __ATOMIC_RELAXED, "agent");
    }
};

template <bool NORM, int NS, bool IDENT>
__global__ __launch_bounds__(NT)
void decode_linear_coop_kernel(const CoopParams p)
{
    extern __shared__ __align__(16) unsigned char smem[];
    const int M = (int)p.g.M;
    if ((int)blockIdx.x < M) {
        // producer: row blockIdx.x through the row routine of the stand-alone front end
        quantize_rows_fast_body<NORM, NS, NT, kPlain, IDENT>(
            reinterpret_cast<float *>(smem), blockIdx.x, M, p.x, M, p.ldx, nullptr, 0, nullptr, 0, p.gamma, p.eps, p.idx,
            p.g.K, p.g.O, p.nbits, p.clip, const_cast<uint8_t *>(p.g.a_q4), const_cast<int8_t *>(p.g.a_q8),
            reinterpret_cast<__half *>(const_cast<uint16_t *>(p.g.a_scale)));
        // every wavefront's stores are out and written back before the row is counted (a release
        // only: __threadfence() would also invalidate the L2)
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
        __syncthreads();
        if (threadIdx.x == 0) __hip_atomic_fetch_add(p.sync, 1u, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
        return;
    }
    const int block = (int)blockIdx.x - M;
    // the word the polling wavefront sets, behind the routine's own LDS
    uint32_t *lds_flag = reinterpret_cast<uint32_t *>(smem + kStageBytes);
    if (threadIdx.x == 0) *lds_flag = 0u;
    __syncthreads();
    const bool poller = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6) == NW - 1;
    const uint32_t consumers = gridDim.x - (uint32_t)M, bucket = (uint32_t)block % kBuckets;
    // (not initialised on purpose: writing a register that a memory instruction in flight is going
    // to fill makes the compiler wait for that instruction on the spot)
    uint32_t before_me;           // (first lane of the polling wavefront) members of the bucket past their wait before this one
    uint32_t first_look;
    const uint32_t members = (consumers - bucket + kBuckets - 1) / kBuckets;
    const WaitForRows wait{p.sync, (uint32_t)M, lds_flag, poller, bucket, members, &before_me, &first_look};
    switch (p.variant) {
    case 0:  decode_staged_body<1, false, 3, true>(p.g, block, smem, wait); break;
    case 1:  decode_staged_body<1, false, 1, true>(p.g, block, smem, wait); break;
    case 2:  decode_staged_body<2, false, 3, true>(p.g, block, smem, wait); break;
    case 3:  decode_staged_body<2, false, 1, true>(p.g, block, smem, wait); break;
    case 4:  decode_staged_body<4, false, 3, true>(p.g, block, smem, wait); break;
    default: decode_staged_body<4, false, 1, true>(p.g, block, smem, wait); break;
    }
    // whoever completes a bucket (its counter is back at zero) counts the bucket; whoever completes
    // the buckets (likewise) zeroes the rows: the counters are as the launch found them
    if (poller && (threadIdx.x & 63) == 0) {
        if (before_me == members - 1) {
            const uint32_t buckets = consumers < (uint32_t)kBuckets ? consumers : (uint32_t)kBuckets;
            if (__builtin_amdgcn_atomic_inc32(p.sync + 32, buckets - 1u, __ATOMIC_RELAXED, "agent") == buckets - 1)
                __hip_atomic_store(p.sync, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
}

template <bool NORM, int NS, bool IDENT>
hipError_t launch_coop_cfg(const CoopParams &p, size_t lds, hipStream_t stream)
{
    auto kern = &decode_linear_coop_kernel<NORM, NS, IDENT>;
    static atom_launch::LdsOptIn opt_in;
    hipError_t err = atom_launch::ensure_dynamic_lds(opt_in, reinterpret_cast<const void *>(kern), lds);
    if (err != hipSuccess) return err;
    const unsigned blocks = (unsigned)p.g.M + (unsigned)((p.g.N + TN - 1) / TN);
    hipLaunchKernelGGL(kern, dim3(blocks), dim3(NT), lds, stream, p);
    return hipGetLastError();
}

template <bool NORM, int NS>
hipError_t launch_coop_ident(const CoopParams &p, size_t lds, hipStream_t stream)
{
    return p.idx ? launch_coop_cfg<NORM, NS, false>(p, lds, stream) : launch_coop_cfg<NORM, NS, true>(p, lds, stream);
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

size_t decode_linear_coop_sync_bytes() { return 4 * (size_t)kSyncWords; }

bool decode_linear_coop_supported(int M, int K, int O, const void *a_scale, const void *w_scale, int64_t N)
{
    GemmParams g{};
    g.a_scale = static_cast<const uint16_t *>(a_scale); g.w_scale = static_cast<const uint16_t *>(w_scale);
    g.M = M; g.N = N; g.K = K; g.O = O;
    return M >= 1 && M <= 16 && K <= 12288 && common_tail(g) != 0;
}

hipError_t launch_decode_linear_coop(const void *x, int M, int64_t ldx, const void *gamma, float eps,
                                     const int32_t *idx, int K, int O, int nbits, float clip,
                                     const void *w_q4, const void *w_q8, const void *w_scale, int64_t N,
                                     void *y, int64_t ldy, void *a_q4, void *a_q8, void *a_scale, void *sync,
                                     hipStream_t stream)
{
    const bool norm = gamma != nullptr;
    CoopParams p;
    p.x = static_cast<const __half *>(x); p.ldx = ldx;
    p.gamma = static_cast<const __half *>(gamma); p.eps = eps; p.idx = idx; p.nbits = nbits; p.clip = clip;
    p.g.a_q4 = static_cast<const uint8_t *>(a_q4); p.g.a_q8 = static_cast<const int8_t *>(a_q8);
    p.g.a_scale = static_cast<const uint16_t *>(a_scale);
    p.g.w_q4 = static_cast<const uint8_t *>(w_q4); p.g.w_q8 = static_cast<const int8_t *>(w_q8);
    p.g.w_scale = static_cast<const uint16_t *>(w_scale);
    p.g.y = static_cast<uint16_t *>(y); p.g.partials = nullptr;
    p.g.M = M; p.g.N = N; p.g.ldy = ldy; p.g.K = K; p.g.O = O;
    p.sync = static_cast<uint32_t *>(sync);
    p.variant = 2 * (M <= 4 ? 0 : M <= 8 ? 1 : 2) + (common_tail(p.g) == 1 ? 1 : 0);
    const size_t front = front_bytes(K, norm, idx == nullptr);
    const size_t lds = (front > (size_t)kStageBytes ? front : (size_t)kStageBytes) + 16;    // and the consumers' flag
    if (K <= 4096) return norm ? launch_coop_ident<true, 1>(p, lds, stream) : launch_coop_ident<false, 1>(p, lds, stream);
    if (K <= 8192) return norm ? launch_coop_ident<true, 2>(p, lds, stream) : launch_coop_ident<false, 2>(p, lds, stream);
    return norm ? launch_coop_ident<true, 3>(p, lds, stream) : launch_coop_ident<false, 3>(p, lds, stream);
}

}  // namespace atom_internal
