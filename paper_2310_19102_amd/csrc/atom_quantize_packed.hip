// The activation front end writing the packed GEMM's unit images directly (Sections 4.1 - 4.3 of
// the paper: reorder and dynamic quantisation fused into the operator before the GEMM; here also
// the re-tiling the packed GEMM wants, so that no pass over the codes stands between front end
// and GEMM).  Same row routine as the stand-alone front end (atom_quantize_rows.h, PACKED): the
// image is byte for byte what the canonical front end followed by the re-tiling pass produces.
//
// Compile WITHOUT fast-math (see atom_quantize_rows.h).

#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include <stdint.h>

#include "atom_internal.h"
#include "atom_launch.h"
#include "atom_quantize_rows.h"

namespace {

using namespace atom_quantize_rows;

template <bool NORM, int NS, int NT, int PRE, bool IDENT>
__global__ __launch_bounds__(NT)
void quantize_rows_packed_kernel(const __half *x, int64_t rows, int64_t ld, const __half *res, int64_t ldr,
                                 __half *sum_out, int64_t ldo, const __half *__restrict__ gamma, float eps,
                                 const int32_t *__restrict__ idx, int K, int O, int nbits, float clip,
                                 uint8_t *__restrict__ pk_out, unsigned pk_lds_off)
{
    extern __shared__ __align__(16) float lds[];
    uint8_t *pk_lds = reinterpret_cast<uint8_t *>(lds) + pk_lds_off;
    // A workgroup takes a run of consecutive rows, and consecutive runs go to workgroups of the same
    // XCD (the hardware deals workgroup ids round-robin to the 8 XCDs): the 16-byte pieces that the
    // rows r .. r+7 of a unit put into one 128-byte line then meet in one L2 instead of eight.
    const int64_t nb = gridDim.x, b = blockIdx.x;
    const int64_t per = nb >> 3, rem = nb & 7, xcd = b & 7;
    const int64_t logical = xcd * per + (xcd < rem ? xcd : rem) + (b >> 3);
    const int64_t rpw = (rows + nb - 1) / nb;
    const int64_t first = logical * rpw, last = first + rpw < rows ? first + rpw : rows;
    quantize_rows_fast_body<NORM, NS, NT, PRE, IDENT, true>(lds, first, 1, x, last, ld, res, ldr, sum_out,
                                                            ldo, gamma, eps, idx, K, O, nbits, clip, nullptr, nullptr,
                                                            nullptr, NoHook(), pk_out, pk_lds);
    // rows past the end of the matrix, up to the end of the last unit: zero codes, zero scales
    const int64_t end = (rows + 63) / 64 * 64;
    if (blockIdx.x == 0 && end > rows) {
        const int K4 = K - O, G4 = K4 >> 7, G8 = O >> 7;
        uint8_t *ubase = pk_out + (rows >> 6) * ((int64_t)G4 * kImg4 + (int64_t)G8 * kImg8);
        const int npad = (int)(end - rows), r0 = (int)(rows & 63);
        // per pad row: 6 chunks per INT4 group, 8 per INT8 group, one scale entry per group (as half a chunk)
        const int per_row = 6 * G4 + 8 * G8;
        for (int i = threadIdx.x; i < npad * per_row; i += NT) {
            const int r = r0 + i / per_row, j = i % per_row;
            uint8_t *dst;
            if (j < 6 * G4) {
                const int g = j / 6, hc = j % 6;
                dst = ubase + (int64_t)g * kImg4 + 2048 * (hc % 3) + 1024 * (hc / 3) + 16 * r;
            } else {
                const int j8 = j - 6 * G4;
                dst = ubase + (int64_t)G4 * kImg4 + (int64_t)(j8 >> 3) * kImg8 + 128 * r + 16 * (j8 & 7);
            }
            *reinterpret_cast<uint4 *>(dst) = make_uint4(0, 0, 0, 0);
        }
        for (int i = threadIdx.x; i < npad * (G4 + G8); i += NT) {
            const int r = r0 + i / (G4 + G8), g = i % (G4 + G8);
            uint8_t *dst = g < G4 ? ubase + (int64_t)g * kImg4 + kSc4 + 8 * r
                                  : ubase + (int64_t)G4 * kImg4 + (int64_t)(g - G4) * kImg8 + kSc8 + 8 * r;
            *reinterpret_cast<uint2 *>(dst) = make_uint2(0, 0);
        }
    }
}

struct PackedArgs {
    const void *x; int64_t rows, ld;
    const void *res; int64_t ldr; void *sum_out; int64_t ldo;
    const void *gamma; float eps; const int32_t *idx; int K, O, nbits; float clip;
    void *out;
};

template <bool NORM, int NS, int NT, int PRE, bool IDENT>
hipError_t launch_cfg(const PackedArgs &a, hipStream_t stream)
{
    auto kern = &quantize_rows_packed_kernel<NORM, NS, NT, PRE, IDENT>;
    const size_t front = sizeof(float) * (size_t)((IDENT ? 0 : a.K) + (NORM ? a.K / 8 : 0));
    const size_t lds = front + 3 * (size_t)((a.K - a.O) / 4) + (size_t)a.O;
    static atom_launch::LdsOptIn opt_in;
    hipError_t err = atom_launch::ensure_dynamic_lds(opt_in, reinterpret_cast<const void *>(kern), lds);
    if (err != hipSuccess) return err;
    const int cus = atom_launch::compute_units();
    int64_t per_cu = (int64_t)(160 * 1024) / (int64_t)(lds > 0 ? lds : 1);
    const int64_t by_waves = 2048 / NT;
    per_cu = per_cu < 1 ? 1 : (per_cu > by_waves ? by_waves : per_cu);
    const int64_t slots = (int64_t)cus * per_cu;
    const int64_t rows_per_wg = (a.rows + slots - 1) / slots;
    const int64_t grid = (a.rows + rows_per_wg - 1) / rows_per_wg;
    hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(NT), lds, stream, (const __half *)a.x, a.rows, a.ld,
                       (const __half *)a.res, a.ldr, (__half *)a.sum_out, a.ldo, (const __half *)a.gamma, a.eps, a.idx,
                       a.K, a.O, a.nbits, a.clip, (uint8_t *)a.out, (unsigned)front);
    return hipGetLastError();
}

template <bool NORM, int PRE, bool IDENT>
hipError_t dispatch_k(const PackedArgs &a, hipStream_t stream)
{
    if (a.K <= 2048)  return launch_cfg<NORM, 1, 256, PRE, IDENT>(a, stream);
    if (a.K <= 4096)  return launch_cfg<NORM, 2, 256, PRE, IDENT>(a, stream);
    if (a.K <= 8192)  return launch_cfg<NORM, 2, 512, PRE, IDENT>(a, stream);
    if (a.K <= 12288) return launch_cfg<NORM, 3, 512, PRE, IDENT>(a, stream);
    if (a.K <= 16384) return launch_cfg<NORM, 4, 512, PRE, IDENT>(a, stream);
    if (a.K <= 24576) return launch_cfg<NORM, 3, 1024, PRE, IDENT>(a, stream);
    return launch_cfg<NORM, 4, 1024, PRE, IDENT>(a, stream);
}

template <bool NORM, int PRE>
hipError_t dispatch_ident(const PackedArgs &a, hipStream_t stream)
{
    return a.idx ? dispatch_k<NORM, PRE, false>(a, stream) : dispatch_k<NORM, PRE, true>(a, stream);
}

}  // namespace

namespace atom_internal {

// LDS bytes of the packed front end (above 160 KB: does not fit)
size_t quantize_packed_lds_bytes(int K, int O, bool norm, bool ident)
{
    return sizeof(float) * (size_t)((ident ? 0 : K) + (norm ? K / 8 : 0)) + 3 * (size_t)((K - O) / 4) + (size_t)O;
}

hipError_t launch_quantize_rows_packed(const void *x, int64_t rows, int64_t ld, int pre, const void *res, int64_t ldr,
                                       void *sum_out, int64_t ldo, const void *gamma, float eps, const int32_t *idx,
                                       int K, int O, int nbits, float clip, void *out, hipStream_t stream)
{
    const PackedArgs a = {x, rows, ld, res, ldr, sum_out, ldo, gamma, eps, idx, K, O, nbits, clip, out};
    const bool norm = gamma != nullptr;
    if (pre == kSwiglu) return dispatch_ident<false, kSwiglu>(a, stream);
    if (pre == kAdd) return norm ? dispatch_ident<true, kAdd>(a, stream) : dispatch_ident<false, kAdd>(a, stream);
    return norm ? dispatch_ident<true, kPlain>(a, stream) : dispatch_ident<false, kPlain>(a, stream);
}

}  // namespace atom_internal
