// Centroid selection, Eq. 2 of section 2.3:
//     g[r] = argmin_j ( ||C_j||^2 - 2 <h_r, C_j> ),  ties to the lowest j,
// with ||C_j||^2 precomputed at build time.  The inner products of 16 rows
// with 16 centroids are one v_mfma_f32_16x16x32_f16 per 32 k-values; every
// lane then holds 4 scores of one row, keeps a running (min, argmin), the
// four lane groups of the wavefront are reduced with cross-lane shuffles and
// the four wavefronts of the workgroup through LDS.  The centroids are split
// into `parts` ranges handled by different workgroups so that small batches
// still fill the chip; whoever needs the clusters next (the planning kernel, or the
// projection workgroups themselves for batches of a few rows) reduces the per-part minima.
#include <hip/hip_runtime.h>
#include "vp_kernels.h"

namespace {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef float floatx4 __attribute__((ext_vector_type(4)));

union Frag {
    uint4 u;
    half8 h;
};

constexpr int CU = 8;   // k-tiles fetched together (k-tile counts are multiples of 8)

__device__ inline bool score_less(float s, int j, float s2, int j2)
{
    return (s < s2) | ((s == s2) & (j < j2));   // (no short-circuit: compares and selects, no branches)
}

__global__ __launch_bounds__(256) void centroid_kernel(
    const uint4 *__restrict__ hidden, int N, int d, const uint4 *__restrict__ cp,
    const float *__restrict__ cnorm, int K, int kt_count, int ctiles, int tiles_per_wave, int parts,
    int2 *__restrict__ cpart)
{
    const int wave = threadIdx.x >> 6;
    const int lane = threadIdx.x & 63;
    const int n = lane & 15;
    const int q = lane >> 4;
    const int part = blockIdx.y;
    const int row = blockIdx.x * 16 + n;
    const bool valid_row = row < N;
    const int t0 = (part * 4 + wave) * tiles_per_wave;
    const int t1 = min(t0 + tiles_per_wave, ctiles);
    const int pieces_per_row = d >> 3;   // 16-byte pieces
    const uint4 *hrow = hidden + (size_t)(valid_row ? row : 0) * pieces_per_row;

    float best_s = __builtin_inff();
    int best_j = VP_IDX_NONE;
    for (int t = t0; t < t1; ++t) {
        floatx4 acc = {0.f, 0.f, 0.f, 0.f};
        const uint4 *ap = cp + (size_t)t * kt_count * 64 + lane;
        for (int kt0 = 0; kt0 < kt_count; kt0 += CU) {
            Frag a[CU], b[CU];
#pragma unroll
            for (int u = 0; u < CU; ++u) {
                a[u].u = ap[(size_t)(kt0 + u) * 64];
                const int piece = (kt0 + u) * 4 + q;
                b[u].u = make_uint4(0, 0, 0, 0);
                if (valid_row && piece < pieces_per_row) b[u].u = hrow[piece];
            }
#pragma unroll
            for (int u = 0; u < CU; ++u) acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(a[u].h, b[u].h, acc, 0, 0, 0);
        }
        const float4 cn = *reinterpret_cast<const float4 *>(cnorm + t * 16 + q * 4);
        const float cnv[4] = {cn.x, cn.y, cn.z, cn.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int j = t * 16 + q * 4 + i;
            const float s = cnv[i] - 2.0f * acc[i];
            if (j < K && s < best_s) {   // j ascends within a lane: strict < keeps the lowest
                best_s = s;
                best_j = j;
            }
        }
    }
#pragma unroll
    for (int off = 16; off <= 32; off <<= 1) {
        const float s2 = __shfl_xor(best_s, off);
        const int j2 = __shfl_xor(best_j, off);
        const bool take = score_less(s2, j2, best_s, best_j);
        best_s = take ? s2 : best_s;
        best_j = take ? j2 : best_j;
    }
    __shared__ float ws[4][16];
    __shared__ int wj[4][16];
    if (q == 0) {
        ws[wave][n] = best_s;
        wj[wave][n] = best_j;
    }
    __syncthreads();
    if (wave == 0 && q == 0 && valid_row) {
#pragma unroll
        for (int w = 1; w < 4; ++w) {
            const bool take = score_less(ws[w][n], wj[w][n], best_s, best_j);
            best_s = take ? ws[w][n] : best_s;
            best_j = take ? wj[w][n] : best_j;
        }
        cpart[(size_t)row * parts + part] = make_int2(__float_as_int(best_s), best_j);
    }
}

// The same for small and medium batches, where the time is one memory latency after the
// other rather than bytes: one workgroup per (tile of 16 centroids, tile of 16 rows), the k-extent split over its
// four wavefronts, so that every wavefront has all of its loads in flight at once (a quarter of
// the tile's k-tiles, and the matching pieces of the rows); the four partial products meet in
// LDS and are added in a fixed order.  cpart then holds one minimum per tile: parts = ctiles.
__global__ __launch_bounds__(256) void centroid_small_kernel(
    const uint4 *__restrict__ hidden, int N, int d, const uint4 *__restrict__ cp,
    const float *__restrict__ cnorm, int K, int kt_count, int2 *__restrict__ cpart)
{
    const int wave = threadIdx.x >> 6;
    const int lane = threadIdx.x & 63;
    const int n = lane & 15;
    const int q = lane >> 4;
    const int t = blockIdx.x;
    const int parts = gridDim.x;
    const int row = blockIdx.y * 16 + n;
    const bool valid_row = row < N;
    const int pieces_per_row = d >> 3;
    const uint4 *hrow = hidden + (size_t)(valid_row ? row : 0) * pieces_per_row;
    const int kq = kt_count >> 2;            // k-tiles per wavefront (k-tile counts are multiples of 8)
    const int k0 = wave * kq;
    const uint4 *ap = cp + ((size_t)t * kt_count + k0) * 64 + lane;

    floatx4 acc = {0.f, 0.f, 0.f, 0.f};
    for (int kk = 0; kk < kq; kk += CU) {
        Frag a[CU], b[CU];
#pragma unroll
        for (int u = 0; u < CU; ++u) {
            a[u].u = make_uint4(0, 0, 0, 0);
            b[u].u = make_uint4(0, 0, 0, 0);
            if (kk + u < kq) {
                a[u].u = ap[(size_t)(kk + u) * 64];
                const int piece = (k0 + kk + u) * 4 + q;
                if (valid_row && piece < pieces_per_row) b[u].u = hrow[piece];
            }
        }
#pragma unroll
        for (int u = 0; u < CU; ++u) acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(a[u].h, b[u].h, acc, 0, 0, 0);
    }
    __shared__ floatx4 part[4][64];
    part[wave][lane] = acc;
    __syncthreads();
    if (wave != 0) return;
    const floatx4 sum = (part[0][lane] + part[1][lane]) + (part[2][lane] + part[3][lane]);
    const float4 cn = *reinterpret_cast<const float4 *>(cnorm + t * 16 + q * 4);
    const float cnv[4] = {cn.x, cn.y, cn.z, cn.w};
    float best_s = __builtin_inff();
    int best_j = VP_IDX_NONE;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int j = t * 16 + q * 4 + i;
        const float s = cnv[i] - 2.0f * sum[i];
        if (j < K && s < best_s) {
            best_s = s;
            best_j = j;
        }
    }
#pragma unroll
    for (int off = 16; off <= 32; off <<= 1) {
        const float s2 = __shfl_xor(best_s, off);
        const int j2 = __shfl_xor(best_j, off);
        const bool take = score_less(s2, j2, best_s, best_j);
        best_s = take ? s2 : best_s;
        best_j = take ? j2 : best_j;
    }
    if (q == 0 && valid_row) cpart[(size_t)row * parts + t] = make_int2(__float_as_int(best_s), best_j);
}

}  // namespace

// One workgroup per (centroid tile, row tile), parts = ctiles (see above).
void vpk_centroid_small(const void *hidden, int N, int d, const void *cp, const float *cnorm, int K, int kt,
                        int ctiles, void *cpart, hipStream_t st)
{
    hipLaunchKernelGGL(centroid_small_kernel, dim3(ctiles, (N + 15) / 16), dim3(256), 0, st, (const uint4 *)hidden, N, d,
                       (const uint4 *)cp, cnorm, K, kt, (int2 *)cpart);
}

// parts: workgroups along the centroid axis; each of their 4 wavefronts takes tiles_per_wave tiles.
void vpk_centroid(const void *hidden, int N, int d, const void *cp, const float *cnorm, int K, int kt,
                  int ctiles, int tiles_per_wave, int parts, void *cpart, hipStream_t st)
{
    dim3 grid((N + 15) / 16, parts);
    hipLaunchKernelGGL(centroid_kernel, grid, dim3(256), 0, st, (const uint4 *)hidden, N, d, (const uint4 *)cp,
                       cnorm, K, kt, ctiles, tiles_per_wave, parts, (int2 *)cpart);
}
