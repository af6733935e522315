// Index-building kernels (run once by vp_build; not on the timed path).
//
// They re-tile W and the centroids into the packed operand layout described in
// vp_layout.h, precompute the squared centroid norms of Eq. 2 (section 2.3: the
// C_j^2 term is constant at inference time and kept in GPU memory), and gather
// each cluster's active-token columns (section 2.2) into its own slab.
#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include "vp_kernels.h"

namespace {

// W[d, V] row-major (one column per token) -> packed tiles of the whole
// vocabulary.  One wavefront per (token group, k-tile).
__global__ __launch_bounds__(64) void pack_w_kernel(const uint16_t *__restrict__ W, int d, int V,
                                                     int kt_count, uint4 *__restrict__ out)
{
    const int group = blockIdx.x;
    const int kt = blockIdx.y;
    const int lane = threadIdx.x;
    const int v = group * VP_TILE_ITEMS + (lane & 15);
    const int k0 = kt * VP_TILE_K + (lane >> 4) * 8;
    uint16_t h[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const int k = k0 + e;
        h[e] = (k < d && v < V) ? W[(size_t)k * V + v] : (uint16_t)0;
    }
    uint4 o;
    o.x = h[0] | ((uint32_t)h[1] << 16);
    o.y = h[2] | ((uint32_t)h[3] << 16);
    o.z = h[4] | ((uint32_t)h[5] << 16);
    o.w = h[6] | ((uint32_t)h[7] << 16);
    out[((size_t)group * kt_count + kt) * 64 + lane] = o;
}

// Packed tiles of the whole vocabulary -> one contiguous row of d_pad k-values per token (the
// transpose of the paper's W[d, V], zero padded): what a run-time gather of single columns reads.
__global__ __launch_bounds__(256) void token_major_kernel(const uint4 *__restrict__ wp, int V, int kt_count,
                                                          uint4 *__restrict__ wt)
{
    const int X = kt_count * 4;   // 16-byte pieces per token
    const size_t e = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (e >= (size_t)V * X) return;
    const int v = (int)(e / X);
    const int x = (int)(e - (size_t)v * X);
    wt[e] = wp[((size_t)(v >> 4) * kt_count + (x >> 2)) * 64 + (x & 3) * 16 + (v & 15)];
}

// M[rows, d] row-major (one row per item, e.g. the centroids) -> packed tiles.
__global__ __launch_bounds__(64) void pack_rows_kernel(const uint16_t *__restrict__ M, int rows, int d,
                                                        int kt_count, uint4 *__restrict__ out)
{
    const int group = blockIdx.x;
    const int kt = blockIdx.y;
    const int lane = threadIdx.x;
    const int j = group * VP_TILE_ITEMS + (lane & 15);
    const int k0 = kt * VP_TILE_K + (lane >> 4) * 8;
    uint4 o = make_uint4(0, 0, 0, 0);
    if (j < rows && k0 + 8 <= d)   // d % 8 == 0: a chunk of 8 is entirely inside or outside
        o = *reinterpret_cast<const uint4 *>(M + (size_t)j * d + k0);
    out[((size_t)group * kt_count + kt) * 64 + lane] = o;
}

// cnorm[j] = sum_i C[j, i]^2 in fp32 (padding entries +inf so they never win).
__global__ __launch_bounds__(64) void cnorm_kernel(const __half *__restrict__ C, int K, int d,
                                                    int K_pad, float *__restrict__ cnorm)
{
    const int j = blockIdx.x;
    const int lane = threadIdx.x;
    if (j >= K) {
        if (lane == 0 && j < K_pad) cnorm[j] = __builtin_inff();
        return;
    }
    float acc = 0.f;
    for (int i = lane; i < d; i += 64) {
        const float c = __half2float(C[(size_t)j * d + i]);
        acc += c * c;
    }
    for (int off = 32; off > 0; off >>= 1) acc += __shfl_xor(acc, off);
    if (lane == 0) cnorm[j] = acc;
}

// fp16 bias of the whole vocabulary -> fp32, zero padded.
__global__ void bias_full_kernel(const __half *__restrict__ b, int V, int V_pad,
                                 float *__restrict__ out)
{
    const int v = blockIdx.x * blockDim.x + threadIdx.x;
    if (v < V_pad) out[v] = v < V ? __half2float(b[v]) : 0.f;
}

// Gathers the slab of every cluster from the packed whole-W copy.  One
// workgroup per candidate group (16 candidates of one cluster); its 4
// wavefronts share the k-tiles.  ids_pad holds each cluster's ascending token
// ids padded with -1 to a multiple of 16 per cluster (same indexing as the
// slab's candidate groups).
__global__ __launch_bounds__(256) void gather_slab_kernel(
    const uint4 *__restrict__ wp, const __half *__restrict__ b, int kt_count,
    const int32_t *__restrict__ ids_pad, long total_groups, uint4 *__restrict__ slabs,
    float *__restrict__ sbias)
{
    const long group = blockIdx.x;
    if (group >= total_groups) return;
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int v = ids_pad[group * VP_TILE_ITEMS + (lane & 15)];
    if (threadIdx.x < 16) sbias[group * VP_TILE_ITEMS + lane] = v >= 0 ? __half2float(b[v]) : 0.f;
    const int q = lane >> 4;
    for (int kt = wave; kt < kt_count; kt += VP_WG_WAVES) {
        uint4 o = make_uint4(0, 0, 0, 0);
        if (v >= 0) o = wp[((size_t)(v >> 4) * kt_count + kt) * 64 + q * 16 + (v & 15)];
        slabs[((size_t)group * kt_count + kt) * 64 + lane] = o;
    }
}

// Membership bit lists: bit v of cluster j's list is set iff token v is in A_j (the
// list must be zero beforehand).  One workgroup of 16 threads' worth of work per group
// of 16 candidates; the cluster of a group is found by bisection of the tile offsets.
__global__ __launch_bounds__(64) void bitmap_kernel(const int32_t *__restrict__ ids_pad,
                                                    const int32_t *__restrict__ tile_off, int K, long total_groups,
                                                    int words, uint32_t *__restrict__ bitmaps)
{
    const long group = (long)blockIdx.x * 4 + (threadIdx.x >> 4);
    if (group >= total_groups) return;
    int lo = 0, hi = K;   // largest j with tile_off[j] <= group
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (tile_off[mid] <= group) lo = mid; else hi = mid;
    }
    const int v = ids_pad[group * VP_TILE_ITEMS + (threadIdx.x & 15)];
    if (v >= 0) atomicOr(&bitmaps[(size_t)lo * words + (v >> 5)], 1u << (v & 31));
}

}  // namespace

void vpk_bitmaps(const int32_t *ids_pad, const int32_t *tile_off, int K, long total_groups, int words,
                 uint32_t *bitmaps, hipStream_t st)
{
    hipLaunchKernelGGL(bitmap_kernel, dim3((unsigned)((total_groups + 3) / 4)), dim3(64), 0, st, ids_pad, tile_off, K,
                       total_groups, words, bitmaps);
}

void vpk_pack_w(const void *W, int d, int V, int kt, void *out, hipStream_t st)
{
    dim3 grid((V + VP_TILE_ITEMS - 1) / VP_TILE_ITEMS, kt);
    hipLaunchKernelGGL(pack_w_kernel, grid, dim3(64), 0, st, (const uint16_t *)W, d, V, kt, (uint4 *)out);
}

void vpk_token_major(const void *wp, int V, int kt, void *wt, hipStream_t st)
{
    const size_t pieces = (size_t)V * kt * 4;
    hipLaunchKernelGGL(token_major_kernel, dim3((unsigned)((pieces + 255) / 256)), dim3(256), 0, st, (const uint4 *)wp, V,
                       kt, (uint4 *)wt);
}

void vpk_pack_rows(const void *M, int rows, int d, int kt, void *out, hipStream_t st)
{
    dim3 grid((rows + VP_TILE_ITEMS - 1) / VP_TILE_ITEMS, kt);
    hipLaunchKernelGGL(pack_rows_kernel, grid, dim3(64), 0, st, (const uint16_t *)M, rows, d, kt, (uint4 *)out);
}

void vpk_cnorm(const void *C, int K, int d, int K_pad, float *cnorm, hipStream_t st)
{
    hipLaunchKernelGGL(cnorm_kernel, dim3(K_pad), dim3(64), 0, st, (const __half *)C, K, d, K_pad, cnorm);
}

void vpk_bias_full(const void *b, int V, int V_pad, float *out, hipStream_t st)
{
    hipLaunchKernelGGL(bias_full_kernel, dim3((V_pad + 255) / 256), dim3(256), 0, st, (const __half *)b, V, V_pad, out);
}

void vpk_gather_slabs(const void *wp, const void *b, int kt, const int32_t *ids_pad, long total_groups,
                      void *slabs, float *sbias, hipStream_t st)
{
    // grid.x is limited to 2^31-1 workgroups; total_groups is checked by the caller
    hipLaunchKernelGGL(gather_slab_kernel, dim3((unsigned)total_groups), dim3(256), 0, st, (const uint4 *)wp,
                       (const __half *)b, kt, ids_pad, total_groups, (uint4 *)slabs, sbias);
}
