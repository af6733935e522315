// Stand-alone caller of the C ABI (include/vp.h): no Python, no PyTorch.  Device memory comes from
// hipMalloc, the index and the workspace live in buffers this program owns.
//
//   vp_cli <input file> <output file>
//
// Input file (little endian): int32 d, V, K, N, k; then fp16 W[d*V], b[V], C[K*d]; int64 off[K+1];
// int32 ids[off[K]]; fp16 H[N*d].  Output file: int32 ids[N*k], fp32 logp[N*k], int32 cluster[N] of
// vp_project, then int32 ids[N*k], fp32 logp[N*k] of vp_project_full.
#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "vp.h"

#define HIP_OK(call)                                                                     \
    do {                                                                                 \
        hipError_t e_ = (call);                                                          \
        if (e_ != hipSuccess) {                                                          \
            std::fprintf(stderr, "%s: %s\n", #call, hipGetErrorString(e_));              \
            return 2;                                                                    \
        }                                                                                \
    } while (0)
#define VP_OK_OR_DIE(call)                                                               \
    do {                                                                                 \
        vp_status s_ = (call);                                                           \
        if (s_ != VP_OK) {                                                               \
            std::fprintf(stderr, "%s: status %d: %s\n", #call, (int)s_, vp_last_error()); \
            return 3;                                                                    \
        }                                                                                \
    } while (0)

template <typename T>
static bool read_vec(FILE *f, std::vector<T> &v, size_t n)
{
    v.resize(n);
    return n == 0 || std::fread(v.data(), sizeof(T), n, f) == n;
}

template <typename T>
static int to_device(const std::vector<T> &h, void **dptr)
{
    HIP_OK(hipMalloc(dptr, h.size() * sizeof(T) + 16));
    HIP_OK(hipMemcpy(*dptr, h.data(), h.size() * sizeof(T), hipMemcpyHostToDevice));
    return 0;
}

int main(int argc, char **argv)
{
    if (argc != 3) {
        std::fprintf(stderr, "usage: %s <input> <output>\n", argv[0]);
        return 1;
    }
    FILE *f = std::fopen(argv[1], "rb");
    if (!f) return 1;
    int32_t hdr[5];
    if (std::fread(hdr, 4, 5, f) != 5) return 1;
    const int d = hdr[0], V = hdr[1], K = hdr[2], N = hdr[3], k = hdr[4];
    std::vector<uint16_t> W, b, C, H;
    std::vector<int64_t> off;
    std::vector<int32_t> ids;
    if (!read_vec(f, W, (size_t)d * V) || !read_vec(f, b, (size_t)V) || !read_vec(f, C, (size_t)K * d) ||
        !read_vec(f, off, (size_t)K + 1) || !read_vec(f, ids, (size_t)off[K]) || !read_vec(f, H, (size_t)N * d))
        return 1;
    std::fclose(f);

    void *dW, *db, *dC, *dH;
    if (to_device(W, &dW) || to_device(b, &db) || to_device(C, &dC) || to_device(H, &dH)) return 2;

    vp_build_desc desc = {};
    desc.d = d;
    desc.V = V;
    desc.K = K;
    desc.W = dW;
    desc.bias = db;
    desc.centroids = dC;
    desc.cand_offsets = off.data();
    desc.cand_ids = ids.data();
    desc.k_max = k;
    const size_t arena_bytes = vp_build_bytes(&desc);
    if (!arena_bytes) {
        std::fprintf(stderr, "vp_build_bytes: %s\n", vp_last_error());
        return 3;
    }
    void *arena;
    HIP_OK(hipMalloc(&arena, arena_bytes));
    desc.arena = arena;
    desc.arena_bytes = arena_bytes;
    hipStream_t st;
    HIP_OK(hipStreamCreate(&st));
    vp_index *index = nullptr;
    VP_OK_OR_DIE(vp_build(&desc, st, &index));
    // the index keeps its own packed copies: the inputs may go
    HIP_OK(hipFree(dW));
    HIP_OK(hipFree(db));
    HIP_OK(hipFree(dC));

    const size_t ws_bytes = vp_workspace_bytes(index, N);
    void *ws, *o_ids, *o_logp, *o_g, *f_ids, *f_logp;
    HIP_OK(hipMalloc(&ws, ws_bytes));
    HIP_OK(hipMalloc(&o_ids, (size_t)N * k * 4 + 16));
    HIP_OK(hipMalloc(&o_logp, (size_t)N * k * 4 + 16));
    HIP_OK(hipMalloc(&o_g, (size_t)N * 4 + 16));
    HIP_OK(hipMalloc(&f_ids, (size_t)N * k * 4 + 16));
    HIP_OK(hipMalloc(&f_logp, (size_t)N * k * 4 + 16));
    VP_OK_OR_DIE(vp_project(index, dH, N, k, (int32_t *)o_ids, (float *)o_logp, (int32_t *)o_g, ws, ws_bytes, st));
    std::vector<int32_t> h_ids((size_t)N * k), h_g(N), hf_ids((size_t)N * k);
    std::vector<float> h_logp((size_t)N * k), hf_logp((size_t)N * k);
    HIP_OK(hipMemcpyAsync(h_ids.data(), o_ids, h_ids.size() * 4, hipMemcpyDeviceToHost, st));
    HIP_OK(hipMemcpyAsync(h_logp.data(), o_logp, h_logp.size() * 4, hipMemcpyDeviceToHost, st));
    HIP_OK(hipMemcpyAsync(h_g.data(), o_g, h_g.size() * 4, hipMemcpyDeviceToHost, st));
    VP_OK_OR_DIE(vp_project_full(index, dH, N, k, (int32_t *)f_ids, (float *)f_logp, ws, ws_bytes, st));
    HIP_OK(hipMemcpyAsync(hf_ids.data(), f_ids, hf_ids.size() * 4, hipMemcpyDeviceToHost, st));
    HIP_OK(hipMemcpyAsync(hf_logp.data(), f_logp, hf_logp.size() * 4, hipMemcpyDeviceToHost, st));
    HIP_OK(hipStreamSynchronize(st));

    FILE *o = std::fopen(argv[2], "wb");
    if (!o) return 1;
    std::fwrite(h_ids.data(), 4, h_ids.size(), o);
    std::fwrite(h_logp.data(), 4, h_logp.size(), o);
    std::fwrite(h_g.data(), 4, h_g.size(), o);
    std::fwrite(hf_ids.data(), 4, hf_ids.size(), o);
    std::fwrite(hf_logp.data(), 4, hf_logp.size(), o);
    std::fclose(o);
    vp_index_info info;
    VP_OK_OR_DIE(vp_get_info(index, &info));
    std::printf("vp_cli: d %d V %d K %d N %d k %d, index %lld bytes, workspace %zu bytes\n", d, V, K, N, k,
                (long long)info.arena_bytes_used, ws_bytes);
    vp_destroy(index);
    return 0;
}
