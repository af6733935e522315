// Host side of the C ABI under AddressSanitizer: every check that runs before any GPU work, with
// exactly sized host arrays (the candidate lists are the only host memory the library reads).
// Built by tests/test_sanitizers.py against the library's API files compiled with
// -Xarch_host -fsanitize=address; needs no GPU.
#include <cstdint>
#include <cstdio>
#include <cstring>
#include <vector>

#include "vp.h"

#define CHECK(c)                                                           \
    do {                                                                   \
        if (!(c)) {                                                        \
            std::fprintf(stderr, "check failed: %s (line %d), last error: %s\n", #c, __LINE__, vp_last_error()); \
            return 1;                                                      \
        }                                                                  \
    } while (0)

int main()
{
    const int d = 64, V = 1000, K = 4;
    const int sizes[K] = {10, 0, 333, 1000};
    int64_t *off = new int64_t[K + 1];
    off[0] = 0;
    for (int j = 0; j < K; ++j) off[j + 1] = off[j] + sizes[j];
    int32_t *ids = new int32_t[off[K]];
    for (int j = 0; j < K; ++j)
        for (int c = 0; c < sizes[j]; ++c) ids[off[j] + c] = (int32_t)((int64_t)c * V / sizes[j]);

    vp_build_desc D;
    std::memset(&D, 0, sizeof(D));
    D.d = d;
    D.V = V;
    D.K = K;
    D.cand_offsets = off;
    D.cand_ids = ids;
    D.k_max = 8;
    const size_t need = vp_build_bytes(&D);
    CHECK(need > 0);
    vp_index *idx = reinterpret_cast<vp_index *>(1);
    // the id lists are scanned in full, then the null device pointers are refused before any GPU call
    CHECK(vp_build(&D, nullptr, &idx) == VP_ERR_INVALID_ARG && idx == nullptr);
    CHECK(std::strstr(vp_last_error(), "null") != nullptr);
    CHECK(vp_build(&D, nullptr, nullptr) == VP_ERR_INVALID_ARG);
    CHECK(vp_build(nullptr, nullptr, &idx) == VP_ERR_INVALID_ARG);
    CHECK(vp_build_bytes(nullptr) == 0);

    // descriptions the host must refuse
    ids[off[2] + 5] = ids[off[2] + 4];                  // a duplicate id
    CHECK(vp_build(&D, nullptr, &idx) == VP_ERR_INVALID_ARG);
    ids[off[2] + 5] = (int32_t)((int64_t)5 * V / sizes[2]);
    ids[off[3] - 1] = V;                                // out of range (last entry of cluster 2)
    CHECK(vp_build(&D, nullptr, &idx) == VP_ERR_INVALID_ARG);
    ids[off[3] - 1] = (int32_t)((int64_t)(sizes[2] - 1) * V / sizes[2]);
    ids[0] = -1;
    CHECK(vp_build(&D, nullptr, &idx) == VP_ERR_INVALID_ARG);
    ids[0] = 0;
    off[2] = off[1] - 1;                                // offsets decrease
    CHECK(vp_build_bytes(&D) == 0);
    off[2] = off[1];
    off[0] = 1;
    CHECK(vp_build_bytes(&D) == 0);
    off[0] = 0;
    CHECK(vp_build_bytes(&D) == need);
    const vp_build_desc good = D;
    D.d = 60;
    CHECK(vp_build_bytes(&D) == 0);
    D = good;
    D.k_max = VP_MAX_TOPK + 1;
    CHECK(vp_build_bytes(&D) == 0);
    D = good;
    D.K = 0;
    CHECK(vp_build_bytes(&D) == 0);
    D = good;
    D.flags = 2;   // an unknown flag bit
    CHECK(vp_build_bytes(&D) == 0);
    D = good;
    D.cand_ids = nullptr;
    CHECK(vp_build_bytes(&D) == 0);

    // calls without an index
    vp_index_info info;
    CHECK(vp_get_info(nullptr, &info) == VP_ERR_INVALID_ARG);
    CHECK(vp_set_option(nullptr, "dispatch", 1) == VP_ERR_INVALID_ARG);
    CHECK(vp_workspace_bytes(nullptr, 16) == 0 && vp_union_workspace_bytes(nullptr, 16) == 0);
    CHECK(vp_project(nullptr, nullptr, 1, 1, nullptr, nullptr, nullptr, nullptr, 0, nullptr) == VP_ERR_INVALID_ARG);
    CHECK(vp_project_full(nullptr, nullptr, 1, 1, nullptr, nullptr, nullptr, 0, nullptr) == VP_ERR_INVALID_ARG);
    CHECK(vp_project_union(nullptr, nullptr, 1, 1, nullptr, nullptr, nullptr, nullptr, nullptr, 0, nullptr) ==
          VP_ERR_INVALID_ARG);
    CHECK(vp_project_debug_logits(nullptr, nullptr, 1, 0, nullptr, nullptr, nullptr, 0, nullptr, 0, nullptr) ==
          VP_ERR_INVALID_ARG);
    double ms;
    int64_t launches;
    CHECK(vp_get_profile(nullptr, &ms, &launches) == VP_ERR_INVALID_ARG);
    vp_destroy(nullptr);

    // training and search: argument errors found on the host
    CHECK(vp_kmeans_workspace_bytes(1000, 64, 10) > 0 && vp_kmeans_workspace_bytes(0, 64, 10) == 0);
    CHECK(vp_kmeans(nullptr, 1000, 64, 10, 5, 0, nullptr, nullptr, nullptr, nullptr, 0, nullptr) != VP_OK);
    CHECK(vp_kmeans(nullptr, 1000, 64, 10, 5, 2u, nullptr, nullptr, nullptr, nullptr, 0, nullptr) != VP_OK);
    CHECK(vp_active_sets_workspace_bytes(10, 1000) > 0);
    int64_t total = -1;
    CHECK(vp_active_sets(nullptr, nullptr, 100, 3, 10, 1000, nullptr, nullptr, 0, &total, nullptr, 0, nullptr) != VP_OK);
    CHECK(vp_beam_step(nullptr, nullptr, nullptr, 1, 4, 8, nullptr, nullptr, nullptr, nullptr) == VP_ERR_INVALID_ARG);
    CHECK(vp_beam_step(nullptr, nullptr, nullptr, 1, 4096, 8, nullptr, nullptr, nullptr, nullptr) == VP_ERR_UNSUPPORTED);
    CHECK(vp_beam_step(nullptr, nullptr, nullptr, 0, 4, 8, nullptr, nullptr, nullptr, nullptr) == VP_OK);
    CHECK(vp_round_to_half(1.0) == 0x3c00 && vp_round_to_half(-2.0) == 0xc000);

    delete[] off;
    delete[] ids;
    std::puts("boundary sanitizer run ok");
    return 0;
}
