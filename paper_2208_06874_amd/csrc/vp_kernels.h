// Host-callable launchers of the HIP kernels (internal to the library).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>
#include "vp_layout.h"

// index building
void vpk_pack_w(const void *W, int d, int V, int kt, void *out, hipStream_t st);
void vpk_token_major(const void *wp, int V, int kt, void *wt, hipStream_t st);
void vpk_pack_rows(const void *M, int rows, int d, int kt, void *out, hipStream_t st);
void vpk_cnorm(const void *C, int K, int d, int K_pad, float *cnorm, hipStream_t st);
void vpk_bias_full(const void *b, int V, int V_pad, float *out, hipStream_t st);
void vpk_gather_slabs(const void *wp, const void *b, int kt, const int32_t *ids_pad, long total_groups,
                      void *slabs, float *sbias, hipStream_t st);

void vpk_bitmaps(const int32_t *ids_pad, const int32_t *tile_off, int K, long total_groups, int words,
                 uint32_t *bitmaps, hipStream_t st);

// centroid selection (Eq. 2)
void vpk_centroid(const void *hidden, int N, int d, const void *cp, const float *cnorm, int K, int kt,
                  int ctiles, int tiles_per_part, int parts, void *cpart, hipStream_t st);

void vpk_centroid_small(const void *hidden, int N, int d, const void *cp, const float *cnorm, int K, int kt,
                        int ctiles, void *cpart, hipStream_t st);

// bucketing + planning
size_t vpk_plan_lds_bytes(int K);
hipError_t vpk_plan_prepare();
void vpk_plan(const void *cpart, int parts, int N, int K, const int32_t *n_cand, const int32_t *tile_off,
              int target_items, int min_items, int max_items, int32_t *g, int32_t *out_cluster, int32_t *perm,
              VpRowPlan *rowplan, unsigned int *floors, VpItem *items, VpPlanHeader *hdr, int64_t *dbg_row_off,
              int dispatch, const VpCostModel &cost, int k, int V, int vtiles, int full_target_items,
              int full_min_items, int max_items_full, hipStream_t st);
void vpk_plan_full(int N, int V, int vtiles, int rpi, int target_items, int min_items, int max_items, int32_t *perm,
                   VpRowPlan *rowplan, unsigned int *floors, VpItem *items, VpPlanHeader *hdr,
                   int64_t *dbg_row_off, hipStream_t st);

// projection + fused log-softmax / top-k partials
size_t vpk_project_lds_bytes(int kt, int k, int row_tiles);
hipError_t vpk_project_prepare();
void vpk_project(const VpSlabSet &set, const void *hidden, int d, const int32_t *perm, const VpItem *items,
                 const VpPlanHeader *hdr, int grid_items, int row_tiles, int k, int rstar, float *partials,
                 unsigned int *floors, float *dbg_logits, const int64_t *dbg_row_off, int raw_ok, hipStream_t st);

void vpk_project_small(const VpSlabSet &set, const void *hidden, int d, const VpSmallArgs &a, int grid_items, int k,
                       int rstar, float *partials, int raw_ok, int pf, hipStream_t st);

void vpk_project_masked(const VpSlabSet &full, const void *hidden, int d, const int32_t *perm, const VpItem *items,
                        const VpPlanHeader *hdr, int grid_items, int k, float *partials, unsigned int *floors,
                        const VpMaskInfo &mask, hipStream_t st);

// GEMM-shaped projection of single-bucket plans with 64 rows per item (mask: nullptr, or the
// membership lists of the masked full projection)
size_t vpk_project_gemm_lds_bytes(int k, int kt);
bool vpk_project_gemm_supported(int kt);
hipError_t vpk_project_gemm_prepare();
void vpk_project_gemm(const VpSlabSet &set, const void *hidden, int d, const int32_t *perm, const VpItem *items,
                      const VpPlanHeader *hdr, int grid_items, int k, float *partials, unsigned int *bounds,
                      const VpMaskInfo *mask, hipStream_t st);

// the same with the 64 rows of an item held in LDS (d_pad <= 1024, k <= 8); floors: [N] per-row bounds
size_t vpk_project_rows_lds_bytes(int k, int kt);
bool vpk_project_rows_lds_supported(int kt, int k);
int vpk_project_rows_lds_row_tiles(int kt);
hipError_t vpk_project_rows_lds_prepare();
void vpk_project_rows_lds(const VpSlabSet &set, const void *hidden, int d, const int32_t *perm, const VpItem *items,
                          const VpPlanHeader *hdr, int grid_items, int k, float *partials, unsigned int *floors,
                          const VpMaskInfo *mask, bool gather, hipStream_t st);

// per-row merge
size_t vpk_merge_lds_bytes(int k);
hipError_t vpk_merge_prepare();
void vpk_merge(const VpSlabSet &set, const VpRowPlan *rowplan, const VpPlanHeader *hdr, const float *partials, int k, int N,
               int32_t *out_ids, float *out_logp, hipStream_t st);

// the paper's batch-union form
hipError_t vpk_union_prepare();
void vpk_union_mark(const void *cpart, int parts, int N, int K, const uint32_t *bitmaps, int bm_words, int mask_words,
                    int32_t *g, int32_t *out_cluster, int32_t *zero_g, unsigned int *mask, int32_t *bsum,
                    hipStream_t st);
int vpk_union_blocks(int mask_words);
void vpk_union_compact(const unsigned int *mask, int mask_words, const int32_t *bsum, int N, int rpi, int target_items,
                       int min_items, int max_items, int32_t *uids, VpUnionHeader *uh, int32_t *out_union_size,
                       int32_t *perm, VpRowPlan *rowplan, unsigned int *floors, VpItem *items, VpPlanHeader *hdr,
                       int allow_full, int V, int vtiles, int k, const VpCostModel &cost, int max_items_full,
                       const float *bias_full, float *ubias, hipStream_t st);
void vpk_union_gather(const void *wt, int kt, const int32_t *uids, const VpUnionHeader *uh, int max_groups, void *slab,
                      hipStream_t st);

// offline training of the clusters (section 2.2)
void vpk_fill_u32(void *p, size_t n, uint32_t v, hipStream_t st);
void vpk_kmeans_assign(const void *cpart, int parts, int rows, int K, int32_t *assign, int32_t *counts,
                       hipStream_t st);
bool vpk_kmeans_assign_gemm(const void *X, long n, int d, const void *cp, const float *cnorm, int K, int kt, int ctiles,
                            int32_t *assign, int32_t *counts, hipStream_t st);
void vpk_kmeans_bucket(const int32_t *assign, long n, const int32_t *counts, int K, int32_t *start, int32_t *cursor,
                       int32_t *perm, hipStream_t st);
void vpk_kmeans_update(const void *X, int d, const int32_t *perm, const int32_t *start, const int32_t *counts, int K,
                       int splits, void *acc, void *C, hipStream_t st);
void vpk_kmeans_split(const int32_t *counts, int K, int d, void *C, hipStream_t st);
void vpk_aset_flags(const int32_t *top, const int32_t *assign, long n, int T, int K, int V, int words,
                    uint32_t *bitmaps, int32_t *sizes, int64_t *cand_off, hipStream_t st);
void vpk_aset_emit(const uint32_t *bitmaps, int words, int K, const int64_t *cand_off, int32_t *cand_ids,
                   hipStream_t st);

// measured ceilings (benchmark aid)
size_t vpk_ceiling_read(const void *buf, size_t bytes, int cus, void *sink, hipStream_t st);
double vpk_ceiling_mfma(int iters, int cus, void *sink, hipStream_t st);

// error message of the calling thread (shared by the translation units of the host API)
int vpi_fail(int status, const char *fmt, ...);
uint16_t vpk_round_to_half(double v);
