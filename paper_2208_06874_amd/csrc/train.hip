// Offline training of the clusters on the GPU (section 2.2 and the training
// settings of section 3.1): Lloyd k-means over recorded hidden vectors and the
// active set of each cluster as the union of its members' recorded tokens.
//
// Memberships are Eq. 2 (nearest centroid, ties to the lowest index), for many vectors as a
// GEMM.  The update is exact: every binary16 value is an integer multiple of 2^-24, so sums
// of members, kept in double precision while they stay below 2^29 in magnitude, or as 64-bit
// integers in that unit where the sums of different threads meet, are exact whatever the
// order of the additions (and of the atomics), and the mean sum / count is rounded once, in
// double precision, to binary16 (nearest, ties to even).  A cluster without members keeps its
// centroid.
#include <hip/hip_runtime.h>
#include "vp_kernels.h"
#include "project_common.h"

namespace {

__device__ inline bool part_less(float s, int j, float s2, int j2) { return s < s2 || (s == s2 && j < j2); }

// Finishes Eq. 2 for a chunk of rows (minimum over the centroid ranges) and counts the members.
__global__ __launch_bounds__(256) void kmeans_assign_kernel(const int2 *__restrict__ cpart, int parts, int rows,
                                                            int K, int32_t *__restrict__ assign,
                                                            int32_t *__restrict__ counts)
{
    const int r = blockIdx.x * 256 + threadIdx.x;
    if (r >= rows) return;
    float bs = __builtin_inff();
    int bj = VP_IDX_NONE;
    for (int p = 0; p < parts; ++p) {
        const int2 e = cpart[(size_t)r * parts + p];
        const float s = __int_as_float(e.x);
        if (part_less(s, e.y, bs, bj)) {
            bs = s;
            bj = e.y;
        }
    }
    if ((unsigned)bj >= (unsigned)K) bj = 0;   // only when every score is NaN: keep the index in range
    assign[r] = bj;
    atomicAdd(&counts[bj], 1);
}

// Membership of many vectors at once: Eq. 2 as a GEMM.  One workgroup takes 64 vectors and
// all centroids.  As in the GEMM-shaped projection kernel the k-extent is split over the four
// wavefronts, each keeping its slice of the 64 vectors in registers in MFMA operand order and
// streaming its slice of every packed centroid tile (the centroids stay in the caches), so
// each 1 KiB load feeds four MFMAs; the partial inner products of a group of 16 centroids meet
// in LDS and wavefront w keeps the running (min, argmin) of vector tile w.
template <int KW>
__global__ __launch_bounds__(256, (KW <= 8 ? 2 : 1)) void kmeans_assign_gemm_kernel(
    const uint4 *__restrict__ X, long n, int d, const uint4 *__restrict__ cp, const float *__restrict__ cnorm, int K,
    int ctiles, int32_t *__restrict__ assign, int32_t *__restrict__ counts)
{
    constexpr int KT = KW * 4;
    constexpr int RT = 4;
    const int wave = threadIdx.x >> 6;
    const int lane = threadIdx.x & 63;
    const int nn = lane & 15;
    const int q = lane >> 4;
    __shared__ floatx4 xbuf[2 * RT * 4 * 64];

    const uint4 *tiles = cp + (size_t)wave * KW * 64 + lane;
    Frag Xb[KW], Yb[KW];
    auto issue = [&](Frag(&buf)[KW], int g) {
        const uint4 *p = tiles + (size_t)g * KT * 64;
#pragma unroll
        for (int i = 0; i < KW; ++i) buf[i].u = p[i * 64];
    };
    issue(Xb, 0);
    if (1 < ctiles) issue(Yb, 1);

    const long r0 = (long)blockIdx.x * (16 * RT);
    const int pieces_per_row = d >> 3;
    Frag B[RT][KW];
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) {
        const long row = r0 + rt * 16 + nn;
#pragma unroll
        for (int i = 0; i < KW; ++i) {
            const int piece = (wave * KW + i) * 4 + q;
            B[rt][i].u = make_uint4(0, 0, 0, 0);
            if (row < n && piece < pieces_per_row) B[rt][i].u = X[(size_t)row * pieces_per_row + piece];
        }
    }

    float best_s = __builtin_inff();
    int best_j = VP_IDX_NONE;
    floatx4 acc[RT];
    auto compute = [&](Frag(&buf)[KW], int gnext) {
        const bool more = gnext < ctiles;
        const uint4 *p = tiles + (size_t)gnext * KT * 64;
#pragma unroll
        for (int i = 0; i < KW; ++i) {
            Frag a;
            a.u = buf[i].u;
            if (more) buf[i].u = p[i * 64];
#pragma unroll
            for (int rt = 0; rt < RT; ++rt)
                acc[rt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a.h, B[rt][i].h,
                                                                 i == 0 ? floatx4{0.f, 0.f, 0.f, 0.f} : acc[rt], 0, 0, 0);
        }
    };
    auto finish = [&](int g, int par) {
        floatx4 *xw = xbuf + (size_t)par * RT * 4 * 64;
#pragma unroll
        for (int rt = 0; rt < RT; ++rt) xw[(rt * 4 + wave) * 64 + lane] = acc[rt];
        const float4 cn = *reinterpret_cast<const float4 *>(cnorm + g * 16 + q * 4);
        __syncthreads();
        const floatx4 dot = (xw[(wave * 4 + 0) * 64 + lane] + xw[(wave * 4 + 1) * 64 + lane]) +
                            (xw[(wave * 4 + 2) * 64 + lane] + xw[(wave * 4 + 3) * 64 + lane]);
        const float cnv[4] = {cn.x, cn.y, cn.z, cn.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int j = g * 16 + q * 4 + i;
            const float s = cnv[i] - 2.0f * dot[i];
            if (j < K && s < best_s) {   // j ascends within a lane: strict < keeps the lowest
                best_s = s;
                best_j = j;
            }
        }
    };
    int g = 0, par = 0;
    while (g < ctiles) {
        compute(Xb, g + 2);
        finish(g, par);
        par ^= 1;
        ++g;
        if (g >= ctiles) break;
        compute(Yb, g + 2);
        finish(g, par);
        par ^= 1;
        ++g;
    }
#pragma unroll
    for (int off = 16; off <= 32; off <<= 1) {
        const float s2 = __shfl_xor(best_s, off);
        const int j2 = __shfl_xor(best_j, off);
        if (part_less(s2, j2, best_s, best_j)) {
            best_s = s2;
            best_j = j2;
        }
    }
    const long row = r0 + wave * 16 + nn;
    if (q == 0 && row < n) {
        if ((unsigned)best_j >= (unsigned)K) best_j = 0;   // only when every score is NaN
        assign[row] = best_j;
        atomicAdd(&counts[best_j], 1);
    }
}

// start[j] = number of members of clusters below j; cursor[j] = start[j].  One workgroup.
__global__ __launch_bounds__(1024) void kmeans_scan_kernel(const int32_t *__restrict__ counts, int K,
                                                           int32_t *__restrict__ start, int32_t *__restrict__ cursor)
{
    __shared__ int wsum[17];
    __shared__ int carry;
    if (threadIdx.x == 0) carry = 0;
    __syncthreads();
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (int base = 0; base < K; base += 1024) {
        const int j = base + threadIdx.x;
        const int v = j < K ? counts[j] : 0;
        int inc = v;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const int up = __shfl_up(inc, off);
            if (lane >= off) inc += up;
        }
        if (lane == 63) wsum[wave] = inc;
        __syncthreads();
        if (threadIdx.x == 0) {
            int run = carry;
            for (int w = 0; w < 16; ++w) {
                const int t = wsum[w];
                wsum[w] = run;
                run += t;
            }
            wsum[16] = run;
        }
        __syncthreads();
        if (j < K) {
            const int ex = wsum[wave] + inc - v;
            start[j] = ex;
            cursor[j] = ex;
        }
        __syncthreads();
        if (threadIdx.x == 0) carry = wsum[16];
        __syncthreads();
    }
    if (threadIdx.x == 0) start[K] = carry;
}

// Row numbers in cluster order (the order inside a cluster is arbitrary: the sums are exact).
__global__ __launch_bounds__(256) void kmeans_scatter_kernel(const int32_t *__restrict__ assign, long n,
                                                             int32_t *__restrict__ cursor, int32_t *__restrict__ perm)
{
    const long r = (long)blockIdx.x * 256 + threadIdx.x;
    if (r >= n) return;
    const int pos = atomicAdd(&cursor[assign[r]], 1);
    perm[pos] = (int32_t)r;
}

// Running sums of 8 coordinates.  They are kept in double precision: every binary16 value is
// a multiple of 2^-24, so while a sum stays below 2^29 in magnitude every addition is exact and
// the order of the additions does not matter.  Where sums of different threads meet they are
// added as 64-bit integers in units of 2^-24 (exact conversions), which keeps that true under
// atomics.
typedef _Float16 half2t __attribute__((ext_vector_type(2)));

__device__ inline void add_units(double (&s)[8], const uint4 v)
{
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const half2t h = __builtin_bit_cast(half2t, w[e]);
        s[2 * e] += (double)(float)h[0];
        s[2 * e + 1] += (double)(float)h[1];
    }
}

__device__ inline unsigned long long to_units(double sum) { return (unsigned long long)(long long)(sum * 0x1p24); }

// Sum of the members of cluster blockIdx.x that fall to this workgroup (every `splits`-th one
// starting at blockIdx.y).  A thread owns one 16-byte piece (8 coordinates) of the vectors; when
// a vector has fewer than 256 pieces the workgroup's threads form several member lanes that take
// the workgroup's members in turn.  Eight rows are in flight per thread.
__global__ __launch_bounds__(256) void kmeans_sum_kernel(const uint4 *__restrict__ X, int pieces,
                                                         const int32_t *__restrict__ perm,
                                                         const int32_t *__restrict__ start, int splits,
                                                         unsigned long long *__restrict__ acc)
{
    const int j = blockIdx.x;
    const int m0 = start[j], m1 = start[j + 1];
    const int lanes = pieces <= 128 ? 256 / pieces : 1;       // member lanes per workgroup
    const int ml = lanes > 1 ? threadIdx.x / pieces : 0;       // this thread's member lane
    __shared__ unsigned long long lsum[128 * 8];
    if (lanes > 1) {
        for (int e = threadIdx.x; e < pieces * 8; e += 256) lsum[e] = 0ull;
        __syncthreads();
    }
    const int step = splits * lanes;
    const int first = m0 + blockIdx.y * lanes + ml;
    for (int piece = lanes > 1 ? threadIdx.x - ml * pieces : threadIdx.x; piece < pieces && ml < lanes; piece += 256) {
        double s[8] = {0, 0, 0, 0, 0, 0, 0, 0};
        int m = first;
        for (; m + 7 * step < m1; m += 8 * step) {
            int r[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) r[u] = perm[m + u * step];
            uint4 v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) v[u] = X[(size_t)r[u] * pieces + piece];
#pragma unroll
            for (int u = 0; u < 8; ++u) add_units(s, v[u]);
        }
        for (; m < m1; m += step) add_units(s, X[(size_t)perm[m] * pieces + piece]);
        if (lanes > 1) {
            // the member lanes meet in LDS; one global addition per coordinate and workgroup
            unsigned long long *slot = lsum + (size_t)piece * 8;
#pragma unroll
            for (int e = 0; e < 8; ++e) atomicAdd(slot + e, to_units(s[e]));
        } else if (first < m1) {
#pragma unroll
            for (int e = 0; e < 8; ++e) atomicAdd(&acc[((size_t)j * pieces + piece) * 8 + e], to_units(s[e]));
        }
    }
    if (lanes > 1) {
        __syncthreads();
        if (m0 + (int)blockIdx.y * lanes < m1) {
            for (int e = threadIdx.x; e < pieces * 8; e += 256)
                atomicAdd(&acc[(size_t)j * pieces * 8 + e], lsum[e]);
        }
    }
}

// double -> binary16 bits, round to nearest, ties to even (integer arithmetic on the bits).
__host__ __device__ inline uint16_t double_to_half_bits(double v)
{
    unsigned long long b;
    __builtin_memcpy(&b, &v, sizeof(b));
    const uint16_t sign = (uint16_t)((b >> 48) & 0x8000);
    const int ex = (int)((b >> 52) & 0x7ff);
    const unsigned long long man = b & ((1ull << 52) - 1);
    if (ex == 0x7ff) return (uint16_t)(sign | (man ? 0x7e00 : 0x7c00));
    if (ex == 0) return sign;                                   // zero (and double subnormals)
    const int e = ex - 1023;
    if (e > 15) return (uint16_t)(sign | 0x7c00);
    unsigned long long q, rem, half;
    uint32_t base;
    if (e >= -14) {                                             // normal binary16 range
        q = man >> 42;
        rem = man & ((1ull << 42) - 1);
        half = 1ull << 41;
        base = (uint32_t)(e + 15) << 10;
    } else {                                                    // multiples of 2^-24
        const int shift = 28 - e;                               // >= 43
        if (shift > 63) return sign;
        const unsigned long long full = man | (1ull << 52);
        q = full >> shift;
        rem = full & ((1ull << shift) - 1);
        half = 1ull << (shift - 1);
        base = 0;
    }
    uint32_t h = base + (uint32_t)q;
    if (rem > half || (rem == half && (q & 1))) h += 1;        // a carry moves into the exponent field
    if (h >= 0x7c00) h = 0x7c00;
    return (uint16_t)(sign | h);
}

// One workgroup per cluster: sums all its members and writes the new centroid at once (no
// sums in memory, no atomics between workgroups).  Used when there are enough clusters to fill
// the chip this way; the member lanes of the workgroup meet in LDS.
__global__ __launch_bounds__(1024) void kmeans_mean_kernel(const uint4 *__restrict__ X, int pieces,
                                                          const int32_t *__restrict__ perm,
                                                          const int32_t *__restrict__ start, uint4 *__restrict__ C)
{
    const int j = blockIdx.x;
    const int m0 = start[j], m1 = start[j + 1];
    if (m0 == m1) return;                                      // no members: the centroid stays
    constexpr int T = 1024;                                   // threads per workgroup
    const int lanes = pieces <= T / 2 ? T / pieces : 1;       // member lanes
    const int ml = lanes > 1 ? threadIdx.x / pieces : 0;
    __shared__ unsigned long long lsum[(T / 2) * 8];
    if (lanes > 1) {
        for (int e = threadIdx.x; e < pieces * 8; e += T) lsum[e] = 0ull;
        __syncthreads();
    }
    const double inv_units = 0x1p-24;
    const double count = (double)(m1 - m0);
    for (int piece = lanes > 1 ? threadIdx.x - ml * pieces : threadIdx.x; piece < pieces && ml < lanes; piece += T) {
        double s[8] = {0, 0, 0, 0, 0, 0, 0, 0};
        int m = m0 + ml;
        for (; m + 7 * lanes < m1; m += 8 * lanes) {
            // row numbers first, then all eight rows: written as one expression the loads of a row
            // number and of its row alternate and every one waits for the one before
            int r[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) r[u] = perm[m + u * lanes];
            uint4 v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) v[u] = X[(size_t)r[u] * pieces + piece];
#pragma unroll
            for (int u = 0; u < 8; ++u) add_units(s, v[u]);
        }
        for (; m < m1; m += lanes) add_units(s, X[(size_t)perm[m] * pieces + piece]);
        if (lanes > 1) {
#pragma unroll
            for (int e = 0; e < 8; ++e) atomicAdd(lsum + (size_t)piece * 8 + e, to_units(s[e]));
        } else {
            uint32_t h[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) h[e] = double_to_half_bits(s[e] / count);
            C[(size_t)j * pieces + piece] = make_uint4(h[0] | (h[1] << 16), h[2] | (h[3] << 16), h[4] | (h[5] << 16),
                                                       h[6] | (h[7] << 16));
        }
    }
    if (lanes > 1) {
        __syncthreads();
        for (int piece = threadIdx.x; piece < pieces; piece += T) {
            uint32_t h[8];
#pragma unroll
            for (int e = 0; e < 8; ++e)
                h[e] = double_to_half_bits((double)(long long)lsum[piece * 8 + e] * inv_units / count);
            C[(size_t)j * pieces + piece] = make_uint4(h[0] | (h[1] << 16), h[2] | (h[3] << 16), h[4] | (h[5] << 16),
                                                       h[6] | (h[7] << 16));
        }
    }
}

// New centroids from the sums; the sums are cleared for the next iteration.
__global__ __launch_bounds__(256) void kmeans_update_kernel(unsigned long long *__restrict__ acc,
                                                            const int32_t *__restrict__ counts, int K, int d,
                                                            uint16_t *__restrict__ C)
{
    const size_t e = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (e >= (size_t)K * d) return;
    const int j = (int)(e / d);
    const int c = counts[j];
    if (c > 0) {
        const double sum = (double)(long long)acc[e];
        C[e] = double_to_half_bits(sum * 0x1p-24 / (double)c);
    }
    acc[e] = 0ull;
}

// binary16 bits -> double, exactly
__device__ inline double half_bits_to_double(uint32_t h)
{
    const _Float16 v = __builtin_bit_cast(_Float16, (unsigned short)h);
    return (double)(float)v;
}

// Optional remedy for clusters without members: in ascending order each takes the cluster that
// has the most members at that moment (ties: lowest index; at least two members), whose centroid
// c becomes c (1 - 2^-10) while c (1 + 2^-10) goes to the empty cluster; half of the members
// (rounded down) are counted for the new cluster.  One workgroup; cnt lives in LDS.
__global__ __launch_bounds__(1024) void kmeans_split_kernel(const int32_t *__restrict__ counts, int K, int d,
                                                            uint16_t *__restrict__ C)
{
    extern __shared__ int cnt[];   // [K]
    __shared__ int red_c[16], red_i[16];
    __shared__ int big_s, any_empty;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    if (tid == 0) any_empty = 0;
    __syncthreads();
    for (int j = tid; j < K; j += 1024) {
        cnt[j] = counts[j];
        if (cnt[j] == 0) any_empty = 1;
    }
    __syncthreads();
    if (!any_empty) return;
    const double eps = 0x1p-10;
    for (int j = 0; j < K; ++j) {
        if (cnt[j] != 0) continue;          // uniform: every thread reads the same LDS word
        int bc = -1, bi = 0x7fffffff;       // largest count, lowest index
        for (int i = tid; i < K; i += 1024) {
            if (cnt[i] > bc) {
                bc = cnt[i];
                bi = i;
            }
        }
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const int c2 = __shfl_xor(bc, off), i2 = __shfl_xor(bi, off);
            if (c2 > bc || (c2 == bc && i2 < bi)) {
                bc = c2;
                bi = i2;
            }
        }
        if (lane == 0) {
            red_c[wave] = bc;
            red_i[wave] = bi;
        }
        __syncthreads();
        if (tid == 0) {
            for (int w = 1; w < 16; ++w) {
                if (red_c[w] > bc || (red_c[w] == bc && red_i[w] < bi)) {
                    bc = red_c[w];
                    bi = red_i[w];
                }
            }
            big_s = bc >= 2 ? bi : -1;
        }
        __syncthreads();
        const int big = big_s;
        if (big < 0) return;                // nothing left to split (uniform)
        for (int e = tid; e < d; e += 1024) {
            const double c = half_bits_to_double(C[(size_t)big * d + e]);
            C[(size_t)j * d + e] = double_to_half_bits(c * (1.0 + eps));
            C[(size_t)big * d + e] = double_to_half_bits(c * (1.0 - eps));
        }
        __syncthreads();
        if (tid == 0) {
            const int c = cnt[big];
            cnt[j] = c / 2;
            cnt[big] = c - c / 2;
        }
        __syncthreads();
    }
}

__global__ void fill_u32_kernel(uint32_t *__restrict__ p, size_t n, uint32_t v)
{
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = v;
}

// ---------------------------------------------------------------- active sets
// bit v of cluster assign[r]'s list is set for every recorded token v of vector r
__global__ __launch_bounds__(256) void aset_flag_kernel(const int32_t *__restrict__ top,
                                                        const int32_t *__restrict__ assign, long n, int T, int K,
                                                        int V, int words, uint32_t *__restrict__ bitmaps)
{
    const long i = (long)blockIdx.x * 256 + threadIdx.x;
    if (i >= n * T) return;
    const int v = top[i];
    const int j = assign[i / T];
    if (v < 0 || v >= V || j < 0 || j >= K) return;
    atomicOr(&bitmaps[(size_t)j * words + (v >> 5)], 1u << (v & 31));
}

__device__ inline int block_sum_256(int v, int *lds)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) lds[threadIdx.x >> 6] = v;
    __syncthreads();
    return lds[0] + lds[1] + lds[2] + lds[3];
}

__global__ __launch_bounds__(256) void aset_count_kernel(const uint32_t *__restrict__ bitmaps, int words,
                                                         int32_t *__restrict__ sizes)
{
    __shared__ int lds[4];
    const uint32_t *bm = bitmaps + (size_t)blockIdx.x * words;
    int c = 0;
    for (int w = threadIdx.x; w < words; w += 256) c += __popc(bm[w]);
    c = block_sum_256(c, lds);
    if (threadIdx.x == 0) sizes[blockIdx.x] = c;
}

// cand_off[j] = sum of the sizes below j (64-bit); one wavefront
__global__ __launch_bounds__(64) void aset_scan_kernel(const int32_t *__restrict__ sizes, int K,
                                                       int64_t *__restrict__ cand_off)
{
    long long carry = 0;
    const int lane = threadIdx.x;
    for (int base = 0; base < K; base += 64) {
        const int j = base + lane;
        const long long v = j < K ? sizes[j] : 0;
        long long inc = v;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const long long up = __shfl_up(inc, off);
            if (lane >= off) inc += up;
        }
        if (j < K) cand_off[j] = carry + inc - v;
        carry += __shfl(inc, 63);
    }
    if (lane == 0) cand_off[K] = carry;
}

// the set bits of cluster blockIdx.x's list as ascending token ids
__global__ __launch_bounds__(256) void aset_emit_kernel(const uint32_t *__restrict__ bitmaps, int words,
                                                        const int64_t *__restrict__ cand_off,
                                                        int32_t *__restrict__ cand_ids)
{
    __shared__ int wsum[4];
    const uint32_t *bm = bitmaps + (size_t)blockIdx.x * words;
    int64_t out = cand_off[blockIdx.x];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (int base = 0; base < words; base += 256) {
        const int w = base + threadIdx.x;
        uint32_t bits = w < words ? bm[w] : 0u;
        const int c = __popc(bits);
        int inc = c;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const int up = __shfl_up(inc, off);
            if (lane >= off) inc += up;
        }
        __syncthreads();   // wsum of the previous round has been read
        if (lane == 63) wsum[wave] = inc;
        __syncthreads();
        int before = inc - c;
        for (int x = 0; x < wave; ++x) before += wsum[x];
        const int round_total = wsum[0] + wsum[1] + wsum[2] + wsum[3];
        int64_t pos = out + before;
        while (bits) {
            const int bit = __ffs(bits) - 1;
            bits &= bits - 1;
            cand_ids[pos++] = w * 32 + bit;
        }
        out += round_total;
    }
}

}  // namespace

uint16_t vpk_round_to_half(double v) { return double_to_half_bits(v); }

void vpk_fill_u32(void *p, size_t n, uint32_t v, hipStream_t st)
{
    if (n == 0) return;
    hipLaunchKernelGGL(fill_u32_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, (uint32_t *)p, n, v);
}

void vpk_kmeans_assign(const void *cpart, int parts, int rows, int K, int32_t *assign, int32_t *counts,
                       hipStream_t st)
{
    hipLaunchKernelGGL(kmeans_assign_kernel, dim3((rows + 255) / 256), dim3(256), 0, st, (const int2 *)cpart, parts,
                       rows, K, assign, counts);
}

bool vpk_kmeans_assign_gemm(const void *X, long n, int d, const void *cp, const float *cnorm, int K, int kt, int ctiles,
                            int32_t *assign, int32_t *counts, hipStream_t st)
{
    const dim3 grid((unsigned)((n + 63) / 64)), block(256);
#define VP_KM_CASE(KW)                                                                                                \
    case KW * 4:                                                                                                      \
        hipLaunchKernelGGL((kmeans_assign_gemm_kernel<KW>), grid, block, 0, st, (const uint4 *)X, n, d,               \
                           (const uint4 *)cp, cnorm, K, ctiles, assign, counts);                                      \
        return true;
    switch (kt) {
        VP_KM_CASE(2)
        VP_KM_CASE(4)
        VP_KM_CASE(8)
        VP_KM_CASE(12)
        default: return false;   // other k-extents: the caller falls back to the decode-time kernel
    }
#undef VP_KM_CASE
}

void vpk_kmeans_bucket(const int32_t *assign, long n, const int32_t *counts, int K, int32_t *start, int32_t *cursor,
                       int32_t *perm, hipStream_t st)
{
    hipLaunchKernelGGL(kmeans_scan_kernel, dim3(1), dim3(1024), 0, st, counts, K, start, cursor);
    hipLaunchKernelGGL(kmeans_scatter_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, assign, n, cursor,
                       perm);
}

void vpk_kmeans_update(const void *X, int d, const int32_t *perm, const int32_t *start, const int32_t *counts, int K,
                       int splits, void *acc, void *C, hipStream_t st)
{
    if (K >= 256) {
        // enough clusters to fill the chip with one workgroup each: no sums in memory at all
        hipLaunchKernelGGL(kmeans_mean_kernel, dim3(K), dim3(1024), 0, st, (const uint4 *)X, d / 8, perm, start,
                           (uint4 *)C);
        return;
    }
    hipLaunchKernelGGL(kmeans_sum_kernel, dim3(K, splits), dim3(256), 0, st, (const uint4 *)X, d / 8, perm, start,
                       splits, (unsigned long long *)acc);
    const size_t e = (size_t)K * d;
    hipLaunchKernelGGL(kmeans_update_kernel, dim3((unsigned)((e + 255) / 256)), dim3(256), 0, st,
                       (unsigned long long *)acc, counts, K, d, (uint16_t *)C);
}

void vpk_kmeans_split(const int32_t *counts, int K, int d, void *C, hipStream_t st)
{
    hipLaunchKernelGGL(kmeans_split_kernel, dim3(1), dim3(1024), (size_t)K * sizeof(int), st, counts, K, d,
                       (uint16_t *)C);
}

void vpk_aset_flags(const int32_t *top, const int32_t *assign, long n, int T, int K, int V, int words,
                    uint32_t *bitmaps, int32_t *sizes, int64_t *cand_off, hipStream_t st)
{
    vpk_fill_u32(bitmaps, (size_t)K * words, 0u, st);
    const long total = n * T;
    if (total > 0)
        hipLaunchKernelGGL(aset_flag_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, top, assign, n,
                           T, K, V, words, bitmaps);
    hipLaunchKernelGGL(aset_count_kernel, dim3(K), dim3(256), 0, st, bitmaps, words, sizes);
    hipLaunchKernelGGL(aset_scan_kernel, dim3(1), dim3(64), 0, st, sizes, K, cand_off);
}

void vpk_aset_emit(const uint32_t *bitmaps, int words, int K, const int64_t *cand_off, int32_t *cand_ids,
                   hipStream_t st)
{
    hipLaunchKernelGGL(aset_emit_kernel, dim3(K), dim3(256), 0, st, bitmaps, words, cand_off, cand_ids);
}
