// Training of the quantizers and encoding (Sec. 3.2, Alg. 2 build_quantizers; the encoding rule of the
// last paragraph of Sec. 3.2).
//
//   step 1  kmeans                 temporary codebook of 2^b centroids per sub-quantizer
//   step 2  kmeans_same_size       the temporary centroids partitioned into 2^bbar groups of equal size
//   step 3  build_final_codebook   the temporary centroids reordered so that the low bbar bits of a
//                                  centroid's index name its group (property P1)
//   encode                         sub-code j of a vector = index of the centroid of C_j nearest to its
//                                  j-th sub-vector
//
// The paper leaves the insides of steps 1 and 2 to standard algorithms; what is computed here:
//   - nearest centroid: smallest (distance, index); distances ||x||^2 + ||c||^2 - 2 <x, c> with the inner
//     products on the double-precision matrix cores (v_mfma_f64_16x16x4_f64), compared in double precision;
//   - a k-means iteration assigns every point and replaces each centroid by the mean of its members
//     (double-precision sums, one division, rounded to fp32); a centroid without members keeps its value;
//     initial centroids are an input; after the last iteration the points are assigned once more;
//   - same-size k-means: an iteration makes a balanced assignment (groups of exactly n / kbar points) and
//     takes the means; the labels returned are those of the last assignment, whose means the returned
//     centroids are;
//   - balanced assignment, in rounds: every point without a group proposes to the group with the smallest
//     (distance, index) among those with room; every group takes, among its proposers, those with the
//     smallest (distance, point) up to its room; until no point is left.  Distances are fp32 table entries
//     (the distance-table kernel of tables_full.hip).
#include "common.h"
#include "device_util.h"
#include "f64_tile.h"

namespace dcpq {


constexpr int kAssignQ = 32;       // points per workgroup (2 row tiles of 16)
constexpr int kAssignC = 256;      // centroids per step of a workgroup (4 wavefronts x 64)

// Smaller of two (value, index) pairs; equal values -> smaller index.
__device__ inline void take_smaller(double &v, uint32_t &i, double ov, uint32_t oi)
{
    if (ov < v || (ov == v && oi < i)) { v = ov; i = oi; }
}

// Nearest centroid of the j-th sub-vector of every point, j = blockIdx.y.  A workgroup owns kAssignQ
// points and walks all centroids of C_j in steps of kAssignC; operand and result layout of the matrix
// instruction as in the distance-table kernel (lane l: A row l % 16, column l / 16; B row l / 16, column
// l % 16; value v of the result is row 4 v + l / 16, column l % 16), centroid columns interleaved by 4.
// The term ||x||^2 is the same for every centroid of a point and is left out of the comparison.
// points: rows of `ld` floats; sub-vector j starts at column j * dsub.  labels: [n][m] of LabelT.
// dist (optional): [n][m] fp32 squared distance to the chosen centroid.
template <typename LabelT>
__global__ __launch_bounds__(256) void assign_kernel(const float *__restrict__ points, uint64_t n, int ld,
                                                     const float *__restrict__ cb, int m, int dsub, int ncent,
                                                     LabelT *__restrict__ labels, float *__restrict__ dist)
{
    __shared__ double red_v[4][kAssignQ];
    __shared__ uint32_t red_i[4][kAssignQ];
    __shared__ double ny[kAssignQ];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int j = blockIdx.y;
    const uint64_t q0 = static_cast<uint64_t>(blockIdx.x) * kAssignQ;
    const float *cbj = cb + static_cast<size_t>(j) * ncent * dsub;
    const int lr = lane & 15, lk = lane >> 4;
    constexpr int MT = kAssignQ / 16;

    double best_v[MT][4];
    uint32_t best_i[MT][4];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int v = 0; v < 4; ++v) { best_v[mt][v] = INFINITY; best_i[mt][v] = 0xFFFFFFFFu; }
    double na[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) na[mt] = 0.0;

    const float *ap[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        const uint64_t q = q0 + mt * 16 + lr;
        ap[mt] = points + static_cast<size_t>(q < n ? q : n - 1) * ld + j * dsub;
    }
    for (int c0 = 0; c0 < ncent; c0 += kAssignC) {                    // uniform
        const int cw = c0 + wave * 64;                                // first centroid of this wavefront
        double4_t acc[MT][4];
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int nt = 0; nt < 4; ++nt) acc[mt][nt] = double4_t{0.0, 0.0, 0.0, 0.0};
        double nb[4] = {0.0, 0.0, 0.0, 0.0};
        // this lane's four centroids, clamped to valid ones (the others are skipped below)
        const float *bp[4];
#pragma unroll
        for (int nt = 0; nt < 4; ++nt) {
            const int c = cw + lr * 4 + nt;
            bp[nt] = cbj + static_cast<size_t>(c < ncent ? c : ncent - 1) * dsub;
        }
        f64_tile_products<MT>(ap, bp, dsub, lk, c0 == 0, acc, na, nb);
#pragma unroll
        for (int nt = 0; nt < 4; ++nt) {
            nb[nt] += __shfl_xor(nb[nt], 16);
            nb[nt] += __shfl_xor(nb[nt], 32);
        }
        // this lane's four centroids against its eight result rows, in increasing centroid index
#pragma unroll
        for (int nt = 0; nt < 4; ++nt) {
            const int c = cw + lr * 4 + nt;
            if (c < ncent) {
#pragma unroll
                for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        // a lane meets its centroids in increasing index, so "strictly smaller" keeps the first of equals
                        const double val = fma(-2.0, acc[mt][nt][v], nb[nt]);
                        const bool better = val < best_v[mt][v];
                        best_v[mt][v] = better ? val : best_v[mt][v];
                        best_i[mt][v] = better ? static_cast<uint32_t>(c) : best_i[mt][v];
                    }
            }
        }
    }
    // the 16 lanes with the same l / 16 hold candidates for the same rows: reduce over them, then over
    // the four wavefronts through LDS
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int v = 0; v < 4; ++v) {
#pragma unroll
            for (int off = 1; off < 16; off <<= 1) {
                const double ov = __shfl_xor(best_v[mt][v], off);
                const uint32_t oi = __shfl_xor(best_i[mt][v], off);
                take_smaller(best_v[mt][v], best_i[mt][v], ov, oi);
            }
            if (lr == 0) { red_v[wave][mt * 16 + v * 4 + lk] = best_v[mt][v]; red_i[wave][mt * 16 + v * 4 + lk] = best_i[mt][v]; }
        }
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        na[mt] += __shfl_xor(na[mt], 16);
        na[mt] += __shfl_xor(na[mt], 32);
        if (wave == 0 && lk == 0) ny[mt * 16 + lr] = na[mt];
    }
    __syncthreads();
    if (tid < kAssignQ && q0 + tid < n) {
        double v = red_v[0][tid];
        uint32_t i = red_i[0][tid];
        for (int w = 1; w < 4; ++w) take_smaller(v, i, red_v[w][tid], red_i[w][tid]);
        const size_t o = (q0 + tid) * static_cast<size_t>(m) + j;
        labels[o] = static_cast<LabelT>(i);
        if (dist) dist[o] = static_cast<float>(fmax(0.0, ny[tid] + v));
    }
}

// sums[label][t] += point[t] (double), counts[label] += 1.  One thread per (point, component).
__global__ __launch_bounds__(256) void accumulate_kernel(const float *__restrict__ points, uint64_t n, int ld, int d,
                                                         const uint32_t *__restrict__ labels, double *__restrict__ sums,
                                                         uint32_t *__restrict__ counts)
{
    const uint64_t e = static_cast<uint64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
    if (e >= n * static_cast<uint64_t>(d)) return;
    const uint64_t i = e / d;
    const int t = static_cast<int>(e % d);
    const uint32_t c = labels[i];
    unsafeAtomicAdd(&sums[static_cast<size_t>(c) * d + t], static_cast<double>(points[i * ld + t]));
    if (t == 0) atomicAdd(&counts[c], 1u);
}

__global__ __launch_bounds__(256) void means_kernel(const double *__restrict__ sums, const uint32_t *__restrict__ counts,
                                                    int k, int d, float *__restrict__ centroids)
{
    const int e = blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= k * d) return;
    const uint32_t c = counts[e / d];
    if (c) centroids[e] = static_cast<float>(sums[e] / static_cast<double>(c));    // no members: keeps its value
}

__global__ __launch_bounds__(256) void clear_kernel(uint32_t *p, size_t nwords)
{
    const size_t i = static_cast<size_t>(blockIdx.x) * blockDim.x + threadIdx.x;
    if (i < nwords) p[i] = 0u;
}

// ---- balanced assignment ----------------------------------------------------------------------------
// state: labels[n] (0xFFFFFFFF = no group yet), room[kbar], left[0] = points without a group
__global__ __launch_bounds__(256) void balanced_init_kernel(uint32_t *labels, int n, uint32_t *room, int kbar, uint32_t *left)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) labels[i] = 0xFFFFFFFFu;
    if (i < kbar) room[i] = static_cast<uint32_t>(n / kbar);
    if (i == 0) left[0] = static_cast<uint32_t>(n);
}

// prop[i] = the group with room nearest to point i (smallest (distance, index)), -1 for a point that has a group
__global__ __launch_bounds__(256) void propose_kernel(const float *__restrict__ T, int n, int kbar,
                                                      const uint32_t *__restrict__ labels, const uint32_t *__restrict__ room,
                                                      int *__restrict__ prop)
{
    __shared__ uint32_t lroom[256];
    if (threadIdx.x < static_cast<unsigned>(kbar)) lroom[threadIdx.x] = room[threadIdx.x];
    __syncthreads();
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    int p = -1;
    if (labels[i] == 0xFFFFFFFFu) {
        float best = INFINITY;
        for (int l = 0; l < kbar; ++l) {
            const float v = T[static_cast<size_t>(i) * kbar + l];
            if (lroom[l] > 0 && (p < 0 || v < best)) { best = v; p = l; }
        }
    }
    prop[i] = p;
}

// One workgroup per group: its proposers ordered by (distance, point), the first `room` of them accepted.
// list: scratch of np2 keys per group (np2 = n rounded up to a power of two).
__global__ __launch_bounds__(1024) void accept_kernel(const float *__restrict__ T, int n, int kbar, const int *__restrict__ prop,
                                                      uint32_t *__restrict__ labels, uint32_t *__restrict__ room,
                                                      uint32_t *__restrict__ left, uint64_t *__restrict__ list, uint32_t np2)
{
    __shared__ uint32_t s_n;
    const int l = blockIdx.x, tid = threadIdx.x;
    const uint32_t have = room[l];
    if (have == 0) return;                                       // uniform
    uint64_t *a = list + static_cast<size_t>(l) * np2;
    if (tid == 0) s_n = 0;
    __syncthreads();
    for (int i = tid; i < n; i += 1024)
        if (prop[i] == l) {
            const uint32_t pos = atomicAdd(&s_n, 1u);
            a[pos] = make_key(__float_as_uint(T[static_cast<size_t>(i) * kbar + l]), static_cast<uint32_t>(i));   // distances are >= +0
        }
    __syncthreads();
    const uint32_t p = s_n;
    if (p == 0) return;                                          // uniform
    uint32_t take = p;
    if (p > have) {                                              // uniform: more proposers than room, keep the closest
        uint32_t s2 = 1;
        while (s2 < p) s2 <<= 1;
        for (uint32_t t = p + tid; t < s2; t += 1024) a[t] = ~0ull;
        __syncthreads();
        bitonic_sort(a, s2);
        take = have;
    }
    for (uint32_t t = tid; t < take; t += 1024) labels[static_cast<uint32_t>(a[t])] = static_cast<uint32_t>(l);
    if (tid == 0) { room[l] = have - take; atomicSub(left, take); }
}

// Step 3: one workgroup per group l walks the labels in index order; the i-th member met gets the final
// index (i << bbar) | l.
__global__ __launch_bounds__(1024) void final_codebook_kernel(const float *__restrict__ temp, int k, int d,
                                                              const uint32_t *__restrict__ labels, int bbar,
                                                              float *__restrict__ final_cb, uint32_t *__restrict__ perm)
{
    __shared__ uint32_t wsum[16];
    __shared__ uint32_t s_base;
    const uint32_t l = blockIdx.x;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    if (tid == 0) s_base = 0;
    __syncthreads();
    for (int i0 = 0; i0 < k; i0 += 1024) {                       // uniform
        const int i = i0 + tid;
        const bool mine = i < k && labels[i] == l;
        const uint64_t mask = __ballot(mine);
        const uint32_t below = __popcll(mask & ((1ull << lane) - 1ull));
        if (lane == 0) wsum[wave] = __popcll(mask);
        __syncthreads();
        uint32_t before = s_base;
        for (int w = 0; w < wave; ++w) before += wsum[w];
        if (mine) {
            const uint32_t f = ((before + below) << bbar) | l;
            if (f < static_cast<uint32_t>(k)) {                  // labels with unequal groups would point past the end
                perm[f] = static_cast<uint32_t>(i);
                for (int t = 0; t < d; ++t) final_cb[static_cast<size_t>(f) * d + t] = temp[static_cast<size_t>(i) * d + t];
            }
        }
        __syncthreads();
        if (tid == 0) { uint32_t tot = 0; for (int w = 0; w < 16; ++w) tot += wsum[w]; s_base += tot; }
        __syncthreads();
    }
}

// ---- host side --------------------------------------------------------------------------------------

static int launch_assign(const float *points, uint64_t n, int ld, const float *cb, int m, int dsub, int ncent, void *labels,
                         int label_bytes, float *dist, hipStream_t st)
{
    if (n == 0) return DCPQ_OK;
    const dim3 grid(static_cast<unsigned>((n + kAssignQ - 1) / kAssignQ), m);
    switch (label_bytes) {
        case 1:
            DCPQ_LAUNCH(kStageTrain, st, assign_kernel<uint8_t>, grid, dim3(256), 0, points, n, ld, cb, m, dsub, ncent,
                        static_cast<uint8_t *>(labels), dist);
            break;
        case 2:
            DCPQ_LAUNCH(kStageTrain, st, assign_kernel<uint16_t>, grid, dim3(256), 0, points, n, ld, cb, m, dsub, ncent,
                        static_cast<uint16_t *>(labels), dist);
            break;
        default:
            DCPQ_LAUNCH(kStageTrain, st, assign_kernel<uint32_t>, grid, dim3(256), 0, points, n, ld, cb, m, dsub, ncent,
                        static_cast<uint32_t *>(labels), dist);
            break;
    }
    DCPQ_CHECK_LAUNCH("assign_kernel");
    return DCPQ_OK;
}

static size_t means_bytes(int k, int d) { return align_up(sizeof(double) * static_cast<size_t>(k) * d + sizeof(uint32_t) * k, 256); }

// centroids[c] = mean of the points labelled c (ws: means_bytes(k, d))
static int launch_means(const float *points, uint64_t n, int ld, int d, const uint32_t *labels, int k, float *centroids,
                        void *ws, hipStream_t st)
{
    double *sums = static_cast<double *>(ws);
    uint32_t *counts = reinterpret_cast<uint32_t *>(sums + static_cast<size_t>(k) * d);
    const size_t nwords = (sizeof(double) * static_cast<size_t>(k) * d + sizeof(uint32_t) * k) / 4;
    DCPQ_LAUNCH(kStageTrain, st, clear_kernel, dim3(static_cast<unsigned>((nwords + 255) / 256)), dim3(256), 0,
                reinterpret_cast<uint32_t *>(ws), nwords);
    DCPQ_CHECK_LAUNCH("clear_kernel");
    const uint64_t e = n * static_cast<uint64_t>(d);
    DCPQ_LAUNCH(kStageTrain, st, accumulate_kernel, dim3(static_cast<unsigned>((e + 255) / 256)), dim3(256), 0, points, n, ld, d,
                labels, sums, counts);
    DCPQ_CHECK_LAUNCH("accumulate_kernel");
    DCPQ_LAUNCH(kStageTrain, st, means_kernel, dim3((k * d + 255) / 256), dim3(256), 0, sums, counts, k, d, centroids);
    DCPQ_CHECK_LAUNCH("means_kernel");
    return DCPQ_OK;
}

static uint32_t pow2_at_least(uint32_t x)
{
    uint32_t p = 1;
    while (p < x) p <<= 1;
    return p;
}

struct SameSizePlan { size_t off_T, off_prop, off_room, off_left, off_list, off_means, total; uint32_t np2; };

static SameSizePlan plan_same_size(int n, int d, int kbar)
{
    SameSizePlan p{};
    p.np2 = pow2_at_least(static_cast<uint32_t>(n));
    size_t off = 0;
    p.off_T = off;     off = align_up(off + sizeof(float) * static_cast<size_t>(n) * kbar, 256);
    p.off_prop = off;  off = align_up(off + sizeof(int) * static_cast<size_t>(n), 256);
    p.off_room = off;  off = align_up(off + sizeof(uint32_t) * kbar, 256);
    p.off_left = off;  off = align_up(off + 256, 256);
    p.off_list = off;  off = align_up(off + sizeof(uint64_t) * static_cast<size_t>(kbar) * p.np2, 256);
    p.off_means = off; off = align_up(off + means_bytes(kbar, d), 256);
    p.total = off;
    return p;
}

}  // namespace dcpq

using namespace dcpq;

extern "C" int dcpq_assign(const float *points, uint64_t n, int ld, const float *codebooks, int m, int dsub, int n_entries,
                           void *labels, int label_bytes, float *dist, void *stream)
{
    clear_error();
    if (!dcpq_shape_supported(m, dsub)) return fail(DCPQ_EUNSUPPORTED, "assign: m=%d dsub=%d not supported", m, dsub);
    DCPQ_REQUIRE(n < (1ull << 32) * kAssignQ, "assign: n out of range");
    DCPQ_REQUIRE(ld >= m * dsub, "assign: row stride %d below m * dsub = %d", ld, m * dsub);
    DCPQ_REQUIRE(label_bytes == 1 || label_bytes == 2 || label_bytes == 4, "assign: label_bytes=%d (1, 2 or 4)", label_bytes);
    DCPQ_REQUIRE(n_entries >= 1 && (label_bytes == 4 || n_entries <= (1 << (8 * label_bytes))),
                 "assign: %d centroids do not fit labels of %d byte(s)", n_entries, label_bytes);
    if (n == 0) return DCPQ_OK;
    DCPQ_REQUIRE(points && codebooks && labels, "assign: null pointer");
    return launch_assign(points, n, ld, codebooks, m, dsub, n_entries, labels, label_bytes, dist, as_stream(stream));
}

extern "C" int dcpq_encode(const float *vectors, uint64_t n, const float *codebooks, int m, int dsub, int b, void *codes,
                           void *stream)
{
    if (!dcpq_bits_supported(b, 1)) {
        clear_error();
        return fail(DCPQ_EUNSUPPORTED, "encode: b=%d not supported", b);
    }
    return dcpq_assign(vectors, n, m * dsub, codebooks, m, dsub, 1 << b, codes, b / 8, nullptr, stream);
}

extern "C" size_t dcpq_kmeans_workspace_bytes(int k, int d)
{
    if (k <= 0 || d <= 0) return 0;
    return means_bytes(k, d);
}

extern "C" int dcpq_kmeans(const float *points, uint64_t n, int ld, int d, int k, int iters, float *centroids,
                           uint32_t *labels, void *workspace, size_t workspace_bytes, void *stream)
{
    clear_error();
    if (!dcpq_shape_supported(1, d)) return fail(DCPQ_EUNSUPPORTED, "kmeans: d=%d not supported", d);
    DCPQ_REQUIRE(n >= 1 && n < (1ull << 32), "kmeans: n out of range");
    DCPQ_REQUIRE(k >= 1 && iters >= 0 && ld >= d, "kmeans: k=%d iters=%d ld=%d", k, iters, ld);
    DCPQ_REQUIRE(points && centroids && labels && workspace, "kmeans: null pointer");
    DCPQ_REQUIRE((reinterpret_cast<uintptr_t>(workspace) & 255) == 0, "kmeans: workspace must be 256-byte aligned");
    if (workspace_bytes < means_bytes(k, d))
        return fail(DCPQ_EWORKSPACE, "kmeans: workspace %zu < %zu bytes", workspace_bytes, means_bytes(k, d));
    hipStream_t st = as_stream(stream);
    for (int it = 0; it < iters; ++it) {
        int rc = launch_assign(points, n, ld, centroids, 1, d, k, labels, 4, nullptr, st);
        if (rc) return rc;
        rc = launch_means(points, n, ld, d, labels, k, centroids, workspace, st);
        if (rc) return rc;
    }
    return launch_assign(points, n, ld, centroids, 1, d, k, labels, 4, nullptr, st);
}

extern "C" size_t dcpq_kmeans_same_size_workspace_bytes(int n, int d, int kbar)
{
    if (n <= 0 || d <= 0 || kbar <= 0 || kbar > 256) return 0;
    return plan_same_size(n, d, kbar).total;
}

extern "C" int dcpq_kmeans_same_size(const float *points, int n, int d, int kbar, int iters, float *centroids,
                                     uint32_t *labels, void *workspace, size_t workspace_bytes, void *stream)
{
    clear_error();
    if (!dcpq_shape_supported(1, d)) return fail(DCPQ_EUNSUPPORTED, "kmeans_same_size: d=%d not supported", d);
    DCPQ_REQUIRE(kbar >= 1 && kbar <= 256, "kmeans_same_size: kbar=%d (1..256)", kbar);
    DCPQ_REQUIRE(n >= kbar && n % kbar == 0 && n <= (1 << 20), "kmeans_same_size: n=%d must be a multiple of kbar=%d, at most 2^20", n, kbar);
    DCPQ_REQUIRE(iters >= 1, "kmeans_same_size: iters=%d", iters);
    DCPQ_REQUIRE(points && centroids && labels && workspace, "kmeans_same_size: null pointer");
    DCPQ_REQUIRE((reinterpret_cast<uintptr_t>(workspace) & 255) == 0, "kmeans_same_size: workspace must be 256-byte aligned");
    const SameSizePlan p = plan_same_size(n, d, kbar);
    if (workspace_bytes < p.total) return fail(DCPQ_EWORKSPACE, "kmeans_same_size: workspace %zu < %zu bytes", workspace_bytes, p.total);
    uint8_t *base = static_cast<uint8_t *>(workspace);
    float *T = reinterpret_cast<float *>(base + p.off_T);
    int *prop = reinterpret_cast<int *>(base + p.off_prop);
    uint32_t *room = reinterpret_cast<uint32_t *>(base + p.off_room);
    uint32_t *left = reinterpret_cast<uint32_t *>(base + p.off_left);
    uint64_t *list = reinterpret_cast<uint64_t *>(base + p.off_list);
    hipStream_t st = as_stream(stream);
    for (int it = 0; it < iters; ++it) {
        int rc = launch_distance_tables(points, n, centroids, 1, d, kbar, T, kStageTrain, st);
        if (rc) return rc;
        const int nb = (n > kbar ? n : kbar);
        DCPQ_LAUNCH(kStageTrain, st, balanced_init_kernel, dim3((nb + 255) / 256), dim3(256), 0, labels, n, room, kbar, left);
        DCPQ_CHECK_LAUNCH("balanced_init_kernel");
        // rounds until every point has a group; every round gives at least one point a group, and the count
        // is read back after each (the only host synchronization in the library)
        uint32_t h_left = static_cast<uint32_t>(n);
        for (int round = 0; h_left > 0; ++round) {
            if (round > n) return fail(DCPQ_EHIP, "kmeans_same_size: balanced assignment did not finish");
            DCPQ_LAUNCH(kStageTrain, st, propose_kernel, dim3((n + 255) / 256), dim3(256), 0, T, n, kbar, labels, room, prop);
            DCPQ_CHECK_LAUNCH("propose_kernel");
            DCPQ_LAUNCH(kStageTrain, st, accept_kernel, dim3(kbar), dim3(1024), 0, T, n, kbar, prop, labels, room, left, list, p.np2);
            DCPQ_CHECK_LAUNCH("accept_kernel");
            DCPQ_CHECK_HIP(hipMemcpyAsync(&h_left, left, sizeof(uint32_t), hipMemcpyDeviceToHost, st));
            DCPQ_CHECK_HIP(hipStreamSynchronize(st));
        }
        rc = launch_means(points, static_cast<uint64_t>(n), d, d, labels, kbar, centroids, base + p.off_means, st);
        if (rc) return rc;
    }
    return DCPQ_OK;
}

extern "C" int dcpq_build_final_codebook(const float *temp_codebook, int k, int d, const uint32_t *labels, int bbar,
                                         float *final_codebook, uint32_t *perm, void *stream)
{
    clear_error();
    DCPQ_REQUIRE(k >= 1 && d >= 1 && bbar >= 0 && bbar <= 8 && k % (1 << bbar) == 0, "build_final_codebook: k=%d d=%d bbar=%d", k, d, bbar);
    DCPQ_REQUIRE(temp_codebook && labels && final_codebook && perm, "build_final_codebook: null pointer");
    DCPQ_REQUIRE(temp_codebook != final_codebook, "build_final_codebook: in place is not supported");
    DCPQ_LAUNCH(kStageTrain, as_stream(stream), final_codebook_kernel, dim3(1 << bbar), dim3(1024), 0, temp_codebook, k, d, labels,
                bbar, final_codebook, perm);
    DCPQ_CHECK_LAUNCH("final_codebook_kernel");
    return DCPQ_OK;
}

// Alg. 2 for all m sub-quantizers.  Workspace: labels of the training points, the temporary codebook, labels
// and order of its centroids, and the larger of the two k-means workspaces.
struct BuildPlan { size_t off_plabels, off_temp, off_clabels, off_perm, off_cbar, off_ws, ws_bytes, total; };

static BuildPlan plan_build(uint64_t n, int dsub, int b, int bbar)
{
    BuildPlan p{};
    const int k = 1 << b, kbar = 1 << bbar;
    size_t off = 0;
    p.off_plabels = off; off = align_up(off + sizeof(uint32_t) * n, 256);
    p.off_temp = off;    off = align_up(off + sizeof(float) * static_cast<size_t>(k) * dsub, 256);
    p.off_clabels = off; off = align_up(off + sizeof(uint32_t) * k, 256);
    p.off_perm = off;    off = align_up(off + sizeof(uint32_t) * k, 256);
    p.off_cbar = off;    off = align_up(off + sizeof(float) * static_cast<size_t>(kbar) * dsub, 256);
    const size_t a = means_bytes(k, dsub), c = plan_same_size(k, dsub, kbar).total;
    p.ws_bytes = a > c ? a : c;
    p.off_ws = off;      off = align_up(off + p.ws_bytes, 256);
    p.total = off;
    return p;
}

extern "C" size_t dcpq_build_quantizers_workspace_bytes(uint64_t n_train, int dsub, int b, int bbar)
{
    if (n_train == 0 || dsub <= 0 || !dcpq_bits_supported(b, bbar)) return 0;
    return plan_build(n_train, dsub, b, bbar).total;
}

extern "C" int dcpq_build_quantizers(const float *train, uint64_t n_train, int m, int dsub, int b, int bbar, int iters,
                                     int iters_same_size, float *codebooks, float *derived, void *workspace,
                                     size_t workspace_bytes, void *stream)
{
    clear_error();
    if (!dcpq_shape_supported(m, dsub)) return fail(DCPQ_EUNSUPPORTED, "build_quantizers: m=%d dsub=%d not supported", m, dsub);
    if (!dcpq_bits_supported(b, bbar)) return fail(DCPQ_EUNSUPPORTED, "build_quantizers: b=%d bbar=%d not supported", b, bbar);
    DCPQ_REQUIRE(n_train >= 1 && n_train < (1ull << 32), "build_quantizers: n_train out of range");
    DCPQ_REQUIRE(iters >= 0 && iters_same_size >= 1, "build_quantizers: iters=%d iters_same_size=%d", iters, iters_same_size);
    DCPQ_REQUIRE(train && codebooks && derived && workspace, "build_quantizers: null pointer");
    DCPQ_REQUIRE((reinterpret_cast<uintptr_t>(workspace) & 255) == 0, "build_quantizers: workspace must be 256-byte aligned");
    const BuildPlan p = plan_build(n_train, dsub, b, bbar);
    if (workspace_bytes < p.total) return fail(DCPQ_EWORKSPACE, "build_quantizers: workspace %zu < %zu bytes", workspace_bytes, p.total);
    uint8_t *base = static_cast<uint8_t *>(workspace);
    uint32_t *plabels = reinterpret_cast<uint32_t *>(base + p.off_plabels);
    float *temp = reinterpret_cast<float *>(base + p.off_temp);
    uint32_t *clabels = reinterpret_cast<uint32_t *>(base + p.off_clabels);
    uint32_t *perm = reinterpret_cast<uint32_t *>(base + p.off_perm);
    float *cbar = reinterpret_cast<float *>(base + p.off_cbar);
    const int k = 1 << b, kbar = 1 << bbar, D = m * dsub;
    hipStream_t st = as_stream(stream);
    for (int j = 0; j < m; ++j) {
        float *cj = codebooks + static_cast<size_t>(j) * k * dsub;
        // step 1: the initial centroids the caller left in codebooks[j] become the temporary codebook
        DCPQ_CHECK_HIP(hipMemcpyAsync(temp, cj, sizeof(float) * static_cast<size_t>(k) * dsub, hipMemcpyDeviceToDevice, st));
        int rc = dcpq_kmeans(train + static_cast<size_t>(j) * dsub, n_train, D, dsub, k, iters, temp, plabels, base + p.off_ws,
                             p.ws_bytes, stream);
        if (rc) return rc;
        // step 2: groups of equal size, started from the first 2^bbar temporary centroids
        DCPQ_CHECK_HIP(hipMemcpyAsync(cbar, temp, sizeof(float) * static_cast<size_t>(kbar) * dsub, hipMemcpyDeviceToDevice, st));
        rc = dcpq_kmeans_same_size(temp, k, dsub, kbar, iters_same_size, cbar, clabels, base + p.off_ws, p.ws_bytes, stream);
        if (rc) return rc;
        // step 3: final order; the derived codebook is the mean of every low-bits group of it
        rc = dcpq_build_final_codebook(temp, k, dsub, clabels, bbar, cj, perm, stream);
        if (rc) return rc;
    }
    return launch_derive(codebooks, m, dsub, b, bbar, derived, st);
}
