// Alg. 3 with an inverted index and residual encoding (Sec. 2.2; Sec. 2.3: every step after the
// Index step is done once per probed list; Sec. 3.3).  List l holds the codes at positions offsets[l] .. offsets[l+1]-1 of the
// code array (a vector's id is its position); codes quantize the residual x - c_l.
//
//   Index   ivf_probe           the nprobe closest cell centres per query (matrix cores, fp64)
//   Tables  ivf_small_tables    per (query, probed list): small tables of the residual query
//                               rho = y - c_l on the derived codebooks; ONE (qmin, qmax) pair per
//                               query -- qmin over all its lists' tables, qmax over the first
//                               min(r, total) codes met walking its lists in probe order -- so that
//                               integer distances from different lists are comparable
//   Scan    ivf_scan            the r smallest (qd, id) over the union of the probed lists, over a
//                               per-query list of "units" (runs of codes inside one list, in
//                               increasing id order), one wavefront per unit with that (query,
//                               list)'s 8-bit tables in LDS: one streaming pass with a running
//                               bucket bound and an exact selection (as in scan_fast.hip), the
//                               three-pass selection of scan.hip for the queries it flags
//   Refine  ivf_refine_topk     Eq. 3 on the residual of each candidate's own list, directly from
//                               the full codebooks in double precision (per-list 2^16-entry tables
//                               would cost nprobe table builds per query), then the k best
#include "common.h"
#include "scan_internal.h"

namespace dcpq {

constexpr int kIvfUnitsPerQuery = 1024;   // upper bound of scan units per query (unit size adapts)
constexpr int kIvfMaxProbe = 512;         // nprobe supported by the per-query planning kernels
constexpr uint32_t kIvfSampleStep = 32;   // the first 1 / kIvfSampleStep of every probed list is the sample that gives the scan its starting bounds
constexpr int kIvfSampleUnits = kIvfMaxProbe + kIvfUnitsPerQuery / static_cast<int>(kIvfSampleStep);   // sample units a query can have

struct IvfUnit {
    uint64_t begin;    // first code of the unit (global position)
    uint32_t count;    // codes in the unit
    uint32_t p;        // index of the list in the query's probe order (selects the tables)
};

// ------------------------------------------------------------------------------------------------
// Index step: nprobe smallest coarse distances per query, ordered by (distance, list id).
// dist: [nq][nlist] fp32 squared distances.  One workgroup per query, 4-level radix select on the
// bit patterns (non-negative floats order like their bits), ties at the cut taken in id order.
// ------------------------------------------------------------------------------------------------
constexpr uint32_t kProbeSteps = 2048;   // histogram steps of the cut by value (two per thread)

__global__ __launch_bounds__(1024) void ivf_select_probe_kernel(const float *__restrict__ dist, int nlist, int nprobe,
                                                               int32_t *__restrict__ probe)
{
    __shared__ uint32_t hist[256];
    __shared__ uint32_t s_prefix, s_need, s_pos;
    __shared__ uint32_t part[1024];
    __shared__ uint64_t sel[kIvfMaxProbe * 2];
    const int q = blockIdx.x, tid = threadIdx.x;
    const uint32_t *d = reinterpret_cast<const uint32_t *>(dist) + static_cast<size_t>(q) * nlist;

    // Cut by value first: a histogram over kProbeSteps equal steps between the smallest and the largest
    // distance locates the step that holds the nprobe-th smallest; the keys up to that step (a superset of
    // the nprobe smallest, usually little more) are gathered and sorted by (distance, id).  The radix
    // select below remains for inputs where that superset is large (many equal distances) or the
    // distances span no finite range.  (Its first levels put all keys into a handful of counters, since
    // distances of similar size share their top bits, which serializes the LDS atomics.)
    {
        __shared__ uint32_t steps[kProbeSteps];
        __shared__ uint32_t s_lo, s_hi, s_step, s_n, wsum[16];
        const int lane = tid & 63, wave = tid >> 6;
        uint32_t lo = 0xFFFFFFFFu, hi = 0;
        // (the row is walked three times, four keys per lane and load where its length allows: 16 instead of 64
        // dependent rounds per walk at 65536 lists)
        const bool vec = (nlist & 3) == 0 && (reinterpret_cast<uintptr_t>(dist) & 15) == 0;    // uniform
        auto for_each_key = [&](auto &&f) {
            if (vec) {
                const uint4 *d4 = reinterpret_cast<const uint4 *>(d);
                for (int l4 = tid; l4 < nlist / 4; l4 += 1024) {
                    const uint4 k4 = d4[l4];
                    f(k4.x, 4 * l4); f(k4.y, 4 * l4 + 1); f(k4.z, 4 * l4 + 2); f(k4.w, 4 * l4 + 3);
                }
            } else {
                for (int l = tid; l < nlist; l += 1024) f(d[l], l);
            }
        };
        for_each_key([&](uint32_t key, int) { lo = min(lo, key); hi = max(hi, key); });
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            lo = min(lo, static_cast<uint32_t>(__shfl_xor(static_cast<int>(lo), o)));
            hi = max(hi, static_cast<uint32_t>(__shfl_xor(static_cast<int>(hi), o)));
        }
        if (tid == 0) { s_lo = 0xFFFFFFFFu; s_hi = 0; s_step = kProbeSteps; s_n = 0; }
        for (uint32_t t = tid; t < kProbeSteps; t += 1024) steps[t] = 0;
        __syncthreads();
        if (lane == 0) { atomicMin(&s_lo, lo); atomicMax(&s_hi, hi); }
        __syncthreads();
        const float dlo = __uint_as_float(s_lo), dhi = __uint_as_float(s_hi);
        const float scale = static_cast<float>(kProbeSteps) / (dhi - dlo);
        // non-decreasing in the distance, so "step <= s" keeps every key below some value
        auto step_of = [&](uint32_t key) -> uint32_t {
            const float x = (__uint_as_float(key) - dlo) * scale;
            return x < static_cast<float>(kProbeSteps - 1) ? static_cast<uint32_t>(x) : kProbeSteps - 1;
        };
        bool cut = scale > 0.0f && scale < INFINITY;
        if (cut) {                                               // uniform
            for_each_key([&](uint32_t key, int) { atomicAdd(&steps[step_of(key)], 1u); });
            __syncthreads();
            const uint32_t h0 = steps[2 * tid], h1 = steps[2 * tid + 1];      // kProbeSteps = 2 x 1024 threads
            uint32_t incl = h0 + h1;
#pragma unroll
            for (int o = 1; o < 64; o <<= 1) {
                const uint32_t other = __shfl(incl, lane >= o ? lane - o : lane);
                if (lane >= o) incl += other;
            }
            if (lane == 63) wsum[wave] = incl;
            __syncthreads();
            uint32_t before = incl - (h0 + h1);
            for (int w2 = 0; w2 < wave; ++w2) before += wsum[w2];
            const uint32_t want = static_cast<uint32_t>(nprobe);
            if (before < want && before + h0 + h1 >= want) {      // exactly one thread (nprobe <= nlist)
                const bool first = before + h0 >= want;
                s_step = first ? 2 * tid : 2 * tid + 1;
                s_n = first ? before + h0 : before + h0 + h1;
            }
            __syncthreads();
            cut = s_step < kProbeSteps && s_n <= kIvfMaxProbe * 2;
        }
        if (cut) {                                               // uniform
            const uint32_t step = s_step, nkeep = s_n;
            uint32_t nf = 1;
            while (nf < nkeep) nf <<= 1;
            __syncthreads();
            if (tid == 0) s_n = 0;
            for (uint32_t t = tid; t < nf; t += 1024) sel[t] = ~0ull;
            __syncthreads();
            for_each_key([&](uint32_t key, int l) {
                if (step_of(key) <= step) {
                    const uint32_t pos = atomicAdd(&s_n, 1u);
                    if (pos < nf) sel[pos] = make_key(key, static_cast<uint32_t>(l));
                }
            });
            bitonic_sort(sel, nf);
            for (int t = tid; t < nprobe; t += 1024)
                probe[static_cast<size_t>(q) * nprobe + t] = static_cast<int32_t>(sel[t] & 0xFFFFFFFFu);
            return;
        }
        __syncthreads();
    }

    // value of the nprobe-th smallest key, one byte at a time from the top
    uint32_t prefix = 0, need = nprobe;
    for (int level = 3; level >= 0; --level) {
        if (tid < 256) hist[tid] = 0;
        __syncthreads();
        const uint32_t shift = 8 * level;
        const uint32_t hi_mask = level == 3 ? 0u : ~0u << (shift + 8);
        for (int l = tid; l < nlist; l += 1024) {
            const uint32_t key = d[l];
            if ((key & hi_mask) == prefix) atomicAdd(&hist[(key >> shift) & 255u], 1u);
        }
        __syncthreads();
        if (tid == 0) {
            uint32_t cum = 0, b = 0;
            for (; b < 256; ++b) {
                if (cum + hist[b] >= need) break;
                cum += hist[b];
            }
            s_prefix = prefix | (b << shift);
            s_need = need - cum;
        }
        __syncthreads();
        prefix = s_prefix;
        need = s_need;
        __syncthreads();
    }
    const uint32_t kth = prefix;          // exact key of the nprobe-th smallest; `need` of the equal keys are taken
    // contiguous id ranges per thread so that equal keys can be ranked in id order
    const int per = (nlist + 1023) / 1024;
    const int lo = tid * per, hi = min(nlist, lo + per);
    uint32_t eq = 0;
    for (int l = lo; l < hi; ++l) eq += d[l] == kth ? 1u : 0u;
    part[tid] = eq;
    if (tid == 0) s_pos = 0;
    __syncthreads();
    for (int off = 1; off < 1024; off <<= 1) {
        const uint32_t add = tid >= off ? part[tid - off] : 0u;
        __syncthreads();
        part[tid] += add;
        __syncthreads();
    }
    uint32_t rank = part[tid] - eq;       // equal keys before this thread's range
    for (int l = lo; l < hi; ++l) {
        const uint32_t key = d[l];
        bool take = key < kth;
        if (key == kth) { take = rank < need; ++rank; }
        if (take) {
            const uint32_t pos = atomicAdd(&s_pos, 1u);
            if (pos < static_cast<uint32_t>(nprobe)) sel[pos] = make_key(key, static_cast<uint32_t>(l));
        }
    }
    __syncthreads();
    uint32_t np2 = 1;
    while (np2 < static_cast<uint32_t>(nprobe)) np2 <<= 1;
    for (uint32_t t = nprobe + tid; t < np2; t += 1024) sel[t] = ~0ull;
    bitonic_sort(sel, np2);
    for (int t = tid; t < nprobe; t += 1024) probe[static_cast<size_t>(q) * nprobe + t] = static_cast<int32_t>(sel[t] & 0xFFFFFFFFu);
}

// ------------------------------------------------------------------------------------------------
// Tables step.  All arithmetic fp32, one rounding per operation, fixed order (feeds integers).
// ------------------------------------------------------------------------------------------------

// MODE 0: smallest entry of the (query, list) tables -> atomic min into qmin_bits[q].
// MODE 1: quantize with the query's bounds -> qtab[q][p][m][256].
// grid (ceil(nprobe / kIvfTabProbes), nq), 256 threads; thread i owns entry i of every table of
// kIvfTabProbes probed lists of the query.  The derived centroid is read once per component and used for
// all of those lists' residuals (the kernel is bound by these reads, which all come from the L2); every
// entry is still the sum over t, in ascending t, of the individually rounded squares.
constexpr int kIvfTabProbes = 8;

template <int MODE>
__global__ __launch_bounds__(256) void ivf_tables_kernel(const float *__restrict__ queries, const float *__restrict__ coarse,
                                                        const int32_t *__restrict__ probe, int nprobe,
                                                        const float *__restrict__ derived, int m, int dsub,
                                                        uint32_t *__restrict__ qmin_bits, const float *__restrict__ bounds,
                                                        uint8_t *__restrict__ qtab, float *__restrict__ keep)
{
    // keep (MODE 0, optional): the entries themselves, [nq][nprobe][m][256], for the quantization to read back
    // instead of computing them a second time
    extern __shared__ __align__(16) float lds[];         // rho [kIvfTabProbes][m*dsub]
    __shared__ float red[4];
    const int p0 = blockIdx.x * kIvfTabProbes, q = blockIdx.y, tid = threadIdx.x;
    const int np = min(kIvfTabProbes, nprobe - p0);
    const int D = m * dsub;
    for (int pp = 0; pp < np; ++pp) {
        const int l = probe[static_cast<size_t>(q) * nprobe + p0 + pp];
        for (int t = tid; t < D; t += 256)
            lds[pp * D + t] = __fsub_rn(queries[static_cast<size_t>(q) * D + t], coarse[static_cast<size_t>(l) * D + t]);
    }
    __syncthreads();
    float qmin = 0.0f, qmax = 0.0f;
    if (MODE == 1) {
        qmin = bounds[2 * q];
        qmax = bounds[2 * q + 1];
    }
    float lo = INFINITY;
    for (int j = 0; j < m; ++j) {
        const float *c = derived + (static_cast<size_t>(j) * kSmallSize + tid) * dsub;
        float acc[kIvfTabProbes];
#pragma unroll
        for (int pp = 0; pp < kIvfTabProbes; ++pp) acc[pp] = 0.0f;
        if ((dsub & 3) == 0) {
            // four components per step: one 16-byte load of the centroid, one 16-byte (broadcast) LDS read per
            // list; the squares are still added one by one in ascending t
            for (int t = 0; t < dsub; t += 4) {
                const float4 c4 = *reinterpret_cast<const float4 *>(c + t);
#pragma unroll
                for (int pp = 0; pp < kIvfTabProbes; ++pp) {
                    if (pp < np) {                                // uniform
                        const float4 r4 = *reinterpret_cast<const float4 *>(lds + pp * D + j * dsub + t);
                        float diff = __fsub_rn(r4.x, c4.x);
                        acc[pp] = __fadd_rn(acc[pp], __fmul_rn(diff, diff));
                        diff = __fsub_rn(r4.y, c4.y);
                        acc[pp] = __fadd_rn(acc[pp], __fmul_rn(diff, diff));
                        diff = __fsub_rn(r4.z, c4.z);
                        acc[pp] = __fadd_rn(acc[pp], __fmul_rn(diff, diff));
                        diff = __fsub_rn(r4.w, c4.w);
                        acc[pp] = __fadd_rn(acc[pp], __fmul_rn(diff, diff));
                    }
                }
            }
        } else {
            for (int t = 0; t < dsub; ++t) {
                const float ct = c[t];
#pragma unroll
                for (int pp = 0; pp < kIvfTabProbes; ++pp) {
                    if (pp < np) {                                // uniform
                        const float diff = __fsub_rn(lds[pp * D + j * dsub + t], ct);
                        acc[pp] = __fadd_rn(acc[pp], __fmul_rn(diff, diff));
                    }
                }
            }
        }
#pragma unroll
        for (int pp = 0; pp < kIvfTabProbes; ++pp) {
            if (pp >= np) continue;                               // uniform
            if (MODE == 0) {
                lo = fminf(lo, acc[pp]);
                if (keep) keep[((static_cast<size_t>(q) * nprobe + p0 + pp) * m + j) * kSmallSize + tid] = acc[pp];
            } else {
                qtab[((static_cast<size_t>(q) * nprobe + p0 + pp) * m + j) * kSmallSize + tid] =
                    quantize_entry(acc[pp], qmin, qmax);
            }
        }
    }
    if (MODE == 0) {
        lo = block_reduce(lo, false, red);
        if (tid == 0) atomicMin(&qmin_bits[q], __float_as_uint(lo));    // entries are >= +0
    }
}

// The quantization of entries kept by the first pass: qtab[e] = quantizer(keep[e]) with the bounds of the
// entry's query (per_query = nprobe * m * 256 entries each).
__global__ __launch_bounds__(256) void ivf_quantize_kept_kernel(const float *__restrict__ keep, size_t n, size_t per_query,
                                                               const float *__restrict__ bounds, uint8_t *__restrict__ qtab)
{
    const size_t e = (static_cast<size_t>(blockIdx.x) * blockDim.x + threadIdx.x) * 4;
    if (e >= n) return;                                         // n is a multiple of 256
    const size_t q = e / per_query;
    const float qmin = bounds[2 * q], qmax = bounds[2 * q + 1];
    const float4 v = *reinterpret_cast<const float4 *>(keep + e);
    uchar4 o;
    o.x = quantize_entry(v.x, qmin, qmax); o.y = quantize_entry(v.y, qmin, qmax);
    o.z = quantize_entry(v.z, qmin, qmax); o.w = quantize_entry(v.w, qmin, qmax);
    *reinterpret_cast<uchar4 *>(qtab + e) = o;
}

// qmax: largest small-table distance over the first min(r, total) codes met walking the probed
// lists in probe order (each code against its own list's residual).  One workgroup per query.
// Also finishes the bounds: (qmin, qmax), or (0, 0) when the probed lists are empty.
__global__ __launch_bounds__(256) void ivf_qmax_kernel(const float *__restrict__ queries, const float *__restrict__ coarse,
                                                      const int32_t *__restrict__ probe, int nprobe,
                                                      const float *__restrict__ derived, int m, int dsub,
                                                      const uint16_t *__restrict__ codes, const int64_t *__restrict__ offsets,
                                                      uint32_t r, const uint32_t *__restrict__ qmin_bits,
                                                      float *__restrict__ bounds)
{
    extern __shared__ __align__(16) float rho[];   // D floats: the query minus the centroid of the list being walked
    __shared__ uint64_t start[kIvfMaxProbe + 1];   // exclusive prefix of the list sizes in probe order
    __shared__ int lst[kIvfMaxProbe];
    __shared__ float red[4];
    const int q = blockIdx.x, tid = threadIdx.x;
    const int D = m * dsub;
    for (int p = tid; p < nprobe; p += 256) lst[p] = probe[static_cast<size_t>(q) * nprobe + p];
    __syncthreads();
    if (tid == 0) {
        uint64_t s = 0;
        for (int p = 0; p < nprobe; ++p) { start[p] = s; s += static_cast<uint64_t>(offsets[lst[p] + 1] - offsets[lst[p]]); }
        start[nprobe] = s;
    }
    __syncthreads();
    const uint64_t total = start[nprobe];
    const uint32_t n_first = static_cast<uint32_t>(total < r ? total : r);
    const float *y = queries + static_cast<size_t>(q) * D;
    const bool vec4 = (dsub & 3) == 0;               // centroid rows of whole 16-byte vectors (derived is 16-byte aligned)
    float hi = -INFINITY;
    // The walk takes the lists in probe order; the codes of one list share the residual of the query against
    // that list's centroid, which the workgroup works out once per list (the walk seldom leaves the first one).
    for (int p = 0; p < nprobe && start[p] < n_first; ++p) {              // uniform
        const uint32_t lo = static_cast<uint32_t>(start[p]);
        const uint32_t up = static_cast<uint32_t>(start[p + 1] < n_first ? start[p + 1] : n_first);
        if (up == lo) continue;                                           // an empty list (uniform)
        const int l = lst[p];
        const float *cl = coarse + static_cast<size_t>(l) * D;
        __syncthreads();                                                  // the previous list's residual is no longer read
        for (int t = tid; t < D; t += 256) rho[t] = __fsub_rn(y[t], cl[t]);
        __syncthreads();
        for (uint32_t i = lo + tid; i < up; i += 256) {
            const uint16_t *c = codes + (static_cast<size_t>(offsets[l]) + (i - lo)) * m;
            float d = 0.0f;
            for (int j = 0; j < m; ++j) {
                const float *cen = derived + (static_cast<size_t>(j) * kSmallSize + (c[j] & 255)) * dsub;
                const float *rj = rho + j * dsub;
                float acc = 0.0f;
                if (vec4) {
                    for (int t = 0; t < dsub; t += 4) {
                        const float4 cv = *reinterpret_cast<const float4 *>(cen + t);
                        const float d0 = __fsub_rn(rj[t], cv.x), d1 = __fsub_rn(rj[t + 1], cv.y);
                        const float d2 = __fsub_rn(rj[t + 2], cv.z), d3 = __fsub_rn(rj[t + 3], cv.w);
                        acc = __fadd_rn(acc, __fmul_rn(d0, d0)); acc = __fadd_rn(acc, __fmul_rn(d1, d1));
                        acc = __fadd_rn(acc, __fmul_rn(d2, d2)); acc = __fadd_rn(acc, __fmul_rn(d3, d3));
                    }
                } else {
                    for (int t = 0; t < dsub; ++t) {
                        const float diff = __fsub_rn(rj[t], cen[t]);
                        acc = __fadd_rn(acc, __fmul_rn(diff, diff));
                    }
                }
                d = j == 0 ? acc : __fadd_rn(d, acc);
            }
            hi = fmaxf(hi, d);
        }
    }
    hi = block_reduce(hi, true, red);
    if (tid == 0) {
        if (total == 0) { bounds[2 * q] = 0.0f; bounds[2 * q + 1] = 0.0f; }
        else { bounds[2 * q] = __uint_as_float(qmin_bits[q]); bounds[2 * q + 1] = hi; }
    }
}

// ------------------------------------------------------------------------------------------------
// Scan step: per-query unit lists.
// ------------------------------------------------------------------------------------------------
// One workgroup per query: probed lists sorted by list id (so that units follow increasing vector
// id), a unit size that keeps the query within kIvfUnitsPerQuery units, and the unit records.
__global__ __launch_bounds__(256) void ivf_plan_kernel(const int32_t *__restrict__ probe, int nprobe,
                                                      const int64_t *__restrict__ offsets, uint32_t r,
                                                      IvfUnit *__restrict__ units, uint32_t *__restrict__ nunits,
                                                      uint32_t *__restrict__ count, IvfUnit *__restrict__ sunits,
                                                      uint32_t *__restrict__ nsunits, uint32_t *__restrict__ probed)
{
    __shared__ uint64_t key[kIvfMaxProbe];         // (list id << 32) | probe position
    __shared__ uint32_t ubase[kIvfMaxProbe + 1];
    __shared__ uint32_t sbase[kIvfMaxProbe + 1];   // the same for the sample units
    __shared__ uint64_t lsize[kIvfMaxProbe];       // codes in the s-th probed list (lists in id order)
    __shared__ uint32_t s_unit;
    const int q = blockIdx.x, tid = threadIdx.x;
    uint32_t np2 = 1;
    while (np2 < static_cast<uint32_t>(nprobe)) np2 <<= 1;
    for (uint32_t p = tid; p < np2; p += 256)
        key[p] = p < static_cast<uint32_t>(nprobe)
                     ? make_key(static_cast<uint32_t>(probe[static_cast<size_t>(q) * nprobe + p]), p) : ~0ull;
    bitonic_sort(key, np2);
    // (the list sizes are fetched by all threads at once: the planning below is one thread's walk over them)
    for (int s = tid; s < nprobe; s += 256) {
        const int l = static_cast<int>(key[s] >> 32);
        lsize[s] = static_cast<uint64_t>(offsets[l + 1] - offsets[l]);
    }
    __syncthreads();
    if (tid == 0) {
        uint64_t total = 0;
        for (int s = 0; s < nprobe; ++s) total += lsize[s];
        // three units per probed list on average, and at least 512 less one per list in all (measured: fewer,
        // longer units leave the chip unevenly loaded, more of them pay the latency of a wavefront's first
        // loads too often); never more than the unit table holds
        uint64_t want = 4ull * nprobe < 512 ? 512 : 4ull * nprobe;
        if (want > static_cast<uint64_t>(kIvfUnitsPerQuery)) want = kIvfUnitsPerQuery;
        uint64_t unit = (total + (want - nprobe) - 1) / (want - nprobe);
        unit = (unit + 63) / 64 * 64;
        if (unit < 256) unit = 256;
        uint32_t u = 0, su = 0;
        for (int s = 0; s < nprobe; ++s) {
            const uint64_t size = lsize[s];
            ubase[s] = u;
            u += static_cast<uint32_t>((size + unit - 1) / unit);
            sbase[s] = su;                                   // (at most one unit per list and one per kIvfSampleStep scan units)
            su += static_cast<uint32_t>(((size + kIvfSampleStep - 1) / kIvfSampleStep + unit - 1) / unit);
        }
        ubase[nprobe] = u;
        sbase[nprobe] = su;
        nsunits[q] = su;
        s_unit = static_cast<uint32_t>(unit);
        nunits[q] = u;
        count[q] = static_cast<uint32_t>(total < r ? total : r);
        probed[q] = static_cast<uint32_t>(total < 0xFFFFFFFFull ? total : 0xFFFFFFFFull);     // codes in the probed lists
    }
    __syncthreads();
    const uint32_t unit = s_unit;
    // The sample that gives the scan its starting bound: the first ceil(size / kIvfSampleStep) codes of every probed
    // list (a list keeps its codes in no order that matters here), so that every list is in it with the same weight; cut
    // into units no longer than the scan's, so that a long list's share is not one wavefront's work.
    for (int s = 0; s < nprobe; ++s) {
        const int l = static_cast<int>(key[s] >> 32);
        const uint64_t lo = static_cast<uint64_t>(offsets[l]), size = static_cast<uint64_t>(offsets[l + 1]) - lo;
        const uint64_t part = (size + kIvfSampleStep - 1) / kIvfSampleStep;
        const uint32_t nu = sbase[s + 1] - sbase[s];
        for (uint32_t c = tid; c < nu; c += 256) {
            IvfUnit rec;
            rec.begin = lo + static_cast<uint64_t>(c) * unit;
            rec.count = static_cast<uint32_t>(min(static_cast<uint64_t>(unit), part - static_cast<uint64_t>(c) * unit));
            rec.p = static_cast<uint32_t>(key[s] & 0xFFFFFFFFu);
            sunits[static_cast<size_t>(q) * kIvfSampleUnits + sbase[s] + c] = rec;
        }
    }
    for (int s = 0; s < nprobe; ++s) {
        const int l = static_cast<int>(key[s] >> 32);
        const uint64_t lo = static_cast<uint64_t>(offsets[l]), size = static_cast<uint64_t>(offsets[l + 1]) - lo;
        const uint32_t nu = ubase[s + 1] - ubase[s];
        for (uint32_t c = tid; c < nu; c += 256) {
            IvfUnit rec;
            rec.begin = lo + static_cast<uint64_t>(c) * unit;
            rec.count = static_cast<uint32_t>(min(static_cast<uint64_t>(unit), size - static_cast<uint64_t>(c) * unit));
            rec.p = static_cast<uint32_t>(key[s] & 0xFFFFFFFFu);
            units[static_cast<size_t>(q) * kIvfUnitsPerQuery + ubase[s] + c] = rec;
        }
    }
}

enum IvfMode { kIvfHist = 0, kIvfTieCount = 1, kIvfCollect = 2 };
constexpr int kIvfAhead = 4;     // 64-code groups whose codes a wavefront loads together

// One wavefront per unit; grid (kIvfUnitsPerQuery / 4, nq), 256 threads.  The wavefront keeps the
// 8-bit tables of its (query, list) in its own LDS slot and walks the unit 64 codes at a time.
// CodeT: uint16_t (the codes as stored) or uint8_t (their low-byte plane).
// One (query, unit) by one wavefront; nothing in it waits for another wavefront.
template <int M, int MODE, typename CodeT>
__device__ inline void ivf_scan_unit(int q, const CodeT *__restrict__ codes, const IvfUnit *__restrict__ units,
                                     const uint32_t *__restrict__ nunits, const uint8_t *__restrict__ qtab,
                                     int nprobe, uint32_t r, uint32_t unit_step,
                                     const uint32_t *__restrict__ flags, uint32_t *__restrict__ hist,
                                     const uint32_t *__restrict__ thr, uint32_t *__restrict__ tie,
                                     uint32_t *__restrict__ counter, uint64_t *__restrict__ keys)
{
    extern __shared__ __align__(16) uint8_t smem[];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const uint32_t u = blockIdx.x * 4 + wave;
    uint8_t *tab = smem + wave * (M * 256);                                      // [M][256]
    uint32_t *lhist = reinterpret_cast<uint32_t *>(smem + 4 * M * 256) + wave * 256;   // kIvfHist only
    // every unit_step-th unit only (sampling), and only the queries with a flag when flags are given
    const bool active = u < nunits[q] && u % unit_step == 0 && (!flags || flags[q] != 0);
    IvfUnit un{0, 0, 0};
    if (active) un = units[static_cast<size_t>(q) * kIvfUnitsPerQuery + u];
    if (active) {
        const uint4 *src = reinterpret_cast<const uint4 *>(qtab + (static_cast<size_t>(q) * nprobe + un.p) * M * 256);
        uint4 *dst = reinterpret_cast<uint4 *>(tab);
        for (int v = lane; v < M * 256 / 16; v += 64) dst[v] = src[v];
        if (MODE == kIvfHist)
            for (int v = lane; v < 256; v += 64) lhist[v] = 0;
    }
    // the tables are this wavefront's own: its lanes run in lockstep, the fences order the LDS accesses
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    if (!active) return;

    uint32_t T = 0, aux = 0;
    if (MODE != kIvfHist) {
        T = thr[2 * q];
        if (MODE == kIvfCollect) aux = tie[static_cast<size_t>(q) * kIvfUnitsPerQuery + u];
    }
    // The unit is walked 64 codes at a time, in id order; the codes of kIvfAhead such groups are loaded
    // together, so that one memory latency covers all of them.
    for (uint32_t base0 = 0; base0 < un.count; base0 += 64 * kIvfAhead) {
        uint32_t low[kIvfAhead][M];
#pragma unroll
        for (int g = 0; g < kIvfAhead; ++g) {
            const uint32_t k = base0 + g * 64 + lane;
            if (k < un.count) {
                load_low_bytes<M>(codes, un.begin + k, low[g]);
            } else {
#pragma unroll
                for (int j = 0; j < M; ++j) low[g][j] = 0;
            }
        }
#pragma unroll
      for (int g = 0; g < kIvfAhead; ++g) {
        const uint32_t base = base0 + g * 64;
        if (base >= un.count) break;                                  // uniform
        const uint32_t k = base + lane;
        const bool live = k < un.count;
        const uint64_t id = un.begin + k;
        uint32_t s = 0;
#pragma unroll
        for (int j = 0; j < M; ++j) s += tab[j * 256 + low[g][j]];
        const uint32_t qd = min(s, 255u);
        if (MODE == kIvfHist) {
            if (live) atomicAdd(&lhist[qd], 1u);
        } else if (MODE == kIvfTieCount) {
            aux += __popcll(__ballot(live && qd == T));
        } else {
            const bool below = live && qd < T;
            const bool tied = live && qd == T;
            const uint64_t tied_mask = __ballot(tied);
            bool take = below;
            if (tied_mask) {
                const uint32_t rank = __popcll(tied_mask & ((1ull << lane) - 1ull));
                take = below || (tied && rank < aux);
                const uint32_t n_tied = __popcll(tied_mask);
                aux = aux > n_tied ? aux - n_tied : 0u;
            }
            const uint64_t take_mask = __ballot(take);
            if (take_mask) {
                uint32_t slot0 = 0;
                if (lane == 0) slot0 = atomicAdd(&counter[q], static_cast<uint32_t>(__popcll(take_mask)));
                slot0 = __shfl(slot0, 0, kWave);
                if (take) {
                    const uint32_t slot = slot0 + __popcll(take_mask & ((1ull << lane) - 1ull));
                    if (slot < r) keys[static_cast<size_t>(q) * r + slot] = make_key(qd, static_cast<uint32_t>(id));
                }
            }
        }
      }
    }
    if (MODE == kIvfHist) {
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        for (int v = lane; v < 256; v += 64) {
            const uint32_t c = lhist[v];
            if (c) atomicAdd(&hist[static_cast<size_t>(q) * 256 + v], c);
        }
    } else if (MODE == kIvfTieCount) {
        if (lane == 0) tie[static_cast<size_t>(q) * kIvfUnitsPerQuery + u] = aux;
    }
}

// Grid (kIvfUnitsPerQuery / 4, min(nq, kIvfRedoRows)): a wavefront takes the same unit number of every
// kIvfRedoRows-th query.  With flags given (nq of them and, as entry nq, whether any is set: ivf_any_flag_kernel)
// only flagged queries are scanned, and since that is the rare case
// (the three passes redo what the single pass could not finish) a row of workgroups serves many queries, so
// that a launch with nothing to do costs a few thousand empty workgroups, not one per (query, 4 units).
constexpr int kIvfRedoRows = 32;

// flags[nq] = whether any of flags[0 .. nq) is set.  One workgroup.
__global__ __launch_bounds__(1024) void ivf_any_flag_kernel(uint32_t *__restrict__ flags, int nq)
{
    __shared__ uint32_t any;
    if (threadIdx.x == 0) any = 0;
    __syncthreads();
    uint32_t mine = 0;
    for (int q = threadIdx.x; q < nq; q += 1024) mine |= flags[q];
    if (mine) any = 1;                                       // benign race: every writer stores 1
    __syncthreads();
    if (threadIdx.x == 0) flags[nq] = any;
}

template <int M, int MODE, typename CodeT>
__global__ __launch_bounds__(256) void ivf_scan_kernel(const CodeT *__restrict__ codes, const IvfUnit *__restrict__ units,
                                                      const uint32_t *__restrict__ nunits, const uint8_t *__restrict__ qtab,
                                                      int nprobe, int nq, uint32_t r, uint32_t unit_step,
                                                      const uint32_t *__restrict__ flags, uint32_t *__restrict__ hist,
                                                      const uint32_t *__restrict__ thr, uint32_t *__restrict__ tie,
                                                      uint32_t *__restrict__ counter, uint64_t *__restrict__ keys)
{
    if (flags && flags[nq] == 0) return;                     // no query is flagged: one load, not nq / gridDim.y
    for (int q = blockIdx.y; q < nq; q += gridDim.y) {
        if (flags && flags[q] == 0) continue;
        ivf_scan_unit<M, MODE, CodeT>(q, codes, units, nunits, qtab, nprobe, r, unit_step, flags, hist, thr, tie, counter, keys);
        // the next query's tables overwrite this one's: every lane is done with them
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    }
}

// The same scan in ONE pass over the probed lists (each pass reads every probed code from HBM, and no
// two queries share them, so passes are what the scan costs).  As in the flat single pass, a query has
// a running bucket bound, initialised from the histogram of a sample (the first 1 / kIvfSampleStep of every list) and
// lowered as exact per-bucket counts of appended candidates accumulate; pairs at or below the bound are
// appended to the query's sliced buffer, the exact r are selected afterwards, and a query whose buffer
// overflows (or whose lists hold fewer than r codes) is redone by the three passes above.
// Grid (nq, kIvfUnitsPerQuery / 4): the query index varies fastest, so only a few wavefronts of one
// query run at a time and the candidates waiting in their queues stay few against r.
//
// The kernel is bound by the stream of codes from HBM, so a wavefront is built around keeping that
// stream in flight: the codes stay in registers as loaded (their low bytes are picked out when they
// are looked up), in two sets of kIvfRawWords words per lane; while one set is processed the loads
// of the next are under way, the first of them issued together with the load of the unit's tables,
// and nothing in the kernel waits for another wavefront.
constexpr int kIvfRawWords = 16;         // registers per lane and set that hold codes in flight

// The bytes of code i as stored, in RW words (a narrower code is zero-extended).
template <int M, typename CodeT, int RW>
__device__ inline void load_raw_code(const CodeT *__restrict__ codes, uint64_t i, uint32_t (&w)[RW])
{
    constexpr int BPC = M * static_cast<int>(sizeof(CodeT));
    const uint8_t *p = reinterpret_cast<const uint8_t *>(codes) + i * BPC;
    if constexpr (BPC >= 16) {
#pragma unroll
        for (int v = 0; v < BPC / 16; ++v) {
            const uint4 x = reinterpret_cast<const uint4 *>(p)[v];
            w[4 * v] = x.x; w[4 * v + 1] = x.y; w[4 * v + 2] = x.z; w[4 * v + 3] = x.w;
        }
    } else if constexpr (BPC == 8) {
        const uint2 x = *reinterpret_cast<const uint2 *>(p);
        w[0] = x.x; w[1] = x.y;
    } else if constexpr (BPC == 4) {
        w[0] = *reinterpret_cast<const uint32_t *>(p);
    } else if constexpr (BPC == 2) {
        w[0] = *reinterpret_cast<const uint16_t *>(p);
    } else {
        w[0] = *p;
    }
}

// Low byte of sub-code j of a code held as loaded (property P1: the derived index is the low 8 bits).
template <typename CodeT, int RW>
__device__ inline uint32_t low_byte_of(const uint32_t (&w)[RW], int j)
{
    if constexpr (sizeof(CodeT) == 2) return (w[j >> 1] >> (16 * (j & 1))) & 255u;
    else return (w[j >> 2] >> (8 * (j & 3))) & 255u;
}

// SAMPLE: the pass that finds the starting bounds -- `units` and `nunits` are the sample's (the first
// 1 / kIvfSampleStep of every probed list), nothing is appended, and `count` is the per-query histogram of the
// integer distances ([nq][256]).
template <int M, typename CodeT, bool SAMPLE>
__global__ __launch_bounds__(256) void ivf_scan_single_kernel(const CodeT *__restrict__ codes,
                                                             const IvfUnit *__restrict__ units,
                                                             const uint32_t *__restrict__ nunits,
                                                             const uint8_t *__restrict__ qtab, int nprobe, uint32_t r,
                                                             uint32_t cap, uint32_t upd, uint32_t qflush, int *t_cur,
                                                             uint32_t *count, uint32_t *chist, uint64_t *__restrict__ keys)
{
    constexpr int BPC = M * static_cast<int>(sizeof(CodeT));
    constexpr int RW = BPC >= 4 ? BPC / 4 : 1;                // words per code
    constexpr int GPB = RW >= kIvfRawWords ? 1 : kIvfRawWords / RW;   // 64-code groups per set
    extern __shared__ __align__(16) uint8_t smem[];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int q = blockIdx.x;
    const uint32_t u = blockIdx.y * 4 + wave;
    // (SAMPLE: `units` and `nunits` are the sample's, kIvfSampleUnits records per query)
    if (u >= nunits[q]) return;                              // uniform per wavefront; the kernel has no workgroup barrier
    uint8_t *tab = smem + wave * (M * 256);                                           // [M][256]
    uint64_t *wq = reinterpret_cast<uint64_t *>(smem + 4 * M * 256) + wave * 64;      // pending candidates
    uint32_t *lhist = reinterpret_cast<uint32_t *>(smem + 4 * M * 256) + wave * 256;  // SAMPLE: this wavefront's histogram
    if constexpr (SAMPLE) {
#pragma unroll
        for (int b = 0; b < 4; ++b) lhist[lane + 64 * b] = 0;
    }
    const IvfUnit un = units[static_cast<size_t>(q) * (SAMPLE ? kIvfSampleUnits : kIvfUnitsPerQuery) + u];
    if (un.count == 0) return;                               // uniform (the planner makes no empty units)

    auto load_set = [&](uint32_t base0, uint32_t (&w)[GPB][RW]) {
#pragma unroll
        for (int g = 0; g < GPB; ++g) {
            const uint32_t k = base0 + g * 64 + lane;
            // past the end of the unit the last code is read again (a valid address); it is masked below
            load_raw_code<M, CodeT, RW>(codes, un.begin + (k < un.count ? k : un.count - 1), w[g]);
        }
    };
    auto load_bound = [&]() {
        if constexpr (SAMPLE) return 0;
        const int t = __hip_atomic_load(&t_cur[q], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        return t >= 255 ? 0x7fffffff : t;
    };
    // The unit's first codes and its tables travel together: the code loads are issued first, the table words
    // follow them and go from their registers straight to LDS.  (Held in an array across the code loads, the table
    // words were put in scratch memory by the compiler: 2 KB written and read back per wavefront, a gigabyte of
    // traffic per batch at 1024 queries x 64 lists.)
    uint32_t wa[GPB][RW], wb[GPB][RW];
    load_set(0, wa);
    int T = load_bound();
    {
        constexpr int NTW = M * 256 / 16;                                // 16-byte words of the tables
        const uint4 *src = reinterpret_cast<const uint4 *>(qtab + (static_cast<size_t>(q) * nprobe + un.p) * M * 256);
        uint4 *dst = reinterpret_cast<uint4 *>(tab);
#pragma unroll
        for (int v = 0; v < (NTW + 63) / 64; ++v)
            if (NTW % 64 == 0 || lane + 64 * v < NTW) dst[lane + 64 * v] = src[lane + 64 * v];
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

    const size_t cell = static_cast<size_t>(q) * kFastSlices + u % kFastSlices;
    uint32_t qlen = 0;                                   // wave-uniform
    auto flush = [&]() {
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        uint32_t first = 0;
        if (lane == 0) first = atomicAdd(&count[cell], qlen);
        first = __builtin_amdgcn_readfirstlane(__shfl(first, 0, kWave));
        if (static_cast<uint32_t>(lane) < qlen) {
            const uint64_t key = wq[lane];
            if (first + lane < cap) keys[cell * cap + first + lane] = key;
            else atomicMin(&t_cur[q], -1);               // slice full: stop appending, the query is redone
            atomicAdd(&chist[static_cast<size_t>(q) * 256 + static_cast<uint32_t>(key >> 32)], 1u);
        }
        if (first / upd != (first + qlen) / upd) lower_bound_of(q, r, t_cur, chist);   // uniform
        qlen = 0;
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    };
    auto process = [&](uint32_t base0, const uint32_t (&w)[GPB][RW], int bound) {
#pragma unroll
        for (int g = 0; g < GPB; ++g) {
            const uint32_t base = base0 + g * 64;
            if (base >= un.count) break;                              // uniform
            const uint32_t k = base + lane;
            uint32_t s = 0;
#pragma unroll
            for (int j = 0; j < M; ++j) s += tab[j * 256 + low_byte_of<CodeT, RW>(w[g], j)];
            const uint32_t qd = min(s, 255u);
            if constexpr (SAMPLE) {
                if (k < un.count) atomicAdd(&lhist[qd], 1u);
                continue;
            }
            const bool h = k < un.count && static_cast<int>(qd) <= bound;
            const uint64_t mask = __builtin_amdgcn_ballot_w64(h);
            if (!mask) continue;                                      // uniform
            const uint32_t cnt = __popcll(mask);
            if (qlen + cnt > 64) flush();                             // uniform
            if (h) {
                const uint32_t rank = __builtin_amdgcn_mbcnt_hi(static_cast<uint32_t>(mask >> 32),
                                                                __builtin_amdgcn_mbcnt_lo(static_cast<uint32_t>(mask), 0u));
                wq[qlen + rank] = make_key(qd, static_cast<uint32_t>(un.begin + k));
            }
            qlen = __builtin_amdgcn_readfirstlane(qlen + cnt);
            if (qlen >= qflush) flush();                              // uniform
        }
    };

    constexpr uint32_t SET = 64 * GPB;
    for (uint32_t base0 = 0; base0 < un.count; base0 += 2 * SET) {
        int Tn = T;
        if (base0 + SET < un.count) { load_set(base0 + SET, wb); Tn = load_bound(); }
        process(base0, wa, T);
        if (base0 + SET >= un.count) break;
        T = Tn;
        if (base0 + 2 * SET < un.count) { load_set(base0 + 2 * SET, wa); Tn = load_bound(); }
        process(base0 + SET, wb, T);
        T = Tn;
    }
    if constexpr (SAMPLE) {
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            const uint32_t c = lhist[lane + 64 * b];
            if (c) atomicAdd(&count[static_cast<size_t>(q) * 256 + lane + 64 * b], c);
        }
        return;
    }
    if (qlen) flush();
}

// ------------------------------------------------------------------------------------------------
// Refine step: Eq. 3 on residuals, double precision, then top-k.  One workgroup per query.
// ------------------------------------------------------------------------------------------------
template <int M>
__global__ __launch_bounds__(1024) void ivf_refine_kernel(const float *__restrict__ queries, const float *__restrict__ coarse,
                                                         const float *__restrict__ cb, int dsub,
                                                         const uint16_t *__restrict__ codes, const int64_t *__restrict__ offsets,
                                                         const int32_t *__restrict__ probe, int nprobe,
                                                         const uint32_t *__restrict__ cand_id, uint32_t r, uint32_t k,
                                                         uint32_t n_pow2, int use_lds, uint64_t *__restrict__ spill,
                                                         uint32_t *__restrict__ ids, float *__restrict__ dist)
{
    extern __shared__ __align__(16) uint8_t smem[];
    __shared__ uint32_t lbeg[kIvfMaxProbe], lend[kIvfMaxProbe];   // ids are 32-bit, so are list bounds
    __shared__ int lst[kIvfMaxProbe];
    const int q = blockIdx.x;
    const int D = M * dsub;
    for (int p = threadIdx.x; p < nprobe; p += blockDim.x) {
        const int l = probe[static_cast<size_t>(q) * nprobe + p];
        lst[p] = l;
        lbeg[p] = static_cast<uint32_t>(offsets[l]);
        lend[p] = static_cast<uint32_t>(offsets[l + 1]);
    }
    __syncthreads();
    uint64_t *a = use_lds ? reinterpret_cast<uint64_t *>(smem) : spill + static_cast<size_t>(q) * n_pow2;
    const float *y = queries + static_cast<size_t>(q) * D;
    // One lane per (candidate, sub-quantizer): the M lanes of a candidate are neighbours in a wavefront.  They
    // share the search for the candidate's list, each computes the squared distance of its own sub-vector
    // (components in ascending order), and the sums are added in ascending j, as a single thread would.
    {
        const uint32_t lane = threadIdx.x & 63u;
        const int j = static_cast<int>(threadIdx.x % M);
        const bool vec4 = (dsub & 3) == 0;
        for (uint32_t base = 0; base < n_pow2; base += blockDim.x / M) {      // uniform trip count
            const uint32_t t = base + threadIdx.x / M;
            uint32_t id = 0xFFFFFFFFu;
            if (t < r) id = cand_id[static_cast<size_t>(q) * r + t];
            int p = -1;                                                      // pad slots (id 0xFFFFFFFF) belong to no probed list
            for (int z = j; z < nprobe; z += M)
                if (id >= lbeg[z] && id < lend[z]) p = z;                    // the lists are disjoint: at most one
#pragma unroll
            for (int off = 1; off < M; off <<= 1) p = max(p, __shfl_xor(p, off));
            double dj = 0.0;
            if (p >= 0) {
                const float *cl = coarse + static_cast<size_t>(lst[p]) * D + j * dsub;
                const float *yj = y + j * dsub;
                const float *cen = cb + (static_cast<size_t>(j) * kFullSize + codes[static_cast<size_t>(id) * M + j]) * dsub;
                if (vec4) {
                    for (int tt = 0; tt < dsub; tt += 4) {
                        const float4 yv = *reinterpret_cast<const float4 *>(yj + tt);
                        const float4 lv = *reinterpret_cast<const float4 *>(cl + tt);
                        const float4 cv = *reinterpret_cast<const float4 *>(cen + tt);
                        double diff = (static_cast<double>(yv.x) - static_cast<double>(lv.x)) - static_cast<double>(cv.x);
                        dj += diff * diff;
                        diff = (static_cast<double>(yv.y) - static_cast<double>(lv.y)) - static_cast<double>(cv.y);
                        dj += diff * diff;
                        diff = (static_cast<double>(yv.z) - static_cast<double>(lv.z)) - static_cast<double>(cv.z);
                        dj += diff * diff;
                        diff = (static_cast<double>(yv.w) - static_cast<double>(lv.w)) - static_cast<double>(cv.w);
                        dj += diff * diff;
                    }
                } else {
                    for (int tt = 0; tt < dsub; ++tt) {
                        const double diff = (static_cast<double>(yj[tt]) - static_cast<double>(cl[tt])) - static_cast<double>(cen[tt]);
                        dj += diff * diff;
                    }
                }
            }
            double d = __shfl(dj, static_cast<int>(lane - j));
#pragma unroll
            for (int jj = 1; jj < M; ++jj) d += __shfl(dj, static_cast<int>(lane - j + jj));
            if (j == 0 && t < n_pow2) a[t] = p >= 0 ? make_key(__float_as_uint(static_cast<float>(d)), id) : ~0ull;
        }
    }
    bitonic_sort(a, n_pow2);
    for (uint32_t t = threadIdx.x; t < k; t += blockDim.x) {
        const uint64_t key = a[t];
        ids[static_cast<size_t>(q) * k + t] = static_cast<uint32_t>(key);
        dist[static_cast<size_t>(q) * k + t] = (key == ~0ull) ? INFINITY : __uint_as_float(static_cast<uint32_t>(key >> 32));
    }
}

// ------------------------------------------------------------------------------------------------
// host side
// ------------------------------------------------------------------------------------------------
struct IvfScanPlan {
    size_t off_hist, off_thr, off_counter, off_nunits, zero_bytes, off_tie, off_units, off_keys, off_spill, total;
    // single pass: sample histogram, cursors, appended histogram (cleared with the rest); bounds, flags, buffers
    size_t off_shist, off_fcount, off_chist, off_tcur, off_flags, off_fkeys, off_fsort, off_probed, off_sunits, off_nsunits;
    uint32_t cap, upd, qflush, sortcap;
};

static IvfScanPlan plan_ivf_scan(int nq, uint32_t r)
{
    IvfScanPlan p{};
    const size_t Q = static_cast<size_t>(nq);
    size_t off = 0;
    p.off_hist = off;    off = align_up(off + sizeof(uint32_t) * 256 * Q, 256);
    p.off_thr = off;     off = align_up(off + sizeof(uint32_t) * 2 * Q, 256);
    p.off_counter = off; off = align_up(off + sizeof(uint32_t) * Q, 256);
    p.off_nunits = off;  off = align_up(off + sizeof(uint32_t) * Q, 256);
    p.off_tie = off;     off = align_up(off + sizeof(uint32_t) * Q * kIvfUnitsPerQuery, 256);
    p.off_shist = off;   off = align_up(off + sizeof(uint32_t) * 256 * Q, 256);
    p.off_fcount = off;  off = align_up(off + sizeof(uint32_t) * Q * kFastSlices, 256);
    p.off_chist = off;   off = align_up(off + sizeof(uint32_t) * 256 * Q, 256);
    p.zero_bytes = off;  // everything above is cleared together
    p.off_units = off;   off = align_up(off + sizeof(IvfUnit) * Q * kIvfUnitsPerQuery, 256);
    p.off_keys = off;    off = align_up(off + sizeof(uint64_t) * Q * r, 256);
    p.off_spill = off;
    if (next_pow2(r) > kSortLdsKeys) off = align_up(off + sizeof(uint64_t) * Q * next_pow2(r), 256);
    p.cap = 2 * r < 1024 ? 1024 : 2 * r;                 // per slice; 32 r per query in all
    p.upd = r / 16 < 16 ? 16 : r / 16;                   // appends to one slice between bound updates
    // Pending candidates a wavefront may hold: the wavefronts of one query that run at the same time
    // (about 2048 workgroups of 4 are resident, the query index varies fastest) together keep at most r / 4
    // candidates away from the bound.
    {
        const size_t resident = 2048 / Q ? 2048 / Q : 1;
        const size_t waves = 4 * resident < static_cast<size_t>(kIvfUnitsPerQuery) ? 4 * resident : kIvfUnitsPerQuery;
        const size_t lim = r / 4 / waves;
        p.qflush = static_cast<uint32_t>(lim < 1 ? 1 : lim > 64 ? 64 : lim);
    }
    p.sortcap = next_pow2(2 * r) < kSortLdsKeys ? kSortLdsKeys : next_pow2(2 * r);
    p.off_tcur = off;    off = align_up(off + sizeof(int32_t) * Q, 256);
    p.off_flags = off;   off = align_up(off + sizeof(uint32_t) * (Q + 1), 256);     // and "any of them"
    p.off_probed = off;  off = align_up(off + sizeof(uint32_t) * Q, 256);
    p.off_sunits = off;  off = align_up(off + sizeof(IvfUnit) * Q * kIvfSampleUnits, 256);
    p.off_nsunits = off; off = align_up(off + sizeof(uint32_t) * Q, 256);
    p.off_fkeys = off;   off = align_up(off + sizeof(uint64_t) * Q * kFastSlices * p.cap, 256);
    p.off_fsort = off;
    if (p.sortcap > kSortLdsKeys) off = align_up(off + sizeof(uint64_t) * Q * p.sortcap, 256);
    p.total = off;
    return p;
}

template <int M, typename CodeT>
static int ivf_scan_m(const CodeT *codes, const int64_t *offsets, const int32_t *probe, int nprobe,
                      const uint8_t *qtab, int nq, uint32_t r, uint32_t *cand_id, uint8_t *cand_qd, uint32_t *count,
                      uint8_t *base, hipStream_t st)
{
    const IvfScanPlan p = plan_ivf_scan(nq, r);
    uint32_t *hist = reinterpret_cast<uint32_t *>(base + p.off_hist);
    uint32_t *thr = reinterpret_cast<uint32_t *>(base + p.off_thr);
    uint32_t *counter = reinterpret_cast<uint32_t *>(base + p.off_counter);
    uint32_t *nunits = reinterpret_cast<uint32_t *>(base + p.off_nunits);
    uint32_t *tie = reinterpret_cast<uint32_t *>(base + p.off_tie);
    IvfUnit *units = reinterpret_cast<IvfUnit *>(base + p.off_units);
    uint64_t *keys = reinterpret_cast<uint64_t *>(base + p.off_keys);
    uint64_t *spill = reinterpret_cast<uint64_t *>(base + p.off_spill);
    int rc = launch_zero_words(reinterpret_cast<uint32_t *>(base), p.zero_bytes / 4, st);
    if (rc) return rc;
    rc = launch_fill_u64(keys, static_cast<size_t>(nq) * r, ~0ull, st);     // unused slots read as padding
    if (rc) return rc;
    uint32_t *probed = reinterpret_cast<uint32_t *>(base + p.off_probed);
    IvfUnit *sunits = reinterpret_cast<IvfUnit *>(base + p.off_sunits);
    uint32_t *nsunits = reinterpret_cast<uint32_t *>(base + p.off_nsunits);
    DCPQ_LAUNCH(kStageIvf, st, ivf_plan_kernel, dim3(nq), dim3(256), 0, probe, nprobe, offsets, r, units, nunits, count, sunits,
                nsunits, probed);
    DCPQ_CHECK_LAUNCH("ivf_plan_kernel");
    const dim3 grid(kIvfUnitsPerQuery / 4, nq < kIvfRedoRows ? nq : kIvfRedoRows);
    const size_t lds_tab = 4 * M * 256;
    uint32_t *shist = reinterpret_cast<uint32_t *>(base + p.off_shist);
    uint32_t *fcount = reinterpret_cast<uint32_t *>(base + p.off_fcount);
    uint32_t *chist = reinterpret_cast<uint32_t *>(base + p.off_chist);
    int *t_cur = reinterpret_cast<int *>(base + p.off_tcur);
    uint32_t *flags = reinterpret_cast<uint32_t *>(base + p.off_flags);
    uint64_t *fkeys = reinterpret_cast<uint64_t *>(base + p.off_fkeys);
    uint64_t *fsort = reinterpret_cast<uint64_t *>(base + p.off_fsort);
    // single pass: bounds from a sample of the probed lists, one pass over all their units, exact selection
    DCPQ_LAUNCH(kStageIvf, st, (ivf_scan_single_kernel<M, CodeT, true>),
                dim3(nq, (nprobe + kIvfUnitsPerQuery / kIvfSampleStep + 3) / 4), dim3(256),
                lds_tab + 4 * 256 * 4, codes, sunits, nsunits, qtab, nprobe, r, p.cap, p.upd, p.qflush, t_cur, shist, chist, fkeys);
    DCPQ_CHECK_LAUNCH("ivf_scan_single_kernel<sample>");
    // As in the flat scan, the bound starts at the bucket where the sample's count reaches what r codes of all the
    // query's probed codes would leave in a sample of that size, plus slack; a query whose bucket holds fewer than
    // r codes after all is flagged by the selection and redone below.
    rc = launch_sample_threshold(shist, nq, r, 0, t_cur, st, probed);
    if (rc) return rc;
    DCPQ_LAUNCH(kStageIvfScan, st, (ivf_scan_single_kernel<M, CodeT, false>), dim3(nq, kIvfUnitsPerQuery / 4), dim3(256),
                lds_tab + 4 * 64 * 8, codes, units, nunits, qtab, nprobe, r, p.cap, p.upd, p.qflush, t_cur, fcount, chist,
                fkeys);
    DCPQ_CHECK_LAUNCH("ivf_scan_single_kernel");
    rc = launch_fast_select(fkeys, fcount, chist, nq, r, kFastSlices, p.cap, p.sortcap, 0, fsort, cand_id, cand_qd, flags, st);
    if (rc) return rc;
    DCPQ_LAUNCH(kStageIvf, st, ivf_any_flag_kernel, dim3(1), dim3(1024), 0, flags, nq);
    DCPQ_CHECK_LAUNCH("ivf_any_flag_kernel");
    // the queries it flagged (a full slice, or fewer than r codes in the probed lists): three passes
    DCPQ_LAUNCH(kStageIvf, st, (ivf_scan_kernel<M, kIvfHist, CodeT>), grid, dim3(256), lds_tab + 4 * 256 * 4, codes, units,
                nunits, qtab, nprobe, nq, r, 1u, flags, hist, thr, tie, counter, keys);
    DCPQ_CHECK_LAUNCH("ivf_scan_kernel<hist>");
    rc = launch_threshold(hist, nq, r, thr, st);
    if (rc) return rc;
    DCPQ_LAUNCH(kStageIvf, st, (ivf_scan_kernel<M, kIvfTieCount, CodeT>), grid, dim3(256), lds_tab, codes, units, nunits, qtab,
                nprobe, nq, r, 1u, flags, hist, thr, tie, counter, keys);
    DCPQ_CHECK_LAUNCH("ivf_scan_kernel<tiecount>");
    rc = launch_tie_quota(tie, kIvfUnitsPerQuery, nq, thr, st);
    if (rc) return rc;
    DCPQ_LAUNCH(kStageIvf, st, (ivf_scan_kernel<M, kIvfCollect, CodeT>), grid, dim3(256), lds_tab, codes, units, nunits, qtab,
                nprobe, nq, r, 1u, flags, hist, thr, tie, counter, keys);
    DCPQ_CHECK_LAUNCH("ivf_scan_kernel<collect>");
    return launch_sort_candidates(keys, nq, r, spill, cand_id, cand_qd, st, flags);
}

static int ivf_check_common(const char *what, int nq, int m, int dsub, int nlist, int nprobe)
{
    DCPQ_REQUIRE(nq >= 0, "%s: nq=%d", what, nq);
    if (!dcpq_shape_supported(m, dsub)) return fail(DCPQ_EUNSUPPORTED, "%s: m=%d dsub=%d not supported", what, m, dsub);
    DCPQ_REQUIRE(nlist >= 1 && nprobe >= 1 && nprobe <= nlist, "%s: needs 1 <= nprobe <= nlist (nprobe=%d nlist=%d)", what, nprobe, nlist);
    if (nprobe > kIvfMaxProbe) return fail(DCPQ_EUNSUPPORTED, "%s: nprobe=%d above the supported %d", what, nprobe, kIvfMaxProbe);
    return DCPQ_OK;
}

}  // namespace dcpq

using namespace dcpq;

extern "C" size_t dcpq_ivf_probe_workspace_bytes(int nq, int nlist)
{
    if (nq <= 0 || nlist <= 0) return 0;
    return align_up(sizeof(float) * static_cast<size_t>(nq) * nlist, 256);
}

extern "C" int dcpq_ivf_probe(const float *queries, int nq, int D, const float *coarse, int nlist, int nprobe,
                              int32_t *probe, void *workspace, size_t workspace_bytes, void *stream)
{
    clear_error();
    DCPQ_REQUIRE(nq >= 0 && D >= 1, "ivf_probe: nq=%d D=%d", nq, D);
    DCPQ_REQUIRE(nlist >= 1 && nprobe >= 1 && nprobe <= nlist, "ivf_probe: needs 1 <= nprobe <= nlist");
    if (nprobe > kIvfMaxProbe) return fail(DCPQ_EUNSUPPORTED, "ivf_probe: nprobe=%d above the supported %d", nprobe, kIvfMaxProbe);
    if (nq == 0) return DCPQ_OK;
    DCPQ_REQUIRE(queries && coarse && probe && workspace, "ivf_probe: null pointer");
    DCPQ_REQUIRE((reinterpret_cast<uintptr_t>(workspace) & 255) == 0, "ivf_probe: workspace must be 256-byte aligned");
    const size_t need = dcpq_ivf_probe_workspace_bytes(nq, nlist);
    if (workspace_bytes < need) return fail(DCPQ_EWORKSPACE, "ivf_probe: workspace %zu < %zu bytes", workspace_bytes, need);
    hipStream_t st = as_stream(stream);
    float *dist = static_cast<float *>(workspace);
    int rc = launch_distance_tables(queries, nq, coarse, 1, D, nlist, dist, kStageIvfProbe, st);
    if (rc) return rc;
    DCPQ_LAUNCH(kStageIvfProbe, st, ivf_select_probe_kernel, dim3(nq), dim3(1024), 0, dist, nlist, nprobe, probe);
    DCPQ_CHECK_LAUNCH("ivf_select_probe_kernel");
    return DCPQ_OK;
}

extern "C" size_t dcpq_ivf_tables_workspace_bytes(int nq) { return nq > 0 ? align_up(sizeof(uint32_t) * static_cast<size_t>(nq), 256) : 0; }

// With this much workspace (or more) dcpq_ivf_build_small_tables keeps the entries of its first pass and
// quantizes them from memory instead of computing them twice.
extern "C" size_t dcpq_ivf_tables_workspace_bytes_fast(int nq, int nprobe, int m)
{
    if (nq <= 0 || nprobe <= 0 || !m_supported(m)) return 0;
    return dcpq_ivf_tables_workspace_bytes(nq) + align_up(sizeof(float) * static_cast<size_t>(nq) * nprobe * m * kSmallSize, 256);
}

extern "C" int dcpq_ivf_build_small_tables(const float *queries, int nq, const float *coarse, int nlist,
                                           const int32_t *probe, int nprobe, const float *derived, int m, int dsub,
                                           const uint16_t *codes, const int64_t *offsets, uint32_t r, uint8_t *qtab,
                                           float *bounds, void *workspace, size_t workspace_bytes, void *stream)
{
    clear_error();
    int rc = ivf_check_common("ivf_build_small_tables", nq, m, dsub, nlist, nprobe);
    if (rc) return rc;
    DCPQ_REQUIRE(r >= 1, "ivf_build_small_tables: r=%u", r);
    if (nq == 0) return DCPQ_OK;
    DCPQ_REQUIRE(queries && coarse && probe && derived && codes && offsets && qtab && bounds && workspace,
                 "ivf_build_small_tables: null pointer");
    DCPQ_REQUIRE((reinterpret_cast<uintptr_t>(derived) & 15) == 0, "ivf_build_small_tables: derived must be 16-byte aligned");
    if (workspace_bytes < dcpq_ivf_tables_workspace_bytes(nq))
        return fail(DCPQ_EWORKSPACE, "ivf_build_small_tables: workspace too small");
    hipStream_t st = as_stream(stream);
    uint32_t *qmin_bits = static_cast<uint32_t *>(workspace);
    // +inf as the starting minimum
    rc = launch_fill_u64(reinterpret_cast<uint64_t *>(qmin_bits), (static_cast<size_t>(nq) + 1) / 2, 0x7f8000007f800000ull, st);
    if (rc) return rc;
    const size_t lds = sizeof(float) * static_cast<size_t>(kIvfTabProbes) * m * dsub;
    const dim3 tgrid((nprobe + kIvfTabProbes - 1) / kIvfTabProbes, nq);
    if (lds > 64 * 1024) {                  // LDS above 64 KiB must be requested per kernel (at most 128 KiB here)
        const int most = static_cast<int>(sizeof(float) * kIvfTabProbes * 32 * 128);
        rc = allow_dynamic_lds(reinterpret_cast<const void *>(&ivf_tables_kernel<0>), most);
        if (rc) return rc;
        rc = allow_dynamic_lds(reinterpret_cast<const void *>(&ivf_tables_kernel<1>), most);
        if (rc) return rc;
    }
    // with room for them, the entries are kept by the first pass and quantized from memory
    const size_t n_entries = static_cast<size_t>(nq) * nprobe * m * kSmallSize;
    float *keep = nullptr;
    if (workspace_bytes >= dcpq_ivf_tables_workspace_bytes_fast(nq, nprobe, m))
        keep = reinterpret_cast<float *>(static_cast<uint8_t *>(workspace) + dcpq_ivf_tables_workspace_bytes(nq));
    DCPQ_LAUNCH(kStageIvfTables, st, ivf_tables_kernel<0>, tgrid, dim3(256), lds, queries, coarse, probe, nprobe,
                derived, m, dsub, qmin_bits, bounds, qtab, keep);
    DCPQ_CHECK_LAUNCH("ivf_tables_kernel<min>");
    DCPQ_LAUNCH(kStageIvfTables, st, ivf_qmax_kernel, dim3(nq), dim3(256), sizeof(float) * m * dsub, queries, coarse, probe, nprobe, derived, m, dsub,
                codes, offsets, r, qmin_bits, bounds);
    DCPQ_CHECK_LAUNCH("ivf_qmax_kernel");
    if (keep) {
        DCPQ_LAUNCH(kStageIvfTables, st, ivf_quantize_kept_kernel, dim3(static_cast<unsigned>((n_entries / 4 + 255) / 256)), dim3(256),
                    0, keep, n_entries, static_cast<size_t>(nprobe) * m * kSmallSize, bounds, qtab);
        DCPQ_CHECK_LAUNCH("ivf_quantize_kept_kernel");
    } else {
        DCPQ_LAUNCH(kStageIvfTables, st, ivf_tables_kernel<1>, tgrid, dim3(256), lds, queries, coarse, probe, nprobe,
                    derived, m, dsub, qmin_bits, bounds, qtab, nullptr);
        DCPQ_CHECK_LAUNCH("ivf_tables_kernel<quantize>");
    }
    return DCPQ_OK;
}

extern "C" size_t dcpq_ivf_scan_workspace_bytes(int nq, uint32_t r)
{
    if (nq <= 0 || r == 0) return 0;
    return plan_ivf_scan(nq, r).total;
}

template <typename CodeT>
static int ivf_scan_checked(const char *what, const CodeT *codes, const int64_t *offsets, int nlist, int m,
                            const int32_t *probe, int nprobe, const uint8_t *qtab, int nq, uint32_t r,
                            uint32_t *cand_id, uint8_t *cand_qd, uint32_t *count, void *workspace,
                            size_t workspace_bytes, void *stream)
{
    clear_error();
    int rc = ivf_check_common(what, nq, m, 1, nlist, nprobe);
    if (rc) return rc;
    DCPQ_REQUIRE(r >= 1 && r <= (1u << 26), "%s: r=%u out of range", what, r);
    if (nq == 0) return DCPQ_OK;
    DCPQ_REQUIRE(codes && offsets && probe && qtab && cand_id && cand_qd && count && workspace, "%s: null pointer", what);
    DCPQ_REQUIRE((reinterpret_cast<uintptr_t>(workspace) & 255) == 0, "%s: workspace must be 256-byte aligned", what);
    DCPQ_REQUIRE((reinterpret_cast<uintptr_t>(qtab) & 15) == 0 && (reinterpret_cast<uintptr_t>(codes) & 15) == 0,
                 "%s: codes and qtab must be 16-byte aligned", what);
    if (workspace_bytes < dcpq_ivf_scan_workspace_bytes(nq, r))
        return fail(DCPQ_EWORKSPACE, "%s: workspace %zu < %zu bytes", what, workspace_bytes, dcpq_ivf_scan_workspace_bytes(nq, r));
    hipStream_t st = as_stream(stream);
    uint8_t *base = static_cast<uint8_t *>(workspace);
    switch (m) {
        case 1: return ivf_scan_m<1>(codes, offsets, probe, nprobe, qtab, nq, r, cand_id, cand_qd, count, base, st);
        case 2: return ivf_scan_m<2>(codes, offsets, probe, nprobe, qtab, nq, r, cand_id, cand_qd, count, base, st);
        case 4: return ivf_scan_m<4>(codes, offsets, probe, nprobe, qtab, nq, r, cand_id, cand_qd, count, base, st);
        case 8: return ivf_scan_m<8>(codes, offsets, probe, nprobe, qtab, nq, r, cand_id, cand_qd, count, base, st);
        case 16: return ivf_scan_m<16>(codes, offsets, probe, nprobe, qtab, nq, r, cand_id, cand_qd, count, base, st);
        case 32: return ivf_scan_m<32>(codes, offsets, probe, nprobe, qtab, nq, r, cand_id, cand_qd, count, base, st);
        default: return fail(DCPQ_EUNSUPPORTED, "m=%d not supported", m);
    }
}

extern "C" int dcpq_ivf_scan_candidates(const uint16_t *codes, const int64_t *offsets, int nlist, int m,
                                        const int32_t *probe, int nprobe, const uint8_t *qtab, int nq, uint32_t r,
                                        uint32_t *cand_id, uint8_t *cand_qd, uint32_t *count, void *workspace,
                                        size_t workspace_bytes, void *stream)
{
    return ivf_scan_checked("ivf_scan_candidates", codes, offsets, nlist, m, probe, nprobe, qtab, nq, r, cand_id, cand_qd,
                            count, workspace, workspace_bytes, stream);
}

extern "C" int dcpq_ivf_scan_candidates_packed(const uint8_t *plane, const int64_t *offsets, int nlist, int m,
                                               const int32_t *probe, int nprobe, const uint8_t *qtab, int nq,
                                               uint32_t r, uint32_t *cand_id, uint8_t *cand_qd, uint32_t *count,
                                               void *workspace, size_t workspace_bytes, void *stream)
{
    return ivf_scan_checked("ivf_scan_candidates_packed", plane, offsets, nlist, m, probe, nprobe, qtab, nq, r, cand_id,
                            cand_qd, count, workspace, workspace_bytes, stream);
}

namespace dcpq {
// plane[i][j] = codes[i][j] & 255, eight sub-codes per thread
__global__ __launch_bounds__(256) void pack_low_bytes_kernel(const uint16_t *__restrict__ codes, uint64_t nsub,
                                                            uint8_t *__restrict__ plane)
{
    const uint64_t t = static_cast<uint64_t>(blockIdx.x) * 256 + threadIdx.x;     // 8 sub-codes per thread
    const uint64_t i = t * 8;
    if (i + 8 <= nsub) {
        const uint4 x = *reinterpret_cast<const uint4 *>(codes + i);
        uint2 o;
        o.x = (x.x & 255u) | ((x.x >> 8) & 0xff00u) | ((x.y & 255u) << 16) | ((x.y << 8) & 0xff000000u);
        o.y = (x.z & 255u) | ((x.z >> 8) & 0xff00u) | ((x.w & 255u) << 16) | ((x.w << 8) & 0xff000000u);
        *reinterpret_cast<uint2 *>(plane + i) = o;
    } else {
        for (uint64_t k = i; k < nsub; ++k) plane[k] = static_cast<uint8_t>(codes[k] & 255u);
    }
}
}  // namespace dcpq

extern "C" int dcpq_pack_low_bytes(const uint16_t *codes, uint64_t n_codes, int m, uint8_t *plane, void *stream)
{
    clear_error();
    DCPQ_REQUIRE(m >= 1 && m <= 64, "pack_low_bytes: m=%d", m);
    if (n_codes == 0) return DCPQ_OK;
    DCPQ_REQUIRE(codes && plane, "pack_low_bytes: null pointer");
    DCPQ_REQUIRE((reinterpret_cast<uintptr_t>(codes) & 15) == 0 && (reinterpret_cast<uintptr_t>(plane) & 15) == 0,
                 "pack_low_bytes: codes and plane must be 16-byte aligned");
    const uint64_t nsub = n_codes * static_cast<uint64_t>(m);
    const uint64_t nthreads = (nsub + 7) / 8;
    hipStream_t st = as_stream(stream);
    DCPQ_LAUNCH(kStageMisc, st, pack_low_bytes_kernel, dim3(static_cast<unsigned>((nthreads + 255) / 256)), dim3(256), 0,
                codes, nsub, plane);
    DCPQ_CHECK_LAUNCH("pack_low_bytes_kernel");
    return DCPQ_OK;
}

extern "C" size_t dcpq_ivf_refine_workspace_bytes(int nq, uint32_t r)
{
    if (nq <= 0 || r == 0) return 0;
    const uint32_t np2 = next_pow2(r);
    return np2 <= kSortLdsKeys ? 0 : sizeof(uint64_t) * static_cast<size_t>(nq) * np2;
}

extern "C" int dcpq_ivf_refine_topk(const float *queries, const float *coarse, int nlist, const float *codebooks, int m,
                                    int dsub, const uint16_t *codes, const int64_t *offsets, const int32_t *probe,
                                    int nprobe, const uint32_t *cand_id, int nq, uint32_t r, uint32_t k, uint32_t *ids,
                                    float *dist, void *workspace, size_t workspace_bytes, void *stream)
{
    clear_error();
    int rc = ivf_check_common("ivf_refine_topk", nq, m, dsub, nlist, nprobe);
    if (rc) return rc;
    DCPQ_REQUIRE(k >= 1 && k <= r, "ivf_refine_topk: needs 1 <= k <= r (k=%u r=%u)", k, r);
    if (nq == 0) return DCPQ_OK;
    DCPQ_REQUIRE(queries && coarse && codebooks && codes && offsets && probe && cand_id && ids && dist, "ivf_refine_topk: null pointer");
    DCPQ_REQUIRE(((reinterpret_cast<uintptr_t>(queries) | reinterpret_cast<uintptr_t>(coarse) | reinterpret_cast<uintptr_t>(codebooks)) & 15) == 0,
                 "ivf_refine_topk: queries, coarse and codebooks must be 16-byte aligned");
    const size_t need = dcpq_ivf_refine_workspace_bytes(nq, r);
    if (need && (!workspace || workspace_bytes < need)) return fail(DCPQ_EWORKSPACE, "ivf_refine_topk: workspace too small");
    hipStream_t st = as_stream(stream);
    const uint32_t np2 = next_pow2(r);
    const int use_lds = np2 <= kSortLdsKeys;
    const size_t lds = use_lds ? sizeof(uint64_t) * np2 : 0;
    uint64_t *spill = static_cast<uint64_t *>(workspace);
#define DCPQ_LAUNCH_IVF_REFINE(MV)                                                                                   \
    case MV:                                                                                                         \
        DCPQ_CHECK_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(&ivf_refine_kernel<MV>),                  \
                                           hipFuncAttributeMaxDynamicSharedMemorySize,                              \
                                           static_cast<int>(sizeof(uint64_t) * kSortLdsKeys)));                      \
        DCPQ_LAUNCH(kStageIvfRefine, st, ivf_refine_kernel<MV>, dim3(nq), dim3(1024), lds, queries, coarse, codebooks, dsub, \
                    codes, offsets, probe, nprobe, cand_id, r, k, np2, use_lds, spill, ids, dist);                   \
        break;
    switch (m) {
        DCPQ_LAUNCH_IVF_REFINE(1) DCPQ_LAUNCH_IVF_REFINE(2) DCPQ_LAUNCH_IVF_REFINE(4) DCPQ_LAUNCH_IVF_REFINE(8)
        DCPQ_LAUNCH_IVF_REFINE(16) DCPQ_LAUNCH_IVF_REFINE(32)
        default: return fail(DCPQ_EUNSUPPORTED, "m=%d not supported", m);
    }
#undef DCPQ_LAUNCH_IVF_REFINE
    DCPQ_CHECK_LAUNCH("ivf_refine_kernel");
    return DCPQ_OK;
}

// ---- the whole inverted-index search in one call ------------------------------------------------
namespace {
struct IvfSearchPlan {
    size_t off_probe, off_qtab, off_bounds, off_cand_id, off_cand_qd, off_count, off_sub, sub_bytes, total;
};
IvfSearchPlan plan_ivf_search(int nq, int nlist, int nprobe, int m, uint32_t r)
{
    IvfSearchPlan p{};
    const size_t Q = static_cast<size_t>(nq);
    size_t off = 0;
    p.off_probe = off;   off = align_up(off + sizeof(int32_t) * Q * nprobe, 256);
    p.off_qtab = off;    off = align_up(off + Q * nprobe * m * kSmallSize, 256);
    p.off_bounds = off;  off = align_up(off + sizeof(float) * 2 * Q, 256);
    p.off_cand_id = off; off = align_up(off + sizeof(uint32_t) * Q * r, 256);
    p.off_cand_qd = off; off = align_up(off + Q * r, 256);
    p.off_count = off;   off = align_up(off + sizeof(uint32_t) * Q, 256);
    // the four steps run one after the other on the stream and share one scratch region
    size_t sub = dcpq_ivf_probe_workspace_bytes(nq, nlist);
    // (the small-table entries are kept between the two table passes when that takes no more than 2 GiB)
    const size_t keep_tables = dcpq_ivf_tables_workspace_bytes_fast(nq, nprobe, m);
    const size_t others[] = {keep_tables <= (static_cast<size_t>(2) << 30) ? keep_tables : dcpq_ivf_tables_workspace_bytes(nq),
                             dcpq_ivf_scan_workspace_bytes(nq, r),
                             dcpq_ivf_refine_workspace_bytes(nq, r)};
    for (size_t o : others) sub = o > sub ? o : sub;
    p.off_sub = off;     p.sub_bytes = align_up(sub, 256); off += p.sub_bytes;
    p.total = off;
    return p;
}
}  // namespace

extern "C" size_t dcpq_ivf_search_workspace_bytes(int nq, int nlist, int nprobe, int m, uint32_t r)
{
    if (nq <= 0 || nlist <= 0 || nprobe <= 0 || nprobe > nlist || !m_supported(m) || r == 0 || r > (1u << 26)) return 0;
    return plan_ivf_search(nq, nlist, nprobe, m, r).total;
}

extern "C" int dcpq_ivf_search(const float *queries, int nq, const float *coarse, int nlist, int nprobe,
                               const float *codebooks, const float *derived, int m, int dsub, const uint16_t *codes,
                               const uint8_t *plane, const int64_t *offsets, uint32_t r, uint32_t k, uint32_t *ids,
                               float *dist, void *workspace, size_t workspace_bytes, void *stream)
{
    clear_error();
    int rc = ivf_check_common("ivf_search", nq, m, dsub, nlist, nprobe);
    if (rc) return rc;
    DCPQ_REQUIRE(r >= 1 && r <= (1u << 26) && k >= 1 && k <= r, "ivf_search: needs 1 <= k <= r <= 2^26 (k=%u r=%u)", k, r);
    if (nq == 0) return DCPQ_OK;
    DCPQ_REQUIRE(queries && coarse && codebooks && derived && codes && offsets && ids && dist && workspace,
                 "ivf_search: null pointer");
    DCPQ_REQUIRE((reinterpret_cast<uintptr_t>(workspace) & 255) == 0, "ivf_search: workspace must be 256-byte aligned");
    const IvfSearchPlan p = plan_ivf_search(nq, nlist, nprobe, m, r);
    if (workspace_bytes < p.total) return fail(DCPQ_EWORKSPACE, "ivf_search: workspace %zu < %zu bytes", workspace_bytes, p.total);
    uint8_t *base = static_cast<uint8_t *>(workspace);
    int32_t *probe = reinterpret_cast<int32_t *>(base + p.off_probe);
    uint8_t *qtab = base + p.off_qtab;
    float *bounds = reinterpret_cast<float *>(base + p.off_bounds);
    uint32_t *cand_id = reinterpret_cast<uint32_t *>(base + p.off_cand_id);
    uint8_t *cand_qd = base + p.off_cand_qd;
    uint32_t *count = reinterpret_cast<uint32_t *>(base + p.off_count);
    void *sub = base + p.off_sub;
    rc = dcpq_ivf_probe(queries, nq, m * dsub, coarse, nlist, nprobe, probe, sub, p.sub_bytes, stream);
    if (rc) return rc;
    rc = dcpq_ivf_build_small_tables(queries, nq, coarse, nlist, probe, nprobe, derived, m, dsub, codes, offsets, r, qtab,
                                     bounds, sub, p.sub_bytes, stream);
    if (rc) return rc;
    rc = plane ? dcpq_ivf_scan_candidates_packed(plane, offsets, nlist, m, probe, nprobe, qtab, nq, r, cand_id, cand_qd,
                                                 count, sub, p.sub_bytes, stream)
               : dcpq_ivf_scan_candidates(codes, offsets, nlist, m, probe, nprobe, qtab, nq, r, cand_id, cand_qd, count, sub,
                                          p.sub_bytes, stream);
    if (rc) return rc;
    return dcpq_ivf_refine_topk(queries, coarse, nlist, codebooks, m, dsub, codes, offsets, probe, nprobe, cand_id, nq, r,
                                k, ids, dist, sub, p.sub_bytes, stream);
}
