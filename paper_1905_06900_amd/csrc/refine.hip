// Pass two of Alg. 3 (Sec. 3.3, "Refine step"): exact asymmetric distance (Eq. 2) of every
// candidate from the full tables, then the result set of the k smallest by (distance, id).
// One workgroup per query: the r keys (distance bits, id) are built in LDS (or in a global spill
// area when they do not fit).  Only k << r of them are wanted, so the keys are first cut down by
// value: a histogram over 2048 equal steps between the smallest and the largest distance locates
// the step that holds the k-th smallest, the keys up to that step (a superset of the k smallest,
// usually little more than k) are gathered and only those are sorted, by the exact (distance, id)
// key.  When that superset is large (many equal distances) all r keys are sorted instead.
// Squared distances are non-negative, so their fp32 bit patterns order like the values.
#include <type_traits>

#include "common.h"
#include "device_util.h"

namespace dcpq {

constexpr uint32_t kRefineLdsKeys = 8192;   // 64 KiB of keys
constexpr uint32_t kRefineSteps = 2048;     // histogram steps between the smallest and the largest distance
constexpr uint32_t kRefineFew = 1024;       // keys gathered and sorted when the cut leaves no more than this

static uint32_t next_pow2_r(uint32_t x)
{
    uint32_t p = 1;
    while (p < x) p <<= 1;
    return p;
}

constexpr int kFromTables = 0, kOnDemand = 1, kFromTerms = 2;     // where refine_topk_kernel takes its entries from

// Double-precision squared distance between a query sub-vector and a centroid row (Eq. 1), rounded to fp32
// once: the value a full table holds.
__device__ inline float entry_on_demand(const float *__restrict__ yj, const float *__restrict__ cen, int dsub, bool vec4)
{
    double dj = 0.0;
    if (vec4) {
#pragma unroll 4
        for (int tt = 0; tt < dsub; tt += 4) {
            const float4 cv = *reinterpret_cast<const float4 *>(cen + tt);
            const float4 yv = *reinterpret_cast<const float4 *>(yj + tt);
            const double d0 = static_cast<double>(yv.x) - static_cast<double>(cv.x);
            const double d1 = static_cast<double>(yv.y) - static_cast<double>(cv.y);
            const double d2 = static_cast<double>(yv.z) - static_cast<double>(cv.z);
            const double d3 = static_cast<double>(yv.w) - static_cast<double>(cv.w);
            dj = fma(d0, d0, dj); dj = fma(d1, d1, dj); dj = fma(d2, d2, dj); dj = fma(d3, d3, dj);
        }
    } else {
        for (int tt = 0; tt < dsub; ++tt) {
            const double df = static_cast<double>(yj[tt]) - static_cast<double>(cen[tt]);
            dj = fma(df, df, dj);
        }
    }
    return static_cast<float>(dj);
}

// CodeT: uint16_t or uint8_t sub-codes; table_size = 2^b entries per sub-quantizer.
// MODE = kFromTables: `src` = the full tables [nq][M][table_size], an entry is looked up.
// MODE = kFromTerms:  `src` = the entries themselves, [M][gridDim.x * r] (sub-quantizer, then query, then
//   candidate), computed on demand by refine_terms_kernel below.
// MODE = kOnDemand:   `src` = the queries [nq][M * dsub]; an entry (Eq. 1: squared distance between the
//   query's sub-vector and the centroid the sub-code names) is computed when a candidate asks for it,
//   straight from the codebook `cb` [M][table_size] rows of dsub floats, cstride floats apart -- the refinement of Alg. 3 computes table
//   entries on demand because only a small part of a 2^16-entry table is ever used (Sec. 3.3,
//   Refine step); the entry is computed in double precision and rounded to fp32 once, which is what the
//   tables hold, and with memo_slots > 0 the entries of a query's distinct sub-codes are computed once and
//   kept in LDS (see the kernel body).  Either way the distance is the fp32 sum of the M entries, j increasing.
template <int M, typename CodeT, int MODE>
__global__ __launch_bounds__(1024) void refine_topk_kernel(const float *__restrict__ src, uint32_t table_size,
                                                          const float *__restrict__ cb, int dsub, int cstride,
                                                          const CodeT *__restrict__ codes, uint32_t n_codes,
                                                          const uint32_t *__restrict__ cand_id, uint32_t r,
                                                          uint32_t k, uint32_t n_pow2, int use_lds,
                                                          uint32_t memo_slots, uint64_t *__restrict__ spill,
                                                          uint32_t *__restrict__ ids, float *__restrict__ dist)
{
    extern __shared__ __align__(16) uint8_t smem[];
    const int q = blockIdx.x;
    uint64_t *a = use_lds ? reinterpret_cast<uint64_t *>(smem) : spill + static_cast<size_t>(q) * n_pow2;
    constexpr bool DIRECT = MODE == kOnDemand;
    const float *tq = nullptr;
    float *ly = nullptr;
    if constexpr (DIRECT) {
        const int D = M * dsub;
        ly = reinterpret_cast<float *>(smem + (use_lds ? sizeof(uint64_t) * n_pow2 : 0));     // the query
        for (int t = threadIdx.x; t < D; t += blockDim.x) ly[t] = src[static_cast<size_t>(q) * D + t];
        __syncthreads();
    } else if constexpr (MODE == kFromTables) {
        tq = src + static_cast<size_t>(q) * M * table_size;
    }
    if constexpr (DIRECT) {
        // Memoized entries (Sec. 3.3, Refine step: a table entry is computed when first asked for and kept).  With
        // encoded data the candidates of a query repeat a few sub-codes (measured on the GIST- and SIFT-shaped
        // workloads: 60 and 26 distinct values per sub-quantizer among 5000 and 2000 candidates), so the workgroup
        // first collects the distinct (sub-quantizer, sub-code) pairs of its query in an LDS hash set of memo_slots
        // slots per sub-quantizer, computes every collected entry once, and then lets each candidate look its
        // entries up.  The value of an entry does not depend on who computes it, so the result is the same bits.
        // With nearly all sub-codes different (random codes) the set fills up, or the first candidates show that
        // little repeats; the entries are then computed per candidate as before.
        const bool vec4 = (dsub & 3) == 0;                               // rows of whole 16-byte vectors
        constexpr uint32_t kEmpty = 0xFFFFFFFFu;
        constexpr uint32_t kMemoFirst = 256;                             // candidates of the first collecting pass
        uint32_t *hkey = reinterpret_cast<uint32_t *>(ly + M * dsub);    // [M][memo_slots] sub-code, or kEmpty
        float *hval = reinterpret_cast<float *>(hkey + M * memo_slots);  // [M][memo_slots] its entry
        uint16_t *hlist = reinterpret_cast<uint16_t *>(hval + M * memo_slots);  // [M * memo_slots / 2] the slots in use
        __shared__ uint32_t s_claimed, s_over;
        const uint32_t hmask = memo_slots - 1u;
        auto first_slot = [&](uint32_t cj) { return ((cj * 40503u) >> 3) & hmask; };
        // the M sub-codes of a candidate, as stored (whole 16-byte words where the code is made of them)
        const bool codes_aligned = (reinterpret_cast<uintptr_t>(codes) & 15) == 0;      // uniform
        auto load_code = [&](uint32_t id, uint32_t (&c)[M]) {
            constexpr int BYTES = M * static_cast<int>(sizeof(CodeT));
            const CodeT *src = codes + static_cast<size_t>(id) * M;
            if constexpr (BYTES % 16 == 0) {
                if (codes_aligned) {
                    uint4 raw[BYTES / 16];
#pragma unroll
                    for (int v = 0; v < BYTES / 16; ++v) raw[v] = reinterpret_cast<const uint4 *>(src)[v];
#pragma unroll
                    for (int jj = 0; jj < M; ++jj) {
                        const int byte = jj * static_cast<int>(sizeof(CodeT));
                        const uint4 w4 = raw[byte / 16];
                        const uint32_t word = (byte % 16) / 4 == 0 ? w4.x : (byte % 16) / 4 == 1 ? w4.y : (byte % 16) / 4 == 2 ? w4.z : w4.w;
                        c[jj] = sizeof(CodeT) == 2 ? (word >> (8 * (byte % 4))) & 0xFFFFu : (word >> (8 * (byte % 4))) & 0xFFu;
                    }
                    return;
                }
            }
#pragma unroll
            for (int jj = 0; jj < M; ++jj) c[jj] = src[jj];
        };
        bool memo = memo_slots != 0;
        if (memo) {                                                      // uniform
            // In the memoized form a lane takes a whole candidate (its entries come from LDS, there is nothing to
            // spread over lanes): collecting pass, then the entries of the collected pairs, then the look-up pass.
            for (uint32_t t = threadIdx.x; t < M * memo_slots; t += blockDim.x) hkey[t] = kEmpty;
            if (threadIdx.x == 0) { s_claimed = 0; s_over = 0; }
            __syncthreads();
            // (a short first pass: it shows whether anything repeats, and after it most pairs are found by a read)
            const uint32_t first = blockDim.x < kMemoFirst ? blockDim.x : kMemoFirst;
            for (uint32_t base = 0; base < r; base += base == 0 ? first : blockDim.x) {  // uniform trip count
                // (given up by some lane already: nothing more to collect; the passes after the first hold no barrier,
                // so each lane may leave as soon as it sees that)
                if (base != 0 && __hip_atomic_load(&s_over, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP)) break;
                const uint32_t t = base + threadIdx.x;
                uint32_t id = kEmpty;
                if (t < r && (base != 0 || threadIdx.x < first)) id = cand_id[static_cast<size_t>(q) * r + t];
                if (id < n_codes) {
                    uint32_t c[M], seen0[M];
                    load_code(id, c);
                    // (the M first slots are read together: nearly every pair is already there, in its first slot)
#pragma unroll
                    for (int jj = 0; jj < M; ++jj)
                        seen0[jj] = __hip_atomic_load(&hkey[jj * memo_slots + first_slot(c[jj])], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
#pragma unroll
                    for (int jj = 0; jj < M; ++jj) {
                        uint32_t *hj = hkey + jj * memo_slots;
                        const uint32_t cj = c[jj];
                        if (seen0[jj] == cj) continue;
                        uint32_t h = first_slot(cj);
                        bool placed = false;
                        for (int probes = 0; probes < 32 && !placed; ++probes) {
                            // a plain read first: nearly every pair is already there
                            uint32_t cur = __hip_atomic_load(&hj[h], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
                            if (cur == kEmpty) {
                                cur = atomicCAS(&hj[h], kEmpty, cj);
                                if (cur == kEmpty) {
                                    const uint32_t at = atomicAdd(&s_claimed, 1u);
                                    if (at < M * memo_slots / 2) hlist[at] = static_cast<uint16_t>(jj * memo_slots + h);
                                    else s_over = 1;                     // the sets are half full: give up
                                    cur = cj;
                                }
                            }
                            if (cur == cj) placed = true;
                            else h = (h + 1u) & hmask;
                        }
                        if (!placed) s_over = 1;                         // benign race: every writer stores 1
                    }
                }
                // after the first pass: does anything repeat?  (more than half of the pairs seen so far new, or the
                // sets half full: give up)
                if (base == 0) {
                    __syncthreads();
                    const uint32_t seen = (r < first ? r : first) * M;
                    if (threadIdx.x == 0 && (s_claimed > seen / 2 || s_claimed > M * memo_slots / 2)) s_over = 1;
                    __syncthreads();
                    if (s_over) break;                                   // uniform
                }
            }
            __syncthreads();
            memo = s_over == 0 && s_claimed <= M * memo_slots / 2;       // (the list of slots in use holds that many)
            if (memo) {                                                  // uniform
                const uint32_t n_used = s_claimed;
                for (uint32_t u = threadIdx.x; u < n_used; u += blockDim.x) {
                    const uint32_t sl = hlist[u], js = sl / memo_slots;
                    hval[sl] = entry_on_demand(ly + js * dsub, cb + (static_cast<size_t>(js) * table_size + hkey[sl]) * cstride, dsub, vec4);
                }
                __syncthreads();
                for (uint32_t t = threadIdx.x; t < n_pow2; t += blockDim.x) {
                    uint64_t key = ~0ull;
                    if (t < r) {
                        const uint32_t id = cand_id[static_cast<size_t>(q) * r + t];
                        if (id < n_codes) {                              // pad slots (and anything out of range) sort last
                            uint32_t c[M], slot[M];
                            float e[M];
                            load_code(id, c);
                            // first slots and their values read together; the few pairs that sit further on are found after
#pragma unroll
                            for (int jj = 0; jj < M; ++jj) slot[jj] = jj * memo_slots + first_slot(c[jj]);
                            bool all_first = true;
#pragma unroll
                            for (int jj = 0; jj < M; ++jj) all_first = all_first && hkey[slot[jj]] == c[jj];
                            if (!all_first) {
#pragma unroll
                                for (int jj = 0; jj < M; ++jj) {
                                    uint32_t h = slot[jj] - jj * memo_slots;
                                    while (hkey[jj * memo_slots + h] != c[jj]) h = (h + 1u) & hmask;  // it is there: every pair was collected
                                    slot[jj] = jj * memo_slots + h;
                                }
                            }
#pragma unroll
                            for (int jj = 0; jj < M; ++jj) e[jj] = hval[slot[jj]];
                            float d = e[0];
#pragma unroll
                            for (int jj = 1; jj < M; ++jj) d = __fadd_rn(d, e[jj]);
                            key = make_key(__float_as_uint(d), id);
                        }
                    }
                    a[t] = key;
                }
            }
        }
        if (!memo) {                                                     // uniform
            // One lane per (candidate, sub-quantizer): the M lanes of a candidate are neighbours in a wavefront, each
            // computes one entry, and the sums are formed in ascending j from the neighbours' values.
            const uint32_t lane = threadIdx.x & 63u;
            const int j = static_cast<int>(threadIdx.x % M);
            const float *yj = ly + j * dsub;
            for (uint32_t base = 0; base < n_pow2; base += blockDim.x / M) {  // uniform trip count
                const uint32_t t = base + threadIdx.x / M;
                uint32_t id = 0xFFFFFFFFu;
                if (t < r) id = cand_id[static_cast<size_t>(q) * r + t];
                float e = 0.0f;
                if (id < n_codes) {                                      // pad slots (and anything out of range) sort last
                    const uint32_t cj = codes[static_cast<size_t>(id) * M + j];
                    const float *cen = cb + (static_cast<size_t>(j) * table_size + cj) * cstride;
                    e = entry_on_demand(yj, cen, dsub, vec4);
                }
                float d = __shfl(e, static_cast<int>(lane - j));
#pragma unroll
                for (int jj = 1; jj < M; ++jj) d = __fadd_rn(d, __shfl(e, static_cast<int>(lane - j + jj)));
                if (j == 0 && t < n_pow2) a[t] = id < n_codes ? make_key(__float_as_uint(d), id) : ~0ull;
            }
        }
    } else if constexpr (MODE == kFromTerms) {
        const size_t total = static_cast<size_t>(gridDim.x) * r;
        for (uint32_t t = threadIdx.x; t < n_pow2; t += blockDim.x) {
            uint64_t key = ~0ull;
            if (t < r) {
                const size_t at = static_cast<size_t>(q) * r + t;
                const uint32_t id = cand_id[at];
                if (id < n_codes) {                 // pad slots (and anything out of range) sort last
                    float d = src[at];
#pragma unroll
                    for (int j = 1; j < M; ++j) d = __fadd_rn(d, src[j * total + at]);
                    key = make_key(__float_as_uint(d), id);
                }
            }
            a[t] = key;
        }
    } else {
        for (uint32_t t = threadIdx.x; t < n_pow2; t += blockDim.x) {
            uint64_t key = ~0ull;
            if (t < r) {
                const uint32_t id = cand_id[static_cast<size_t>(q) * r + t];
                if (id < n_codes) {                 // pad slots (and anything out of range) sort last
                    const CodeT *c = codes + static_cast<size_t>(id) * M;
                    float d = tq[c[0]];
#pragma unroll
                    for (int j = 1; j < M; ++j) d = __fadd_rn(d, tq[static_cast<size_t>(j) * table_size + c[j]]);
                    key = make_key(__float_as_uint(d), id);
                }
            }
            a[t] = key;
        }
    }
    __syncthreads();
    // ---- cut down by value ----------------------------------------------------------------
    __shared__ uint32_t hist[kRefineSteps];
    __shared__ uint64_t few[kRefineFew];
    __shared__ uint32_t s_lo, s_hi, s_step, s_n, wsum[16];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    uint32_t lo = 0xFFFFFFFFu, hi = 0;
    for (uint32_t t = tid; t < r; t += blockDim.x) {
        const uint64_t key = a[t];
        if (key != ~0ull) {
            const uint32_t d = static_cast<uint32_t>(key >> 32);
            lo = min(lo, d); hi = max(hi, d);
        }
    }
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        lo = min(lo, static_cast<uint32_t>(__shfl_xor(static_cast<int>(lo), d)));
        hi = max(hi, static_cast<uint32_t>(__shfl_xor(static_cast<int>(hi), d)));
    }
    if (tid == 0) { s_lo = 0xFFFFFFFFu; s_hi = 0; s_step = kRefineSteps; s_n = 0; }
    for (uint32_t t = tid; t < kRefineSteps; t += blockDim.x) hist[t] = 0;
    __syncthreads();
    if (lane == 0) { atomicMin(&s_lo, lo); atomicMax(&s_hi, hi); }
    __syncthreads();
    const float dlo = __uint_as_float(s_lo), dhi = __uint_as_float(s_hi);
    const float scale = static_cast<float>(kRefineSteps) / (dhi - dlo);
    // step of a distance: non-decreasing in the distance, so "step <= s" keeps every key below some value
    auto step_of = [&](uint64_t key) -> uint32_t {
        const float x = (__uint_as_float(static_cast<uint32_t>(key >> 32)) - dlo) * scale;
        return x < static_cast<float>(kRefineSteps - 1) ? static_cast<uint32_t>(x) : kRefineSteps - 1;
    };
    bool all = !(scale > 0.0f) || !(scale < INFINITY);       // one value only, or nothing finite to scale by
    if (!all) {
        for (uint32_t t = tid; t < r; t += blockDim.x) {
            const uint64_t key = a[t];
            if (key != ~0ull) atomicAdd(&hist[step_of(key)], 1u);
        }
        __syncthreads();
        // thread t owns steps 2t and 2t + 1 (1024 threads); inclusive prefix over the threads
        const uint32_t h0 = hist[2 * tid], h1 = hist[2 * tid + 1];
        uint32_t incl = h0 + h1;
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) {
            const uint32_t other = __shfl(incl, lane >= d ? lane - d : lane);
            if (lane >= d) incl += other;
        }
        if (lane == 63) wsum[wave] = incl;
        __syncthreads();
        uint32_t before = incl - (h0 + h1);
        for (int w2 = 0; w2 < wave; ++w2) before += wsum[w2];
        if (before < k && before + h0 + h1 >= k) {                // exactly one thread, if k keys exist at all
            const bool first = before + h0 >= k;
            s_step = first ? 2 * tid : 2 * tid + 1;
            s_n = first ? before + h0 : before + h0 + h1;
        }
        __syncthreads();
        all = s_step == kRefineSteps || s_n > kRefineFew;          // fewer than k real keys, or too many to gather
    }
    if (!all) {
        const uint32_t step = s_step, nkeep = s_n;
        uint32_t nf = 1;
        while (nf < nkeep) nf <<= 1;
        __syncthreads();
        if (tid == 0) s_n = 0;
        for (uint32_t t = tid; t < nf; t += blockDim.x) few[t] = ~0ull;
        __syncthreads();
        for (uint32_t t = tid; t < r; t += blockDim.x) {
            const uint64_t key = a[t];
            if (key != ~0ull && step_of(key) <= step) {
                const uint32_t pos = atomicAdd(&s_n, 1u);
                if (pos < nf) few[pos] = key;
            }
        }
        bitonic_sort(few, nf);
        a = few;
    } else {
        bitonic_sort(a, n_pow2);
    }
    for (uint32_t t = threadIdx.x; t < k; t += blockDim.x) {
        const uint64_t key = a[t];
        ids[static_cast<size_t>(q) * k + t] = static_cast<uint32_t>(key);
        dist[static_cast<size_t>(q) * k + t] = (key == ~0ull) ? INFINITY : __uint_as_float(static_cast<uint32_t>(key >> 32));
    }
}

template <int M, typename CodeT, int MODE>
static int launch_refine_m(const float *src, uint32_t table_size, const float *cb, int dsub, int cstride, const CodeT *codes,
                           uint64_t n_codes, const uint32_t *cand_id, int nq, uint32_t r, uint32_t k, uint32_t *ids,
                           float *dist, void *ws, hipStream_t st)
{
    const uint32_t np2 = next_pow2_r(r);
    const int use_lds = np2 <= kRefineLdsKeys;
    size_t lds = (use_lds ? sizeof(uint64_t) * np2 : 0) + (MODE == kOnDemand ? sizeof(float) * M * dsub : 0);
    // on demand: a hash set of the query's distinct (sub-quantizer, sub-code) pairs with their entries, as many
    // slots per sub-quantizer (a power of two, at most 512) as the LDS left beside the keys, the query and the
    // kernel's static arrays (17 KB) holds; none if that is fewer than 64
    // (below 8192 (candidate, sub-quantizer) pairs per query collecting and looking up costs more than it saves:
    // measured at r = 1000, m = 4)
    uint32_t memo_slots = 0;
    if (MODE == kOnDemand && static_cast<uint64_t>(r) * M >= 8u * 1024u) {
        memo_slots = 512;
        while (memo_slots >= 64 && lds + static_cast<size_t>(9) * M * memo_slots > static_cast<size_t>(140) * 1024) memo_slots /= 2;
        if (memo_slots < 64) memo_slots = 0;
        lds += static_cast<size_t>(9) * M * memo_slots;                 // keys, entries, and the list of slots in use
    }
    const int rc = allow_dynamic_lds(reinterpret_cast<const void *>(&refine_topk_kernel<M, CodeT, MODE>), static_cast<int>(lds));
    if (rc) return rc;
    DCPQ_LAUNCH(kStageRefine, st, (refine_topk_kernel<M, CodeT, MODE>), dim3(nq), dim3(1024), lds, src, table_size, cb, dsub,
                cstride, codes, static_cast<uint32_t>(n_codes), cand_id, r, k, np2, use_lds, memo_slots, static_cast<uint64_t *>(ws),
                ids, dist);
    DCPQ_CHECK_LAUNCH("refine_topk_kernel");
    return DCPQ_OK;
}

// rows of dsub floats copied to rows cstride floats apart (the tail of a row is not written: it is never read)
__global__ __launch_bounds__(256) void pad_rows_kernel(const float *__restrict__ src, size_t nrows, int dsub, int cstride,
                                                       float *__restrict__ dst)
{
    const size_t e = static_cast<size_t>(blockIdx.x) * blockDim.x + threadIdx.x;
    if (e >= nrows * dsub) return;
    dst[(e / dsub) * cstride + e % dsub] = src[e];
}

int launch_pad_rows(const float *src, size_t nrows, int dsub, int cstride, float *dst, hipStream_t st)
{
    const size_t e = nrows * dsub;
    DCPQ_LAUNCH(kStageRefine, st, pad_rows_kernel, dim3(static_cast<unsigned>((e + 255) / 256)), dim3(256), 0, src, nrows, dsub,
                cstride, dst);
    DCPQ_CHECK_LAUNCH("pad_rows_kernel");
    return DCPQ_OK;
}

template <typename CodeT, int MODE>
static int launch_refine_t(const float *src, uint32_t table_size, const float *cb, int dsub, int cstride, const CodeT *codes,
                           uint64_t n_codes, int m, const uint32_t *cand_id, int nq, uint32_t r, uint32_t k, uint32_t *ids,
                           float *dist, void *ws, hipStream_t st)
{
    if (nq == 0) return DCPQ_OK;
#define DCPQ_LAUNCH_REFINE(MV)                                                                                      \
    case MV:                                                                                                        \
        return launch_refine_m<MV, CodeT, MODE>(src, table_size, cb, dsub, cstride, codes, n_codes, cand_id, nq, r, k, ids, dist, ws, st);
    switch (m) {
        DCPQ_LAUNCH_REFINE(1) DCPQ_LAUNCH_REFINE(2) DCPQ_LAUNCH_REFINE(4) DCPQ_LAUNCH_REFINE(8)
        DCPQ_LAUNCH_REFINE(16) DCPQ_LAUNCH_REFINE(32)
        default: return fail(DCPQ_EUNSUPPORTED, "m=%d not supported", m);
    }
#undef DCPQ_LAUNCH_REFINE
}

int launch_refine(const float *tables, uint32_t table_size, const void *codes, int code_bytes, uint64_t n_codes, int m,
                  const uint32_t *cand_id, int nq, uint32_t r, uint32_t k, uint32_t *ids, float *dist, void *ws,
                  hipStream_t st)
{
    if (code_bytes == 1)
        return launch_refine_t<uint8_t, kFromTables>(tables, table_size, nullptr, 0, 0, static_cast<const uint8_t *>(codes), n_codes, m,
                                               cand_id, nq, r, k, ids, dist, ws, st);
    return launch_refine_t<uint16_t, kFromTables>(tables, table_size, nullptr, 0, 0, static_cast<const uint16_t *>(codes), n_codes, m,
                                            cand_id, nq, r, k, ids, dist, ws, st);
}

int launch_refine_direct(const float *queries, const float *codebooks, int dsub, int cstride, uint32_t table_size, const void *codes,
                         int code_bytes, uint64_t n_codes, int m, const uint32_t *cand_id, int nq, uint32_t r, uint32_t k,
                         uint32_t *ids, float *dist, void *ws, hipStream_t st)
{
    if (code_bytes == 1)
        return launch_refine_t<uint8_t, kOnDemand>(queries, table_size, codebooks, dsub, cstride, static_cast<const uint8_t *>(codes), n_codes,
                                              m, cand_id, nq, r, k, ids, dist, ws, st);
    return launch_refine_t<uint16_t, kOnDemand>(queries, table_size, codebooks, dsub, cstride, static_cast<const uint16_t *>(codes), n_codes, m,
                                           cand_id, nq, r, k, ids, dist, ws, st);
}


// ---- on demand, split by sub-quantizer ---------------------------------------------------------
// The one-kernel form above gathers, for every candidate, m centroid rows out of codebooks of tens of
// megabytes: nearly every row misses the 4 MB second-level cache of the XCD the workgroup runs on, and the
// kernel is bound by the number of memory lines it moves.  A sub-quantizer's own codebook (2^16 rows of
// dsub floats: 3 MB at dsub = 12) does fit one such cache, and the chip has 8 of them; workgroups are handed
// to the 8 XCDs in turn, so workgroup number w runs on XCD w mod 8.  The split form therefore lets the
// workgroups with w mod 8 = x compute the entries of sub-quantizers j = x, x + 8, ... only (for m < 8: of
// j = x mod m, for one part in 8 / m of the candidates), so that each cache keeps seeing the same few
// megabytes of rows.  Should the hardware hand workgroups out differently, the result is the same and only
// the time changes.  Three kernels:
//   gather_codes_kernel   sub-codes of all candidates of the batch, by sub-quantizer: plane[j][candidate]
//                         (one scattered read of a whole code per candidate, contiguous writes)
//   refine_terms_kernel   entry[j][candidate] (Eq. 1, as in the one-kernel form: fp64, rounded to fp32 once)
//   refine_topk_kernel<kFromTerms>   fp32 sum over j increasing, then the k smallest by (distance, id)
// Candidates are numbered query * r + position, as in cand_id.
constexpr uint32_t kSplitChunk = 2048;      // candidates per workgroup of refine_terms_kernel (256 threads x 8)

template <int M, typename CodeT>
__global__ __launch_bounds__(256) void gather_codes_kernel(const CodeT *__restrict__ codes, uint32_t n_codes,
                                                           const uint32_t *__restrict__ cand_id, uint32_t total,
                                                           CodeT *__restrict__ plane)
{
    const uint32_t t = blockIdx.x * 256u + threadIdx.x;
    if (t >= total) return;
    const uint32_t id = cand_id[t];
    constexpr int BYTES = M * static_cast<int>(sizeof(CodeT));
    CodeT c[M];
#pragma unroll
    for (int j = 0; j < M; ++j) c[j] = 0;                              // pad slots: any valid sub-code
    if (id < n_codes) {
        const uint8_t *src = reinterpret_cast<const uint8_t *>(codes) + static_cast<size_t>(id) * BYTES;
        if constexpr (BYTES % 16 == 0) {
#pragma unroll
            for (int v = 0; v < BYTES / 16; ++v) reinterpret_cast<uint4 *>(c)[v] = reinterpret_cast<const uint4 *>(src)[v];
        } else if constexpr (BYTES == 8) {
            *reinterpret_cast<uint2 *>(c) = *reinterpret_cast<const uint2 *>(src);
        } else if constexpr (BYTES == 4) {
            *reinterpret_cast<uint32_t *>(c) = *reinterpret_cast<const uint32_t *>(src);
        } else {
#pragma unroll
            for (int j = 0; j < M; ++j) c[j] = reinterpret_cast<const CodeT *>(src)[j];
        }
    }
#pragma unroll
    for (int j = 0; j < M; ++j) plane[static_cast<size_t>(j) * total + t] = c[j];
}

// P > 0: rows of P 16-byte parts (dsub = 4 P).  Lane l of a wavefront reading its own row with P loads would
// send P separate requests per row to the second-level cache, whose request rate is what bounds this kernel
// (2.9 requests per entry measured at dsub = 12); instead the P * 64 parts of the wavefront's 64 rows are
// fetched in row order, lane after lane, so that the parts of a row travel in one request (two when the row
// lies across a 64-byte boundary), parked in LDS, and each lane then picks up its row there.
// P = 0: rows of any length, each read by its own lane.
template <typename CodeT, int P>
__global__ __launch_bounds__(256) void refine_terms_kernel(const float *__restrict__ queries, int m, int dsub,
                                                           const float *__restrict__ cb, uint32_t table_size,
                                                           const CodeT *__restrict__ plane, uint32_t total, uint32_t r,
                                                           float *__restrict__ terms)
{
    __shared__ float4 stage[P ? 256 * P : 1];
    const uint32_t x = blockIdx.x & 7u;                                // the XCD this workgroup is expected on
    const uint32_t first = (blockIdx.x >> 3) * kSplitChunk;            // its stretch of candidates
    const bool vec4 = (dsub & 3) == 0;
    const int D = m * dsub;
    const uint32_t lane = threadIdx.x & 63u;
    float4 *ws = stage + (threadIdx.x >> 6) * (64 * P);                // this wavefront's rows
    // m >= 8: sub-quantizers x, x + 8, ..., every candidate of the stretch; m < 8: sub-quantizer x mod m, the
    // candidates of part x / m out of 8 / m (threads are dealt to the parts in turn)
    const uint32_t parts = m >= 8 ? 1u : 8u / static_cast<uint32_t>(m), part = m >= 8 ? 0u : x / static_cast<uint32_t>(m);
    for (int j = m >= 8 ? static_cast<int>(x) : static_cast<int>(x % static_cast<uint32_t>(m)); j < m; j += 8) {
        const CodeT *pj = plane + static_cast<size_t>(j) * total;
        const float *cj = cb + static_cast<size_t>(j) * table_size * dsub;
        float *tj = terms + static_cast<size_t>(j) * total;
        // (the same number of rounds for every thread: kSplitChunk is a multiple of 256 * parts)
#pragma unroll 2
        for (uint32_t i = threadIdx.x + 256u * part; i < kSplitChunk; i += 256u * parts) {
            const uint32_t t = first + i;
            const bool live = t < total;
            const uint32_t code = live ? pj[t] : 0u;                   // past the end: any valid row, result dropped
            const float *yj = queries + static_cast<size_t>(live ? t / r : 0u) * D + j * dsub;
            float e;
            if constexpr (P > 0) {
#pragma unroll
                for (int c = 0; c < P; ++c) {
                    const uint32_t f = 64u * c + lane;                 // part f % P of the row of lane f / P
                    const uint32_t owner = f / P;
                    const uint32_t oc = static_cast<uint32_t>(__shfl(static_cast<int>(code), static_cast<int>(owner)));
                    ws[f] = *reinterpret_cast<const float4 *>(cj + static_cast<size_t>(oc) * dsub + 4u * (f - owner * P));
                }
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                __builtin_amdgcn_wave_barrier();
                __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
                double dj = 0.0;
#pragma unroll
                for (int c = 0; c < P; ++c) {                          // the arithmetic of entry_on_demand, part by part
                    const float4 cv = ws[lane * P + c];
                    const float4 yv = *reinterpret_cast<const float4 *>(yj + 4 * c);
                    const double d0 = static_cast<double>(yv.x) - static_cast<double>(cv.x);
                    const double d1 = static_cast<double>(yv.y) - static_cast<double>(cv.y);
                    const double d2 = static_cast<double>(yv.z) - static_cast<double>(cv.z);
                    const double d3 = static_cast<double>(yv.w) - static_cast<double>(cv.w);
                    dj = fma(d0, d0, dj); dj = fma(d1, d1, dj); dj = fma(d2, d2, dj); dj = fma(d3, d3, dj);
                }
                e = static_cast<float>(dj);
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");     // every lane has its row before the next round parks new ones
                __builtin_amdgcn_wave_barrier();
                __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            } else {
                e = entry_on_demand(yj, cj + static_cast<size_t>(code) * dsub, dsub, vec4);
            }
            if (live) tj[t] = e;
        }
    }
}

// bytes of the two intermediate arrays (sub-code planes, then entries) for nq queries
size_t refine_split_bytes(int nq, uint32_t r, int m, int code_bytes)
{
    const size_t total = static_cast<size_t>(nq) * r;
    return align_up(total * m * code_bytes, 256) + total * m * sizeof(float);
}

template <typename CodeT>
static int launch_refine_split_t(const float *queries, const float *codebooks, int dsub, uint32_t table_size, const CodeT *codes,
                                 uint64_t n_codes, int m, const uint32_t *cand_id, int nq, uint32_t r, uint32_t k, uint32_t *ids,
                                 float *dist, void *mid, void *ws, hipStream_t st)
{
    const uint32_t total = static_cast<uint32_t>(static_cast<size_t>(nq) * r);
    CodeT *plane = static_cast<CodeT *>(mid);
    float *terms = reinterpret_cast<float *>(static_cast<uint8_t *>(mid) + align_up(static_cast<size_t>(total) * m * sizeof(CodeT), 256));
    const dim3 g1((total + 255u) / 256u);
#define DCPQ_LAUNCH_GATHER(MV)                                                                                      \
    case MV:                                                                                                        \
        DCPQ_LAUNCH(kStageRefine, st, (gather_codes_kernel<MV, CodeT>), g1, dim3(256), 0, codes,                     \
                    static_cast<uint32_t>(n_codes), cand_id, total, plane);                                        \
        break;
    switch (m) {
        DCPQ_LAUNCH_GATHER(1) DCPQ_LAUNCH_GATHER(2) DCPQ_LAUNCH_GATHER(4) DCPQ_LAUNCH_GATHER(8)
        DCPQ_LAUNCH_GATHER(16) DCPQ_LAUNCH_GATHER(32)
        default: return fail(DCPQ_EUNSUPPORTED, "m=%d not supported", m);
    }
#undef DCPQ_LAUNCH_GATHER
    DCPQ_CHECK_LAUNCH("gather_codes_kernel");
    const uint32_t stretches = (total + kSplitChunk - 1) / kSplitChunk;
#define DCPQ_LAUNCH_TERMS(PV)                                                                                       \
    case PV:                                                                                                        \
        DCPQ_LAUNCH(kStageRefine, st, (refine_terms_kernel<CodeT, PV>), dim3(8u * stretches), dim3(256), 0, queries, m, dsub,    \
                    codebooks, table_size, plane, total, r, terms);                                                 \
        break;
    // rows of up to 8 whole 16-byte parts go through LDS (codebooks are 16-byte aligned: the callers check)
    switch (dsub % 4 == 0 && dsub <= 32 ? dsub / 4 : 0) {
        DCPQ_LAUNCH_TERMS(1) DCPQ_LAUNCH_TERMS(2) DCPQ_LAUNCH_TERMS(3) DCPQ_LAUNCH_TERMS(4) DCPQ_LAUNCH_TERMS(5)
        DCPQ_LAUNCH_TERMS(6) DCPQ_LAUNCH_TERMS(7) DCPQ_LAUNCH_TERMS(8)
        default: DCPQ_LAUNCH(kStageRefine, st, (refine_terms_kernel<CodeT, 0>), dim3(8u * stretches), dim3(256), 0, queries, m,
                             dsub, codebooks, table_size, plane, total, r, terms);
    }
#undef DCPQ_LAUNCH_TERMS
    DCPQ_CHECK_LAUNCH("refine_terms_kernel");
    return launch_refine_t<CodeT, kFromTerms>(terms, table_size, nullptr, 0, 0, codes, n_codes, m, cand_id, nq, r, k, ids, dist, ws, st);
}

// mid: refine_split_bytes(nq, r, m, code_bytes) bytes, 256-byte aligned; nq * r must fit 32 bits (the caller checks both)
int launch_refine_split(const float *queries, const float *codebooks, int dsub, uint32_t table_size, const void *codes,
                        int code_bytes, uint64_t n_codes, int m, const uint32_t *cand_id, int nq, uint32_t r, uint32_t k,
                        uint32_t *ids, float *dist, void *mid, void *ws, hipStream_t st)
{
    if (nq == 0) return DCPQ_OK;
    if (code_bytes == 1)
        return launch_refine_split_t<uint8_t>(queries, codebooks, dsub, table_size, static_cast<const uint8_t *>(codes), n_codes, m,
                                              cand_id, nq, r, k, ids, dist, mid, ws, st);
    return launch_refine_split_t<uint16_t>(queries, codebooks, dsub, table_size, static_cast<const uint16_t *>(codes), n_codes, m,
                                           cand_id, nq, r, k, ids, dist, mid, ws, st);
}

}  // namespace dcpq

using namespace dcpq;

extern "C" size_t dcpq_refine_workspace_bytes(int nq, uint32_t r)
{
    if (nq <= 0 || r == 0) return 0;
    const uint32_t np2 = next_pow2_r(r);
    return np2 <= kRefineLdsKeys ? 0 : sizeof(uint64_t) * static_cast<size_t>(nq) * np2;
}

extern "C" int dcpq_refine_topk_bits(const float *tables, uint32_t n_entries, const void *codes, int code_bytes,
                                     uint64_t n_codes, int m, const uint32_t *cand_id, int nq, uint32_t r, uint32_t k,
                                     uint32_t *ids, float *dist, void *workspace, size_t workspace_bytes, void *stream)
{
    clear_error();
    DCPQ_REQUIRE(nq >= 0, "refine_topk: nq=%d", nq);
    if (!m_supported(m)) return fail(DCPQ_EUNSUPPORTED, "refine_topk: m=%d not supported", m);
    DCPQ_REQUIRE(code_bytes == 1 || code_bytes == 2, "refine_topk: code_bytes=%d (1 or 2)", code_bytes);
    DCPQ_REQUIRE(n_entries == (code_bytes == 1 ? 256u : 65536u),
                 "refine_topk: tables of %u entries do not cover every value of a %d-byte sub-code", n_entries, code_bytes);
    DCPQ_REQUIRE(k >= 1 && k <= r, "refine_topk: needs 1 <= k <= r (k=%u r=%u)", k, r);
    DCPQ_REQUIRE(n_codes >= 1 && n_codes < (1ull << 32), "refine_topk: n_codes out of range");
    if (nq == 0) return DCPQ_OK;
    DCPQ_REQUIRE(tables && codes && cand_id && ids && dist, "refine_topk: null pointer");
    const size_t need = dcpq_refine_workspace_bytes(nq, r);
    if (need && (!workspace || workspace_bytes < need))
        return fail(DCPQ_EWORKSPACE, "refine_topk: workspace %zu < %zu bytes", workspace_bytes, need);
    return launch_refine(tables, n_entries, codes, code_bytes, n_codes, m, cand_id, nq, r, k, ids, dist, workspace,
                         as_stream(stream));
}

extern "C" int dcpq_refine_direct_topk(const float *queries, const float *codebooks, int m, int dsub, int b,
                                       const void *codes, uint64_t n_codes, const uint32_t *cand_id, int nq, uint32_t r,
                                       uint32_t k, uint32_t *ids, float *dist, void *workspace, size_t workspace_bytes,
                                       void *stream)
{
    clear_error();
    DCPQ_REQUIRE(nq >= 0, "refine_direct_topk: nq=%d", nq);
    if (!dcpq_shape_supported(m, dsub)) return fail(DCPQ_EUNSUPPORTED, "refine_direct_topk: m=%d dsub=%d not supported", m, dsub);
    if (!dcpq_bits_supported(b, 1)) return fail(DCPQ_EUNSUPPORTED, "refine_direct_topk: b=%d not supported", b);
    DCPQ_REQUIRE(k >= 1 && k <= r, "refine_direct_topk: needs 1 <= k <= r (k=%u r=%u)", k, r);
    DCPQ_REQUIRE(n_codes >= 1 && n_codes < (1ull << 32), "refine_direct_topk: n_codes out of range");
    if (nq == 0) return DCPQ_OK;
    DCPQ_REQUIRE(queries && codebooks && codes && cand_id && ids && dist, "refine_direct_topk: null pointer");
    DCPQ_REQUIRE((reinterpret_cast<uintptr_t>(codebooks) & 15) == 0, "refine_direct_topk: codebooks must be 16-byte aligned");
    const size_t need = dcpq_refine_workspace_bytes(nq, r);
    if (need && (!workspace || workspace_bytes < need))
        return fail(DCPQ_EWORKSPACE, "refine_direct_topk: workspace %zu < %zu bytes", workspace_bytes, need);
    return launch_refine_direct(queries, codebooks, dsub, dsub, 1u << b, codes, b / 8, n_codes, m, cand_id, nq, r, k, ids, dist,
                                workspace, as_stream(stream));
}

extern "C" int dcpq_refine_topk(const float *tables, const uint16_t *codes, uint64_t n_codes, int m,
                                const uint32_t *cand_id, int nq, uint32_t r, uint32_t k, uint32_t *ids,
                                float *dist, void *workspace, size_t workspace_bytes, void *stream)
{
    return dcpq_refine_topk_bits(tables, kFullSize, codes, 2, n_codes, m, cand_id, nq, r, k, ids, dist, workspace,
                                 workspace_bytes, stream);
}
