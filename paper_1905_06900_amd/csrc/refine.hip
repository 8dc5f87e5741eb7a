// Pass two of Alg. 3 (Sec. 3.3, "Refine step"): exact asymmetric distance (Eq. 2) of every
// candidate from the full tables, then the result set of the k smallest by (distance, id).
// One workgroup per query: the r keys (distance bits, id) are built and sorted in LDS (or in a
// global spill area when they do not fit) and the first k are written out.  Squared distances
// are non-negative, so their fp32 bit patterns order like the values.
#include "common.h"

namespace dcpq {

constexpr uint32_t kRefineLdsKeys = 8192;   // 64 KiB of keys

static uint32_t next_pow2_r(uint32_t x)
{
    uint32_t p = 1;
    while (p < x) p <<= 1;
    return p;
}

__device__ inline void bitonic_sort_keys(uint64_t *a, uint32_t n_pow2)
{
    for (uint32_t size = 2; size <= n_pow2; size <<= 1) {
        for (uint32_t stride = size >> 1; stride > 0; stride >>= 1) {
            __syncthreads();
            for (uint32_t t = threadIdx.x; t < (n_pow2 >> 1); t += blockDim.x) {
                const uint32_t lo = 2 * t - (t & (stride - 1));
                const uint32_t hi = lo + stride;
                const bool up = (lo & size) == 0;
                const uint64_t x = a[lo], y = a[hi];
                if ((x > y) == up) { a[lo] = y; a[hi] = x; }
            }
        }
    }
    __syncthreads();
}

template <int M>
__global__ __launch_bounds__(1024) void refine_topk_kernel(const float *__restrict__ tables,
                                                          const uint16_t *__restrict__ codes, uint32_t n_codes,
                                                          const uint32_t *__restrict__ cand_id, uint32_t r,
                                                          uint32_t k, uint32_t n_pow2, int use_lds,
                                                          uint64_t *__restrict__ spill,
                                                          uint32_t *__restrict__ ids, float *__restrict__ dist)
{
    extern __shared__ __align__(16) uint8_t smem[];
    const int q = blockIdx.x;
    uint64_t *a = use_lds ? reinterpret_cast<uint64_t *>(smem) : spill + static_cast<size_t>(q) * n_pow2;
    const float *tq = tables + static_cast<size_t>(q) * M * kFullSize;
    for (uint32_t t = threadIdx.x; t < n_pow2; t += blockDim.x) {
        uint64_t key = ~0ull;
        if (t < r) {
            const uint32_t id = cand_id[static_cast<size_t>(q) * r + t];
            if (id < n_codes) {                 // pad slots (and anything out of range) sort last
                const uint16_t *c = codes + static_cast<size_t>(id) * M;
                float d = tq[c[0]];
#pragma unroll
                for (int j = 1; j < M; ++j) d = __fadd_rn(d, tq[static_cast<size_t>(j) * kFullSize + c[j]]);
                key = make_key(__float_as_uint(d), id);
            }
        }
        a[t] = key;
    }
    bitonic_sort_keys(a, n_pow2);
    for (uint32_t t = threadIdx.x; t < k; t += blockDim.x) {
        const uint64_t key = a[t];
        ids[static_cast<size_t>(q) * k + t] = static_cast<uint32_t>(key);
        dist[static_cast<size_t>(q) * k + t] = (key == ~0ull) ? INFINITY : __uint_as_float(static_cast<uint32_t>(key >> 32));
    }
}

int launch_refine(const float *tables, const uint16_t *codes, uint64_t n_codes, int m, const uint32_t *cand_id,
                  int nq, uint32_t r, uint32_t k, uint32_t *ids, float *dist, void *ws, hipStream_t st)
{
    if (nq == 0) return DCPQ_OK;
    const uint32_t np2 = next_pow2_r(r);
    const int use_lds = np2 <= kRefineLdsKeys;
    const size_t lds = use_lds ? sizeof(uint64_t) * np2 : 0;
    uint64_t *spill = static_cast<uint64_t *>(ws);
#define DCPQ_LAUNCH_REFINE(MV)                                                                            \
    case MV:                                                                                              \
        DCPQ_LAUNCH(kStageRefine, st, refine_topk_kernel<MV>, dim3(nq), dim3(1024), lds, tables, codes,   \
                    static_cast<uint32_t>(n_codes), cand_id, r, k, np2, use_lds, spill, ids, dist);       \
        break;
    switch (m) {
        DCPQ_LAUNCH_REFINE(1) DCPQ_LAUNCH_REFINE(2) DCPQ_LAUNCH_REFINE(4) DCPQ_LAUNCH_REFINE(8)
        DCPQ_LAUNCH_REFINE(16) DCPQ_LAUNCH_REFINE(32)
        default: return fail(DCPQ_EUNSUPPORTED, "m=%d not supported", m);
    }
#undef DCPQ_LAUNCH_REFINE
    DCPQ_CHECK_LAUNCH("refine_topk_kernel");
    return DCPQ_OK;
}

}  // namespace dcpq

using namespace dcpq;

extern "C" size_t dcpq_refine_workspace_bytes(int nq, uint32_t r)
{
    if (nq <= 0 || r == 0) return 0;
    const uint32_t np2 = next_pow2_r(r);
    return np2 <= kRefineLdsKeys ? 0 : sizeof(uint64_t) * static_cast<size_t>(nq) * np2;
}

extern "C" int dcpq_refine_topk(const float *tables, const uint16_t *codes, uint64_t n_codes, int m,
                                const uint32_t *cand_id, int nq, uint32_t r, uint32_t k, uint32_t *ids,
                                float *dist, void *workspace, size_t workspace_bytes, void *stream)
{
    clear_error();
    DCPQ_REQUIRE(nq >= 0, "refine_topk: nq=%d", nq);
    if (!m_supported(m)) return fail(DCPQ_EUNSUPPORTED, "refine_topk: m=%d not supported", m);
    DCPQ_REQUIRE(k >= 1 && k <= r, "refine_topk: needs 1 <= k <= r (k=%u r=%u)", k, r);
    DCPQ_REQUIRE(n_codes >= 1 && n_codes < (1ull << 32), "refine_topk: n_codes out of range");
    if (nq == 0) return DCPQ_OK;
    DCPQ_REQUIRE(tables && codes && cand_id && ids && dist, "refine_topk: null pointer");
    const size_t need = dcpq_refine_workspace_bytes(nq, r);
    if (need && (!workspace || workspace_bytes < need))
        return fail(DCPQ_EWORKSPACE, "refine_topk: workspace %zu < %zu bytes", workspace_bytes, need);
    return launch_refine(tables, codes, n_codes, m, cand_id, nq, r, k, ids, dist, workspace, as_stream(stream));
}
