// Conventional single-pass search (Alg. 1, Sec. 2.3): asymmetric distance of every code with the
// full floating-point tables (Eq. 2), the k smallest by (distance, id).  This is the method the
// derived codebooks are measured against -- with 2^16-entry tables ("plain 16-bit": the tables, 256
// KiB per sub-quantizer and query, live in the L2 / HBM and every lookup is a gather from there) and
// with 2^8-entry tables of an 8-bit product quantizer ("plain 8-bit": tables in LDS).  It is a
// comparison system here, not the product path: plain and exact rather than fast.
//
//   d(q, i) = sum over j increasing of tables[q][j][codes[i][j]]   (fp32 adds, as in the refinement)
//
// Selection.  A workgroup owns one stretch of the codes for a tile of queries and keeps, per query,
// the k best keys seen so far (key = order-preserving bits of d, then the id: all keys are distinct,
// so "the k smallest keys" does not depend on the order of arrival).  A code whose key is below the
// query's current k-th best is appended to the query's buffer in LDS; when a buffer is nearly full
// it is sorted and cut back to k.  Every workgroup writes its k keys per query, and a second kernel
// merges the parts of a query.
#include "common.h"
#include "scan_internal.h"

namespace dcpq {

constexpr int kPlainThreads = 256;
constexpr int kPlainQT = 8;             // queries per workgroup
constexpr uint32_t kPlainBuf = 1024;    // keys per query in a workgroup's buffer (power of two, > k + threads)
constexpr uint32_t kPlainMerge = 8192;  // keys the merge sorts in LDS
constexpr uint32_t kPlainMostK = kPlainBuf - kPlainThreads;

// Bits of a float as an unsigned integer with the same order (negative zero and tiny negative
// entries, which the rounded tables may hold, sort below the positives).
__device__ inline uint32_t ordered_bits(float d)
{
    const uint32_t u = __float_as_uint(d);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
__device__ inline float from_ordered_bits(uint32_t o)
{
    return __uint_as_float((o & 0x80000000u) ? (o & 0x7fffffffu) : ~o);
}

// Workgroup-wide: sorts the first `count` keys of buf (padding up to the buffer size), keeps the k
// smallest, returns the new count; *tau = the k-th smallest when there are k, else "no bound".
__device__ inline uint32_t cut_to_k(uint64_t *buf, uint32_t count, uint32_t k, uint64_t *tau)
{
    for (uint32_t t = count + threadIdx.x; t < kPlainBuf; t += kPlainThreads) buf[t] = ~0ull;
    bitonic_sort(buf, kPlainBuf);
    const uint32_t keep = count < k ? count : k;
    if (threadIdx.x == 0) *tau = keep == k ? buf[k - 1] : ~0ull;
    return keep;
}

// Grid (parts, ceil(nq / kPlainQT)).  CodeT: uint8_t (8-bit sub-codes) or uint16_t.
// LDS_TABLES: the tile's tables (K <= 256 entries each) are staged in LDS.
template <int M, typename CodeT, bool LDS_TABLES>
__global__ __launch_bounds__(kPlainThreads) void plain_scan_kernel(const float *__restrict__ tables, uint32_t K,
                                                                  const CodeT *__restrict__ codes, uint64_t n_codes,
                                                                  int nq, uint32_t k, uint64_t codes_per_part,
                                                                  uint64_t *__restrict__ partial)
{
    extern __shared__ __align__(16) uint8_t smem[];
    uint64_t *buf = reinterpret_cast<uint64_t *>(smem);                                  // [QT][kPlainBuf]
    float *ltab = reinterpret_cast<float *>(smem + sizeof(uint64_t) * kPlainQT * kPlainBuf);   // [QT][M][K]
    __shared__ uint32_t cnt[kPlainQT];
    __shared__ uint64_t tau[kPlainQT];
    const int tid = threadIdx.x;
    const int q0 = blockIdx.y * kPlainQT;
    const int nqt = min(kPlainQT, nq - q0);
    const uint64_t begin = static_cast<uint64_t>(blockIdx.x) * codes_per_part;
    const uint64_t end = min(n_codes, begin + codes_per_part);
    if (tid < kPlainQT) { cnt[tid] = 0; tau[tid] = ~0ull; }
    if constexpr (LDS_TABLES) {
        const size_t per_q = static_cast<size_t>(M) * K;
        for (size_t v = tid; v < static_cast<size_t>(nqt) * per_q; v += kPlainThreads)
            ltab[v] = tables[static_cast<size_t>(q0) * per_q + v];
    }
    __syncthreads();

    for (uint64_t base = begin; base < end; base += kPlainThreads) {
        const uint64_t i = base + tid;
        const bool live = i < end;
        uint32_t c[M];
#pragma unroll
        for (int j = 0; j < M; ++j) c[j] = live ? static_cast<uint32_t>(codes[i * M + j]) : 0u;
        for (int q = 0; q < nqt; ++q) {                                  // uniform
            float d;
            if constexpr (LDS_TABLES) {
                const float *t = ltab + static_cast<size_t>(q) * M * K;
                d = t[c[0]];
#pragma unroll
                for (int j = 1; j < M; ++j) d = __fadd_rn(d, t[static_cast<size_t>(j) * K + c[j]]);
            } else {
                const float *t = tables + static_cast<size_t>(q0 + q) * M * K;
                d = t[c[0]];
#pragma unroll
                for (int j = 1; j < M; ++j) d = __fadd_rn(d, t[static_cast<size_t>(j) * K + c[j]]);
            }
            const uint64_t key = make_key(ordered_bits(d), static_cast<uint32_t>(i));
            if (live && key < tau[q]) {
                const uint32_t pos = atomicAdd(&cnt[q], 1u);            // below kPlainBuf: at most kPlainMostK before this batch
                buf[q * kPlainBuf + pos] = key;
            }
        }
        __syncthreads();
        for (int q = 0; q < nqt; ++q) {                                  // uniform
            const uint32_t have = cnt[q];
            if (have > kPlainMostK) {                                    // uniform: no room for another batch
                const uint32_t keep = cut_to_k(buf + q * kPlainBuf, have, k, &tau[q]);
                if (tid == 0) cnt[q] = keep;
                __syncthreads();
            }
        }
    }
    for (int q = 0; q < nqt; ++q) {
        const uint32_t keep = cut_to_k(buf + q * kPlainBuf, cnt[q], k, &tau[q]);
        __syncthreads();
        uint64_t *out = partial + (static_cast<size_t>(q0 + q) * gridDim.x + blockIdx.x) * k;
        for (uint32_t t = tid; t < k; t += kPlainThreads) out[t] = t < keep ? buf[q * kPlainBuf + t] : ~0ull;
        __syncthreads();
    }
}

// One workgroup per query: the k smallest of its parts' keys.
__global__ __launch_bounds__(1024) void plain_merge_kernel(const uint64_t *__restrict__ partial, uint32_t nkeys, uint32_t k,
                                                          uint32_t *__restrict__ ids, float *__restrict__ dist)
{
    extern __shared__ __align__(16) uint8_t smem[];
    uint64_t *a = reinterpret_cast<uint64_t *>(smem);
    const int q = blockIdx.x;
    uint32_t np2 = 1;
    while (np2 < nkeys) np2 <<= 1;
    for (uint32_t t = threadIdx.x; t < np2; t += blockDim.x) a[t] = t < nkeys ? partial[static_cast<size_t>(q) * nkeys + t] : ~0ull;
    bitonic_sort(a, np2);
    for (uint32_t t = threadIdx.x; t < k; t += blockDim.x) {
        const uint64_t key = a[t];
        ids[static_cast<size_t>(q) * k + t] = static_cast<uint32_t>(key);
        dist[static_cast<size_t>(q) * k + t] = from_ordered_bits(static_cast<uint32_t>(key >> 32));
    }
}

static uint32_t plain_parts(uint64_t n_codes, uint32_t k)
{
    uint64_t parts = kPlainMerge / k;                      // what the merge can sort
    if (parts > 64) parts = 64;
    const uint64_t most = (n_codes + 4095) / 4096;         // at least 4096 codes per part
    if (parts > most) parts = most;
    return static_cast<uint32_t>(parts < 1 ? 1 : parts);
}

template <int M, typename CodeT>
static int plain_launch(const float *tables, uint32_t K, const CodeT *codes, uint64_t n_codes, int nq, uint32_t k,
                        uint32_t *ids, float *dist, uint64_t *partial, hipStream_t st)
{
    const uint32_t parts = plain_parts(n_codes, k);
    const uint64_t cpp = (n_codes + parts - 1) / parts;
    const dim3 grid(parts, (nq + kPlainQT - 1) / kPlainQT);
    const size_t buf_bytes = sizeof(uint64_t) * kPlainQT * kPlainBuf;
    const size_t lds = buf_bytes + sizeof(float) * kPlainQT * M * K;
    if (lds <= 144 * 1024) {                               // the tile's tables fit beside the buffers
        int rc = allow_dynamic_lds(reinterpret_cast<const void *>(&plain_scan_kernel<M, CodeT, true>), static_cast<int>(lds));
        if (rc) return rc;
        DCPQ_LAUNCH(kStagePlainScan, st, (plain_scan_kernel<M, CodeT, true>), grid, dim3(kPlainThreads), lds, tables, K, codes,
                    n_codes, nq, k, cpp, partial);
    } else {
        int rc = allow_dynamic_lds(reinterpret_cast<const void *>(&plain_scan_kernel<M, CodeT, false>), static_cast<int>(buf_bytes));
        if (rc) return rc;
        DCPQ_LAUNCH(kStagePlainScan, st, (plain_scan_kernel<M, CodeT, false>), grid, dim3(kPlainThreads), buf_bytes, tables, K,
                    codes, n_codes, nq, k, cpp, partial);
    }
    DCPQ_CHECK_LAUNCH("plain_scan_kernel");
    int rc = allow_dynamic_lds(reinterpret_cast<const void *>(&plain_merge_kernel), static_cast<int>(sizeof(uint64_t) * kPlainMerge));
    if (rc) return rc;
    uint32_t np2 = 1;
    while (np2 < parts * k) np2 <<= 1;
    DCPQ_LAUNCH(kStageSelect, st, plain_merge_kernel, dim3(nq), dim3(1024), sizeof(uint64_t) * np2, partial, parts * k, k, ids, dist);
    DCPQ_CHECK_LAUNCH("plain_merge_kernel");
    return DCPQ_OK;
}

template <typename CodeT>
static int plain_dispatch(const float *tables, uint32_t K, const CodeT *codes, uint64_t n_codes, int m, int nq, uint32_t k,
                          uint32_t *ids, float *dist, uint64_t *partial, hipStream_t st)
{
    switch (m) {
        case 1: return plain_launch<1>(tables, K, codes, n_codes, nq, k, ids, dist, partial, st);
        case 2: return plain_launch<2>(tables, K, codes, n_codes, nq, k, ids, dist, partial, st);
        case 4: return plain_launch<4>(tables, K, codes, n_codes, nq, k, ids, dist, partial, st);
        case 8: return plain_launch<8>(tables, K, codes, n_codes, nq, k, ids, dist, partial, st);
        case 16: return plain_launch<16>(tables, K, codes, n_codes, nq, k, ids, dist, partial, st);
        case 32: return plain_launch<32>(tables, K, codes, n_codes, nq, k, ids, dist, partial, st);
        default: return fail(DCPQ_EUNSUPPORTED, "plain_search: m=%d not supported", m);
    }
}

}  // namespace dcpq

using namespace dcpq;

extern "C" size_t dcpq_plain_workspace_bytes(uint64_t n_codes, int nq, uint32_t k)
{
    if (nq <= 0 || k == 0 || k > kPlainMostK || n_codes == 0) return 0;
    return align_up(sizeof(uint64_t) * static_cast<size_t>(nq) * plain_parts(n_codes, k) * k, 256);
}

extern "C" int dcpq_plain_search(const float *tables, uint32_t n_entries, const void *codes, int code_bytes,
                                 uint64_t n_codes, int m, int nq, uint32_t k, uint32_t *ids, float *dist,
                                 void *workspace, size_t workspace_bytes, void *stream)
{
    clear_error();
    DCPQ_REQUIRE(nq >= 0, "plain_search: nq=%d", nq);
    if (!m_supported(m)) return fail(DCPQ_EUNSUPPORTED, "plain_search: m=%d not supported", m);
    DCPQ_REQUIRE(code_bytes == 1 || code_bytes == 2, "plain_search: code_bytes=%d (1 or 2)", code_bytes);
    DCPQ_REQUIRE(n_entries >= 1 && n_entries <= (code_bytes == 1 ? 256u : 65536u),
                 "plain_search: n_entries=%u does not fit a sub-code of %d byte(s)", n_entries, code_bytes);
    DCPQ_REQUIRE(n_codes >= 1 && n_codes < (1ull << 32), "plain_search: n_codes out of range");
    DCPQ_REQUIRE(k >= 1 && k <= n_codes, "plain_search: needs 1 <= k <= n_codes (k=%u)", k);
    if (k > kPlainMostK) return fail(DCPQ_EUNSUPPORTED, "plain_search: k=%u above the supported %u", k, kPlainMostK);
    if (nq == 0) return DCPQ_OK;
    DCPQ_REQUIRE(tables && codes && ids && dist && workspace, "plain_search: null pointer");
    DCPQ_REQUIRE((reinterpret_cast<uintptr_t>(workspace) & 255) == 0, "plain_search: workspace must be 256-byte aligned");
    const size_t need = dcpq_plain_workspace_bytes(n_codes, nq, k);
    if (workspace_bytes < need) return fail(DCPQ_EWORKSPACE, "plain_search: workspace %zu < %zu bytes", workspace_bytes, need);
    uint64_t *partial = static_cast<uint64_t *>(workspace);
    hipStream_t st = as_stream(stream);
    if (code_bytes == 1)
        return plain_dispatch(tables, n_entries, static_cast<const uint8_t *>(codes), n_codes, m, nq, k, ids, dist, partial, st);
    return plain_dispatch(tables, n_entries, static_cast<const uint16_t *>(codes), n_codes, m, nq, k, ids, dist, partial, st);
}
