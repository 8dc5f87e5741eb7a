// Pass one of Alg. 3 (Sec. 3.3, "Scan step"): adc_low_bits over the whole code array with the
// 8-bit quantized small tables, and the candidate set of exactly the r smallest by (qd, id).
//
// The paper's capped buckets (one bucket per integer distance 0..254, ids appended in list
// order, read out by increasing bucket) have an order-independent meaning: a 256-bin histogram
// of qd fixes the threshold bucket T that holds the r-th candidate; every id with qd < T is a
// candidate and bucket T contributes its smallest ids.  That is what is computed here, exactly
// and deterministically, in three streaming passes over the codes:
//   pass A  histogram of qd per query                       -> T and the number still needed from T
//   pass B  per (query, scan unit) count of qd == T         -> quota of bucket T per unit (prefix in id order)
//   pass C  collect ids with qd < T, and the first `quota` ids of bucket T in each unit
// followed by a per-query sort of the r keys (qd, id).
//
// Work layout: a wavefront owns one "unit" of consecutive codes and walks it 64 codes at a time
// (lane = code, fully coalesced 2m-byte loads), so id order inside a unit is (iteration, lane).
// A workgroup is 4 wavefronts and serves a tile of QT queries whose u8 tables (QT * m * 256
// bytes) sit in LDS; each lane gathers its m table bytes per query from LDS.
#include "common.h"

namespace dcpq {

constexpr int kScanThreads = 256;
constexpr int kScanWaves = kScanThreads / kWave;

enum ScanMode { kHist = 0, kTieCount = 1, kCollect = 2 };

// Low bytes of the m sub-codes of code i (property P1: the derived index is the low 8 bits).
template <int M>
__device__ inline void load_low_bytes(const uint16_t *__restrict__ codes, uint64_t i, uint32_t (&low)[M])
{
    if constexpr (M % 8 == 0) {
        const uint4 *p = reinterpret_cast<const uint4 *>(codes + i * M);
#pragma unroll
        for (int v = 0; v < M / 8; ++v) {
            const uint4 x = p[v];
            low[8 * v + 0] = x.x & 255u; low[8 * v + 1] = (x.x >> 16) & 255u;
            low[8 * v + 2] = x.y & 255u; low[8 * v + 3] = (x.y >> 16) & 255u;
            low[8 * v + 4] = x.z & 255u; low[8 * v + 5] = (x.z >> 16) & 255u;
            low[8 * v + 6] = x.w & 255u; low[8 * v + 7] = (x.w >> 16) & 255u;
        }
    } else if constexpr (M == 4) {
        const uint2 x = *reinterpret_cast<const uint2 *>(codes + i * 4);
        low[0] = x.x & 255u; low[1] = (x.x >> 16) & 255u;
        low[2] = x.y & 255u; low[3] = (x.y >> 16) & 255u;
    } else if constexpr (M == 2) {
        const uint32_t x = *reinterpret_cast<const uint32_t *>(codes + i * 2);
        low[0] = x & 255u; low[1] = (x >> 16) & 255u;
    } else {
        low[0] = codes[i] & 255u;
    }
}

template <int M, int QT, int MODE>
__global__ __launch_bounds__(kScanThreads) void scan_kernel(
    const uint16_t *__restrict__ codes, uint64_t n_codes, uint32_t unit, uint32_t nunits,
    const uint8_t *__restrict__ qtab, int nq, uint32_t r,
    uint32_t *__restrict__ hist,        // [nq][256]          (kHist: accumulated)
    const uint32_t *__restrict__ thr,   // [nq][2]            (kTieCount, kCollect: read)
    uint32_t *__restrict__ tie,         // [nq][nunits]       (kTieCount: counts out; kCollect: quotas in)
    uint32_t *__restrict__ counter,     // [nq]               (kCollect)
    uint64_t *__restrict__ keys)        // [nq][r]            (kCollect)
{
    extern __shared__ __align__(16) uint8_t smem[];
    uint8_t *ltab = smem;                                                   // [QT][M][256]
    uint32_t *lhist = reinterpret_cast<uint32_t *>(smem + QT * M * 256);    // [QT][256] (kHist)

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int q0 = blockIdx.y * QT;
    const int nqt = min(QT, nq - q0);

    // Stage the tile's tables; rows of absent queries are never read.
    {
        const uint4 *src = reinterpret_cast<const uint4 *>(qtab + static_cast<size_t>(q0) * M * 256);
        uint4 *dst = reinterpret_cast<uint4 *>(ltab);
        const int nvec = nqt * M * 256 / 16;
        for (int v = tid; v < nvec; v += kScanThreads) dst[v] = src[v];
        if (MODE == kHist)
            for (int v = tid; v < QT * 256; v += kScanThreads) lhist[v] = 0;
    }
    __syncthreads();

    const uint32_t u = blockIdx.x * kScanWaves + wave;          // this wavefront's unit
    const uint64_t begin = static_cast<uint64_t>(u) * unit;
    const uint64_t end = (u < nunits) ? min(n_codes, begin + unit) : begin;

    uint32_t T[QT], aux[QT];   // threshold bucket; kTieCount: running count, kCollect: quota left
#pragma unroll
    for (int q = 0; q < QT; ++q) {
        T[q] = 0; aux[q] = 0;
        if (MODE != kHist && q < nqt) {
            T[q] = thr[2 * (q0 + q)];
            if (MODE == kCollect && u < nunits) aux[q] = tie[static_cast<size_t>(q0 + q) * nunits + u];
        }
    }

    for (uint64_t base = begin; base < end; base += kWave) {
        const uint64_t i = base + lane;
        const bool live = i < end;
        uint32_t low[M];
        if (live) {
            load_low_bytes<M>(codes, i, low);
        } else {
#pragma unroll
            for (int j = 0; j < M; ++j) low[j] = 0;
        }
#pragma unroll
        for (int q = 0; q < QT; ++q) {
            if (q >= nqt) continue;                               // uniform
            const uint8_t *t = ltab + q * (M * 256);
            uint32_t s = 0;
#pragma unroll
            for (int j = 0; j < M; ++j) s += t[j * 256 + low[j]];
            const uint32_t qd = min(s, 255u);                     // saturate: 255 = beyond qmax
            if (MODE == kHist) {
                if (live) atomicAdd(&lhist[q * 256 + qd], 1u);
            } else if (MODE == kTieCount) {
                aux[q] += __popcll(__ballot(live && qd == T[q]));
            } else {
                const bool below = live && qd < T[q];
                const bool tied = live && qd == T[q];
                const uint64_t tied_mask = __ballot(tied);
                bool take = below;
                if (tied_mask) {                                  // uniform
                    const uint32_t rank = __popcll(tied_mask & ((1ull << lane) - 1ull));
                    take = below || (tied && rank < aux[q]);
                    const uint32_t n_tied = __popcll(tied_mask);
                    aux[q] = aux[q] > n_tied ? aux[q] - n_tied : 0u;
                }
                const uint64_t take_mask = __ballot(take);
                if (take_mask) {                                  // uniform, rare
                    const uint32_t n_take = __popcll(take_mask);
                    uint32_t slot0 = 0;
                    if (lane == 0) slot0 = atomicAdd(&counter[q0 + q], n_take);
                    slot0 = __shfl(slot0, 0, kWave);
                    if (take) {
                        const uint32_t slot = slot0 + __popcll(take_mask & ((1ull << lane) - 1ull));
                        if (slot < r)   // exactly r ids are taken over the whole scan; guard anyway
                            keys[static_cast<size_t>(q0 + q) * r + slot] = make_key(qd, static_cast<uint32_t>(i));
                    }
                }
            }
        }
    }

    if (MODE == kHist) {
        __syncthreads();
        for (int v = tid; v < nqt * 256; v += kScanThreads) {
            const uint32_t c = lhist[v];
            if (c) atomicAdd(&hist[static_cast<size_t>(q0) * 256 + v], c);
        }
    } else if (MODE == kTieCount) {
        if (u < nunits && lane == 0) {
#pragma unroll
            for (int q = 0; q < QT; ++q)
                if (q < nqt) tie[static_cast<size_t>(q0 + q) * nunits + u] = aux[q];
        }
    }
}

// T = bucket holding the r-th smallest qd; need = ids still to take from bucket T.
__global__ __launch_bounds__(256) void threshold_kernel(const uint32_t *__restrict__ hist, uint32_t r,
                                                        uint32_t *__restrict__ thr)
{
    __shared__ uint32_t cum[256];
    const int q = blockIdx.x, b = threadIdx.x;
    cum[b] = hist[static_cast<size_t>(q) * 256 + b];
    __syncthreads();
    for (int off = 1; off < 256; off <<= 1) {            // inclusive scan (Hillis-Steele)
        const uint32_t add = b >= off ? cum[b - off] : 0u;
        __syncthreads();
        cum[b] += add;
        __syncthreads();
    }
    const uint32_t before = b ? cum[b - 1] : 0u;
    if (before < r && cum[b] >= r) { thr[2 * q] = b; thr[2 * q + 1] = r - before; }
}

// Turns per-unit counts of bucket T into per-unit quotas: units are in id order, so unit u may
// take min(count_u, need - sum of counts before u) ids (its smallest ones).
__global__ __launch_bounds__(256) void tie_quota_kernel(uint32_t *__restrict__ tie, uint32_t nunits,
                                                        const uint32_t *__restrict__ thr)
{
    __shared__ uint32_t part[256];
    __shared__ uint32_t carry;
    const int q = blockIdx.x, t = threadIdx.x;
    uint32_t *row = tie + static_cast<size_t>(q) * nunits;
    const uint32_t need = thr[2 * q + 1];
    if (t == 0) carry = 0;
    __syncthreads();
    for (uint32_t base = 0; base < nunits; base += 256) {
        const uint32_t u = base + t;
        const uint32_t c = u < nunits ? row[u] : 0u;
        part[t] = c;
        __syncthreads();
        for (int off = 1; off < 256; off <<= 1) {
            const uint32_t add = t >= off ? part[t - off] : 0u;
            __syncthreads();
            part[t] += add;
            __syncthreads();
        }
        const uint32_t before = carry + part[t] - c;       // exclusive prefix in id order
        if (u < nunits) row[u] = before >= need ? 0u : min(c, need - before);
        __syncthreads();
        if (t == 255) carry += part[255];
        __syncthreads();
    }
}

// In-place bitonic sort of n_pow2 64-bit keys by one workgroup (array in LDS or global memory).
__device__ inline void bitonic_sort(uint64_t *a, uint32_t n_pow2)
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

// Sort the r collected keys of each query by (qd, id) and split them into the two outputs.
// use_lds: the padded array fits the dynamic LDS allocation; otherwise it is sorted in `spill`.
__global__ __launch_bounds__(1024) void sort_candidates_kernel(const uint64_t *__restrict__ keys, uint32_t r,
                                                              uint32_t n_pow2, int use_lds,
                                                              uint64_t *__restrict__ spill,
                                                              uint32_t *__restrict__ cand_id,
                                                              uint8_t *__restrict__ cand_qd)
{
    extern __shared__ __align__(16) uint8_t smem[];
    const int q = blockIdx.x;
    uint64_t *a = use_lds ? reinterpret_cast<uint64_t *>(smem) : spill + static_cast<size_t>(q) * n_pow2;
    for (uint32_t t = threadIdx.x; t < n_pow2; t += blockDim.x)
        a[t] = t < r ? keys[static_cast<size_t>(q) * r + t] : ~0ull;
    bitonic_sort(a, n_pow2);
    for (uint32_t t = threadIdx.x; t < r; t += blockDim.x) {
        const uint64_t key = a[t];
        cand_id[static_cast<size_t>(q) * r + t] = static_cast<uint32_t>(key);
        cand_qd[static_cast<size_t>(q) * r + t] = static_cast<uint8_t>(key >> 32);
    }
}

static uint32_t next_pow2(uint32_t x)
{
    uint32_t p = 1;
    while (p < x) p <<= 1;
    return p;
}

constexpr uint32_t kSortLdsKeys = 8192;   // 64 KiB of keys

constexpr int scan_qt(int m) { return m <= 8 ? 16 : 128 / m; }   // tables of a tile: <= 32 KiB of LDS

ScanPlan plan_scan(uint64_t n_codes, int m, int nq, uint32_t r)
{
    ScanPlan p{};
    p.qt = scan_qt(m);
    // Unit: enough wavefronts to fill the chip (256 CUs) several times over, 64..16384 codes each.
    const uint64_t qtiles = (static_cast<uint64_t>(nq) + p.qt - 1) / p.qt;
    uint64_t unit = 16384;
    while (unit > 64 && (n_codes + unit - 1) / unit * (qtiles ? qtiles : 1) < 8192) unit >>= 1;
    p.unit = static_cast<uint32_t>(unit);
    p.nunits = static_cast<uint32_t>((n_codes + unit - 1) / unit);
    const uint32_t np2 = next_pow2(r);
    size_t off = 0;
    p.off_hist = off;    off = align_up(off + sizeof(uint32_t) * 256 * static_cast<size_t>(nq), 256);
    p.off_thr = off;     off = align_up(off + sizeof(uint32_t) * 2 * static_cast<size_t>(nq), 256);
    p.off_counter = off; off = align_up(off + sizeof(uint32_t) * static_cast<size_t>(nq), 256);
    p.off_tie = off;     off = align_up(off + sizeof(uint32_t) * static_cast<size_t>(nq) * p.nunits, 256);
    p.off_keys = off;    off = align_up(off + sizeof(uint64_t) * static_cast<size_t>(nq) * r, 256);
    p.off_spill = off;   // sort area in global memory, only when r keys do not fit the LDS sort
    if (np2 > kSortLdsKeys) off = align_up(off + sizeof(uint64_t) * static_cast<size_t>(nq) * np2, 256);
    p.total = off;
    return p;
}

// Clears `n` 32-bit words (a fill kernel rather than a memset node, so that the call sequence
// stays safe to capture into a HIP graph).
__global__ void zero_words_kernel(uint32_t *p, size_t n)
{
    const size_t i = static_cast<size_t>(blockIdx.x) * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0u;
}

template <int M>
static int launch_scan_m(const uint16_t *codes, uint64_t n_codes, const uint8_t *qtab, int nq, uint32_t r,
                         uint32_t *cand_id, uint8_t *cand_qd, void *ws, hipStream_t st)
{
    constexpr int QT = scan_qt(M);
    const ScanPlan p = plan_scan(n_codes, M, nq, r);
    uint8_t *base = static_cast<uint8_t *>(ws);
    uint32_t *hist = reinterpret_cast<uint32_t *>(base + p.off_hist);
    uint32_t *thr = reinterpret_cast<uint32_t *>(base + p.off_thr);
    uint32_t *counter = reinterpret_cast<uint32_t *>(base + p.off_counter);
    uint32_t *tie = reinterpret_cast<uint32_t *>(base + p.off_tie);
    const bool spill = next_pow2(r) > kSortLdsKeys;
    uint64_t *keys = reinterpret_cast<uint64_t *>(base + p.off_keys);
    uint64_t *sorted = reinterpret_cast<uint64_t *>(base + p.off_spill);

    // hist, thr and counter are contiguous at the head of the workspace: one clear.
    const size_t nwords = p.off_tie / sizeof(uint32_t);
    DCPQ_LAUNCH(kStageMisc, st, zero_words_kernel, dim3((nwords + 255) / 256), dim3(256), 0,
                reinterpret_cast<uint32_t *>(base), nwords);
    DCPQ_CHECK_LAUNCH("zero_words_kernel");

    const dim3 grid((p.nunits + kScanWaves - 1) / kScanWaves, (nq + QT - 1) / QT);
    const size_t lds_tab = static_cast<size_t>(QT) * M * 256;
    DCPQ_LAUNCH(kStageScanHist, st, (scan_kernel<M, QT, kHist>), grid, dim3(kScanThreads), lds_tab + QT * 256 * 4,
                codes, n_codes, p.unit, p.nunits, qtab, nq, r, hist, thr, tie, counter, keys);
    DCPQ_CHECK_LAUNCH("scan_kernel<hist>");
    DCPQ_LAUNCH(kStageSelect, st, threshold_kernel, dim3(nq), dim3(256), 0, hist, r, thr);
    DCPQ_CHECK_LAUNCH("threshold_kernel");
    DCPQ_LAUNCH(kStageScanTieCount, st, (scan_kernel<M, QT, kTieCount>), grid, dim3(kScanThreads), lds_tab, codes,
                n_codes, p.unit, p.nunits, qtab, nq, r, hist, thr, tie, counter, keys);
    DCPQ_CHECK_LAUNCH("scan_kernel<tiecount>");
    DCPQ_LAUNCH(kStageSelect, st, tie_quota_kernel, dim3(nq), dim3(256), 0, tie, p.nunits, thr);
    DCPQ_CHECK_LAUNCH("tie_quota_kernel");
    DCPQ_LAUNCH(kStageScanCollect, st, (scan_kernel<M, QT, kCollect>), grid, dim3(kScanThreads), lds_tab, codes,
                n_codes, p.unit, p.nunits, qtab, nq, r, hist, thr, tie, counter, keys);
    DCPQ_CHECK_LAUNCH("scan_kernel<collect>");
    const uint32_t np2 = next_pow2(r);
    DCPQ_LAUNCH(kStageSelect, st, sort_candidates_kernel, dim3(nq), dim3(1024), spill ? 0 : sizeof(uint64_t) * np2,
                keys, r, np2, spill ? 0 : 1, sorted, cand_id, cand_qd);
    DCPQ_CHECK_LAUNCH("sort_candidates_kernel");
    return DCPQ_OK;
}

int launch_scan(const uint16_t *codes, uint64_t n_codes, int m, const uint8_t *qtab, int nq, uint32_t r,
                uint32_t *cand_id, uint8_t *cand_qd, void *ws, hipStream_t st)
{
    if (nq == 0) return DCPQ_OK;
    switch (m) {
        case 1: return launch_scan_m<1>(codes, n_codes, qtab, nq, r, cand_id, cand_qd, ws, st);
        case 2: return launch_scan_m<2>(codes, n_codes, qtab, nq, r, cand_id, cand_qd, ws, st);
        case 4: return launch_scan_m<4>(codes, n_codes, qtab, nq, r, cand_id, cand_qd, ws, st);
        case 8: return launch_scan_m<8>(codes, n_codes, qtab, nq, r, cand_id, cand_qd, ws, st);
        case 16: return launch_scan_m<16>(codes, n_codes, qtab, nq, r, cand_id, cand_qd, ws, st);
        case 32: return launch_scan_m<32>(codes, n_codes, qtab, nq, r, cand_id, cand_qd, ws, st);
        default: return fail(DCPQ_EUNSUPPORTED, "m=%d not supported", m);
    }
}

}  // namespace dcpq

using namespace dcpq;

extern "C" int dcpq_scan_query_tile(int m) { return m_supported(m) ? scan_qt(m) : 0; }

extern "C" size_t dcpq_scan_workspace_bytes(uint64_t n_codes, int m, int nq, uint32_t r)
{
    if (nq <= 0 || !m_supported(m) || n_codes == 0 || r == 0) return 0;
    return plan_scan(n_codes, m, nq, r).total;
}

extern "C" int dcpq_scan_candidates(const uint16_t *codes, uint64_t n_codes, int m, const uint8_t *qtab, int nq,
                                    uint32_t r, uint32_t *cand_id, uint8_t *cand_qd, void *workspace,
                                    size_t workspace_bytes, void *stream)
{
    clear_error();
    DCPQ_REQUIRE(nq >= 0, "scan_candidates: nq=%d", nq);
    if (!m_supported(m)) return fail(DCPQ_EUNSUPPORTED, "scan_candidates: m=%d not supported", m);
    DCPQ_REQUIRE(n_codes >= 1 && n_codes < (1ull << 32), "scan_candidates: n_codes=%llu must be in [1, 2^32)",
                 static_cast<unsigned long long>(n_codes));
    DCPQ_REQUIRE(r >= 1 && r <= n_codes, "scan_candidates: r=%u must be in [1, n_codes]", r);
    if (nq == 0) return DCPQ_OK;
    DCPQ_REQUIRE(codes && qtab && cand_id && cand_qd && workspace, "scan_candidates: null pointer");
    DCPQ_REQUIRE((reinterpret_cast<uintptr_t>(workspace) & 255) == 0, "scan_candidates: workspace must be 256-byte aligned");
    DCPQ_REQUIRE((reinterpret_cast<uintptr_t>(codes) & 15) == 0 && (reinterpret_cast<uintptr_t>(qtab) & 15) == 0,
                 "scan_candidates: codes and qtab must be 16-byte aligned");
    const size_t need = dcpq_scan_workspace_bytes(n_codes, m, nq, r);
    if (workspace_bytes < need)
        return fail(DCPQ_EWORKSPACE, "scan_candidates: workspace %zu < %zu bytes", workspace_bytes, need);
    return launch_scan(codes, n_codes, m, qtab, nq, r, cand_id, cand_qd, workspace, as_stream(stream));
}
