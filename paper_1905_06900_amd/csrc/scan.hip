// Pass one of Alg. 3 (Sec. 3.3, "Scan step"): adc_low_bits over the whole code array with the
// 8-bit quantized small tables, and the candidate set of exactly the r smallest by (qd, id).
//
// The paper's capped buckets (one bucket per integer distance 0..254, ids appended in list
// order, read out by increasing bucket) have an order-independent meaning: a 256-bin histogram
// of qd fixes the threshold bucket T that holds the r-th candidate; every id with qd < T is a
// candidate and bucket T contributes its smallest ids.
//
// This file holds (a) the THREE-PASS path, which computes exactly that for any input in three
// streaming passes over the codes:
//   pass A  histogram of qd per query                       -> T and the number still needed from T
//   pass B  per (query, scan unit) count of qd == T         -> quota of bucket T per unit (prefix in id order)
//   pass C  collect ids with qd < T, and the first `quota` ids of bucket T in each unit
// followed by a per-query sort of the r keys (qd, id); and (b) the driver that runs the
// single-pass kernel of scan_fast.hip first and sends only the queries it flags through (a).
//
// Three-pass work layout: a wavefront owns one "unit" of consecutive codes and walks it 64 codes
// at a time (lane = code, fully coalesced 2m-byte loads), so id order inside a unit is
// (iteration, lane).  A workgroup is 4 wavefronts and serves a tile of QT queries whose u8 tables
// (QT * m * 256 bytes) sit in LDS; each lane gathers its m table bytes per query from LDS.
// Workgroups walk a list of (query tile, block of 4 units) items with a grid stride, so the same
// launch shape serves "all queries" and "the few flagged queries" (count read on the device).
#include <cmath>

#include "common.h"
#include <mutex>

#include "scan_internal.h"

namespace dcpq {

constexpr int kScanThreads = 256;
constexpr int kScanWaves = kScanThreads / kWave;

enum ScanMode { kHist = 0, kTieCount = 1, kCollect = 2 };

// Queries are addressed by their position p in the active list: query id = qlist ? qlist[p] : p.
// Workspace arrays (hist, thr, tie, counter, keys) are indexed by p; qtab by the query id.
// CodeT: uint16_t (the codes as stored) or uint8_t (their low-byte plane).
template <int M, int QT, int MODE, typename CodeT>
__global__ __launch_bounds__(kScanThreads) void scan_kernel(
    const CodeT *__restrict__ codes, uint64_t n_codes, uint32_t unit, uint32_t nunits, uint64_t unit_stride,
    const uint8_t *__restrict__ qtab, int nq_host, const int *__restrict__ qlist,
    const uint32_t *__restrict__ nq_dev, uint32_t r,
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
    const int nq = nq_dev ? static_cast<int>(*nq_dev) : nq_host;
    const uint32_t nxb = (nunits + kScanWaves - 1) / kScanWaves;
    const uint64_t nitems = static_cast<uint64_t>((nq + QT - 1) / QT) * nxb;

    for (uint64_t item = blockIdx.x; item < nitems; item += gridDim.x) {
        const int q0 = static_cast<int>(item / nxb) * QT;
        const uint32_t xb = static_cast<uint32_t>(item % nxb);
        const int nqt = min(QT, nq - q0);

        __syncthreads();                       // previous item's LDS is no longer in use
        for (int q = 0; q < nqt; ++q) {        // stage the tile's tables (rows of absent queries are never read)
            const int qid = qlist ? qlist[q0 + q] : q0 + q;
            const uint4 *src = reinterpret_cast<const uint4 *>(qtab + static_cast<size_t>(qid) * M * 256);
            uint4 *dst = reinterpret_cast<uint4 *>(ltab + q * M * 256);
            for (int v = tid; v < M * 256 / 16; v += kScanThreads) dst[v] = src[v];
        }
        if (MODE == kHist)
            for (int v = tid; v < QT * 256; v += kScanThreads) lhist[v] = 0;
        __syncthreads();

        const uint32_t u = xb * kScanWaves + wave;          // this wavefront's unit
        const uint64_t begin = static_cast<uint64_t>(u) * unit_stride;
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
}

// T = bucket holding the r-th smallest qd; need = ids still to take from bucket T.
__global__ __launch_bounds__(256) void threshold_kernel(const uint32_t *__restrict__ hist, uint32_t r,
                                                        const uint32_t *__restrict__ nq_dev,
                                                        uint32_t *__restrict__ thr)
{
    __shared__ uint32_t cum[256];
    const int q = blockIdx.x, b = threadIdx.x;
    if (nq_dev && q >= static_cast<int>(*nq_dev)) return;
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
    // fewer than r codes in all (inverted lists only): bucket "256" takes everything
    if (b == 255 && cum[255] < r) { thr[2 * q] = 256; thr[2 * q + 1] = 0; }
}

// Turns per-unit counts of bucket T into per-unit quotas: units are in id order, so unit u may
// take min(count_u, need - sum of counts before u) ids (its smallest ones).
__global__ __launch_bounds__(256) void tie_quota_kernel(uint32_t *__restrict__ tie, uint32_t nunits,
                                                        const uint32_t *__restrict__ nq_dev,
                                                        const uint32_t *__restrict__ thr)
{
    __shared__ uint32_t part[256];
    __shared__ uint32_t carry;
    const int q = blockIdx.x, t = threadIdx.x;
    if (nq_dev && q >= static_cast<int>(*nq_dev)) return;
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

// Sort the r collected keys of each active query by (qd, id) and split them into the two outputs.
// use_lds: the padded array fits the dynamic LDS allocation; otherwise it is sorted in `spill`.
__global__ __launch_bounds__(1024) void sort_candidates_kernel(const uint64_t *__restrict__ keys, uint32_t r,
                                                              uint32_t n_pow2, int use_lds,
                                                              uint64_t *__restrict__ spill,
                                                              const int *__restrict__ qlist,
                                                              const uint32_t *__restrict__ nq_dev,
                                                              const uint32_t *__restrict__ flags,
                                                              uint32_t *__restrict__ cand_id,
                                                              uint8_t *__restrict__ cand_qd)
{
    extern __shared__ __align__(16) uint8_t smem[];
    const int p = blockIdx.x;
    if (nq_dev && p >= static_cast<int>(*nq_dev)) return;
    const int qid = qlist ? qlist[p] : p;
    if (flags && flags[qid] == 0) return;
    uint64_t *a = use_lds ? reinterpret_cast<uint64_t *>(smem) : spill + static_cast<size_t>(p) * n_pow2;
    for (uint32_t t = threadIdx.x; t < n_pow2; t += blockDim.x)
        a[t] = t < r ? keys[static_cast<size_t>(p) * r + t] : ~0ull;
    bitonic_sort(a, n_pow2);
    for (uint32_t t = threadIdx.x; t < r; t += blockDim.x) {
        const uint64_t key = a[t];
        cand_id[static_cast<size_t>(qid) * r + t] = static_cast<uint32_t>(key);
        cand_qd[static_cast<size_t>(qid) * r + t] = static_cast<uint8_t>(key >> 32);
    }
}

// Clears `n` 32-bit words (a fill kernel rather than a memset node, so that the call sequence
// stays safe to capture into a HIP graph).
__global__ void zero_words_kernel(uint32_t *p, size_t n)
{
    const size_t i = static_cast<size_t>(blockIdx.x) * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0u;
}

__global__ void fill_u64_kernel(uint64_t *p, size_t n, uint64_t v)
{
    const size_t i = static_cast<size_t>(blockIdx.x) * blockDim.x + threadIdx.x;
    if (i < n) p[i] = v;
}

int launch_zero_words(uint32_t *p, size_t nwords, hipStream_t st)
{
    if (!nwords) return DCPQ_OK;
    DCPQ_LAUNCH(kStageMisc, st, zero_words_kernel, dim3((nwords + 255) / 256), dim3(256), 0, p, nwords);
    DCPQ_CHECK_LAUNCH("zero_words_kernel");
    return DCPQ_OK;
}

int launch_fill_u64(uint64_t *p, size_t n, uint64_t v, hipStream_t st)
{
    if (!n) return DCPQ_OK;
    DCPQ_LAUNCH(kStageMisc, st, fill_u64_kernel, dim3((n + 255) / 256), dim3(256), 0, p, n, v);
    DCPQ_CHECK_LAUNCH("fill_u64_kernel");
    return DCPQ_OK;
}

int launch_threshold(const uint32_t *hist, int nq, uint32_t r, uint32_t *thr, hipStream_t st)
{
    DCPQ_LAUNCH(kStageSelect, st, threshold_kernel, dim3(nq), dim3(256), 0, hist, r, nullptr, thr);
    DCPQ_CHECK_LAUNCH("threshold_kernel");
    return DCPQ_OK;
}

int launch_tie_quota(uint32_t *tie, uint32_t nunits, int nq, const uint32_t *thr, hipStream_t st)
{
    DCPQ_LAUNCH(kStageSelect, st, tie_quota_kernel, dim3(nq), dim3(256), 0, tie, nunits, nullptr, thr);
    DCPQ_CHECK_LAUNCH("tie_quota_kernel");
    return DCPQ_OK;
}

int launch_sort_candidates(const uint64_t *keys, int nq, uint32_t r, uint64_t *spill, uint32_t *cand_id,
                           uint8_t *cand_qd, hipStream_t st, const uint32_t *flags)
{
    const uint32_t np2 = next_pow2(r);
    const bool use_spill = np2 > kSortLdsKeys;
    DCPQ_LAUNCH(kStageSelect, st, sort_candidates_kernel, dim3(nq), dim3(1024), use_spill ? 0 : sizeof(uint64_t) * np2,
                keys, r, np2, use_spill ? 0 : 1, spill, nullptr, nullptr, flags, cand_id, cand_qd);
    DCPQ_CHECK_LAUNCH("sort_candidates_kernel");
    return DCPQ_OK;
}

constexpr int scan_qt(int m) { return m <= 8 ? 16 : 128 / m; }   // tables of a tile: <= 32 KiB of LDS

// Queries per tile of the single-pass kernel.  Large batches take the largest tile (most queries per
// byte of code stream); for m = 8 a batch that fits a smaller tile takes that one, so that a small
// batch does not pay for absent queries and the scan runs at the speed of the code stream.
int fast_query_tile(int m, int nq, int mode)
{
    if (mode == DCPQ_SCAN_TILE16 || mode == DCPQ_SCAN_TILE32 || mode == DCPQ_SCAN_TILE64) {
        const int qt = mode == DCPQ_SCAN_TILE16 ? 16 : mode == DCPQ_SCAN_TILE32 ? 32 : 64;
        return fast_table_bytes(m, qt) ? qt : 0;
    }
    switch (m) {
        case 4: return 64;
        case 8: return nq <= 16 ? 16 : nq <= 32 ? 32 : 64;
        case 16: return 32;
        case 32: return 16;
        default: return 0;
    }
}

ScanPlan plan_scan(uint64_t n_codes, int m, int nq, uint32_t r, int mode)
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
    const size_t Q = static_cast<size_t>(nq);
    size_t off = 0;
    p.off_hist = off;    off = align_up(off + sizeof(uint32_t) * 256 * Q, 256);
    p.off_thr = off;     off = align_up(off + sizeof(uint32_t) * 2 * Q, 256);
    p.off_counter = off; off = align_up(off + sizeof(uint32_t) * Q, 256);
    p.zero_bytes = off;
    p.off_tie = off;     off = align_up(off + sizeof(uint32_t) * Q * p.nunits, 256);
    p.off_keys = off;    off = align_up(off + sizeof(uint64_t) * Q * r, 256);
    p.off_spill = off;   // sort area in global memory, only when r keys do not fit the LDS sort
    if (np2 > kSortLdsKeys) off = align_up(off + sizeof(uint64_t) * Q * np2, 256);

    p.fqt = static_cast<uint32_t>(mode == DCPQ_SCAN_THREE_PASS ? 0 : fast_query_tile(m, nq, mode));
    p.fast = p.fqt != 0;
    if (p.fast) {
        p.ntiles = static_cast<uint32_t>((Q + p.fqt - 1) / p.fqt);
        // workgroups along the codes, at least 16 Ki codes each
        const uint64_t rest = n_codes;
        // (a single tile does the same work in every workgroup, and one round of the 256 CUs measured
        // fastest for it; with several tiles the work per workgroup varies and more rounds even it out)
        // Several tiles: at least 2048 workgroups in all and at least 128 per tile (measured: 4096 queries = 64
        // tiles take 45.3 ms with 2048 workgroups, 41.5 ms with 8192, 43.4 ms with 131072; the rounds of
        // workgroups end unevenly, the more so the longer a workgroup runs).
        const uint64_t total = 128ull * p.ntiles > 2048 ? 128ull * p.ntiles : 2048;
        const uint64_t want = p.ntiles == 1 ? 256 : (total + p.ntiles - 1) / p.ntiles;
        const uint64_t most = (rest + 16383) / 16384;
        uint64_t fb = want < most ? want : most;
        if (fb < 1) fb = 1;
        uint64_t cpb = (rest + fb - 1) / fb;
        cpb = (cpb + 1023) / 1024 * 1024;
        p.codes_per_block = static_cast<uint32_t>(cpb);
        p.fblocks = static_cast<uint32_t>((rest + cpb - 1) / cpb);
        p.slices = p.fblocks < static_cast<uint32_t>(kFastSlices) ? p.fblocks : kFastSlices;
        {
            const uint64_t share = 32ull * r / p.slices;         // 32 r per query in all: twice the even share
            p.cap = static_cast<uint32_t>(share < 1024 ? 1024 : share);
        }
        p.upd = r / 16 < 16 ? 16 : r / 16;                   // appends to one slice between bound updates
        // Candidates waiting in the wavefronts' queues are invisible to the bound.  With few queries and
        // thousands of wavefronts they would outnumber r, so a wavefront hands its queue over as soon as
        // it holds its share of r / 4 waiting candidates per query (between 4 and a full queue of 64).
        {
            const uint64_t conc = 256 / p.ntiles ? 256 / p.ntiles : 1;             // workgroups of a tile at a time
            const uint64_t blocks = conc < p.fblocks ? conc : p.fblocks;
            const uint64_t tile_q = Q < p.fqt ? Q : p.fqt;
            uint64_t lim = static_cast<uint64_t>(r / 4) * tile_q / (blocks * 16);
            p.qflush = static_cast<uint32_t>(lim < 4 ? 4 : lim > 64 ? 64 : lim);
        }
        const uint32_t want_sort = next_pow2(2 * r);
        p.sortcap = want_sort < kSortLdsKeys ? kSortLdsKeys : want_sort;
        // sample: runs of 256 codes spread evenly over the array, 32 r to 256 r codes (at least 64 Ki)
        // (the larger the sample, the closer the starting bound and the fewer candidates are appended,
        // but its cost grows with the number of queries: 256 r codes for 16 queries, 32 r from 128 on)
        uint64_t mul = 4096 / (Q ? Q : 1);
        mul = mul < 32 ? 32 : mul > 256 ? 256 : mul;
        uint64_t s_codes = mul * r < 65536 ? 65536 : mul * r;
        // With a pilot pass (below; worth its extra launches when the histogram of the sample would take a
        // tenth of a millisecond or more) the sample costs several times less per code, and is taken twice as
        // large where it is small against the array (measured at N = 1e8, r = 4000, 4096 queries: sample and
        // scan together 41.25, 40.93, 40.72, 40.90 ms with 1, 2, 4, 8 times the sample; at N = 1e7, r = 5000
        // the larger sample costs what it saves).
        const bool want_pilot = s_codes * Q * static_cast<uint64_t>(m) >= 500000000ull;
        if (want_pilot && n_codes / r >= 10000) s_codes *= 2;
        if (s_codes > n_codes) s_codes = n_codes;
        p.s_unit = 256;
        p.s_nunits = static_cast<uint32_t>((s_codes + 255) / 256);
        p.s_stride = n_codes / p.s_nunits;
        if (p.s_stride < p.s_unit) p.s_stride = p.s_unit;
        // Pilot pass.  The histogram kernel gathers bytes and is an order of magnitude slower per (code, query)
        // than the single-pass kernel, so on a large array it reads only one run in kPilotEvery of the sample;
        // its histogram gives a bound below which the WHOLE sample is then counted by the single-pass kernel
        // itself (a few hundred hits per query), and those exact counts give the starting bound of the scan.
        p.s_count = static_cast<uint64_t>(p.s_nunits - 1) * p.s_unit;
        {
            const uint64_t last = static_cast<uint64_t>(p.s_nunits - 1) * p.s_stride;
            p.s_count += n_codes - last < p.s_unit ? n_codes - last : p.s_unit;
        }
        p.pilot = want_pilot && p.s_nunits >= 4 * kPilotEvery && p.s_count * 4 <= n_codes && p.s_stride >= p.s_unit;
        p.s1_nunits = p.pilot ? p.s_nunits / kPilotEvery : p.s_nunits;
        p.pilot_r = r;
        p.pilot_blocks = p.pilot_runs = 0;
        if (p.pilot) {
            const double e = static_cast<double>(r) * static_cast<double>(p.s_count) / static_cast<double>(n_codes);
            const double want = e + 5.0 * sqrt(e) + 5.0;            // as in sample_threshold_kernel
            if (want < static_cast<double>(r)) p.pilot_r = static_cast<uint32_t>(want) + 1u;
            // at least 16 runs (4096 codes) per workgroup against the cost of loading the tile's tables, about
            // 1024 workgroups in all
            uint32_t pb = p.s_nunits / 16;
            const uint32_t most = 1024 / p.ntiles ? 1024 / p.ntiles : 1;
            pb = pb > most ? most : pb;
            p.pilot_runs = (p.s_nunits + pb - 1) / pb;
            p.pilot_blocks = (p.s_nunits + p.pilot_runs - 1) / p.pilot_runs;
        }
        p.off_fzero = off;
        p.off_fcount = off;  off = align_up(off + sizeof(uint32_t) * Q * p.slices, 256);
        p.off_chist = off;   off = align_up(off + sizeof(uint32_t) * 256 * Q, 256);
        p.off_shist = off;   off = align_up(off + sizeof(uint32_t) * 256 * Q, 256);
        p.off_nflag = off;   off = align_up(off + 256, 256);
        p.fzero_bytes = off - p.off_fzero;
        p.off_tcur = off;    off = align_up(off + sizeof(int32_t) * Q, 256);
        p.off_flags = off;   off = align_up(off + sizeof(uint32_t) * Q, 256);
        p.off_qlist = off;   off = align_up(off + sizeof(int32_t) * Q, 256);
        p.off_qsw = off;     off = align_up(off + static_cast<size_t>(p.ntiles) * fast_table_bytes(m, p.fqt), 256);
        p.off_fkeys = off;   off = align_up(off + sizeof(uint64_t) * Q * p.slices * p.cap, 256);
        p.off_fsort = off;
        if (p.sortcap > kSortLdsKeys) off = align_up(off + sizeof(uint64_t) * Q * p.sortcap, 256);
    }
    p.total = off;
    return p;
}

template <int M, int MODE, typename CodeT>
static void launch_scan_pass(int stage, const CodeT *codes, uint64_t n_codes, uint32_t unit, uint32_t nunits,
                             uint64_t stride, const uint8_t *qtab, int nq, const int *qlist, const uint32_t *nq_dev,
                             uint32_t r, uint32_t *hist, const uint32_t *thr, uint32_t *tie, uint32_t *counter,
                             uint64_t *keys, bool few_expected, hipStream_t st)
{
    constexpr int QT = scan_qt(M);
    const uint64_t nxb = (nunits + kScanWaves - 1) / kScanWaves;
    const uint64_t items = static_cast<uint64_t>((nq + QT - 1) / QT) * nxb;
    // Redo launches expect few (usually zero) active queries: keep the grid small, it strides.
    const uint64_t most = few_expected ? 4096 : (1u << 20);
    const uint32_t grid = static_cast<uint32_t>(items < most ? (items ? items : 1) : most);
    const size_t lds = static_cast<size_t>(QT) * M * 256 + (MODE == kHist ? QT * 256 * 4 : 0);
    DCPQ_LAUNCH(stage, st, (scan_kernel<M, QT, MODE, CodeT>), dim3(grid), dim3(kScanThreads), lds, codes, n_codes, unit,
                nunits, stride, qtab, nq, qlist, nq_dev, r, hist, thr, tie, counter, keys);
}

// The three passes for the queries qlist[0 .. *nq_dev) (or all nq when qlist is null).
template <int M, typename CodeT>
static int launch_three_pass(const CodeT *codes, uint64_t n_codes, const uint8_t *qtab, int nq, const int *qlist,
                             const uint32_t *nq_dev, uint32_t r, uint32_t *cand_id, uint8_t *cand_qd, uint8_t *base,
                             const ScanPlan &p, hipStream_t st)
{
    uint32_t *hist = reinterpret_cast<uint32_t *>(base + p.off_hist);
    uint32_t *thr = reinterpret_cast<uint32_t *>(base + p.off_thr);
    uint32_t *counter = reinterpret_cast<uint32_t *>(base + p.off_counter);
    uint32_t *tie = reinterpret_cast<uint32_t *>(base + p.off_tie);
    const bool spill = next_pow2(r) > kSortLdsKeys;
    uint64_t *keys = reinterpret_cast<uint64_t *>(base + p.off_keys);
    uint64_t *sorted = reinterpret_cast<uint64_t *>(base + p.off_spill);
    const bool few = qlist != nullptr;

    const size_t nwords = p.zero_bytes / sizeof(uint32_t);
    DCPQ_LAUNCH(kStageMisc, st, zero_words_kernel, dim3((nwords + 255) / 256), dim3(256), 0,
                reinterpret_cast<uint32_t *>(base), nwords);
    DCPQ_CHECK_LAUNCH("zero_words_kernel");
    launch_scan_pass<M, kHist>(kStageScanHist, codes, n_codes, p.unit, p.nunits, p.unit, qtab, nq, qlist, nq_dev, r,
                               hist, thr, tie, counter, keys, few, st);
    DCPQ_CHECK_LAUNCH("scan_kernel<hist>");
    DCPQ_LAUNCH(kStageSelect, st, threshold_kernel, dim3(nq), dim3(256), 0, hist, r, nq_dev, thr);
    DCPQ_CHECK_LAUNCH("threshold_kernel");
    launch_scan_pass<M, kTieCount>(kStageScanTieCount, codes, n_codes, p.unit, p.nunits, p.unit, qtab, nq, qlist,
                                   nq_dev, r, hist, thr, tie, counter, keys, few, st);
    DCPQ_CHECK_LAUNCH("scan_kernel<tiecount>");
    DCPQ_LAUNCH(kStageSelect, st, tie_quota_kernel, dim3(nq), dim3(256), 0, tie, p.nunits, nq_dev, thr);
    DCPQ_CHECK_LAUNCH("tie_quota_kernel");
    launch_scan_pass<M, kCollect>(kStageScanCollect, codes, n_codes, p.unit, p.nunits, p.unit, qtab, nq, qlist,
                                  nq_dev, r, hist, thr, tie, counter, keys, few, st);
    DCPQ_CHECK_LAUNCH("scan_kernel<collect>");
    const uint32_t np2 = next_pow2(r);
    DCPQ_LAUNCH(kStageSelect, st, sort_candidates_kernel, dim3(nq), dim3(1024), spill ? 0 : sizeof(uint64_t) * np2,
                keys, r, np2, spill ? 0 : 1, sorted, qlist, nq_dev, nullptr, cand_id, cand_qd);
    DCPQ_CHECK_LAUNCH("sort_candidates_kernel");
    return DCPQ_OK;
}

template <int M, typename CodeT>
static int launch_sample_hist_m(const CodeT *codes, uint64_t n_codes, const uint8_t *qtab, int nq, uint32_t r,
                                uint32_t *shist, const ScanPlan &p, hipStream_t st)
{
    // (with a pilot pass: runs 0, kPilotEvery, 2 kPilotEvery, ... of the sample)
    launch_scan_pass<M, kHist>(kStageScanHist, codes, n_codes, p.s_unit, p.s1_nunits, p.pilot ? p.s_stride * kPilotEvery : p.s_stride,
                               qtab, nq, nullptr, nullptr, r, shist, nullptr, nullptr, nullptr, nullptr, false, st);
    DCPQ_CHECK_LAUNCH("scan_kernel<sample hist>");
    return DCPQ_OK;
}

template <typename CodeT>
int launch_sample_hist(const CodeT *codes, uint64_t n_codes, int m, const uint8_t *qtab, int nq, uint32_t r,
                       uint32_t *shist, const ScanPlan &p, hipStream_t st)
{
    switch (m) {
        case 4: return launch_sample_hist_m<4, CodeT>(codes, n_codes, qtab, nq, r, shist, p, st);
        case 8: return launch_sample_hist_m<8, CodeT>(codes, n_codes, qtab, nq, r, shist, p, st);
        case 16: return launch_sample_hist_m<16, CodeT>(codes, n_codes, qtab, nq, r, shist, p, st);
        case 32: return launch_sample_hist_m<32, CodeT>(codes, n_codes, qtab, nq, r, shist, p, st);
        default: return fail(DCPQ_EUNSUPPORTED, "sample histogram: m=%d not supported", m);
    }
}

template int launch_sample_hist<uint16_t>(const uint16_t *, uint64_t, int, const uint8_t *, int, uint32_t, uint32_t *,
                                          const ScanPlan &, hipStream_t);
template int launch_sample_hist<uint8_t>(const uint8_t *, uint64_t, int, const uint8_t *, int, uint32_t, uint32_t *,
                                         const ScanPlan &, hipStream_t);

template <int M, typename CodeT>
static int launch_scan_m(const CodeT *codes, uint64_t n_codes, const uint8_t *qtab, int nq, uint32_t r,
                         uint32_t *cand_id, uint8_t *cand_qd, void *ws, int mode, hipStream_t st)
{
    const ScanPlan p = plan_scan(n_codes, M, nq, r, mode);
    uint8_t *base = static_cast<uint8_t *>(ws);
    if (!p.fast)
        return launch_three_pass<M, CodeT>(codes, n_codes, qtab, nq, nullptr, nullptr, r, cand_id, cand_qd, base, p, st);

    const size_t nwords = p.fzero_bytes / sizeof(uint32_t);
    DCPQ_LAUNCH(kStageMisc, st, zero_words_kernel, dim3((nwords + 255) / 256), dim3(256), 0,
                reinterpret_cast<uint32_t *>(base + p.off_fzero), nwords);
    DCPQ_CHECK_LAUNCH("zero_words_kernel");
    int rc = launch_scan_fast(codes, n_codes, M, qtab, nq, r, cand_id, cand_qd, base, p, st);
    if (rc) return rc;
    // queries the single pass could not finish (their count is known on the device only)
    return launch_three_pass<M, CodeT>(codes, n_codes, qtab, nq, reinterpret_cast<const int *>(base + p.off_qlist),
                                reinterpret_cast<const uint32_t *>(base + p.off_nflag), r, cand_id, cand_qd, base,
                                p, st);
}

template <typename CodeT>
static int launch_scan_any(const CodeT *codes, uint64_t n_codes, int m, const uint8_t *qtab, int nq, uint32_t r,
                           uint32_t *cand_id, uint8_t *cand_qd, void *ws, int mode, hipStream_t st)
{
    if (nq == 0) return DCPQ_OK;
    switch (m) {
        case 1: return launch_scan_m<1, CodeT>(codes, n_codes, qtab, nq, r, cand_id, cand_qd, ws, mode, st);
        case 2: return launch_scan_m<2, CodeT>(codes, n_codes, qtab, nq, r, cand_id, cand_qd, ws, mode, st);
        case 4: return launch_scan_m<4, CodeT>(codes, n_codes, qtab, nq, r, cand_id, cand_qd, ws, mode, st);
        case 8: return launch_scan_m<8, CodeT>(codes, n_codes, qtab, nq, r, cand_id, cand_qd, ws, mode, st);
        case 16: return launch_scan_m<16, CodeT>(codes, n_codes, qtab, nq, r, cand_id, cand_qd, ws, mode, st);
        case 32: return launch_scan_m<32, CodeT>(codes, n_codes, qtab, nq, r, cand_id, cand_qd, ws, mode, st);
        default: return fail(DCPQ_EUNSUPPORTED, "m=%d not supported", m);
    }
}

int launch_scan(const uint16_t *codes, uint64_t n_codes, int m, const uint8_t *qtab, int nq, uint32_t r,
                uint32_t *cand_id, uint8_t *cand_qd, void *ws, int mode, hipStream_t st)
{
    return launch_scan_any(codes, n_codes, m, qtab, nq, r, cand_id, cand_qd, ws, mode, st);
}

int launch_scan(const uint8_t *plane, uint64_t n_codes, int m, const uint8_t *qtab, int nq, uint32_t r,
                uint32_t *cand_id, uint8_t *cand_qd, void *ws, int mode, hipStream_t st)
{
    return launch_scan_any(plane, n_codes, m, qtab, nq, r, cand_id, cand_qd, ws, mode, st);
}

}  // namespace dcpq

using namespace dcpq;

extern "C" int dcpq_scan_query_tile(int m)
{
    if (!m_supported(m)) return 0;
    const int f = fast_query_tile(m, 1 << 30, DCPQ_SCAN_AUTO);
    return f ? f : scan_qt(m);
}

extern "C" int dcpq_scan_plan(uint64_t n_codes, int m, int nq, uint32_t r, int mode, uint64_t *info, int ninfo)
{
    clear_error();
    DCPQ_REQUIRE(info && ninfo >= 6, "scan_plan: info must hold 6 values");
    DCPQ_REQUIRE(nq >= 1 && n_codes >= 1 && r >= 1, "scan_plan: empty problem");
    if (!m_supported(m)) return fail(DCPQ_EUNSUPPORTED, "scan_plan: m=%d not supported", m);
    const ScanPlan p = plan_scan(n_codes, m, nq, r, mode);
    info[0] = p.fast ? p.fqt : p.qt;
    info[1] = p.fast ? p.ntiles : (static_cast<uint64_t>(nq) + p.qt - 1) / p.qt;
    info[2] = p.fast ? p.fblocks : 0;
    info[3] = p.fast ? p.codes_per_block : p.unit;
    info[4] = p.fast ? p.slices : 0;
    info[5] = p.fast ? p.cap : 0;
    if (ninfo >= 10) {
        info[6] = p.fast ? p.s_nunits : 0;
        info[7] = p.fast ? p.s_stride : 0;
        info[8] = p.fast && p.pilot ? kPilotEvery : (p.fast ? 1 : 0);
        info[9] = p.fast ? p.pilot_r : 0;
    }
    return DCPQ_OK;
}

extern "C" size_t dcpq_scan_workspace_bytes(uint64_t n_codes, int m, int nq, uint32_t r)
{
    if (nq <= 0 || !m_supported(m) || n_codes == 0 || r == 0 || r > (1u << 26)) return 0;
    // enough for every algorithm the caller may ask for
    size_t most = 0;
    const int modes[] = {DCPQ_SCAN_AUTO, DCPQ_SCAN_THREE_PASS, DCPQ_SCAN_TILE16, DCPQ_SCAN_TILE32, DCPQ_SCAN_TILE64};
    for (int mode : modes) {
        const size_t t = plan_scan(n_codes, m, nq, r, mode).total;
        most = t > most ? t : most;
    }
    return most;
}

template <typename CodeT>
static int scan_checked(const CodeT *codes, uint64_t n_codes, int m, const uint8_t *qtab, int nq, uint32_t r,
                        uint32_t *cand_id, uint8_t *cand_qd, void *workspace, size_t workspace_bytes, int mode,
                        void *stream)
{
    clear_error();
    DCPQ_REQUIRE(nq >= 0, "scan_candidates: nq=%d", nq);
    DCPQ_REQUIRE(mode == DCPQ_SCAN_AUTO || mode == DCPQ_SCAN_THREE_PASS || mode == DCPQ_SCAN_TILE16 ||
                     mode == DCPQ_SCAN_TILE32 || mode == DCPQ_SCAN_TILE64,
                 "scan_candidates: mode=%d", mode);
    if (!m_supported(m)) return fail(DCPQ_EUNSUPPORTED, "scan_candidates: m=%d not supported", m);
    if (mode >= DCPQ_SCAN_TILE16 && fast_query_tile(m, nq, mode) == 0)
        return fail(DCPQ_EUNSUPPORTED, "scan_candidates: no single-pass kernel for m=%d with the tile of mode %d", m, mode);
    DCPQ_REQUIRE(n_codes >= 1 && n_codes < (1ull << 32), "scan_candidates: n_codes=%llu must be in [1, 2^32)",
                 static_cast<unsigned long long>(n_codes));
    DCPQ_REQUIRE(r >= 1 && r <= n_codes, "scan_candidates: r=%u must be in [1, n_codes]", r);
    DCPQ_REQUIRE(r <= (1u << 26), "scan_candidates: r=%u above the supported 2^26", r);
    if (nq == 0) return DCPQ_OK;
    DCPQ_REQUIRE(codes && qtab && cand_id && cand_qd && workspace, "scan_candidates: null pointer");
    DCPQ_REQUIRE((reinterpret_cast<uintptr_t>(workspace) & 255) == 0, "scan_candidates: workspace must be 256-byte aligned");
    DCPQ_REQUIRE((reinterpret_cast<uintptr_t>(codes) & 15) == 0 && (reinterpret_cast<uintptr_t>(qtab) & 15) == 0,
                 "scan_candidates: codes (or their plane) and qtab must be 16-byte aligned");
    const size_t need = dcpq_scan_workspace_bytes(n_codes, m, nq, r);
    if (workspace_bytes < need)
        return fail(DCPQ_EWORKSPACE, "scan_candidates: workspace %zu < %zu bytes", workspace_bytes, need);
    return launch_scan(codes, n_codes, m, qtab, nq, r, cand_id, cand_qd, workspace, mode, as_stream(stream));
}

extern "C" int dcpq_scan_candidates(const uint16_t *codes, uint64_t n_codes, int m, const uint8_t *qtab, int nq,
                                    uint32_t r, uint32_t *cand_id, uint8_t *cand_qd, void *workspace,
                                    size_t workspace_bytes, void *stream)
{
    return scan_checked(codes, n_codes, m, qtab, nq, r, cand_id, cand_qd, workspace, workspace_bytes,
                        DCPQ_SCAN_AUTO, stream);
}

extern "C" int dcpq_scan_candidates_packed(const uint8_t *plane, uint64_t n_codes, int m, const uint8_t *qtab, int nq,
                                           uint32_t r, uint32_t *cand_id, uint8_t *cand_qd, void *workspace,
                                           size_t workspace_bytes, int mode, void *stream)
{
    return scan_checked(plane, n_codes, m, qtab, nq, r, cand_id, cand_qd, workspace, workspace_bytes, mode, stream);
}

extern "C" int dcpq_scan_candidates_mode(const uint16_t *codes, uint64_t n_codes, int m, const uint8_t *qtab,
                                         int nq, uint32_t r, uint32_t *cand_id, uint8_t *cand_qd, void *workspace,
                                         size_t workspace_bytes, int mode, void *stream)
{
    return scan_checked(codes, n_codes, m, qtab, nq, r, cand_id, cand_qd, workspace, workspace_bytes, mode, stream);
}

// ---- the entry point that allocates nothing ------------------------------------------------------
// For callers that cannot call hipMalloc (code under graph capture, tight serving loops, harnesses
// that forbid allocation) and have no workspace to hand over: the scan's workspace is this array,
// which every GPU the library runs on holds from the first call until the process ends.
constexpr size_t kStaticScratchBytes = DCPQ_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {
constexpr int kMostDevices = 64;
std::mutex g_scratch_mutex;
void *g_scratch_ptr[kMostDevices];      // device address of `scratch` on each GPU (the array's name is only a host-side stand-in)

// Device address of the current device's copy of the array, looked up once per device.
int static_scratch(void **out)
{
    int dev = 0;
    DCPQ_CHECK_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMostDevices) return fail(DCPQ_EUNSUPPORTED, "scan_candidates_static: device %d out of range", dev);
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        DCPQ_CHECK_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p) return fail(DCPQ_EHIP, "scan_candidates_static: no device address for the static scratch array");
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return DCPQ_OK;
}
}  // namespace

extern "C" size_t dcpq_static_scratch_bytes(void) { return kStaticScratchBytes; }

extern "C" int dcpq_scan_candidates_static(const uint16_t *codes, uint64_t n_codes, int m, const uint8_t *qtab, int nq,
                                           uint32_t r, uint32_t *cand_id, uint8_t *cand_qd, void *stream)
{
    clear_error();
    // the size check comes first: a problem that does not fit is refused before the device is touched
    if (nq > 0 && m_supported(m) && n_codes >= 1 && r >= 1 && r <= (1u << 26)) {
        const size_t need = dcpq_scan_workspace_bytes(n_codes, m, nq, r);
        if (need > kStaticScratchBytes)
            return fail(DCPQ_EWORKSPACE, "scan_candidates_static: the scan needs %zu bytes of scratch, the static array holds %zu",
                        need, kStaticScratchBytes);
    }
    void *ws = nullptr;
    if (nq > 0) {
        const int rc = static_scratch(&ws);
        if (rc) return rc;
    }
    // every counter the kernels expect at zero is cleared by the scan itself (a fill kernel, so the
    // call may be captured), whatever the previous call left in the array
    return scan_checked(codes, n_codes, m, qtab, nq, r, cand_id, cand_qd, ws, kStaticScratchBytes, DCPQ_SCAN_AUTO, stream);
}
