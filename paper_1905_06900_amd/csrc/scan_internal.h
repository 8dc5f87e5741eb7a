// Shared between the two translation units of the scan stage (not part of the ABI).
#pragma once

#include "common.h"

namespace dcpq {

constexpr uint32_t kSortLdsKeys = 8192;   // keys a workgroup sorts in LDS (64 KiB)

inline uint32_t next_pow2(uint32_t x)
{
    uint32_t p = 1;
    while (p < x) p <<= 1;
    return p;
}

// Sizes and workspace layout of one scan_candidates call (offsets in bytes from a 256-byte
// aligned base).  The three-pass path can always run; the single-pass path exists for m >= 4.
// Each query's candidate buffer and append cursor are split into slices, one per residue of the
// workgroup's position along the codes: workgroups that run at the same time append to different
// cursors, which keeps same-address atomics (they serialize in the L2) off the critical path.
constexpr int kFastSlices = 16;      // at most; fewer when there are fewer workgroups along the codes

constexpr uint32_t kPilotEvery = 16;

struct ScanPlan {
    // three-pass path
    uint32_t unit;        // codes scanned by one wavefront
    uint32_t nunits;      // ceil(n_codes / unit)
    uint32_t qt;          // queries per workgroup tile
    size_t off_hist;      // uint32 [nq][256]
    size_t off_thr;       // uint32 [nq][2]   (threshold bucket, ids still needed from it)
    size_t off_counter;   // uint32 [nq]
    size_t zero_bytes;    // the three arrays above are contiguous from offset 0 and cleared together
    size_t off_tie;       // uint32 [nq][nunits]
    size_t off_keys;      // uint64 [nq][r]
    size_t off_spill;     // uint64 [nq][next_pow2(r)], only when r keys do not fit the LDS sort
    // single-pass path
    bool fast;
    uint32_t fqt;             // queries per tile
    uint32_t ntiles;
    uint32_t fblocks;         // workgroups along the code axis
    uint32_t codes_per_block;
    uint32_t slices;          // slices per query: min(kFastSlices, fblocks)
    uint32_t cap;             // candidate-buffer entries per query and slice
    uint32_t upd;             // appended candidates between two bound updates
    uint32_t qflush;          // a wavefront appends its pending candidates once it holds this many
    uint32_t sortcap;         // keys the final selection can sort (power of two)
    uint32_t s_unit, s_nunits;    // sample: s_nunits runs of s_unit codes ...
    uint64_t s_stride;            // ... starting every s_stride codes
    // pilot pass (large arrays): the histogram pass reads only every kPilotEvery-th run of the sample, and the
    // sample itself goes through the single-pass kernel, counting only
    bool pilot;
    uint32_t s1_nunits;           // runs the histogram pass reads
    uint64_t s_count;             // codes in the sample
    uint32_t pilot_r;             // rank wanted within the sample: what r codes of the array leave in it, plus slack
    uint32_t pilot_blocks;        // workgroups per tile of the pilot pass ...
    uint32_t pilot_runs;          // ... and sample runs per workgroup
    size_t off_fzero, fzero_bytes;   // fcount, chist, shist, nflag: cleared together
    size_t off_fcount;    // uint32 [nq][slices]
    size_t off_chist;     // uint32 [nq][256]
    size_t off_shist;     // uint32 [nq][256]
    size_t off_nflag;     // uint32 [1] (+ padding)
    size_t off_tcur;      // int32 [nq]
    size_t off_flags;     // uint32 [nq]
    size_t off_qlist;     // int32 [nq]
    size_t off_qsw;       // uint8 [ntiles][fast_table_bytes(m, fqt)]
    size_t off_fkeys;     // uint64 [nq][slices][cap]
    size_t off_fsort;     // uint64 [nq][sortcap], only when sortcap exceeds the LDS sort
    size_t total;
};
// mode: DCPQ_SCAN_AUTO picks the single-pass query tile from the batch size; DCPQ_SCAN_TILE16/32/64 force it
ScanPlan plan_scan(uint64_t n_codes, int m, int nq, uint32_t r, int mode = 0);

int fast_query_tile(int m, int nq, int mode);   // 0 when the single-pass path does not exist for this m (and tile)
size_t fast_table_bytes(int m, int qt);
// CodeT: uint16_t (the codes as stored) or uint8_t (their low-byte plane); both are instantiated.
template <typename CodeT>
int launch_sample_hist(const CodeT *codes, uint64_t n_codes, int m, const uint8_t *qtab, int nq,
                       uint32_t r, uint32_t *shist, const ScanPlan &p, hipStream_t st);
template <typename CodeT>
int launch_scan_fast(const CodeT *codes, uint64_t n_codes, int m, const uint8_t *qtab, int nq,
                     uint32_t r, uint32_t *cand_id, uint8_t *cand_qd, uint8_t *base, const ScanPlan &p,
                     hipStream_t st);

// Steps of the single-pass selection that the inverted-list variant reuses.
// n_codes: size of the array the sample was drawn from (the sample's own size is the histogram's total)
// n_each (optional): the number of codes each query scans, where it is not the same n_codes for all of them
int launch_sample_threshold(const uint32_t *shist, int nq, uint32_t r, uint64_t n_codes, int *t_cur, hipStream_t st,
                            const uint32_t *n_each = nullptr);
// n_ids: the ids are below this (0 = unknown)
int launch_fast_select(const uint64_t *keys, const uint32_t *count, const uint32_t *chist, int nq, uint32_t r,
                       uint32_t nslices, uint32_t cap, uint32_t sortcap, uint64_t n_ids, uint64_t *spill, uint32_t *cand_id,
                       uint8_t *cand_qd, uint32_t *flags, hipStream_t st);

// Small shared steps of the three-pass selection, reused by the inverted-list variant.
int launch_zero_words(uint32_t *p, size_t nwords, hipStream_t st);
int launch_fill_u64(uint64_t *p, size_t n, uint64_t v, hipStream_t st);
int launch_threshold(const uint32_t *hist, int nq, uint32_t r, uint32_t *thr, hipStream_t st);
int launch_tie_quota(uint32_t *tie, uint32_t nunits, int nq, const uint32_t *thr, hipStream_t st);
// flags (may be null): only queries with a non-zero flag are sorted and written
int launch_sort_candidates(const uint64_t *keys, int nq, uint32_t r, uint64_t *spill, uint32_t *cand_id,
                           uint8_t *cand_qd, hipStream_t st, const uint32_t *flags = nullptr);

#ifdef __HIPCC__
}  // namespace dcpq
#include "device_util.h"
namespace dcpq {
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

// Lowers query q's bucket bound to the bucket that holds its r-th best appended candidate (nothing
// happens while fewer than r are appended).  Called by
// a whole wavefront: lane l reads the counts of buckets 4l .. 4l+3, a wavefront prefix sum locates the
// bucket.  The counts only grow, so any snapshot of them gives a bound that is still valid later.
static __device__ __noinline__ void lower_bound_of(int q, uint32_t r, int *t_cur, const uint32_t *chist)
{
    const int lane = threadIdx.x & 63;
    uint32_t c[4];
#pragma unroll
    for (int z = 0; z < 4; ++z)
        c[z] = __hip_atomic_load(&chist[static_cast<size_t>(q) * 256 + 4 * lane + z], __ATOMIC_RELAXED,
                                 __HIP_MEMORY_SCOPE_AGENT);
    const uint32_t mine = c[0] + c[1] + c[2] + c[3];
    uint32_t incl = mine;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const uint32_t other = __shfl(incl, lane >= d ? lane - d : lane);
        if (lane >= d) incl += other;
    }
    uint32_t cum = incl - mine;                          // appended candidates in buckets below 4 * lane
    if (cum < r && incl >= r) {                          // at most one lane
        int tn = 4 * lane;
#pragma unroll
        for (int z = 0; z < 3; ++z) {
            cum += c[z];
            if (cum < r) tn = 4 * lane + z + 1;
        }
        atomicMin(&t_cur[q], tn);
    }
}

// The same from the low-byte plane of the codes (uint8 [n][m], the bytes pass one consumes).
template <int M>
__device__ inline void load_low_bytes(const uint8_t *__restrict__ plane, uint64_t i, uint32_t (&low)[M])
{
    if constexpr (M % 8 == 0) {
        const uint2 *p = reinterpret_cast<const uint2 *>(plane + i * M);
#pragma unroll
        for (int v = 0; v < M / 8; ++v) {
            const uint2 x = p[v];
#pragma unroll
            for (int z = 0; z < 4; ++z) {
                low[8 * v + z] = (x.x >> (8 * z)) & 255u;
                low[8 * v + 4 + z] = (x.y >> (8 * z)) & 255u;
            }
        }
    } else if constexpr (M == 4) {
        const uint32_t x = *reinterpret_cast<const uint32_t *>(plane + i * 4);
#pragma unroll
        for (int z = 0; z < 4; ++z) low[z] = (x >> (8 * z)) & 255u;
    } else if constexpr (M == 2) {
        const uint32_t x = *reinterpret_cast<const uint16_t *>(plane + i * 2);
        low[0] = x & 255u; low[1] = (x >> 8) & 255u;
    } else {
        low[0] = plane[i];
    }
}
#endif

}  // namespace dcpq
