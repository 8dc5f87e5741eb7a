// Pass one of Alg. 3 (Sec. 3.3, "Scan step") -- the single-pass kernel.
//
// What is computed is the same as in scan.hip: qd = min(255, sum_j Q_j[low8(c[j])]) for every
// (query, code) and the r smallest by (qd, id).  How it is computed differs from the paper's CPU
// loop in three ways that matter on this chip:
//
// 1. Row lookups instead of byte lookups.  A tile of QT queries keeps its tables in LDS
//    transposed, T[j][e][q] with the query fastest, so that the table entries of one (code, j)
//    for 16 queries are 16 contiguous bytes.  One ds_read_b128 per lane then delivers 1024
//    lookups per wavefront instruction, against 64 for byte gathers.  Rows of the same
//    sub-quantizer group are interleaved over a 256-byte LDS line (row slot = j mod NSLOT) and
//    every lane group of a wavefront reads a different slot, which keeps the reads free of bank
//    conflicts whatever the code bytes are.
//
// 2. The sum over j runs on the matrix cores as an exact integer accumulation: with A = the
//    gathered rows (16 x 64 bytes: 16 (code, query-block) rows, 4 sub-quantizers x 16 queries) and
//    B = four stacked 16 x 16 identities, v_mfma_i32_16x16x64_i8 returns
//    D[row][n] = sum over the 4 sub-quantizers of T[j][e][16 * qb + n], and chaining M/4 of them
//    through the accumulator gives the unsaturated integer distance.  The instruction multiplies
//    SIGNED bytes, so the LDS copy of the tables holds x - 128 (the byte with its top bit flipped)
//    and the accumulator starts at 128 * M instead of 0, which restores the unsigned sum exactly.  This is not a reshaping of
//    the scan into a dense product (no one-hot expansion: every byte multiplied is a byte the
//    method looks up); the matrix unit only replaces the byte unpack-and-add that the vector ALU
//    would otherwise spend three instructions per four lookups on.
//
// 3. Capped buckets become a running threshold.  Each query has a bucket bound T_cur that is
//    never below the bucket of its r-th best candidate: it starts as the exact r-th smallest qd
//    of a strided sample of the codes and is lowered whenever the exact per-bucket counts of the
//    candidates appended so far reach r below a smaller bucket (the paper's "distance of the
//    r2-th farthest vector as upper bound").  A pair with qd <= T_cur is appended to the query's
//    candidate buffer.  Whatever the timing of the updates, the buffer ends up a superset of the
//    true candidate set, from which the exact, id-tie-broken r are then selected; the result does
//    not depend on the order of arrival.  If a buffer overflows (pathological ties), the query is
//    flagged and redone by the three-pass path of scan.hip.
#include "common.h"
#include "scan_internal.h"

namespace dcpq {

typedef int v4i __attribute__((ext_vector_type(4)));

template <int M, int QT, int WAVES>
struct FastCfg {
    static constexpr int NQB = QT / 16;             // 16-query blocks per table row
    static constexpr int CPS = 16 / NQB;            // codes per MFMA step
    static constexpr int NSLOT = 256 / QT;          // table rows per 256-byte LDS line
    static constexpr int NMF = M / 4;               // chained MFMAs per step
    static constexpr int STEPS = 64 / CPS;          // steps per 64-code group
    static constexpr int UNROLL = NMF >= 8 ? 1 : 8 / NMF;   // steps issued together (8 row reads in flight)
    static constexpr int PREFETCH = M <= 8 ? 4 : M == 16 ? 2 : 1;   // 64-code groups fetched ahead per wavefront
    static constexpr int CLS = M / 4;               // bytes per residue class j mod 4 in the code scratch
    static constexpr int TAB_BYTES = M * 256 * QT;
    static constexpr int SCR_BYTES = WAVES * 64 * M;
    static constexpr int QCAP = 64;                 // pending-candidate queue entries per wavefront (>= 64)
    static constexpr int Q_BYTES = WAVES * QCAP * 8;
    static constexpr int LDS_BYTES = TAB_BYTES + SCR_BYTES + Q_BYTES;
    static_assert(NSLOT <= M && M % 4 == 0, "row slots must rotate within the sub-quantizers");
    static_assert(STEPS % UNROLL == 0, "unroll must divide the steps of a group");
};

// Sub-quantizer read by MFMA u, chunk s (= lane / 16), for code slot c: rotate within aligned
// groups of NSLOT sub-quantizers so that the 16 lanes of one chunk hit NSLOT different row slots.
template <int NSLOT>
__device__ inline int rotated_j(int u, int s, int c)
{
    const int g = 4 * u + s;
    return (g & ~(NSLOT - 1)) | ((g + c) & (NSLOT - 1));
}

// Byte offset of T[j][e][q] in the swizzled tile layout (shared by the transposition kernel and
// the scan kernel).
template <int QT>
__host__ __device__ inline uint32_t swz_offset(int j, int e, int q)
{
    constexpr int NSLOT = 256 / QT;
    return (static_cast<uint32_t>(j / NSLOT) * 256u + e) * 256u + (j % NSLOT) * QT + q;
}

// qtab [nq][M][256] -> per-tile swizzled tables [ntiles][M*256*QT], each byte stored as x - 128
// (x ^ 0x80) for the signed matrix instruction; absent queries read 255.
template <int M, int QT>
__global__ __launch_bounds__(256) void swizzle_tables_kernel(const uint8_t *__restrict__ qtab, int nq,
                                                             uint8_t *__restrict__ out)
{
    const int tile = blockIdx.y;
    const int idx = blockIdx.x * 256 + threadIdx.x;      // (j, e, qb)
    constexpr int NQB = QT / 16;
    if (idx >= M * 256 * NQB) return;
    const int qb = idx % NQB, e = (idx / NQB) % 256, j = idx / (NQB * 256);
    uint32_t w[4] = {0, 0, 0, 0};
#pragma unroll
    for (int t = 0; t < 16; ++t) {
        const int q = tile * QT + qb * 16 + t;
        const uint32_t v = q < nq ? qtab[(static_cast<size_t>(q) * M + j) * 256 + e] : 255u;
        w[t >> 2] |= (v ^ 0x80u) << (8 * (t & 3));
    }
    uint8_t *dst = out + static_cast<size_t>(tile) * (M * 256 * QT) + swz_offset<QT>(j, e, qb * 16);
    *reinterpret_cast<uint4 *>(dst) = make_uint4(w[0], w[1], w[2], w[3]);
}

// T_cur[q] = bucket of the r-th smallest qd of the sample (255 if the sample holds fewer than r).
__global__ __launch_bounds__(256) void sample_threshold_kernel(const uint32_t *__restrict__ shist, uint32_t r,
                                                               int *__restrict__ t_cur)
{
    __shared__ uint32_t cum[256];
    const int q = blockIdx.x, b = threadIdx.x;
    cum[b] = shist[static_cast<size_t>(q) * 256 + b];
    __syncthreads();
    for (int off = 1; off < 256; off <<= 1) {
        const uint32_t add = b >= off ? cum[b - off] : 0u;
        __syncthreads();
        cum[b] += add;
        __syncthreads();
    }
    const uint32_t before = b ? cum[b - 1] : 0u;
    if (before < r && cum[b] >= r) t_cur[q] = b;
    if (b == 255 && cum[255] < r) t_cur[q] = 255;
}

// Low bytes of the M sub-codes of one code, reordered by residue class: byte (j & 3) * CLS + (j >> 2).
template <int M>
__device__ inline void transposed_low_bytes(const uint32_t (&w)[M / 2], uint32_t (&out)[M / 4])
{
    // w[i] holds sub-codes 2i (bits 0..15) and 2i+1 (bits 16..31); low byte of j is byte 2*(j&1) of w[j/2]
#pragma unroll
    for (int d = 0; d < M / 4; ++d) out[d] = 0;
#pragma unroll
    for (int j = 0; j < M; ++j) {
        const uint32_t b = (w[j >> 1] >> (16 * (j & 1))) & 255u;
        const int p = (j & 3) * (M / 4) + (j >> 2);
        out[p >> 2] |= b << (8 * (p & 3));
    }
}

// Appends one candidate (rec: id in bits 0..31, qd in 32..39, query-in-tile in 40..47) to its
// query's buffer, counts it in the query's exact per-bucket histogram, and every `upd` appends
// lowers the query's bucket bound to the bucket that now holds its r-th best appended candidate.
// Kept out of line: it is the rare path and would otherwise be replicated at every call site.
__device__ __noinline__ void append_candidate(uint64_t rec, int q0, uint32_t r, uint32_t cap, uint32_t upd,
                                              int *t_cur, uint32_t *count, uint32_t *chist, uint64_t *keys)
{
    const uint32_t q = q0 + static_cast<uint32_t>(rec >> 40);
    const uint32_t qd = static_cast<uint32_t>(rec >> 32) & 255u;
    const uint32_t pos = atomicAdd(&count[q], 1u);
    if (pos < cap) keys[static_cast<size_t>(q) * cap + pos] = rec & 0xFFFFFFFFFFull;
    else atomicMin(&t_cur[q], -1);                     // buffer full: stop appending, query is redone
    atomicAdd(&chist[static_cast<size_t>(q) * 256 + qd], 1u);
    if (pos + 1 >= r && (pos + 1) % upd == 0) {
        uint32_t cum = 0;
        int tn = -1;
#pragma unroll 1
        for (int b = 0; b < 256; b += 4) {
            uint32_t c[4];
#pragma unroll
            for (int z = 0; z < 4; ++z)
                c[z] = __hip_atomic_load(&chist[static_cast<size_t>(q) * 256 + b + z], __ATOMIC_RELAXED,
                                         __HIP_MEMORY_SCOPE_AGENT);
#pragma unroll
            for (int z = 0; z < 4; ++z) {
                cum += c[z];
                if (tn < 0 && cum >= r) tn = b + z;
            }
            if (tn >= 0) break;
        }
        if (tn >= 0) atomicMin(&t_cur[q], tn);
    }
}

template <int M, int QT, int WAVES>
__global__ __launch_bounds__(WAVES * 64) void scan_fast_kernel(
    const uint16_t *__restrict__ codes, uint64_t n_codes, uint32_t codes_per_block,
    const uint8_t *__restrict__ qsw, int nq, uint32_t r, uint32_t cap, uint32_t upd,
    int *t_cur, uint32_t *count, uint32_t *chist, uint64_t *__restrict__ keys)
{
    using C = FastCfg<M, QT, WAVES>;
    extern __shared__ __align__(16) uint8_t smem[];
    uint8_t *ltab = smem;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    uint8_t *scr = smem + C::TAB_BYTES + wave * (64 * M);
    uint64_t *wq = reinterpret_cast<uint64_t *>(smem + C::TAB_BYTES + C::SCR_BYTES) + wave * C::QCAP;

    const int tile = blockIdx.x;
    const int q0 = tile * QT;
    {
        const uint4 *src = reinterpret_cast<const uint4 *>(qsw + static_cast<size_t>(tile) * C::TAB_BYTES);
        uint4 *dst = reinterpret_cast<uint4 *>(ltab);
        for (int v = tid; v < C::TAB_BYTES / 16; v += WAVES * 64) dst[v] = src[v];
    }
    __syncthreads();

    // ---- per-lane constants -------------------------------------------------------------
    const int s = lane >> 4, i = lane & 15;
    const int ca = i / C::NQB, qba = i % C::NQB;          // A operand: code slot, query block
    uint32_t laneoff[C::NMF];
    int shift[C::NMF];
#pragma unroll
    for (int u = 0; u < C::NMF; ++u) {
        const int j = rotated_j<C::NSLOT>(u, s, ca);
        laneoff[u] = swz_offset<QT>(j, 0, qba * 16);
        shift[u] = 8 * (j >> 2);
    }
    const int cls = (s + ca) & 3;                          // residue class j mod 4 read by this lane
    const uint32_t scr_rd = ca * M + cls * C::CLS;         // + step * CPS * M
    v4i bsel = {0, 0, 0, 0};                               // B: four stacked identities
    bsel[i >> 2] = 1 << (8 * (i & 3));
    // D operand: value v of this lane is row 4 * (lane / 16) + v, column lane % 16
    int cd[4], ql[4];
#pragma unroll
    for (int v = 0; v < 4; ++v) {
        const int row = 4 * s + v;
        cd[v] = row / C::NQB;
        ql[v] = (row % C::NQB) * 16 + i;
    }

    const uint64_t cbeg = static_cast<uint64_t>(blockIdx.y) * codes_per_block;
    const uint64_t cend = min(n_codes, cbeg + codes_per_block);
    const uint32_t ngroups = cbeg < cend ? static_cast<uint32_t>((cend - cbeg + 63) / 64) : 0u;

    auto insert = [&](uint64_t rec) { append_candidate(rec, q0, r, cap, upd, t_cur, count, chist, keys); };

    // Pending candidates of this wavefront: records wq[0 .. qlen).  qlen is wave-uniform (it only
    // changes by ballot counts), so it lives in a scalar register and the queue needs no atomics.
    uint32_t qlen = 0;
    auto flush = [&]() {
        // the wavefront runs in lockstep; the barriers say that every push is in place before the
        // entries are read, and that every lane has read its entry before the next push overwrites it
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        for (uint32_t e = lane; e < qlen; e += 64) insert(wq[e]);
        qlen = 0;
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    };

    // ---- main loop: one 64-code group per iteration ---------------------------------------
    auto load_group = [&](uint32_t g, uint32_t (&dst)[M / 2]) {
        const uint64_t id = cbeg + static_cast<uint64_t>(g) * 64 + lane;
        if (g < ngroups && id < cend) {
            if constexpr (M % 8 == 0) {
                const uint4 *p = reinterpret_cast<const uint4 *>(codes + id * M);
#pragma unroll
                for (int v = 0; v < M / 8; ++v) {
                    const uint4 x = p[v];
                    dst[4 * v] = x.x; dst[4 * v + 1] = x.y; dst[4 * v + 2] = x.z; dst[4 * v + 3] = x.w;
                }
            } else {
                const uint2 x = *reinterpret_cast<const uint2 *>(codes + id * M);
                dst[0] = x.x; dst[1] = x.y;
            }
        } else {
#pragma unroll
            for (int v = 0; v < M / 2; ++v) dst[v] = 0;
        }
    };
    // Groups are fetched PF at a time and one batch ahead of their use, so that each wavefront
    // keeps PF kilobytes of the code stream in flight (HBM latency x bandwidth needs that much).
    constexpr int PF = C::PREFETCH;
    uint32_t wb[PF][M / 2];
    auto load_batch = [&](uint32_t g0) {
#pragma unroll
        for (int pf = 0; pf < PF; ++pf) load_group(g0 + pf * WAVES, wb[pf]);
    };
    load_batch(wave);
    // bucket bounds of this lane's four (code, query) outputs, re-read once per batch and one
    // batch ahead of their use; absent queries never match
    auto load_bounds = [&](int (&dst)[4]) {
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int q = q0 + ql[v];
            const int t = q < nq ? __hip_atomic_load(&t_cur[q], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : -1;
            dst[v] = t >= 255 ? 0x7fffffff : t;
        }
    };
    int tl_next[4];
    load_bounds(tl_next);

    for (uint32_t g0 = wave; g0 < ngroups; g0 += PF * WAVES) {
        uint32_t tbp[PF][M / 4];
#pragma unroll
        for (int pf = 0; pf < PF; ++pf) transposed_low_bytes<M>(wb[pf], tbp[pf]);
        load_batch(g0 + PF * WAVES);                                 // prefetch the next batch
        int tl[4];
#pragma unroll
        for (int v = 0; v < 4; ++v) tl[v] = tl_next[v];
        load_bounds(tl_next);
        v4i acc0;
#pragma unroll
        for (int v = 0; v < 4; ++v)
            acc0[v] = static_cast<int>(128u * M - static_cast<uint32_t>(tl[v]) - 1u);
#pragma unroll 1
      for (int pf = 0; pf < PF; ++pf) {
        const uint32_t g = g0 + pf * WAVES;
        if (g >= ngroups) break;                                     // uniform
        const uint64_t gbase = cbeg + static_cast<uint64_t>(g) * 64;
        const int nlive = static_cast<int>(min(static_cast<uint64_t>(64), cend - gbase));   // codes in this group
        // publish the low bytes of the group's codes to the wavefront's scratch
        {
            uint32_t tb[M / 4];
#pragma unroll
            for (int d = 0; d < M / 4; ++d) {
                tb[d] = tbp[0][d];
#pragma unroll
                for (int z = 1; z < PF; ++z) tb[d] = pf == z ? tbp[z][d] : tb[d];
            }
            uint32_t *dst = reinterpret_cast<uint32_t *>(scr + lane * M);
#pragma unroll
            for (int d = 0; d < M / 4; ++d) dst[d] = tb[d];
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

        // this lane's M/4 code bytes of a step (class cls of code slot ca), read one step ahead
        auto read_word = [&](int t) -> uint64_t {
            const uint8_t *sp = scr + scr_rd + t * (C::CPS * M);
            if constexpr (C::CLS == 1) return *sp;
            else if constexpr (C::CLS == 2) return *reinterpret_cast<const uint16_t *>(sp);
            else if constexpr (C::CLS == 4) return *reinterpret_cast<const uint32_t *>(sp);
            else return *reinterpret_cast<const uint64_t *>(sp);
        };
        // U steps are issued together: all their row reads first, then U independent MFMA chains,
        // so that several kilobytes of LDS reads per wavefront are in flight at any time.
        constexpr int U = C::UNROLL;
#pragma unroll 1
        for (int t0 = 0; t0 < C::STEPS; t0 += U) {
            uint64_t word[U];
#pragma unroll
            for (int u = 0; u < U; ++u) word[u] = read_word(t0 + u);
            v4i a[U][C::NMF];
#pragma unroll
            for (int u = 0; u < U; ++u)
#pragma unroll
                for (int f = 0; f < C::NMF; ++f) {
                    const uint32_t e = static_cast<uint32_t>(word[u] >> shift[f]) & 255u;
                    a[u][f] = *reinterpret_cast<const v4i *>(ltab + laneoff[f] + e * 256u);
                }
            // Each accumulator starts at 128 * M - (T + 1): the 128 * M undoes the -128 bias of the M
            // signed bytes and the rest turns "qd <= T" into "result < 0", so one sign test of the
            // OR of all results of the U steps decides whether anything was hit.
            v4i acc[U];
#pragma unroll
            for (int u = 0; u < U; ++u) acc[u] = acc0;
#pragma unroll
            for (int f = 0; f < C::NMF; ++f)
#pragma unroll
                for (int u = 0; u < U; ++u)
                    acc[u] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a[u][f], bsel, acc[u], 0, 0, 0);
            int sign = 0;
#pragma unroll
            for (int u = 0; u < U; ++u) sign |= acc[u][0] | acc[u][1] | acc[u][2] | acc[u][3];
            if (__ballot(sign < 0)) {                                // uniform, rare
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const int su = acc[u][0] | acc[u][1] | acc[u][2] | acc[u][3];
                    if (!__ballot(su < 0)) continue;                 // uniform: no hit in this step
                    const int first = (t0 + u) * C::CPS;             // first code of the step within the group
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        const bool h = acc[u][v] < 0 && first + cd[v] < nlive;
                        const uint64_t mask = __ballot(h);
                        if (!mask) continue;                         // uniform
                        const uint32_t cnt = __popcll(mask);
                        if (qlen + cnt > C::QCAP) flush();           // uniform: make room (cnt <= 64 = QCAP)
                        if (h) {
                            const uint64_t id = gbase + first + cd[v];
                            // result + T + 1 is the unsaturated sum (unsigned wrap-around is intended)
                            const uint32_t sum = static_cast<uint32_t>(acc[u][v]) + static_cast<uint32_t>(tl[v]) + 1u;
                            const uint32_t qd = min(sum, 255u);
                            wq[qlen + __popcll(mask & ((1ull << lane) - 1ull))] =
                                (static_cast<uint64_t>(ql[v]) << 40) | (static_cast<uint64_t>(qd) << 32) | id;
                        }
                        qlen += cnt;
                    }
                }
            }
        }
      }
    }
    flush();
}

// One workgroup per query: pick the exact r smallest (qd, id) out of the appended superset.
// flags[q] = 1 when the query must be redone (buffer overflow, or a tie bucket too large to sort).
__global__ __launch_bounds__(1024) void fast_select_kernel(const uint64_t *__restrict__ keys,
                                                          const uint32_t *__restrict__ count,
                                                          const uint32_t *__restrict__ chist, uint32_t r,
                                                          uint32_t cap, uint32_t sortcap, int use_lds,
                                                          uint64_t *__restrict__ spill,
                                                          uint32_t *__restrict__ cand_id,
                                                          uint8_t *__restrict__ cand_qd,
                                                          uint32_t *__restrict__ flags)
{
    extern __shared__ __align__(16) uint8_t smem[];
    __shared__ uint32_t cum[256];
    __shared__ uint32_t s_t, s_keep, s_pos;
    const int q = blockIdx.x, tid = threadIdx.x;
    const uint32_t n = count[q];
    if (n > cap || n < r) {                     // overflow (n < r cannot happen: the bound is safe)
        if (tid == 0) flags[q] = 1;
        return;
    }
    if (tid < 256) cum[tid] = chist[static_cast<size_t>(q) * 256 + tid];
    if (tid == 0) { s_t = 255; s_keep = n; s_pos = 0; }
    __syncthreads();
    for (int off = 1; off < 256; off <<= 1) {
        uint32_t add = 0;
        if (tid < 256 && tid >= off) add = cum[tid - off];
        __syncthreads();
        if (tid < 256) cum[tid] += add;
        __syncthreads();
    }
    if (tid < 256) {
        const uint32_t before = tid ? cum[tid - 1] : 0u;
        if (before < r && cum[tid] >= r) { s_t = tid; s_keep = cum[tid]; }
    }
    __syncthreads();
    const uint32_t T = s_t, keep = s_keep;
    if (keep > sortcap) {                        // tie bucket does not fit the sort area
        if (tid == 0) flags[q] = 1;
        return;
    }
    uint32_t np2 = 1;
    while (np2 < keep) np2 <<= 1;
    uint64_t *a = use_lds ? reinterpret_cast<uint64_t *>(smem) : spill + static_cast<size_t>(q) * sortcap;
    for (uint32_t t = tid; t < np2; t += 1024) a[t] = ~0ull;
    __syncthreads();
    for (uint32_t t = tid; t < n; t += 1024) {
        const uint64_t key = keys[static_cast<size_t>(q) * cap + t];
        if (static_cast<uint32_t>(key >> 32) <= T) {
            const uint32_t pos = atomicAdd(&s_pos, 1u);
            if (pos < np2) a[pos] = key;
        }
    }
    bitonic_sort(a, np2);
    for (uint32_t t = tid; t < r; t += 1024) {
        const uint64_t key = a[t];
        cand_id[static_cast<size_t>(q) * r + t] = static_cast<uint32_t>(key);
        cand_qd[static_cast<size_t>(q) * r + t] = static_cast<uint8_t>(key >> 32);
    }
    if (tid == 0) flags[q] = 0;
}

// Ordered list of the flagged queries and their number (one wavefront).
__global__ __launch_bounds__(64) void collect_flags_kernel(const uint32_t *__restrict__ flags, int nq,
                                                           int *__restrict__ qlist, uint32_t *__restrict__ nflag)
{
    const int lane = threadIdx.x;
    uint32_t total = 0;
    for (int base = 0; base < nq; base += 64) {
        const int q = base + lane;
        const bool f = q < nq && flags[q] != 0;
        const uint64_t mask = __ballot(f);
        if (f) qlist[total + __popcll(mask & ((1ull << lane) - 1ull))] = q;
        total += __popcll(mask);
    }
    if (lane == 0) *nflag = total;
}

// ---- host side ------------------------------------------------------------------------------

template <int M, int QT, int WAVES>
static int launch_fast_t(const uint16_t *codes, uint64_t n_codes, const uint8_t *qtab, int nq, uint32_t r,
                         uint32_t *cand_id, uint8_t *cand_qd, uint8_t *base, const ScanPlan &p, hipStream_t st)
{
    using C = FastCfg<M, QT, WAVES>;
    uint8_t *qsw = base + p.off_qsw;
    int *t_cur = reinterpret_cast<int *>(base + p.off_tcur);
    uint32_t *fcount = reinterpret_cast<uint32_t *>(base + p.off_fcount);
    uint32_t *chist = reinterpret_cast<uint32_t *>(base + p.off_chist);
    uint32_t *shist = reinterpret_cast<uint32_t *>(base + p.off_shist);
    uint64_t *fkeys = reinterpret_cast<uint64_t *>(base + p.off_fkeys);
    uint64_t *fsort = reinterpret_cast<uint64_t *>(base + p.off_fsort);
    uint32_t *flags = reinterpret_cast<uint32_t *>(base + p.off_flags);
    int *qlist = reinterpret_cast<int *>(base + p.off_qlist);
    uint32_t *nflag = reinterpret_cast<uint32_t *>(base + p.off_nflag);

    static bool attr_done = false;          // LDS above 64 KiB must be requested once per kernel
    if (!attr_done) {
        DCPQ_CHECK_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(&scan_fast_kernel<M, QT, WAVES>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, C::LDS_BYTES));
        DCPQ_CHECK_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(&fast_select_kernel),
                                           hipFuncAttributeMaxDynamicSharedMemorySize,
                                           static_cast<int>(sizeof(uint64_t) * kSortLdsKeys)));
        attr_done = true;
    }

    // swizzled tables
    DCPQ_LAUNCH(kStageMisc, st, (swizzle_tables_kernel<M, QT>), dim3((M * 256 * C::NQB + 255) / 256, p.ntiles),
                dim3(256), 0, qtab, nq, qsw);
    DCPQ_CHECK_LAUNCH("swizzle_tables_kernel");
    // sample histogram -> starting bounds
    int rc = launch_sample_hist(codes, n_codes, M, qtab, nq, r, shist, p, st);
    if (rc) return rc;
    DCPQ_LAUNCH(kStageSelect, st, sample_threshold_kernel, dim3(nq), dim3(256), 0, shist, r, t_cur);
    DCPQ_CHECK_LAUNCH("sample_threshold_kernel");
    // the scan
    DCPQ_LAUNCH(kStageScanFast, st, (scan_fast_kernel<M, QT, WAVES>), dim3(p.ntiles, p.fblocks), dim3(WAVES * 64),
                C::LDS_BYTES, codes, n_codes, p.codes_per_block, qsw, nq, r, p.cap, p.upd, t_cur, fcount, chist,
                fkeys);
    DCPQ_CHECK_LAUNCH("scan_fast_kernel");
    // exact selection + list of queries to redo
    const int use_lds = p.sortcap <= kSortLdsKeys;
    DCPQ_LAUNCH(kStageSelect, st, fast_select_kernel, dim3(nq), dim3(1024), use_lds ? sizeof(uint64_t) * p.sortcap : 0,
                fkeys, fcount, chist, r, p.cap, p.sortcap, use_lds, fsort, cand_id, cand_qd, flags);
    DCPQ_CHECK_LAUNCH("fast_select_kernel");
    DCPQ_LAUNCH(kStageSelect, st, collect_flags_kernel, dim3(1), dim3(64), 0, flags, nq, qlist, nflag);
    DCPQ_CHECK_LAUNCH("collect_flags_kernel");
    return DCPQ_OK;
}

int fast_lds_bytes(int m)
{
    switch (m) {
        case 4: return FastCfg<4, 64, 16>::LDS_BYTES;
        case 8: return FastCfg<8, 64, 16>::LDS_BYTES;
        case 16: return FastCfg<16, 32, 16>::LDS_BYTES;
        case 32: return FastCfg<32, 16, 8>::LDS_BYTES;
        default: return 0;
    }
}

int launch_scan_fast(const uint16_t *codes, uint64_t n_codes, int m, const uint8_t *qtab, int nq, uint32_t r,
                     uint32_t *cand_id, uint8_t *cand_qd, uint8_t *base, const ScanPlan &p, hipStream_t st)
{
    switch (m) {
        case 4: return launch_fast_t<4, 64, 16>(codes, n_codes, qtab, nq, r, cand_id, cand_qd, base, p, st);
        case 8: return launch_fast_t<8, 64, 16>(codes, n_codes, qtab, nq, r, cand_id, cand_qd, base, p, st);
        case 16: return launch_fast_t<16, 32, 16>(codes, n_codes, qtab, nq, r, cand_id, cand_qd, base, p, st);
        case 32: return launch_fast_t<32, 16, 8>(codes, n_codes, qtab, nq, r, cand_id, cand_qd, base, p, st);
        default: return fail(DCPQ_EUNSUPPORTED, "single-pass scan: m=%d not supported", m);
    }
}

}  // namespace dcpq
