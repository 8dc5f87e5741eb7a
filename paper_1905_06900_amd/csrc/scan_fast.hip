// Pass one of Alg. 3 (Sec. 3.3, Scan step) -- the single-pass kernel.
//
// What is computed is the same as in scan.hip: qd = min(255, sum_j Q_j[low8(c[j])]) for every
// (query, code) and the r smallest by (qd, id).  How it is computed differs from the paper's CPU
// loop in five ways that matter on this chip:
//
// 1. Row lookups instead of byte lookups.  A tile of QT queries keeps its tables in LDS
//    transposed, T[j][e][q] with the query fastest, so that the table entries of one (code, j)
//    for 16 queries are 16 contiguous bytes.  One ds_read_b128 per lane then delivers 1024
//    lookups per wavefront instruction, against 64 for byte gathers.  Rows of the same
//    sub-quantizer group are interleaved over a 256-byte LDS line (row slot = j mod NSLOT), and
//    which sub-quantizer a lane reads is rotated with its code slot so that the 16 lanes of a
//    lane group always touch 16 different 16-byte units of their lines (see rotated_j).
//
// 2. The sum over j runs on the matrix cores as an exact integer accumulation.  The 16-byte rows
//    are one operand; the other is constant and only says which bytes belong to which output:
//    for m = 4 four stacked 16 x 16 identities (v_mfma_i32_16x16x64_i8 adds 4 sub-quantizers), for
//    m >= 8 a structured-sparse pattern of ones (v_smfmac_i32_16x16x128_i8 adds 8 sub-quantizers
//    in the same time).  The instructions multiply SIGNED bytes, so the LDS copy of the tables
//    holds x - 128 (the byte with its top bit flipped) and the accumulator starts at 128 * M
//    instead of 0, which restores the unsigned sum exactly.  This is not a reshaping of the scan
//    into a dense product (no one-hot expansion: every byte multiplied is a byte the method looks
//    up); the matrix unit only replaces the byte unpack-and-add that the vector ALU would
//    otherwise spend three instructions per four lookups on.
//
// 3. Capped buckets become a running threshold.  Each query has a bucket bound T_cur that the
//    scan never lets fall below the bucket of its r-th best candidate: it starts from the histogram
//    of a strided sample of the codes, at the bucket where the sample's count reaches what r
//    codes of the whole array would leave in a sample of that size (plus five standard
//    deviations; when the sample is large the byte-gathering histogram kernel reads a sixteenth
//    of it and this kernel itself, in a pilot pass, counts the whole sample below the bound that
//    gives), and it is lowered whenever the exact per-bucket counts of the candidates
//    appended so far reach r below a smaller bucket (Sec. 3.3, Scan step: the dynamic upper bound
//    of the capped buckets).  A pair with qd <= T_cur is appended to the query's candidate buffer.
//    Whatever the timing of the updates, the buffer ends up a superset of the true candidate set,
//    from which the exact, id-tie-broken r are then selected; the result does not depend on the
//    order of arrival.  If a buffer overflows (pathological ties), or the estimated starting bound
//    turns out too low (fewer than r appended), the query is flagged and redone by the three-pass
//    path of scan.hip.
//
// 4. Appends stay off the critical path.  A query's buffer and append cursor are split into slices by
//    the workgroup's position along the codes (same-address returning atomics serialize in the L2),
//    and a wavefront hands its pending candidates over early when few queries face many
//    wavefronts, so that candidates waiting in queues never outnumber r.
//
// 5. The inner loop is a software pipeline.  The vector instruction port of a SIMD (matrix and
//    ordinary vector instructions share it) and the LDS are both close to full, and an LDS read
//    comes back hundreds of clocks after its issue; so (64-query tiles) the rows of the next
//    iteration and the code bytes of the one after it are always in flight, and everything
//    per-iteration that is not a row read, a matrix instruction, an address permute or the sign
//    test has been moved out of the loop (bounds live in LDS, code bytes are published a batch at
//    a time).  The 16- and 32-query tiles, which serve small batches where the code stream from
//    memory sets the pace, keep a single set of row registers: a second set would push per-lane
//    constants into scratch memory, and their reloads would queue behind the code prefetch.
#include <type_traits>

#include "common.h"
#include "lds_access.h"
#include "scan_internal.h"

namespace dcpq {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v8i __attribute__((ext_vector_type(8)));

template <int M, int QT, int WAVES>
struct FastCfg {
    static constexpr int NQB = QT / 16;             // 16-query blocks per table row
    static constexpr int CPS = 16 / NQB;            // codes per MFMA step
    static constexpr int NSLOT = 256 / QT;          // table rows per 256-byte LDS line
    static constexpr int NMF = M / 4;               // chained MFMAs per step
    static constexpr int STEPS = 64 / CPS;          // steps per 64-code group
    static constexpr int UNROLL = NMF >= 8 ? 1 : 8 / NMF;   // steps issued together (8 row reads in flight)
    static constexpr int CLS = M / 4;               // bytes per residue class j mod 4 of one code
    static constexpr bool ADJ = NQB != 4;           // lanes of one table row adjacent (else strided by CPS)
    static constexpr bool SPARSE = M >= 8;          // sum 8 rows per matrix instruction (else 4)
    static constexpr int REGION = STEPS * CLS;      // scratch bytes per (code slot, class): all steps of a group
    // Table rows per code value: when a line has more row slots than there are sub-quantizers the
    // tables are stored NSLOT / M times, so that every lane still finds its row in the slot its
    // position in the wavefront asks for.
    static constexpr int VJ = NSLOT > M ? NSLOT : M;
    static constexpr int TAB_BYTES = VJ * 256 * QT;
    static constexpr int QCAP = 64;                 // pending-candidate queue entries per wavefront (>= 64)
    static constexpr int Q_BYTES = WAVES * QCAP * 8;
    // 64-code groups fetched ahead per wavefront (and published to its scratch together): as many
    // as the LDS left beside the tables holds, at most 4
    static constexpr int BND_BYTES = 4 * QT;        // starting values of the accumulators, one per query of the tile
    static constexpr int ROOM = (160 * 1024 - TAB_BYTES - Q_BYTES - BND_BYTES) / (WAVES * 64 * M);
    static constexpr int PREFETCH = ROOM >= 4 ? 4 : ROOM >= 2 ? 2 : 1;
    static constexpr int SCR_BYTES = WAVES * PREFETCH * 64 * M;
    static constexpr int LDS_BYTES = TAB_BYTES + SCR_BYTES + Q_BYTES + BND_BYTES;
    static_assert(M % 4 == 0 && VJ % M == 0, "row slots rotate within the (possibly repeated) sub-quantizers");
    static_assert(ROOM >= 1 && LDS_BYTES <= 160 * 1024, "one workgroup must fit the LDS of a CU");
    static_assert(STEPS % UNROLL == 0, "unroll must divide the steps of a group");
    static_assert(UNROLL * CLS == 8, "the steps issued together read one 8-byte word of code bytes");
    static_assert(CPS * 4 * REGION == 64 * M, "scratch regions tile the group");
};

// Table row set jv read by MFMA u, chunk s (= lane / 16), for code slot c; the sub-quantizer is
// j = jv mod M (row sets M and above are the repeated copies).  For a fixed c the map (u, s) -> j is
// a bijection onto 0..M-1, j mod 4 does not depend on u, and the row slots (jv mod NSLOT) of the 16
// lanes of a chunk are all different.  The rotations are the ones that
// measured fastest for ds_read_b128: with 4 slots, slot = s + c and the four lanes of a row strided
// by 4; with 8 slots, slot = s + 2c (+4u); with 16 slots, the low two slot bits rotate with c and the
// high two with c / 4.
template <int NSLOT>
__device__ inline int rotated_j(int u, int s, int c)
{
    const int g = 4 * u + s;
    if constexpr (NSLOT == 4) return (g & ~3) | ((g + c) & 3);
    else if constexpr (NSLOT == 8) return (g & ~7) | ((g + 2 * c) & 7);
    else {
        static_assert(NSLOT == 16, "row slots per line: 4, 8 or 16");
        return (g & ~15) | ((s + c) & 3) | (((u + (c >> 2)) & 3) << 2);
    }
}

// Byte offset of T[j][e][q] in the swizzled tile layout (shared by the transposition kernel and
// the scan kernel).
template <int QT>
__host__ __device__ inline uint32_t swz_offset(int j, int e, int q)
{
    constexpr int NSLOT = 256 / QT;
    return (static_cast<uint32_t>(j / NSLOT) * 256u + e) * 256u + (j % NSLOT) * QT + q;
}

// qtab [nq][M][256] -> per-tile swizzled tables [ntiles][VJ*256*QT], each byte stored as x - 128
// (x ^ 0x80) for the signed matrix instruction; absent queries read 255.
template <int M, int QT>
__global__ __launch_bounds__(256) void swizzle_tables_kernel(const uint8_t *__restrict__ qtab, int nq,
                                                             uint8_t *__restrict__ out)
{
    const int tile = blockIdx.y;
    const int idx = blockIdx.x * 256 + threadIdx.x;      // (jv, e, qb)
    constexpr int NQB = QT / 16;
    constexpr int VJ = 256 / QT > M ? 256 / QT : M;      // row sets, repeated copies included
    if (idx >= VJ * 256 * NQB) return;
    const int qb = idx % NQB, e = (idx / NQB) % 256, jv = idx / (NQB * 256), j = jv % M;
    uint32_t w[4] = {0, 0, 0, 0};
#pragma unroll
    for (int t = 0; t < 16; ++t) {
        const int q = tile * QT + qb * 16 + t;
        const uint32_t v = q < nq ? qtab[(static_cast<size_t>(q) * M + j) * 256 + e] : 255u;
        w[t >> 2] |= (v ^ 0x80u) << (8 * (t & 3));
    }
    uint8_t *dst = out + static_cast<size_t>(tile) * (VJ * 256 * QT) + swz_offset<QT>(jv, e, qb * 16);
    *reinterpret_cast<uint4 *>(dst) = make_uint4(w[0], w[1], w[2], w[3]);
}

// Starting bucket bound of every query from the histogram of a sample of S of the n codes.
// The bucket of the sample's r-th smallest qd is a bound that cannot fail (the sample is part of the
// array), but it lets r / S of all codes through.  The array's r-th smallest qd is about the sample's
// (r S / n)-th smallest, so the bound starts at the bucket where the sample's cumulative count reaches
// e + 5 sqrt(e) + 5 with e = r S / n (five standard deviations of the count above its mean: a query in
// ten million starts too low), or r if that is smaller.  Should that bucket hold fewer than r codes of the whole array after all, the
// selection sees fewer than r appended candidates and has the query redone by the three-pass path.
__global__ __launch_bounds__(256) void sample_threshold_kernel(const uint32_t *__restrict__ shist, uint32_t r,
                                                               uint64_t n_codes, const uint32_t *__restrict__ n_each,
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
    uint32_t rs = r;
    if (n_each) n_codes = n_each[q];                      // every query scans its own codes (probed lists)
    if (n_codes) {                                        // 0: the sample's own r-th smallest
        const float e = static_cast<float>(r) * static_cast<float>(cum[255]) / static_cast<float>(n_codes);
        const float want = e + 5.0f * sqrtf(e) + 5.0f;
        if (want < static_cast<float>(r)) rs = static_cast<uint32_t>(want) + 1u;
    }
    const uint32_t before = b ? cum[b - 1] : 0u;
    if (before < rs && cum[b] >= rs) t_cur[q] = b;
    if (b == 255 && cum[255] < rs) t_cur[q] = 255;
}

// Low bytes of the M sub-codes of one code, reordered by residue class: byte (j & 3) * CLS + (j >> 2).
// w: the code as stored -- uint16 sub-codes (sub-codes 2i and 2i+1 in w[i]; the low byte of j is byte
// 2 * (j & 1) of w[j / 2]) or, for the low-byte plane, the bytes themselves (byte j & 3 of w[j / 4]).
template <int M, typename CodeT>
__device__ inline void transposed_low_bytes(const uint32_t (&w)[M * sizeof(CodeT) / 4], uint32_t (&out)[M / 4])
{
    constexpr bool WIDE = sizeof(CodeT) == 2;
    if constexpr (M == 4) {
        out[0] = WIDE ? __builtin_amdgcn_perm(w[WIDE ? 1 : 0], w[0], 0x06040200u) : w[0];      // j = 0, 1, 2, 3
    } else if constexpr (M == 8 && WIDE) {
        out[0] = __builtin_amdgcn_perm(w[2], w[0], 0x06020400u);       // j = 0, 4, 1, 5
        out[1] = __builtin_amdgcn_perm(w[3], w[1], 0x06020400u);       // j = 2, 6, 3, 7
    } else if constexpr (M == 8) {
        out[0] = __builtin_amdgcn_perm(w[1], w[0], 0x05010400u);       // j = 0, 4, 1, 5
        out[1] = __builtin_amdgcn_perm(w[1], w[0], 0x07030602u);       // j = 2, 6, 3, 7
    } else {
#pragma unroll
        for (int d = 0; d < M / 4; ++d) out[d] = 0;
#pragma unroll
        for (int j = 0; j < M; ++j) {
            const uint32_t b = WIDE ? (w[j >> 1] >> (16 * (j & 1))) & 255u : (w[j >> 2] >> (8 * (j & 3))) & 255u;
            const int p = (j & 3) * (M / 4) + (j >> 2);
            out[p >> 2] |= b << (8 * (p & 3));
        }
    }
}

// Appends one candidate (rec: id in bits 0..31, qd in 32..39, query-in-tile in 40..47) to slice
// `slice` of its query's buffer (unless cap = 0) and counts it in the query's exact per-bucket histogram.  Returns the
// query when this append is one of those (every `upd`-th of the slice) after which the query's bucket
// bound is to be recomputed, else -1.  Kept out of line: it is the rare path and would otherwise be
// replicated at every call site.
__device__ __noinline__ int append_candidate(uint64_t rec, int q0, uint32_t slice, uint32_t nslices, uint32_t cap, uint32_t upd,
                                             int *t_cur, uint32_t *count, uint32_t *chist, uint64_t *keys)
{
    const uint32_t q = q0 + static_cast<uint32_t>(rec >> 40);
    const uint32_t qd = static_cast<uint32_t>(rec >> 32) & 255u;
    const size_t cell = static_cast<size_t>(q) * nslices + slice;
    const uint32_t pos = atomicAdd(&count[cell], 1u);
    if (pos < cap) keys[cell * cap + pos] = rec & 0xFFFFFFFFFFull;
    else if (cap) atomicMin(&t_cur[q], -1);            // slice full: stop appending, query is redone
    // (cap = 0: the pilot pass, which only counts)
    atomicAdd(&chist[static_cast<size_t>(q) * 256 + qd], 1u);
    return (pos + 1) % upd == 0 ? static_cast<int>(q) : -1;
}

template <int M, int QT, int WAVES, typename CodeT>
__global__ __launch_bounds__(WAVES * 64) void scan_fast_kernel(
    const CodeT *__restrict__ codes, uint64_t code_end, uint64_t block_stride, uint32_t block_groups, uint32_t total_groups,
    uint32_t gshift, uint32_t gstride, const uint8_t *__restrict__ qsw, int nq, uint32_t r, uint32_t nslices, uint32_t cap,
    uint32_t upd, uint32_t qflush, int *t_cur, uint32_t *count, uint32_t *chist, uint64_t *__restrict__ keys)
{
    // The codes of workgroup y (blockIdx.y) are 64-code groups y * block_groups ... (block_groups of them, fewer
    // at the end: total_groups in all); group g of the workgroup starts at code
    //   y * block_stride + (g >> gshift) * gstride + (g mod 2^gshift) * 64
    // and ends before code_end.  The scan of the whole array is gshift = 0, gstride = 64, block_stride = 64 *
    // block_groups (one contiguous stretch per workgroup); the pilot pass over a sample reads runs of 2^gshift
    // groups that start every gstride codes.  cap = 0 (pilot pass): candidates are counted in chist but not
    // stored, and a bound of 255 lets nothing through instead of everything.
    using C = FastCfg<M, QT, WAVES>;
    constexpr int PF = C::PREFETCH;
    extern __shared__ __align__(16) uint8_t smem[];
    uint8_t *ltab = smem;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);      // wave-uniform: keep it (and what derives from it) scalar
    uint8_t *scr = smem + C::TAB_BYTES + wave * (PF * 64 * M);
    uint64_t *wq = reinterpret_cast<uint64_t *>(smem + C::TAB_BYTES + C::SCR_BYTES) + wave * C::QCAP;
    int *lbnd = reinterpret_cast<int *>(smem + C::TAB_BYTES + C::SCR_BYTES + C::Q_BYTES);

    const int tile = blockIdx.x;
    const int q0 = tile * QT;
    // Bucket bound T of a query as the value its accumulators start from, 128 * M - (T + 1): the
    // 128 * M undoes the -128 bias of the M signed bytes and the rest turns "qd <= T" into
    // "result < 0".  A bound of 255 lets every code through (the sum itself is not capped), an
    // absent query has the bound -1 that nothing reaches.
    auto start_value = [&](int q) {
        int t = -1;
        if (q < nq) t = __hip_atomic_load(&t_cur[q], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (cap == 0 && t >= 255) t = -1;
        return t >= 255 ? static_cast<int>(128u * M - 0x80000000u) : static_cast<int>(128u * M - static_cast<uint32_t>(t) - 1u);
    };
    {
        const uint4 *src = reinterpret_cast<const uint4 *>(qsw + static_cast<size_t>(tile) * C::TAB_BYTES);
        uint4 *dst = reinterpret_cast<uint4 *>(ltab);
        for (int v = tid; v < C::TAB_BYTES / 16; v += WAVES * 64) dst[v] = src[v];
        if (tid < QT) lbnd[tid] = start_value(q0 + tid);
    }
    __syncthreads();

    // ---- per-lane constants -------------------------------------------------------------
    const int s = lane >> 4, i = lane & 15;
    // position i of a 16-lane chunk stands for (code slot ca, query block qba)
    const int ca = C::ADJ ? i / C::NQB : i % C::CPS, qba = C::ADJ ? i % C::NQB : i / C::CPS;
    // Address of row read f = laneoff[f] with its (zero) second byte replaced by the code byte, one
    // v_perm_b32: sel[f] picks, out of a 32-bit word of class bytes, the byte of this lane's
    // sub-quantizer j (byte j / 4 of the class word j mod 4).
    // The tables start at LDS offset lds0 = 0 (the kernel has no static LDS; the host checks that),
    // so every laneoff has a zero second byte.
    const uint32_t lds0 = lds_offset_of(ltab);
    uint32_t laneoff[C::NMF], selb[C::NMF];
#pragma unroll
    for (int f = 0; f < C::NMF; ++f) {
        const int jv = rotated_j<C::NSLOT>(f, s, ca);
        laneoff[f] = lds0 + swz_offset<QT>(jv, 0, qba * 16);
        selb[f] = C::NSLOT == 4 ? static_cast<uint32_t>(f) : static_cast<uint32_t>((jv % M) >> 2);
    }
    const int cls = rotated_j<C::NSLOT>(0, s, ca) & 3;     // residue class j mod 4 read by this lane
    const uint32_t scr_rd = lds_offset_of(scr) + (ca * 4 + cls) * C::REGION;    // + 64 M (group of the batch) + 8 (iteration)
    // Dense form (M = 4): A = the gathered rows (row i of the matrix = this chunk position), B = four
    // stacked 16 x 16 identities; output value v of this lane belongs to chunk position
    // 4 * (lane / 16) + v and to query lane % 16 of the block.
    // Sparse form (M >= 8): the roles are swapped and the structured-sparse operand (two stored
    // values out of every four along K = 128) is the constant one: its row n holds a 1 wherever K
    // addresses byte n of one of the 8 gathered rows of a column, so one instruction adds 8
    // sub-quantizers.  The stored values sit in 8 pairs per lane; pair g of lane (n, k) with index p
    // meets byte 16 * (k / 2) + 4 * (g mod 4) + p of the dense operand's lane 2 * (k mod 2) + g / 4 of
    // the same column (found by feeding the instruction single ones).  Output value v of this lane
    // belongs to query 4 * (lane / 16) + v of the block and to chunk position lane % 16.
    constexpr bool SP = C::SPARSE;
    v4i bsel = {0, 0, 0, 0};
    int spidx = 0;
    if constexpr (SP) {
        const int t1 = 2 * (i >> 2), t2 = 8 + 2 * (i >> 2);        // first value of pairs i / 4 and 4 + i / 4
        bsel[t1 >> 2] |= 1 << (8 * (t1 & 3));
        bsel[t2 >> 2] |= 1 << (8 * (t2 & 3));
        spidx = ((i & 3) << (2 * t1)) | ((i & 3) << (2 * t2));
    } else {
        bsel[i >> 2] = 1 << (8 * (i & 3));
    }
    // code slot and query (within the tile) of output value v
    auto code_slot_of = [&](int v) { return SP ? ca : (C::ADJ ? (4 * s + v) / C::NQB : (4 * s + v) % C::CPS); };
    auto query_at = [](int ln, int v) {
        const int ss = ln >> 4, ii = ln & 15;
        if constexpr (SP) return (C::ADJ ? ii % C::NQB : ii / C::CPS) * 16 + 4 * ss + v;
        else return (C::ADJ ? (4 * ss + v) % C::NQB : (4 * ss + v) / C::CPS) * 16 + ii;
    };
    auto query_of = [&](int v) { return query_at(lane, v); };

    // this workgroup's codes (ids fit 32 bits: the host checks n_codes)
    const uint32_t cbeg = static_cast<uint32_t>(static_cast<uint64_t>(blockIdx.y) * block_stride);
    const uint32_t cend = static_cast<uint32_t>(code_end);
    const uint32_t gfirst = blockIdx.y * block_groups;
    const uint32_t ngroups = gfirst < total_groups ? min(block_groups, total_groups - gfirst) : 0u;
    const uint32_t gmask = (1u << gshift) - 1u;
    auto group_base = [&](uint32_t g) { return cbeg + (g >> gshift) * gstride + (g & gmask) * 64u; };     // for g < ngroups

    // Pending candidates of this wavefront: records wq[0 .. qlen), qlen <= QCAP = 64.  qlen is
    // wave-uniform (it only changes by ballot counts), so it lives in a scalar register and the queue
    // needs no atomics.
    static_assert(C::QCAP == 64, "flush hands one record to each lane");
    uint32_t qlen = 0;
    const uint32_t slice = blockIdx.y % nslices;
    auto flush = [&]() {
        // the wavefront runs in lockstep; the barriers say that every push is in place before the
        // entries are read, and that every lane has read its entry before the next push overwrites it
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        int qu = -1;
        if (static_cast<uint32_t>(lane) < qlen) qu = append_candidate(wq[lane], q0, slice, nslices, cap, upd, t_cur, count, chist, keys);
        // the queries whose bound is due, one after the other, each by the whole wavefront
        uint64_t due = __builtin_amdgcn_ballot_w64(qu >= 0);
        while (due) {                                    // uniform
            const int src = __builtin_ctzll(due);
            due &= due - 1;
            lower_bound_of(__shfl(qu, src), r, t_cur, chist);
        }
        qlen = 0;
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    };

    // ---- the code stream ------------------------------------------------------------------
    // This wavefront's groups are wave, wave + WAVES, ...; they are fetched PF at a time and one batch
    // ahead of their use, so that each wavefront keeps PF kilobytes of the code stream in flight.
    const uint32_t ng_w = ngroups > static_cast<uint32_t>(wave) ? (ngroups - wave + WAVES - 1) / WAVES : 0u;
    constexpr int RW = M * static_cast<int>(sizeof(CodeT)) / 4;     // words per code as stored
    auto load_group = [&](uint32_t g, uint32_t (&dst)[RW]) {
        const uint32_t id = group_base(g) + lane;
        if (g < ngroups && id < cend) {
            const uint8_t *src = reinterpret_cast<const uint8_t *>(codes) + static_cast<uint64_t>(id) * (4 * RW);
            if constexpr (RW % 4 == 0) {
#pragma unroll
                for (int v = 0; v < RW / 4; ++v) {
                    const uint4 x = reinterpret_cast<const uint4 *>(src)[v];
                    dst[4 * v] = x.x; dst[4 * v + 1] = x.y; dst[4 * v + 2] = x.z; dst[4 * v + 3] = x.w;
                }
            } else if constexpr (RW == 2) {
                const uint2 x = *reinterpret_cast<const uint2 *>(src);
                dst[0] = x.x; dst[1] = x.y;
            } else {
                static_assert(RW == 1, "codes of 4, 8 or a multiple of 16 bytes");
                dst[0] = *reinterpret_cast<const uint32_t *>(src);
            }
        } else {
#pragma unroll
            for (int v = 0; v < RW; ++v) dst[v] = 0;
        }
    };
    uint32_t wb[PF][RW];
    auto load_batch = [&](uint32_t g0) {
#pragma unroll
        for (int pf = 0; pf < PF; ++pf) load_group(g0 + pf * WAVES, wb[pf]);
    };
    load_batch(wave);
    uint32_t g_load = wave + PF * WAVES;                     // first group of the batch to fetch next

    // Bucket bounds.  The workgroup keeps the accumulator start values of its tile's queries in LDS;
    // once per batch every wavefront re-reads those of its four outputs, and now and then (every
    // batch at first, when the bounds move fastest, every fourth later) one wavefront, in turn,
    // renews the array from the bounds in global memory (lane = query).  A stale bound is still a
    // valid one (bounds only go down), so neither step needs any ordering, and only one wavefront per
    // workgroup touches the cache line that holds the tile's bounds.
    uint32_t batch = 0;

    // ---- the pipeline ---------------------------------------------------------------------
    // One iteration = U steps = 8 table-row reads per lane and the matrix instructions that add
    // them; a 64-code group is NI iterations.  All iterations of the wavefront form one software
    // pipeline, because with 16 wavefronts queueing on one LDS a read comes back hundreds of clocks
    // after it was issued: while the matrix instructions of iteration n run, the row reads of
    // iteration n + 1 and the 8-byte read of the code bytes of iteration n + 2 are already in flight.
    // Two register sets of rows (ra, rb) and two code-byte words alternate; the loop body is one
    // group (two when a group is a single iteration), so that every LDS instruction has a fixed
    // place in it and the waits can count.  The pipeline runs up to two iterations past the
    // wavefront's last group: those reads find zero code bytes and valid table rows, and their
    // results are never used.
    constexpr int U = C::UNROLL, NI = C::STEPS / U, GB = NI == 1 ? 2 : 1;
    static_assert(NI == 1 || NI % 2 == 0, "the two row sets alternate evenly over a group");
    static_assert(PF % GB == 0, "a batch is a whole number of loop bodies");

    // Makes the next group the current one: `area` is the scratch offset of its code bytes.  When
    // the fetched batch is used up, the low bytes of the next one are published to the wavefront's
    // scratch, PF groups side by side.  Lane l holds code l = step l / CPS, code slot l % CPS of its
    // group; its M / 4 bytes of class k go to region (slot, k) at the step's position, so that a
    // reader finds the bytes of the U steps of an iteration in one 8-byte word.  Overwriting the
    // scratch is safe: the LDS executes a wavefront's instructions in order, and every read of the
    // previous batch has been issued by now (the code-byte reads run two iterations ahead).
    uint32_t ring = PF;                                      // groups of the published batch used up
    uint32_t area = 0;
    auto next_group = [&]() {
        if (ring == PF) {                                    // uniform
            uint8_t *dst = scr + (lane % C::CPS) * (4 * C::REGION) + (lane / C::CPS) * C::CLS;
#pragma unroll
            for (int pf = 0; pf < PF; ++pf) {
                uint32_t tb[M / 4];
                transposed_low_bytes<M, CodeT>(wb[pf], tb);
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    uint8_t *d = dst + pf * (64 * M) + k * C::REGION;
                    if constexpr (C::CLS == 1) *d = static_cast<uint8_t>(tb[0] >> (8 * k));
                    else if constexpr (C::CLS == 2) *reinterpret_cast<uint16_t *>(d) = static_cast<uint16_t>(tb[k >> 1] >> (16 * (k & 1)));
                    else if constexpr (C::CLS == 4) *reinterpret_cast<uint32_t *>(d) = tb[k];
                    else *reinterpret_cast<uint2 *>(d) = make_uint2(tb[2 * k], tb[2 * k + 1]);
                }
            }
            load_batch(g_load);                              // fetch the batch after it
            g_load += PF * WAVES;
            ring = 0;
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        }
        area = ring * (64 * M);
        ++ring;
    };
    // code bytes of the U steps at position p of the current group
    auto read_word = [&](int p) -> uint2 {
        typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
        typedef const u32x2 __attribute__((address_space(3))) *ptr_t;
        const u32x2 x = *reinterpret_cast<ptr_t>(static_cast<uintptr_t>(scr_rd + area + p * 8));
        return make_uint2(x[0], x[1]);
    };
    // the 8 row reads of an iteration
    auto issue_rows = [&](const uint2 word, v4i (&a)[U][C::NMF]) {
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int f = 0; f < C::NMF; ++f) {
                // byte u * CLS + j / 4 of the 8-byte word; which of its two halves is known statically
                const int stat = u * C::CLS + (C::CLS == 8 ? 4 * (f >> 2) : 0);
                const uint32_t half = stat >= 4 ? word.y : word.x;
                const uint32_t sel = 0x07060004u | (((static_cast<uint32_t>(stat) + selb[f]) & 3u) << 8);
                const uint32_t addr = __builtin_amdgcn_perm(laneoff[f], half, sel);
                a[u][f] = lds_read_v4i(addr);
            }
    };
    // The accumulations over the rows of the iteration at position p of group g (independent chains,
    // UC steps at a time so that few accumulators are live at once), the sign test of each such
    // chunk, and (for a few per cent of the chunks) the hits
    constexpr int UC = U < 4 ? U : 4;
    auto compute = [&](const v4i (&a)[U][C::NMF], const v4i acc0, uint32_t g, int p) {
#pragma unroll
        for (int uc = 0; uc < U; uc += UC) {
            v4i acc[UC];
#pragma unroll
            for (int u = 0; u < UC; ++u) acc[u] = acc0;
            if constexpr (SP) {
#pragma unroll
                for (int f = 0; f < C::NMF; f += 2)
#pragma unroll
                    for (int u = 0; u < UC; ++u) {
                        const v8i rows = __builtin_shufflevector(a[uc + u][f], a[uc + u][f + 1], 0, 1, 2, 3, 4, 5, 6, 7);
                        acc[u] = __builtin_amdgcn_smfmac_i32_16x16x128_i8(bsel, rows, acc[u], spidx, 0, 0);
                    }
            } else {
#pragma unroll
                for (int f = 0; f < C::NMF; ++f)
#pragma unroll
                    for (int u = 0; u < UC; ++u)
                        acc[u] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a[uc + u][f], bsel, acc[u], 0, 0, 0);
            }
            // OR of all 4 UC results, two new values per three-input OR
            int sign = acc[0][0];
#pragma unroll
            for (int x = 1; x + 1 < 4 * UC; x += 2) sign = sign | acc[x >> 2][x & 3] | acc[(x + 1) >> 2][(x + 1) & 3];
            sign = sign | acc[UC - 1][3];
            if (!__builtin_amdgcn_ballot_w64(sign < 0)) continue;    // uniform
            // codes in this group: fewer than 64 in the last group of the stretch, none past it
            const uint32_t gbase = group_base(g);
            const int nlive = g < ngroups && gbase < cend ? static_cast<int>(min(64u, cend - gbase)) : 0;
            // Which of the 4 UC results hold the hit(s): one compare per result, whose outcome is a lane mask
            // in scalar registers, so that the search for the (usually single) result with a hit runs on the
            // scalar unit and only that result is decoded on the vector unit.
#pragma unroll
            for (int u = 0; u < UC; ++u) {
                const int first = (p * U + uc + u) * C::CPS;    // first code of the step within the group
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    if (!__builtin_amdgcn_ballot_w64(acc[u][v] < 0)) continue;      // uniform
                    // (the empty asm keeps the compiler from precomputing, and then spilling, this sum for
                    // every step of a group outside the loop)
                    int slot = code_slot_of(v);
                    asm volatile("" : "+v"(slot));
                    const int code = first + slot;
                    const bool h = acc[u][v] < 0 && code < nlive;
                    const uint64_t mask = __builtin_amdgcn_ballot_w64(h);
                    if (!mask) continue;                         // uniform
                    const uint32_t cnt = __popcll(mask);
                    if (qlen + cnt > C::QCAP) flush();           // uniform: make room (cnt <= 64 = QCAP)
                    if (h) {
                        const uint32_t id = gbase + static_cast<uint32_t>(code);
                        // result - start value + 128 M is the unsaturated sum (unsigned wrap-around is intended)
                        const uint32_t sum = static_cast<uint32_t>(acc[u][v]) - static_cast<uint32_t>(acc0[v]) + 128u * M;
                        const uint32_t qd = min(sum, 255u);
                        const uint32_t rank = __builtin_amdgcn_mbcnt_hi(
                            static_cast<uint32_t>(mask >> 32),
                            __builtin_amdgcn_mbcnt_lo(static_cast<uint32_t>(mask), 0u));
                        wq[qlen + rank] = (static_cast<uint64_t>((static_cast<uint32_t>(query_of(v)) << 8) | qd) << 32) | id;
                    }
                    qlen = __builtin_amdgcn_readfirstlane(qlen + cnt);      // wave-uniform: keep it scalar
                }
            }
            if (qlen >= qflush) flush();                       // uniform: keep the invisible backlog small
        }
    };

    // With 64-query tiles the rows of the next iteration are in flight while this one is summed (two
    // register sets).  The smaller tiles keep one set: they are used where few queries face the code
    // stream, the memory system rather than the LDS sets their pace, and the second set would push
    // per-lane constants out of the register file into scratch memory, whose reloads wait behind
    // (and so serialize with) the prefetched code loads.
    constexpr bool DEEP = C::NSLOT == 4;
    if (ng_w) {
        v4i ra[U][C::NMF], rb[DEEP ? U : 1][C::NMF];
        uint2 w[2];
        next_group();
        w[0] = read_word(0);
        if constexpr (NI == 1) next_group();
        w[1] = read_word(NI == 1 ? 0 : 1);
        if constexpr (DEEP) issue_rows(w[0], ra);
#pragma unroll 1
        for (uint32_t gi = 0; gi < ng_w; gi += GB) {
            if (gi % PF == 0) {                                  // uniform
                if ((batch < 8 || (batch & 3u) == 0) && batch % WAVES == static_cast<uint32_t>(wave)) {
                    if (lane < QT) lbnd[lane] = start_value(q0 + lane);      // this wavefront's turn to renew them
                }
                ++batch;
            }
            // start values of this lane's four accumulator values, re-read for every loop body: one sign
            // test of the OR of all results of a chunk decides whether anything was hit
            // (the lane index is taken afresh so that the addresses are recomputed here rather than
            // kept, spilled, in registers over the whole loop)
            v4i acc0;
            {
                uint32_t zero = 0;
                asm volatile("" : "+v"(zero));
                const int ln = static_cast<int>(__builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, zero)));
#pragma unroll
                for (int v = 0; v < 4; ++v) acc0[v] = lbnd[query_at(ln, v)];
            }
            const uint32_t g = wave + gi * WAVES;
#pragma unroll
            for (int t = 0; t < GB * NI; ++t) {
                // code bytes of the iteration after the next (into the word whose rows are already
                // on their way), then the rows of the next iteration
                if constexpr (DEEP) {
                    if ((t + 2) % NI == 0) next_group();
                    w[t % 2] = read_word((t + 2) % NI);
                    if (t % 2 == 0) issue_rows(w[1], rb); else issue_rows(w[0], ra);
                    if (t % 2 == 0) compute(ra, acc0, g + (t / NI) * WAVES, t % NI);
                    else compute(rb, acc0, g + (t / NI) * WAVES, t % NI);
                } else {
                    issue_rows(w[t % 2], ra);
                    if ((t + 2) % NI == 0) next_group();
                    w[t % 2] = read_word((t + 2) % NI);
                    compute(ra, acc0, g + (t / NI) * WAVES, t % NI);
                }
            }
        }
    }
    flush();
}

// The selection orders candidates by counting ranks inside small groups (the work grows with the
// square of the group size); a query with a group larger than this goes through the bitonic network.
constexpr uint32_t kRankGroup = 2048;
constexpr int kRangeBits = 11;                          // finest split of the ids: 2048 equal ranges
constexpr uint32_t kGroups = 2048;                      // (bucket, id range) groups the counting sort holds
constexpr size_t kSelectLdsMost = 120 * 1024;

// LDS of the rank-counting selection: group counters and group starts (uint32 each), then the ids
// (uint32) and group numbers (uint16) of up to sortcap candidates.
static size_t rank_lds_bytes(uint32_t sortcap) { return 8 * static_cast<size_t>(kGroups) + 6 * static_cast<size_t>(sortcap); }

// One workgroup per query: pick the exact r smallest (qd, id) out of the appended superset.
// flags[q] = 1 when the query must be redone (buffer overflow, fewer than r candidates, or more
// candidates at or below the bound than the sort area holds).
// The candidates at or below the bound are dealt into groups -- (bucket, one of 2^s equal ranges of the
// ids), over the buckets from the first one that holds a candidate up to the bound's (the r smallest of
// an array sit in a handful of buckets, with nothing below them), s as large as 2048 groups allow: 8
// ranges if all 256 buckets were in play, 2048 when everything ties in one bucket -- by a counting sort:
// one pass over the buffer counts the groups, a prefix sum gives every group its place in the output
// (groups ordered by bucket, then by id range, are already in (qd, id) order), a second pass deals the
// ids out, and inside a group a candidate's rank is the number of ids below its own.  With the ids spread
// over the array the groups hold a few ids, so this is several times cheaper than a sorting network
// over the whole set, which remains for queries with a very large group (many equal qd in one stretch
// of ids).
// id_mul: the finest id range of an id is the high word of id * id_mul (below 2048 for every id of the
// array, and non-decreasing in the id, which is all the order needs); coarser ranges are its top bits.
__global__ __launch_bounds__(1024) void fast_select_kernel(const uint64_t *__restrict__ keys,
                                                          const uint32_t *__restrict__ count,
                                                          const uint32_t *__restrict__ chist, uint32_t r, uint32_t nslices,
                                                          uint32_t cap, uint32_t sortcap, int use_lds, int rank_ok,
                                                          uint32_t id_mul, uint64_t *__restrict__ spill,
                                                          uint32_t *__restrict__ cand_id,
                                                          uint8_t *__restrict__ cand_qd,
                                                          uint32_t *__restrict__ flags)
{
    extern __shared__ __align__(16) uint8_t smem[];
    __shared__ uint32_t cum[256];                // inclusive prefix of the bucket counts
    __shared__ uint32_t wsum[16];
    __shared__ uint32_t s_t, s_keep, s_pos, s_big, s_b0;
    const int q = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    uint32_t n = 0;
    bool over = false;
    for (uint32_t sl = 0; sl < nslices; ++sl) {
        const uint32_t c = count[static_cast<size_t>(q) * nslices + sl];
        over = over || c > cap;
        n += c;
    }
    if (over || n < r) {                        // a slice overflowed, or the starting bound was too low after all
        if (tid == 0) flags[q] = 1;
        return;
    }
    if (tid < 256) cum[tid] = chist[static_cast<size_t>(q) * 256 + tid];
    if (tid == 0) { s_t = 255; s_keep = n; s_pos = 0; s_big = 0; s_b0 = 0; }
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
        if (before == 0 && cum[tid] > 0) s_b0 = tid;                      // the first bucket that holds a candidate
    }
    __syncthreads();
    const uint32_t T = s_t, keep = s_keep, b0 = s_b0;
    if (keep > sortcap) {                        // tie bucket does not fit the sort area
        if (tid == 0) flags[q] = 1;
        return;
    }
    if (rank_ok) {
        uint32_t *gcnt = reinterpret_cast<uint32_t *>(smem);              // [kGroups] count, later the deal-out cursor
        uint32_t *gstart = gcnt + kGroups;                                // [kGroups] first output position of the group
        uint32_t *ids = gstart + kGroups;                                 // [sortcap]
        uint16_t *grp = reinterpret_cast<uint16_t *>(ids + sortcap);      // [sortcap]
        // the groups cover the buckets b0 .. T only (the r smallest of an array sit in a few buckets just below T, and
        // the buckets under them are empty: counting them would leave most groups unused and the rest large)
        const uint32_t nbuckets = T - b0 + 1;
        int sub_bits = 0;
        while (sub_bits < kRangeBits && (nbuckets << (sub_bits + 1)) <= kGroups) ++sub_bits;
        const int range_shift = kRangeBits - sub_bits;
        const uint32_t ngroups = nbuckets << sub_bits;
        for (uint32_t t = tid; t < ngroups; t += 1024) gcnt[t] = 0;
        __syncthreads();
        // count the groups: one wavefront per slice at a time, so that the slices' loads are in flight together
        for (uint32_t sl = wave; sl < nslices; sl += 16) {
            const size_t cell = static_cast<size_t>(q) * nslices + sl;
            const uint32_t c = count[cell];
#pragma unroll 4
            for (uint32_t t = lane; t < c; t += 64) {
                const uint64_t key = keys[cell * cap + t];
                const uint32_t qd = static_cast<uint32_t>(key >> 32);
                if (qd <= T) atomicAdd(&gcnt[((qd - b0) << sub_bits) + (__umulhi(static_cast<uint32_t>(key), id_mul) >> range_shift)], 1u);
            }
        }
        __syncthreads();
        // exclusive prefix over the groups (two per thread), and the largest group
        {
            const uint32_t g0 = 2 * tid, g1 = 2 * tid + 1;
            const uint32_t c0 = g0 < ngroups ? gcnt[g0] : 0u, c1 = g1 < ngroups ? gcnt[g1] : 0u;
            uint32_t incl = c0 + c1;
#pragma unroll
            for (int d = 1; d < 64; d <<= 1) {
                const uint32_t other = __shfl(incl, lane >= d ? lane - d : lane);
                if (lane >= d) incl += other;
            }
            if (lane == 63) wsum[wave] = incl;
            if (c0 > kRankGroup || c1 > kRankGroup) s_big = 1;            // benign race: every writer stores 1
            __syncthreads();
            uint32_t before = incl - (c0 + c1);
            for (int w2 = 0; w2 < wave; ++w2) before += wsum[w2];
            if (g0 < ngroups) { gstart[g0] = before; gcnt[g0] = 0; }
            if (g1 < ngroups) { gstart[g1] = before + c0; gcnt[g1] = 0; }
            __syncthreads();
        }
        if (!s_big) {
            for (uint32_t sl = wave; sl < nslices; sl += 16) {
                const size_t cell = static_cast<size_t>(q) * nslices + sl;
                const uint32_t c = count[cell];
#pragma unroll 4
                for (uint32_t t = lane; t < c; t += 64) {
                    const uint64_t key = keys[cell * cap + t];
                    const uint32_t qd = static_cast<uint32_t>(key >> 32);
                    if (qd <= T) {
                        const uint32_t g = ((qd - b0) << sub_bits) + (__umulhi(static_cast<uint32_t>(key), id_mul) >> range_shift);
                        const uint32_t pos = gstart[g] + atomicAdd(&gcnt[g], 1u);
                        if (pos < sortcap) { ids[pos] = static_cast<uint32_t>(key); grp[pos] = static_cast<uint16_t>(g); }
                    }
                }
            }
            __syncthreads();
            for (uint32_t t = tid; t < keep; t += 1024) {
                const uint32_t id = ids[t], g = grp[t];
                const uint32_t lo = gstart[g], hi = g + 1 < ngroups ? gstart[g + 1] : keep;
                // rank inside the group: ids read four at a time where they are aligned (one LDS read per four compares)
                uint32_t rank = 0, k = lo;
                for (; k < hi && (k & 3u); ++k) rank += ids[k] < id ? 1u : 0u;
                for (; k + 4 <= hi; k += 4) {
                    const uint4 v = *reinterpret_cast<const uint4 *>(ids + k);
                    rank += (v.x < id ? 1u : 0u) + (v.y < id ? 1u : 0u) + (v.z < id ? 1u : 0u) + (v.w < id ? 1u : 0u);
                }
                for (; k < hi; ++k) rank += ids[k] < id ? 1u : 0u;
                const uint32_t out = lo + rank;
                if (out < r) {
                    cand_id[static_cast<size_t>(q) * r + out] = id;
                    cand_qd[static_cast<size_t>(q) * r + out] = static_cast<uint8_t>((g >> sub_bits) + b0);
                }
            }
            if (tid == 0) flags[q] = 0;
            return;
        }
        __syncthreads();
    }
    uint64_t *a = use_lds ? reinterpret_cast<uint64_t *>(smem) : spill + static_cast<size_t>(q) * sortcap;
    uint32_t np2 = 1;
    while (np2 < keep) np2 <<= 1;
    for (uint32_t t = tid; t < np2; t += 1024) a[t] = ~0ull;
    __syncthreads();
    for (uint32_t sl = 0; sl < nslices; ++sl) {
        const size_t cell = static_cast<size_t>(q) * nslices + sl;
        const uint32_t c = count[cell];
        for (uint32_t t = tid; t < c; t += 1024) {
            const uint64_t key = keys[cell * cap + t];
            if (static_cast<uint32_t>(key >> 32) <= T) {
                const uint32_t pos = atomicAdd(&s_pos, 1u);
                if (pos < np2) a[pos] = key;
            }
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

template <int M, int QT, int WAVES, typename CodeT>
static int launch_fast_t(const CodeT *codes, uint64_t n_codes, const uint8_t *qtab, int nq, uint32_t r,
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

    // LDS above 64 KiB must be requested; the kernel addresses its tables by LDS offset and assumes that they
    // start at offset 0
    {
        const int arc = allow_dynamic_lds(reinterpret_cast<const void *>(&scan_fast_kernel<M, QT, WAVES, CodeT>), C::LDS_BYTES, true);
        if (arc) return arc;
    }

    // swizzled tables
    DCPQ_LAUNCH(kStageMisc, st, (swizzle_tables_kernel<M, QT>), dim3((C::VJ * 256 * C::NQB + 255) / 256, p.ntiles),
                dim3(256), 0, qtab, nq, qsw);
    DCPQ_CHECK_LAUNCH("swizzle_tables_kernel");
    // sample histogram -> starting bounds
    int rc = launch_sample_hist(codes, n_codes, M, qtab, nq, r, shist, p, st);
    if (rc) return rc;
    if (p.pilot) {
        if (p.s_unit != 256) return fail(DCPQ_EINVAL, "single-pass scan: the pilot pass reads runs of 256 codes");
        // The histogram covered one run in kPilotEvery of the sample.  It gives a bound for the pilot pass: the
        // bucket below which the whole sample (taken as the array, its wanted rank pilot_r as r) should hold
        // pilot_r codes with the usual slack.  The pilot pass counts every sample code at or below that bound
        // exactly, and the starting bound of the scan is the bucket where those counts reach pilot_r -- the bucket
        // a histogram of the whole sample would have given (255, and with it the redo path, if the counts never
        // get there).
        rc = launch_sample_threshold(shist, nq, p.pilot_r, p.s_count, t_cur, st);
        if (rc) return rc;
        DCPQ_LAUNCH(kStageScanHist, st, (scan_fast_kernel<M, QT, WAVES, CodeT>), dim3(p.ntiles, p.pilot_blocks), dim3(WAVES * 64),
                    C::LDS_BYTES, codes, n_codes, static_cast<uint64_t>(p.pilot_runs) * p.s_stride, p.pilot_runs * (p.s_unit / 64),
                    p.s_nunits * (p.s_unit / 64), 2u, static_cast<uint32_t>(p.s_stride), qsw, nq, p.pilot_r, p.slices, 0u, 16u, 4u,
                    t_cur, fcount, chist, fkeys);
        DCPQ_CHECK_LAUNCH("scan_fast_kernel<pilot>");
        rc = launch_sample_threshold(chist, nq, p.pilot_r, 0, t_cur, st);      // 0: the counted codes' own pilot_r-th smallest
        if (rc) return rc;
        rc = launch_zero_words(reinterpret_cast<uint32_t *>(base + p.off_fzero), p.fzero_bytes / sizeof(uint32_t), st);
        if (rc) return rc;
    } else {
        rc = launch_sample_threshold(shist, nq, r, n_codes, t_cur, st);
        if (rc) return rc;
    }
    // the scan: one contiguous stretch of codes per workgroup
    DCPQ_LAUNCH(kStageScanFast, st, (scan_fast_kernel<M, QT, WAVES, CodeT>), dim3(p.ntiles, p.fblocks), dim3(WAVES * 64),
                C::LDS_BYTES, codes, n_codes, static_cast<uint64_t>(p.codes_per_block), p.codes_per_block / 64,
                static_cast<uint32_t>((n_codes + 63) / 64), 0u, 64u, qsw, nq, r, p.slices, p.cap, p.upd, p.qflush, t_cur, fcount,
                chist, fkeys);
    DCPQ_CHECK_LAUNCH("scan_fast_kernel");
    // exact selection + list of queries to redo
    rc = launch_fast_select(fkeys, fcount, chist, nq, r, p.slices, p.cap, p.sortcap, n_codes, fsort, cand_id, cand_qd, flags, st);
    if (rc) return rc;
    DCPQ_LAUNCH(kStageSelect, st, collect_flags_kernel, dim3(1), dim3(64), 0, flags, nq, qlist, nflag);
    DCPQ_CHECK_LAUNCH("collect_flags_kernel");
    return DCPQ_OK;
}

int launch_sample_threshold(const uint32_t *shist, int nq, uint32_t r, uint64_t n_codes, int *t_cur, hipStream_t st,
                            const uint32_t *n_each)
{
    DCPQ_LAUNCH(kStageSelect, st, sample_threshold_kernel, dim3(nq), dim3(256), 0, shist, r, n_codes, n_each, t_cur);
    DCPQ_CHECK_LAUNCH("sample_threshold_kernel");
    return DCPQ_OK;
}

int launch_fast_select(const uint64_t *keys, const uint32_t *count, const uint32_t *chist, int nq, uint32_t r,
                       uint32_t nslices, uint32_t cap, uint32_t sortcap, uint64_t n_ids, uint64_t *spill, uint32_t *cand_id,
                       uint8_t *cand_qd, uint32_t *flags, hipStream_t st)
{
    {
        const int arc = allow_dynamic_lds(reinterpret_cast<const void *>(&fast_select_kernel), static_cast<int>(kSelectLdsMost));
        if (arc) return arc;
    }
    const int use_lds = sortcap <= kSortLdsKeys;
    const int rank_ok = rank_lds_bytes(sortcap) <= kSelectLdsMost;
    size_t lds = use_lds ? sizeof(uint64_t) * sortcap : 0;
    if (rank_ok && rank_lds_bytes(sortcap) > lds) lds = rank_lds_bytes(sortcap);
    // 2048 equal id ranges: high word of id * floor(2048 * 2^32 / n_ids); ids are below n_ids (2^32 when unknown)
    const uint64_t n = n_ids ? n_ids : (1ull << 32);
    const uint64_t mul64 = (2048ull << 32) / n;
    const uint32_t id_mul = mul64 > 0xFFFFFFFFull ? 0xFFFFFFFFu : static_cast<uint32_t>(mul64);
    DCPQ_LAUNCH(kStageSelect, st, fast_select_kernel, dim3(nq), dim3(1024), lds,
                keys, count, chist, r, nslices, cap, sortcap, use_lds, rank_ok, id_mul, spill, cand_id, cand_qd, flags);
    DCPQ_CHECK_LAUNCH("fast_select_kernel");
    return DCPQ_OK;
}

// Bytes of swizzled tables per query tile, 0 when the single-pass kernel does not exist for (m, qt).
size_t fast_table_bytes(int m, int qt)
{
    switch (m * 1000 + qt) {
        case 4064: return FastCfg<4, 64, 16>::TAB_BYTES;
        case 8064: return FastCfg<8, 64, 16>::TAB_BYTES;
        case 8032: return FastCfg<8, 32, 16>::TAB_BYTES;
        case 8016: return FastCfg<8, 16, 16>::TAB_BYTES;
        case 16032: return FastCfg<16, 32, 16>::TAB_BYTES;
        case 32016: return FastCfg<32, 16, 8>::TAB_BYTES;
        default: return 0;
    }
}

template <typename CodeT>
int launch_scan_fast(const CodeT *codes, uint64_t n_codes, int m, const uint8_t *qtab, int nq, uint32_t r,
                     uint32_t *cand_id, uint8_t *cand_qd, uint8_t *base, const ScanPlan &p, hipStream_t st)
{
    switch (m * 1000 + static_cast<int>(p.fqt)) {
        case 4064: return launch_fast_t<4, 64, 16, CodeT>(codes, n_codes, qtab, nq, r, cand_id, cand_qd, base, p, st);
        case 8064: return launch_fast_t<8, 64, 16, CodeT>(codes, n_codes, qtab, nq, r, cand_id, cand_qd, base, p, st);
        case 8032: return launch_fast_t<8, 32, 16, CodeT>(codes, n_codes, qtab, nq, r, cand_id, cand_qd, base, p, st);
        case 8016: return launch_fast_t<8, 16, 16, CodeT>(codes, n_codes, qtab, nq, r, cand_id, cand_qd, base, p, st);
        case 16032: return launch_fast_t<16, 32, 16, CodeT>(codes, n_codes, qtab, nq, r, cand_id, cand_qd, base, p, st);
        case 32016: return launch_fast_t<32, 16, 8, CodeT>(codes, n_codes, qtab, nq, r, cand_id, cand_qd, base, p, st);
        default: return fail(DCPQ_EUNSUPPORTED, "single-pass scan: m=%d with tiles of %u queries not supported", m, p.fqt);
    }
}

template int launch_scan_fast<uint16_t>(const uint16_t *, uint64_t, int, const uint8_t *, int, uint32_t, uint32_t *, uint8_t *,
                                        uint8_t *, const ScanPlan &, hipStream_t);
template int launch_scan_fast<uint8_t>(const uint8_t *, uint64_t, int, const uint8_t *, int, uint32_t, uint32_t *, uint8_t *,
                                       uint8_t *, const ScanPlan &, hipStream_t);

}  // namespace dcpq
