// Alg. 3 nns_derived end to end (no index): Tables -> Scan -> Refine for a batch of queries,
// in chunks so that the full 2^b-entry tables of one chunk fit the workspace.  b (bits of a sub-code,
// 16 or 8) and bbar (bits of a derived-codebook index, 1..8) are run-time parameters (the PQ m x bbar,b
// family of Sec. 3.1); sub-codes are stored in 2 bytes for b = 16 and in 1 byte for b = 8.
#include "common.h"

namespace dcpq {

struct SearchPlan {
    int chunk;
    size_t off_qtab, off_bounds, off_cand_id, off_cand_qd, off_tables, tables_bytes, off_scan, off_refine, total;
};

static SearchPlan plan_search(uint64_t n_codes, int m, int nq, uint32_t r, int full_bits, int chunk_queries)
{
    SearchPlan p{};
    int chunk = chunk_queries;
    if (chunk <= 0) {   // default: about 8 GiB of full tables per chunk (sized for a 288 GB device; the larger
                        // the chunk, the fewer launches share the scan's start-up and tail)
        const size_t per_q = sizeof(float) * (static_cast<size_t>(m) << full_bits);
        chunk = static_cast<int>((static_cast<size_t>(8) << 30) / per_q);
        if (chunk < 64) chunk = 64;
    }
    if (chunk > nq) chunk = nq;
    p.chunk = chunk;
    size_t off = 0;
    p.off_qtab = off;    off = align_up(off + static_cast<size_t>(chunk) * m * kSmallSize, 256);
    p.off_bounds = off;  off = align_up(off + sizeof(float) * 2 * static_cast<size_t>(chunk), 256);
    p.off_cand_id = off; off = align_up(off + sizeof(uint32_t) * static_cast<size_t>(chunk) * r, 256);
    p.off_cand_qd = off; off = align_up(off + static_cast<size_t>(chunk) * r, 256);
    // the full tables of a chunk (table mode), or the codebooks with their rows padded to whole 64-byte units
    // (on-demand mode with rows shorter than that; 16 floats per row), or the sub-code planes and entries of the
    // split on-demand mode (used only where they fit): the region holds the larger of the first two
    {
        const size_t tables = sizeof(float) * ((static_cast<size_t>(chunk) * m) << full_bits);
        const size_t padded = sizeof(float) * ((static_cast<size_t>(m) * 16) << full_bits);
        p.tables_bytes = tables > padded ? tables : padded;
        p.off_tables = off;  off = align_up(off + p.tables_bytes, 256);
    }
    // The scan and the refinement lay their scratch out for the number of queries they are given, and
    // a smaller batch does not always need less (fewer queries can mean more units or slices), so
    // the regions hold the larger of what a full chunk and what the ragged last chunk need: those
    // are the only two batch sizes the loop below ever passes.
    const int tail = nq % chunk;
    size_t scan_bytes = dcpq_scan_workspace_bytes(n_codes, m, chunk, r);
    size_t refine_bytes = dcpq_refine_workspace_bytes(chunk, r);
    if (tail) {
        const size_t st = dcpq_scan_workspace_bytes(n_codes, m, tail, r), rt = dcpq_refine_workspace_bytes(tail, r);
        scan_bytes = st > scan_bytes ? st : scan_bytes;
        refine_bytes = rt > refine_bytes ? rt : refine_bytes;
    }
    p.off_scan = off;    off = align_up(off + scan_bytes, 256);
    p.off_refine = off;  off = align_up(off + refine_bytes, 256);
    p.total = off;
    return p;
}

}  // namespace dcpq

using namespace dcpq;

extern "C" int dcpq_search_bits_chunk(int m, int nq, int b, int chunk_queries)
{
    if (nq <= 0 || !m_supported(m) || !dcpq_bits_supported(b, 1)) return 0;
    return plan_search(1, m, nq, 1, b, chunk_queries).chunk;
}

extern "C" int dcpq_search_chunk(int m, int nq, int chunk_queries) { return dcpq_search_bits_chunk(m, nq, kFullBits, chunk_queries); }

extern "C" size_t dcpq_search_bits_workspace_bytes(uint64_t n_codes, int m, int nq, uint32_t r, int b, int chunk_queries)
{
    if (nq <= 0 || !m_supported(m) || n_codes == 0 || r == 0 || r > (1u << 26) || !dcpq_bits_supported(b, 1)) return 0;
    return plan_search(n_codes, m, nq, r, b, chunk_queries).total;
}

extern "C" size_t dcpq_search_workspace_bytes(uint64_t n_codes, int m, int nq, uint32_t r, int chunk_queries)
{
    return dcpq_search_bits_workspace_bytes(n_codes, m, nq, r, kFullBits, chunk_queries);
}

// How pass two gets its table entries: looked up in full tables built first (DCPQ_REFINE_TABLES), or computed
// on demand, in one kernel (DCPQ_REFINE_DIRECT) or split by sub-quantizer (DCPQ_REFINE_SPLIT).  On demand a
// query gathers r m centroid rows; with tables it writes 2^b m entries and then makes r m scattered 4-byte
// lookups.  Measured on MI355X a gathered row costs about 8 ps more than a table lookup (27 against 19 ps for
// random 16-bit sub-codes, dsub = 12) and a 2^16-entry table 60 to 200 ns to build (dsub = 12 to 60), which
// puts the break-even near r = 8000 for b = 16; the rule below scales that with the table size.
// The split form pays when the sub-codebooks that one XCD would serve (one in eight of them) fit its 4 MB
// cache with room to spare while the codebooks as a whole do not (measured at m = 8, dsub = 12, r = 4000:
// 2.9 times faster with 64 queries, 2.2 times with 4096; with rows of exactly 4 MB per sub-quantizer and
// codes that follow the queries, 1.4 times slower), and the batch is not tiny; it is possible when its
// intermediate arrays fit the table region and candidate numbers 32 bits.
static bool split_possible(const SearchPlan &p, int m, int b, int nq, uint32_t r, const float *queries)
{
    // (its kernels read query sub-vectors 16 bytes at a time from where the caller keeps them)
    return static_cast<uint64_t>(nq) * r < (1ull << 32) && refine_split_bytes(nq, r, m, b / 8) <= p.tables_bytes &&
           (reinterpret_cast<uintptr_t>(queries) & 15) == 0;
}

static bool split_pays(int m, int dsub, int b, int nq, uint32_t r)
{
    const size_t sub = (sizeof(float) * static_cast<size_t>(dsub)) << b;
    return sub * ((m + 7) / 8) < (4u << 20) && sub * m > (4u << 20) && static_cast<uint64_t>(nq) * r >= (1u << 16);
}

static int refine_mode_for(int requested, const SearchPlan &p, int m, int dsub, int b, int nq, uint32_t r, const float *queries)
{
    if (requested != DCPQ_REFINE_AUTO) return requested;
    if (r > (1u << b) / 8) return DCPQ_REFINE_TABLES;
    return split_possible(p, m, b, nq, r, queries) && split_pays(m, dsub, b, nq, r) ? DCPQ_REFINE_SPLIT : DCPQ_REFINE_DIRECT;
}

extern "C" int dcpq_search_bits(const float *queries, int nq, const float *codebooks, const float *derived, int m,
                                int dsub, int b, int bbar, const void *codes, uint64_t n_codes, uint32_t r, uint32_t k,
                                int refine_mode, uint32_t *ids, float *dist, int chunk_queries, void *workspace,
                                size_t workspace_bytes, void *stream)
{
    clear_error();
    DCPQ_REQUIRE(nq >= 0, "search: nq=%d", nq);
    if (!dcpq_shape_supported(m, dsub)) return fail(DCPQ_EUNSUPPORTED, "search: m=%d dsub=%d not supported", m, dsub);
    if (!dcpq_bits_supported(b, bbar)) return fail(DCPQ_EUNSUPPORTED, "search: b=%d bbar=%d not supported", b, bbar);
    DCPQ_REQUIRE(n_codes >= 1 && n_codes < (1ull << 32), "search: n_codes out of range");
    DCPQ_REQUIRE(r >= 1 && r <= n_codes && k >= 1 && k <= r, "search: needs 1 <= k <= r <= n_codes");
    DCPQ_REQUIRE(r <= (1u << 26), "search: r=%u above the supported 2^26", r);
    DCPQ_REQUIRE(refine_mode == DCPQ_REFINE_AUTO || refine_mode == DCPQ_REFINE_TABLES || refine_mode == DCPQ_REFINE_DIRECT ||
                     refine_mode == DCPQ_REFINE_SPLIT,
                 "search: refine_mode=%d", refine_mode);
    if (nq == 0) return DCPQ_OK;
    DCPQ_REQUIRE(queries && codebooks && derived && codes && ids && dist && workspace, "search: null pointer");
    DCPQ_REQUIRE((reinterpret_cast<uintptr_t>(codebooks) & 15) == 0, "search: codebooks must be 16-byte aligned");
    DCPQ_REQUIRE((reinterpret_cast<uintptr_t>(workspace) & 255) == 0, "search: workspace must be 256-byte aligned");
    DCPQ_REQUIRE((reinterpret_cast<uintptr_t>(codes) & 15) == 0, "search: codes must be 16-byte aligned");
    const SearchPlan p = plan_search(n_codes, m, nq, r, b, chunk_queries);
    if (workspace_bytes < p.total)
        return fail(DCPQ_EWORKSPACE, "search: workspace %zu < %zu bytes", workspace_bytes, p.total);
    uint8_t *base = static_cast<uint8_t *>(workspace);
    uint8_t *qtab = base + p.off_qtab;
    float *bounds = reinterpret_cast<float *>(base + p.off_bounds);
    uint32_t *cand_id = reinterpret_cast<uint32_t *>(base + p.off_cand_id);
    uint8_t *cand_qd = base + p.off_cand_qd;
    float *tables = reinterpret_cast<float *>(base + p.off_tables);
    hipStream_t st = as_stream(stream);
    const int D = m * dsub;
    const int code_bytes = b / 8;
    const int tail = nq % p.chunk;
    const int mode_full = refine_mode_for(refine_mode, p, m, dsub, b, p.chunk, r, queries);
    const int mode_tail = tail ? refine_mode_for(refine_mode, p, m, dsub, b, tail, r, queries) : mode_full;
    if (mode_full == DCPQ_REFINE_SPLIT && !split_possible(p, m, b, p.chunk, r, queries))
        return fail(DCPQ_EINVAL, "search: DCPQ_REFINE_SPLIT: %zu bytes of sub-codes and entries per chunk do not fit the table "
                                 "region (%zu bytes), or chunk * r reaches 2^32, or the queries are not 16-byte aligned",
                    refine_split_bytes(p.chunk, r, m, b / 8), p.tables_bytes);
    const bool any_split = mode_full == DCPQ_REFINE_SPLIT || mode_tail == DCPQ_REFINE_SPLIT;
    const bool any_direct = mode_full == DCPQ_REFINE_DIRECT || mode_tail == DCPQ_REFINE_DIRECT;
    // On demand in one kernel, a candidate gathers m centroid rows; a row shorter than a 64-byte unit that does not divide it
    // lies across two memory lines more often than it has to, so such codebooks are copied once per call into
    // rows of 16 floats (25 -> 33 MB at m = 8, dsub = 12: 30 microseconds, 6 % off the refinement).  Longer rows
    // gain nothing and the copy costs more (measured at dsub = 60), so they are read in place.
    const float *rows = codebooks;
    int cstride = dsub;
    // (the split form reads the codebooks in place and uses the region for its own arrays: no copy then)
    if (any_direct && !any_split && dsub < 16 && 16 % dsub != 0) {
        cstride = 16;
        int rc = launch_pad_rows(codebooks, static_cast<size_t>(m) << b, dsub, cstride, tables, st);
        if (rc) return rc;
        rows = tables;
    }
    for (int q0 = 0; q0 < nq; q0 += p.chunk) {
        const int nc = (nq - q0 < p.chunk) ? nq - q0 : p.chunk;
        const float *y = queries + static_cast<size_t>(q0) * D;
        int rc = launch_small_tables(y, nc, derived, m, dsub, bbar, codes, code_bytes, n_codes, r, qtab, bounds, nullptr, st);
        if (rc) return rc;
        // the quantized tables have 256 entries whatever bbar is, and 1-byte sub-codes are their own low-byte plane
        if (code_bytes == 1)
            rc = launch_scan(static_cast<const uint8_t *>(codes), n_codes, m, qtab, nc, r, cand_id, cand_qd, base + p.off_scan,
                             DCPQ_SCAN_AUTO, st);
        else
            rc = launch_scan(static_cast<const uint16_t *>(codes), n_codes, m, qtab, nc, r, cand_id, cand_qd,
                             base + p.off_scan, DCPQ_SCAN_AUTO, st);
        if (rc) return rc;
        uint32_t *ids_c = ids + static_cast<size_t>(q0) * k;
        float *dist_c = dist + static_cast<size_t>(q0) * k;
        const int mode = nc == p.chunk ? mode_full : mode_tail;
        if (mode == DCPQ_REFINE_SPLIT) {
            rc = launch_refine_split(y, codebooks, dsub, 1u << b, codes, code_bytes, n_codes, m, cand_id, nc, r, k, ids_c, dist_c,
                                     tables, base + p.off_refine, st);
        } else if (mode == DCPQ_REFINE_DIRECT) {
            rc = launch_refine_direct(y, rows, dsub, cstride, 1u << b, codes, code_bytes, n_codes, m, cand_id, nc, r, k, ids_c,
                                      dist_c, base + p.off_refine, st);
        } else {
            rc = launch_distance_tables(y, nc, codebooks, m, dsub, 1 << b, tables, kStageFullTables, st);
            if (rc) return rc;
            rc = launch_refine(tables, 1u << b, codes, code_bytes, n_codes, m, cand_id, nc, r, k, ids_c, dist_c,
                               base + p.off_refine, st);
        }
        if (rc) return rc;
    }
    return DCPQ_OK;
}

extern "C" int dcpq_search(const float *queries, int nq, const float *codebooks, const float *derived, int m,
                           int dsub, const uint16_t *codes, uint64_t n_codes, uint32_t r, uint32_t k,
                           uint32_t *ids, float *dist, int chunk_queries, void *workspace,
                           size_t workspace_bytes, void *stream)
{
    return dcpq_search_bits(queries, nq, codebooks, derived, m, dsub, kFullBits, kSmallBits, codes, n_codes, r, k,
                            DCPQ_REFINE_AUTO, ids, dist, chunk_queries, workspace, workspace_bytes, stream);
}

extern "C" int dcpq_search_refine_mode(int m, int dsub, int b, int nq, uint32_t r, int refine_mode)
{
    if (nq <= 0 || !m_supported(m) || !dcpq_bits_supported(b, 1) || r == 0) return refine_mode;
    const SearchPlan p = plan_search(1, m, nq, r, b, 0);
    return refine_mode_for(refine_mode, p, m, dsub, b, p.chunk, r, nullptr);
}
