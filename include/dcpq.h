/*
 * dcpq.h -- C ABI of libdcpq: two-pass product-quantization nearest-neighbour search with derived
 * codebooks ("Derived Codebooks for High-Accuracy Nearest Neighbor Search", Alg. 3), hand-written
 * HIP for gfx950 (MI355X).
 *
 * Letters: m sub-quantizers of b = 16 bits (2^16 centroids of dsub floats each); derived codebooks
 * of bbar = 8 bits (2^8 centroids) indexed by the LOW 8 bits of a sub-code (Sec. 3.2, property
 * P1); r = size of the candidate set kept by pass one (the paper's r2); k = size of the result set
 * (the paper's r); D = m * dsub.
 *
 * Conventions for every call
 *   - All array arguments are DEVICE pointers owned by the caller, row-major and contiguous, unless
 *     a parameter is documented as "host".  The library never allocates, frees or retains them.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls only enqueue
 *     work on that stream and never synchronise; outputs are valid once the stream has drained.
 *   - Scratch memory is a caller-provided device workspace of at least the number of bytes the
 *     matching *_workspace_bytes call returns; its contents on entry do not matter, and two calls
 *     that share a workspace must not overlap in time.
 *   - Return value: DCPQ_OK or an error code; dcpq_last_error() then holds a message (thread
 *     local).  Arguments are validated on the host before anything is launched: on DCPQ_EINVAL,
 *     DCPQ_EWORKSPACE or DCPQ_EUNSUPPORTED nothing has been enqueued.  DCPQ_EHIP (a launch the
 *     runtime refused) can come from any kernel of a call, after earlier ones were enqueued; the
 *     outputs are then undefined.
 *   - Ties are always broken by the smaller vector id.  Ids are 32-bit: N < 2^32.
 */
#ifndef DCPQ_H
#define DCPQ_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define DCPQ_OK 0
#define DCPQ_EINVAL 1        /* bad argument (null pointer, size out of range, k > r, r > N, ...) */
#define DCPQ_EWORKSPACE 2    /* workspace smaller than *_workspace_bytes */
#define DCPQ_EHIP 3          /* a HIP runtime call failed */
#define DCPQ_EUNSUPPORTED 4  /* shape outside what the kernels are built for */

#define DCPQ_PAD_ID 0xFFFFFFFFu /* id written into unused output slots (IVF variant only) */

/* Message of the last error on this thread ("" if none). */
const char *dcpq_last_error(void);

/* Library ABI version (bumped when a signature changes). */
int dcpq_version(void);

/* Shapes the kernels accept: m in {1,2,4,8,16,32}, 1 <= dsub <= 128.  Returns 1 / 0. */
int dcpq_shape_supported(int m, int dsub);

/* ---------------------------------------------------------------------------------------------
 * derive_codebooks -- Sec. 3.2 (Step 2 and property P1).
 * derived[j][l][:] = mean of the 256 centroids codebooks[j][(i << 8) | l][:], i = 0..255, in
 * fp32, added in increasing i and divided once by 256 (bit-reproducible).
 *   codebooks : const float [m][65536][dsub]      derived : float [m][256][dsub]   (output)
 * Done once per index, not per query.
 * ------------------------------------------------------------------------------------------- */
int dcpq_derive_codebooks(const float *codebooks, int m, int dsub, float *derived, void *stream);

/* ---------------------------------------------------------------------------------------------
 * build_small_tables -- Sec. 3.3 "Tables step": small lookup tables from the derived codebooks
 * (Eq. 1), the qmin / qmax bounds, and the 8-bit quantized tables Q_j.
 *   small[q][j][i] = sum_t (y_q[j*dsub+t] - derived[j][i][t])^2, fp32, t increasing, unfused.
 *   qmin[q] = min over all m*256 entries; qmax[q] = max over the first min(r, n_codes) codes of
 *   the fp32 sum over j (increasing) of small[q][j][code[j] & 255].
 *   qtab[q][j][i] = 255 if (small - qmin) / (qmax - qmin) * 255 >= 255, else its floor; all zero
 *   when qmax <= qmin.
 *   queries : const float [nq][D]          derived : const float [m][256][dsub]
 *   codes   : const uint16_t [n_codes][m]  (only the first min(r, n_codes) rows are read)
 *   qtab    : uint8_t [nq][m][256] (output)   bounds : float [nq][2] = (qmin, qmax) (output)
 *   small   : float [nq][m][256] (output) or NULL
 * Needs no workspace.
 * ------------------------------------------------------------------------------------------- */
int dcpq_build_small_tables(const float *queries, int nq, const float *derived, int m, int dsub,
                            const uint16_t *codes, uint64_t n_codes, uint32_t r, uint8_t *qtab,
                            float *bounds, float *small, void *stream);

/* ---------------------------------------------------------------------------------------------
 * build_tables -- Eq. 1 with the full 16-bit codebooks ("Tables step" of Alg. 1), batched over
 * queries as a matrix product on the matrix cores (double-precision accumulate, one rounding to
 * fp32 on output).
 *   tables[q][j][i] = || y_q^j - codebooks[j][i] ||^2
 *   queries : const float [nq][D]   codebooks : const float [m][65536][dsub]
 *   tables  : float [nq][m][65536] (output; nq * m * 256 KiB)
 * Needs no workspace.
 * ------------------------------------------------------------------------------------------- */
int dcpq_build_tables(const float *queries, int nq, const float *codebooks, int m, int dsub,
                      float *tables, void *stream);
/* The same for codebooks of any size (n_entries centroids per sub-quantizer, e.g. the 256 of an 8-bit
 * product quantizer):  codebooks : const float [m][n_entries][dsub]   tables : float [nq][m][n_entries] */
int dcpq_build_tables_n(const float *queries, int nq, const float *codebooks, int m, int dsub, int n_entries,
                        float *tables, void *stream);


/* ---------------------------------------------------------------------------------------------
 * scan_candidates -- Sec. 3.3 "Scan step" (Alg. 3 scan / adc_low_bits, capped buckets).
 * For every query q and code i: qd = min(255, sum_j qtab[q][j][codes[i][j] & 255]); the candidate
 * set is exactly the r smallest by (qd, i), written in that order.
 *   codes   : const uint16_t [n_codes][m]     qtab : const uint8_t [nq][m][256]
 *   cand_id : uint32_t [nq][r] (output)       cand_qd : uint8_t [nq][r] (output)
 *   workspace : at least dcpq_scan_workspace_bytes(n_codes, m, nq, r) bytes, 256-byte aligned
 * Requires 1 <= r <= n_codes < 2^32; codes and qtab 16-byte aligned.
 * ------------------------------------------------------------------------------------------- */
size_t dcpq_scan_workspace_bytes(uint64_t n_codes, int m, int nq, uint32_t r);
/* Queries that share one pass over the codes inside the scan kernels for a large batch (their tables
 * sit in LDS). */
int dcpq_scan_query_tile(int m);
/* How scan_candidates(_mode) lays out its work for a problem, for benchmarks and reports (host only, no
 * device work).  info (host pointer, ninfo >= 6) receives: [0] queries per tile, [1] number of tiles,
 * [2] workgroups along the codes in the single-pass launch, [3] codes per workgroup (for the three-pass
 * algorithm: codes per wavefront unit), [4] slices of a query's candidate buffer, [5] entries per slice.
 * [2], [4], [5] are 0 for the three-pass algorithm.  With ninfo >= 10 also the sample that gives the
 * single-pass scan its starting bounds: [6] runs of 256 codes, [7] codes between the starts of two runs,
 * [8] 16 when the histogram pass reads one run in 16 and the single-pass kernel counts the whole sample
 * below the bound that gives (the pilot pass, large arrays), 1 when the histogram pass reads every run,
 * [9] the rank wanted within the sample (all 0 for the three-pass algorithm). */
int dcpq_scan_plan(uint64_t n_codes, int m, int nq, uint32_t r, int mode, uint64_t *info, int ninfo);
int dcpq_scan_candidates(const uint16_t *codes, uint64_t n_codes, int m, const uint8_t *qtab, int nq,
                         uint32_t r, uint32_t *cand_id, uint8_t *cand_qd, void *workspace,
                         size_t workspace_bytes, void *stream);
/* Same call with the algorithm chosen by the caller (same outputs either way):
 *   DCPQ_SCAN_AUTO        single pass over the codes with a running bucket bound (the paper's
 *                         capped-buckets upper bound); queries whose candidate buffer overflows are
 *                         redone by the three-pass algorithm.  m = 1, 2 always use three passes.
 *   DCPQ_SCAN_THREE_PASS  histogram pass, tie-count pass, collect pass: exact for any input.
 *   DCPQ_SCAN_TILE16/32/64  the single pass with tiles of 16, 32 or 64 queries sharing one pass over the
 *                         codes (AUTO takes the largest tile the kernel has for m, and for m = 8 the
 *                         smallest of 16, 32, 64 that holds the whole batch); DCPQ_EUNSUPPORTED when the
 *                         kernel does not exist for (m, tile).  Tiles: m = 4: 64; m = 8: 16, 32, 64;
 *                         m = 16: 32; m = 32: 16. */
#define DCPQ_SCAN_AUTO 0
#define DCPQ_SCAN_THREE_PASS 1
#define DCPQ_SCAN_TILE16 2
#define DCPQ_SCAN_TILE32 3
#define DCPQ_SCAN_TILE64 4
int dcpq_scan_candidates_mode(const uint16_t *codes, uint64_t n_codes, int m, const uint8_t *qtab, int nq,
                              uint32_t r, uint32_t *cand_id, uint8_t *cand_qd, void *workspace,
                              size_t workspace_bytes, int mode, void *stream);

/* The same scan reading the low-byte plane of the codes (dcpq_pack_low_bytes: uint8_t [n_codes][m], the
 * only bytes pass one consumes, Sec. 3.3 adc_low_bits) instead of the codes: half the bytes per code
 * and pass.  Same outputs; `mode` as in dcpq_scan_candidates_mode. */
int dcpq_scan_candidates_packed(const uint8_t *plane, uint64_t n_codes, int m, const uint8_t *qtab, int nq,
                                uint32_t r, uint32_t *cand_id, uint8_t *cand_qd, void *workspace,
                                size_t workspace_bytes, int mode, void *stream);

/* The same scan for callers that cannot allocate (code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc) and have no workspace to pass: the scratch memory is an array
 * inside the library, DCPQ_STATIC_SCRATCH_BYTES per GPU, held from the first call on that GPU until
 * the process ends.  Inputs, outputs, order and error behaviour as dcpq_scan_candidates; the call
 * itself allocates nothing.  A problem whose dcpq_scan_workspace_bytes exceeds
 * dcpq_static_scratch_bytes() is refused with DCPQ_EWORKSPACE before anything is launched.  All
 * calls on one GPU share the one array: two of them must not overlap in time (they would race),
 * whichever streams they use. */
#define DCPQ_STATIC_SCRATCH_BYTES (64u << 20)
size_t dcpq_static_scratch_bytes(void);
int dcpq_scan_candidates_static(const uint16_t *codes, uint64_t n_codes, int m, const uint8_t *qtab, int nq,
                                uint32_t r, uint32_t *cand_id, uint8_t *cand_qd, void *stream);

/* ---------------------------------------------------------------------------------------------
 * refine_topk -- Sec. 3.3 "Refine step" (Alg. 3 refine / adc_refine, Eq. 2): exact re-ranking of
 * the candidates with the full tables, then the k best.
 *   d(q, i) = sum over j increasing of tables[q][j][codes[i][j]] (fp32 adds)
 *   ids[q][:], dist[q][:] = the k smallest by (d, i), ascending.
 *   tables : const float [nq][m][65536]   codes : const uint16_t [n_codes][m]
 *   cand_id : const uint32_t [nq][r]      ids : uint32_t [nq][k]   dist : float [nq][k] (outputs)
 *   workspace : at least dcpq_refine_workspace_bytes(nq, r) bytes
 * Requires 1 <= k <= r.
 * ------------------------------------------------------------------------------------------- */
size_t dcpq_refine_workspace_bytes(int nq, uint32_t r);
int dcpq_refine_topk(const float *tables, const uint16_t *codes, uint64_t n_codes, int m,
                     const uint32_t *cand_id, int nq, uint32_t r, uint32_t k, uint32_t *ids,
                     float *dist, void *workspace, size_t workspace_bytes, void *stream);

/* ---------------------------------------------------------------------------------------------
 * search -- Alg. 3 nns_derived end to end for a batch of queries without an index: small tables,
 * quantization, scan, full tables, refine, top-k.  Queries are processed in chunks of
 * `chunk_queries` (0 = library default) so that the full tables of one chunk live in the
 * workspace.
 *   derived : const float [m][256][dsub] from dcpq_derive_codebooks
 *   workspace : at least dcpq_search_workspace_bytes(...) bytes
 * ------------------------------------------------------------------------------------------- */
size_t dcpq_search_workspace_bytes(uint64_t n_codes, int m, int nq, uint32_t r, int chunk_queries);
/* Queries per chunk dcpq_search will use for this shape (chunk_queries = 0: the default). */
int dcpq_search_chunk(int m, int nq, int chunk_queries);
int dcpq_search(const float *queries, int nq, const float *codebooks, const float *derived, int m,
                int dsub, const uint16_t *codes, uint64_t n_codes, uint32_t r, uint32_t k,
                uint32_t *ids, float *dist, int chunk_queries, void *workspace,
                size_t workspace_bytes, void *stream);

/* ---------------------------------------------------------------------------------------------
 * The PQ m x bbar,b family (Sec. 3.1 notation; Sec. 6 names 4-, 5- and 6-bit derived codebooks for an
 * 8-bit quantizer as the next step): the same stages with the two bit widths as arguments.
 *   b    : bits of a sub-code, 16 (sub-codes stored as uint16) or 8 (stored as uint8); 2^b centroids
 *   bbar : bits of a derived-codebook index, 1 <= bbar <= 8, bbar <= b; derived centroid l is the
 *          mean of the 2^(b-bbar) centroids whose index has low bits l (sum in increasing index
 *          order, one division), and a sub-code's derived code is its low bbar bits (P1).
 * The calls above are these with b = 16, bbar = 8.  Layouts as above with 65536 -> 2^b and, for
 * `derived` and `small`, 256 -> 2^bbar.  The QUANTIZED tables keep 256 entries per sub-quantizer
 * for every bbar:  qtab[q][j][e] = quantized distance to derived centroid (e mod 2^bbar),  so the
 * scan calls (which look up by the low byte of a sub-code) serve every bbar unchanged:
 *   b = 16: dcpq_scan_candidates(codes, ...);   b = 8: dcpq_scan_candidates_packed(codes, ...)
 *   (1-byte sub-codes are their own low-byte plane).  Full tables: dcpq_build_tables_n with
 *   n_entries = 2^b.  dcpq_refine_topk_bits needs n_entries = 2^(8 code_bytes).
 * Unsupported widths -> DCPQ_EUNSUPPORTED.
 * ------------------------------------------------------------------------------------------- */
int dcpq_bits_supported(int b, int bbar);
int dcpq_derive_codebooks_bits(const float *codebooks, int m, int dsub, int b, int bbar, float *derived,
                               void *stream);
int dcpq_build_small_tables_bits(const float *queries, int nq, const float *derived, int m, int dsub,
                                 int bbar, const void *codes, int code_bytes, uint64_t n_codes, uint32_t r,
                                 uint8_t *qtab, float *bounds, float *small, void *stream);
int dcpq_refine_topk_bits(const float *tables, uint32_t n_entries, const void *codes, int code_bytes,
                          uint64_t n_codes, int m, const uint32_t *cand_id, int nq, uint32_t r, uint32_t k,
                          uint32_t *ids, float *dist, void *workspace, size_t workspace_bytes, void *stream);
size_t dcpq_search_bits_workspace_bytes(uint64_t n_codes, int m, int nq, uint32_t r, int b, int chunk_queries);
int dcpq_search_bits_chunk(int m, int nq, int b, int chunk_queries);
/* refine_mode: how pass two gets its table entries (Sec. 3.3, Refine step: the entries of the full
 * tables are computed on demand, since a query uses a small part of them).
 *   DCPQ_REFINE_TABLES  build the full tables of the chunk first, then look entries up
 *   DCPQ_REFINE_DIRECT  compute every entry a candidate needs from the codebooks (fp64, rounded to
 *                       fp32 once: the value the tables would hold, up to the last bit); no tables
 *   DCPQ_REFINE_SPLIT   the same entries, bit for bit, computed in three kernels split by sub-quantizer
 *                       so that each of the 8 second-level caches keeps serving one sub-codebook;
 *                       its two intermediate arrays, chunk * r * m * (4 + b / 8) bytes, live in the
 *                       region of the workspace that the tables would take: they fit whenever
 *                       r * (4 + b / 8) <= 4 * 2^b; DCPQ_EINVAL if they do not, if chunk * r
 *                       reaches 2^32, or if `queries` is not 16-byte aligned
 *   DCPQ_REFINE_AUTO    TABLES when r > 2^b / 8; else SPLIT when it is possible, a sub-codebook (two
 *                       for m = 16, four for m = 32) is smaller than 4 MB, the codebooks as a whole
 *                       are not, and the chunk has at least 2^16 candidates; else DIRECT (dcpq_search
 *                       uses this).
 *                       dcpq_search_refine_mode reports the choice for the first chunk of a batch of
 *                       nq queries under the default chunking
 * All give the fp32 sum, j increasing, of the M entries; TABLES and the on-demand modes agree within
 * the 1e-5 bar and may differ in the last bit (and then in the order of near-ties). */
#define DCPQ_REFINE_AUTO 0
#define DCPQ_REFINE_TABLES 1
#define DCPQ_REFINE_DIRECT 2
#define DCPQ_REFINE_SPLIT 3
int dcpq_search_refine_mode(int m, int dsub, int b, int nq, uint32_t r, int refine_mode);
int dcpq_search_bits(const float *queries, int nq, const float *codebooks, const float *derived, int m,
                     int dsub, int b, int bbar, const void *codes, uint64_t n_codes, uint32_t r, uint32_t k,
                     int refine_mode, uint32_t *ids, float *dist, int chunk_queries, void *workspace,
                     size_t workspace_bytes, void *stream);
/* Pass two on its own with on-demand entries:  queries [nq][m*dsub], codebooks [m][2^b][dsub] (16-byte
 * aligned), codes of b/8 bytes per sub-code; otherwise as dcpq_refine_topk. */
int dcpq_refine_direct_topk(const float *queries, const float *codebooks, int m, int dsub, int b,
                            const void *codes, uint64_t n_codes, const uint32_t *cand_id, int nq, uint32_t r,
                            uint32_t k, uint32_t *ids, float *dist, void *workspace, size_t workspace_bytes,
                            void *stream);

/* ---------------------------------------------------------------------------------------------
 * plain_search -- Alg. 1 (Sec. 2.3): the conventional single-pass search the paper compares with:
 * asymmetric distance of EVERY code from the full floating-point tables (Eq. 2), no derived
 * codebooks, no candidate set:
 *   d(q, i) = sum over j increasing of tables[q][j][codes[i][j]] (fp32 adds)
 *   ids[q][:], dist[q][:] = the k smallest by (d, i), ascending.
 * With n_entries = 65536 and 2-byte sub-codes this is "plain 16-bit" PQ (tables from
 * dcpq_build_tables), with n_entries = 256 and 1-byte sub-codes "plain 8-bit" PQ (tables from
 * dcpq_build_tables_n on an 8-bit codebook).  A comparison system: exact, not tuned.
 *   tables : const float [nq][m][n_entries]   codes : [n_codes][m] sub-codes of code_bytes (1 or 2) each
 *   workspace : dcpq_plain_workspace_bytes(n_codes, nq, k), 256-byte aligned.  1 <= k <= 768.
 * ------------------------------------------------------------------------------------------- */
size_t dcpq_plain_workspace_bytes(uint64_t n_codes, int nq, uint32_t k);
int dcpq_plain_search(const float *tables, uint32_t n_entries, const void *codes, int code_bytes,
                      uint64_t n_codes, int m, int nq, uint32_t k, uint32_t *ids, float *dist,
                      void *workspace, size_t workspace_bytes, void *stream);

/* ---------------------------------------------------------------------------------------------
 * Training and encoding -- Sec. 3.2, Alg. 2 (build_quantizers) and the encoding rule of the last
 * paragraph of Sec. 3.2.  The paper names the steps and leaves their insides to standard algorithms;
 * what these calls compute:
 *   nearest centroid    the smallest (squared distance, index), distances in double precision from
 *                       the fp32 inputs (matrix cores);
 *   k-means (step 1)    `iters` times { assign every point; centroid = mean of its members, double
 *                       precision sums rounded to fp32 once; a centroid without members keeps its
 *                       value }, then one more assignment; the initial centroids are an input;
 *   same-size k-means   (step 2) `iters` times { balanced assignment into groups of exactly n / kbar
 *                       points; means }; the labels are those of the last assignment, whose means
 *                       the centroids are.  Balanced assignment, in rounds: every point without a
 *                       group proposes to the group with the smallest (distance, index) among those
 *                       with room, every group keeps the proposers with the smallest (distance,
 *                       point) up to its room, until no point is left; distances as fp32;
 *   final codebook      (step 3) the members of group l in increasing temporary index get the final
 *                       indices (0 << bbar) | l, (1 << bbar) | l, ...  (property P1).
 * dcpq_kmeans_same_size (and dcpq_build_quantizers, which calls it) reads a counter back after every
 * round and so SYNCHRONIZES the stream; the other calls only enqueue.  Workspaces 256-byte aligned.
 *
 *   dcpq_assign   points: n rows of ld floats, sub-vector j in columns j*dsub .. (j+1)*dsub-1;
 *                 codebooks [m][n_entries][dsub]; labels [n][m] of label_bytes (1, 2 or 4) each;
 *                 dist (NULL or float [n][m]): squared distance to the chosen centroid.
 *   dcpq_encode   = dcpq_assign on [n][m*dsub] vectors with 2^b centroids, codes of b/8 bytes per sub-code.
 *   dcpq_kmeans   points as above with one sub-vector (ld >= d); centroids float [k][d] in/out; labels uint32 [n].
 *   dcpq_kmeans_same_size   points float [n][d] (the temporary codebook), n a multiple of kbar <= 256;
 *                 centroids float [kbar][d] in/out; labels uint32 [n].
 *   dcpq_build_final_codebook   temp/final float [k][d] (distinct), labels uint32 [k] with groups of equal
 *                 size (not checked), perm uint32 [k]: perm[final index] = temporary index.
 *   dcpq_build_quantizers   all of Alg. 2 for m sub-quantizers: train float [n_train][m*dsub]; codebooks
 *                 float [m][2^b][dsub] hold the INITIAL centroids on entry and the final codebooks on
 *                 return; step 2 starts from the first 2^bbar temporary centroids; derived float
 *                 [m][2^bbar][dsub] = dcpq_derive_codebooks_bits of the result.
 * ------------------------------------------------------------------------------------------- */
int dcpq_assign(const float *points, uint64_t n, int ld, const float *codebooks, int m, int dsub, int n_entries,
                void *labels, int label_bytes, float *dist, void *stream);
int dcpq_encode(const float *vectors, uint64_t n, const float *codebooks, int m, int dsub, int b, void *codes,
                void *stream);
size_t dcpq_kmeans_workspace_bytes(int k, int d);
int dcpq_kmeans(const float *points, uint64_t n, int ld, int d, int k, int iters, float *centroids,
                uint32_t *labels, void *workspace, size_t workspace_bytes, void *stream);
size_t dcpq_kmeans_same_size_workspace_bytes(int n, int d, int kbar);
int dcpq_kmeans_same_size(const float *points, int n, int d, int kbar, int iters, float *centroids,
                          uint32_t *labels, void *workspace, size_t workspace_bytes, void *stream);
int dcpq_build_final_codebook(const float *temp_codebook, int k, int d, const uint32_t *labels, int bbar,
                              float *final_codebook, uint32_t *perm, void *stream);
size_t dcpq_build_quantizers_workspace_bytes(uint64_t n_train, int dsub, int b, int bbar);
int dcpq_build_quantizers(const float *train, uint64_t n_train, int m, int dsub, int b, int bbar, int iters,
                          int iters_same_size, float *codebooks, float *derived, void *workspace,
                          size_t workspace_bytes, void *stream);

/* =============================================================================================
 * Inverted-index variant (Sec. 2.2: inverted lists with residual encoding; Sec. 2.3: the Index step,
 * and every later step done once per probed list; Sec. 3.3 with derived codebooks).
 *
 * Layout: nlist cells with centres coarse[nlist][D]; list l holds the codes at positions
 * offsets[l] .. offsets[l+1]-1 of the code array (offsets: int64 [nlist+1], increasing, last one =
 * number of codes < 2^32); a vector's id is its position in the code array; codes quantize the
 * residual x - coarse[l].  nprobe (the paper's ma) lists are scanned per query, nprobe <= 512, and
 * the lists named in one row of `probe` must be distinct.
 * ============================================================================================= */

/* Index step: probe[q][:] = the nprobe cells with the smallest || y_q - coarse[l] ||^2 (matrix
 * cores, double-precision accumulate, compared after rounding to fp32), ordered by (distance, l).
 *   probe : int32_t [nq][nprobe] (output)   workspace : dcpq_ivf_probe_workspace_bytes(nq, nlist) */
size_t dcpq_ivf_probe_workspace_bytes(int nq, int nlist);
int dcpq_ivf_probe(const float *queries, int nq, int D, const float *coarse, int nlist, int nprobe,
                   int32_t *probe, void *workspace, size_t workspace_bytes, void *stream);

/* Tables step: for every query q and probed list p, the residual rho = y_q - coarse[probe[q][p]]
 * (fp32), its small tables on the derived codebooks (as in dcpq_build_small_tables), and their
 * 8-bit quantization with ONE pair of bounds per query: qmin = smallest entry over all nprobe
 * tables of the query; qmax = largest small-table distance over the first min(r, total) codes met
 * when walking the probed lists in probe order, each code against its own list's tables.  If the
 * probed lists are empty the bounds are (0, 0) and the tables all zero.
 *   qtab : uint8_t [nq][nprobe][m][256] (output)   bounds : float [nq][2] (output)
 *   workspace : dcpq_ivf_tables_workspace_bytes(nq) */
size_t dcpq_ivf_tables_workspace_bytes(int nq);
/* Optional: with at least this much workspace dcpq_ivf_build_small_tables keeps the table entries of its
 * first pass (float [nq][nprobe][m][256]) and quantizes them from memory instead of computing them twice;
 * the results are the same bit for bit. */
size_t dcpq_ivf_tables_workspace_bytes_fast(int nq, int nprobe, int m);
int dcpq_ivf_build_small_tables(const float *queries, int nq, const float *coarse, int nlist,
                                const int32_t *probe, int nprobe, const float *derived, int m, int dsub,
                                const uint16_t *codes, const int64_t *offsets, uint32_t r, uint8_t *qtab,
                                float *bounds, void *workspace, size_t workspace_bytes, void *stream);

/* Scan step over the probed lists: the r smallest by (qd, id) over their union, qd computed with
 * the tables of the list the code lies in.  If the probed lists hold fewer than r codes the tail
 * is padded with id DCPQ_PAD_ID and qd 255; count[q] = number of valid candidates.
 *   cand_id : uint32_t [nq][r]  cand_qd : uint8_t [nq][r]  count : uint32_t [nq]  (outputs)
 *   workspace : dcpq_ivf_scan_workspace_bytes(nq, r), 256-byte aligned; codes and qtab 16-byte aligned */
size_t dcpq_ivf_scan_workspace_bytes(int nq, uint32_t r);
int dcpq_ivf_scan_candidates(const uint16_t *codes, const int64_t *offsets, int nlist, int m,
                             const int32_t *probe, int nprobe, const uint8_t *qtab, int nq, uint32_t r,
                             uint32_t *cand_id, uint8_t *cand_qd, uint32_t *count, void *workspace,
                             size_t workspace_bytes, void *stream);

/* Low-byte plane of a code array.  Pass one consumes only the low bbar = 8 bits of every sub-code
 * (Sec. 3.3, adc_low_bits), and the scan of probed lists is bound by the bytes it streams from HBM, so a
 * copy of just those bytes halves its cost:  plane[i][j] = codes[i][j] & 255,  uint8_t [n_codes][m]
 * (device, caller-owned, 16-byte aligned like codes).  An index-build step, like derive_codebooks. */
int dcpq_pack_low_bytes(const uint16_t *codes, uint64_t n_codes, int m, uint8_t *plane, void *stream);
/* dcpq_ivf_scan_candidates reading the plane instead of the codes: same arguments otherwise, same outputs. */
int dcpq_ivf_scan_candidates_packed(const uint8_t *plane, const int64_t *offsets, int nlist, int m,
                                    const int32_t *probe, int nprobe, const uint8_t *qtab, int nq, uint32_t r,
                                    uint32_t *cand_id, uint8_t *cand_qd, uint32_t *count, void *workspace,
                                    size_t workspace_bytes, void *stream);

/* Refine step: d(q, i) = sum_j || (y_q - coarse[l(i)])^j - codebooks[j][codes[i][j]] ||^2 with l(i)
 * the probed list holding i, computed directly in double precision (Eq. 3 on the residual) and
 * rounded to fp32; the k smallest by (d, i), ascending; padded candidates give id DCPQ_PAD_ID and
 * distance +inf.
 *   ids : uint32_t [nq][k]  dist : float [nq][k] (outputs)
 *   workspace : dcpq_ivf_refine_workspace_bytes(nq, r) (may be 0) */
size_t dcpq_ivf_refine_workspace_bytes(int nq, uint32_t r);
int dcpq_ivf_refine_topk(const float *queries, const float *coarse, int nlist, const float *codebooks, int m,
                         int dsub, const uint16_t *codes, const int64_t *offsets, const int32_t *probe,
                         int nprobe, const uint32_t *cand_id, int nq, uint32_t r, uint32_t k, uint32_t *ids,
                         float *dist, void *workspace, size_t workspace_bytes, void *stream);

/* The four steps above in one call (Alg. 3 with an index: Index, Tables, Scan, Refine) for a batch
 * of queries.  `plane` is the low-byte plane of `codes` from dcpq_pack_low_bytes, or NULL to scan
 * the codes themselves; the probe lists, tables and candidates live in the workspace.  Short lists
 * are padded as in the staged calls (id DCPQ_PAD_ID, distance +inf).
 *   ids : uint32_t [nq][k]  dist : float [nq][k] (outputs)
 *   workspace : dcpq_ivf_search_workspace_bytes(nq, nlist, nprobe, m, r), 256-byte aligned */
size_t dcpq_ivf_search_workspace_bytes(int nq, int nlist, int nprobe, int m, uint32_t r);
int dcpq_ivf_search(const float *queries, int nq, const float *coarse, int nlist, int nprobe,
                    const float *codebooks, const float *derived, int m, int dsub, const uint16_t *codes,
                    const uint8_t *plane, const int64_t *offsets, uint32_t r, uint32_t k, uint32_t *ids,
                    float *dist, void *workspace, size_t workspace_bytes, void *stream);

/* ---------------------------------------------------------------------------------------------
 * Optional per-kernel timing (measurement aid, not part of the search).  While enabled, every
 * kernel the library launches is bracketed by two HIP events recorded on the stream it is launched
 * on.  dcpq_profile_enable(on) clears the accumulated figures; dcpq_profile_read waits for the
 * pending events (it synchronises with them) and returns the total milliseconds and the number of
 * launches of one stage; stage names come from dcpq_profile_stage_name(0 .. stage_count-1).
 * total_ms and launches are HOST pointers.
 * ------------------------------------------------------------------------------------------- */
int dcpq_profile_enable(int on);
int dcpq_profile_stage_count(void);
const char *dcpq_profile_stage_name(int stage);
int dcpq_profile_read(int stage, double *total_ms, uint64_t *launches);
/* Plain device-to-device copy of `bytes` (multiple of 16) by a kernel named
 * calibration_copy_kernel: reads `bytes`, writes `bytes`.  Hardware traffic counters collected for
 * the search kernels are scaled by what the same counters report for this copy of known size. */
int dcpq_profile_copy(const void *src, void *dst, size_t bytes, void *stream);
/* Read-only stream over `bytes` (multiple of 16) of device memory by a kernel named
 * stream_read_kernel (stage "misc" of the timing above): the rate a kernel that reads an array once
 * reaches on this device, the yardstick beside the published HBM peak for the scans that are bound
 * by the code stream.  `sink` receives dcpq_profile_stream_read_sink_bytes() bytes of checksums. */
size_t dcpq_profile_stream_read_sink_bytes(void);
int dcpq_profile_stream_read(const void *src, size_t bytes, void *sink, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* DCPQ_H */
