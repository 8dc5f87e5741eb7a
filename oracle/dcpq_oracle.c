/*
 * dcpq_oracle.c -- plain, slow, CPU-only statement of the two-pass product-quantization
 * search with derived codebooks ("Derived Codebooks for High-Accuracy Nearest Neighbor
 * Search", Sec. 2.3 Alg. 1 / Eq. 1-3, Sec. 3.2 Alg. 2, Sec. 3.3 Alg. 3).
 *
 * THIS IS TEST INFRASTRUCTURE.  It defines what the GPU library must compute; it shares no
 * code, header, table or helper with the GPU library, and only the tests, the smoke check
 * and the benchmark's cpu_baseline leg may call it.  It is never tuned for speed.
 *
 * Naming: r = size of the candidate set kept by pass one (the paper's r2), k = size of the
 * final result set (the paper's r), m = number of sub-quantizers, b = bits per sub-code,
 * bbar = bits of a derived codebook index (the low bbar bits of a sub-code, property P1).
 *
 * Arithmetic contract
 *   - Everything that decides an integer in pass one (derived codebooks, small tables,
 *     qmin/qmax, 8-bit table quantization) is single precision IEEE-754, one rounding per
 *     written operation, in exactly the order written here; build with
 *     -ffp-contract=off -fno-fast-math so the compiler neither fuses nor reorders.
 *   - Pass two (exact re-ranking, Eq. 3) is double precision from the fp32 inputs.
 *   - Ties are always broken by the smaller id.
 *
 * Parity pins: every function below is pinned by tests/test_oracle_*.py (brute force in
 * numpy/fractions, closed forms, the paper's printed index example, the reduction of the
 * two-pass search to exhaustive 16-bit ADC when r = N; for the training functions at the end
 * of the file also scikit-learn's Lloyd iteration, a hand-worked balanced assignment and the
 * invariants of Alg. 2).  Unpinned: none of the paper's
 * recall or latency figures (its datasets and trained codebooks are not available).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* ------------------------------------------------------------------------------------------
 * Sec. 3.2, step 2 + property P1: the derived centroid l of sub-quantizer j is the mean of
 * the group G_l, and by P1 the members of G_l are the full centroids whose index has low
 * bbar bits equal to l, i.e. indices (i << bbar) | l for i = 0 .. 2^(b-bbar)-1.
 * C    : [m][2^b][dsub]     Cbar : [m][2^bbar][dsub]
 * fp32, members added in increasing i, then one division by the group size.
 * ---------------------------------------------------------------------------------------- */
void dcpq_oracle_derive_codebooks(const float *C, int m, int dsub, int b, int bbar, float *Cbar)
{
    const size_t k = (size_t)1 << b, kbar = (size_t)1 << bbar, gsize = (size_t)1 << (b - bbar);
    for (int j = 0; j < m; ++j)
        for (size_t l = 0; l < kbar; ++l)
            for (int t = 0; t < dsub; ++t) {
                float acc = 0.0f;
                for (size_t i = 0; i < gsize; ++i)
                    acc = acc + C[((size_t)j * k + ((i << bbar) | l)) * dsub + t];
                Cbar[((size_t)j * kbar + l) * dsub + t] = acc / (float)gsize;
            }
}

/* ------------------------------------------------------------------------------------------
 * Eq. 1 (compute_tables) in the fp32 contract: D[j][i] = sum_t (y^j_t - C_j[i]_t)^2,
 * t increasing, each of subtract / multiply / add rounded to fp32.
 * Used for the small tables (Sec. 3.3, Tables step) that feed the integer quantizer.
 * y : [m*dsub]   C : [m][kc][dsub]   D : [m][kc]
 * ---------------------------------------------------------------------------------------- */
void dcpq_oracle_compute_tables_f32(const float *y, const float *C, int m, int kc, int dsub, float *D)
{
    for (int j = 0; j < m; ++j)
        for (int i = 0; i < kc; ++i) {
            const float *c = C + ((size_t)j * kc + i) * dsub;
            float acc = 0.0f;
            for (int t = 0; t < dsub; ++t) {
                float diff = y[j * dsub + t] - c[t];
                float sq = diff * diff;
                acc = acc + sq;
            }
            D[(size_t)j * kc + i] = acc;
        }
}

/* Eq. 1 in double precision (the reference for the full 2^b-entry tables). */
void dcpq_oracle_compute_tables_f64(const float *y, const float *C, int m, int kc, int dsub, double *D)
{
    for (int j = 0; j < m; ++j)
        for (int i = 0; i < kc; ++i) {
            const float *c = C + ((size_t)j * kc + i) * dsub;
            double acc = 0.0;
            for (int t = 0; t < dsub; ++t) {
                double diff = (double)y[j * dsub + t] - (double)c[t];
                acc += diff * diff;
            }
            D[(size_t)j * kc + i] = acc;
        }
}

/* low_bbar(c): the lowest bbar bits of a sub-code (Sec. 3.2, P1; Alg. 3 adc_low_bits). */
static inline unsigned low_bits(unsigned c, int bbar) { return c & ((1u << bbar) - 1u); }

/* Small-table ADC of one code in fp32: ((Dbar_0[.] + Dbar_1[.]) + ...) over j increasing. */
static float adc_small_f32(const uint16_t *code, const float *Dbar, int m, int bbar)
{
    const int kbar = 1 << bbar;
    float acc = Dbar[low_bits(code[0], bbar)];
    for (int j = 1; j < m; ++j)
        acc = acc + Dbar[(size_t)j * kbar + low_bits(code[j], bbar)];
    return acc;
}

/* ------------------------------------------------------------------------------------------
 * Sec. 3.3, Tables step: qmin = smallest entry of all small tables; qmax = largest small-table
 * distance between the query and the first n_first codes of the list.
 * Dbar : [m][2^bbar]   codes : [n_first][m]
 * ---------------------------------------------------------------------------------------- */
void dcpq_oracle_bounds(const float *Dbar, int m, int bbar, const uint16_t *codes, uint64_t n_first,
                        float *qmin, float *qmax)
{
    const int kbar = 1 << bbar;
    float lo = Dbar[0];
    for (int e = 1; e < m * kbar; ++e)
        if (Dbar[e] < lo) lo = Dbar[e];
    float hi = -INFINITY;
    for (uint64_t i = 0; i < n_first; ++i) {
        float d = adc_small_f32(codes + i * (size_t)m, Dbar, m, bbar);
        if (d > hi) hi = d;
    }
    *qmin = lo;
    *qmax = hi;
}

/* ------------------------------------------------------------------------------------------
 * Sec. 3.3 quantization formula: Q = floor((Dbar - qmin) / (qmax - qmin) * 255); entries at or
 * above qmax become 255 (bins 0..254 lie below qmax).  A non-positive range gives all zeros.
 * ---------------------------------------------------------------------------------------- */
void dcpq_oracle_quantize(const float *Dbar, int n_entries, float qmin, float qmax, uint8_t *Qt)
{
    const float den = qmax - qmin;
    for (int e = 0; e < n_entries; ++e) {
        if (!(den > 0.0f)) { Qt[e] = 0; continue; }
        float num = Dbar[e] - qmin;
        float t = num / den;
        float u = t * 255.0f;
        Qt[e] = (u >= 255.0f) ? (uint8_t)255 : (uint8_t)floorf(u);
    }
}

/* ------------------------------------------------------------------------------------------
 * Alg. 3 adc_low_bits for every code of a list: qd[i] = min(255, sum_j Q_j[low_bbar(c_i[j])]).
 * The sum is saturated at 255: bucket ids are one byte and 255 means "beyond qmax".
 * ---------------------------------------------------------------------------------------- */
void dcpq_oracle_adc_low_bits(const uint16_t *codes, uint64_t n, int m, int bbar, const uint8_t *Qt,
                              uint8_t *qd)
{
    const int kbar = 1 << bbar;
    for (uint64_t i = 0; i < n; ++i) {
        unsigned s = 0;
        for (int j = 0; j < m; ++j)
            s += Qt[(size_t)j * kbar + low_bits(codes[i * (size_t)m + j], bbar)];
        qd[i] = (uint8_t)(s > 255u ? 255u : s);
    }
}

/* ------------------------------------------------------------------------------------------
 * Capped buckets (Sec. 3.3, Scan step) read out as in the Refine step: one bucket per integer
 * distance, ids appended in list order, buckets visited by increasing distance.  The candidate
 * set is cut at exactly r ids, i.e. the r smallest by (qd, position); ids[] maps a position in
 * the scanned sequence to the reported id and must be increasing where qd ties matter (NULL =
 * the position itself).
 * Returns the number of candidates written (min(r, n)).
 * ---------------------------------------------------------------------------------------- */
uint64_t dcpq_oracle_select(const uint8_t *qd, const uint32_t *ids, uint64_t n, uint64_t r,
                            uint32_t *cand_id, uint8_t *cand_qd)
{
    uint64_t hist[256];
    memset(hist, 0, sizeof hist);
    for (uint64_t i = 0; i < n; ++i) hist[qd[i]]++;
    uint64_t start[257];
    start[0] = 0;
    for (int bkt = 0; bkt < 256; ++bkt) start[bkt + 1] = start[bkt] + hist[bkt];
    const uint64_t keep = r < n ? r : n;
    uint64_t fill[256];
    memset(fill, 0, sizeof fill);
    for (uint64_t i = 0; i < n; ++i) {
        const unsigned bkt = qd[i];
        const uint64_t slot = start[bkt] + fill[bkt]++;
        if (slot < keep) {
            cand_id[slot] = ids ? ids[i] : (uint32_t)i;
            cand_qd[slot] = (uint8_t)bkt;
        }
    }
    return keep;
}

/* Eq. 3: exact asymmetric distance of one code, double precision. */
static double adc_exact_f64(const float *y, const float *C, int m, int dsub, int b, const uint16_t *code)
{
    const size_t k = (size_t)1 << b;
    double d = 0.0;
    for (int j = 0; j < m; ++j) {
        const float *c = C + ((size_t)j * k + code[j]) * dsub;
        double dj = 0.0;
        for (int t = 0; t < dsub; ++t) {
            double diff = (double)y[j * dsub + t] - (double)c[t];
            dj += diff * diff;
        }
        d += dj;
    }
    return d;
}

/* Alg. 3 refine / adc_refine: exact distance of every candidate (values of Eq. 3; the lazily
 * filled table of the listing holds exactly these sub-distances). */
void dcpq_oracle_refine(const float *y, const float *C, int m, int dsub, int b, const uint16_t *codes,
                        const uint32_t *cand_id, uint64_t n_cand, double *dist)
{
    for (uint64_t c = 0; c < n_cand; ++c)
        dist[c] = adc_exact_f64(y, C, m, dsub, b, codes + (size_t)cand_id[c] * m);
}

typedef struct { double d; uint32_t id; } pair_t;
static int pair_cmp(const void *a, const void *b_)
{
    const pair_t *x = (const pair_t *)a, *z = (const pair_t *)b_;
    if (x->d < z->d) return -1;
    if (x->d > z->d) return 1;
    return (x->id > z->id) - (x->id < z->id);
}

/* Result set of size k (the binary heap of Alg. 1 / Alg. 3): k smallest by (distance, id),
 * ascending.  Returns min(k, n). */
uint64_t dcpq_oracle_topk(const double *dist, const uint32_t *ids, uint64_t n, uint64_t k,
                          uint32_t *out_id, double *out_dist)
{
    pair_t *p = (pair_t *)malloc((n ? n : 1) * sizeof(pair_t));
    for (uint64_t i = 0; i < n; ++i) { p[i].d = dist[i]; p[i].id = ids[i]; }
    qsort(p, n, sizeof(pair_t), pair_cmp);
    const uint64_t keep = k < n ? k : n;
    for (uint64_t i = 0; i < keep; ++i) { out_id[i] = p[i].id; out_dist[i] = p[i].d; }
    free(p);
    return keep;
}

/* ------------------------------------------------------------------------------------------
 * Alg. 3 nns_derived without an index (exhaustive search), for nq queries (OpenMP over queries).
 * Inputs : C [m][2^b][dsub], Cbar [m][2^bbar][dsub], codes [N][m], queries [nq][m*dsub].
 * Outputs (any may be NULL): small [nq][m][2^bbar] fp32 small tables, bounds [nq][2] (qmin,qmax),
 *          qtab [nq][m][2^bbar], cand_id/cand_qd [nq][r], ids [nq][k], dist [nq][k] (double).
 * Requires k <= r <= N.  Returns 0, or -1 on bad arguments.
 * ---------------------------------------------------------------------------------------- */
int dcpq_oracle_search_flat(const float *C, const float *Cbar, int m, int dsub, int b, int bbar,
                            const uint16_t *codes, uint64_t N, const float *queries, int nq,
                            uint64_t r, uint64_t k, float *small, float *bounds, uint8_t *qtab,
                            uint32_t *cand_id, uint8_t *cand_qd, uint32_t *ids, double *dist)
{
    if (m <= 0 || dsub <= 0 || bbar <= 0 || b < bbar || b > 16 || r > N || k > r) return -1;
    const int kbar = 1 << bbar, ntab = m * kbar;
    int failed = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int q = 0; q < nq; ++q) {
        const float *y = queries + (size_t)q * m * dsub;
        float *Dbar = (float *)malloc(sizeof(float) * ntab);
        uint8_t *Qt = (uint8_t *)malloc(ntab);
        uint8_t *qd = (uint8_t *)malloc(N ? N : 1);
        uint32_t *cid = (uint32_t *)malloc(sizeof(uint32_t) * (r ? r : 1));
        uint8_t *cqd = (uint8_t *)malloc(r ? r : 1);
        double *cd = (double *)malloc(sizeof(double) * (r ? r : 1));
        if (!Dbar || !Qt || !qd || !cid || !cqd || !cd) {
            failed = 1;
        } else {
            float qmin, qmax;
            dcpq_oracle_compute_tables_f32(y, Cbar, m, kbar, dsub, Dbar);        /* Tables */
            dcpq_oracle_bounds(Dbar, m, bbar, codes, r < N ? r : N, &qmin, &qmax);
            dcpq_oracle_quantize(Dbar, ntab, qmin, qmax, Qt);
            dcpq_oracle_adc_low_bits(codes, N, m, bbar, Qt, qd);                 /* Scan */
            dcpq_oracle_select(qd, NULL, N, r, cid, cqd);
            dcpq_oracle_refine(y, C, m, dsub, b, codes, cid, r, cd);             /* Refine */
            if (small) memcpy(small + (size_t)q * ntab, Dbar, sizeof(float) * ntab);
            if (bounds) { bounds[2 * q] = qmin; bounds[2 * q + 1] = qmax; }
            if (qtab) memcpy(qtab + (size_t)q * ntab, Qt, ntab);
            if (cand_id) memcpy(cand_id + (size_t)q * r, cid, sizeof(uint32_t) * r);
            if (cand_qd) memcpy(cand_qd + (size_t)q * r, cqd, r);
            if (ids && dist) dcpq_oracle_topk(cd, cid, r, k, ids + (size_t)q * k, dist + (size_t)q * k);
        }
        free(Dbar); free(Qt); free(qd); free(cid); free(cqd); free(cd);
    }
    return failed ? -2 : 0;
}

/* ------------------------------------------------------------------------------------------
 * Alg. 1 (conventional search) with the full 2^b tables, exhaustive: the k smallest by
 * (Eq. 3 distance, id) over the whole list.  This is what the two-pass search returns when r = N.
 * ---------------------------------------------------------------------------------------- */
int dcpq_oracle_search_exhaustive(const float *C, int m, int dsub, int b, const uint16_t *codes,
                                  uint64_t N, const float *queries, int nq, uint64_t k,
                                  uint32_t *ids, double *dist)
{
    if (k > N) return -1;
#pragma omp parallel for schedule(dynamic, 1)
    for (int q = 0; q < nq; ++q) {
        const float *y = queries + (size_t)q * m * dsub;
        double *d = (double *)malloc(sizeof(double) * (N ? N : 1));
        uint32_t *id = (uint32_t *)malloc(sizeof(uint32_t) * (N ? N : 1));
        for (uint64_t i = 0; i < N; ++i) {
            id[i] = (uint32_t)i;
            d[i] = adc_exact_f64(y, C, m, dsub, b, codes + i * (size_t)m);
        }
        dcpq_oracle_topk(d, id, N, k, ids + (size_t)q * k, dist + (size_t)q * k);
        free(d); free(id);
    }
    return 0;
}

/* ------------------------------------------------------------------------------------------
 * Index step (Sec. 2.3): the nprobe inverted lists whose cell centres are closest to y, ordered
 * by (squared distance in double precision, list id).
 * coarse : [nlist][D]    probe : [nprobe]
 * ---------------------------------------------------------------------------------------- */
void dcpq_oracle_ivf_probe(const float *y, const float *coarse, int nlist, int D, int nprobe, int32_t *probe)
{
    pair_t *p = (pair_t *)malloc(sizeof(pair_t) * (size_t)nlist);
    for (int l = 0; l < nlist; ++l) {
        double d = 0.0;
        for (int t = 0; t < D; ++t) {
            double diff = (double)y[t] - (double)coarse[(size_t)l * D + t];
            d += diff * diff;
        }
        p[l].d = d; p[l].id = (uint32_t)l;
    }
    qsort(p, (size_t)nlist, sizeof(pair_t), pair_cmp);
    for (int i = 0; i < nprobe; ++i) probe[i] = (int32_t)p[i].id;
    free(p);
}

/* ------------------------------------------------------------------------------------------
 * Alg. 3 with an inverted index and residual encoding (Sec. 2.2, Sec. 2.3 "each step is repeated
 * ma times", Sec. 3.3).  List l holds the codes at positions offsets[l] .. offsets[l+1]-1 of the
 * code array; a vector's id is its position in that array.  For each probed list the residual
 * rho = y - c_l is formed in fp32 and the small tables are computed on rho.  One (qmin, qmax)
 * pair per query: qmin over the tables of all probed lists, qmax over the first min(r, total)
 * codes met when walking the probed lists in probe order.  Candidates are the r smallest by
 * (qd, id) over the union of the probed lists; refinement is Eq. 3 on the residual of the
 * candidate's own list, in double precision from the fp32 inputs.
 * probe : [nq][nprobe] (from dcpq_oracle_ivf_probe).  If the probed lists hold fewer than r (or
 * k) codes the tail of the outputs is padded with id 0xFFFFFFFF, qd 255, distance +inf; count[q]
 * receives the number of valid candidates.
 * Outputs (any may be NULL): bounds [nq][2], qtab [nq][nprobe][m][2^bbar], cand_id/cand_qd
 * [nq][r], count [nq], ids [nq][k], dist [nq][k].
 * ---------------------------------------------------------------------------------------- */
int dcpq_oracle_search_ivf(const float *C, const float *Cbar, int m, int dsub, int b, int bbar,
                           const uint16_t *codes, const int64_t *offsets, const float *coarse, int nlist,
                           const float *queries, int nq, const int32_t *probe, int nprobe,
                           uint64_t r, uint64_t k, float *bounds, uint8_t *qtab,
                           uint32_t *cand_id, uint8_t *cand_qd, uint32_t *count,
                           uint32_t *ids, double *dist)
{
    if (m <= 0 || dsub <= 0 || k > r || nprobe > nlist) return -1;
    const int kbar = 1 << bbar, ntab = m * kbar, D = m * dsub;
    int failed = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int q = 0; q < nq; ++q) {
        const float *y = queries + (size_t)q * D;
        const int32_t *pl = probe + (size_t)q * nprobe;
        uint64_t total = 0;
        for (int p = 0; p < nprobe; ++p) total += (uint64_t)(offsets[pl[p] + 1] - offsets[pl[p]]);
        float *rho = (float *)malloc(sizeof(float) * (size_t)nprobe * D);
        float *Dbar = (float *)malloc(sizeof(float) * (size_t)nprobe * ntab);
        uint8_t *Qt = (uint8_t *)malloc((size_t)nprobe * ntab);
        uint8_t *qd = (uint8_t *)malloc(total ? total : 1);
        uint32_t *gid = (uint32_t *)malloc(sizeof(uint32_t) * (total ? total : 1));
        uint32_t *cid = (uint32_t *)malloc(sizeof(uint32_t) * (r ? r : 1));
        uint8_t *cqd = (uint8_t *)malloc(r ? r : 1);
        double *cd = (double *)malloc(sizeof(double) * (r ? r : 1));
        if (!rho || !Dbar || !Qt || !qd || !gid || !cid || !cqd || !cd) {
            failed = 1;
        } else {
            /* Index + Tables, once per probed list */
            float qmin = INFINITY, qmax = -INFINITY;
            for (int p = 0; p < nprobe; ++p) {
                const float *c = coarse + (size_t)pl[p] * D;
                for (int t = 0; t < D; ++t) rho[(size_t)p * D + t] = y[t] - c[t];
                dcpq_oracle_compute_tables_f32(rho + (size_t)p * D, Cbar, m, kbar, dsub, Dbar + (size_t)p * ntab);
                for (int e = 0; e < ntab; ++e)
                    if (Dbar[(size_t)p * ntab + e] < qmin) qmin = Dbar[(size_t)p * ntab + e];
            }
            /* qmax: the first min(r, total) vectors in probe order */
            uint64_t seen = 0;
            for (int p = 0; p < nprobe && seen < r; ++p) {
                const int64_t lo = offsets[pl[p]], hi = offsets[pl[p] + 1];
                for (int64_t i = lo; i < hi && seen < r; ++i, ++seen) {
                    float d = adc_small_f32(codes + (size_t)i * m, Dbar + (size_t)p * ntab, m, bbar);
                    if (d > qmax) qmax = d;
                }
            }
            if (total == 0) { qmin = 0.0f; qmax = 0.0f; }
            dcpq_oracle_quantize(Dbar, nprobe * ntab, qmin, qmax, Qt);
            /* Scan: lists are visited in increasing list id so that positions in the scanned
             * sequence increase with the global id, as dcpq_oracle_select requires. */
            int32_t *order = (int32_t *)malloc(sizeof(int32_t) * (size_t)nprobe);
            for (int p = 0; p < nprobe; ++p) order[p] = p;
            for (int a = 1; a < nprobe; ++a) {          /* insertion sort by list id */
                int32_t v = order[a]; int z = a - 1;
                while (z >= 0 && pl[order[z]] > pl[v]) { order[z + 1] = order[z]; --z; }
                order[z + 1] = v;
            }
            uint64_t pos = 0;
            for (int a = 0; a < nprobe; ++a) {
                const int p = order[a];
                const int64_t lo = offsets[pl[p]], hi = offsets[pl[p] + 1];
                dcpq_oracle_adc_low_bits(codes + (size_t)lo * m, (uint64_t)(hi - lo), m, bbar,
                                         Qt + (size_t)p * ntab, qd + pos);
                for (int64_t i = lo; i < hi; ++i) gid[pos++] = (uint32_t)i;
            }
            const uint64_t ncand = dcpq_oracle_select(qd, gid, total, r, cid, cqd);
            /* Refine on the residual of each candidate's list */
            for (uint64_t c = 0; c < ncand; ++c) {
                int p_of = -1;
                for (int p = 0; p < nprobe; ++p)
                    if ((int64_t)cid[c] >= offsets[pl[p]] && (int64_t)cid[c] < offsets[pl[p] + 1]) { p_of = p; break; }
                const float *cc = coarse + (size_t)pl[p_of] * D;
                const uint16_t *code = codes + (size_t)cid[c] * m;
                const size_t kfull = (size_t)1 << b;
                double d = 0.0;
                for (int j = 0; j < m; ++j) {
                    const float *cen = C + ((size_t)j * kfull + code[j]) * dsub;
                    double dj = 0.0;
                    for (int t = 0; t < dsub; ++t) {
                        double diff = ((double)y[j * dsub + t] - (double)cc[j * dsub + t]) - (double)cen[t];
                        dj += diff * diff;
                    }
                    d += dj;
                }
                cd[c] = d;
            }
            for (uint64_t c = ncand; c < r; ++c) { cid[c] = 0xFFFFFFFFu; cqd[c] = 255; cd[c] = INFINITY; }
            if (bounds) { bounds[2 * q] = qmin; bounds[2 * q + 1] = qmax; }
            if (qtab) memcpy(qtab + (size_t)q * nprobe * ntab, Qt, (size_t)nprobe * ntab);
            if (cand_id) memcpy(cand_id + (size_t)q * r, cid, sizeof(uint32_t) * r);
            if (cand_qd) memcpy(cand_qd + (size_t)q * r, cqd, r);
            if (count) count[q] = (uint32_t)ncand;
            if (ids && dist) dcpq_oracle_topk(cd, cid, r, k, ids + (size_t)q * k, dist + (size_t)q * k);
            free(order);
        }
        free(rho); free(Dbar); free(Qt); free(qd); free(gid); free(cid); free(cqd); free(cd);
    }
    return failed ? -2 : 0;
}

int dcpq_oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* ==========================================================================================
 * Training (Sec. 3.2, Alg. 2: build_quantizers) and encoding (Sec. 3.2, last paragraph).
 *
 * The paper names its three steps and leaves their insides to "a standard implementation of
 * k-means" and to a same-size k-means variant it cites; the readings taken here:
 *   - distances are double precision from the fp32 inputs, components added in increasing
 *     order; the nearest centroid is the one with the smallest (distance, index);
 *   - a k-means iteration is: assign every point, then replace each centroid by the mean of
 *     its members (double precision sum in increasing point order, one division, rounded to
 *     fp32); a centroid without members keeps its value; the initial centroids are an input;
 *     after the last iteration the points are assigned once more, to the final centroids;
 *   - same-size k-means: an iteration assigns the points to clusters of exactly n / kbar
 *     members each (balanced assignment, below) and then takes the means as above; the
 *     labels returned are those of the last assignment, so that the returned centroids are
 *     the means of the returned groups (Sec. 3.2, step 2);
 *   - balanced assignment, in rounds: every point without a cluster proposes to the cluster
 *     with the smallest (distance, index) among those that still have room; every cluster
 *     takes, among its proposers, the ones with the smallest (distance, point) up to the room
 *     it has; repeat until no point is left.  Distances are rounded to fp32 first (they are
 *     compared as fp32 by the GPU library, which reads them from a table of floats).
 * ======================================================================================== */

/* squared distance between an fp32 point and an fp32 centroid, double precision */
static double dist2_f64(const float *x, const float *c, int d)
{
    double acc = 0.0;
    for (int t = 0; t < d; ++t) {
        const double diff = (double)x[t] - (double)c[t];
        acc += diff * diff;
    }
    return acc;
}

/* X : n rows of d floats, row stride ld floats.   C : [k][d].   label : [n]   dist2 : [n] or NULL */
void dcpq_oracle_assign(const float *X, uint64_t n, int d, int ld, const float *C, int k, uint32_t *label,
                        double *dist2)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < (int64_t)n; ++i) {
        double best = INFINITY;
        uint32_t arg = 0;
        for (int c = 0; c < k; ++c) {
            const double dd = dist2_f64(X + (size_t)i * ld, C + (size_t)c * d, d);
            if (dd < best) { best = dd; arg = (uint32_t)c; }      /* strict: the smaller index wins a tie */
        }
        label[i] = arg;
        if (dist2) dist2[i] = best;
    }
}

/* means of the members of every cluster; a cluster without members keeps its centroid */
static void update_means(const float *X, uint64_t n, int d, int ld, const uint32_t *label, int k, float *C)
{
    double *sum = (double *)calloc((size_t)k * d, sizeof(double));
    uint64_t *cnt = (uint64_t *)calloc((size_t)k, sizeof(uint64_t));
    for (uint64_t i = 0; i < n; ++i) {
        const uint32_t c = label[i];
        cnt[c] += 1;
        for (int t = 0; t < d; ++t) sum[(size_t)c * d + t] += (double)X[(size_t)i * ld + t];
    }
    for (int c = 0; c < k; ++c)
        if (cnt[c])
            for (int t = 0; t < d; ++t) C[(size_t)c * d + t] = (float)(sum[(size_t)c * d + t] / (double)cnt[c]);
    free(sum); free(cnt);
}

/* Alg. 2 step 1.  C : [k][d], initial centroids in, final centroids out.  label : [n] out. */
void dcpq_oracle_kmeans(const float *X, uint64_t n, int d, int ld, int k, int iters, float *C, uint32_t *label)
{
    for (int it = 0; it < iters; ++it) {
        dcpq_oracle_assign(X, n, d, ld, C, k, label, NULL);
        update_means(X, n, d, ld, label, k, C);
    }
    dcpq_oracle_assign(X, n, d, ld, C, k, label, NULL);
}

typedef struct { float d; uint32_t i; } prop_t;
static int prop_cmp(const void *a, const void *b)
{
    const prop_t *x = (const prop_t *)a, *y = (const prop_t *)b;
    if (x->d < y->d) return -1;
    if (x->d > y->d) return 1;
    return x->i < y->i ? -1 : (x->i > y->i ? 1 : 0);
}

/* Balanced assignment of n points to kbar clusters of n / kbar members each (n % kbar == 0).
 * D : [n][kbar] fp32 distances.  label : [n] out.  Returns the number of rounds, -1 on bad sizes. */
int dcpq_oracle_balanced_assign(const float *D, int n, int kbar, uint32_t *label)
{
    if (kbar <= 0 || n <= 0 || n % kbar) return -1;
    int *room = (int *)malloc(sizeof(int) * kbar);
    int *prop = (int *)malloc(sizeof(int) * n);
    prop_t *list = (prop_t *)malloc(sizeof(prop_t) * n);
    for (int l = 0; l < kbar; ++l) room[l] = n / kbar;
    for (int i = 0; i < n; ++i) label[i] = 0xFFFFFFFFu;
    int left = n, rounds = 0;
    while (left > 0) {
        ++rounds;
        for (int i = 0; i < n; ++i) {
            prop[i] = -1;
            if (label[i] != 0xFFFFFFFFu) continue;
            float best = INFINITY;
            for (int l = 0; l < kbar; ++l)
                if (room[l] > 0 && (prop[i] < 0 || D[(size_t)i * kbar + l] < best)) { best = D[(size_t)i * kbar + l]; prop[i] = l; }
        }
        for (int l = 0; l < kbar; ++l) {
            if (room[l] == 0) continue;
            int p = 0;
            for (int i = 0; i < n; ++i)
                if (prop[i] == l) { list[p].d = D[(size_t)i * kbar + l]; list[p].i = (uint32_t)i; ++p; }
            qsort(list, (size_t)p, sizeof(prop_t), prop_cmp);
            const int take = p < room[l] ? p : room[l];
            for (int t = 0; t < take; ++t) label[list[t].i] = (uint32_t)l;
            room[l] -= take;
            left -= take;
        }
    }
    free(room); free(prop); free(list);
    return rounds;
}

/* Alg. 2 step 2.  P : [n][d] (the centroids of the temporary codebook), Cbar : [kbar][d] initial in, final out.
 * label : [n] out, the groups whose means Cbar holds.  Returns 0, -1 on bad sizes. */
int dcpq_oracle_kmeans_same_size(const float *P, int n, int d, int kbar, int iters, float *Cbar, uint32_t *label)
{
    if (kbar <= 0 || n <= 0 || n % kbar || iters < 1) return -1;
    float *D = (float *)malloc(sizeof(float) * (size_t)n * kbar);
    for (int it = 0; it < iters; ++it) {
        for (int i = 0; i < n; ++i)
            for (int l = 0; l < kbar; ++l)
                D[(size_t)i * kbar + l] = (float)dist2_f64(P + (size_t)i * d, Cbar + (size_t)l * d, d);
        dcpq_oracle_balanced_assign(D, n, kbar, label);
        update_means(P, (uint64_t)n, d, d, label, kbar, Cbar);
    }
    free(D);
    return 0;
}

/* Alg. 2 step 3 (build_final_codebook): the members of group l, taken in increasing index of the
 * temporary codebook, get the final indices (0 << bbar) | l, (1 << bbar) | l, ... (property P1).
 * Ct : [k][d] temporary codebook, label : [k] group of each of its centroids (2^bbar groups of equal size).
 * Cf : [k][d] final codebook out, perm : [k] out, perm[final index] = temporary index.  Returns 0, -1 if
 * the groups are not of equal size. */
int dcpq_oracle_build_final_codebook(const float *Ct, int k, int d, const uint32_t *label, int bbar, float *Cf,
                                     uint32_t *perm)
{
    const int kbar = 1 << bbar;
    if (k % kbar) return -1;
    int *seen = (int *)calloc((size_t)kbar, sizeof(int));
    int rc = 0;
    for (int i = 0; i < k && !rc; ++i) {
        const uint32_t l = label[i];
        if (l >= (uint32_t)kbar || seen[l] >= k / kbar) { rc = -1; break; }
        const uint32_t f = ((uint32_t)seen[l] << bbar) | l;
        seen[l] += 1;
        perm[f] = (uint32_t)i;
        memcpy(Cf + (size_t)f * d, Ct + (size_t)i * d, sizeof(float) * d);
    }
    free(seen);
    return rc;
}

/* Encoding: sub-code j of vector i = index of the centroid of C_j nearest to the j-th sub-vector.
 * X : [n][m*dsub]   C : [m][kc][dsub]   codes : [n][m] */
void dcpq_oracle_encode(const float *X, uint64_t n, const float *C, int m, int kc, int dsub, uint16_t *codes)
{
    uint32_t *lab = (uint32_t *)malloc(sizeof(uint32_t) * n);
    for (int j = 0; j < m; ++j) {
        dcpq_oracle_assign(X + (size_t)j * dsub, n, dsub, m * dsub, C + (size_t)j * kc * dsub, kc, lab, NULL);
        for (uint64_t i = 0; i < n; ++i) codes[i * m + j] = (uint16_t)lab[i];
    }
    free(lab);
}
