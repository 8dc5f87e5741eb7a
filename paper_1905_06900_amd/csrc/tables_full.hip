// Full lookup tables of Alg. 1 / Eq. 1 for a batch of queries:
//   tables[q][j][i] = || y_q^j - C_j[i] ||^2 = ||y_q^j||^2 + ||C_j[i]||^2 - 2 <y_q^j, C_j[i]>.
// The inner products of (queries x 65536 centroids) per sub-quantizer are a dense contraction and
// run on the matrix cores.  They run in DOUBLE precision (v_mfma_f64_16x16x4_f64): the expanded
// form cancels (norms are 10-100x the distances on SIFT-like data), so fp32 products would not
// hold 1e-5 relative, while fp64 costs nothing here -- K = dsub is tiny (12..60), so the kernel
// is bound by writing the fp32 tables to HBM, not by the matrix pipe.  One rounding to fp32 at
// the store.
#include "common.h"
#include "f64_tile.h"

namespace dcpq {


constexpr int kTileQ = 32;     // queries per workgroup   (2 row tiles of 16)
constexpr int kTileC = 256;    // centroids per workgroup (4 wavefronts x 64)

// MFMA operand/result layout (16x16x4, fp64), lane l = 0..63:
//   A (16x4):  row l % 16, column l / 16          B (4x16): row l / 16, column l % 16
//   D (16x16): 4 values per lane, value v is row 4 * v + l / 16, column l % 16
// Centroid columns are interleaved so that a lane ends up with 4 consecutive centroids of one
// query row: column c of column-tile nt is centroid c * 4 + nt of the wavefront's 64, which
// turns the stores into 16-byte vectors, 256 contiguous bytes per 16 lanes.
// ncent = centroids per sub-quantizer (65536 for the product quantizer; any count for the coarse
// quantizer of the inverted index, which is the same computation with m = 1 and dsub = D).
__global__ __launch_bounds__(256) void full_tables_kernel(const float *__restrict__ queries, int nq,
                                                          const float *__restrict__ cb, int m, int dsub,
                                                          int ncent, float *__restrict__ tables)
{
    __shared__ double ny[kTileQ];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    // The query tile varies fastest over the workgroups: those that run at the same time then share their
    // centroids (which they fetch through the caches of 8 XCDs, not once per query tile from memory: 1.1 GB ->
    // about 0.3 GB for 1024 queries x 65536 centroids of 128 components), and the few queries stay cached anyway.
    const int qtiles = (nq + kTileQ - 1) / kTileQ;
    const int j = blockIdx.z;
    const int q0 = static_cast<int>(blockIdx.x % qtiles) * kTileQ;
    const int c0 = static_cast<int>(blockIdx.x / qtiles) * kTileC;
    const int D = m * dsub;
    const float *cbj = cb + static_cast<size_t>(j) * ncent * dsub;

    constexpr int MT = kTileQ / 16;
    double4_t acc[MT][4];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int nt = 0; nt < 4; ++nt) acc[mt][nt] = double4_t{0.0, 0.0, 0.0, 0.0};

    const int lr = lane & 15, lk = lane >> 4;
    const int cw = c0 + wave * 64;                     // first centroid of this wavefront
    // this lane's rows, clamped to valid ones (rows past the end compute values that are never stored)
    const float *ap[MT], *bp[4];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        const int q = q0 + mt * 16 + lr;
        ap[mt] = queries + static_cast<size_t>(q < nq ? q : nq - 1) * D + j * dsub;
    }
#pragma unroll
    for (int nt = 0; nt < 4; ++nt) {
        const int c = cw + lr * 4 + nt;
        bp[nt] = cbj + static_cast<size_t>(c < ncent ? c : ncent - 1) * dsub;
    }
    double na[MT], nb[4] = {0.0, 0.0, 0.0, 0.0};
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) na[mt] = 0.0;
    // (the queries' norms are wanted once per workgroup: the first wavefront computes them)
    f64_tile_products<MT>(ap, bp, dsub, lk, __builtin_amdgcn_readfirstlane(wave) == 0, acc, na, nb);
    // sum the four component residues: lane (lr, *) then holds the norms of queries q0 + 16 mt + lr and of
    // its own four centroids; the queries' norms go through LDS, because the outputs of a lane belong to
    // other queries than its A operands
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        na[mt] += __shfl_xor(na[mt], 16);
        na[mt] += __shfl_xor(na[mt], 32);
        if (wave == 0 && lk == 0) ny[mt * 16 + lr] = na[mt];
    }
#pragma unroll
    for (int nt = 0; nt < 4; ++nt) {
        nb[nt] += __shfl_xor(nb[nt], 16);
        nb[nt] += __shfl_xor(nb[nt], 32);
    }
    __syncthreads();   // query norms visible

    const int cl = wave * 64 + lr * 4;                 // this lane's 4 centroids within the tile
    const double n0 = nb[0], n1 = nb[1], n2 = nb[2], n3 = nb[3];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int ql = mt * 16 + v * 4 + lk;
            const int q = q0 + ql;
            if (q >= nq) continue;
            const double yy = ny[ql];
            float4 o;
            o.x = static_cast<float>(fmax(0.0, (yy + n0) - 2.0 * acc[mt][0][v]));
            o.y = static_cast<float>(fmax(0.0, (yy + n1) - 2.0 * acc[mt][1][v]));
            o.z = static_cast<float>(fmax(0.0, (yy + n2) - 2.0 * acc[mt][2][v]));
            o.w = static_cast<float>(fmax(0.0, (yy + n3) - 2.0 * acc[mt][3][v]));
            float *dst = tables + (static_cast<size_t>(q) * m + j) * ncent + c0 + cl;
            if (c0 + cl + 3 < ncent && (ncent & 3) == 0) {
                *reinterpret_cast<float4 *>(dst) = o;
            } else {
                const float ov[4] = {o.x, o.y, o.z, o.w};
                for (int z = 0; z < 4; ++z)
                    if (c0 + cl + z < ncent) dst[z] = ov[z];
            }
        }
    }
}

// Same computation for sub-spaces of at most 64 dimensions, laid out for the store stream: a workgroup
// keeps its 256 centroids (as MFMA B operands, 4 * KS doubles per lane, KS = ceil(dsub / 4)) and their
// norms in registers and walks TQ queries in sub-tiles of 16, so the codebook is read once per
// TQ queries and every wavefront alternates a few MFMAs with 16 KiB of table stores.  Loading the B
// operands is a strided, latency-bound read (one centroid per lane and component); for wide sub-spaces
// (many components, and 64 cycles of MFMA per component step) TQ is larger so that it stays a small
// part of a workgroup's time.
template <int KS, int TQ>
__global__ __launch_bounds__(256) void full_tables_stream_kernel(const float *__restrict__ queries, int nq,
                                                                 const float *__restrict__ cb, int m, int dsub,
                                                                 int ncent, float *__restrict__ tables)
{
    __shared__ double ny[TQ];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int j = blockIdx.z;
    const int q0 = blockIdx.y * TQ;
    const int c0 = blockIdx.x * kTileC;
    const int D = m * dsub;
    const float *cbj = cb + static_cast<size_t>(j) * ncent * dsub;
    const int lr = lane & 15, lk = lane >> 4;

    for (int ql = tid; ql < TQ; ql += 256) {             // query norms in fp64
        double sy = 0.0;
        if (q0 + ql < nq) {
            const float *y = queries + static_cast<size_t>(q0 + ql) * D + j * dsub;
            for (int t = 0; t < dsub; ++t) { const double v = y[t]; sy += v * v; }
        }
        ny[ql] = sy;
    }

    // B operands: lane (lr, lk) holds components 4 * ks + lk of centroids cw + 4 * lr + nt
    const int cw = c0 + wave * 64;
    double b[KS][4];
    double nc[4] = {0.0, 0.0, 0.0, 0.0};
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
        const int k = 4 * ks + lk;
#pragma unroll
        for (int nt = 0; nt < 4; ++nt) {
            const int c = cw + lr * 4 + nt;
            // the load itself is unconditional (clamped address): a guarded load would be waited for on its own
            const float bv = cbj[static_cast<size_t>(c < ncent ? c : ncent - 1) * dsub + (k < dsub ? k : dsub - 1)];
            b[ks][nt] = (k < dsub && c < ncent) ? static_cast<double>(bv) : 0.0;
            nc[nt] += b[ks][nt] * b[ks][nt];
        }
    }
#pragma unroll
    for (int nt = 0; nt < 4; ++nt) {                     // sum the four component residues: full squared norms
        nc[nt] += __shfl_xor(nc[nt], 16);
        nc[nt] += __shfl_xor(nc[nt], 32);
    }
    __syncthreads();                                     // query norms visible

    const int cl = wave * 64 + lr * 4;                   // this lane's 4 centroids within the tile
    const bool vec_ok = c0 + cl + 3 < ncent && (ncent & 3) == 0;
    for (int mt = 0; mt < TQ / 16; ++mt) {
        if (q0 + mt * 16 >= nq) break;                   // uniform
        const int qa = q0 + mt * 16 + lr;
        double4_t acc[4];
#pragma unroll
        for (int nt = 0; nt < 4; ++nt) acc[nt] = double4_t{0.0, 0.0, 0.0, 0.0};
        double a[KS];
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            const int k = 4 * ks + lk;
            const float av = queries[static_cast<size_t>(qa < nq ? qa : nq - 1) * D + j * dsub + (k < dsub ? k : dsub - 1)];
            a[ks] = (k < dsub && qa < nq) ? static_cast<double>(av) : 0.0;
        }
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
#pragma unroll
            for (int nt = 0; nt < 4; ++nt)
                acc[nt] = __builtin_amdgcn_mfma_f64_16x16x4f64(a[ks], b[ks][nt], acc[nt], 0, 0, 0);
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int ql = mt * 16 + v * 4 + lk;
            const int q = q0 + ql;
            if (q >= nq) continue;
            const double yy = ny[ql];
            float4 o;
            o.x = static_cast<float>(fmax(0.0, (yy + nc[0]) - 2.0 * acc[0][v]));
            o.y = static_cast<float>(fmax(0.0, (yy + nc[1]) - 2.0 * acc[1][v]));
            o.z = static_cast<float>(fmax(0.0, (yy + nc[2]) - 2.0 * acc[2][v]));
            o.w = static_cast<float>(fmax(0.0, (yy + nc[3]) - 2.0 * acc[3][v]));
            float *dst = tables + (static_cast<size_t>(q) * m + j) * ncent + c0 + cl;
            if (vec_ok) {
                *reinterpret_cast<float4 *>(dst) = o;
            } else {
                const float ov[4] = {o.x, o.y, o.z, o.w};
                for (int z = 0; z < 4; ++z)
                    if (c0 + cl + z < ncent) dst[z] = ov[z];
            }
        }
    }
}

template <int KS, int TQ>
static void launch_stream(const float *queries, int nq, const float *codebooks, int m, int dsub, int ncent,
                          float *tables, int stage, hipStream_t st)
{
    const dim3 grid((ncent + kTileC - 1) / kTileC, (nq + TQ - 1) / TQ, m);
    DCPQ_LAUNCH(stage, st, (full_tables_stream_kernel<KS, TQ>), grid, dim3(256), 0, queries, nq, codebooks, m, dsub, ncent,
                tables);
}

int launch_distance_tables(const float *queries, int nq, const float *codebooks, int m, int dsub, int ncent,
                           float *tables, int stage, hipStream_t st)
{
    if (nq == 0) return DCPQ_OK;
    const int ks = (dsub + 3) / 4;
    if (ks <= 3) launch_stream<3, 128>(queries, nq, codebooks, m, dsub, ncent, tables, stage, st);
    else if (ks <= 4) launch_stream<4, 128>(queries, nq, codebooks, m, dsub, ncent, tables, stage, st);
    else if (ks <= 8) launch_stream<8, 256>(queries, nq, codebooks, m, dsub, ncent, tables, stage, st);
    else if (ks <= 16) launch_stream<16, 512>(queries, nq, codebooks, m, dsub, ncent, tables, stage, st);
    else {
        const uint64_t wgs = static_cast<uint64_t>((ncent + kTileC - 1) / kTileC) * static_cast<uint64_t>((nq + kTileQ - 1) / kTileQ);
        if (wgs > 0x7fffffffull) return fail(DCPQ_EINVAL, "distance tables: %d queries x %d centroids are too many for one launch", nq, ncent);
        const dim3 grid(static_cast<unsigned>(wgs), 1, m);
        DCPQ_LAUNCH(stage, st, full_tables_kernel, grid, dim3(256), 0, queries, nq, codebooks, m, dsub, ncent, tables);
    }
    DCPQ_CHECK_LAUNCH("full_tables_kernel");
    return DCPQ_OK;
}

int launch_full_tables(const float *queries, int nq, const float *codebooks, int m, int dsub,
                       float *tables, hipStream_t st)
{
    return launch_distance_tables(queries, nq, codebooks, m, dsub, kFullSize, tables, kStageFullTables, st);
}

}  // namespace dcpq

using namespace dcpq;

extern "C" int dcpq_build_tables(const float *queries, int nq, const float *codebooks, int m, int dsub,
                                 float *tables, void *stream)
{
    clear_error();
    DCPQ_REQUIRE(nq >= 0, "build_tables: nq=%d", nq);
    if (!dcpq_shape_supported(m, dsub)) return fail(DCPQ_EUNSUPPORTED, "build_tables: m=%d dsub=%d not supported", m, dsub);
    if (nq == 0) return DCPQ_OK;
    DCPQ_REQUIRE(queries && codebooks && tables, "build_tables: null pointer");
    DCPQ_REQUIRE((reinterpret_cast<uintptr_t>(tables) & 15) == 0, "build_tables: tables must be 16-byte aligned");
    return launch_full_tables(queries, nq, codebooks, m, dsub, tables, as_stream(stream));
}

extern "C" int dcpq_build_tables_n(const float *queries, int nq, const float *codebooks, int m, int dsub, int n_entries,
                                   float *tables, void *stream)
{
    clear_error();
    DCPQ_REQUIRE(nq >= 0, "build_tables_n: nq=%d", nq);
    if (!dcpq_shape_supported(m, dsub)) return fail(DCPQ_EUNSUPPORTED, "build_tables_n: m=%d dsub=%d not supported", m, dsub);
    DCPQ_REQUIRE(n_entries >= 1 && n_entries <= kFullSize, "build_tables_n: n_entries=%d", n_entries);
    if (nq == 0) return DCPQ_OK;
    DCPQ_REQUIRE(queries && codebooks && tables, "build_tables_n: null pointer");
    DCPQ_REQUIRE((reinterpret_cast<uintptr_t>(tables) & 15) == 0, "build_tables_n: tables must be 16-byte aligned");
    return launch_distance_tables(queries, nq, codebooks, m, dsub, n_entries, tables, kStageFullTables, as_stream(stream));
}
