// Derived codebooks (Sec. 3.2) and the small-table / quantization stage of Alg. 3 (Sec. 3.3,
// "Tables step").  Everything here feeds an integer decision, so the arithmetic is plain fp32
// with one rounding per operation in a fixed order: no FMA contraction (explicit *_rn
// intrinsics), correctly rounded division, sequential accumulation.
#include "common.h"

namespace dcpq {

// derived[j][l][t] = (sum_{i=0}^{255} cb[j][(i << 8) | l][t]) / 256, i increasing.
// One thread per output element; for a fixed i the threads of a block read one contiguous
// run of 256*dsub floats, so the loads coalesce.
__global__ __launch_bounds__(256) void derive_kernel(const float *__restrict__ cb, int dsub,
                                                     float *__restrict__ derived)
{
    const int j = blockIdx.y;
    const int per_sub = kSmallSize * dsub;                 // floats in one derived codebook
    const int e = blockIdx.x * blockDim.x + threadIdx.x;   // l * dsub + t
    if (e >= per_sub) return;
    const float *base = cb + static_cast<size_t>(j) * kFullSize * dsub + e;
    float acc = 0.0f;
    for (int i = 0; i < kFullSize / kSmallSize; ++i)
        acc = __fadd_rn(acc, base[static_cast<size_t>(i) * per_sub]);
    derived[static_cast<size_t>(j) * per_sub + e] = __fdiv_rn(acc, 256.0f);
}

__device__ inline float block_reduce(float v, bool want_max, float *red)
{
    // 256 threads = 4 wavefronts; wave reduction by cross-lane shuffles, then via LDS.
    for (int off = 32; off > 0; off >>= 1) {
        float o = __shfl_xor(v, off, kWave);
        v = want_max ? fmaxf(v, o) : fminf(v, o);
    }
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    __syncthreads();
    if (lane == 0) red[wave] = v;
    __syncthreads();
    float out = red[0];
    for (int w = 1; w < 4; ++w) out = want_max ? fmaxf(out, red[w]) : fminf(out, red[w]);
    return out;
}

// One workgroup per query.  LDS: the query (D floats) and its m*256 small-table entries.
template <int M>
__global__ __launch_bounds__(256) void small_tables_kernel(
    const float *__restrict__ queries, const float *__restrict__ derived, int dsub,
    const uint16_t *__restrict__ codes, uint32_t n_first, uint8_t *__restrict__ qtab,
    float *__restrict__ bounds, float *__restrict__ small)
{
    extern __shared__ float lds[];
    float *ly = lds;                       // [M*dsub]
    float *ltab = lds + M * dsub;          // [M][256]
    __shared__ float red[4];
    const int q = blockIdx.x, tid = threadIdx.x;
    const int D = M * dsub;
    for (int t = tid; t < D; t += 256) ly[t] = queries[static_cast<size_t>(q) * D + t];
    __syncthreads();

    // Eq. 1 on the derived codebooks: thread i owns entry i of every table.
    float lo = INFINITY;
    for (int j = 0; j < M; ++j) {
        const float *c = derived + (static_cast<size_t>(j) * kSmallSize + tid) * dsub;
        float acc = 0.0f;
        for (int t = 0; t < dsub; ++t) {
            const float diff = __fsub_rn(ly[j * dsub + t], c[t]);
            acc = __fadd_rn(acc, __fmul_rn(diff, diff));
        }
        ltab[j * kSmallSize + tid] = acc;
        lo = fminf(lo, acc);
    }
    const float qmin = block_reduce(lo, false, red);   // also publishes ltab (barriers inside)

    // qmax: largest small-table distance to the first n_first codes, sum over j increasing.
    float hi = -INFINITY;
    for (uint32_t i = tid; i < n_first; i += 256) {
        const uint16_t *c = codes + static_cast<size_t>(i) * M;
        float d = ltab[c[0] & 255];
        for (int j = 1; j < M; ++j) d = __fadd_rn(d, ltab[j * kSmallSize + (c[j] & 255)]);
        hi = fmaxf(hi, d);
    }
    const float qmax = block_reduce(hi, true, red);

    const float den = __fsub_rn(qmax, qmin);
    for (int j = 0; j < M; ++j) {
        const float v = ltab[j * kSmallSize + tid];
        uint8_t code = 0;
        if (den > 0.0f) {
            const float u = __fmul_rn(__fdiv_rn(__fsub_rn(v, qmin), den), 255.0f);
            code = (u >= 255.0f) ? static_cast<uint8_t>(255) : static_cast<uint8_t>(floorf(u));
        }
        const size_t o = (static_cast<size_t>(q) * M + j) * kSmallSize + tid;
        qtab[o] = code;
        if (small) small[o] = v;
    }
    if (tid == 0) { bounds[2 * q] = qmin; bounds[2 * q + 1] = qmax; }
}

int launch_small_tables(const float *queries, int nq, const float *derived, int m, int dsub,
                        const uint16_t *codes, uint64_t n_codes, uint32_t r, uint8_t *qtab,
                        float *bounds, float *small, hipStream_t st)
{
    if (nq == 0) return DCPQ_OK;
    const uint32_t n_first = static_cast<uint32_t>(r < n_codes ? r : n_codes);
    const size_t lds = sizeof(float) * (static_cast<size_t>(m) * dsub + static_cast<size_t>(m) * kSmallSize);
#define DCPQ_LAUNCH_SMALL(MV)                                                                        \
    case MV:                                                                                         \
        DCPQ_LAUNCH(kStageSmallTables, st, small_tables_kernel<MV>, dim3(nq), dim3(256), lds, queries,   \
                    derived, dsub, codes, n_first, qtab, bounds, small);                             \
        break;
    switch (m) {
        DCPQ_LAUNCH_SMALL(1) DCPQ_LAUNCH_SMALL(2) DCPQ_LAUNCH_SMALL(4) DCPQ_LAUNCH_SMALL(8)
        DCPQ_LAUNCH_SMALL(16) DCPQ_LAUNCH_SMALL(32)
        default: return fail(DCPQ_EUNSUPPORTED, "m=%d not supported", m);
    }
#undef DCPQ_LAUNCH_SMALL
    DCPQ_CHECK_LAUNCH("small_tables_kernel");
    return DCPQ_OK;
}

}  // namespace dcpq

using namespace dcpq;

extern "C" int dcpq_shape_supported(int m, int dsub)
{
    return (m_supported(m) && dsub >= 1 && dsub <= 128) ? 1 : 0;
}

extern "C" int dcpq_derive_codebooks(const float *codebooks, int m, int dsub, float *derived, void *stream)
{
    clear_error();
    DCPQ_REQUIRE(codebooks && derived, "derive_codebooks: null pointer");
    if (!dcpq_shape_supported(m, dsub)) return fail(DCPQ_EUNSUPPORTED, "derive_codebooks: m=%d dsub=%d not supported", m, dsub);
    const int per_sub = kSmallSize * dsub;
    hipLaunchKernelGGL(derive_kernel, dim3((per_sub + 255) / 256, m), dim3(256), 0, as_stream(stream),
                       codebooks, dsub, derived);
    DCPQ_CHECK_LAUNCH("derive_kernel");
    return DCPQ_OK;
}

extern "C" int dcpq_build_small_tables(const float *queries, int nq, const float *derived, int m, int dsub,
                                       const uint16_t *codes, uint64_t n_codes, uint32_t r, uint8_t *qtab,
                                       float *bounds, float *small, void *stream)
{
    clear_error();
    DCPQ_REQUIRE(nq >= 0, "build_small_tables: nq=%d", nq);
    if (!dcpq_shape_supported(m, dsub)) return fail(DCPQ_EUNSUPPORTED, "build_small_tables: m=%d dsub=%d not supported", m, dsub);
    if (nq == 0) return DCPQ_OK;
    DCPQ_REQUIRE(queries && derived && qtab && bounds, "build_small_tables: null pointer");
    DCPQ_REQUIRE(r >= 1 && n_codes >= 1 && codes, "build_small_tables: needs r >= 1 and at least one code (qmax is taken over the first r codes)");
    return launch_small_tables(queries, nq, derived, m, dsub, codes, n_codes, r, qtab, bounds, small, as_stream(stream));
}
