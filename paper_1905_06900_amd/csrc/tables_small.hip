// Derived codebooks (Sec. 3.2) and the small-table / quantization stage of Alg. 3 (Sec. 3.3,
// "Tables step").  Everything here feeds an integer decision, so the arithmetic is plain fp32
// with one rounding per operation in a fixed order: no FMA contraction (explicit *_rn
// intrinsics), correctly rounded division, sequential accumulation.
#include "common.h"
#include "device_util.h"

namespace dcpq {

// derived[j][l][t] = (sum_i cb[j][(i << bbar) | l][t]) / 2^(b - bbar), i = 0 .. 2^(b - bbar) - 1 increasing
// (Sec. 3.2: the derived centroid is the mean of the group of centroids that share the low bbar
// bits).  One thread per output element; for a fixed i the threads of a block read one contiguous
// run of 2^bbar * dsub floats, so the loads coalesce.
__global__ __launch_bounds__(256) void derive_kernel(const float *__restrict__ cb, int dsub, int full_size,
                                                     int small_bits, float *__restrict__ derived)
{
    const int j = blockIdx.y;
    const int per_sub = dsub << small_bits;                // floats in one derived codebook
    const int groups = full_size >> small_bits;
    const int e = blockIdx.x * blockDim.x + threadIdx.x;   // l * dsub + t
    if (e >= per_sub) return;
    const float *base = cb + static_cast<size_t>(j) * full_size * dsub + e;
    float acc = 0.0f;
    for (int i = 0; i < groups; ++i)
        acc = __fadd_rn(acc, base[static_cast<size_t>(i) * per_sub]);
    derived[static_cast<size_t>(j) * per_sub + e] = __fdiv_rn(acc, static_cast<float>(groups));
}

// One workgroup per query.  LDS: the query (D floats) and its m * 2^bbar small-table entries.
// The quantized tables are written with 256 entries each whatever bbar is: entry e holds the
// quantized distance of derived centroid (e mod 2^bbar), so that a scan which looks a table up by
// the low BYTE of a sub-code gets the entry of its low bbar BITS (property P1 of Sec. 3.1 for any
// bbar <= 8).  `small`, when asked for, keeps the 2^bbar floating-point entries as they are.
template <int M, typename CodeT>
__global__ __launch_bounds__(256) void small_tables_kernel(
    const float *__restrict__ queries, const float *__restrict__ derived, int dsub, int small_bits,
    const CodeT *__restrict__ codes, uint32_t n_first, uint8_t *__restrict__ qtab,
    float *__restrict__ bounds, float *__restrict__ small)
{
    extern __shared__ float lds[];
    float *ly = lds;                       // [M*dsub]
    float *ltab = lds + M * dsub;          // [M][2^bbar]
    __shared__ float red[4];
    const int q = blockIdx.x, tid = threadIdx.x;
    const int D = M * dsub;
    const int ks = 1 << small_bits, mask = ks - 1;
    for (int t = tid; t < D; t += 256) ly[t] = queries[static_cast<size_t>(q) * D + t];
    __syncthreads();

    // Eq. 1 on the derived codebooks: thread i owns entry i of every table.
    const bool vec4 = (dsub & 3) == 0 && (reinterpret_cast<uintptr_t>(derived) & 15) == 0;      // uniform
    float lo = INFINITY;
    if (tid < ks) {
        for (int j = 0; j < M; ++j) {
            const float *c = derived + (static_cast<size_t>(j) * ks + tid) * dsub;
            float acc = 0.0f;
            if (vec4) {
                // a centroid row as 16-byte vectors (a thread reads its own row: 4-byte loads would touch as many
                // memory lines four times as often); the squares are still added one by one in ascending t
                for (int t = 0; t < dsub; t += 4) {
                    const float4 c4 = *reinterpret_cast<const float4 *>(c + t);
                    float diff = __fsub_rn(ly[j * dsub + t], c4.x);
                    acc = __fadd_rn(acc, __fmul_rn(diff, diff));
                    diff = __fsub_rn(ly[j * dsub + t + 1], c4.y);
                    acc = __fadd_rn(acc, __fmul_rn(diff, diff));
                    diff = __fsub_rn(ly[j * dsub + t + 2], c4.z);
                    acc = __fadd_rn(acc, __fmul_rn(diff, diff));
                    diff = __fsub_rn(ly[j * dsub + t + 3], c4.w);
                    acc = __fadd_rn(acc, __fmul_rn(diff, diff));
                }
            } else {
                for (int t = 0; t < dsub; ++t) {
                    const float diff = __fsub_rn(ly[j * dsub + t], c[t]);
                    acc = __fadd_rn(acc, __fmul_rn(diff, diff));
                }
            }
            ltab[j * ks + tid] = acc;
            lo = fminf(lo, acc);
        }
    }
    const float qmin = block_reduce(lo, false, red);   // also publishes ltab (barriers inside)

    // qmax: largest small-table distance to the first n_first codes, sum over j increasing.
    float hi = -INFINITY;
    for (uint32_t i = tid; i < n_first; i += 256) {
        const CodeT *c = codes + static_cast<size_t>(i) * M;
        float d = ltab[c[0] & mask];
        for (int j = 1; j < M; ++j) d = __fadd_rn(d, ltab[j * ks + (c[j] & mask)]);
        hi = fmaxf(hi, d);
    }
    const float qmax = block_reduce(hi, true, red);

    for (int j = 0; j < M; ++j) {
        const float v = ltab[j * ks + (tid & mask)];
        qtab[(static_cast<size_t>(q) * M + j) * kSmallSize + tid] = quantize_entry(v, qmin, qmax);
        if (small && tid < ks) small[(static_cast<size_t>(q) * M + j) * ks + tid] = v;
    }
    if (tid == 0) { bounds[2 * q] = qmin; bounds[2 * q + 1] = qmax; }
}

template <typename CodeT>
static int launch_small_tables_t(const float *queries, int nq, const float *derived, int m, int dsub, int small_bits,
                                 const CodeT *codes, uint64_t n_codes, uint32_t r, uint8_t *qtab,
                                 float *bounds, float *small, hipStream_t st)
{
    if (nq == 0) return DCPQ_OK;
    const uint32_t n_first = static_cast<uint32_t>(r < n_codes ? r : n_codes);
    const size_t lds = sizeof(float) * (static_cast<size_t>(m) * dsub + (static_cast<size_t>(m) << small_bits));
#define DCPQ_LAUNCH_SMALL(MV)                                                                                 \
    case MV:                                                                                                  \
        DCPQ_LAUNCH(kStageSmallTables, st, (small_tables_kernel<MV, CodeT>), dim3(nq), dim3(256), lds, queries, \
                    derived, dsub, small_bits, codes, n_first, qtab, bounds, small);                          \
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

int launch_small_tables(const float *queries, int nq, const float *derived, int m, int dsub, int small_bits,
                        const void *codes, int code_bytes, uint64_t n_codes, uint32_t r, uint8_t *qtab,
                        float *bounds, float *small, hipStream_t st)
{
    if (code_bytes == 1)
        return launch_small_tables_t(queries, nq, derived, m, dsub, small_bits, static_cast<const uint8_t *>(codes),
                                     n_codes, r, qtab, bounds, small, st);
    return launch_small_tables_t(queries, nq, derived, m, dsub, small_bits, static_cast<const uint16_t *>(codes),
                                 n_codes, r, qtab, bounds, small, st);
}

int launch_derive(const float *codebooks, int m, int dsub, int full_bits, int small_bits, float *derived, hipStream_t st)
{
    const int per_sub = dsub << small_bits;
    hipLaunchKernelGGL(derive_kernel, dim3((per_sub + 255) / 256, m), dim3(256), 0, st, codebooks, dsub, 1 << full_bits,
                       small_bits, derived);
    DCPQ_CHECK_LAUNCH("derive_kernel");
    return DCPQ_OK;
}

}  // namespace dcpq

using namespace dcpq;

extern "C" int dcpq_shape_supported(int m, int dsub)
{
    return (m_supported(m) && dsub >= 1 && dsub <= 128) ? 1 : 0;
}

extern "C" int dcpq_bits_supported(int b, int bbar)
{
    return ((b == 8 || b == 16) && bbar >= 1 && bbar <= 8 && bbar <= b) ? 1 : 0;
}

extern "C" int dcpq_derive_codebooks_bits(const float *codebooks, int m, int dsub, int b, int bbar, float *derived,
                                          void *stream)
{
    clear_error();
    DCPQ_REQUIRE(codebooks && derived, "derive_codebooks: null pointer");
    if (!dcpq_shape_supported(m, dsub)) return fail(DCPQ_EUNSUPPORTED, "derive_codebooks: m=%d dsub=%d not supported", m, dsub);
    if (!dcpq_bits_supported(b, bbar)) return fail(DCPQ_EUNSUPPORTED, "derive_codebooks: b=%d bbar=%d not supported", b, bbar);
    return launch_derive(codebooks, m, dsub, b, bbar, derived, as_stream(stream));
}

extern "C" int dcpq_derive_codebooks(const float *codebooks, int m, int dsub, float *derived, void *stream)
{
    return dcpq_derive_codebooks_bits(codebooks, m, dsub, kFullBits, kSmallBits, derived, stream);
}

extern "C" int dcpq_build_small_tables_bits(const float *queries, int nq, const float *derived, int m, int dsub,
                                            int bbar, const void *codes, int code_bytes, uint64_t n_codes, uint32_t r,
                                            uint8_t *qtab, float *bounds, float *small, void *stream)
{
    clear_error();
    DCPQ_REQUIRE(nq >= 0, "build_small_tables: nq=%d", nq);
    if (!dcpq_shape_supported(m, dsub)) return fail(DCPQ_EUNSUPPORTED, "build_small_tables: m=%d dsub=%d not supported", m, dsub);
    DCPQ_REQUIRE(code_bytes == 1 || code_bytes == 2, "build_small_tables: code_bytes=%d (1 or 2)", code_bytes);
    if (!dcpq_bits_supported(8 * code_bytes, bbar))
        return fail(DCPQ_EUNSUPPORTED, "build_small_tables: bbar=%d with %d-byte sub-codes not supported", bbar, code_bytes);
    if (nq == 0) return DCPQ_OK;
    DCPQ_REQUIRE(queries && derived && qtab && bounds, "build_small_tables: null pointer");
    DCPQ_REQUIRE(r >= 1 && n_codes >= 1 && codes, "build_small_tables: needs r >= 1 and at least one code (qmax is taken over the first r codes)");
    return launch_small_tables(queries, nq, derived, m, dsub, bbar, codes, code_bytes, n_codes, r, qtab, bounds, small,
                               as_stream(stream));
}

extern "C" int dcpq_build_small_tables(const float *queries, int nq, const float *derived, int m, int dsub,
                                       const uint16_t *codes, uint64_t n_codes, uint32_t r, uint8_t *qtab,
                                       float *bounds, float *small, void *stream)
{
    return dcpq_build_small_tables_bits(queries, nq, derived, m, dsub, kSmallBits, codes, 2, n_codes, r, qtab, bounds,
                                        small, stream);
}
