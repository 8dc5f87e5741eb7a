// Inner products of a 16 MT x 64 tile on the double-precision matrix cores, shared by the distance-table
// kernel and the nearest-centroid kernel (HIP translation units only).
#pragma once

#include <type_traits>

#include "common.h"

namespace dcpq {

typedef double double4_t __attribute__((ext_vector_type(4)));

// Four consecutive floats that need only 4-byte alignment (rows of 12 or 60 floats start anywhere).
struct __attribute__((packed, aligned(4))) float4_any { float v[4]; };

// Up to four consecutive floats of a row; n is uniform over the wavefront.
__device__ inline void load_run(const float *p, int n, float (&out)[4])
{
    if (n == 4) {
        const float4_any x = *reinterpret_cast<const float4_any *>(p);
        out[0] = x.v[0]; out[1] = x.v[1]; out[2] = x.v[2]; out[3] = x.v[3];
    } else {
        out[0] = p[0];
        out[1] = n > 1 ? p[1] : 0.0f;
        out[2] = n > 2 ? p[2] : 0.0f;
        out[3] = 0.0f;
    }
}

// acc[mt][nt] += A_mt x B_nt over the dsub components (v_mfma_f64_16x16x4_f64: lane l supplies row l % 16 of A
// and column l % 16 of B for component slot l / 16 of every step), na / nb += this lane's share of the squared
// norms of its A rows / B columns (the four slots l / 16 together hold a whole norm).
//   arow[mt], brow[nt]: this lane's rows (16 mt + l % 16 of A; its four columns of B), already clamped to
//   valid rows -- rows past the end give values the caller never uses.
// A sum over components does not care in which order they come, so when dsub is a multiple of 4 slot g does
// not take components g, g + 4, g + 8, ... (a 4-byte load per lane, row and step, 64 scattered requests per
// instruction: the address path, not the matrix pipe, then sets the pace) but runs of four consecutive floats,
// fetched as 16-byte loads four steps ahead of their use: the g-th 16 bytes of every 64-byte piece of the row
// when dsub is a multiple of 16, else the g-th quarter of the row.
template <int MT>
__device__ inline void f64_tile_products(const float *const (&arow)[MT], const float *const (&brow)[4], int dsub, int slot,
                                         bool want_na, double4_t (&acc)[MT][4], double (&na)[MT], double (&nb)[4])
{
    if ((dsub & 15) == 0) {
        // Rows of whole 64-byte pieces: the four slots share each piece (slot g its g-th 16 bytes), so that the 64
        // loads of an instruction fall into 16 memory lines and the next piece finds the other half of each line
        // still in the first-level cache.  (With a quarter of the row per slot every lane walks a line of its own,
        // 16 bytes every four steps, and at 128 components the 256 lines a wavefront has open are the whole cache:
        // measured 115 M requests to the L2 per 1024 x 65536 distances instead of 21 M.)  Two sets of registers take the pieces in turn, so
        // that the loads of one are under way while the other is multiplied, and nothing is copied between them:
        // the ordinary vector instructions share the issue port with the matrix instructions, and at 8 matrix
        // instructions per step every one of them saved counts (6 conversions and 4 to 6 fused norm updates remain).
        const float *ap[MT], *bp[4];
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) ap[mt] = arow[mt] + slot * 4;
#pragma unroll
        for (int nt = 0; nt < 4; ++nt) bp[nt] = brow[nt] + slot * 4;
        auto load_piece = [&](int c, float4_any (&A)[MT], float4_any (&B)[4]) {
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) A[mt] = *reinterpret_cast<const float4_any *>(ap[mt] + 16 * c);
#pragma unroll
            for (int nt = 0; nt < 4; ++nt) B[nt] = *reinterpret_cast<const float4_any *>(bp[nt] + 16 * c);
        };
        // (WANT: std::true_type or std::false_type, so that the norms of the A rows cost nothing where they are
        // not wanted; every load is unconditional, the last one of a piece that is there already: loads behind a
        // branch make the compiler wait for ALL loads in flight where the paths join)
        auto run = [&](auto WANT) {
            auto multiply = [&](const float4_any (&A)[MT], const float4_any (&B)[4]) {
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    double a[MT], b[4];
#pragma unroll
                    for (int mt = 0; mt < MT; ++mt) a[mt] = static_cast<double>(A[mt].v[t]);
#pragma unroll
                    for (int nt = 0; nt < 4; ++nt) b[nt] = static_cast<double>(B[nt].v[t]);
                    if constexpr (decltype(WANT)::value) {
#pragma unroll
                        for (int mt = 0; mt < MT; ++mt) na[mt] = __builtin_fma(a[mt], a[mt], na[mt]);
                    }
#pragma unroll
                    for (int nt = 0; nt < 4; ++nt) nb[nt] = __builtin_fma(b[nt], b[nt], nb[nt]);
#pragma unroll
                    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                        for (int nt = 0; nt < 4; ++nt)
                            acc[mt][nt] = __builtin_amdgcn_mfma_f64_16x16x4f64(a[mt], b[nt], acc[mt][nt], 0, 0, 0);
                }
            };
            const int pieces = dsub >> 4;
            float4_any a0[MT], b0[4], a1[MT], b1[4];
            load_piece(0, a0, b0);
            int c = 0;
            for (; c + 2 <= pieces; c += 2) {
                load_piece(c + 1, a1, b1);
                multiply(a0, b0);
                load_piece(c + 2 < pieces ? c + 2 : pieces - 1, a0, b0);
                multiply(a1, b1);
            }
            if (c < pieces) multiply(a0, b0);                  // an odd count: the last piece is in the first set
        };
        if (want_na) run(std::true_type{});                    // uniform
        else run(std::false_type{});
        return;
    }
    if ((dsub & 3) == 0) {
        const int q = dsub >> 2;
        const float *ap[MT], *bp[4];
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) ap[mt] = arow[mt] + slot * q;
#pragma unroll
        for (int nt = 0; nt < 4; ++nt) bp[nt] = brow[nt] + slot * q;
        float an[MT][4], bn[4][4];
        auto load_chunk = [&](int t0) {
            const int n = q - t0 < 4 ? q - t0 : 4;             // uniform
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) load_run(ap[mt] + t0, n, an[mt]);
#pragma unroll
            for (int nt = 0; nt < 4; ++nt) load_run(bp[nt] + t0, n, bn[nt]);
        };
        load_chunk(0);
        for (int t0 = 0; t0 < q; t0 += 4) {
            float ac[MT][4], bc[4][4];
#pragma unroll
            for (int t = 0; t < 4; ++t) {
#pragma unroll
                for (int mt = 0; mt < MT; ++mt) ac[mt][t] = an[mt][t];
#pragma unroll
                for (int nt = 0; nt < 4; ++nt) bc[nt][t] = bn[nt][t];
            }
            if (t0 + 4 < q) load_chunk(t0 + 4);                // uniform
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                if (t0 + t >= q) break;                        // uniform
                double a[MT], b[4];
#pragma unroll
                for (int mt = 0; mt < MT; ++mt) a[mt] = static_cast<double>(ac[mt][t]);
#pragma unroll
                for (int nt = 0; nt < 4; ++nt) b[nt] = static_cast<double>(bc[nt][t]);
                if (want_na) {
#pragma unroll
                    for (int mt = 0; mt < MT; ++mt) na[mt] += a[mt] * a[mt];
                }
#pragma unroll
                for (int nt = 0; nt < 4; ++nt) nb[nt] += b[nt] * b[nt];
#pragma unroll
                for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                    for (int nt = 0; nt < 4; ++nt)
                        acc[mt][nt] = __builtin_amdgcn_mfma_f64_16x16x4f64(a[mt], b[nt], acc[mt][nt], 0, 0, 0);
            }
        }
        return;
    }
    // any dsub: slot g takes components g, g + 4, ...; the operands of step k0 + 4 are loaded while the matrix
    // instructions of step k0 run, unconditionally from a clamped component (a guarded load would be waited
    // for on its own), and the components past dsub are zeroed in the one tail step
    float av[MT], bv[4];
    auto load_step = [&](int k0) {
        const int k = k0 + slot < dsub ? k0 + slot : dsub - 1;
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) av[mt] = arow[mt][k];
#pragma unroll
        for (int nt = 0; nt < 4; ++nt) bv[nt] = brow[nt][k];
    };
    auto step = [&](int k0, bool tail) {
        const bool kin = !tail || k0 + slot < dsub;
        double a[MT], b[4];
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) a[mt] = kin ? static_cast<double>(av[mt]) : 0.0;
#pragma unroll
        for (int nt = 0; nt < 4; ++nt) b[nt] = kin ? static_cast<double>(bv[nt]) : 0.0;
        if (k0 + 4 < dsub) load_step(k0 + 4);                  // uniform
        if (want_na) {
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) na[mt] += a[mt] * a[mt];
        }
#pragma unroll
        for (int nt = 0; nt < 4; ++nt) nb[nt] += b[nt] * b[nt];
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int nt = 0; nt < 4; ++nt)
                acc[mt][nt] = __builtin_amdgcn_mfma_f64_16x16x4f64(a[mt], b[nt], acc[mt][nt], 0, 0, 0);
    };
    load_step(0);
    const int whole = dsub & ~3;
    for (int k0 = 0; k0 < whole; k0 += 4) step(k0, false);
    if (whole < dsub) step(whole, true);
}

}  // namespace dcpq
