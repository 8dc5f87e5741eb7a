// Internal helpers shared by the translation units of libdcpq (not part of the ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>

#include "dcpq.h"

namespace dcpq {

constexpr int kFullBits = 16;          // b: bits of a sub-code
constexpr int kFullSize = 1 << 16;     // centroids per sub-quantizer
constexpr int kSmallBits = 8;          // bbar: bits of a derived-codebook index
constexpr int kSmallSize = 1 << 8;     // centroids per derived codebook
constexpr int kWave = 64;              // wavefront width on gfx950

// Records a message for dcpq_last_error() and returns `code`.
int fail(int code, const char *fmt, ...);
void clear_error();

inline hipStream_t as_stream(void *s) { return reinterpret_cast<hipStream_t>(s); }

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

#define DCPQ_CHECK_HIP(expr)                                                                   \
    do {                                                                                       \
        hipError_t e_ = (expr);                                                                \
        if (e_ != hipSuccess)                                                                  \
            return ::dcpq::fail(DCPQ_EHIP, "%s failed: %s", #expr, hipGetErrorString(e_));     \
    } while (0)

#define DCPQ_CHECK_LAUNCH(name)                                                                \
    do {                                                                                       \
        hipError_t e_ = hipGetLastError();                                                     \
        if (e_ != hipSuccess)                                                                  \
            return ::dcpq::fail(DCPQ_EHIP, "launch of %s failed: %s", name,                    \
                                hipGetErrorString(e_));                                        \
    } while (0)

#define DCPQ_REQUIRE(cond, ...)                                                                \
    do {                                                                                       \
        if (!(cond)) return ::dcpq::fail(DCPQ_EINVAL, __VA_ARGS__);                            \
    } while (0)

// Stages reported by the optional event-based profiler (dcpq_profile_*).
enum Stage {
    kStageSmallTables = 0, kStageScanHist, kStageScanTieCount, kStageScanCollect, kStageScanFast,
    kStageSelect, kStageFullTables, kStageRefine, kStageIvf, kStageMisc,
    kStageIvfProbe, kStageIvfTables, kStageIvfScan, kStageIvfRefine, kStagePlainScan, kStageTrain, kNumStages
};
namespace prof {
bool enabled();
void *begin(int stage, hipStream_t st);      // returns a token for end(), or nullptr when disabled
void end(void *token, hipStream_t st);
}  // namespace prof

// Launches a kernel, bracketed by profiler events when profiling is on.
#define DCPQ_LAUNCH(stage, st, kernel, grid, block, lds, ...)                                  \
    do {                                                                                       \
        void *tok_ = ::dcpq::prof::begin(stage, st);                                           \
        hipLaunchKernelGGL(kernel, grid, block, lds, st, __VA_ARGS__);                         \
        ::dcpq::prof::end(tok_, st);                                                           \
    } while (0)

// Raises a kernel's dynamic LDS limit to `bytes` (needed above 64 KiB) once per (device, kernel); when
// `no_static_lds` is set, also checks that the kernel has no static LDS of its own (kernels that
// address their dynamic LDS from offset 0 rely on it).  Thread-safe.
int allow_dynamic_lds(const void *kernel, int bytes, bool no_static_lds = false);

inline bool m_supported(int m) { return m == 1 || m == 2 || m == 4 || m == 8 || m == 16 || m == 32; }

// Sortable 64-bit key: major part in the high word, vector id in the low word.
__host__ __device__ inline uint64_t make_key(uint32_t major, uint32_t id)
{
    return (static_cast<uint64_t>(major) << 32) | id;
}

// Internal launchers used by dcpq_search (same contracts as the public calls, no validation).
// small_bits = bbar; codes: uint8 (code_bytes 1) or uint16 (2) sub-codes
int launch_small_tables(const float *queries, int nq, const float *derived, int m, int dsub, int small_bits,
                        const void *codes, int code_bytes, uint64_t n_codes, uint32_t r, uint8_t *qtab,
                        float *bounds, float *small, hipStream_t st);
int launch_derive(const float *codebooks, int m, int dsub, int full_bits, int small_bits, float *derived, hipStream_t st);
int launch_full_tables(const float *queries, int nq, const float *codebooks, int m, int dsub,
                       float *tables, hipStream_t st);
// Same kernel for any number of centroids (the coarse quantizer: m = 1, dsub = D, ncent = nlist).
int launch_distance_tables(const float *queries, int nq, const float *codebooks, int m, int dsub, int ncent,
                           float *tables, int stage, hipStream_t st);
// mode: DCPQ_SCAN_AUTO or DCPQ_SCAN_THREE_PASS
int launch_scan(const uint16_t *codes, uint64_t n_codes, int m, const uint8_t *qtab, int nq,
                uint32_t r, uint32_t *cand_id, uint8_t *cand_qd, void *ws, int mode, hipStream_t st);
// the same reading the low-byte plane of the codes (uint8 [n_codes][m])
int launch_scan(const uint8_t *plane, uint64_t n_codes, int m, const uint8_t *qtab, int nq,
                uint32_t r, uint32_t *cand_id, uint8_t *cand_qd, void *ws, int mode, hipStream_t st);
int launch_refine(const float *tables, uint32_t table_size, const void *codes, int code_bytes, uint64_t n_codes, int m,
                  const uint32_t *cand_id, int nq, uint32_t r, uint32_t k, uint32_t *ids, float *dist, void *ws,
                  hipStream_t st);
// the same with every table entry computed on demand from the codebooks (no tables)
// codebooks: rows of dsub floats, cstride floats apart (16-byte aligned rows when dsub is a multiple of 4)
int launch_pad_rows(const float *src, size_t nrows, int dsub, int cstride, float *dst, hipStream_t st);
int launch_refine_direct(const float *queries, const float *codebooks, int dsub, int cstride, uint32_t table_size, const void *codes,
                         int code_bytes, uint64_t n_codes, int m, const uint32_t *cand_id, int nq, uint32_t r, uint32_t k,
                         uint32_t *ids, float *dist, void *ws, hipStream_t st);
// the same in three kernels, split by sub-quantizer so that each XCD's cache keeps one sub-codebook; `mid`:
// refine_split_bytes(...) bytes, 256-byte aligned; nq * r must fit 32 bits
size_t refine_split_bytes(int nq, uint32_t r, int m, int code_bytes);
int launch_refine_split(const float *queries, const float *codebooks, int dsub, uint32_t table_size, const void *codes,
                        int code_bytes, uint64_t n_codes, int m, const uint32_t *cand_id, int nq, uint32_t r, uint32_t k,
                        uint32_t *ids, float *dist, void *mid, void *ws, hipStream_t st);

}  // namespace dcpq
