// Host-side launchers of the gfx950 kernels (internal to the library; the public surface is
// include/picospec.h).  Every launcher enqueues on `stream` and returns the launch status.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>
#include <cmath>

#include "rowspan.hpp"

namespace picospec {

constexpr int kMaxK = 4096;          // candidate buffer in LDS holds 16384 entries; k beyond this is refused
constexpr int kMaxV = 1 << 20;
// picospec_round: draft + target rows up to which the two-launch schedule is used (the chip holds 512 compress
// workgroups at a time; beyond that the separate kernels, each with its own launch shape, are as fast or faster)
constexpr int kRoundSmallRows = 512;

// The optimistic pass of the compress kernel takes its threshold from a sample of m elements of a row of V: the value
// of rank r in the sample, and every row element at or above it becomes a candidate.  With f = m / V the sample holds
// X ~ Binomial(k, f) of the row's k largest; the pass finds fewer than k candidates iff X >= r, so
//     r = k f + z sqrt(k f (1 - f)) + z^2 / 3      (mean + z standard deviations + the term that covers small means)
// with z = 4.5 (or 4, see below).  It overflows a buffer of `cap` slots iff the sample holds fewer than r of the row's
// `cap` largest, Binomial(cap, f): r must stay z_over standard deviations below cap f.  A pass that fails either way is
// repeated the careful way, so the margins only trade a rare slow row against the candidates every row carries.
// 0: no rank satisfies both (the careful pass takes the row).  The host evaluates the same function, with a slightly
// larger z_over, to choose the kernel variant.
__host__ __device__ inline int optimistic_rank(int k, int V, int m, int cap, float z_over = 4.45f) {
    const float f = (float)m / (float)V;
    const float lam = (float)k * f, lam_cap = (float)cap * f;
    const float sd_cap = sqrtf(lam_cap * (1.f - f));
    const float zs[2] = {4.5f, 4.0f};
    for (int i = 0; i < 2; ++i) {
        const float r = ceilf(lam + zs[i] * sqrtf(lam * (1.f - f)) + zs[i] * zs[i] * (1.f / 3.f));
        if (lam_cap - r >= z_over * sd_cap) return (int)r;           // (r may exceed k: a short record still takes the fast pass)
    }
    return 0;
}

// Kernels whose dynamic LDS exceeds the 64 KB default need their limit raised once per device and kernel.
// `done` is the caller's per-device record for that kernel; the current device's ordinal comes back in `dev`.
// The record is atomic and the attribute call idempotent: two threads that meet here on a kernel's first use
// both set the same value, and a thread that reads `true` (acquire) finds the attribute set.
constexpr int kMaxDevices = 64;
using DeviceFlags = std::atomic<bool>[kMaxDevices];
inline hipError_t raise_lds_limit_once(const void* kernel, size_t bytes, DeviceFlags& done, int& dev) {
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    if (!done[dev].load(std::memory_order_acquire)) {
        e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
        if (e != hipSuccess) return e;
        done[dev].store(true, std::memory_order_release);
    }
    return hipSuccess;
}

// seq_off / n_accept: both null (record r from row r), or the downlink's row map (record b from target
// row seq_off[b] + b + n_accept[b])
hipError_t launch_compress(const void* logits, int dtype, int64_t ld, int n_rows, int V, float temperature,
                           int k, float top_p, int32_t* idx, float* prob, int32_t* count, float* mass,
                           float* lse, const int32_t* seq_off, const int32_t* n_accept, hipStream_t stream);

// the draft rows' compression and the target rows' statistics in one launch (small rounds)
hipError_t launch_round_stream(const void* draft_logits, int dtype, int64_t ld_d, int n_draft, int V, float temperature,
                               int k, float top_p, int32_t* idx, float* prob, int32_t* count, float* mass, float* lse,
                               const void* tgt_logits, int64_t ld_t, int n_target,
                               float* tgt_max, float* tgt_sum, float* tgt_lse, void* seg_table, hipStream_t stream);

hipError_t launch_sample_draft(const int32_t* idx, const float* prob, const int32_t* count, const float* mass,
                               int k, int n_rows, const float* uniforms, int32_t* tok, float* q_scalar,
                               hipStream_t stream);

// Launch shape of the row statistics (threads per row, 16-byte vectors per thread and trip) for a dtype and a row
// count, and with it the layout of the optional segment table: a segment is what one wave reads per trip, seg_vecs
// consecutive vectors; a row owns `stride` entries (float2: sum, reference exponent).
struct StatsShape { int threads, nv, seg_vecs, stride; };
inline StatsShape stats_shape(int dtype, int64_t n_rows, int V) {
    StatsShape sh;
    if (dtype != 1)            { sh.threads = 1024; sh.nv = 4; }   // fp32 rows are HBM-bound with any shape
    else if (n_rows >= 2048)   { sh.threads = 256;  sh.nv = 4; }   // bf16: twice the arithmetic per byte; small workgroups,
    else if (n_rows >= 1024)   { sh.threads = 512;  sh.nv = 2; }   // many per CU, keep the vector ALUs busier as long as
    else                       { sh.threads = 1024; sh.nv = 2; }   // there are rows enough to fill the chip with them
    const int esz = dtype == 1 ? 2 : 4;
    const int64_t nq_max = ((int64_t)V * esz + 15) / 16 + 1;       // (a row off the 16-byte boundary spans one vector more)
    const int tile_vecs = sh.threads * sh.nv;
    sh.seg_vecs = 64 * sh.nv;
    sh.stride = (int)((nq_max + tile_vecs - 1) / tile_vecs) * (sh.threads / 64);
    return sh;
}
// ... and of the target rows of a small round, whose statistics run in 512-thread workgroups next to the compression
// (launch_round_stream): vectors per lane and trip chosen so that a row of the longest vocabulary has as many
// segments as above
template <bool BF16> constexpr int kRoundStatsNV = BF16 ? 2 : 4;
inline StatsShape round_stats_shape(int dtype, int V) {
    StatsShape sh;
    sh.threads = kCompressThreads;
    sh.nv = dtype == 1 ? kRoundStatsNV<true> : kRoundStatsNV<false>;
    const int esz = dtype == 1 ? 2 : 4;
    const int64_t nq_max = ((int64_t)V * esz + 15) / 16 + 1;
    const int tile_vecs = sh.threads * sh.nv;
    sh.seg_vecs = 64 * sh.nv;
    sh.stride = (int)((nq_max + tile_vecs - 1) / tile_vecs) * (sh.threads / 64);
    return sh;
}
// bytes of the segment table of `rows` rows (16-byte header in front: see SegHeader)
struct SegHeader { int32_t magic, seg_vecs, stride, rows; };
constexpr int32_t kSegMagic = 0x53454731;
inline size_t seg_table_bytes(int dtype, int64_t rows, int V) {
    return sizeof(SegHeader) + (size_t)rows * (size_t)stats_shape(dtype, rows, V).stride * 8;
}
// ... of a round's target rows, whichever of the two schedules the round takes
inline size_t round_seg_table_bytes(int dtype, int64_t rows, int V) {
    const size_t small = sizeof(SegHeader) + (size_t)rows * (size_t)round_stats_shape(dtype, V).stride * 8;
    return small > seg_table_bytes(dtype, rows, V) ? small : seg_table_bytes(dtype, rows, V);
}

// seg (nullable): the segment table, seg_stride entries per row
hipError_t launch_row_stats(const void* logits, int dtype, int64_t ld, int n_rows, int V, float temperature,
                            float* row_max, float* row_sum, float* row_lse, void* seg_table, hipStream_t stream);

// the same for the target rows pos_begin[b]..pos_end[b] of every sequence only (nullable: 0 / gamma_b)
hipError_t launch_row_stats_range(const void* logits, int dtype, int64_t ld, int V, float temperature, int B,
                                  int gamma_max, const int32_t* seq_off, const int32_t* pos_begin,
                                  const int32_t* pos_end, float* row_max, float* row_sum, float* row_lse,
                                  hipStream_t stream);

hipError_t launch_accept(const void* tgt_logits, int dtype, int64_t ld, int V, float temperature,
                         int B, const int32_t* seq_off, const int32_t* draft_tok,
                         const int32_t* q_idx, const float* q_prob, const int32_t* q_count, const float* q_mass,
                         int k, int renorm, const float* q_scalar, const float* uniforms,
                         const float* tgt_max, const float* tgt_sum,
                         int32_t* n_accept, float* p_tok, float* q_tok, uint32_t* flags,
                         const int32_t* pos_begin, const int32_t* pos_end, hipStream_t stream);

hipError_t launch_residual(const void* tgt_logits, int dtype, int64_t ld, int V, float temperature,
                           int B, const int32_t* seq_off, const int32_t* n_accept,
                           const float* tgt_max, const float* tgt_sum,
                           const int32_t* q_idx, const float* q_prob, const int32_t* q_count, const float* q_mass,
                           int k, int renorm, const float* uniforms,
                           int32_t* out_tok, float* resid_mass, uint32_t* flags, const void* seg_table, int64_t n_rows, hipStream_t stream);

// acceptance and residual draw of every sequence in one launch; seg_table (nullable, also in launch_residual): the
// table of the n_rows target rows from launch_row_stats (small_round_table: from launch_round_stream, whose layout
// differs), with which the draw does not stream its row again
hipError_t launch_decide(const void* tgt_logits, int dtype, int64_t ld, int V, float temperature,
                         int B, const int32_t* seq_off, const int32_t* draft_tok,
                         const int32_t* q_idx, const float* q_prob, const int32_t* q_count, const float* q_mass,
                         int k, int renorm, const float* uniforms, const float* tgt_max, const float* tgt_sum,
                         int32_t* n_accept, float* p_tok, float* q_tok, uint32_t* flags,
                         int32_t* out_tok, float* resid_mass, uint32_t* res_flags, const void* seg_table, int64_t n_rows,
                         bool small_round_table, hipStream_t stream);

hipError_t launch_resample_sparse(const void* draft_logits, int dtype, int64_t ld, int V, float temperature,
                                  int B, const int32_t* seq_off, const int32_t* n_accept,
                                  const float* draft_max, const float* draft_sum,
                                  const int32_t* p_idx, const float* p_prob, const int32_t* p_count, const float* p_mass,
                                  int k, int renorm, const float* uniforms,
                                  int32_t* out_tok, float* resid_mass, uint32_t* flags, hipStream_t stream);

// device self-check of the buffer loads' range check (csrc/selfcheck.hip); the workspace holds kCheckBytes
constexpr int kCheckBytes = 64 * 1024;
hipError_t launch_check_device(void* workspace, uint32_t* status, hipStream_t stream);
hipError_t launch_probe_clock(uint64_t* out, hipStream_t stream);

// ---- wire messages (csrc/wire.hip); fmt: 0 fp32, 1 fp16, 2 bf16 probabilities
int64_t downlink_bytes_max(int B, int k, int fmt);
int64_t uplink_bytes(int B, int n_draft, int fmt);

hipError_t launch_pack_downlink(int B, const int32_t* seq_off, const int32_t* n_accept, const int32_t* token,
                                const int32_t* idx, const float* prob, const int32_t* count, int k, int fmt,
                                void* wire, int64_t capacity, int64_t* wire_bytes, uint32_t* status, hipStream_t stream);

hipError_t launch_unpack_downlink(const void* wire, int64_t wire_bytes, int B, int k, int32_t* n_accept,
                                  int32_t* token, int32_t* idx, float* prob, int32_t* count, float* mass,
                                  uint32_t* status, hipStream_t stream);

hipError_t launch_pack_uplink(int B, int n_draft, const int32_t* seq_off, const int32_t* draft_tok,
                              const float* q_scalar, int fmt, void* wire, int64_t* wire_bytes, hipStream_t stream);

hipError_t launch_unpack_uplink(const void* wire, int64_t wire_bytes, int B, int n_max, int32_t* seq_off,
                                int32_t* draft_tok, float* q_scalar, uint32_t* status, hipStream_t stream);

}  // namespace picospec
