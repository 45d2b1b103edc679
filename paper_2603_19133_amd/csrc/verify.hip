// Parallel verification (paper Section 3.3): softmax statistics of every target row in one
// streaming pass, then per sequence the sparse lookup of the drafted token's probability, the
// acceptance test u < min(1, p/qhat) and the first rejected position.
#include "common.hpp"
#include "decide.hpp"
#include "kernels.hpp"

namespace picospec {

namespace {

template <bool BF16, int NV, int THREADS>
__global__ __launch_bounds__(THREADS) void row_stats_kernel(
    const void* __restrict__ logits, int64_t ld, int V, float inv_T,
    float* __restrict__ row_max, float* __restrict__ row_sum, float* __restrict__ row_lse)
{
    row_stats_row<BF16, NV, THREADS>(blockIdx.x, logits, ld, V, inv_T, row_max, row_sum, row_lse);
}

// The statistics together with the row's segment table (row_stats_seg_row); workgroup 0 also writes the table's header.
template <bool BF16, int NV, int THREADS>
__global__ __launch_bounds__(THREADS) void row_stats_seg_kernel(
    const void* __restrict__ logits, int64_t ld, int V, float inv_T,
    float* __restrict__ row_max, float* __restrict__ row_sum, float* __restrict__ row_lse,
    SegHeader* __restrict__ header, int seg_stride)
{
    if (blockIdx.x == 0 && threadIdx.x == 0) *header = SegHeader{kSegMagic, NV * kWave, seg_stride, (int32_t)gridDim.x};
    row_stats_seg_row<BF16, NV, THREADS>(blockIdx.x, logits, ld, V, inv_T, row_max, row_sum, row_lse,
                                         reinterpret_cast<float2*>(header + 1), seg_stride);
}

// The same for the target rows begin_b..end_b of every sequence only (verification of a part of the
// draft): workgroup (t, b) of a (gamma_max + 1) x B grid takes position t of sequence b or leaves.
template <bool BF16, int NV, int THREADS>
__global__ __launch_bounds__(THREADS) void row_stats_range_kernel(
    const void* __restrict__ logits, int64_t ld, int V, float inv_T,
    const int32_t* __restrict__ seq_off, const int32_t* __restrict__ pos_begin, const int32_t* __restrict__ pos_end,
    float* __restrict__ row_max, float* __restrict__ row_sum, float* __restrict__ row_lse)
{
    const int b = blockIdx.y, t = blockIdx.x;
    const int d0 = seq_off[b];
    int g = seq_off[b + 1] - d0;
    if (g < 0) g = 0;
    int begin, end;
    clamp_range(pos_begin, pos_end, b, g, begin, end);
    if (t < begin || t > end) return;
    row_stats_row<BF16, NV, THREADS>((int64_t)d0 + b + t, logits, ld, V, inv_T, row_max, row_sum, row_lse);
}

// picospec_verify's second kernel: one workgroup per sequence (accept_sequence, decide.hpp).
template <bool BF16>
__global__ __launch_bounds__(kThreads) void accept_kernel(
    const void* __restrict__ tgt_logits, int64_t ld, int V, float inv_T, int B,
    const int32_t* __restrict__ seq_off, const int32_t* __restrict__ draft_tok,
    const int32_t* __restrict__ q_idx, const float* __restrict__ q_prob,
    const int32_t* __restrict__ q_count, const float* __restrict__ q_mass, int k, int renorm,
    const float* __restrict__ q_scalar, const float* __restrict__ uniforms,
    const float* __restrict__ tgt_max, const float* __restrict__ tgt_sum,
    int32_t* __restrict__ n_accept, float* __restrict__ p_tok, float* __restrict__ q_tok,
    uint32_t* __restrict__ flags, const int32_t* __restrict__ pos_begin, const int32_t* __restrict__ pos_end)
{
    accept_sequence<BF16>(blockIdx.x, tgt_logits, ld, V, inv_T, seq_off, draft_tok, q_idx, q_prob, q_count, q_mass, k,
                          renorm, q_scalar, uniforms, tgt_max, tgt_sum, n_accept, p_tok, q_tok, flags, pos_begin, pos_end);
}

}  // namespace

hipError_t launch_row_stats_range(const void* logits, int dtype, int64_t ld, int V, float temperature, int B,
                                  int gamma_max, const int32_t* seq_off, const int32_t* pos_begin,
                                  const int32_t* pos_end, float* row_max, float* row_sum, float* row_lse,
                                  hipStream_t stream)
{
    if (B == 0) return hipSuccess;
    const float inv_T = 1.0f / temperature;
    const int64_t n_rows = (int64_t)B * (gamma_max + 1);          // (an upper bound: workgroups outside the ranges leave at once)
    const dim3 grid(gamma_max + 1, B);
#define PICOSPEC_ROW_STATS_RANGE(BF, NVV, TH) \
    hipLaunchKernelGGL((row_stats_range_kernel<BF, NVV, TH>), grid, dim3(TH), 0, stream, logits, ld, V, inv_T, seq_off, pos_begin, pos_end, row_max, row_sum, row_lse)
    if (dtype != 1)           PICOSPEC_ROW_STATS_RANGE(false, 4, kThreads);
    else if (n_rows >= 2048)  PICOSPEC_ROW_STATS_RANGE(true, 4, 256);
    else if (n_rows >= 1024)  PICOSPEC_ROW_STATS_RANGE(true, 2, 512);
    else                      PICOSPEC_ROW_STATS_RANGE(true, 2, kThreads);
#undef PICOSPEC_ROW_STATS_RANGE
    return hipGetLastError();
}

hipError_t launch_row_stats(const void* logits, int dtype, int64_t ld, int n_rows, int V, float temperature,
                            float* row_max, float* row_sum, float* row_lse, void* seg_table, hipStream_t stream)
{
    if (n_rows == 0) return hipSuccess;
    const float inv_T = 1.0f / temperature;
    const StatsShape sh = stats_shape(dtype, n_rows, V);
#define PICOSPEC_ROW_STATS(BF, NVV, TH) \
    do { if (seg_table) hipLaunchKernelGGL((row_stats_seg_kernel<BF, NVV, TH>), dim3(n_rows), dim3(TH), 0, stream, logits, ld, V, inv_T, row_max, row_sum, row_lse, (SegHeader*)seg_table, sh.stride); \
         else hipLaunchKernelGGL((row_stats_kernel<BF, NVV, TH>), dim3(n_rows), dim3(TH), 0, stream, logits, ld, V, inv_T, row_max, row_sum, row_lse); } while (0)
    if (dtype != 1)              PICOSPEC_ROW_STATS(false, 4, kThreads);
    else if (sh.threads == 256)  PICOSPEC_ROW_STATS(true, 4, 256);
    else if (sh.threads == 512)  PICOSPEC_ROW_STATS(true, 2, 512);
    else                         PICOSPEC_ROW_STATS(true, 2, kThreads);
#undef PICOSPEC_ROW_STATS
    return hipGetLastError();
}

hipError_t launch_accept(const void* tgt_logits, int dtype, int64_t ld, int V, float temperature,
                         int B, const int32_t* seq_off, const int32_t* draft_tok,
                         const int32_t* q_idx, const float* q_prob, const int32_t* q_count, const float* q_mass,
                         int k, int renorm, const float* q_scalar, const float* uniforms,
                         const float* tgt_max, const float* tgt_sum,
                         int32_t* n_accept, float* p_tok, float* q_tok, uint32_t* flags,
                         const int32_t* pos_begin, const int32_t* pos_end, hipStream_t stream)
{
    if (B == 0) return hipSuccess;
    const float inv_T = 1.0f / temperature;
    if (dtype == 1) hipLaunchKernelGGL(accept_kernel<true>, dim3(B), dim3(kThreads), 0, stream, tgt_logits, ld, V, inv_T, B, seq_off, draft_tok, q_idx, q_prob, q_count, q_mass, k, renorm, q_scalar, uniforms, tgt_max, tgt_sum, n_accept, p_tok, q_tok, flags, pos_begin, pos_end);
    else            hipLaunchKernelGGL(accept_kernel<false>, dim3(B), dim3(kThreads), 0, stream, tgt_logits, ld, V, inv_T, B, seq_off, draft_tok, q_idx, q_prob, q_count, q_mass, k, renorm, q_scalar, uniforms, tgt_max, tgt_sum, n_accept, p_tok, q_tok, flags, pos_begin, pos_end);
    return hipGetLastError();
}

}  // namespace picospec
