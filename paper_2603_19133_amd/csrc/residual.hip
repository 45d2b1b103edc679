// Correction / bonus token (paper Section 3.3): one draw per sequence from
// norm(max(0, P_j - qhat_j)) by inverse CDF in ascending vocabulary id.
//
// One workgroup per sequence streams target row j once, in tiles of 16384 elements.  The sparse qhat
// of the matching draft row is scattered into an LDS image of the tile, so the dense pass sees
// qhat(x) at LDS speed; two images alternate, and instead of clearing an image the entries written
// for a tile are taken back after it, so that an image costs k writes per row, not V.  Within a tile
// each wave owns 1024 consecutive ids (a "segment") and leaves one partial sum per segment; the
// segment sums are kept in LDS in id order.  The crossing of u*R is then located among the segments
// and only that one segment (4 KB at most) is read again to name the token.
#include "common.hpp"
#include "decide.hpp"
#include "kernels.hpp"

namespace picospec {

namespace {

template <bool BF16>
__global__ __launch_bounds__(kThreads) void residual_kernel(
    const void* __restrict__ tgt_logits, int64_t ld, int V, float inv_T,
    const int32_t* __restrict__ seq_off, const int32_t* __restrict__ n_accept,
    const float* __restrict__ tgt_max, const float* __restrict__ tgt_sum,
    const int32_t* __restrict__ q_idx, const float* __restrict__ q_prob,
    const int32_t* __restrict__ q_count, const float* __restrict__ q_mass, int k, int renorm,
    const float* __restrict__ uniforms,
    int32_t* __restrict__ out_tok, float* __restrict__ resid_mass, uint32_t* __restrict__ flags)
{
    residual_sequence<BF16>(blockIdx.x, n_accept[blockIdx.x], tgt_logits, ld, V, inv_T, seq_off, tgt_max, tgt_sum,
                            q_idx, q_prob, q_count, q_mass, k, renorm, uniforms, out_tok, resid_mass, flags);
}

// The two decisions of a sequence in one workgroup (small rounds): acceptance of its draft positions, then the
// draw at the first rejected position, without the trip of that position through device memory.
template <bool BF16>
__global__ __launch_bounds__(kThreads) void decide_kernel(
    const void* __restrict__ tgt_logits, int64_t ld, int V, float inv_T,
    const int32_t* __restrict__ seq_off, const int32_t* __restrict__ draft_tok,
    const int32_t* __restrict__ q_idx, const float* __restrict__ q_prob,
    const int32_t* __restrict__ q_count, const float* __restrict__ q_mass, int k, int renorm,
    const float* __restrict__ uniforms, const float* __restrict__ tgt_max, const float* __restrict__ tgt_sum,
    int32_t* __restrict__ n_accept, float* __restrict__ p_tok, float* __restrict__ q_tok, uint32_t* __restrict__ flags,
    int32_t* __restrict__ out_tok, float* __restrict__ resid_mass, uint32_t* __restrict__ res_flags)
{
    const int first = accept_sequence<BF16>(blockIdx.x, tgt_logits, ld, V, inv_T, seq_off, draft_tok, q_idx, q_prob,
                                            q_count, q_mass, k, renorm, nullptr, uniforms, tgt_max, tgt_sum,
                                            n_accept, p_tok, q_tok, flags, nullptr, nullptr);
    residual_sequence<BF16>(blockIdx.x, first, tgt_logits, ld, V, inv_T, seq_off, tgt_max, tgt_sum,
                            q_idx, q_prob, q_count, q_mass, k, renorm, uniforms, out_tok, resid_mass, res_flags);
}

// The same two kernels with the target rows' segment table at hand (no second pass over a row).
template <bool BF16>
__global__ __launch_bounds__(kThreads) void residual_seg_kernel(
    const void* __restrict__ tgt_logits, int64_t ld, int V, float inv_T,
    const int32_t* __restrict__ seq_off, const int32_t* __restrict__ n_accept,
    const float* __restrict__ tgt_max, const SegHeader* __restrict__ table, int seg_vecs, int stride,
    const int32_t* __restrict__ q_idx, const float* __restrict__ q_prob,
    const int32_t* __restrict__ q_count, const float* __restrict__ q_mass, int k, int renorm,
    const float* __restrict__ uniforms,
    int32_t* __restrict__ out_tok, float* __restrict__ resid_mass, uint32_t* __restrict__ flags)
{
    residual_seg_sequence<BF16>(blockIdx.x, n_accept[blockIdx.x], tgt_logits, ld, V, inv_T, seq_off, tgt_max, table, seg_vecs, stride,
                                q_idx, q_prob, q_count, q_mass, k, renorm, uniforms, out_tok, resid_mass, flags);
}

template <bool BF16>
__global__ __launch_bounds__(kThreads) void decide_seg_kernel(
    const void* __restrict__ tgt_logits, int64_t ld, int V, float inv_T,
    const int32_t* __restrict__ seq_off, const int32_t* __restrict__ draft_tok,
    const int32_t* __restrict__ q_idx, const float* __restrict__ q_prob,
    const int32_t* __restrict__ q_count, const float* __restrict__ q_mass, int k, int renorm,
    const float* __restrict__ uniforms, const float* __restrict__ tgt_max, const float* __restrict__ tgt_sum,
    const SegHeader* __restrict__ table, int seg_vecs, int stride,
    int32_t* __restrict__ n_accept, float* __restrict__ p_tok, float* __restrict__ q_tok, uint32_t* __restrict__ flags,
    int32_t* __restrict__ out_tok, float* __restrict__ resid_mass, uint32_t* __restrict__ res_flags)
{
    const int first = accept_sequence<BF16>(blockIdx.x, tgt_logits, ld, V, inv_T, seq_off, draft_tok, q_idx, q_prob,
                                            q_count, q_mass, k, renorm, nullptr, uniforms, tgt_max, tgt_sum,
                                            n_accept, p_tok, q_tok, flags, nullptr, nullptr);
    residual_seg_sequence<BF16>(blockIdx.x, first, tgt_logits, ld, V, inv_T, seq_off, tgt_max, table, seg_vecs, stride,
                                q_idx, q_prob, q_count, q_mass, k, renorm, uniforms, out_tok, resid_mass, res_flags);
}

}  // namespace

hipError_t launch_residual(const void* tgt_logits, int dtype, int64_t ld, int V, float temperature,
                           int B, const int32_t* seq_off, const int32_t* n_accept,
                           const float* tgt_max, const float* tgt_sum,
                           const int32_t* q_idx, const float* q_prob, const int32_t* q_count, const float* q_mass,
                           int k, int renorm, const float* uniforms,
                           int32_t* out_tok, float* resid_mass, uint32_t* flags, const void* seg_table, int64_t n_rows, hipStream_t stream)
{
    if (seg_table) {
        if (B == 0) return hipSuccess;
        const float it = 1.0f / temperature;
        const StatsShape sh = stats_shape(dtype, n_rows, V);
        if (dtype == 1) hipLaunchKernelGGL(residual_seg_kernel<true>, dim3(B), dim3(kThreads), 0, stream, tgt_logits, ld, V, it, seq_off, n_accept, tgt_max, (const SegHeader*)seg_table, sh.seg_vecs, sh.stride, q_idx, q_prob, q_count, q_mass, k, renorm, uniforms, out_tok, resid_mass, flags);
        else            hipLaunchKernelGGL(residual_seg_kernel<false>, dim3(B), dim3(kThreads), 0, stream, tgt_logits, ld, V, it, seq_off, n_accept, tgt_max, (const SegHeader*)seg_table, sh.seg_vecs, sh.stride, q_idx, q_prob, q_count, q_mass, k, renorm, uniforms, out_tok, resid_mass, flags);
        return hipGetLastError();
    }
    static DeviceFlags limit_raised[2] = {};
    const size_t smem = sizeof(ResidualShared);
    auto f32 = residual_kernel<false>;
    auto b16 = residual_kernel<true>;
    const int which = dtype == 1;
    {
        int dev = 0;
        hipError_t e = raise_lds_limit_once(which ? (const void*)b16 : (const void*)f32, smem, limit_raised[which], dev);
        if (e != hipSuccess) return e;
    }
    if (B == 0) return hipSuccess;
    const float inv_T = 1.0f / temperature;
    if (which) hipLaunchKernelGGL(b16, dim3(B), dim3(kThreads), smem, stream, tgt_logits, ld, V, inv_T, seq_off, n_accept, tgt_max, tgt_sum, q_idx, q_prob, q_count, q_mass, k, renorm, uniforms, out_tok, resid_mass, flags);
    else       hipLaunchKernelGGL(f32, dim3(B), dim3(kThreads), smem, stream, tgt_logits, ld, V, inv_T, seq_off, n_accept, tgt_max, tgt_sum, q_idx, q_prob, q_count, q_mass, k, renorm, uniforms, out_tok, resid_mass, flags);
    return hipGetLastError();
}

hipError_t launch_decide(const void* tgt_logits, int dtype, int64_t ld, int V, float temperature,
                         int B, const int32_t* seq_off, const int32_t* draft_tok,
                         const int32_t* q_idx, const float* q_prob, const int32_t* q_count, const float* q_mass,
                         int k, int renorm, const float* uniforms, const float* tgt_max, const float* tgt_sum,
                         int32_t* n_accept, float* p_tok, float* q_tok, uint32_t* flags,
                         int32_t* out_tok, float* resid_mass, uint32_t* res_flags, const void* seg_table, int64_t n_rows,
                         bool small_round_table, hipStream_t stream)
{
    if (seg_table) {
        if (B == 0) return hipSuccess;
        const float it = 1.0f / temperature;
        const StatsShape sh = small_round_table ? round_stats_shape(dtype, V) : stats_shape(dtype, n_rows, V);
        if (dtype == 1) hipLaunchKernelGGL(decide_seg_kernel<true>, dim3(B), dim3(kThreads), 0, stream, tgt_logits, ld, V, it, seq_off, draft_tok, q_idx, q_prob, q_count, q_mass, k, renorm, uniforms, tgt_max, tgt_sum, (const SegHeader*)seg_table, sh.seg_vecs, sh.stride, n_accept, p_tok, q_tok, flags, out_tok, resid_mass, res_flags);
        else            hipLaunchKernelGGL(decide_seg_kernel<false>, dim3(B), dim3(kThreads), 0, stream, tgt_logits, ld, V, it, seq_off, draft_tok, q_idx, q_prob, q_count, q_mass, k, renorm, uniforms, tgt_max, tgt_sum, (const SegHeader*)seg_table, sh.seg_vecs, sh.stride, n_accept, p_tok, q_tok, flags, out_tok, resid_mass, res_flags);
        return hipGetLastError();
    }
    static DeviceFlags limit_raised[2] = {};
    const size_t smem = sizeof(ResidualShared);
    auto f32 = decide_kernel<false>;
    auto b16 = decide_kernel<true>;
    const int which = dtype == 1;
    {
        int dev = 0;
        hipError_t e = raise_lds_limit_once(which ? (const void*)b16 : (const void*)f32, smem, limit_raised[which], dev);
        if (e != hipSuccess) return e;
    }
    if (B == 0) return hipSuccess;
    const float inv_T = 1.0f / temperature;
    if (which) hipLaunchKernelGGL(b16, dim3(B), dim3(kThreads), smem, stream, tgt_logits, ld, V, inv_T, seq_off, draft_tok, q_idx, q_prob, q_count, q_mass, k, renorm, uniforms, tgt_max, tgt_sum, n_accept, p_tok, q_tok, flags, out_tok, resid_mass, res_flags);
    else       hipLaunchKernelGGL(f32, dim3(B), dim3(kThreads), smem, stream, tgt_logits, ld, V, inv_T, seq_off, draft_tok, q_idx, q_prob, q_count, q_mass, k, renorm, uniforms, tgt_max, tgt_sum, n_accept, p_tok, q_tok, flags, out_tok, resid_mass, res_flags);
    return hipGetLastError();
}

}  // namespace picospec
