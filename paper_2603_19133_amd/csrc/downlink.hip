// Edge-side local resampling on the sparse downlink (paper Section 3.3: on a rejection the cloud
// sends only the Top-K record of the target distribution, Eq. 4, and the edge draws the corrected
// token from norm(max(0, P_j - Q_j)) with its own dense Q_j).  The target is known here only
// through the record, so the residual lives on the record's slots: one workgroup per sequence
// gathers the draft logits at the record's ids, forms r_s = max(0, Pt(id_s) - Q_j(id_s)) in fp64,
// and takes the inverse CDF over the slots in slot order.
#include "common.hpp"
#include "kernels.hpp"

namespace picospec {

namespace {

constexpr int kRT = 256;                      // threads per workgroup (4 waves)
constexpr int kRW = kRT / kWave;
constexpr int kPer = kMaxK / kRT;             // slots per thread at most (consecutive slots)

template <bool BF16>
__global__ __launch_bounds__(kRT) void resample_sparse_kernel(
    const void* __restrict__ draft_logits, int64_t ld, int V, float inv_T,
    const int32_t* __restrict__ seq_off, const int32_t* __restrict__ n_accept,
    const float* __restrict__ draft_max, const float* __restrict__ draft_sum,
    const int32_t* __restrict__ p_idx, const float* __restrict__ p_prob,
    const int32_t* __restrict__ p_count, const float* __restrict__ p_mass, int k, int renorm,
    const float* __restrict__ uniforms,
    int32_t* __restrict__ out_tok, float* __restrict__ resid_mass, uint32_t* __restrict__ flags)
{
    __shared__ double s_wave[kRW];
    __shared__ int s_pick, s_last;
    __shared__ unsigned s_flags;
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
    const int b = blockIdx.x;
    const int d0 = seq_off[b];
    int g = seq_off[b + 1] - d0;
    unsigned fl = 0;
    if (g < 0) { fl |= 8u; g = 0; }
    int j = n_accept[b];
    if (j < 0 || j > g) { fl |= 8u; j = j < 0 ? 0 : g; }
    const bool has_q = j < g;
    const int64_t rd = (int64_t)d0 + j;
    int cnt = p_count[b];
    cnt = cnt < 0 ? 0 : (cnt > k ? k : cnt);
    const double scale = renorm ? 1.0 / (double)p_mass[b] : 1.0;
    const double cd = 1.4426950408889634 * (double)inv_T;
    float M = 0.f;
    double invS = 0.0;
    if (has_q) { M = draft_max[rd]; invS = 1.0 / (double)draft_sum[rd]; }
    const int32_t* ids = p_idx + (int64_t)b * k;
    const float* pp = p_prob + (int64_t)b * k;
    if (tid == 0) { s_pick = 0x7FFFFFFF; s_last = -1; s_flags = 0; }

    // this thread's consecutive slots [s0, s1) and their weights
    const int per = (cnt + kRT - 1) / kRT;
    const int s0 = min(cnt, tid * per), s1 = min(cnt, s0 + per);
    double r[kPer], pt[kPer];
    double mine = 0.0;
#pragma unroll
    for (int z = 0; z < kPer; ++z) {
        r[z] = 0.0; pt[z] = 0.0;
        const int s = s0 + z;
        if (s < s1) {
            pt[z] = (double)pp[s] * scale;
            double w = pt[z];
            if (has_q) {
                const int x = ids[s];
                double q = 0.0;
                if (x >= 0 && x < V) q = exp_emit(logit_at<BF16>(draft_logits, ld, rd, x), M, cd) * invS;
                else fl |= 8u;
                w = w - q > 0.0 ? w - q : 0.0;
            }
            r[z] = w;
            mine += w;
        }
    }
    // block prefix in slot order
    auto block_scan = [&](double v, double& before, double& total) {
        const double incl = wave_scan_incl(v);
        __syncthreads();                                   // (s_wave may still be read from the last scan)
        if (lane == kWave - 1) s_wave[wave] = incl;
        __syncthreads();
        before = incl - v;
        total = 0.0;
#pragma unroll
        for (int w = 0; w < kRW; ++w) { const double t = s_wave[w]; if (w < wave) before += t; total += t; }
    };
    double before, R;
    block_scan(mine, before, R);
    if (!(R > 0.0)) {            // nothing of the record exceeds Q: draw from the record itself
        fl |= 4u;
        mine = 0.0;
#pragma unroll
        for (int z = 0; z < kPer; ++z) { r[z] = pt[z]; mine += pt[z]; }
        block_scan(mine, before, R);
    }
    const double target = (double)uniforms[(int64_t)d0 + b + g] * R;
    int my_pick = 0x7FFFFFFF, my_last = -1;
    double cum = before;
#pragma unroll
    for (int z = 0; z < kPer; ++z) {
        const int s = s0 + z;
        if (s < s1) {
            if (r[z] > 0.0) my_last = s;
            cum += r[z];
            if (my_pick == 0x7FFFFFFF && cum > target) my_pick = s;
        }
    }
    if (my_pick != 0x7FFFFFFF) atomicMin(&s_pick, my_pick);
    if (my_last >= 0) atomicMax(&s_last, my_last);
    if (fl) atomicOr(&s_flags, fl);
    __syncthreads();
    if (tid == 0) {
        int pick = s_pick;
        if (pick == 0x7FFFFFFF) pick = s_last < 0 ? (cnt > 0 ? cnt - 1 : -1) : s_last;   // rounding: last slot with weight
        if (pick > 0 && s_last < 0) pick = 0;                                              // (no weight anywhere: slot 0, as the plain definition ends up)
        const unsigned f = s_flags;
        out_tok[b] = pick >= 0 ? ids[pick] : -1;
        resid_mass[b] = (f & 4u) ? 0.f : (float)R;
        flags[b] = f;
    }
}

}  // namespace

hipError_t launch_resample_sparse(const void* draft_logits, int dtype, int64_t ld, int V, float temperature,
                                  int B, const int32_t* seq_off, const int32_t* n_accept,
                                  const float* draft_max, const float* draft_sum,
                                  const int32_t* p_idx, const float* p_prob, const int32_t* p_count, const float* p_mass,
                                  int k, int renorm, const float* uniforms,
                                  int32_t* out_tok, float* resid_mass, uint32_t* flags, hipStream_t stream)
{
    if (B == 0) return hipSuccess;
    const float inv_T = 1.0f / temperature;
    if (dtype == 1) hipLaunchKernelGGL(resample_sparse_kernel<true>, dim3(B), dim3(kRT), 0, stream, draft_logits, ld, V, inv_T, seq_off, n_accept, draft_max, draft_sum, p_idx, p_prob, p_count, p_mass, k, renorm, uniforms, out_tok, resid_mass, flags);
    else            hipLaunchKernelGGL(resample_sparse_kernel<false>, dim3(B), dim3(kRT), 0, stream, draft_logits, ld, V, inv_T, seq_off, n_accept, draft_max, draft_sum, p_idx, p_prob, p_count, p_mass, k, renorm, uniforms, out_tok, resid_mass, flags);
    return hipGetLastError();
}

}  // namespace picospec
