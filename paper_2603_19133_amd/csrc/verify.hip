// Parallel verification (paper Section 3.3): softmax statistics of every target row in one
// streaming pass, then per sequence the sparse lookup of the drafted token's probability, the
// acceptance test u < min(1, p/qhat) and the first rejected position.
#include "common.hpp"
#include "kernels.hpp"

namespace picospec {

namespace {

// One workgroup of THREADS threads per row, NV 16-byte vectors per thread and trip: M = max z, S = sum exp((z - M)/T), lse = M/T + ln S.
template <bool BF16, int NV, int THREADS>
__device__ __forceinline__ void row_stats_row(
    const int64_t row, const void* __restrict__ logits, int64_t ld, int V, float inv_T,
    float* __restrict__ row_max, float* __restrict__ row_sum, float* __restrict__ row_lse)
{
    __shared__ double red[2 * (THREADS / kWave)];
    constexpr int N = Vec<BF16>::N, E = NV * N, TILE = THREADS * E;
    static_assert(E <= 32, "one bit of the validity mask per element");
    const int tid = threadIdx.x;
    const RowView rv = row_view<BF16>(logits, ld, row, V);
    const int n_tiles = (rv.L + TILE - 1) / TILE;
    const float c = 1.4426950408889634f * inv_T;

    uint4 cur[NV], nxt[NV];
    auto load_tile = [&](int it, uint4 (&dst)[NV]) {
#pragma unroll
        for (int j = 0; j < NV; ++j) {
            int q = it * (THREADS * NV) + j * THREADS + tid;
            dst[j] = make_uint4(0, 0, 0, 0);
            if (vec_in_row<BF16>(rv, q)) dst[j] = load16_stream(rv.base + q);
        }
    };
    load_tile(0, cur);
    OnlineSum os;
    for (int it = 0; it < n_tiles; ++it) {
        if (it + 1 < n_tiles) load_tile(it + 1, nxt);
        float v[E];
#pragma unroll
        for (int j = 0; j < NV; ++j) {
            float t[N];
            unpack<BF16>(cur[j], t);
#pragma unroll
            for (int e = 0; e < N; ++e) v[j * N + e] = t[e];
        }
        if (it == 0 || it == n_tiles - 1) {
            unsigned vm = 0;
#pragma unroll
            for (int j = 0; j < NV; ++j) vm |= vec_valid_mask<BF16>(rv, it * (THREADS * NV) + j * THREADS + tid) << (j * N);
#pragma unroll
            for (int e = 0; e < E; ++e) v[e] = (vm >> e) & 1u ? v[e] : kNegInf;
        }
        float bm = v[0];
#pragma unroll
        for (int e = 1; e < E; ++e) bm = fmaxf(bm, v[e]);
        const float mref = os.rebase(bm, c);
        float acc = 0.f;
#pragma unroll
        for (int e = 0; e < E; ++e) acc += exp_stream(v[e], mref, c);
        os.s += acc;
#pragma unroll
        for (int j = 0; j < NV; ++j) cur[j] = nxt[j];
    }
    float M; double S;
    block_softmax_stats<THREADS / kWave>(os.m, os.s, c, red, M, S);
    if (tid == 0) {
        row_max[row] = M;
        row_sum[row] = (float)S;
        if (row_lse) row_lse[row] = (float)((double)M * (double)inv_T + log(S));
    }
}

template <bool BF16, int NV, int THREADS>
__global__ __launch_bounds__(THREADS) void row_stats_kernel(
    const void* __restrict__ logits, int64_t ld, int V, float inv_T,
    float* __restrict__ row_max, float* __restrict__ row_sum, float* __restrict__ row_lse)
{
    row_stats_row<BF16, NV, THREADS>(blockIdx.x, logits, ld, V, inv_T, row_max, row_sum, row_lse);
}

// Clamp a range of draft positions to 0 <= begin <= end <= g; reports whether it had to.
__device__ __forceinline__ bool clamp_range(const int32_t* pos_begin, const int32_t* pos_end, int b, int g, int& begin, int& end) {
    const int rb = pos_begin ? pos_begin[b] : 0, re = pos_end ? pos_end[b] : g;
    end = re < 0 ? 0 : (re > g ? g : re);
    begin = rb < 0 ? 0 : (rb > end ? end : rb);
    return rb != begin || re != end;
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

// One workgroup (16 waves) per sequence, one wave per draft position.  The wave looks the drafted
// token up in the position's sparse record with 16-byte loads (four in flight per lane), front
// first, and stops once it is found.
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
    __shared__ int s_first;
    __shared__ unsigned s_flags;
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
    const int b = blockIdx.x;
    const int d0 = seq_off[b];
    int g = seq_off[b + 1] - d0;
    unsigned fl = 0;
    if (g < 0) { fl |= 8u; g = 0; }
    int begin, end;                                   // the draft positions this call verifies (all of them by default)
    if (clamp_range(pos_begin, pos_end, b, g, begin, end)) fl |= 8u;
    if (tid == 0) { s_first = end; s_flags = 0; }
    __syncthreads();
    const int64_t t0 = (int64_t)d0 + b;
    const double cd = 1.4426950408889634 * (double)inv_T;

    // every target row of the range must have finite statistics
    for (int t = begin + tid; t <= end; t += kThreads) {
        float M = tgt_max[t0 + t], S = tgt_sum[t0 + t];
        if (!(fabsf(M) < __builtin_huge_valf()) || !(S > 0.f) || !(S < __builtin_huge_valf())) fl |= 2u;
    }

    for (int i = begin + wave; i < end; i += kWaves) {
        const int64_t rd = (int64_t)d0 + i, rt = t0 + i;
        const int x = draft_tok[rd];
        const bool bad = x < 0 || x >= V;
        // everything the decision needs besides qhat is asked for now (every lane the same address), so that it
        // arrives while the record is scanned instead of after it
        const float M_t = tgt_max[rt], S_t = tgt_sum[rt], u_t = uniforms[rt];
        const float z_t = bad ? 0.f : logit_at<BF16>(tgt_logits, ld, rt, x);
        const float mass_d = (!q_scalar && renorm) ? q_mass[rd] : 1.f;
        double qh = 0.0;
        if (q_scalar) {
            qh = (double)q_scalar[rd];
        } else {
            int cnt = q_count[rd];
            cnt = cnt < 0 ? 0 : (cnt > k ? k : cnt);
            const int32_t* ids = q_idx + rd * k;
            int slot = -1;
            // The record is ordered by probability and the token was drawn from it, so it sits near the
            // front more often than not: the scan goes in rounds of 1024 ids and stops at the round
            // that holds it.
            if ((((uintptr_t)ids) & 15u) == 0) {
                const int4* ids4 = reinterpret_cast<const int4*>(ids);
                const int n4 = cnt >> 2;
                for (int s0 = 0; s0 < n4; s0 += 4 * kWave) {
#pragma unroll
                    for (int u = 0; u < 4; ++u) {
                        const int s = s0 + u * kWave + lane;
                        if (s < n4) {
                            const int4 q = ids4[s];
                            if (q.x == x) slot = 4 * s;
                            if (q.y == x) slot = 4 * s + 1;
                            if (q.z == x) slot = 4 * s + 2;
                            if (q.w == x) slot = 4 * s + 3;
                        }
                    }
                    if (__ballot(slot >= 0)) break;
                }
                if (!__ballot(slot >= 0))
                    for (int s = 4 * n4 + lane; s < cnt; s += kWave)
                        if (ids[s] == x) slot = s;
            } else {
                for (int s0 = 0; s0 < cnt; s0 += 8 * kWave) {
#pragma unroll
                    for (int u = 0; u < 8; ++u) {
                        const int s = s0 + u * kWave + lane;
                        if (s < cnt && ids[s] == x) slot = s;
                    }
                    if (__ballot(slot >= 0)) break;
                }
            }
#pragma unroll
            for (int o = 32; o > 0; o >>= 1) slot = max(slot, __shfl_xor(slot, o, kWave));
            if (slot >= 0 && !bad) {
                qh = (double)q_prob[rd * k + slot];
                if (renorm) qh /= (double)mass_d;
            } else if (lane == 0) {
                fl |= 1u;
            }
        }
        if (lane == 0) {
            if (bad) fl |= 8u;
            double p = 0.0;
            if (!bad) p = exp_emit(z_t, M_t, cd) / (double)S_t;
            const double u = (double)u_t;
            // u < min(1, p/qhat), without forming the quotient; qhat = 0 counts as ratio = +inf
            const bool accept = (u < 1.0) && (qh > 0.0 ? (u * qh < p) : true);
            if (!accept) atomicMin(&s_first, i);
            if (p_tok) p_tok[rd] = (float)p;
            if (q_tok) q_tok[rd] = (float)qh;
        }
    }
    if (fl) atomicOr(&s_flags, fl);
    __syncthreads();
    if (tid == 0) {
        n_accept[b] = s_first;
        flags[b] = s_flags;
    }
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
                            float* row_max, float* row_sum, float* row_lse, hipStream_t stream)
{
    if (n_rows == 0) return hipSuccess;
    const float inv_T = 1.0f / temperature;
    // fp32 rows are HBM-bound with any shape.  bf16 rows carry twice the arithmetic per byte: small
    // workgroups (many per CU, out of step, short ragged tails) keep the vector ALUs busier, as long as
    // there are enough rows to fill the chip with them.
#define PICOSPEC_ROW_STATS(BF, NVV, TH) \
    hipLaunchKernelGGL((row_stats_kernel<BF, NVV, TH>), dim3(n_rows), dim3(TH), 0, stream, logits, ld, V, inv_T, row_max, row_sum, row_lse)
    if (dtype != 1)           PICOSPEC_ROW_STATS(false, 4, kThreads);
    else if (n_rows >= 2048)  PICOSPEC_ROW_STATS(true, 4, 256);
    else if (n_rows >= 1024)  PICOSPEC_ROW_STATS(true, 2, 512);
    else                      PICOSPEC_ROW_STATS(true, 2, kThreads);
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
