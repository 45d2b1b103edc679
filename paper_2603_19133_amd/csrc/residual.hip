// Correction / bonus token (paper Section 3.3): one draw per sequence from
// norm(max(0, P_j - qhat_j)) by inverse CDF in ascending vocabulary id.
//
// One workgroup per sequence streams target row j once.  The sparse qhat of the matching draft
// row is scattered into an LDS image of the current tile, so the dense pass sees qhat(x) at LDS
// speed.  Each wave leaves one partial sum per 16-byte-vector column it owns ("segment": 64 lanes
// x 4 or 8 consecutive ids per lane, contiguous in id); segment sums are kept in LDS in id order.
// The crossing of u*R is then located among the segments and only that one segment (1 KB) is read
// again to name the token.
#include "common.hpp"
#include "kernels.hpp"

namespace picospec {

namespace {

constexpr int kTile = 16384;                                  // elements per tile (both dtypes)
constexpr int kMaxTiles = (kMaxV + 16) / kTile + 1;
constexpr int kMaxSeg = kMaxTiles * 4 * kWaves;               // fp32: 4 vector columns per tile

struct __align__(16) ResidualShared {
    float qtile[kTile];         // qhat image of the current tile (0 off-support)
    double seg[kMaxSeg];        // residual mass of each segment, id order
    double red[2 * kWaves];
    double before;              // cumulative residual in front of the chosen segment
    int seg_pick, seg_last;
};

static_assert(sizeof(ResidualShared) <= 160 * 1024, "LDS budget of one gfx950 CU");

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
    extern __shared__ __align__(16) unsigned char smem_raw[];
    ResidualShared& sh = *reinterpret_cast<ResidualShared*>(smem_raw);
    constexpr int N = Vec<BF16>::N, NV = kTile / (kThreads * N);
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
    const int b = blockIdx.x;
    const int d0 = seq_off[b];
    int g = seq_off[b + 1] - d0;
    unsigned fl = 0;
    if (g < 0) { fl |= 8u; g = 0; }
    int j = n_accept[b];
    if (j < 0 || j > g) { fl |= 8u; j = j < 0 ? 0 : g; }
    const int64_t rt = (int64_t)d0 + b + j;
    const int64_t rd = (int64_t)d0 + j;
    bool has_q = j < g;
    int cnt = 0;
    float q_scale = 1.f;
    if (has_q) {
        cnt = q_count[rd];
        cnt = cnt < 0 ? 0 : (cnt > k ? k : cnt);
        if (renorm) q_scale = 1.f / q_mass[rd];
    }
    const float M = tgt_max[rt];
    const float invS = 1.f / tgt_sum[rt];
    const float c = 1.4426950408889634f * inv_T;
    const RowView rv = row_view<BF16>(tgt_logits, ld, rt, V);
    const int n_tiles = (rv.L + kTile - 1) / kTile;
    const int n_seg = n_tiles * NV * kWaves;
    const int32_t* ids = q_idx + rd * k;
    const float* qp = q_prob + rd * k;

    // residual of the N elements of the 16-byte vector `raw` = vector q of the row, given the qhat image
    auto residual_of = [&](const uint4& raw, int q, const float* qimg, float (&r)[N]) {
        float v[N];
        unpack<BF16>(raw, v);
        const unsigned vm = vec_valid_mask<BF16>(rv, q);
#pragma unroll
        for (int e = 0; e < N; ++e) {
            const float p = exp_stream(v[e], M, c) * invS;
            const float d = p - qimg[e];
            r[e] = ((vm >> e) & 1u) && d > 0.f ? d : 0.f;
        }
    };
    const int nq = (rv.L + N - 1) / N;
    auto load_vec = [&](int q) { return load16_stream(rv.base + min(q, nq - 1)); };   // behind the row: its last vector, masked later

    // this thread's share of the sparse record (k <= kMaxK), kept in registers across tiles
    constexpr int SP = kMaxK / kThreads;
    int my_id[SP];
    float my_q[SP];
#pragma unroll
    for (int z = 0; z < SP; ++z) {
        const int s = z * kThreads + tid;
        my_id[z] = -1;
        my_q[z] = 0.f;
        if (s < cnt) { my_id[z] = ids[s]; my_q[z] = qp[s] * q_scale; }
    }

    double R = 0.0;
    for (int attempt = 0; attempt < 2; ++attempt) {
        uint4 cur[NV], nxt[NV];
#pragma unroll
        for (int jv = 0; jv < NV; ++jv) cur[jv] = load_vec(jv * kThreads + tid);
        for (int it = 0; it < n_tiles; ++it) {
            if (it + 1 < n_tiles) {
#pragma unroll
                for (int jv = 0; jv < NV; ++jv) nxt[jv] = load_vec((it + 1) * (kThreads * NV) + jv * kThreads + tid);
            }
            // qhat image of this tile
            float4* qt4 = reinterpret_cast<float4*>(sh.qtile);
#pragma unroll
            for (int z = 0; z < kTile / 4 / kThreads; ++z) qt4[z * kThreads + tid] = make_float4(0.f, 0.f, 0.f, 0.f);
            __syncthreads();
            if (has_q) {
                const int lo = it * kTile - rv.o;            // id of the tile's first virtual element
#pragma unroll
                for (int z = 0; z < SP; ++z) {
                    const int off = my_id[z] - lo;
                    if (my_id[z] >= 0 && off >= 0 && off < kTile) sh.qtile[off] = my_q[z];
                }
            }
            __syncthreads();
#pragma unroll
            for (int jv = 0; jv < NV; ++jv) {
                float r[N];
                residual_of(cur[jv], it * (kThreads * NV) + jv * kThreads + tid, sh.qtile + (jv * kThreads + tid) * N, r);
                double sum = 0.0;
#pragma unroll
                for (int e = 0; e < N; ++e) sum += (double)r[e];
                sum = wave_sum(sum);
                if (lane == 0) sh.seg[(it * NV + jv) * kWaves + wave] = sum;
            }
            __syncthreads();
#pragma unroll
            for (int jv = 0; jv < NV; ++jv) cur[jv] = nxt[jv];
        }
        // total residual mass
        double part = 0.0;
        for (int s = tid; s < n_seg; s += kThreads) part += sh.seg[s];
        part = wave_sum(part);
        if (lane == 0) sh.red[wave] = part;
        __syncthreads();
        R = 0.0;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) R += sh.red[w];
        __syncthreads();
        if (R > 0.0 || !has_q) break;
        // P == qhat numerically: draw from P itself
        fl |= 4u;
        has_q = false;
    }

    // locate the segment in which the cumulative residual first exceeds u*R
    const double target = (double)uniforms[(int64_t)d0 + b + g] * R;
    const int per = (n_seg + kThreads - 1) / kThreads;       // contiguous segments per thread
    const int s0 = min(n_seg, tid * per), s1 = min(n_seg, s0 + per);
    double mine = 0.0;
    for (int s = s0; s < s1; ++s) mine += sh.seg[s];
    double incl = wave_scan_incl(mine);
    if (lane == kWave - 1) sh.red[wave] = incl;
    if (tid == 0) { sh.seg_pick = 0x7FFFFFFF; sh.seg_last = -1; sh.before = 0.0; }
    __syncthreads();
    double before = 0.0;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) if (w < wave) before += sh.red[w];
    double cum = before + incl - mine;
    int my_pick = 0x7FFFFFFF, my_last = -1;
    for (int s = s0; s < s1; ++s) {
        const double v = sh.seg[s];
        if (v > 0.0) my_last = s;
        if (my_pick == 0x7FFFFFFF && cum + v > target) my_pick = s;
        if (my_pick == 0x7FFFFFFF) cum += v;
    }
    if (my_pick != 0x7FFFFFFF) atomicMin(&sh.seg_pick, my_pick);
    if (my_last >= 0) atomicMax(&sh.seg_last, my_last);
    __syncthreads();
    int pick = sh.seg_pick;
    const bool crossed = pick != 0x7FFFFFFF;
    if (!crossed) pick = sh.seg_last < 0 ? 0 : sh.seg_last;   // rounding: last segment with mass
    if (crossed && my_pick == pick) sh.before = cum;          // exactly one thread owns the chosen segment
    __syncthreads();

    // re-read that one segment and name the token (wave 0)
    const int col = pick / kWaves, pw = pick % kWaves, it = col / NV, jv = col % NV;
    const int seg_lo = (it * (kThreads * NV) + jv * kThreads + pw * kWave) * N - rv.o;   // id of the segment's first element
    if (wave == 0) {
#pragma unroll
        for (int e = 0; e < N; ++e) sh.qtile[lane * N + e] = 0.f;
    }
    __syncthreads();
    if (has_q) {
#pragma unroll
        for (int z = 0; z < SP; ++z) {
            const int off = my_id[z] - seg_lo;
            if (my_id[z] >= 0 && off >= 0 && off < kWave * N) sh.qtile[off] = my_q[z];
        }
    }
    __syncthreads();
    if (wave == 0) {
        float r[N];
        const int qv = it * (kThreads * NV) + jv * kThreads + pw * kWave + lane;
        residual_of(load_vec(qv), qv, sh.qtile + lane * N, r);
        double sum = 0.0;
#pragma unroll
        for (int e = 0; e < N; ++e) sum += (double)r[e];
        const double inc = wave_scan_incl(sum);
        const double base = sh.before;
        int tok = -1;
        const unsigned long long hit = crossed ? __ballot(base + inc > target) : 0ull;
        if (hit) {
            const int owner = __ffsll((long long)hit) - 1;
            if (lane == owner) {
                double cu = base + inc - sum;
#pragma unroll
                for (int e = 0; e < N; ++e) {
                    cu += (double)r[e];
                    if (tok < 0 && cu > target) tok = seg_lo + lane * N + e;
                }
                if (tok < 0) tok = seg_lo + lane * N + N - 1;
            }
            tok = __shfl(tok, owner, kWave);
        } else {   // rounding: the last id of the segment with residual mass
            const unsigned long long any = __ballot(sum > 0.0);
            if (any) {
                const int owner = 63 - __clzll((long long)any);
                if (lane == owner) {
#pragma unroll
                    for (int e = 0; e < N; ++e) if (r[e] > 0.f) tok = seg_lo + lane * N + e;
                }
                tok = __shfl(tok, owner, kWave);
            } else {
                tok = min(max(seg_lo, 0), V - 1);
            }
        }
        if (lane == 0) {
            out_tok[b] = tok;
            resid_mass[b] = (fl & 4u) ? 0.f : (float)R;
            flags[b] = fl;
        }
    }
}

}  // namespace

hipError_t launch_residual(const void* tgt_logits, int dtype, int64_t ld, int V, float temperature,
                           int B, const int32_t* seq_off, const int32_t* n_accept,
                           const float* tgt_max, const float* tgt_sum,
                           const int32_t* q_idx, const float* q_prob, const int32_t* q_count, const float* q_mass,
                           int k, int renorm, const float* uniforms,
                           int32_t* out_tok, float* resid_mass, uint32_t* flags, hipStream_t stream)
{
    static bool attr_set[2] = {false, false};
    const size_t smem = sizeof(ResidualShared);
    auto f32 = residual_kernel<false>;
    auto b16 = residual_kernel<true>;
    const int which = dtype == 1;
    if (!attr_set[which]) {
        hipError_t e = hipFuncSetAttribute(which ? (const void*)b16 : (const void*)f32,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        if (e != hipSuccess) return e;
        attr_set[which] = true;
    }
    if (B == 0) return hipSuccess;
    const float inv_T = 1.0f / temperature;
    if (which) hipLaunchKernelGGL(b16, dim3(B), dim3(kThreads), smem, stream, tgt_logits, ld, V, inv_T, seq_off, n_accept, tgt_max, tgt_sum, q_idx, q_prob, q_count, q_mass, k, renorm, uniforms, out_tok, resid_mass, flags);
    else       hipLaunchKernelGGL(f32, dim3(B), dim3(kThreads), smem, stream, tgt_logits, ld, V, inv_T, seq_off, n_accept, tgt_max, tgt_sum, q_idx, q_prob, q_count, q_mass, k, renorm, uniforms, out_tok, resid_mass, flags);
    return hipGetLastError();
}

}  // namespace picospec
