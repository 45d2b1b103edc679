// The per-sequence decisions of a round (paper Section 3.3), as device functions that a workgroup of kThreads
// threads runs for one sequence: accept_sequence (the acceptance test of every draft position and the first
// rejection) and residual_sequence (the correction or bonus token from norm(max(0, P_j - qhat_j))).  The
// library's kernels call them one per launch, or both from one workgroup.
#pragma once

#include "common.hpp"
#include "kernels.hpp"
#include "rowspan.hpp"

namespace picospec {

namespace {

// Clamp a range of draft positions to 0 <= begin <= end <= g; reports whether it had to.
__device__ __forceinline__ bool clamp_range(const int32_t* pos_begin, const int32_t* pos_end, int b, int g, int& begin, int& end) {
    const int rb = pos_begin ? pos_begin[b] : 0, re = pos_end ? pos_end[b] : g;
    end = re < 0 ? 0 : (re > g ? g : re);
    begin = rb < 0 ? 0 : (rb > end ? end : rb);
    return rb != begin || re != end;
}

// One workgroup (16 waves) per sequence, one wave per draft position.  The wave looks the drafted
// token up in the position's sparse record with 16-byte loads (four in flight per lane), front
// first, and stops once it is found.
// Returns the sequence's first rejected position (in every thread; a barrier stands behind the decision).
template <bool BF16>
__device__ __forceinline__ int accept_sequence(
    const int b, const void* __restrict__ tgt_logits, int64_t ld, int V, float inv_T,
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
            // u < min(1, p/qhat), without forming the quotient; qhat = 0 counts as ratio = +inf.  An id outside the
            // vocabulary has p = 0 whatever qhat is said to be: it is rejected, so the accepted prefix ends in front of it
            const bool accept = !bad && (u < 1.0) && (qh > 0.0 ? (u * qh < p) : true);
            if (!accept) atomicMin(&s_first, i);
            if (p_tok) p_tok[rd] = (float)p;
            if (q_tok) q_tok[rd] = (float)qh;
        }
    }
    if (fl) atomicOr(&s_flags, fl);
    __syncthreads();
    const int first = s_first;
    if (tid == 0) {
        n_accept[b] = first;
        flags[b] = s_flags;
    }
    return first;
}


constexpr int kTile = kResidualTile;                          // elements per tile (both dtypes)
static_assert(kResidualThreads == kThreads, "one workgroup of kThreads threads per sequence");
constexpr int kSegLen = kTile / kWaves;                       // 1024 consecutive ids per wave and tile
constexpr int kMaxTiles = (kMaxV + 16) / kTile + 1;
constexpr int kMaxSeg = kMaxTiles * kWaves;

struct __align__(16) ResidualShared {
    float qimg[2][kTile];       // qhat images of two consecutive tiles (0 off-support)
    double seg[kMaxSeg];        // residual mass of each segment, id order
    double red[2 * kWaves];
    double before;              // cumulative residual in front of the chosen segment
    int seg_pick, seg_last;
};

static_assert(sizeof(ResidualShared) <= 160 * 1024, "LDS budget of one gfx950 CU");

// The draw of sequence b at its target row j_in (the first rejected position, or gamma_b for the bonus token).
template <bool BF16>
__device__ __forceinline__ void residual_sequence(
    const int b, const int j_in, const void* __restrict__ tgt_logits, int64_t ld, int V, float inv_T,
    const int32_t* __restrict__ seq_off,
    const float* __restrict__ tgt_max, const float* __restrict__ tgt_sum,
    const int32_t* __restrict__ q_idx, const float* __restrict__ q_prob,
    const int32_t* __restrict__ q_count, const float* __restrict__ q_mass, int k, int renorm,
    const float* __restrict__ uniforms,
    int32_t* __restrict__ out_tok, float* __restrict__ resid_mass, uint32_t* __restrict__ flags)
{
    extern __shared__ __align__(16) unsigned char smem_raw[];
    ResidualShared& sh = *reinterpret_cast<ResidualShared*>(smem_raw);
    using Geom = ResidualGeom<BF16>;
    constexpr int N = Vec<BF16>::N, NV = Geom::NV;                     // vectors per thread and tile
    constexpr int kSegVec = Geom::SEG_VECS;                            // vectors per segment
    static_assert(Geom::TILE_VECS == kThreads * NV && kSegVec == NV * kWave, "tile geometry");
    const int tid = threadIdx.x, lane = tid & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(tid / kWave);   // uniform: it forms scalar load offsets
    const int d0 = seq_off[b];
    int g = seq_off[b + 1] - d0;
    unsigned fl = 0;
    if (g < 0) { fl |= 8u; g = 0; }
    int j = j_in;
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
    const float c = 1.4426950408889634f * inv_T;
    const RowView rv = row_view<BF16>(tgt_logits, ld, rt, V);
    const int n_tiles = (rv.L + kTile - 1) / kTile;
    const int n_seg = n_tiles * kWaves;
    const int32_t* ids = q_idx + rd * k;
    const float* qp = q_prob + rd * k;
    const int nq = (rv.L + N - 1) / N;
    // row loads: descriptor base + scalar offset of the vector group + this lane's offset.  On gfx950 a raw
    // buffer load compares scalar offset + lane offset + 16 with the descriptor's size (measured;
    // picospec_check_device() tests it), so vectors behind the row read as zero without touching memory
    const __amdgpu_buffer_rsrc_t row_rsrc = __builtin_amdgcn_make_buffer_rsrc((void*)rv.base, 0, nq * 16, 0x00020000);
    // vector `first + lane` of the row (first is uniform across the wave)
    auto load_vec = [&](int first) {
        const u32x4_t t = __builtin_amdgcn_raw_buffer_load_b128(row_rsrc, lane * 16, first * 16, 2 /* non-temporal */);
        return make_uint4(t.x, t.y, t.z, t.w);
    };

    // P(x) = 2^(z*c + kappa), kappa = -M*c - log2 S, so that one fused multiply-add and one exponential
    // form each probability.  kappa is rounded to fp32 once; that would scale every P by the same
    // factor 1 + eps, so qhat is scaled by it as well (the residuals then all carry it) and the sums
    // are divided by it at the end: the arithmetic stays that of P - qhat.
    const double kappa_d = -(double)M * (double)c - log2((double)tgt_sum[rt]);
    const float kappa = (float)kappa_d;
    const double common = exp2((double)kappa - kappa_d);       // 1 + eps
    // residual of the N elements of the 16-byte vector `raw` = vector q of the row, given the qhat image
    auto residual_of = [&](const uint4& raw, int q, const float* qimg, bool edge, float (&r)[N]) {
        float v[N];
        unpack<BF16>(raw, v);
        if (edge) {
            const unsigned vm = vec_valid_mask<BF16>(rv, q);
#pragma unroll
            for (int e = 0; e < N; ++e) {
                const float d = __builtin_amdgcn_exp2f(fmaf(v[e], c, kappa)) - qimg[e];
                r[e] = ((vm >> e) & 1u) && d > 0.f ? d : 0.f;
            }
        } else {
#pragma unroll
            for (int e = 0; e < N; ++e) r[e] = fmaxf(__builtin_amdgcn_exp2f(fmaf(v[e], c, kappa)) - qimg[e], 0.f);
        }
    };

    // this thread's share of the sparse record (k <= kMaxK), kept in registers across tiles
    constexpr int SP = kMaxK / kThreads;
    int my_id[SP];
    float my_q[SP];
#pragma unroll
    for (int z = 0; z < SP; ++z) {
        const int s = z * kThreads + tid;
        my_id[z] = -1;
        my_q[z] = 0.f;
        if (s < cnt) { my_id[z] = ids[s]; my_q[z] = (float)((double)qp[s] * (double)q_scale * common); }
    }
    // write (or take back) this thread's record entries that fall into ids [lo, lo + len)
    auto scatter = [&](float* img, int lo, int len, bool take_back) {
#pragma unroll
        for (int z = 0; z < SP; ++z) {
            const int off = my_id[z] - lo;
            if (my_id[z] >= 0 && off >= 0 && off < len) img[off] = take_back ? 0.f : my_q[z];
        }
    };

    {   // both images start empty
        float4* z4 = reinterpret_cast<float4*>(&sh.qimg[0][0]);
#pragma unroll
        for (int z = 0; z < 2 * kTile / 4 / kThreads; ++z) z4[z * kThreads + tid] = make_float4(0.f, 0.f, 0.f, 0.f);
    }
    __syncthreads();

    // vector of (tile it, wave, jv, lane): it * (kThreads * NV) + wave * kSegVec + jv * kWave + lane
    const int wave_vec = wave * kSegVec;
    double R = 0.0;
    for (int attempt = 0; attempt < 2; ++attempt) {
        // three tiles in registers: one in use, two in flight (loads behind the row read zeros)
        uint4 tb[3][NV];
        auto load_tile = [&](int it, uint4 (&dst)[NV]) {
#pragma unroll
            for (int jv = 0; jv < NV; ++jv) dst[jv] = load_vec(Geom::group_first(it, wave, jv));
        };
        load_tile(0, tb[0]);
        load_tile(1, tb[1]);
        load_tile(2, tb[2]);
        if (has_q) scatter(sh.qimg[0], -rv.o, kTile, false);
        __syncthreads();
        auto step = [&](int it, uint4 (&buf)[NV]) {
            const float* img = sh.qimg[it & 1];
            const bool edge = it == 0 || it + 1 == n_tiles;
            double sum = 0.0;
#pragma unroll
            for (int jv = 0; jv < NV; ++jv) {
                float r[N];
                const int ql = wave_vec + jv * kWave + lane;             // vector within the tile
                residual_of(buf[jv], it * (kThreads * NV) + ql, img + ql * N, edge, r);
                float part = 0.f;
#pragma unroll
                for (int e = 0; e < N; ++e) part += r[e];
                sum += (double)part;
            }
            load_tile(it + 3, buf);
            sum = wave_sum(sum);
            if (lane == 0) sh.seg[it * kWaves + wave] = sum;
            __syncthreads();                                             // the image of this tile has been read
            if (has_q) {
                scatter(sh.qimg[it & 1], it * kTile - rv.o, kTile, true);
                if (it + 1 < n_tiles) scatter(sh.qimg[(it + 1) & 1], (it + 1) * kTile - rv.o, kTile, false);
            }
            __syncthreads();
        };
        // (whole groups of three in the loop, so that its body has one path and the waits for the loads
        // in flight stay exact; the last one or two tiles follow it)
        int it = 0;
        for (; it + 3 <= n_tiles; it += 3) {
            step(it, tb[0]);
            step(it + 1, tb[1]);
            step(it + 2, tb[2]);
        }
        if (it < n_tiles) step(it, tb[0]);
        if (it + 1 < n_tiles) step(it + 1, tb[1]);
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
        if (R > 0.0 || !has_q) break;   // (R still carries the common factor)
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
    int pick = __builtin_amdgcn_readfirstlane(sh.seg_pick);   // (uniform: it forms scalar load offsets below)
    const bool crossed = pick != 0x7FFFFFFF;
    if (!crossed) pick = max(__builtin_amdgcn_readfirstlane(sh.seg_last), 0);   // rounding: last segment with mass
    if (crossed && my_pick == pick) sh.before = cum;          // exactly one thread owns the chosen segment
    // (both images are empty again: every entry was taken back after its tile)
    const int pt = pick / kWaves, pw = pick % kWaves;
    const int seg_vec = pt * (kThreads * NV) + pw * kSegVec;  // first vector of the segment
    const int seg_lo = seg_vec * N - rv.o;                    // id of its first element
    if (has_q) scatter(sh.qimg[0], seg_lo, kSegLen, false);
    __syncthreads();

    // re-read that one segment and name the token (wave 0): ids ascend with (jv, lane, element)
    if (wave == 0) {
        const double base0 = sh.before;
        double base = base0;
        int tok = -1, last_tok = -1;
#pragma unroll
        for (int jv = 0; jv < NV; ++jv) {
            float r[N];
            const int ql = jv * kWave + lane;
            residual_of(load_vec(Geom::group_first(pt, pw, jv)), seg_vec + ql, sh.qimg[0] + ql * N, true, r);
            double sum = 0.0;
#pragma unroll
            for (int e = 0; e < N; ++e) sum += (double)r[e];
            const double inc = wave_scan_incl(sum);
            const unsigned long long hit = (crossed && tok < 0) ? __ballot(base + inc > target) : 0ull;
            if (hit) {
                const int owner = __ffsll((long long)hit) - 1;
                int t = -1;
                if (lane == owner) {
                    double cu = base + inc - sum;
#pragma unroll
                    for (int e = 0; e < N; ++e) {
                        cu += (double)r[e];
                        if (t < 0 && cu > target) t = seg_lo + ql * N + e;
                    }
                    if (t < 0) t = seg_lo + ql * N + N - 1;
                }
                tok = __shfl(t, owner, kWave);
            }
            // rounding fallback: the last id of the segment with residual mass
            const unsigned long long any = __ballot(sum > 0.0);
            if (any) {
                const int owner = 63 - __clzll((long long)any);
                int t = -1;
                if (lane == owner) {
#pragma unroll
                    for (int e = 0; e < N; ++e) if (r[e] > 0.f) t = seg_lo + ql * N + e;
                }
                last_tok = __shfl(t, owner, kWave);
            }
            base += __shfl(inc, kWave - 1, kWave);
        }
        if (tok < 0) tok = last_tok >= 0 ? last_tok : min(max(seg_lo, 0), V - 1);
        if (lane == 0) {
            out_tok[b] = tok;
            resid_mass[b] = (fl & 4u) ? 0.f : (float)(R / common);
            flags[b] = fl;
        }
    }
}

// ---------------------------------------------------------------- the same draw from the row's segment table
//
// With the exponential sums of the target row's segments at hand (written by the statistics pass: row_stats_seg_row)
// the row is not streamed again.  R = sum_x max(0, P(x) - qhat(x)) = sum over segments of (P(segment) - T(segment)),
// T = sum over the record's entries in the segment of min(P(x), qhat(x)): one gathered logit per record entry.  The
// segment in which the cumulative residual crosses u R is then read (one to four KB) and the token named as before.
// T is summed in 2^-62 fixed point (integer LDS atomics: the order of the additions does not change the result).

constexpr int kMaxSegTable = 1040;                               // segments of the longest row (2^20 elements: 1025 of 4 KB or of 2 KB)
constexpr int kMaxSegElems = 256 * 8;                            // elements of the largest segment (256 vectors of bf16)

struct __align__(16) SegResidualShared {
    double pseg[kMaxSegTable];                 // P of each segment, then its residual mass
    unsigned long long tfix[kMaxSegTable];     // T of each segment, 2^-62 fixed point
    float qimg[kMaxSegElems];                  // qhat image of the chosen segment
    double red[2 * kWaves];
    double before;
    int seg_pick, seg_last;
};

template <bool BF16>
__device__ __forceinline__ void residual_seg_sequence(
    const int b, const int j_in, const void* __restrict__ tgt_logits, int64_t ld, int V, float inv_T,
    const int32_t* __restrict__ seq_off, const float* __restrict__ tgt_max, const SegHeader* __restrict__ table,
    const int seg_vecs, const int stride,
    const int32_t* __restrict__ q_idx, const float* __restrict__ q_prob,
    const int32_t* __restrict__ q_count, const float* __restrict__ q_mass, int k, int renorm,
    const float* __restrict__ uniforms,
    int32_t* __restrict__ out_tok, float* __restrict__ resid_mass, uint32_t* __restrict__ flags)
{
    __shared__ SegResidualShared sh;
    constexpr int N = Vec<BF16>::N;
    constexpr int SP = kMaxK / kThreads;
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
    const int d0 = seq_off[b];
    int g = seq_off[b + 1] - d0;
    unsigned fl = 0;
    if (g < 0) { fl |= 8u; g = 0; }
    int j = j_in;
    if (j < 0 || j > g) { fl |= 8u; j = j < 0 ? 0 : g; }
    const int64_t rt = (int64_t)d0 + b + j;
    const int64_t rd = (int64_t)d0 + j;
    bool has_q = j < g;
    const RowView rv = row_view<BF16>(tgt_logits, ld, rt, V);
    const int nq = (rv.L + N - 1) / N;
    const int seg_elems = seg_vecs * N;
    const int n_seg = (nq + seg_vecs - 1) / seg_vecs;
    const float2* seg_row = reinterpret_cast<const float2*>(table + 1) + rt * (int64_t)stride;
    // Everything that depends only on the two rows is asked for at once (one trip to memory): the table's header
    // (checked below), the target row's maximum, the record's count and mass, this thread's entries of the record and
    // its entries of the segment table.
    const SegHeader hd = *table;
    const float M = tgt_max[rt];
    int cnt = 0;
    float mass_d = 1.f;
    int my_id[SP];
    float my_p[SP];
    if (has_q) {
        cnt = q_count[rd];
        if (renorm) mass_d = q_mass[rd];
#pragma unroll
        for (int z = 0; z < SP; ++z) {
            const int sl = z * kThreads + tid;
            my_id[z] = -1;
            my_p[z] = 0.f;
            if (sl < k) { my_id[z] = q_idx[rd * k + sl]; my_p[z] = q_prob[rd * k + sl]; }
        }
        cnt = cnt < 0 ? 0 : (cnt > k ? k : cnt);
    } else {
#pragma unroll
        for (int z = 0; z < SP; ++z) { my_id[z] = -1; my_p[z] = 0.f; }
    }
    const bool table_ok = n_seg <= stride && n_seg <= kMaxSegTable && seg_elems <= kMaxSegElems;
    float2 my_seg[(kMaxSegTable + kThreads - 1) / kThreads];
#pragma unroll
    for (int u = 0; u < (kMaxSegTable + kThreads - 1) / kThreads; ++u) {
        const int sg = u * kThreads + tid;
        my_seg[u] = make_float2(0.f, 0.f);
        if (table_ok && sg < n_seg) my_seg[u] = seg_row[sg];
    }
    // ... and, one trip later, the target's logit at each of this thread's record entries
    float my_z[SP];
#pragma unroll
    for (int z = 0; z < SP; ++z) {
        const int sl = z * kThreads + tid;
        if (!(sl < cnt && my_id[z] >= 0 && my_id[z] < V)) my_id[z] = -1;
        my_z[z] = my_id[z] >= 0 ? logit_at<BF16>(tgt_logits, ld, rt, my_id[z]) : 0.f;
    }
    const float c = 1.4426950408889634f * inv_T;
    const double cd = 1.4426950408889634 * (double)inv_T;
    const double q_scale = 1.0 / (double)mass_d;
    if (!table_ok || hd.magic != kSegMagic || rt >= hd.rows || hd.stride != stride || hd.seg_vecs != seg_vecs) {
        if (tid == 0) { out_tok[b] = 0; resid_mass[b] = 0.f; flags[b] = fl | 8u; }     // (not the table of these rows)
        return;
    }

    // P of every segment, up to the common factor 1 / S
    double part = 0.0;
#pragma unroll
    for (int u = 0; u < (kMaxSegTable + kThreads - 1) / kThreads; ++u) {
        const int sg = u * kThreads + tid;
        if (sg < n_seg) {
            const float2 e = my_seg[u];
            const double p = e.x > 0.f ? (double)e.x * exp2_split((double)e.y - (double)M * (double)c) : 0.0;
            sh.pseg[sg] = p;
            sh.tfix[sg] = 0ull;
            part += p;
        }
    }
    part = wave_sum(part);
    if (lane == 0) sh.red[wave] = part;
    if (tid == 0) { sh.seg_pick = 0x7FFFFFFF; sh.seg_last = -1; sh.before = 0.0; }
    __syncthreads();
    double S = 0.0;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) S += sh.red[w];
    const double invS = 1.0 / S;
    __syncthreads();

    // this thread's share of the record: qhat and min(P, qhat) into the segment's T
    float my_q[SP];
#pragma unroll
    for (int z = 0; z < SP; ++z) {
        my_q[z] = 0.f;
        if (my_id[z] >= 0) {
            const double qh = (double)my_p[z] * q_scale;
            const double p = exp_emit(my_z[z], M, cd) * invS;
            const double m = p < qh ? p : qh;
            my_q[z] = (float)qh;
            atomicAdd(&sh.tfix[(my_id[z] + rv.o) / seg_elems], (unsigned long long)llrint(m * 4611686018427387904.0));
        }
    }
    __syncthreads();

    // residual mass of every segment, the total, and the segment in which the cumulative residual crosses u R
    const int per = (n_seg + kThreads - 1) / kThreads;        // contiguous segments per thread
    const int s0 = min(n_seg, tid * per), s1 = min(n_seg, s0 + per);
    double R = 0.0, mine = 0.0;
    for (int attempt = 0; attempt < 2; ++attempt) {
        mine = 0.0;
        for (int s = s0; s < s1; ++s) {
            double r = sh.pseg[s] * invS;
            if (has_q) { r -= (double)sh.tfix[s] * (1.0 / 4611686018427387904.0); r = r > 0.0 ? r : 0.0; }
            mine += r;
        }
        const double tot = wave_sum(mine);
        __syncthreads();
        if (lane == 0) sh.red[wave] = tot;
        __syncthreads();
        R = 0.0;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) R += sh.red[w];
        if (R > 0.0 || !has_q) break;
        fl |= 4u;                                              // P == qhat numerically: draw from P itself
        has_q = false;
    }
    auto seg_mass = [&](int s) {
        double r = sh.pseg[s] * invS;
        if (has_q) { r -= (double)sh.tfix[s] * (1.0 / 4611686018427387904.0); r = r > 0.0 ? r : 0.0; }
        return r;
    };
    const double target = (double)uniforms[(int64_t)d0 + b + g] * R;
    const double incl = wave_scan_incl(mine);
    __syncthreads();
    if (lane == kWave - 1) sh.red[kWaves + wave] = incl;
    __syncthreads();
    double cum = incl - mine;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) if (w < wave) cum += sh.red[kWaves + w];
    int my_pick = 0x7FFFFFFF, my_last = -1;
    for (int s = s0; s < s1; ++s) {
        const double v = seg_mass(s);
        if (v > 0.0) my_last = s;
        if (my_pick == 0x7FFFFFFF && cum + v > target) my_pick = s;
        if (my_pick == 0x7FFFFFFF) cum += v;
    }
    if (my_pick != 0x7FFFFFFF) atomicMin(&sh.seg_pick, my_pick);
    if (my_last >= 0) atomicMax(&sh.seg_last, my_last);
    __syncthreads();
    int pick = sh.seg_pick;
    const bool crossed = pick != 0x7FFFFFFF;
    if (!crossed) pick = max(sh.seg_last, 0);                 // rounding: last segment with mass
    if (crossed && my_pick == pick) sh.before = cum;          // exactly one thread owns the chosen segment
    const int seg_vec = pick * seg_vecs;                      // first vector of the segment
    const int seg_lo = seg_vec * N - rv.o;                    // id of its first element
    for (int i = tid; i < seg_elems; i += kThreads) sh.qimg[i] = 0.f;
    __syncthreads();
    if (has_q) {
#pragma unroll
        for (int z = 0; z < SP; ++z) {
            const int off = my_id[z] - seg_lo;
            if (my_id[z] >= 0 && off >= 0 && off < seg_elems) sh.qimg[off] = my_q[z];
        }
    }
    __syncthreads();

    // read that one segment and name the token (wave 0): ids ascend with (jv, lane, element)
    if (wave == 0) {
        const double kappa = -(double)M * cd - log2(S);
        double base = sh.before;
        int tok = -1, last_tok = -1;
        for (int jv = 0; jv * kWave < seg_vecs; ++jv) {
            const int ql = jv * kWave + lane, q = seg_vec + ql;
            uint4 raw = make_uint4(0, 0, 0, 0);
            if (vec_in_row<BF16>(rv, q)) raw = load16_stream(rv.base + q);
            float v[N];
            unpack<BF16>(raw, v);
            const unsigned vm = vec_valid_mask<BF16>(rv, q);
            double r[N], sum = 0.0;
#pragma unroll
            for (int e = 0; e < N; ++e) {
                const double d = exp2_split((double)v[e] * cd + kappa) - (double)sh.qimg[ql * N + e];
                r[e] = ((vm >> e) & 1u) && d > 0.0 ? d : 0.0;
                sum += r[e];
            }
            const double inc = wave_scan_incl(sum);
            const unsigned long long hit = (crossed && tok < 0) ? __ballot(base + inc > target) : 0ull;
            if (hit) {
                const int owner = __ffsll((long long)hit) - 1;
                int t = -1;
                if (lane == owner) {
                    double cu = base + inc - sum;
#pragma unroll
                    for (int e = 0; e < N; ++e) {
                        cu += r[e];
                        if (t < 0 && cu > target) t = seg_lo + ql * N + e;
                    }
                    if (t < 0) t = seg_lo + ql * N + N - 1;
                }
                tok = __shfl(t, owner, kWave);
            }
            const unsigned long long any = __ballot(sum > 0.0);   // rounding fallback: the last id of the segment with mass
            if (any) {
                const int owner = 63 - __clzll((long long)any);
                int t = -1;
                if (lane == owner) {
#pragma unroll
                    for (int e = 0; e < N; ++e) if (r[e] > 0.0) t = seg_lo + ql * N + e;
                }
                last_tok = __shfl(t, owner, kWave);
            }
            base += __shfl(inc, kWave - 1, kWave);
        }
        if (tok < 0) tok = last_tok >= 0 ? last_tok : min(max(seg_lo, 0), V - 1);
        if (lane == 0) {
            out_tok[b] = tok;
            resid_mass[b] = (fl & 4u) ? 0.f : (float)R;
            flags[b] = fl;
        }
    }
}

}  // namespace

}  // namespace picospec
