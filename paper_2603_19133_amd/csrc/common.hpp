// Device-side helpers shared by the gfx950 kernels: 16-byte row streaming with an alignment
// prologue, order-preserving keys, wave64 reductions, accurate exponentials for emitted values.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

namespace picospec {

constexpr int kWave = 64;
constexpr int kThreads = 1024;            // one workgroup = 16 waves = one row (or one sequence)
constexpr int kWaves = kThreads / kWave;
constexpr float kNegInf = -__builtin_huge_valf();

// ---------------------------------------------------------------- wave64 / workgroup reductions
//
// Cross-lane steps inside a row of 16 lanes use DPP operand modifiers (no trip through the LDS
// crossbar); the four rows of a wave are combined through scalar registers (v_readlane).

constexpr int kDppQuadXor1 = 0xB1;        // quad_perm:[1,0,3,2]
constexpr int kDppQuadXor2 = 0x4E;        // quad_perm:[2,3,0,1]
constexpr int kDppRowHalfMirror = 0x141;  // lane i <-> 7 - i within each half row
constexpr int kDppRowMirror = 0x140;      // lane i <-> 15 - i within each row
constexpr int kDppRowShr = 0x110;         // + n: lane i reads lane i - n of its row (0 where there is none)

template <int CTRL>
__device__ __forceinline__ int dpp_word(int v) { return __builtin_amdgcn_update_dpp(0, v, CTRL, 0xF, 0xF, true); }

template <int CTRL, typename T>
__device__ __forceinline__ T dpp(T v) {
    static_assert(sizeof(T) == 4 || sizeof(T) == 8, "32- or 64-bit lanes");
    if constexpr (sizeof(T) == 4) {
        int w;
        __builtin_memcpy(&w, &v, 4);
        w = dpp_word<CTRL>(w);
        __builtin_memcpy(&v, &w, 4);
    } else {
        int w[2];
        __builtin_memcpy(w, &v, 8);
        w[0] = dpp_word<CTRL>(w[0]);
        w[1] = dpp_word<CTRL>(w[1]);
        __builtin_memcpy(&v, w, 8);
    }
    return v;
}

// value of `v` in lane `lane` (a constant), in every lane
template <typename T>
__device__ __forceinline__ T read_lane(T v, int lane) {
    if constexpr (sizeof(T) == 4) {
        int w;
        __builtin_memcpy(&w, &v, 4);
        w = __builtin_amdgcn_readlane(w, lane);
        __builtin_memcpy(&v, &w, 4);
    } else {
        int w[2];
        __builtin_memcpy(w, &v, 8);
        w[0] = __builtin_amdgcn_readlane(w[0], lane);
        w[1] = __builtin_amdgcn_readlane(w[1], lane);
        __builtin_memcpy(&v, w, 8);
    }
    return v;
}

// sum over the 64 lanes, in every lane (the same bits in every lane: each step adds a pair both ways)
template <typename T>
__device__ __forceinline__ T wave_sum(T v) {
    v += dpp<kDppQuadXor1>(v);
    v += dpp<kDppQuadXor2>(v);
    v += dpp<kDppRowHalfMirror>(v);
    v += dpp<kDppRowMirror>(v);
    return (read_lane(v, 0) + read_lane(v, 16)) + (read_lane(v, 32) + read_lane(v, 48));
}

// sum over the 64 lanes, valid in lane 63 only: four shift-and-add steps inside each row of 16 lanes, then the rows'
// totals handed on to the rows behind them (six instructions, none of them reads a lane into a scalar)
__device__ __forceinline__ float wave_sum_last(float v) {
    auto step = [](float x, auto ctrl, auto row_mask) {
        int w;
        __builtin_memcpy(&w, &x, 4);
        w = __builtin_amdgcn_update_dpp(0, w, decltype(ctrl)::value, decltype(row_mask)::value, 0xF, true);
        float y;
        __builtin_memcpy(&y, &w, 4);
        return y;
    };
    using all = std::integral_constant<int, 0xF>;
    v += step(v, std::integral_constant<int, kDppRowShr + 1>{}, all{});
    v += step(v, std::integral_constant<int, kDppRowShr + 2>{}, all{});
    v += step(v, std::integral_constant<int, kDppRowShr + 4>{}, all{});
    v += step(v, std::integral_constant<int, kDppRowShr + 8>{}, all{});
    v += step(v, std::integral_constant<int, 0x142>{}, std::integral_constant<int, 0xA>{});   // row_bcast:15 into rows 1 and 3
    v += step(v, std::integral_constant<int, 0x143>{}, std::integral_constant<int, 0xC>{});   // row_bcast:31 into rows 2 and 3
    return v;
}

__device__ __forceinline__ float wave_max(float v) {
    v = fmaxf(v, dpp<kDppQuadXor1>(v));
    v = fmaxf(v, dpp<kDppQuadXor2>(v));
    v = fmaxf(v, dpp<kDppRowHalfMirror>(v));
    v = fmaxf(v, dpp<kDppRowMirror>(v));
    return fmaxf(fmaxf(read_lane(v, 0), read_lane(v, 16)), fmaxf(read_lane(v, 32), read_lane(v, 48)));
}

__device__ __forceinline__ uint64_t shfl_xor_u64(uint64_t v, int o) {
    uint32_t lo = __shfl_xor((uint32_t)v, o, kWave), hi = __shfl_xor((uint32_t)(v >> 32), o, kWave);
    return ((uint64_t)hi << 32) | lo;
}

__device__ __forceinline__ uint64_t wave_min_u64(uint64_t v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) { uint64_t w = shfl_xor_u64(v, o); v = w < v ? w : v; }
    return v;
}

__device__ __forceinline__ uint64_t wave_max_u64(uint64_t v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) { uint64_t w = shfl_xor_u64(v, o); v = w > v ? w : v; }
    return v;
}

// inclusive prefix sum across the 64 lanes of a wave: four shift-and-add steps inside each row, then
// the totals of the rows in front
template <typename T>
__device__ __forceinline__ T wave_scan_incl(T v) {
    const int lane = threadIdx.x & (kWave - 1);
    v += dpp<kDppRowShr + 1>(v);
    v += dpp<kDppRowShr + 2>(v);
    v += dpp<kDppRowShr + 4>(v);
    v += dpp<kDppRowShr + 8>(v);
    const T r0 = read_lane(v, 15), r1 = read_lane(v, 31), r2 = read_lane(v, 47);
    T before = T(0);
    if (lane >= 16) before += r0;
    if (lane >= 32) before += r1;
    if (lane >= 48) before += r2;
    return v + before;
}

// ---------------------------------------------------------------- order-preserving keys

// fp32 bit pattern -> uint32 whose unsigned order is the numeric order; -0.0 maps onto +0.0.
__device__ __forceinline__ uint32_t key_of_bits(uint32_t b) {
    if (b == 0x80000000u) b = 0u;
    return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}

__device__ __forceinline__ uint32_t bits_of_key(uint32_t k) {
    return (k & 0x80000000u) ? (k ^ 0x80000000u) : ~k;
}

// (logit descending, id ascending) == composite descending.  Composites of distinct ids differ.
__device__ __forceinline__ uint64_t composite_of(uint32_t bits, uint32_t id) {
    return ((uint64_t)key_of_bits(bits) << 32) | (uint64_t)(0xFFFFFFFFu - id);
}

// ---------------------------------------------------------------- exponentials

// exp((x - m) / T) for the streaming sums: one subtract, one multiply, one v_exp_f32.
// c = log2(e) / T.
__device__ __forceinline__ float exp_stream(float x, float m, float c) {
    return __builtin_amdgcn_exp2f((x - m) * c);
}

// exp((x - m) / T) for values that are emitted (probabilities): the exponent is formed in fp64 and
// split into integer and fraction so that its magnitude does not cost relative accuracy.
__device__ __forceinline__ double exp_emit(float x, float m, double c) {
    double a = ((double)x - (double)m) * c;      // <= 0 for x <= m
    if (!(a > -1100.0)) return 0.0;               // also catches x = -inf
    double n = rint(a);
    float f = (float)(a - n);                     // |f| <= 0.5, exact difference
    return ldexp((double)exp2f(f), (int)n);
}

// 2^a for a double exponent of any magnitude (split into integer and fraction as in exp_emit).
__device__ __forceinline__ double exp2_split(double a) {
    if (!(a > -1100.0)) return 0.0;
    double n = rint(a);
    return ldexp((double)exp2f((float)(a - n)), (int)n);
}

// ---------------------------------------------------------------- row streaming
//
// A row of V elements is read as 16-byte vectors.  If the row does not start on a 16-byte
// boundary the vectors are taken from the aligned address below it and the elements in front of
// the row (and behind its end) are masked: an aligned 16-byte block that contains one valid byte
// never leaves the page that byte lives on.  `o` = number of masked elements in front (0 for
// aligned rows), virtual element v = o + x.

template <bool BF16> struct Vec;
template <> struct Vec<false> { static constexpr int N = 4; };   // 4 x fp32
template <> struct Vec<true>  { static constexpr int N = 8; };   // 8 x bf16

struct RowView {
    const uint4* base;   // 16-byte aligned
    int o;               // leading masked elements
    int L;               // o + V
};

template <bool BF16>
__device__ __forceinline__ RowView row_view(const void* logits, int64_t ld, int64_t row, int V) {
    const int esz = BF16 ? 2 : 4;
    const int64_t byte_off = row * ld * esz;
    const int mis = (int)(((uintptr_t)logits + (uintptr_t)byte_off) & 15u);
    RowView r;
    r.o = mis / esz;
    r.base = (const uint4*)((const char*)logits + (byte_off - mis));   // pointer arithmetic keeps the global address space
    r.L = r.o + V;
    return r;
}

// Bit e of the result is set iff element e of vector q lies inside the row.
template <bool BF16>
__device__ __forceinline__ unsigned vec_valid_mask(const RowView& r, int q) {
    const int n = Vec<BF16>::N;
    const int x = q * n - r.o;                  // id of the vector's element 0
    const int lo = x < 0 ? (x < -n ? n : -x) : 0;
    const int V = r.L - r.o;
    const int hi = V - x < 0 ? 0 : (V - x > n ? n : V - x);
    return hi > lo ? (((1u << hi) - 1u) & ~((1u << lo) - 1u)) : 0u;
}

// Vector q (in units of 16 bytes from base); returns false (and leaves `out` untouched) if the
// vector lies wholly outside [o, L).
template <bool BF16>
__device__ __forceinline__ bool vec_in_row(const RowView& r, int q) {
    const int n = Vec<BF16>::N;
    int v0 = q * n;
    return (v0 < r.L) && (v0 + n > r.o);
}

// 16-byte streaming load: the logits are read once, so they are marked non-temporal (measured on
// gfx950: 7.0 TB/s against 6.3 TB/s for plain loads in a read-only sweep).
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint4 load16_stream(const uint4* p) {
    const u32x4_t v = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(p));
    return make_uint4(v.x, v.y, v.z, v.w);
}

// Unpack a 16-byte vector into fp32 values (exact widening for bf16).
template <bool BF16>
__device__ __forceinline__ void unpack(const uint4& raw, float (&out)[Vec<BF16>::N]) {
    if constexpr (BF16) {
        out[0] = __uint_as_float(raw.x << 16); out[1] = __uint_as_float(raw.x & 0xFFFF0000u);
        out[2] = __uint_as_float(raw.y << 16); out[3] = __uint_as_float(raw.y & 0xFFFF0000u);
        out[4] = __uint_as_float(raw.z << 16); out[5] = __uint_as_float(raw.z & 0xFFFF0000u);
        out[6] = __uint_as_float(raw.w << 16); out[7] = __uint_as_float(raw.w & 0xFFFF0000u);
    } else {
        out[0] = __uint_as_float(raw.x); out[1] = __uint_as_float(raw.y);
        out[2] = __uint_as_float(raw.z); out[3] = __uint_as_float(raw.w);
    }
}

// One logit by vocabulary id (random access).
template <bool BF16>
__device__ __forceinline__ float logit_at(const void* logits, int64_t ld, int64_t row, int x) {
    if constexpr (BF16) {
        const uint16_t* p = (const uint16_t*)logits + row * ld + x;
        return __uint_as_float((uint32_t)(*p) << 16);
    } else {
        return ((const float*)logits)[row * ld + x];
    }
}

// Per-thread online softmax state: s = sum exp((x - m)/T) over the elements this thread has seen.
struct OnlineSum {
    float m = kNegInf;
    float s = 0.f;
    // raise the reference to at least bm (the maximum of the next elements) before adding them
    __device__ __forceinline__ float rebase(float bm, float c) {
        if (bm > m) {
            s *= __builtin_amdgcn_exp2f((m - bm) * c);   // m = -inf: exp2(-inf) = 0, s stays 0
            m = bm;
        }
        return m == kNegInf ? 0.f : m;                    // reference for rows of only -inf so far
    }
};

// Combine the per-thread (m, s) of a workgroup of WAVES waves.  Result in every thread: M = max m,
// S = sum s * exp((m - M)/T) accumulated in fp64.  `sh` needs 2*WAVES doubles.
template <int WAVES = kWaves>
__device__ __forceinline__ void block_softmax_stats(float m, float s, float c, double* sh, float& M, double& S) {
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
    float wm = wave_max(m);
    if (lane == 0) sh[wave] = (double)wm;
    __syncthreads();
    float bm = kNegInf;
#pragma unroll
    for (int w = 0; w < WAVES; ++w) bm = fmaxf(bm, (float)sh[w]);
    float scaled = (m == kNegInf) ? 0.f : s * __builtin_amdgcn_exp2f((m - bm) * c);
    double ws = wave_sum((double)scaled);
    if (lane == 0) sh[WAVES + wave] = ws;
    __syncthreads();
    double tot = 0.0;
#pragma unroll
    for (int w = 0; w < WAVES; ++w) tot += sh[WAVES + w];
    __syncthreads();
    M = bm;
    S = tot;
}

// ---------------------------------------------------------------- streaming row statistics

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

// The same statistics, and besides them the row's exponential sums segment by segment (what lets the residual draw
// locate its token without a second pass over the row).  A wave owns NV * 64 consecutive vectors per trip, one
// segment; segment `it * WAVES + wave` of the row gets (t, r): the sum over its elements of 2^(z c - r), c = log2(e) / T,
// with r an integer-valued reference exponent that is the same for the whole wave (every lane adds against it, so the
// trip's sum is one wave-wide addition; it moves up, and the lanes' running sums are rescaled, only when an element
// lies more than 2^64 above it: the check is one compare per trip).  Row layout of the table: seg[row * seg_stride + s].
// STAGE_GIVEN: the caller lends kSegStage float2 of LDS for the row's table (a kernel whose workgroups hold a
// large buffer for another job); otherwise the function owns them.
constexpr int kSegStage = 1040;                  // segments of the longest row (2^20 elements)
template <bool BF16, int NV, int THREADS, bool STAGE_GIVEN = false>
__device__ __forceinline__ void row_stats_seg_row(
    const int64_t row, const void* __restrict__ logits, int64_t ld, int V, float inv_T,
    float* __restrict__ row_max, float* __restrict__ row_sum, float* __restrict__ row_lse,
    float2* __restrict__ seg, int seg_stride, float2* stage = nullptr)
{
    constexpr int WAVES = THREADS / kWave;
    __shared__ double red[2 * WAVES];
    // the row's table is gathered in LDS and written once, in whole lines, at the end of the row
    constexpr int kSegLds = kSegStage;
    float2* seg_lds = stage;
    if constexpr (!STAGE_GIVEN) {
        __shared__ float2 own_stage[kSegLds];
        seg_lds = own_stage;
    }
    constexpr int N = Vec<BF16>::N, E = NV * N, TILE_VECS = THREADS * NV;
    static_assert(E <= 32, "one bit of the validity mask per element");
    const int tid = threadIdx.x, lane = tid & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(tid / kWave);
    const RowView rv = row_view<BF16>(logits, ld, row, V);
    const int nq = (rv.L + N - 1) / N;
    const int n_tiles = (nq + TILE_VECS - 1) / TILE_VECS;
    const float c = 1.4426950408889634f * inv_T;
    float2* const seg_row = seg + row * (int64_t)seg_stride;

    uint4 cur[NV], nxt[NV];
    // vector j of this lane in trip `it`: it * TILE_VECS + wave * (NV * 64) + j * 64 + lane
    const int q_lane = wave * (NV * kWave) + lane;
    auto load_tile = [&](int it, uint4 (&dst)[NV]) {
#pragma unroll
        for (int j = 0; j < NV; ++j) {
            const int q = it * TILE_VECS + q_lane + j * kWave;
            dst[j] = make_uint4(0, 0, 0, 0);
            if (vec_in_row<BF16>(rv, q)) dst[j] = load16_stream(rv.base + q);
        }
    };
    load_tile(0, cur);
    float mx = kNegInf;          // this lane's largest value
    float r_w = kNegInf;         // the wave's reference exponent (uniform)
    float s = 0.f;               // this lane's sum of 2^(z c - r_w)
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
            for (int j = 0; j < NV; ++j) vm |= vec_valid_mask<BF16>(rv, it * TILE_VECS + q_lane + j * kWave) << (j * N);
#pragma unroll
            for (int e = 0; e < E; ++e) v[e] = (vm >> e) & 1u ? v[e] : kNegInf;
        }
        float bm = v[0];
#pragma unroll
        for (int e = 1; e < E; ++e) bm = fmaxf(bm, v[e]);
        mx = fmaxf(mx, bm);
        if (__ballot(bm * c > r_w + 64.f)) {                     // (uniform; the first trip, and outliers)
            const float rn = ceilf(wave_max(bm) * c);
            if (rn > r_w) { s *= __builtin_amdgcn_exp2f(r_w - rn); r_w = rn; }   // r_w = -inf: s is 0 and stays 0
        }
        const float nr = r_w == kNegInf ? 0.f : -r_w;           // waves that have seen only -inf so far
        float acc = 0.f;
#pragma unroll
        for (int e = 0; e < E; ++e) acc += __builtin_amdgcn_exp2f(fmaf(v[e], c, nr));
        s += acc;
        const float t = wave_sum_last(acc);
        if (lane == kWave - 1 && it * WAVES + wave < kSegLds) seg_lds[it * WAVES + wave] = make_float2(t, r_w);   // (r_w = -inf with t = 0: the reader skips it)
#pragma unroll
        for (int j = 0; j < NV; ++j) cur[j] = nxt[j];
    }
    // M = max over the block; S = sum of s 2^(r_w - M c), combined in fp64
    const float wm = wave_max(mx);
    if (lane == 0) red[wave] = (double)wm;
    __syncthreads();
    {   // (non-temporal stores: ordinary ones, which allocate their lines in the L2, cost this pass 5 % of its bandwidth)
        typedef float f32x2_t __attribute__((ext_vector_type(2)));
        for (int sg = tid; sg < min(n_tiles * WAVES, min(seg_stride, kSegLds)); sg += THREADS) {
            const float2 e = seg_lds[sg];
            const f32x2_t ev = {e.x, e.y};
            __builtin_nontemporal_store(ev, reinterpret_cast<f32x2_t*>(&seg_row[sg]));
        }
    }
    float M = kNegInf;
#pragma unroll
    for (int w = 0; w < WAVES; ++w) M = fmaxf(M, (float)red[w]);
    const double mine = r_w == kNegInf ? 0.0 : (double)s * exp2_split((double)r_w - (double)M * (double)c);
    const double ws = wave_sum(mine);
    if (lane == 0) red[WAVES + wave] = ws;
    __syncthreads();
    double S = 0.0;
#pragma unroll
    for (int w = 0; w < WAVES; ++w) S += red[WAVES + w];
    if (tid == 0) {
        row_max[row] = M;
        row_sum[row] = (float)S;
        if (row_lse) row_lse[row] = (float)((double)M * (double)inv_T + log(S));
    }
}

// Largest float below x (x finite or +inf); -inf stays -inf.  x >= t  <=>  x > float_below(t) for non-NaN x.
__device__ __forceinline__ float float_below(float t) {
    uint32_t b = __float_as_uint(t);
    if (t == kNegInf) return t;
    if ((b << 1) == 0u) return __uint_as_float(0x80000001u);   // +-0 -> smallest negative subnormal
    return __uint_as_float((b & 0x80000000u) ? b + 1u : b - 1u);
}

}  // namespace picospec
