// Sparse Top-K compression of vocabulary distributions (paper Section 3.3, Eq. 4) fused with the
// softmax statistics, one workgroup per row, one HBM pass per row.
//
// Streaming selection: a row is read in tiles of 16-byte vectors.  Elements above the running
// threshold tau (the k-th largest logit seen so far; everything is admitted until tau exists) are
// appended to a candidate buffer in LDS.  When the buffer is full it is pruned back to the exact
// top k by a radix select on the 64-bit composite (order-preserving logit key, ~id); tau rises and
// the stream continues.  Rows are streamed in ascending id order, so among equal logits the ones
// already held win: after a prune the admission test is strict.  At the end the k survivors are
// sorted by composite (logit descending, id ascending), their probabilities are formed from the
// row's (max, sum) and the record is written once.
#include "common.hpp"
#include "kernels.hpp"

namespace picospec {

namespace {

constexpr int kCap = 16384;                 // candidate slots in LDS (8 bytes each)
constexpr int kPer = kCap / kThreads;       // candidates a thread holds during a prune
constexpr int kBins = 256;

struct __align__(16) CompressShared {
    uint2 cand[kCap];                       // (fp32 bit pattern, id); reused as uint64 composites for the sort
    unsigned hist[kBins];
    double red[2 * kWaves];
    unsigned long long red64[2 * kWaves];
    int cnt;                                // candidates held
    int bucket, above, bcount;              // radix-select broadcast
    unsigned minkey[kWaves];
    int epoch_overflow[3];                  // per attempt epoch: some wave did not fit
    int epoch_valid[3];                     // per attempt epoch: first reservation that did not fit
};

static_assert(sizeof(CompressShared) <= 160 * 1024, "LDS budget of one gfx950 CU");

// Reduce the n > k candidates in sh.cand to exactly the k largest composites.  Returns the new
// threshold (the smallest kept logit).  All threads of the workgroup call this together.
__device__ float prune_to_k(CompressShared& sh, int n, int k) {
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
    uint64_t c[kPer];
    unsigned act = 0, kept = 0;
    uint64_t mn = ~0ull, mx = 0ull;
#pragma unroll
    for (int j = 0; j < kPer; ++j) {
        int i = tid + j * kThreads;
        c[j] = 0;
        if (i < n) {
            uint2 e = sh.cand[i];
            c[j] = composite_of(e.x, e.y);
            act |= 1u << j;
            mn = c[j] < mn ? c[j] : mn;
            mx = c[j] > mx ? c[j] : mx;
        }
    }
    mn = wave_min_u64(mn);
    mx = wave_max_u64(mx);
    if (lane == 0) { sh.red64[wave] = mn; sh.red64[kWaves + wave] = mx; }
    __syncthreads();
    uint64_t lo = ~0ull, hi = 0ull;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) {
        uint64_t a = sh.red64[w], b = sh.red64[kWaves + w];
        lo = a < lo ? a : lo;
        hi = b > hi ? b : hi;
    }
    const uint64_t range = hi - lo;
    const int nb = range ? 64 - __clzll((long long)range) : 1;
    int shift = nb > 8 ? nb - 8 : 0;
    int need = k;
    for (;;) {
        if (tid < kBins) sh.hist[tid] = 0;
        __syncthreads();
#pragma unroll
        for (int j = 0; j < kPer; ++j)
            if (act & (1u << j)) atomicAdd(&sh.hist[(unsigned)((c[j] - lo) >> shift) & (kBins - 1)], 1u);
        __syncthreads();
        if (wave == 0) {   // bins scanned from the top: lane l owns bins 255-4l .. 252-4l
            const int b0 = kBins - 1 - 4 * lane;
            const int h0 = sh.hist[b0], h1 = sh.hist[b0 - 1], h2 = sh.hist[b0 - 2], h3 = sh.hist[b0 - 3];
            const int loc = h0 + h1 + h2 + h3;
            const int incl = wave_scan_incl(loc), excl = incl - loc;
            if (excl < need && need <= incl) {
                int a = excl, b = b0, hb = h0;
                if (a + h0 < need) { a += h0; b = b0 - 1; hb = h1;
                    if (a + h1 < need) { a += h1; b = b0 - 2; hb = h2;
                        if (a + h2 < need) { a += h2; b = b0 - 3; hb = h3; } } }
                sh.bucket = b; sh.above = a; sh.bcount = hb;
            }
        }
        __syncthreads();
        const unsigned bucket = sh.bucket;
        const int above = sh.above, bcount = sh.bcount;
#pragma unroll
        for (int j = 0; j < kPer; ++j)
            if (act & (1u << j)) {
                unsigned d = (unsigned)((c[j] - lo) >> shift) & (kBins - 1);
                if (d > bucket) { kept |= 1u << j; act &= ~(1u << j); }
                else if (d < bucket) act &= ~(1u << j);
            }
        need -= above;
        if (need == bcount || shift == 0) { kept |= act; break; }   // shift == 0: composites are distinct, so bcount == need == 1
        shift = shift > 8 ? shift - 8 : 0;
    }
    // smallest kept key -> new threshold; compact the survivors to the front
    unsigned mk = 0xFFFFFFFFu;
#pragma unroll
    for (int j = 0; j < kPer; ++j)
        if (kept & (1u << j)) { unsigned kk = (unsigned)(c[j] >> 32); mk = kk < mk ? kk : mk; }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) { unsigned w = __shfl_xor(mk, o, kWave); mk = w < mk ? w : mk; }
    if (lane == 0) sh.minkey[wave] = mk;
    if (tid == 0) sh.cnt = 0;
    __syncthreads();
    const int ck = __popc(kept);
    const int incl = wave_scan_incl(ck), total = __shfl(incl, kWave - 1, kWave);
    int base = 0;
    if (lane == kWave - 1 && total > 0) base = atomicAdd(&sh.cnt, total);
    base = __shfl(base, kWave - 1, kWave);
    int p = base + incl - ck;
#pragma unroll
    for (int j = 0; j < kPer; ++j)
        if (kept & (1u << j)) sh.cand[p++] = make_uint2(bits_of_key((unsigned)(c[j] >> 32)), 0xFFFFFFFFu - (unsigned)c[j]);
    unsigned tk = 0xFFFFFFFFu;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) { unsigned a = sh.minkey[w]; tk = a < tk ? a : tk; }
    __syncthreads();
    return __uint_as_float(bits_of_key(tk));
}

// Descending bitonic sort of P (power of two) uint64 values in LDS.
__device__ void bitonic_sort_desc(uint64_t* a, int P) {
    for (int size = 2; size <= P; size <<= 1)
        for (int stride = size >> 1; stride > 0; stride >>= 1) {
            __syncthreads();
            for (int t = threadIdx.x; t < (P >> 1); t += kThreads) {
                int i = 2 * t - (t & (stride - 1)), j = i + stride;
                bool desc = (i & size) == 0;
                uint64_t x = a[i], y = a[j];
                if ((x < y) == desc) { a[i] = y; a[j] = x; }
            }
        }
    __syncthreads();
}

template <bool BF16, int NV>
__global__ __launch_bounds__(kThreads) void compress_kernel(
    const void* __restrict__ logits, int64_t ld, int V, float inv_T, int k, float top_p,
    int32_t* __restrict__ idx, float* __restrict__ prob, int32_t* __restrict__ count,
    float* __restrict__ mass, float* __restrict__ lse)
{
    extern __shared__ __align__(16) unsigned char smem_raw[];
    CompressShared& sh = *reinterpret_cast<CompressShared*>(smem_raw);
    constexpr int N = Vec<BF16>::N, E = NV * N, TILE = kThreads * E;
    const int tid = threadIdx.x, lane = tid & (kWave - 1);
    const int64_t row = blockIdx.x;
    const RowView rv = row_view<BF16>(logits, ld, row, V);
    const int n_tiles = (rv.L + TILE - 1) / TILE;
    const float c = 1.4426950408889634f * inv_T;

    if (tid == 0) {
        sh.cnt = 0;
        for (int e = 0; e < 3; ++e) { sh.epoch_overflow[e] = 0; sh.epoch_valid[e] = 0x7FFFFFFF; }
    }
    __syncthreads();

    uint4 cur[NV], nxt[NV];
    auto load_tile = [&](int it, uint4 (&dst)[NV]) {
#pragma unroll
        for (int j = 0; j < NV; ++j) {
            int q = it * (kThreads * NV) + j * kThreads + tid;
            dst[j] = make_uint4(0, 0, 0, 0);
            if (vec_in_row<BF16>(rv, q)) dst[j] = rv.base[q];
        }
    };
    load_tile(0, cur);

    OnlineSum os;
    float tau = kNegInf;
    bool admit_all = true;
    int epoch = 0;

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
        // elements outside the row (alignment prologue, tail) are masked
        unsigned vm = (1u << E) - 1u;   // E <= 16
        const int x0 = it * TILE - rv.o;          // id of this tile's virtual element 0
        if (it == 0 || it == n_tiles - 1) {
#pragma unroll
            for (int j = 0; j < NV; ++j)
#pragma unroll
                for (int e = 0; e < N; ++e) {
                    int x = x0 + (j * kThreads + tid) * N + e;
                    if (x < 0 || x >= V) { vm &= ~(1u << (j * N + e)); v[j * N + e] = kNegInf; }
                }
        }
        // softmax statistics
        float bm = v[0];
#pragma unroll
        for (int e = 1; e < E; ++e) bm = fmaxf(bm, v[e]);
        const float mref = os.rebase(bm, c);
        float acc = 0.f;
#pragma unroll
        for (int e = 0; e < E; ++e) acc += exp_stream(v[e], mref, c);
        os.s += acc;

        // candidate admission; retried after a prune when the buffer overflowed
        bool pending = true;
        for (;;) {
            if (pending) {
                unsigned pm = 0;
#pragma unroll
                for (int e = 0; e < E; ++e) {
                    bool pass = admit_all ? (v[e] >= kNegInf) : (v[e] > tau);
                    pm |= (pass ? 1u : 0u) << e;
                }
                pm &= vm;
                const int ck = __popc(pm);
                const int incl = wave_scan_incl(ck), total = __shfl(incl, kWave - 1, kWave);
                if (total > 0) {
                    int base = 0;
                    if (lane == kWave - 1) base = atomicAdd(&sh.cnt, total);
                    base = __shfl(base, kWave - 1, kWave);
                    if (base + total <= kCap) {
                        int p = base + incl - ck;
#pragma unroll
                        for (int j = 0; j < NV; ++j)
#pragma unroll
                            for (int e = 0; e < N; ++e)
                                if (pm & (1u << (j * N + e)))
                                    sh.cand[p++] = make_uint2(__float_as_uint(v[j * N + e]),
                                                              (unsigned)(x0 + (j * kThreads + tid) * N + e));
                        pending = false;
                    } else if (lane == kWave - 1) {
                        atomicMin(&sh.epoch_valid[epoch], base);
                        sh.epoch_overflow[epoch] = 1;
                    }
                } else {
                    pending = false;
                }
            }
            __syncthreads();
            const int overflow = sh.epoch_overflow[epoch];
            const int n_valid = sh.epoch_valid[epoch];
            // the slot two epochs ahead was last read before the barrier above and is next written
            // after the next barrier
            if (tid == 0) { int e2 = (epoch + 2) % 3; sh.epoch_overflow[e2] = 0; sh.epoch_valid[e2] = 0x7FFFFFFF; }
            epoch = (epoch + 1) % 3;
            if (!overflow) break;
            tau = prune_to_k(sh, n_valid, k);
            admit_all = false;
        }
#pragma unroll
        for (int j = 0; j < NV; ++j) cur[j] = nxt[j];
    }

    // ---- final selection, ordering and emission
    int n = sh.cnt;
    if (n > k) { prune_to_k(sh, n, k); n = k; }
    float M; double S;
    block_softmax_stats(os.m, os.s, c, sh.red, M, S);

    int P = 1;
    while (P < n) P <<= 1;
    uint64_t* comp = reinterpret_cast<uint64_t*>(sh.cand);
    for (int i = tid; i < P; i += kThreads) {
        uint64_t cv = 0;
        if (i < n) { uint2 e = sh.cand[i]; cv = composite_of(e.x, e.y); }
        comp[i] = cv;
    }
    bitonic_sort_desc(comp, P);

    const double cd = 1.4426950408889634 * (double)inv_T;
    const double invS = 1.0 / S;
    const bool use_top_p = top_p > 0.f && top_p < 1.f;
    const int wave = tid / kWave;
    double carry = 0.0, my_mass = 0.0;
    int my_count = 0;
    int32_t* idx_row = idx + row * (int64_t)k;
    float* prob_row = prob + row * (int64_t)k;
    for (int j0 = 0; j0 < k; j0 += kThreads) {
        const int slot = j0 + tid;
        int id = -1;
        float pr = 0.f;
        if (slot < n) {
            uint64_t cv = comp[slot];
            id = (int)(0xFFFFFFFFu - (unsigned)cv);
            float x = __uint_as_float(bits_of_key((unsigned)(cv >> 32)));
            pr = (float)(exp_emit(x, M, cd) * invS);
        }
        bool keep = slot < n;
        if (use_top_p) {   // keep a slot iff the probability before it has not reached top_p
            double mine = (double)pr;
            double incl = wave_scan_incl(mine);
            if (lane == kWave - 1) sh.red[wave] = incl;
            __syncthreads();
            double before = carry, tot = 0.0;
#pragma unroll
            for (int w = 0; w < kWaves; ++w) { double t = sh.red[w]; if (w < wave) before += t; tot += t; }
            __syncthreads();
            keep = keep && (before + incl - mine) < (double)top_p;
            carry += tot;
        }
        if (slot < k) {
            idx_row[slot] = keep ? id : -1;
            prob_row[slot] = keep ? pr : 0.f;
        }
        if (keep) { my_mass += (double)pr; ++my_count; }
    }
    double wm = wave_sum(my_mass);
    int wc = wave_sum(my_count);
    if (lane == 0) { sh.red[wave] = wm; sh.red[kWaves + wave] = (double)wc; }
    __syncthreads();
    if (tid == 0) {
        double tm = 0.0, tc = 0.0;
        for (int w = 0; w < kWaves; ++w) { tm += sh.red[w]; tc += sh.red[kWaves + w]; }
        mass[row] = (float)tm;
        count[row] = (int)tc;
        lse[row] = (float)((double)M * (double)inv_T + log(S));
    }
}

// The drafter's draw: inverse CDF over the used slots, one wave per row.
__global__ __launch_bounds__(256) void sample_draft_kernel(
    const int32_t* __restrict__ idx, const float* __restrict__ prob, const int32_t* __restrict__ count,
    const float* __restrict__ mass, int k, int n_rows, const float* __restrict__ uniforms,
    int32_t* __restrict__ tok, float* __restrict__ q_scalar)
{
    const int lane = threadIdx.x & (kWave - 1);
    const int64_t row = (int64_t)blockIdx.x * (blockDim.x / kWave) + threadIdx.x / kWave;
    if (row >= n_rows) return;
    const float* p = prob + row * k;
    int cnt = count[row];
    cnt = cnt < 0 ? 0 : (cnt > k ? k : cnt);
    if (cnt == 0) { if (lane == 0) { tok[row] = -1; if (q_scalar) q_scalar[row] = 0.f; } return; }
    // lane l owns the contiguous slots [l*per, (l+1)*per)
    const int per = (cnt + kWave - 1) / kWave;
    const int s0 = lane * per, s1 = min(cnt, s0 + per);
    double mine = 0.0;
    for (int s = s0; s < s1; ++s) mine += (double)p[s];
    const double incl = wave_scan_incl(mine);
    const double total = __shfl(incl, kWave - 1, kWave);
    const double target = (double)uniforms[row] * total;
    // first lane whose inclusive sum exceeds the target holds the slot
    const unsigned long long ball = __ballot(incl > target);
    int pick = -1;
    if (ball) {
        const int owner = __ffsll((long long)ball) - 1;
        if (lane == owner) {
            double cum = incl - mine;
            for (int s = s0; s < s1; ++s) { cum += (double)p[s]; if (cum > target) { pick = s; break; } }
            if (pick < 0) pick = s1 - 1;
        }
        pick = __shfl(pick, owner, kWave);
    } else {   // rounding: last slot with weight
        if (lane == 0) { pick = cnt - 1; while (pick > 0 && !(p[pick] > 0.f)) --pick; }
        pick = __shfl(pick, 0, kWave);
    }
    if (lane == 0) {
        tok[row] = idx[row * k + pick];
        if (q_scalar) q_scalar[row] = p[pick] / mass[row];
    }
}

}  // namespace

hipError_t launch_compress(const void* logits, int dtype, int64_t ld, int n_rows, int V, float temperature,
                           int k, float top_p, int32_t* idx, float* prob, int32_t* count, float* mass,
                           float* lse, hipStream_t stream)
{
    static bool attr_set[2] = {false, false};
    const size_t smem = sizeof(CompressShared);
    auto f32 = compress_kernel<false, 4>;
    auto b16 = compress_kernel<true, 2>;
    const int which = dtype == 1;
    if (!attr_set[which]) {
        hipError_t e = hipFuncSetAttribute(which ? (const void*)b16 : (const void*)f32,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        if (e != hipSuccess) return e;
        attr_set[which] = true;
    }
    if (n_rows == 0) return hipSuccess;
    const float inv_T = 1.0f / temperature;
    if (which) hipLaunchKernelGGL(b16, dim3(n_rows), dim3(kThreads), smem, stream, logits, ld, V, inv_T, k, top_p, idx, prob, count, mass, lse);
    else       hipLaunchKernelGGL(f32, dim3(n_rows), dim3(kThreads), smem, stream, logits, ld, V, inv_T, k, top_p, idx, prob, count, mass, lse);
    return hipGetLastError();
}

hipError_t launch_sample_draft(const int32_t* idx, const float* prob, const int32_t* count, const float* mass,
                               int k, int n_rows, const float* uniforms, int32_t* tok, float* q_scalar,
                               hipStream_t stream)
{
    if (n_rows == 0) return hipSuccess;
    const int rows_per_block = 256 / kWave;
    hipLaunchKernelGGL(sample_draft_kernel, dim3((n_rows + rows_per_block - 1) / rows_per_block), dim3(256), 0, stream,
                       idx, prob, count, mass, k, n_rows, uniforms, tok, q_scalar);
    return hipGetLastError();
}

}  // namespace picospec
