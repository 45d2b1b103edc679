// Sparse Top-K compression of vocabulary distributions (paper Section 3.3, Eq. 4) fused with the
// softmax statistics, one workgroup per row, one HBM pass per row.
//
// Streaming selection: a row is read in tiles of 16-byte vectors.  Elements above the running
// threshold tau (the k-th largest logit seen so far; everything is admitted until tau exists) are
// appended to a candidate buffer in LDS.  When the buffer is full it is pruned back to the exact
// top k by a radix select (12-bit digits, LDS histogram) on a composite key
//     (order-preserving logit key) << 20 | (2^20 - 1 - id)
// whose descending order is (logit descending, id ascending); tau rises and the stream continues.
// Rows are streamed in ascending id order, so among equal logits the ones already held win: after
// a prune the admission test is strict.  At the end the k survivors are ordered by a histogram
// rank sort, their probabilities are formed from the row's (max, sum) and the record is written
// once.
#include "common.hpp"
#include "kernels.hpp"

namespace picospec {

namespace {

constexpr int kCap = 16384;                 // candidate slots in LDS (8 bytes each)
constexpr int kPer = kCap / kThreads;       // candidates per thread during a prune
constexpr int kBinsLog2 = 12;
constexpr int kBins = 1 << kBinsLog2;       // histogram bins of the radix select / rank sort
constexpr int kBinsPer = kBins / kThreads;
constexpr int kIdBits = 20;                 // ids < 2^20 (kMaxV)
constexpr unsigned kIdMask = (1u << kIdBits) - 1u;
constexpr int kSortMaxBin = 48;             // rank sort falls back to a bitonic network beyond this bin size

static_assert(kMaxK * 3 <= kCap, "the rank sort uses three k-sized regions of the candidate buffer");
static_assert(kMaxV <= (1 << kIdBits), "id field of the composite key");
static_assert(kCap <= 65536 && 2 * kMaxK * 2 <= kBins * 4, "prune keeps two 16-bit index lists in the histogram");

struct __align__(16) CompressShared {
    uint2 cand[kCap];                       // (fp32 bit pattern, id); the sort reuses it as uint64 regions
    unsigned hist[kBins];
    double red[2 * kWaves];
    unsigned long long red64[2 * kWaves];
    int wtot[kWaves];
    unsigned minkey[kWaves];
    int cnt;                                // candidates held
    int n_holes, n_fills;                   // compaction lists of a prune
    int piv_rbin, piv_above, piv_count;     // radix-select broadcast
    int maxbin;
    int epoch_overflow[3];                  // per attempt epoch: some wave did not fit
    int epoch_valid[3];                     // per attempt epoch: first reservation that did not fit
};

static_assert(sizeof(CompressShared) <= 160 * 1024, "LDS budget of one gfx950 CU");

// Composite key.  For bf16 rows the low 16 bits of every fp32 key are zero and are dropped, so the
// key field has no dead bits between the logit and the id.
template <bool BF16>
__device__ __forceinline__ uint64_t composite(uint2 e) {
    uint32_t key = key_of_bits(e.x);
    if constexpr (BF16) key >>= 16;
    return ((uint64_t)key << kIdBits) | (uint64_t)(kIdMask - e.y);
}

template <bool BF16>
__device__ __forceinline__ uint2 entry_of(uint64_t c) {
    uint32_t key = (uint32_t)(c >> kIdBits);
    if constexpr (BF16) key = (key << 16) | ((key & 0x8000u) ? 0u : 0xFFFFu);   // keys of negative values end in ones
    return make_uint2(bits_of_key(key), kIdMask - ((uint32_t)c & kIdMask));
}

// Exclusive prefix sum over the kBins counters in sh.hist (in place), each thread owning kBinsPer
// consecutive bins.  Returns this thread's first exclusive prefix; `loc` receives its bins' total.
// Also records the largest bin in sh.maxbin when `track_max`.
__device__ __forceinline__ int scan_hist(CompressShared& sh, int (&h)[kBinsPer], int& loc) {
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
    loc = 0;
#pragma unroll
    for (int j = 0; j < kBinsPer; ++j) { h[j] = (int)sh.hist[tid * kBinsPer + j]; loc += h[j]; }
    const int incl = wave_scan_incl(loc);
    if (lane == kWave - 1) sh.wtot[wave] = incl;
    __syncthreads();
    int before = 0;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) before += (w < wave) ? sh.wtot[w] : 0;
    return before + incl - loc;
}

// Composite threshold T with exactly `need` of the n > need candidates >= T.
template <bool BF16>
__device__ __forceinline__ uint64_t select_threshold(CompressShared& sh, int n, int need) {
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
    uint64_t mn = ~0ull, mx = 0ull;
#pragma unroll
    for (int j = 0; j < kPer; ++j) {
        const int i = tid + j * kThreads;
        if (i < n) {
            const uint64_t c = composite<BF16>(sh.cand[i]);
            mn = c < mn ? c : mn;
            mx = c > mx ? c : mx;
        }
    }
    mn = wave_min_u64(mn);
    mx = wave_max_u64(mx);
    if (lane == 0) { sh.red64[wave] = mn; sh.red64[kWaves + wave] = mx; }
    __syncthreads();
    uint64_t lo = ~0ull, hi = 0ull;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) {
        const uint64_t a = sh.red64[w], b = sh.red64[kWaves + w];
        lo = a < lo ? a : lo;
        hi = b > hi ? b : hi;
    }
    const uint64_t range = hi - lo;
    const int nb = range ? 64 - __clzll((long long)range) : 1;
    int shift = nb > kBinsLog2 ? nb - kBinsLog2 : 0;
    int wbits = 63;   // the window [lo, lo + 2^wbits) holds the candidates still undecided (composites are < 2^52)
    for (;;) {
#pragma unroll
        for (int j = 0; j < kBinsPer; ++j) sh.hist[tid + j * kThreads] = 0;
        __syncthreads();
#pragma unroll
        for (int j = 0; j < kPer; ++j) {
            const int i = tid + j * kThreads;
            if (i < n) {
                const uint64_t d = composite<BF16>(sh.cand[i]) - lo;   // below the window wraps to >= 2^63
                if ((d >> wbits) == 0) atomicAdd(&sh.hist[kBins - 1 - (int)(d >> shift)], 1u);   // reversed: descending
            }
        }
        __syncthreads();
        int h[kBinsPer], loc;
        const int excl = scan_hist(sh, h, loc);
        if (excl < need && need <= excl + loc) {   // exactly one thread owns the pivot bin
            int a = excl, j = 0;
            while (a + h[j] < need) { a += h[j]; ++j; }
            sh.piv_rbin = tid * kBinsPer + j;
            sh.piv_above = a;
            sh.piv_count = h[j];
        }
        __syncthreads();
        const int bin = kBins - 1 - sh.piv_rbin;
        need -= sh.piv_above;
        const int bcount = sh.piv_count;
        lo += (uint64_t)bin << shift;
        if (need == bcount || shift == 0) return lo;   // the whole pivot bin is kept
        wbits = shift;
        shift = shift > kBinsLog2 ? shift - kBinsLog2 : 0;
    }
}

// Reduce the n > k candidates to exactly the k largest composites, compacted to the front in any
// order: survivors already in the first k slots stay, the other survivors fill the slots that
// were vacated there.  Returns the new threshold: the smallest kept logit.
template <bool BF16>
__device__ __forceinline__ float prune_to_k(CompressShared& sh, int n, int k) {
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
    const uint64_t T = select_threshold<BF16>(sh, n, k);
    // the histogram is free now: it holds the two index lists (k <= kMaxK <= kBins * 2 / 2 entries of 16 bits each)
    uint16_t* holes = reinterpret_cast<uint16_t*>(sh.hist);
    uint16_t* fills = holes + kMaxK;
    if (tid == 0) { sh.n_holes = 0; sh.n_fills = 0; }
    __syncthreads();
    unsigned mk = 0xFFFFFFFFu;
#pragma unroll 4
    for (int j = 0; j < kPer; ++j) {
        const int i = tid + j * kThreads;
        bool hole = false, fill = false;
        if (i < n) {
            const uint2 e = sh.cand[i];
            const bool kept = composite<BF16>(e) >= T;
            if (kept) { const unsigned key = key_of_bits(e.x); mk = key < mk ? key : mk; }
            hole = !kept && i < k;
            fill = kept && i >= k;
        }
        const unsigned long long hm = __ballot(hole), fm = __ballot(fill);
        const unsigned long long below = (1ull << lane) - 1ull;
        if (hm) {
            int base = 0;
            if (lane == 0) base = atomicAdd(&sh.n_holes, __popcll(hm));
            base = __shfl(base, 0, kWave);
            if (hole) holes[base + __popcll(hm & below)] = (uint16_t)i;
        }
        if (fm) {
            int base = 0;
            if (lane == 0) base = atomicAdd(&sh.n_fills, __popcll(fm));
            base = __shfl(base, 0, kWave);
            if (fill) fills[base + __popcll(fm & below)] = (uint16_t)i;
        }
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) { const unsigned w = __shfl_xor(mk, o, kWave); mk = w < mk ? w : mk; }
    if (lane == 0) sh.minkey[wave] = mk;
    __syncthreads();
    const int nh = sh.n_holes;   // == n_fills: exactly k candidates are kept
    for (int t = tid; t < nh; t += kThreads) sh.cand[holes[t]] = sh.cand[fills[t]];
    unsigned tk = 0xFFFFFFFFu;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) { const unsigned a = sh.minkey[w]; tk = a < tk ? a : tk; }
    if (tid == 0) sh.cnt = k;
    __syncthreads();
    return __uint_as_float(bits_of_key(tk));
}

// Descending bitonic sort of P (power of two) uint64 values in LDS.
__device__ __forceinline__ void bitonic_sort_desc(uint64_t* a, int P) {
    for (int size = 2; size <= P; size <<= 1)
        for (int stride = size >> 1; stride > 0; stride >>= 1) {
            __syncthreads();
            for (int t = threadIdx.x; t < (P >> 1); t += kThreads) {
                const int i = 2 * t - (t & (stride - 1)), j = i + stride;
                const bool desc = (i & size) == 0;
                const uint64_t x = a[i], y = a[j];
                if ((x < y) == desc) { a[i] = y; a[j] = x; }
            }
        }
    __syncthreads();
}

// Order the n <= kMaxK candidates at the front of sh.cand by composite, descending.  Returns the
// LDS array holding the sorted composites.  Histogram rank sort: one pass bins the composites
// (12 bits below the highest differing bit), a prefix sum places the bins, and each element's
// place inside its bin is the number of larger bin-mates.
template <bool BF16>
__device__ __forceinline__ const uint64_t* sort_candidates(CompressShared& sh, int n) {
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
    constexpr int PER = kMaxK / kThreads;
    uint64_t* region = reinterpret_cast<uint64_t*>(sh.cand);
    uint64_t* tmp = region + kMaxK;
    uint64_t* out = region + 2 * kMaxK;
    uint64_t c[PER];
    uint64_t mn = ~0ull, mx = 0ull;
#pragma unroll
    for (int j = 0; j < PER; ++j) {
        const int i = tid + j * kThreads;
        c[j] = 0;
        if (i < n) {
            c[j] = composite<BF16>(sh.cand[i]);
            mn = c[j] < mn ? c[j] : mn;
            mx = c[j] > mx ? c[j] : mx;
        }
    }
    mn = wave_min_u64(mn);
    mx = wave_max_u64(mx);
    if (lane == 0) { sh.red64[wave] = mn; sh.red64[kWaves + wave] = mx; }
#pragma unroll
    for (int j = 0; j < kBinsPer; ++j) sh.hist[tid + j * kThreads] = 0;
    if (tid == 0) sh.maxbin = 0;
    __syncthreads();
    uint64_t lo = ~0ull, hi = 0ull;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) {
        const uint64_t a = sh.red64[w], b = sh.red64[kWaves + w];
        lo = a < lo ? a : lo;
        hi = b > hi ? b : hi;
    }
    const uint64_t range = hi >= lo ? hi - lo : 0;
    const int nb = range ? 64 - __clzll((long long)range) : 1;
    const int shift = nb > kBinsLog2 ? nb - kBinsLog2 : 0;
    int rbin[PER], arrival[PER];
#pragma unroll
    for (int j = 0; j < PER; ++j) {
        const int i = tid + j * kThreads;
        rbin[j] = 0; arrival[j] = 0;
        if (i < n) {
            rbin[j] = kBins - 1 - (int)((c[j] - lo) >> shift);
            arrival[j] = (int)atomicAdd(&sh.hist[rbin[j]], 1u);
        }
    }
    __syncthreads();
    int h[kBinsPer], loc;
    int excl = scan_hist(sh, h, loc);
    int big = 0;
#pragma unroll
    for (int j = 0; j < kBinsPer; ++j) big = max(big, h[j]);
    if (big > kSortMaxBin) atomicMax(&sh.maxbin, big);
    __syncthreads();   // every thread has read its counters
#pragma unroll
    for (int j = 0; j < kBinsPer; ++j) { sh.hist[tid * kBinsPer + j] = (unsigned)excl; excl += h[j]; }
    __syncthreads();
    if (sh.maxbin > kSortMaxBin) {   // degenerate spread (one outlier stretching the range): plain network
        int P = 1;
        while (P < n) P <<= 1;
        for (int i = tid; i < P; i += kThreads) tmp[i] = 0;
        __syncthreads();
#pragma unroll
        for (int j = 0; j < PER; ++j) { const int i = tid + j * kThreads; if (i < n) tmp[i] = c[j]; }
        bitonic_sort_desc(tmp, P);
        return tmp;
    }
#pragma unroll
    for (int j = 0; j < PER; ++j) {
        const int i = tid + j * kThreads;
        if (i < n) tmp[(int)sh.hist[rbin[j]] + arrival[j]] = c[j];
    }
    __syncthreads();
#pragma unroll
    for (int j = 0; j < PER; ++j) {
        const int i = tid + j * kThreads;
        if (i < n) {
            const int s = (int)sh.hist[rbin[j]];
            const int e = rbin[j] + 1 < kBins ? (int)sh.hist[rbin[j] + 1] : n;
            int larger = 0;
            for (int q = s; q < e; ++q) larger += tmp[q] > c[j] ? 1 : 0;
            out[s + larger] = c[j];
        }
    }
    __syncthreads();
    return out;
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
    static_assert(E <= 16, "pass mask is 16 bits wide");
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
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
            const int q = it * (kThreads * NV) + j * kThreads + tid;
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
        const bool last = it + 1 == n_tiles;
        if (!last) load_tile(it + 1, nxt);
        float v[E];
#pragma unroll
        for (int j = 0; j < NV; ++j) {
            float t[N];
            unpack<BF16>(cur[j], t);
#pragma unroll
            for (int e = 0; e < N; ++e) v[j * N + e] = t[e];
        }
        // elements outside the row (alignment prologue, tail) are masked
        unsigned vm = (1u << E) - 1u;
        const int x0 = it * TILE - rv.o;          // id of this tile's virtual element 0
        if (it == 0 || last) {
            vm = 0;
#pragma unroll
            for (int j = 0; j < NV; ++j)
                vm |= vec_valid_mask<BF16>(rv, it * (kThreads * NV) + j * kThreads + tid) << (j * N);
#pragma unroll
            for (int e = 0; e < E; ++e) v[e] = (vm >> e) & 1u ? v[e] : kNegInf;
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
                    const bool pass = admit_all ? (v[e] >= kNegInf) : (v[e] > tau);
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
                                if (pm & (1u << (j * N + e))) {
                                    sh.cand[p] = make_uint2(__float_as_uint(v[j * N + e]),
                                                            (unsigned)(x0 + (j * kThreads + tid) * N + e));
                                    ++p;
                                }
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
            int n_held = sh.epoch_valid[epoch];
            // the slot two epochs ahead was last read before the barrier above and is next written
            // after the next barrier
            if (tid == 0) { const int e2 = (epoch + 2) % 3; sh.epoch_overflow[e2] = 0; sh.epoch_valid[e2] = 0x7FFFFFFF; }
            epoch = (epoch + 1) % 3;
            // after the last tile the survivors are cut to k by the same code
            bool final_cut = false;
            if (!overflow) {
                if (!last) break;
                n_held = sh.cnt;
                if (n_held <= k) break;
                final_cut = true;
            }
            tau = prune_to_k<BF16>(sh, n_held, k);
            admit_all = false;
            if (final_cut) break;
        }
#pragma unroll
        for (int j = 0; j < NV; ++j) cur[j] = nxt[j];
    }

    // ---- ordering and emission
    const int n = sh.cnt;
    float M; double S;
    block_softmax_stats(os.m, os.s, c, sh.red, M, S);
    const uint64_t* sorted = sort_candidates<BF16>(sh, n);

    const double cd = 1.4426950408889634 * (double)inv_T;
    const double invS = 1.0 / S;
    const bool use_top_p = top_p > 0.f && top_p < 1.f;
    double carry = 0.0, my_mass = 0.0;
    int my_count = 0;
    int32_t* idx_row = idx + row * (int64_t)k;
    float* prob_row = prob + row * (int64_t)k;
    for (int j0 = 0; j0 < k; j0 += kThreads) {
        const int slot = j0 + tid;
        int id = -1;
        float pr = 0.f;
        if (slot < n) {
            const uint2 e = entry_of<BF16>(sorted[slot]);
            id = (int)e.y;
            pr = (float)(exp_emit(__uint_as_float(e.x), M, cd) * invS);
        }
        bool keep = slot < n;
        if (use_top_p) {   // keep a slot iff the probability before it has not reached top_p
            const double mine = (double)pr;
            const double incl = wave_scan_incl(mine);
            if (lane == kWave - 1) sh.red[wave] = incl;
            __syncthreads();
            double before = carry, tot = 0.0;
#pragma unroll
            for (int w = 0; w < kWaves; ++w) { const double t = sh.red[w]; if (w < wave) before += t; tot += t; }
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
    const double wm = wave_sum(my_mass);
    const int wc = wave_sum(my_count);
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
    const int s0 = min(cnt, lane * per), s1 = min(cnt, s0 + per);
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
