// Sparse Top-K compression of vocabulary distributions (paper Section 3.3, Eq. 4) fused with the
// softmax statistics: one workgroup of 512 threads per row, two workgroups per CU, one HBM pass
// per row.
//
// Streaming selection.  A row is read in tiles of 16-byte vectors (8192 elements per tile).
//   * Tile 0 is copied whole into a candidate buffer in LDS.  A radix select (11-bit digits, LDS
//     histogram) on the composite key
//         (order-preserving logit key) << 20 | (2^20 - 1 - id)
//     (descending composite == logit descending, id ascending) cuts it down and yields a threshold.
//   * Optimistic mode: the cut keeps the r largest of tile 0, r chosen so that about 1.3 k elements
//     of the whole row are expected at or above the r-th value (z = 4.5 sigma above k for
//     exchangeable rows).  Later tiles append every element >= that value.  If the row ends with
//     at least k candidates the exact top k is among them (nothing at or above the threshold was
//     dropped) and one final select finishes the job.
//   * Safe mode: the cut keeps the k largest seen so far; later elements must be strictly larger
//     than the k-th (rows are streamed in ascending id, so equal logits that come later lose).
//     Whenever the buffer would overflow it is pruned back to the exact top k, in either mode,
//     which also switches to safe mode.  A row whose optimistic threshold was too high (fewer
//     than k candidates at the end) is streamed again in safe mode.
//   * The k survivors are ordered by a histogram rank sort, their probabilities formed from the
//     row's (max, sum), and the record written once.
#include "common.hpp"
#include "kernels.hpp"

namespace picospec {

namespace {

constexpr int kT = 512;                     // threads per workgroup (8 waves)
constexpr int kW = kT / kWave;
constexpr int kCap = 8192;                  // candidate slots in LDS (8 bytes each)
constexpr int kPer = kCap / kT;             // candidates per thread during a select
constexpr int kBinsLog2 = 11;
constexpr int kBins = 1 << kBinsLog2;       // histogram bins of the radix select / rank sort
constexpr int kBinsPer = kBins / kT;
constexpr int kIdBits = 20;                 // ids < 2^20 (kMaxV)
constexpr unsigned kIdMask = (1u << kIdBits) - 1u;
constexpr int kSortMaxBin = 48;             // rank sort falls back to a bitonic network beyond this bin size
constexpr int kSortPer = kMaxK / kT;

static_assert(kMaxK * 2 <= kCap, "the rank sort uses two k-sized regions of the candidate buffer");
static_assert(kMaxV <= (1 << kIdBits), "id field of the composite key");
static_assert(kCap <= 65536 && kCap / 2 * 2 <= kBins * 4, "a prune keeps a 16-bit index list in the histogram");

struct __align__(16) CompressShared {
    unsigned cand_val[kCap];                // candidates: fp32 bit pattern ...
    unsigned cand_id[kCap];                 // ... and vocabulary id (the sort reuses both arrays as uint64 regions)
    unsigned hist[kBins];
    double red[2 * kW];
    int wtot[kW];
    unsigned wkey[2 * kW];
    int cnt;                                // candidates held
    int n_holes, n_fills;                   // compaction of a prune
    int piv_rbin, piv_above, piv_count;     // radix-select broadcast
    int maxbin;
    int epoch_overflow[3];                  // per attempt epoch: some wave did not fit
    int epoch_valid[3];                     // per attempt epoch: first reservation that did not fit
};

static_assert(sizeof(CompressShared) <= 80 * 1024, "two workgroups share the 160 KB of LDS of a gfx950 CU");

template <bool BF16>
__device__ __forceinline__ uint32_t short_key(uint32_t bits) {
    uint32_t key = key_of_bits(bits);
    if constexpr (BF16) key >>= 16;          // the low half of a widened bf16 key carries nothing
    return key;
}

// Composite key; for bf16 rows the key field is 16 bits wide so that no dead bits sit between
// the logit and the id.
template <bool BF16>
__device__ __forceinline__ uint64_t composite(uint2 e) {
    return ((uint64_t)short_key<BF16>(e.x) << kIdBits) | (uint64_t)(kIdMask - e.y);
}

template <bool BF16>
__device__ __forceinline__ uint2 entry_of(uint64_t c) {
    uint32_t key = (uint32_t)(c >> kIdBits);
    if constexpr (BF16) key = (key << 16) | ((key & 0x8000u) ? 0u : 0xFFFFu);   // keys of negative values end in ones
    return make_uint2(bits_of_key(key), kIdMask - ((uint32_t)c & kIdMask));
}

// Exclusive prefix sum over the kBins counters in sh.hist, each thread owning kBinsPer consecutive
// bins.  Returns this thread's first exclusive prefix; h[] its counters, `loc` their total.
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
    for (int w = 0; w < kW; ++w) before += (w < wave) ? sh.wtot[w] : 0;
    return before + incl - loc;
}

// Composite threshold T with exactly `need` of the n > need candidates >= T.  Every candidate's
// short key lies in [key_lo, key_hi].
template <bool BF16>
__device__ __forceinline__ uint64_t select_threshold(CompressShared& sh, int n, int need, uint32_t key_lo, uint32_t key_hi) {
    const int tid = threadIdx.x;
    uint64_t lo = (uint64_t)key_lo << kIdBits;
    const uint64_t range = (((uint64_t)key_hi << kIdBits) | kIdMask) - lo;
    const int nb = 64 - __clzll((long long)range);          // range >= kIdMask > 0
    int shift = nb > kBinsLog2 ? nb - kBinsLog2 : 0;
    int wbits = 63;   // the window [lo, lo + 2^wbits) holds the candidates still undecided (composites are < 2^52)
    for (;;) {
#pragma unroll
        for (int j = 0; j < kBinsPer; ++j) sh.hist[tid + j * kT] = 0;
        __syncthreads();
#pragma unroll 4
        for (int j = 0; j < kPer; ++j) {
            const int i = tid + j * kT;
            if (i < n) {
                const uint64_t d = composite<BF16>(make_uint2(sh.cand_val[i], sh.cand_id[i])) - lo;   // below the window wraps to >= 2^63
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

// Reduce the n > target candidates to exactly the `target` largest composites, compacted to the
// front in any order: survivors already in the first `target` slots stay, the others fill the slots
// vacated there.  With `with_ties` every candidate whose logit equals the target-th one is kept as
// well (sh.cnt then exceeds target).  Returns the smallest kept logit.
template <bool BF16>
__device__ __forceinline__ float prune_to(CompressShared& sh, int n, int target, uint32_t key_lo, uint32_t key_hi,
                                          bool with_ties) {
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
    uint64_t T = select_threshold<BF16>(sh, n, target, key_lo, key_hi);
    if (with_ties) {   // keep every candidate whose logit equals the target-th one: count them first
        T = (T >> kIdBits) << kIdBits;
        int mine = 0;
#pragma unroll 4
        for (int j = 0; j < kPer; ++j) {
            const int i = tid + j * kT;
            if (i < n) mine += composite<BF16>(make_uint2(sh.cand_val[i], sh.cand_id[i])) >= T ? 1 : 0;
        }
        mine = wave_sum(mine);
        if (lane == 0) sh.wtot[wave] = mine;
        __syncthreads();
        target = 0;
#pragma unroll
        for (int w = 0; w < kW; ++w) target += sh.wtot[w];
    }
    uint16_t* holes = reinterpret_cast<uint16_t*>(sh.hist);   // the histogram is free now
    if (tid == 0) { sh.n_holes = 0; sh.n_fills = 0; }
    __syncthreads();
    const unsigned long long below = (1ull << lane) - 1ull;
    unsigned mk = 0xFFFFFFFFu;
#pragma unroll 4
    for (int j = 0; j < kPer; ++j) {   // list the vacated slots; track the smallest kept key
        const int i = tid + j * kT;
        bool hole = false;
        if (i < n) {
            const uint2 e = make_uint2(sh.cand_val[i], sh.cand_id[i]);
            const bool kept = composite<BF16>(e) >= T;
            if (kept) { const unsigned key = key_of_bits(e.x); mk = key < mk ? key : mk; }
            hole = !kept && i < target;
        }
        const unsigned long long hm = __ballot(hole);
        if (hm) {
            int base = 0;
            if (lane == 0) base = atomicAdd(&sh.n_holes, __popcll(hm));
            base = __shfl(base, 0, kWave);
            if (hole) holes[base + __popcll(hm & below)] = (uint16_t)i;
        }
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) { const unsigned w = __shfl_xor(mk, o, kWave); mk = w < mk ? w : mk; }
    if (lane == 0) sh.wkey[wave] = mk;
    __syncthreads();
#pragma unroll 4
    for (int j = 0; j < kPer; ++j) {   // survivors behind `target` move into the vacated slots
        const int i = tid + j * kT;
        bool fill = false;
        uint2 e = make_uint2(0, 0);
        if (i >= target && i < n) {
            e = make_uint2(sh.cand_val[i], sh.cand_id[i]);
            fill = composite<BF16>(e) >= T;
        }
        const unsigned long long fm = __ballot(fill);
        if (fm) {
            int base = 0;
            if (lane == 0) base = atomicAdd(&sh.n_fills, __popcll(fm));
            base = __shfl(base, 0, kWave);
            if (fill) { const int h = holes[base + __popcll(fm & below)]; sh.cand_val[h] = e.x; sh.cand_id[h] = e.y; }
        }
    }
    unsigned tk = 0xFFFFFFFFu;
#pragma unroll
    for (int w = 0; w < kW; ++w) { const unsigned a = sh.wkey[w]; tk = a < tk ? a : tk; }
    if (tid == 0) sh.cnt = target;
    __syncthreads();
    return __uint_as_float(bits_of_key(tk));
}

// Descending bitonic sort of P (power of two) uint64 values in LDS.
__device__ __forceinline__ void bitonic_sort_desc(uint64_t* a, int P) {
    for (int size = 2; size <= P; size <<= 1)
        for (int stride = size >> 1; stride > 0; stride >>= 1) {
            __syncthreads();
            for (int t = threadIdx.x; t < (P >> 1); t += kT) {
                const int i = 2 * t - (t & (stride - 1)), j = i + stride;
                const bool desc = (i & size) == 0;
                const uint64_t x = a[i], y = a[j];
                if ((x < y) == desc) { a[i] = y; a[j] = x; }
            }
        }
    __syncthreads();
}

// Order the n <= kMaxK candidates at the front of sh.cand by composite, descending; every
// candidate's short key lies in [key_lo, key_hi].  Returns the LDS array holding the sorted
// composites.  Histogram rank sort: one pass bins the composites (11 bits below the highest bit of
// the range), a prefix sum places the bins, and each element's place inside its bin is the number
// of larger bin-mates.
template <bool BF16>
__device__ __forceinline__ const uint64_t* sort_candidates(CompressShared& sh, int n, uint32_t key_lo, uint32_t key_hi) {
    const int tid = threadIdx.x;
    uint64_t* out = reinterpret_cast<uint64_t*>(sh.cand_val);
    uint64_t* tmp = out + kMaxK;
    const uint64_t lo = (uint64_t)key_lo << kIdBits;
    const uint64_t range = (((uint64_t)key_hi << kIdBits) | kIdMask) - lo;
    const int nb = 64 - __clzll((long long)range);
    const int shift = nb > kBinsLog2 ? nb - kBinsLog2 : 0;
#pragma unroll
    for (int j = 0; j < kBinsPer; ++j) sh.hist[tid + j * kT] = 0;
    if (tid == 0) sh.maxbin = 0;
    __syncthreads();
    uint64_t c[kSortPer];
    int rbin[kSortPer], arrival[kSortPer];
#pragma unroll
    for (int j = 0; j < kSortPer; ++j) {
        const int i = tid + j * kT;
        c[j] = 0; rbin[j] = 0; arrival[j] = 0;
        if (i < n) {
            c[j] = composite<BF16>(make_uint2(sh.cand_val[i], sh.cand_id[i]));
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
    if (sh.maxbin > kSortMaxBin) {   // degenerate spread (e.g. one outlier stretching the range): plain network
        int P = 1;
        while (P < n) P <<= 1;
        for (int i = tid; i < P; i += kT) tmp[i] = 0;
        __syncthreads();
#pragma unroll
        for (int j = 0; j < kSortPer; ++j) { const int i = tid + j * kT; if (i < n) tmp[i] = c[j]; }
        bitonic_sort_desc(tmp, P);
        return tmp;
    }
#pragma unroll
    for (int j = 0; j < kSortPer; ++j) {
        const int i = tid + j * kT;
        if (i < n) tmp[(int)sh.hist[rbin[j]] + arrival[j]] = c[j];
    }
    __syncthreads();   // all candidates are in registers and in tmp: their old slots may be overwritten
#pragma unroll
    for (int j = 0; j < kSortPer; ++j) {
        const int i = tid + j * kT;
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

// Rank r of tile 0 (m elements of a row of V) whose value is expected to have about
// k + z*sqrt(k) + z^2 row elements at or above it, z = 4.5; 0 if the optimistic mode does not pay.
__device__ __forceinline__ int optimistic_rank(int k, int V, int m) {
    const float r0 = (float)k * (float)m / (float)V;                  // expected rank of the row's k-th value in the tile
    const float r = r0 + 4.5f * sqrtf(r0) + 20.25f;
    const float expected = r * (float)V / (float)m;                   // candidates at the end of the row
    if (r >= (float)k || expected > 0.8f * (float)kCap) return 0;
    return (int)ceilf(r);
}

template <bool BF16, int NV>
__global__ __launch_bounds__(kT, 4) void compress_kernel(
    const void* __restrict__ logits, int64_t ld, int V, float inv_T, int k, float top_p,
    int32_t* __restrict__ idx, float* __restrict__ prob, int32_t* __restrict__ count,
    float* __restrict__ mass, float* __restrict__ lse)
{
    extern __shared__ __align__(16) unsigned char smem_raw[];
    CompressShared& sh = *reinterpret_cast<CompressShared*>(smem_raw);
    constexpr int N = Vec<BF16>::N, E = NV * N, TILE = kT * E;
    static_assert(TILE <= kCap, "tile 0 is copied whole into the candidate buffer");
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
    const int64_t row = blockIdx.x;
    const RowView rv = row_view<BF16>(logits, ld, row, V);
    const int n_tiles = (rv.L + TILE - 1) / TILE;
    const float c = 1.4426950408889634f * inv_T;

    uint4 cur[NV], nxt[NV];
    const int nq = (rv.L + N - 1) / N;           // 16-byte vectors that overlap the row
    auto load_tile = [&](int it, uint4 (&dst)[NV]) {
        // vectors behind the row's last one re-read that last vector (always a valid address); unpack_tile masks them
#pragma unroll
        for (int j = 0; j < NV; ++j) dst[j] = rv.base[min(it * (kT * NV) + j * kT + tid, nq - 1)];
    };
    // unpack a tile; elements outside the row (alignment prologue, tail) become -inf
    auto unpack_tile = [&](int it, const uint4 (&src)[NV], float (&v)[E]) {
#pragma unroll
        for (int j = 0; j < NV; ++j) {
            float t[N];
            unpack<BF16>(src[j], t);
#pragma unroll
            for (int e = 0; e < N; ++e) v[j * N + e] = t[e];
        }
        if (it == 0 || it + 1 == n_tiles) {
            unsigned vm = 0;
#pragma unroll
            for (int j = 0; j < NV; ++j) vm |= vec_valid_mask<BF16>(rv, it * (kT * NV) + j * kT + tid) << (j * N);
#pragma unroll
            for (int e = 0; e < E; ++e) v[e] = (vm >> e) & 1u ? v[e] : kNegInf;
        }
    };

    const int n0 = min(V, TILE - rv.o);          // row elements in tile 0
    const int r_opt = n_tiles > 1 ? optimistic_rank(k, V, n0) : 0;
    OnlineSum os;
    float M = kNegInf;
    double S = 0.0;
    uint32_t key_lo = 0, key_hi = 0;

    for (int attempt = 0; attempt < 2; ++attempt) {
        const bool optimistic = attempt == 0 && r_opt > 0;
        if (tid == 0) {
            sh.cnt = n0;
            for (int e = 0; e < 3; ++e) { sh.epoch_overflow[e] = 0; sh.epoch_valid[e] = 0x7FFFFFFF; }
        }
        os = OnlineSum();
        int epoch = 0;
        load_tile(0, cur);
        if (n_tiles > 1) load_tile(1, nxt);

        // ---- tile 0: statistics, whole tile into the buffer, first cut
        float tau_adm = kNegInf;                 // later elements are admitted iff > tau_adm
        {
            float v[E];
            unpack_tile(0, cur, v);
            float bm = v[0], bn = v[0];
#pragma unroll
            for (int e = 1; e < E; ++e) { bm = fmaxf(bm, v[e]); bn = fminf(bn, v[e]); }
            const float mref = os.rebase(bm, c);
            float acc = 0.f;
#pragma unroll
            for (int e = 0; e < E; ++e) acc += exp_stream(v[e], mref, c);
            os.s += acc;
#pragma unroll
            for (int j = 0; j < NV; ++j)
#pragma unroll
                for (int e = 0; e < N; ++e) {
                    const int x = (j * kT + tid) * N + e - rv.o;
                    if (x >= 0 && x < n0) { sh.cand_val[x] = __float_as_uint(v[j * N + e]); sh.cand_id[x] = (unsigned)x; }
                }
            // key range of the tile (masked elements are -inf, which only widens it)
            const float wmax = wave_max(bm), wmin = -wave_max(-bn);
            if (lane == 0) { sh.wkey[wave] = short_key<BF16>(__float_as_uint(wmax)); sh.wkey[kW + wave] = short_key<BF16>(__float_as_uint(wmin)); }
            __syncthreads();
            key_hi = 0; key_lo = 0xFFFFFFFFu;
#pragma unroll
            for (int w = 0; w < kW; ++w) { key_hi = max(key_hi, sh.wkey[w]); key_lo = min(key_lo, sh.wkey[kW + w]); }
            __syncthreads();
            if (n_tiles > 1) {
                const int target = optimistic ? r_opt : k;
                if (n0 > target) {
                    const float tau = prune_to<BF16>(sh, n0, target, key_lo, key_hi, optimistic);
                    tau_adm = optimistic ? float_below(tau) : tau;
                    key_lo = short_key<BF16>(__float_as_uint(tau));
                }
            }
        }

        // ---- tiles 1 .. : admit what beats the threshold
        bool safe = !optimistic;
        for (int it = 1; it < n_tiles; ++it) {
#pragma unroll
            for (int j = 0; j < NV; ++j) cur[j] = nxt[j];
            if (it + 1 < n_tiles) load_tile(it + 1, nxt);
            float v[E];
            unpack_tile(it, cur, v);
            float bm = v[0];
#pragma unroll
            for (int e = 1; e < E; ++e) bm = fmaxf(bm, v[e]);
            const float mref = os.rebase(bm, c);
            float acc = 0.f;
#pragma unroll
            for (int e = 0; e < E; ++e) acc += exp_stream(v[e], mref, c);
            os.s += acc;

            const int x0 = it * TILE - rv.o + tid * N;      // id of this thread's element (j = 0, e = 0)
            bool pending = true;
            for (;;) {
                if (pending) {
                    // one ballot per element column: which lanes hold a candidate there
                    int total = 0;
#pragma unroll
                    for (int e = 0; e < E; ++e) total += __popcll(__ballot(v[e] > tau_adm));
                    if (total > 0) {
                        int base = 0;
                        if (lane == 0) base = atomicAdd(&sh.cnt, total);
                        base = __builtin_amdgcn_readfirstlane(base);
                        if (base + total <= kCap) {
                            int run = base;
                            float tau_keep = tau_adm;
                            asm volatile("" : "+v"(tau_keep));
#pragma unroll
                            for (int j = 0; j < NV; ++j)
#pragma unroll
                                for (int e = 0; e < N; ++e) {
                                    // the lane masks are formed again rather than kept: sixteen of them would not fit the scalar file
                                    const bool pass = v[j * N + e] > tau_keep;
                                    const unsigned long long m = __ballot(pass);
                                    const int pos = (int)__builtin_amdgcn_mbcnt_hi((unsigned)(m >> 32),
                                                        __builtin_amdgcn_mbcnt_lo((unsigned)m, (unsigned)run));
                                    if (pass) {
                                        sh.cand_val[pos] = __float_as_uint(v[j * N + e]);
                                        sh.cand_id[pos] = (unsigned)(x0 + j * kT * N + e);
                                    }
                                    run += __popcll(m);
                                }
                            pending = false;
                        } else if (lane == 0) {
                            atomicMin(&sh.epoch_valid[epoch], base);
                            sh.epoch_overflow[epoch] = 1;
                        }
                    } else {
                        pending = false;
                    }
                }
                __syncthreads();
                const int overflow = sh.epoch_overflow[epoch];
                const int n_held = sh.epoch_valid[epoch];
                // the slot two epochs ahead was last read before the barrier above and is next
                // written after the next barrier
                if (tid == 0) { const int e2 = (epoch + 2) % 3; sh.epoch_overflow[e2] = 0; sh.epoch_valid[e2] = 0x7FFFFFFF; }
                epoch = (epoch + 1) % 3;
                if (!overflow) break;
                // the buffer is full: back to the exact top k of everything seen; strict admission from here on
                const float wmax = wave_max(os.m);
                if (lane == 0) sh.wkey[wave] = short_key<BF16>(__float_as_uint(wmax));
                __syncthreads();
#pragma unroll
                for (int w = 0; w < kW; ++w) key_hi = max(key_hi, sh.wkey[w]);
                const float tau = prune_to<BF16>(sh, n_held, k, key_lo, key_hi, false);
                tau_adm = tau;
                key_lo = short_key<BF16>(__float_as_uint(tau));
                safe = true;
            }
        }

        // ---- end of row
        block_softmax_stats<kW>(os.m, os.s, c, sh.red, M, S);
        key_hi = short_key<BF16>(__float_as_uint(M));
        const int n = sh.cnt;
        if (n > k) prune_to<BF16>(sh, n, k, key_lo, key_hi, false);
        if (n >= k || safe) break;               // an optimistic threshold that kept fewer than k: stream again, safely
        __syncthreads();
    }

    // ---- ordering and emission
    const int n = min(sh.cnt, k);
    const uint64_t* sorted = sort_candidates<BF16>(sh, n, key_lo, key_hi);

    const double cd = 1.4426950408889634 * (double)inv_T;
    const double invS = 1.0 / S;
    const bool use_top_p = top_p > 0.f && top_p < 1.f;
    double carry = 0.0, my_mass = 0.0;
    int my_count = 0;
    int32_t* idx_row = idx + row * (int64_t)k;
    float* prob_row = prob + row * (int64_t)k;
    for (int j0 = 0; j0 < k; j0 += kT) {
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
            for (int w = 0; w < kW; ++w) { const double t = sh.red[w]; if (w < wave) before += t; tot += t; }
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
    if (lane == 0) { sh.red[wave] = wm; sh.red[kW + wave] = (double)wc; }
    __syncthreads();
    if (tid == 0) {
        double tm = 0.0, tc = 0.0;
        for (int w = 0; w < kW; ++w) { tm += sh.red[w]; tc += sh.red[kW + w]; }
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
    if (which) hipLaunchKernelGGL(b16, dim3(n_rows), dim3(kT), smem, stream, logits, ld, V, inv_T, k, top_p, idx, prob, count, mass, lse);
    else       hipLaunchKernelGGL(f32, dim3(n_rows), dim3(kT), smem, stream, logits, ld, V, inv_T, k, top_p, idx, prob, count, mass, lse);
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
