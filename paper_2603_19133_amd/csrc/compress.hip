// Sparse Top-K compression of vocabulary distributions (paper Section 3.3, Eq. 4) fused with the
// softmax statistics: one workgroup of 512 threads per row, two workgroups per CU (three with the
// small candidate buffer), one HBM pass per row.  Three kernels per dtype share the code below
// (launch_compress chooses): the general one (optimistic pass, then the safe pass for the rows that
// lose it), the fast ones that hold the optimistic pass only, with the large or the small candidate
// buffer, and mark the rows they give up, and the retry kernel that runs the general code on those.
//
// Streaming selection.  A row is read with buffer loads (descriptor base + scalar offset + one
// constant per-lane offset) in sub-tiles of two 16-byte vectors per thread through a ring of four
// register buffers (three sub-tiles in flight behind the one being processed; one vector and a ring
// of five in the bf16 kernel with the small buffer).
//   * A sample of 8192 elements stays in registers while a histogram over their values (one pass on a
//     linear scale, else two radix passes over the order-preserving keys) finds a threshold: a value
//     with at least r of the sample's elements at or above it.
//   * Optimistic pass: the sample is 256 runs of 128 bytes spread evenly over the row (logits trend with
//     the vocabulary id, so the head of a row would misplace the threshold); it is only looked at.  r is
//     chosen (optimistic_rank, kernels.hpp) so that the row is expected to hold k plus a safety margin at or above the
//     threshold.  The row is then streamed from its start: every element at or above the threshold
//     claims a slot of the candidate buffer in LDS with an atomic of its own and writes (value, id)
//     there; the softmax arithmetic sits between claim and write, and runs against a reference exponent
//     fixed from the sample (no running maximum: the row's maximum is its largest candidate).  If the row ends with at least k
//     candidates that fit the buffer, the exact top k is among them, because nothing at or above the
//     threshold was dropped.  Waves run free in this pass; too many or too few candidates give the
//     pass up.
//   * Safe pass (only after a failed optimistic pass, or when the optimistic rank would not pay):
//     the sample is the row's first 8192 elements, which are kept as candidates, and r = k, so the
//     threshold is at or below the k-th largest of the sample.  The waves meet after
//     every sub-tile; when the buffer is full it is pruned to the exact top k of everything seen,
//     and from then on an element of a later sub-tile must be strictly larger than the k-th (rows
//     are streamed in ascending id, so equal logits that come later lose the tie; the waves of the
//     sub-tile in which the prune happened append in any order and are admitted from the k-th on).
//   * Vocabulary masks: -inf entries stay out of the optimistic pass's value range; when the sample
//     shows fewer entries above -inf than the rank aimed at, every such entry of the row becomes a
//     candidate, and a record they do not fill goes on with masked ids in ascending order.
//   * The candidates are cut to exactly k and ordered in one step by a histogram rank sort on the
//     composite
//         (key << 20) | (2^20 - 1 - id)
//     (larger logit first, lower id first among equal logits), their probabilities formed from the
//     row's (max, sum), and the record written once.  The cut of a mid-row prune is a radix select
//     on the key, ties at the k-th key cut by a radix select on the id.
#include <type_traits>

#include "common.hpp"
#include "kernels.hpp"
#include "rowspan.hpp"

namespace picospec {

namespace {

constexpr int kT = kCompressThreads;        // threads per workgroup
constexpr int kW = kT / kWave;
constexpr int kRetryRow = -2;               // count of a row that the small variant leaves to the general kernel
constexpr int kCapBig = 8192;               // candidate slots in LDS (value + id, 8 bytes): records of up to kMaxK entries
constexpr int kCapSmall = 5120;             // ... and the variant for records of up to kMaxK / 2: three workgroups per CU
constexpr int kBinsLog2 = 11;
constexpr int kBins = 1 << kBinsLog2;       // histogram bins of the radix selects / rank sort
constexpr int kBinsPer = kBins / kT;
constexpr int kFine = 2 * kBins;            // fine bins of the rank sort: 16-bit counters, two to a histogram word
constexpr int kIdBits = 20;                 // ids < 2^20 (kMaxV)
constexpr unsigned kIdMask = (1u << kIdBits) - 1u;
constexpr int kSortMaxBin = 128;            // beyond this bin size the ordering falls back to a sorting network
constexpr int kCoarseLog2 = 9;
constexpr int kCoarse = 1 << kCoarseLog2;   // coarse ranges that steer the fine bins of the rank sort

static_assert(kMaxK <= kCapBig && (kMaxK & (kMaxK - 1)) == 0, "the sorting network pads to a power of two inside the buffer");
static_assert(kFine <= 32768, "bin and arrival order of a candidate share one register");
static_assert(kMaxV <= (1 << kIdBits), "id field of the composite key");

template <int CAP>
struct __align__(16) CompressShared {
    static constexpr int kCap = CAP;        // candidate slots
    static constexpr int kRecMax = CAP >= 2 * kMaxK ? kMaxK : kMaxK / 2;   // longest record this buffer serves
    static_assert(CAP % (2 * kT) == 0 && CAP < 65536, "whole slots per thread; a prune keeps a 16-bit index list");
    static_assert(kRecMax <= kBins * 2 && kRecMax <= CAP, "a prune's 16-bit index list (one entry per kept slot) lives in the histogram");
    unsigned cand_val[CAP];                 // candidates: fp32 bit pattern ...
    unsigned cand_id[CAP];                  // ... and vocabulary id (the sort reuses both arrays as uint64 regions)
    unsigned hist[kBins];
    unsigned coarse[kCoarse];               // rank sort: count, then (fine bins << 16) | first fine bin, per coarse range
    double red[2 * kW];
    int wtot[kW];
    unsigned wkey[3 * kW];                  // per wave: largest key, smallest key, "saw a masked entry" (sample of the optimistic pass)
    int cnt;                                // candidates held
    int n_holes, n_fills;                   // compaction of a prune
    int piv_bin, piv_before, piv_count;     // radix-select broadcast
    int maxbin;
    int overflowed;                         // a reservation of the sample did not fit (cannot happen: kept as a guard)
    int epoch_overflow[3];                  // safe pass, per attempt epoch: some wave did not fit
    int epoch_valid[3];                     // safe pass, per attempt epoch: first reservation that did not fit
};

static_assert(sizeof(CompressShared<kCapBig>) <= 80 * 1024, "two workgroups share the 160 KB of LDS of a gfx950 CU");
static_assert(sizeof(CompressShared<kCapSmall>) <= 160 * 1024 / 3, "three workgroups of the small variant share a CU's LDS");

template <bool BF16>
__device__ __forceinline__ uint32_t short_key(uint32_t bits) {
    uint32_t key = key_of_bits(bits);
    if constexpr (BF16) key >>= 16;          // the low half of a widened bf16 key carries nothing
    return key;
}

template <bool BF16>
__device__ __forceinline__ uint32_t bits_of_short_key(uint32_t key) {
    if constexpr (BF16) key = (key << 16) | ((key & 0x8000u) ? 0u : 0xFFFFu);   // keys of negative values end in ones
    return bits_of_key(key);
}

// Composite key; for bf16 rows the key field is 16 bits wide so that no dead bits sit between
// the logit and the id.
template <bool BF16>
__device__ __forceinline__ uint64_t composite(uint32_t bits, uint32_t id) {
    return ((uint64_t)short_key<BF16>(bits) << kIdBits) | (uint64_t)(kIdMask - id);
}

template <class SH>
__device__ __forceinline__ void zero_hist(SH& sh) {
#pragma unroll
    for (int j = 0; j < kBinsPer; ++j) sh.hist[threadIdx.x + j * kT] = 0;
}

// Scan the kBins counters in sh.hist (each thread owning kBinsPer consecutive bins) and find the
// bin in which the running count first reaches `need`.  Broadcasts its index, the count in front of
// it and its own count through sh.piv_*; read them after the call.  Returns the total count.  A histogram
// that holds fewer than `need` has no such bin: the last bin is reported then, with the count 0.
template <class SH>
__device__ __forceinline__ int find_pivot_bin(SH& sh, int need) {
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
    int h[kBinsPer], loc = 0;
#pragma unroll
    for (int j = 0; j < kBinsPer; ++j) { h[j] = (int)sh.hist[tid * kBinsPer + j]; loc += h[j]; }
    const int incl = wave_scan_incl(loc);
    if (lane == kWave - 1) sh.wtot[wave] = incl;
    if (tid == 0) { sh.piv_bin = kBins - 1; sh.piv_before = 0; sh.piv_count = 0; }   // (the owner below writes after the barrier)
    __syncthreads();
    int before = 0, total = 0;
#pragma unroll
    for (int w = 0; w < kW; ++w) { before += (w < wave) ? sh.wtot[w] : 0; total += sh.wtot[w]; }
    const int excl = before + incl - loc;
    if (excl < need && need <= excl + loc) {   // exactly one thread owns the pivot bin
        int a = excl, j = 0;
        while (a + h[j] < need) { a += h[j]; ++j; }
        sh.piv_bin = tid * kBinsPer + j;
        sh.piv_before = a;
        sh.piv_count = h[j];
    }
    __syncthreads();
    return total;
}

// What a prune keeps: key > K, or key == K and id <= I.
struct KeepRule {
    uint32_t K, I;
    __device__ __forceinline__ bool keeps(uint32_t key, uint32_t id) const { return key > K || (key == K && id <= I); }
};

// Exact cut: the rule that keeps exactly `need` of the n > need candidates in LDS, largest keys
// first, lower ids first among equal keys.  Every candidate's short key lies in [key_lo, key_hi].
// Radix select on the key, 11 bits per pass below the highest bit of the range; if the pivot key
// is shared by more candidates than are still needed, a radix select on the id cuts the tie.
template <bool BF16, class SH>
__device__ __forceinline__ KeepRule select_exact(SH& sh, int n, int need, uint32_t key_lo, uint32_t key_hi) {
    const int tid = threadIdx.x;
    uint32_t lo = key_lo;
    const uint32_t range = key_hi - key_lo;
    const int nb = range ? 32 - __clz((int)range) : 1;
    int shift = nb > kBinsLog2 ? nb - kBinsLog2 : 0;
    int wbits = 31;   // undecided candidates have key - lo < 2^(wbits+1); keys below lo wrap far above
    bool first = true;
    for (;;) {
        zero_hist(sh);
        __syncthreads();
        for (int i = tid; i < n; i += kT) {
            const uint32_t d = short_key<BF16>(sh.cand_val[i]) - lo;
            if (first || (d >> wbits) == 0) atomicAdd(&sh.hist[kBins - 1 - (int)min(d >> shift, (uint32_t)(kBins - 1))], 1u);   // reversed: descending
        }
        __syncthreads();
        find_pivot_bin(sh, need);
        const int bin = kBins - 1 - sh.piv_bin;
        need -= sh.piv_before;
        const int bcount = sh.piv_count;
        lo += (uint32_t)bin << shift;
        if (need == bcount) return KeepRule{lo, 0xFFFFFFFFu};   // the whole pivot bin is kept: key >= lo
        if (shift == 0) break;                                   // lo is the pivot key, shared by bcount > need candidates
        first = false;
        wbits = shift;
        shift = shift > kBinsLog2 ? shift - kBinsLog2 : 0;
    }
    // tie on the pivot key: keep the `need` lowest ids among its holders (ids < 2^20: 11 + 9 bits)
    uint32_t id_lo = 0;
    for (int pass = 0; pass < 2; ++pass) {
        const int sh_bits = pass == 0 ? kIdBits - kBinsLog2 : 0;
        zero_hist(sh);
        __syncthreads();
        for (int i = tid; i < n; i += kT) {
            if (short_key<BF16>(sh.cand_val[i]) == lo) {
                const uint32_t d = sh.cand_id[i] - id_lo;
                if (pass == 0 || d < (1u << (kIdBits - kBinsLog2))) atomicAdd(&sh.hist[min(d >> sh_bits, (uint32_t)(kBins - 1))], 1u);
            }
        }
        __syncthreads();
        find_pivot_bin(sh, need);
        need -= sh.piv_before;
        id_lo += (uint32_t)sh.piv_bin << sh_bits;
        if (pass == 0 && need == sh.piv_count) return KeepRule{lo, id_lo + (1u << sh_bits) - 1u};   // the whole id bin
    }
    return KeepRule{lo, id_lo};
}

// Reduce the n > k candidates to exactly the k that `select_exact` keeps, compacted to the front in
// any order: survivors already in the first k slots stay, the others fill the slots vacated there.
// Returns a logit not above the smallest kept one (the new admission threshold).
template <bool BF16, class SH>
__device__ __forceinline__ float prune_to_k(SH& sh, int n, int k, uint32_t key_lo, uint32_t key_hi) {
    const int tid = threadIdx.x, lane = tid & (kWave - 1);
    const KeepRule rule = select_exact<BF16>(sh, n, k, key_lo, key_hi);
    uint16_t* holes = reinterpret_cast<uint16_t*>(sh.hist);   // the histogram is free now
    if (tid == 0) { sh.n_holes = 0; sh.n_fills = 0; }
    __syncthreads();
    const unsigned long long below = (1ull << lane) - 1ull;
    for (int i0 = 0; i0 < k; i0 += kT) {   // list the vacated slots among the first k
        const int i = i0 + tid;
        const bool hole = i < k && !rule.keeps(short_key<BF16>(sh.cand_val[i]), sh.cand_id[i]);
        const unsigned long long hm = __ballot(hole);
        if (hm) {
            int base = 0;
            if (lane == 0) base = atomicAdd(&sh.n_holes, __popcll(hm));
            base = __builtin_amdgcn_readfirstlane(base);
            if (hole) holes[base + __popcll(hm & below)] = (uint16_t)i;
        }
    }
    __syncthreads();
    for (int i0 = k; i0 < n; i0 += kT) {   // survivors behind k move into the vacated slots
        const int i = i0 + tid;
        unsigned val = 0, id = 0;
        bool fill = false;
        if (i < n) {
            val = sh.cand_val[i];
            id = sh.cand_id[i];
            fill = rule.keeps(short_key<BF16>(val), id);
        }
        const unsigned long long fm = __ballot(fill);
        if (fm) {
            int base = 0;
            if (lane == 0) base = atomicAdd(&sh.n_fills, __popcll(fm));
            base = __builtin_amdgcn_readfirstlane(base);
            if (fill) { const int h = holes[base + __popcll(fm & below)]; sh.cand_val[h] = val; sh.cand_id[h] = id; }
        }
    }
    if (tid == 0) sh.cnt = k;
    __syncthreads();
    return __uint_as_float(bits_of_short_key<BF16>(rule.K));
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

// Clears what order_top_k counts in; a barrier must lie between this and the call.
template <class SH>
__device__ __forceinline__ void order_prepare(SH& sh, int n) {
    int t = threadIdx.x;
    asm volatile("" : "+v"(t));                  // (the address is formed here, not held in a register from the top of the kernel)
    for (int i = t; i < kCoarse; i += kT) sh.coarse[i] = 0;
    zero_hist(sh);
    if (threadIdx.x == 0) { sh.maxbin = 0; sh.piv_bin = kFine - 1; sh.piv_before = n; }
}

// Cut the n <= kCap candidates in the buffer to the min(n, k) largest by composite and order them,
// descending; every candidate's short key lies in [key_lo, key_hi].  Returns the LDS array that
// holds the ordered composites.  A histogram rank sort does both jobs, on candidates held in
// registers from here on.
//   * A candidate's place p = ((key_hi - key) << ib) | (leading ib bits of its id) is a 32-bit
//     integer that never decreases along the wanted order (larger logit first, lower id first);
//     ib is as many id bits as fit next to the key range (all of them for rows with few distinct
//     logits, so that equal logits spread over the bins by id).
//   * A coarse histogram of p (kCoarse equal ranges) measures where the candidates lie; each
//     coarse range then gets a share of the kFine fine bins in proportion to its count, so that
//     fine bins hold one or two candidates each whatever the distribution of the logits.
//   * A prefix sum over the fine bins finds the bin in which the k-th largest falls; the
//     candidates of the bins up to that one are gathered bin by bin, each one's position inside
//     its bin is the number of larger bin-mates, and the positions below k are kept.
// A bin too crowded for that sends the row through the radix select and a sorting network.
template <bool BF16, class SH>
__device__ __forceinline__ const uint64_t* order_top_k(SH& sh, int n, int k, int V, uint32_t key_lo, uint32_t key_hi) {
    constexpr int kCap = SH::kCap, kCandPer = kCap / kT, kSortPer = SH::kRecMax / kT;
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
    uint64_t* buf = reinterpret_cast<uint64_t*>(sh.cand_val);   // cand_val and cand_id, back to back
    const uint32_t kr = key_hi - key_lo;
    const int kb = kr ? 32 - __clz((int)kr) : 0;                 // bits of the key range
    const int vb = V > 1 ? 32 - __clz(V - 1) : 0;                // bits of an id
    const int ib = min(32 - kb, vb);                             // id bits that take part
    const int id_drop = vb - ib;
    // The coarse ranges tile the places that occur, [0, (kr + 1) << ib), exactly: range = floor(p * kCoarse / that),
    // as the high word of p times a 0.32 fixed-point factor; the low word is the position inside the range.  (Ranges
    // that tile the next power of two leave up to half of them, and of the fine bins of the range that holds the
    // threshold - the most crowded one - to places that do not occur.)  Few places: one range per place.
    const uint64_t n_places = ((uint64_t)kr + 1u) << ib;           // <= 2^32
    const bool one_each = n_places <= (uint64_t)kCoarse;
    const uint32_t to_range = one_each ? 0u : (uint32_t)(((uint64_t)kCoarse << 32) / n_places);   // < 2^32 as n_places > kCoarse
    auto range_of = [&](uint32_t p) { return one_each ? min(p, (uint32_t)(kCoarse - 1)) : min(__umulhi(p, to_range), (uint32_t)(kCoarse - 1)); };
    auto within_range = [&](uint32_t p) { return one_each ? 0u : p * to_range; };   // position inside the range, as a 0.32 fraction
    static_assert(kCoarse <= kT && kCoarse % kWave == 0 && kCoarse <= kFine / 4 && kFine < 65536, "coarse histogram geometry; (fine bins, first fine bin) share a word");
    static_assert(kCap < 65536, "positions and bin counts are kept in 16 bits");
    // (order_prepare and a barrier behind it have cleared the histograms)
    uint64_t c[kCandPer];
    uint32_t place[kCandPer];
#pragma unroll
    for (int j = 0; j < kCandPer; ++j) {
        const int i = tid + j * kT;
        c[j] = 0; place[j] = 0;
        if (i < n) {
            const uint32_t bits = sh.cand_val[i], id = sh.cand_id[i];
            c[j] = composite<BF16>(bits, id);
            place[j] = ib < 32 ? ((key_hi - short_key<BF16>(bits)) << ib) | (id >> id_drop) : (id >> id_drop);
            atomicAdd(&sh.coarse[range_of(place[j])], 1u);
        }
    }
    __syncthreads();
    // fine bins per coarse range, in proportion to its count (at least one where there is a candidate); one
    // wave builds the table, kCoarse / 64 consecutive ranges per lane
    if (wave == 0) {
        constexpr int kPerLane = kCoarse / kWave;
        constexpr int kShared = kFine - kCoarse - kCoarse / 2;      // leaves room for the "at least one" and for rounding
        const float share = (float)kShared / (float)n;
        unsigned nf[kPerLane], loc = 0;
#pragma unroll
        for (int u = 0; u < kPerLane; ++u) {
            const unsigned cnt = sh.coarse[lane * kPerLane + u];
            nf[u] = cnt ? max(1u, (unsigned)((float)cnt * share)) : 0u;
            loc += nf[u];
        }
        unsigned first = wave_scan_incl(loc) - loc;                 // first fine bin of this lane's ranges
#pragma unroll
        for (int u = 0; u < kPerLane; ++u) { sh.coarse[lane * kPerLane + u] = (nf[u] << 16) | first; first += nf[u]; }
    }
    __syncthreads();
    int meta[kCandPer];                      // (fine bin << 16) | arrival order within the bin; -1: no candidate
#pragma unroll
    for (int j = 0; j < kCandPer; ++j) {
        const int i = tid + j * kT;
        meta[j] = -1;
        if (i < n) {
            const unsigned t = sh.coarse[range_of(place[j])];
            const uint32_t frac = within_range(place[j]);
            const int bin = (int)(t & 0xFFFFu) + (int)__umulhi(frac, t >> 16);
            // (bin 2w in the low half of word w, bin 2w+1 in the high half: a bin holds fewer than 2^16 candidates, so
            //  the low half never carries into the high one)
            const int half = (bin & 1) * 16;
            meta[j] = (bin << 16) | (int)((atomicAdd(&sh.hist[bin >> 1], 1u << half) >> half) & 0xFFFFu);
        }
    }
    __syncthreads();
    // exclusive prefix over the bins, in place (16 bits each: at most kCap candidates); the bin that holds the k-th
    // largest; the most crowded bin in front of it
    constexpr int kFinePer = kFine / kT;
    int h[kFinePer], loc = 0;
#pragma unroll
    for (int j = 0; j < kBinsPer; ++j) {
        const unsigned w = sh.hist[tid * kBinsPer + j];
        h[2 * j] = (int)(w & 0xFFFFu); h[2 * j + 1] = (int)(w >> 16);
        loc += h[2 * j] + h[2 * j + 1];
    }
    const int incl = wave_scan_incl(loc);
    if (lane == kWave - 1) sh.wtot[wave] = incl;
    __syncthreads();   // every thread has read its counters
    int excl = incl - loc;
#pragma unroll
    for (int w = 0; w < kW; ++w) excl += (w < wave) ? sh.wtot[w] : 0;
    int big = 0;
    const uint16_t* const start_of = reinterpret_cast<const uint16_t*>(sh.hist);    // first position of a fine bin, below
#pragma unroll
    for (int j = 0; j < kBinsPer; ++j) {
        unsigned w = 0;
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const int b = 2 * j + u;
            w |= (unsigned)excl << (16 * u);
            if (excl < k) {
                big = max(big, h[b]);
                if (excl + h[b] >= k) { sh.piv_bin = tid * kFinePer + b; sh.piv_before = excl + h[b]; }
            }
            excl += h[b];
        }
        sh.hist[tid * kBinsPer + j] = w;
    }
    if (big > kSortMaxBin) atomicMax(&sh.maxbin, big);
    __syncthreads();
    if (sh.maxbin > kSortMaxBin) {
        __syncthreads();                     // (prune_to_k writes the words read above)
        if (n > k) { prune_to_k<BF16>(sh, n, k, key_lo, key_hi); n = k; }
        // the survivors' composites go to registers, then into the buffer padded to a power of two
#pragma unroll
        for (int j = 0; j < kSortPer; ++j) {
            const int i = tid + j * kT;
            c[j] = i < n ? composite<BF16>(sh.cand_val[i], sh.cand_id[i]) : 0;
        }
        int P = 1;
        while (P < n) P <<= 1;
        __syncthreads();
#pragma unroll
        for (int j = 0; j < kSortPer; ++j) { const int i = tid + j * kT; if (i < P) buf[i] = c[j]; }
        bitonic_sort_desc(buf, P);
        return buf;
    }
    const int piv = sh.piv_bin, n_keep = sh.piv_before;
    // gather bin by bin (every candidate is in registers: the buffer may be overwritten)
#pragma unroll
    for (int j = 0; j < kCandPer; ++j)
        if (meta[j] >= 0 && (meta[j] >> 16) <= piv) buf[(int)start_of[meta[j] >> 16] + (meta[j] & 0xFFFF)] = c[j];
    __syncthreads();
    int pos[kCandPer];
#pragma unroll
    for (int j = 0; j < kCandPer; ++j) {
        pos[j] = k;
        if (meta[j] >= 0 && (meta[j] >> 16) <= piv) {
            const int bin = meta[j] >> 16;
            const int s = (int)start_of[bin];
            const int e = bin < piv ? (int)start_of[bin + 1] : n_keep;
            int larger = 0;
            for (int q = s; q < e; q += 4) {         // four bin-mates per round trip to LDS
                uint64_t m[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) m[u] = buf[min(q + u, kCap - 1)];
#pragma unroll
                for (int u = 0; u < 4; ++u) larger += (q + u < e && m[u] > c[j]) ? 1 : 0;
            }
            pos[j] = s + larger;
        }
    }
    __syncthreads();                         // all positions are known before the ordered list overwrites the bins
#pragma unroll
    for (int j = 0; j < kCandPer; ++j) if (pos[j] < k) buf[pos[j]] = c[j];
    __syncthreads();
    return buf;
}

// One row of the compression: the workgroup that runs this writes record `row` of `n_rows`.
// SMALL: records of up to kMaxK / 2 entries on rows whose expected candidates fit the smaller buffer (the host
// decides: launch_compress) - 51 KB of LDS and at most 80 registers, so that three workgroups share a CU.
// FAST: the optimistic pass only (what the careful pass keeps alive across it costs registers, those that the third
// workgroup needs among them): a row whose pass fails, or to which it does not apply, gets count = kRetryRow and
// nothing else, and a second, small launch that runs the general code on the marked rows takes it.
template <bool BF16, bool SMALL, bool FAST = SMALL>
__device__ __forceinline__ void compress_row(
    const int64_t row, const int n_rows,
    const void* __restrict__ logits, int64_t ld, int V, float inv_T, int k, float top_p,
    int32_t* __restrict__ idx, float* __restrict__ prob, int32_t* __restrict__ count,
    float* __restrict__ mass, float* __restrict__ lse,
    const int32_t* __restrict__ seq_off, const int32_t* __restrict__ n_accept, int ahead)
{
    using SH = CompressShared<SMALL ? kCapSmall : kCapBig>;
    constexpr int kCap = SH::kCap, kRecMax = SH::kRecMax, kSortPer = kRecMax / kT;
    extern __shared__ __align__(16) unsigned char smem_raw[];
    SH& sh = *reinterpret_cast<SH*>(smem_raw);
    // A row is streamed in sub-tiles of SV 16-byte vectors per thread.  The sample from which the first
    // threshold is taken has the size of T0 sub-tiles (8192 elements) and is processed in one piece.
    using Geom = CompressGeom<BF16, SMALL>;
    constexpr int N = Vec<BF16>::N;
    constexpr int SAMPLE = kCompressSample;
    constexpr int SV = Geom::SV, ES = SV * N, SUB = kT * ES;
    constexpr int T0 = SAMPLE / SUB, NV0 = T0 * SV, E0 = NV0 * N;
    constexpr int RING = Geom::RING;             // sub-tile buffers: one in use, the others in flight
    static_assert(Geom::N == N, "vector width");
    static_assert(T0 >= 1 && T0 < RING && E0 <= 16 && (FAST || SAMPLE <= kCap), "sample geometry (the careful pass keeps its sample as candidates)");
    const int tid = threadIdx.x, lane = tid & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(tid / kWave);   // uniform: what is indexed by it is addressed from a scalar
    // Row read: the same one, or (downlink record, Section 3.3) the target row of sequence `row` at its
    // first rejected or bonus position, seq_off[b] + b + n_accept[b] (n_accept clamped to 0..gamma_b).
    int64_t in_row = row;
    if (seq_off) {
        const int d0 = seq_off[row], g = max(seq_off[row + 1] - d0, 0);
        in_row = (int64_t)d0 + row + min(max(n_accept[row], 0), g);
    }
    const RowView rv = row_view<BF16>(logits, ld, in_row, V);
    const int n_sub = (rv.L + SUB - 1) / SUB;
    const int nq = (rv.L + N - 1) / N;           // 16-byte vectors that overlap the row
    const float c = 1.4426950408889634f * inv_T;
    const float qnan = __uint_as_float(0x7FC00000u);

    // Row loads go through a buffer descriptor that spans the row's nq vectors: the address is the
    // descriptor's base + a scalar offset (sub-tile, vector group) + this lane's constant offset, so that no
    // vector arithmetic forms it.  On gfx950 a raw buffer load (stride 0) compares scalar offset + lane
    // offset + 16 with the descriptor's size (measured; picospec_check_device() tests it on the device at
    // hand), so vectors behind the row read as zero without touching memory: the look-ahead loads behind
    // the last sub-tile need no guard (rowspan.hpp states the rule; unpack masks the elements anyway).
    const __amdgpu_buffer_rsrc_t row_rsrc = __builtin_amdgcn_make_buffer_rsrc((void*)rv.base, 0, nq * 16, 0x00020000);
    const int lane_off = tid * 16;
    auto load_sub = [&](int sub, uint4 (&dst)[SV]) {
#pragma unroll
        for (int j = 0; j < SV; ++j) {
            const u32x4_t t = __builtin_amdgcn_raw_buffer_load_b128(row_rsrc, lane_off, Geom::group_first(sub, j) * 16, 2 /* non-temporal */);
            dst[j] = make_uint4(t.x, t.y, t.z, t.w);
        }
    };
    // Unpack NVV vectors, vector jj being vector q0 + jj*kT of the row.  With `edge`, elements outside
    // the row (alignment prologue, tail) become NaN, which fails every admission test.
    auto unpack_vecs = [&](auto nvv_tag, int q0, const uint4* src, float* v, bool edge) {
        constexpr int NVV = decltype(nvv_tag)::value;
#pragma unroll
        for (int j = 0; j < NVV; ++j) {
            float t[N];
            unpack<BF16>(src[j], t);
#pragma unroll
            for (int e = 0; e < N; ++e) v[j * N + e] = t[e];
        }
        if (edge) {
            unsigned vm = 0;
#pragma unroll
            for (int j = 0; j < NVV; ++j) vm |= vec_valid_mask<BF16>(rv, q0 + j * kT) << (j * N);
#pragma unroll
            for (int e = 0; e < NVV * N; ++e) v[e] = (vm >> e) & 1u ? v[e] : qnan;
        }
    };
    // The sample that places the optimistic pass's threshold: E0 elements per thread, taken from PIECES runs of
    // 128 bytes spread evenly over the row.  (Logits trend with the vocabulary id - frequent tokens sit at low
    // ids - so the head of a row alone misplaces the threshold and loses the pass.)  The sample is only looked
    // at; its elements are streamed again with the rest of the row, so these loads are ordinary, cached ones.
    constexpr int PIECES = NV0 * (kT / 8);
    // vector of thread tid in run j*(kT/8) + tid/8 of a row of n_vec vectors at `base`: the runs start on 128-byte
    // lines of memory (one line fetched per run), at least 8 vectors apart once n_vec >= 8*PIECES + 8
    auto sample_vec_of = [&](int j, int n_vec, const uint4* base) {
        const int shift = (int)(((uintptr_t)base >> 4) & 7u);
        const int a = ((j * (kT / 8) + (tid >> 3)) * (n_vec - 16)) / (PIECES - 1) + shift;
        return ((a + 7) & ~7) - shift + (tid & 7);
    };
    auto sample_vec = [&](int j) { return sample_vec_of(j, nq, rv.base); };
    auto load_sample = [&](uint4* dst) {
#pragma unroll
        for (int j = 0; j < NV0; ++j) {
            const u32x4_t t = __builtin_amdgcn_raw_buffer_load_b128(row_rsrc, sample_vec(j) * 16, 0, 0);
            dst[j] = make_uint4(t.x, t.y, t.z, t.w);
        }
    };
    auto unpack_sample = [&](const uint4* src, float* v) {      // elements outside the row become NaN
#pragma unroll
        for (int j = 0; j < NV0; ++j) {
            float t[N];
            unpack<BF16>(src[j], t);
            const unsigned vm = vec_valid_mask<BF16>(rv, sample_vec(j));
#pragma unroll
            for (int e = 0; e < N; ++e) v[j * N + e] = (vm >> e) & 1u ? t[e] : qnan;
        }
    };
    // Running softmax sum of this thread: s = sum 2^(v*c - r) with an integer reference exponent
    // r >= c * (largest value seen), so that one fused multiply-add forms each exponent (and a change
    // of reference scales s by an exact power of two); mx = largest value seen.
    struct { float mx, r, s; } os;
    // add EE elements to the running sum; returns this thread's maximum over them
    auto add_stats = [&](auto ee_tag, const float* v, bool edge) {
        constexpr int EE = decltype(ee_tag)::value;
        float bm = kNegInf;
#pragma unroll
        for (int e = 0; e < EE; ++e) bm = fmaxf(bm, v[e]);          // fmaxf skips the NaN of masked elements
        if (bm > os.mx) {
            os.mx = bm;
            const float rn = ceilf(bm * c);
            if (rn > os.r) { os.s *= __builtin_amdgcn_exp2f(os.r - rn); os.r = rn; }   // r = -inf: s is 0 and stays 0
        }
        const float nr = os.r == kNegInf ? 0.f : -os.r;             // rows of only -inf so far
        float acc = 0.f;
        if (edge) {
#pragma unroll
            for (int e = 0; e < EE; ++e) acc += v[e] == v[e] ? __builtin_amdgcn_exp2f(fmaf(v[e], c, nr)) : 0.f;
        } else {
#pragma unroll
            for (int e = 0; e < EE; ++e) acc += __builtin_amdgcn_exp2f(fmaf(v[e], c, nr));
        }
        os.s += acc;
        return bm;
    };
    // The optimistic pass's form: the reference exponent is fixed for the whole row (set from the sample's largest
    // value, the same for every thread), so an element costs its exponent, the exponential and an add, and neither
    // the largest value nor the reference is followed: the row's largest value is the largest candidate, and a row
    // whose values rise so far above the sample's that the sum could overflow gives the pass up at its end.
    auto add_sum = [&](auto ee_tag, const float* v, bool edge, float nr) {
        constexpr int EE = decltype(ee_tag)::value;
        float acc = 0.f;
        if (edge) {
#pragma unroll
            for (int e = 0; e < EE; ++e) acc += v[e] == v[e] ? __builtin_amdgcn_exp2f(fmaf(v[e], c, nr)) : 0.f;
        } else {
#pragma unroll
            for (int e = 0; e < EE; ++e) acc += __builtin_amdgcn_exp2f(fmaf(v[e], c, nr));
        }
        os.s += acc;
    };
    // Safe pass: appending the elements that pass (v > tau, or with ALL every element that is not NaN)
    // by wave-wide reservation, so that a reservation that does not fit writes nothing and can be
    // repeated after a prune.  reserve_vecs counts the wave's candidates (one ballot per element
    // column) and reserves their slots with one LDS atomic; place_vecs forms the lane masks again and
    // writes (value, id).  x0 = id of this thread's first element; vector jj starts kT*N ids after
    // vector jj-1.
    struct Reservation { int total, base; };   // base is valid in lane 0 until place_vecs broadcasts it
    auto reserve_vecs = [&](auto nvv_tag, auto all_tag, const float* v, float tau) {
        constexpr int NVV = decltype(nvv_tag)::value;
        constexpr bool ALL = decltype(all_tag)::value;
        Reservation r{0, 0};
#pragma unroll
        for (int e = 0; e < NVV * N; ++e) r.total += __popcll(__ballot(ALL ? v[e] == v[e] : v[e] > tau));
        if (r.total > 0 && lane == 0) r.base = atomicAdd(&sh.cnt, r.total);
        return r;
    };
    // Returns the first slot of a reservation that does not fit (nothing is written then), else -1.
    auto place_vecs = [&](auto nvv_tag, auto all_tag, const float* v, float tau, int x0, Reservation r) {
        constexpr int NVV = decltype(nvv_tag)::value;
        constexpr bool ALL = decltype(all_tag)::value;
        if (r.total == 0) return -1;
        const int base = __builtin_amdgcn_readfirstlane(r.base);
        if (base + r.total > kCap) return base;
        int run = base;
        float tau2 = tau;
        int xb = x0;
        asm volatile("" : "+v"(tau2), "+v"(xb));   // also keeps the ids from being formed ahead of time
#pragma unroll
        for (int j = 0; j < NVV; ++j)
#pragma unroll
            for (int e = 0; e < N; ++e) {
                const bool pass = ALL ? v[j * N + e] == v[j * N + e] : v[j * N + e] > tau2;
                const unsigned long long m = __ballot(pass);
                if (m) {
                    const int pos = run + (int)__builtin_amdgcn_mbcnt_hi((unsigned)(m >> 32),
                                              __builtin_amdgcn_mbcnt_lo((unsigned)m, 0u));
                    if (pass) {
                        sh.cand_val[pos] = __float_as_uint(v[j * N + e]);
                        sh.cand_id[pos] = (unsigned)(xb + j * kT * N + e);
                    }
                    run += __popcll(m);
                }
            }
        return -1;
    };
    auto append = [&](auto nvv_tag, const float* v, float tau, bool all, int x0) {
        if (all) return place_vecs(nvv_tag, std::true_type{}, v, tau, x0, reserve_vecs(nvv_tag, std::true_type{}, v, tau));
        return place_vecs(nvv_tag, std::false_type{}, v, tau, x0, reserve_vecs(nvv_tag, std::false_type{}, v, tau));
    };
    using sv_t = std::integral_constant<int, SV>;
    using es_t = std::integral_constant<int, ES>;
    using nv0_t = std::integral_constant<int, NV0>;
    using e0_t = std::integral_constant<int, E0>;

    // Optimistic pass: every element above the threshold claims a slot with an LDS atomic of its own (a
    // few lanes per instruction) and later writes (value, id) there.  Both steps are hand-issued so
    // that they stay straight-line code (predication by EXEC, no branches for the compiler to lay
    // out): claim_asm forms the lane mask, claims under it and hands the mask on; put_asm waits for
    // the claimed slots and writes under the same masks.  The counter
    // starts at the LDS address of cand_val and counts bytes (4 per candidate), so that a claimed slot, clamped,
    // is the address to write to; slots behind the buffer's end fall onto its last one: once the count has
    // passed the end the pass is lost anyway.
    typedef __attribute__((address_space(3))) unsigned lds_u32;
    const unsigned cnt_addr = (unsigned)(uintptr_t)(lds_u32*)&sh.cnt;
    const unsigned val_addr = (unsigned)(uintptr_t)(lds_u32*)&sh.cand_val[0];
    unsigned four = 4u, last_slot = val_addr + (unsigned)(kCap * 4 - 4);
    asm volatile("" : "+v"(four), "+v"(last_slot));
    auto claim_asm = [&, four](auto ee_tag, const float* v, float tau, int* slot, unsigned long long* passed) {
        constexpr int EE = decltype(ee_tag)::value;
        unsigned ca = cnt_addr;
        asm volatile("" : "+v"(ca));
#pragma unroll
        for (int e = 0; e < EE; ++e) {
            unsigned long long saved;
            asm volatile("v_cmp_gt_f32_e64 %[m], %[x], %[t]\n\t"
                         "s_and_saveexec_b64 %[sv], %[m]\n\t"
                         "ds_add_rtn_u32 %[slot], %[ca], %[four]\n\t"
                         "s_mov_b64 exec, %[sv]"
                         : [slot] "=&v"(slot[e]), [m] "=&s"(passed[e]), [sv] "=&s"(saved)
                         : [x] "v"(v[e]), [t] "v"(tau), [ca] "v"(ca), [four] "v"(four)
                         : "memory", "scc");
        }
    };
    auto put_asm = [&, last_slot](auto nvv_tag, const float* v, int* slot, const unsigned long long* passed, int x0) {
        constexpr int NVV = decltype(nvv_tag)::value;
        static_assert(NVV * N == 8 || NVV * N == 16, "the wait names every slot");
        // the claimed slots have arrived (the running sum is named so that the statistics stay in front)
        if constexpr (NVV * N == 8)
            asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(slot[0]), "+v"(slot[1]), "+v"(slot[2]), "+v"(slot[3]),
                         "+v"(slot[4]), "+v"(slot[5]), "+v"(slot[6]), "+v"(slot[7]), "+v"(os.s));
        else {
            asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(slot[0]), "+v"(slot[1]), "+v"(slot[2]), "+v"(slot[3]),
                         "+v"(slot[4]), "+v"(slot[5]), "+v"(slot[6]), "+v"(slot[7]), "+v"(os.s));
            asm volatile("" : "+v"(slot[8]), "+v"(slot[9]), "+v"(slot[10]), "+v"(slot[11]),
                         "+v"(slot[12]), "+v"(slot[13]), "+v"(slot[14]), "+v"(slot[15]));
        }
        // eight columns at a time: their addresses and ids first (every lane, back to back), then only the write
        // under each column's mask
        static_assert((NVV * N) % 8 == 0, "writes go in blocks of eight columns");
#pragma unroll
        for (int i0 = 0; i0 < NVV * N; i0 += 8) {
            unsigned at[8], id[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int i = i0 + u;
                                at[u] = min((unsigned)slot[i], last_slot);
                id[u] = (unsigned)(x0 + (i / N) * kT * N + i % N);
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                unsigned long long saved;
                asm volatile("s_and_saveexec_b64 %[sv], %[m]\n\t"
                             "ds_write2st64_b32 %[at], %[x], %[id] offset1:%c[o1]\n\t"
                             "s_mov_b64 exec, %[sv]"
                             : [sv] "=&s"(saved)
                             : [m] "s"(passed[i0 + u]), [at] "v"(at[u]), [id] "v"(id[u]), [x] "v"(v[i0 + u]), [o1] "n"(kCap / 64)
                             : "memory", "scc");
            }
        }
    };
    static_assert(offsetof(SH, cand_id) - offsetof(SH, cand_val) == (kCap / 64) * 64 * 4,
                  "ds_write2st64 offset1 reaches cand_id from cand_val");

    const bool more = n_sub > T0;                // the row goes on behind the sample
    const int r_opt = more ? optimistic_rank(k, V, SAMPLE, kCap) : 0;
    float M = kNegInf;
    double S = 0.0;
    uint32_t key_lo = 0, key_hi = 0;
    int n_held = -1;                             // candidates held at the end of the row (-1: read the counter)
    bool fill = false;                           // fewer entries above -inf than k: masked entries fill the record up

    bool row_done = false;
    static_assert(FAST || !SMALL, "the small buffer cannot hold the careful pass's sample");
    for (int attempt = r_opt > 0 ? 0 : 1; attempt < (FAST ? 1 : 2); ++attempt) {
        const bool optimistic = FAST || attempt == 0;
        if (tid == 0) {
            sh.cnt = optimistic ? (int)val_addr : 0;      // (the optimistic pass's counter is the LDS address of the next slot)
            sh.overflowed = 0;
            for (int e = 0; e < 3; ++e) { sh.epoch_overflow[e] = 0; sh.epoch_valid[e] = 0x7FFFFFFF; }
        }
        os.mx = kNegInf; os.r = kNegInf; os.s = 0.f;
        // Sub-tile buffers.  Optimistic pass: the first T0 take the spread sample, the others the row's first
        // sub-tiles (sub-tile s lives in buffer (T0 + s) % RING).  Safe pass: the row's first T0 sub-tiles are
        // the sample and are kept as candidates.
        uint4 rb[RING][SV];
        if (optimistic) {
            load_sample(&rb[0][0]);
#pragma unroll
            for (int t = T0; t < RING; ++t) load_sub(t - T0, rb[t]);
        } else {
#pragma unroll
            for (int t = 0; t < RING; ++t) load_sub(t, rb[t]);
        }
        const int n0 = optimistic ? SAMPLE : min(V, SAMPLE - rv.o);   // row elements in the sample

        // ---- the sample: the first threshold (and, in the safe pass, the statistics of its elements)
        float tau = kNegInf;                     // elements are admitted iff > tau ...
        bool admit_all = true;                   // ... or, before a threshold exists, all of them
        {
            float v[E0];
            float bm;
            if (optimistic) {
                unpack_sample(&rb[0][0], v);
                bm = kNegInf;
#pragma unroll
                for (int e = 0; e < E0; ++e) bm = fmaxf(bm, v[e]);      // fmaxf skips the NaN of masked elements
            } else {
                unpack_vecs(nv0_t{}, tid, &rb[0][0], v, true);
                bm = add_stats(e0_t{}, v, true);
            }
            // smallest value of the sample; the optimistic pass leaves masked vocabulary entries (-inf) out of it,
            // so that the value range it bins is that of the entries a threshold can fall between
            float bn = __builtin_huge_valf();
            bool saw_masked = false;             // (an element in front of or behind the row counts as one: it only costs a
                                                 //  constant row that is cut at both ends a pass that fails)
#pragma unroll
            for (int e = 0; e < E0; ++e) {
                const bool above = v[e] > kNegInf;
                bn = fminf(bn, (optimistic && !above) ? __builtin_huge_valf() : v[e]);
                saw_masked |= !above;
            }
            // key range of the sample
            const float wmax = wave_max(bm), wmin = -wave_max(-bn);
            const unsigned wave_masked = __ballot(saw_masked) != 0ull;
            if (lane == 0) {
                sh.wkey[wave] = short_key<BF16>(__float_as_uint(wmax));
                sh.wkey[kW + wave] = short_key<BF16>(__float_as_uint(wmin));
                sh.wkey[2 * kW + wave] = wave_masked;
            }
            const int target = optimistic ? r_opt : k;
            const bool one_pass = optimistic && more && n0 > target;
            if (one_pass) zero_hist(sh);         // (for the histogram below: the barrier of the key range serves it too)
            __syncthreads();
            key_hi = 0; key_lo = 0xFFFFFFFFu;
            unsigned masked = 0;
#pragma unroll
            for (int w = 0; w < kW; ++w) { key_hi = max(key_hi, sh.wkey[w]); key_lo = min(key_lo, sh.wkey[kW + w]); masked |= sh.wkey[2 * kW + w]; }
            bool have_tau = false;
            if (one_pass) {
                // Optimistic pass: the threshold only has to be about right (the count at the end of the row
                // decides), so one histogram pass over a linear scale of the sample's value range does: bin
                // 0 holds the largest values.  A crowded pivot bin (a value range stretched by outliers)
                // leaves the job to the exact radix passes below.
                const float vmax = __uint_as_float(bits_of_short_key<BF16>(key_hi));
                const float vmin = __uint_as_float(bits_of_short_key<BF16>(key_lo));
                if (vmax > vmin && vmin > kNegInf && vmax < __builtin_huge_valf()) {
                    const float width = (vmax - vmin) * (1.0f / (float)kBins);
                    const float scale = 1.0f / width;
#pragma unroll
                    for (int e = 0; e < E0; ++e)
                        if (v[e] > kNegInf) atomicAdd(&sh.hist[min((int)((vmax - v[e]) * scale), kBins - 1)], 1u);
                    __syncthreads();
                    const int n_finite = find_pivot_bin(sh, target);
                    if (n_finite < target) {
                        // A row that is mostly masked: fewer entries above -inf than the rank aimed at.  Every one
                        // of them becomes a candidate (there are about n_finite * V / SAMPLE, which fits); should
                        // the row hold fewer than k, masked entries fill the record up in id order at the end.
                        have_tau = true;
                        tau = kNegInf;
                        admit_all = false;
                        key_lo = short_key<BF16>(0xFF800000u);
                    } else if (scale < __builtin_huge_valf() && sh.piv_count <= max(8, target / 4)) {
                        const float t = vmax - ((float)(sh.piv_bin + 1) + 0.01f) * width;   // below every element of the bins up to the pivot
                        if (t > kNegInf) {
                            tau = float_below(t);
                            admit_all = false;
                            have_tau = true;
                            key_lo = short_key<BF16>(__float_as_uint(tau));
                        }
                    }
                    __syncthreads();             // (the histogram and the pivot words are reused below)
                } else if (masked && !(vmax > vmin) && vmax < __builtin_huge_valf()) {
                    // masked entries and at most one value above -inf in the whole sample (a vocabulary mask that
                    // leaves a handful of ids): every entry above -inf becomes a candidate
                    have_tau = true;
                    tau = kNegInf;
                    admit_all = false;
                    key_lo = short_key<BF16>(0xFF800000u);
                    __syncthreads();
                }
            }
            if (!have_tau && more && n0 > target && key_hi > key_lo) {
                // two histogram passes over the keys in registers: a key with >= target elements of the sample at or above it
                uint32_t lo = key_lo;
                const uint32_t range = key_hi - key_lo;
                const int nb = 32 - __clz((int)range);
                int shift = nb > kBinsLog2 ? nb - kBinsLog2 : 0;
                int need = target;
                int wbits = 31;                  // undecided keys have key - lo < 2^(wbits+1) ...
                for (int pass = 0; pass < 2; ++pass) {
                    zero_hist(sh);
                    __syncthreads();
#pragma unroll
                    for (int e = 0; e < E0; ++e) {
                        const uint32_t d = short_key<BF16>(__float_as_uint(v[e])) - lo;   // ... keys below lo wrap far above (masked entries below
                                                                                          //     the optimistic pass's range: left out)
                        if (v[e] == v[e] && d <= range && (pass == 0 || (d >> wbits) == 0)) atomicAdd(&sh.hist[kBins - 1 - (int)(d >> shift)], 1u);
                    }
                    __syncthreads();
                    find_pivot_bin(sh, need);
                    need -= sh.piv_before;
                    lo += (uint32_t)(kBins - 1 - sh.piv_bin) << shift;
                    if (shift == 0) break;
                    wbits = shift;
                    shift = shift > kBinsLog2 ? shift - kBinsLog2 : 0;
                }
                const float t = __uint_as_float(bits_of_short_key<BF16>(lo));   // lower edge of the pivot bin
                if (t > kNegInf) { tau = float_below(t); admit_all = false; key_lo = lo; }
            }
            if (admit_all && more) key_lo = 0;   // later sub-tiles may go below the sample's minimum
            if (!have_tau) __syncthreads();      // (with a one-pass threshold the barrier behind the pivot stands here already)
            if (!optimistic) {
                const int failed_at = append(nv0_t{}, v, tau, admit_all, tid * N - rv.o);
                if (failed_at >= 0 && lane == 0) sh.overflowed = 1;   // cannot happen: the sample fits the empty buffer
            }
        }

        bool enough = true;
        if (optimistic) {
            // ---- the row from its start, optimistic: waves run free; a reservation that does not fit gives the
            //      pass up.  The ring buffers rotate by role (no copies): while one sub-tile is processed
            //      three are in flight; loads behind the row read zero without touching memory (load_sub).
            // a sample without a threshold (rows of -inf), or with +inf in it, leaves the row to the safe pass
            const float sample_max = __uint_as_float(bits_of_short_key<BF16>(key_hi));
            const bool applies = !admit_all && sample_max < __builtin_huge_valf();
            os.r = sample_max > kNegInf ? ceilf(sample_max * c) : 0.f;      // (the reference exponent of add_sum)
            float nr = -os.r;
            asm volatile("" : "+v"(nr));
            if (applies) {
#pragma unroll
                for (int t = 0; t < T0; ++t) load_sub(RING - T0 + t, rb[t]);
                auto full = [&](int sub, uint4 (&buf)[SV]) {        // a sub-tile wholly inside the row
                    float v[ES];
                    int slot[ES];
                    unsigned long long passed[ES];
                    unpack_vecs(sv_t{}, 0, buf, v, false);
                    claim_asm(es_t{}, v, tau, slot, passed);
                    add_sum(es_t{}, v, false, nr);
                    put_asm(sv_t{}, v, slot, passed, sub * SUB - rv.o + tid * N);
                    load_sub(sub + RING, buf);
                };
                auto ragged = [&](int sub, uint4 (&buf)[SV]) {      // the last sub-tiles: what lies behind the row is masked
                    if (sub < n_sub) {
                        float v[ES];
                        int slot[ES];
                        unsigned long long passed[ES];
                        const bool edge = sub + 1 == n_sub;
                        unpack_vecs(sv_t{}, sub * (kT * SV) + tid, buf, v, edge);
                        claim_asm(es_t{}, v, tau, slot, passed);
                        add_sum(es_t{}, v, edge, nr);
                        put_asm(sv_t{}, v, slot, passed, sub * SUB - rv.o + tid * N);
                    }
                };
                {   // sub-tile 0 may begin in front of the row (rows off the 16-byte boundary): masked like an edge
                    float v[ES];
                    int slot[ES];
                    unsigned long long passed[ES];
                    unpack_vecs(sv_t{}, tid, rb[T0], v, true);
                    claim_asm(es_t{}, v, tau, slot, passed);
                    add_sum(es_t{}, v, true, nr);
                    put_asm(sv_t{}, v, slot, passed, tid * N - rv.o);
                    load_sub(RING, rb[T0]);
                }
                // the hot loop holds nothing but the common case, RING times (one copy per buffer role)
                int sub = 1;
                for (; sub + RING < n_sub; sub += RING) {
#pragma unroll
                    for (int r = 0; r < RING; ++r) full(sub + r, rb[(T0 + 1 + r) % RING]);
                }
#pragma unroll
                for (int r = 0; r < RING; ++r) ragged(sub + r, rb[(T0 + 1 + r) % RING]);
            }
            __syncthreads();
            const int held = (int)((unsigned)sh.cnt - val_addr) >> 2;   // (this pass's counter is an LDS byte address)
            // (a threshold of -inf: every entry above -inf is held, so fewer than k of them are still the whole answer)
            enough = applies && !sh.overflowed && held <= kCap && (held >= k || (tau == kNegInf && held >= 1));
            n_held = enough ? held : -1;
            fill = enough && held < k;
            // the row's largest value is its largest candidate (slots behind the last one hold stale values)
            float cm = kNegInf;
            if (enough) {
#pragma unroll
                for (int j = 0; j < kCap / kT; ++j) {
                    const float x = __uint_as_float(sh.cand_val[tid + j * kT]);
                    cm = tid + j * kT < held ? fmaxf(cm, x) : cm;
                }
            }
            os.mx = cm;
            __syncthreads();                     // everyone has read the verdict before the next attempt resets it
        } else {
            // ---- behind the sample, safe: all waves meet after every sub-tile; a full buffer is pruned back to
            //      the exact top k of everything seen, after which admission is strict for the sub-tiles that follow.
            //      (Rare path: no prefetch.)
            int epoch = 0;
            __syncthreads();
            for (int sub = T0; sub < n_sub; ++sub) {
                uint4 cur[SV];
                load_sub(sub, cur);
                float v[ES];
                const bool edge = sub + 1 == n_sub;
                unpack_vecs(sv_t{}, sub * (kT * SV) + tid, cur, v, edge);
                add_stats(es_t{}, v, edge);
                const int x0 = sub * SUB - rv.o + tid * N;
                bool pending = true;
                // Admission is strict (v > tau) against what earlier sub-tiles left in the buffer: an equal value that
                // comes later has the higher id and loses the tie.  Inside a sub-tile the waves append in any order, so
                // after a prune in mid sub-tile the waves still waiting may hold values equal to the k-th with LOWER ids
                // than entries the prune kept: they are admitted from the k-th value on (the next prune sorts it out).
                float tau_sub = tau;
                bool all_sub = admit_all;
                for (;;) {
                    if (pending) {
                        const int failed_at = append(sv_t{}, v, tau_sub, all_sub, x0);
                        pending = failed_at >= 0;
                        if (pending && lane == 0) {
                            atomicMin(&sh.epoch_valid[epoch], failed_at);
                            sh.epoch_overflow[epoch] = 1;
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
                    const float wmax = wave_max(os.mx);
                    if (lane == 0) sh.wkey[wave] = short_key<BF16>(__float_as_uint(wmax));
                    __syncthreads();
#pragma unroll
                    for (int w = 0; w < kW; ++w) key_hi = max(key_hi, sh.wkey[w]);
                    tau = prune_to_k<BF16>(sh, n_held, k, key_lo, key_hi);
                    admit_all = false;
                    key_lo = short_key<BF16>(__float_as_uint(tau));
                    tau_sub = float_below(tau);
                    all_sub = tau == kNegInf;    // (the k-th is a masked entry: the waiting waves' masked entries count too)
                }
            }
        }
        if (!enough) continue;                   // optimistic threshold too high, or buffer full: stream again, safely

        // ---- end of row
        if (n_held < 0) n_held = sh.cnt;
        order_prepare(sh, n_held);               // (the barriers of the combine below stand behind it)
        {   // M = max over the threads; S = sum s * 2^(r - M*c), combined in fp64
            const float wm = wave_max(os.mx);
            if (lane == 0) sh.red[wave] = (double)wm;
            __syncthreads();
            M = kNegInf;
#pragma unroll
            for (int w = 0; w < kW; ++w) M = fmaxf(M, (float)sh.red[w]);
            // (optimistic pass: values so far above the sample's that the sums may have overflowed; the same for every thread)
            if (optimistic && !(M * c - os.r < 100.f)) { enough = false; n_held = -1; fill = false; }
            const double mine = os.r == kNegInf ? 0.0 : (double)os.s * exp2_split((double)os.r - (double)M * (double)c);
            const double ws = wave_sum(mine);
            if (lane == 0) sh.red[kW + wave] = ws;
            __syncthreads();
            S = 0.0;
#pragma unroll
            for (int w = 0; w < kW; ++w) S += sh.red[kW + w];
            if (tid == kT - 1) {                 // (off the last wave's critical path later on)
                float it = inv_T;
                asm volatile("" : "+s"(it));     // widened here: hoisted to the top of the kernel it would hold two registers throughout
                lse[row] = (float)((double)M * (double)it + log(S));     // (rewritten by the pass that follows a pass given up here)
            }
        }
        if (!enough) continue;
        key_hi = short_key<BF16>(__float_as_uint(M));
        row_done = true;
        break;
    }
    if (FAST && !row_done) {                     // (uniform: the verdict was read from LDS behind a barrier)
        if (tid == 0) count[row] = kRetryRow;
        return;
    }

    // ---- While this row is ordered and emitted, the first sub-tiles of the row that will take a slot like
    //      this one next (`ahead` rows further: as many rows as the chip holds at a time, same XCD) are pulled
    //      into the caches with ordinary loads whose data is dropped, so that row does not start by waiting
    //      for HBM: what its first loads will ask for, i.e. its spread sample (if it takes the optimistic pass)
    //      and the sub-tiles behind it.  One register quadruple takes all of them (tied operand: loads return in order).
    u32x4_t dropped = {0u, 0u, 0u, 0u};
    if (ahead > 0 && row + ahead < (int64_t)n_rows) {
        const RowView nv = row_view<BF16>(logits, ld, row + ahead, V);
        const int nq2 = (nv.L + N - 1) / N;
        const int n_spread = (r_opt > 0 && nq2 >= 8 * PIECES + 8) ? NV0 : 0;
#pragma unroll
        for (int j = 0; j < RING * SV; ++j) {
            const int q = j < n_spread ? sample_vec_of(j, nq2, nv.base) : (j - n_spread) * kT + tid;
            const uint4* p = nv.base + min(q, nq2 - 1);
            asm volatile("global_load_dwordx4 %0, %1, off" : "+v"(dropped) : "v"(p));
        }
    }

    // ---- exact cut to k, ordering and emission
    const int n = min(n_held, k);
    const uint64_t* sorted = order_top_k<BF16>(sh, n_held, n, V, key_lo, key_hi);

    // A mostly masked row with fewer entries above -inf than k (all of them are held): the record goes on with
    // masked entries (probability 0), lowest ids first, i.e. with the lowest ids that are not held.  There are
    // k - n of them among the ids below n + (k - n) <= 2 * kRecMax: a bitmap of the held ids in that range and the
    // number of free ids in front of each of its words locate the j-th.
    constexpr int kFillWords = 2 * kRecMax / 32;
    static_assert(kFillWords <= kT && 2 * kFillWords <= kBins, "the bitmap and its prefix live in the histogram");
    uint32_t* const held_bits = sh.hist;
    uint32_t* const free_before = sh.hist + kFillWords;
    if (fill) {
        int t = tid;
        asm volatile("" : "+v"(t));              // (addresses formed here, in this rare branch, not held from the top of the kernel)
        if (t < kFillWords) held_bits[t] = 0u;
        __syncthreads();
        for (int i = t; i < n; i += kT) {
            const uint32_t id = kIdMask - ((uint32_t)sorted[i] & kIdMask);
            if (id < 2u * kRecMax) atomicOr(&held_bits[id >> 5], 1u << (id & 31u));
        }
        __syncthreads();
        const int z = t < kFillWords ? 32 - __popc(held_bits[t]) : 0;
        const int incl = wave_scan_incl(z);
        if (lane == kWave - 1) sh.wtot[wave] = incl;
        __syncthreads();
        int before = 0;
#pragma unroll
        for (int w = 0; w < kW; ++w) before += (w < wave) ? sh.wtot[w] : 0;
        if (t < kFillWords) free_before[t] = (uint32_t)(before + incl - z);
        __syncthreads();
    }
    auto filler = [&](int j) {                   // the j-th lowest id that is not held
        int lo = 0, hi = kFillWords - 1;         // the last word with at most j free ids in front of it
        while (lo < hi) {
            const int mid = (lo + hi + 1) >> 1;
            if ((int)free_before[mid] <= j) lo = mid; else hi = mid - 1;
        }
        uint32_t free = ~held_bits[lo];
        for (int r = j - (int)free_before[lo]; r > 0; --r) free &= free - 1u;
        return lo * 32 + __ffs((int)free) - 1;
    };

    // the dropped loads have landed (they were issued a whole ordering ago); waiting here, in front of the
    // record's stores, keeps the wave from waiting for those at its end
    asm volatile("s_waitcnt vmcnt(0)" : "+v"(dropped));

    const double cd = 1.4426950408889634 * (double)inv_T;
    const double invS = 1.0 / S;
    const bool use_top_p = top_p > 0.f && top_p < 1.f;
    double carry = 0.0, my_mass = 0.0;
    int my_count = 0;
    int32_t* idx_row = idx + row * (int64_t)k;
    float* prob_row = prob + row * (int64_t)k;
    auto emit_value = [&](int slot, int& id, float& pr) {
        const uint64_t cv = sorted[slot];
        id = (int)(kIdMask - ((uint32_t)cv & kIdMask));
        const float x = __uint_as_float(bits_of_short_key<BF16>((uint32_t)(cv >> kIdBits)));
        pr = (float)(exp_emit(x, M, cd) * invS);
    };
    const bool rows_aligned = (k & 3) == 0 && ((((uintptr_t)idx_row) | ((uintptr_t)prob_row)) & 15u) == 0;
    if (fill && !use_top_p) {
        // (rare: a plain loop; with top-p the entries above -inf carry all of the mass, so the prefix that reaches
        //  top_p ends among them and the loop below needs no fillers)
        for (int slot = tid; slot < k; slot += kT) {
            int id;
            float pr = 0.f;
            if (slot < n) { emit_value(slot, id, pr); my_mass += (double)pr; } else id = filler(slot - n);
            ++my_count;
            idx_row[slot] = id;
            prob_row[slot] = pr;
        }
    } else if (!use_top_p && rows_aligned) {
        // every slot is independent.  A thread takes four consecutive slots and writes them with one
        // 16-byte store per array; the record is not read again by this kernel: non-temporal stores.
        static_assert(kSortPer % 4 == 0, "four slots per thread and step");
#pragma unroll
        for (int j = 0; j < kSortPer / 4; ++j) {
            const int s0 = 4 * (tid + j * kT);
            if (s0 < k) {
                typedef int i32x4_t __attribute__((ext_vector_type(4)));
                typedef float f32x4_t __attribute__((ext_vector_type(4)));
                i32x4_t ids = {-1, -1, -1, -1};
                f32x4_t prs = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    if (s0 + e < n) {
                        int id; float pr;
                        emit_value(s0 + e, id, pr);
                        ids[e] = id; prs[e] = pr;
                        my_mass += (double)pr; ++my_count;
                    }
                __builtin_nontemporal_store(ids, reinterpret_cast<i32x4_t*>(idx_row + s0));
                __builtin_nontemporal_store(prs, reinterpret_cast<f32x4_t*>(prob_row + s0));
            }
        }
    } else if (!use_top_p) {
#pragma unroll
        for (int j = 0; j < kSortPer; ++j) {
            const int slot = tid + j * kT;
            if (slot < k) {
                int id = -1;
                float pr = 0.f;
                if (slot < n) { emit_value(slot, id, pr); my_mass += (double)pr; ++my_count; }
                __builtin_nontemporal_store(id, &idx_row[slot]);
                __builtin_nontemporal_store(pr, &prob_row[slot]);
            }
        }
    } else {
        for (int j0 = 0; j0 < k; j0 += kT) {   // keep a slot iff the probability before it has not reached top_p
            const int slot = j0 + tid;
            int id = -1;
            float pr = 0.f;
            if (slot < n) emit_value(slot, id, pr);
            const double mine = (double)pr;
            const double incl = wave_scan_incl(mine);
            if (lane == kWave - 1) sh.red[wave] = incl;
            __syncthreads();
            double before = carry, tot = 0.0;
#pragma unroll
            for (int w = 0; w < kW; ++w) { const double t = sh.red[w]; if (w < wave) before += t; tot += t; }
            __syncthreads();
            const bool keep = slot < n && (before + incl - mine) < (double)top_p;
            carry += tot;
            if (slot < k) {
                idx_row[slot] = keep ? id : -1;
                prob_row[slot] = keep ? pr : 0.f;
            }
            if (keep) { my_mass += (double)pr; ++my_count; }
        }
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
    }
}

template <bool BF16, bool SMALL, bool FAST>
__global__ __launch_bounds__(kT, SMALL ? 6 : 4) void compress_kernel(
    const void* __restrict__ logits, int64_t ld, int V, float inv_T, int k, float top_p,
    int32_t* __restrict__ idx, float* __restrict__ prob, int32_t* __restrict__ count,
    float* __restrict__ mass, float* __restrict__ lse,
    const int32_t* __restrict__ seq_off, const int32_t* __restrict__ n_accept, int ahead)
{
    compress_row<BF16, SMALL, FAST>(blockIdx.x, (int)gridDim.x, logits, ld, V, inv_T, k, top_p, idx, prob, count, mass, lse,
                                    seq_off, n_accept, ahead);
}

// The rows that the small variant marked with count = kRetryRow, through the general code: a few workgroups, each
// looking through its share of the counts (one row per thread and step) and compressing the rows it finds marked.
// (Launching one general workgroup per row just to look would cost tens of microseconds: its LDS makes the launch slow.)
template <bool BF16>
__global__ __launch_bounds__(kT, 4) void compress_retry_kernel(
    const void* __restrict__ logits, int64_t ld, int n_rows, int V, float inv_T, int k, float top_p,
    int32_t* __restrict__ idx, float* __restrict__ prob, int32_t* __restrict__ count,
    float* __restrict__ mass, float* __restrict__ lse,
    const int32_t* __restrict__ seq_off, const int32_t* __restrict__ n_accept)
{
    __shared__ int marked[kT];
    __shared__ int n_marked;
    const int per = (n_rows + (int)gridDim.x - 1) / (int)gridDim.x;
    const int first = (int)blockIdx.x * per, last = min(first + per, n_rows);
    for (int r0 = first; r0 < last; r0 += kT) {
        if (threadIdx.x == 0) n_marked = 0;
        __syncthreads();
        const int r = r0 + (int)threadIdx.x;
        if (r < last && count[r] == kRetryRow) marked[atomicAdd(&n_marked, 1)] = r;
        __syncthreads();
        const int n = n_marked;
        for (int i = 0; i < n; ++i) {
            const int row = marked[i];
            compress_row<BF16, false, false>(row, n_rows, logits, ld, V, inv_T, k, top_p, idx, prob, count, mass, lse,
                                      seq_off, n_accept, 0);
            __syncthreads();                     // (the row's last reads of LDS are done before the next one resets it)
        }
        __syncthreads();
    }
}

// Both streams of a small round in one launch (the draft rows' compression and the target rows' statistics do
// not depend on each other): workgroups 0..n_draft-1 compress, the others take one target row each.
// (For rounds of a few rows: registers are not held down to four waves per SIMD here.)
template <bool BF16>
__global__ __launch_bounds__(kT, 2) void round_stream_kernel(
    const void* __restrict__ draft_logits, int64_t ld_d, int n_draft, int V, float inv_T, int k, float top_p,
    int32_t* __restrict__ idx, float* __restrict__ prob, int32_t* __restrict__ count,
    float* __restrict__ mass, float* __restrict__ lse,
    const void* __restrict__ tgt_logits, int64_t ld_t,
    float* __restrict__ tgt_max, float* __restrict__ tgt_sum, float* __restrict__ tgt_lse,
    SegHeader* __restrict__ seg_header, int seg_stride)
{
    if ((int)blockIdx.x < n_draft) {
        compress_row<BF16, false, false>(blockIdx.x, n_draft, draft_logits, ld_d, V, inv_T, k, top_p, idx, prob, count, mass, lse,
                                  nullptr, nullptr, 0);
    } else if (seg_header) {
        // with the target rows' segment table (the draw then needs no second pass over its row); the row's table is
        // staged in the LDS that a compressing workgroup uses for its candidates
        extern __shared__ __align__(16) unsigned char smem_raw[];
        static_assert(sizeof(CompressShared<kCapBig>) >= kSegStage * sizeof(float2), "the staged table fits the candidate buffer");
        if ((int)blockIdx.x == n_draft && threadIdx.x == 0)
            *seg_header = SegHeader{kSegMagic, kRoundStatsNV<BF16> * kWave, seg_stride, (int32_t)(gridDim.x - n_draft)};
        row_stats_seg_row<BF16, kRoundStatsNV<BF16>, kT, true>((int64_t)blockIdx.x - n_draft, tgt_logits, ld_t, V, inv_T, tgt_max, tgt_sum,
                                                                tgt_lse, reinterpret_cast<float2*>(seg_header + 1), seg_stride,
                                                                reinterpret_cast<float2*>(smem_raw));
    } else {
        row_stats_row<BF16, 2, kT>((int64_t)blockIdx.x - n_draft, tgt_logits, ld_t, V, inv_T, tgt_max, tgt_sum, tgt_lse);
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

// The same draw for records whose rows start on 16-byte boundaries (k a multiple of 4): the wave reads the row
// with 16-byte loads, 1 KB per instruction, and keeps it in registers; lane l of load i owns the four slots
// 4 * (64 i + l) ..., so a chunk of 256 slots is summed by a wave scan and the chunks by a running carry.
template <int CHUNKS>
__global__ __launch_bounds__(256) void sample_draft_vec_kernel(
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
    const float4* p4 = reinterpret_cast<const float4*>(p);
    float4 v[CHUNKS];
    double incl[CHUNKS];                      // inclusive sum over the chunk up to and including this lane's four
    double carry[CHUNKS + 1];                 // sum of the chunks in front
    carry[0] = 0.0;
#pragma unroll
    for (int i = 0; i < CHUNKS; ++i) {
        const int s0 = 4 * (i * kWave + lane);
        v[i] = make_float4(0.f, 0.f, 0.f, 0.f);
        if (s0 < cnt) v[i] = p4[i * kWave + lane];
        if (s0 + 1 >= cnt) v[i].y = 0.f;      // slots behind the count carry no weight
        if (s0 + 2 >= cnt) v[i].z = 0.f;
        if (s0 + 3 >= cnt) v[i].w = 0.f;
    }
#pragma unroll
    for (int i = 0; i < CHUNKS; ++i) {
        const double mine = (((double)v[i].x + (double)v[i].y) + (double)v[i].z) + (double)v[i].w;
        incl[i] = wave_scan_incl(mine);
        carry[i + 1] = carry[i] + read_lane(incl[i], kWave - 1);
    }
    const double target = (double)uniforms[row] * carry[CHUNKS];
    int pick = -1;
#pragma unroll
    for (int i = 0; i < CHUNKS; ++i) {
        if (pick < 0) {                       // (uniform across the wave)
            const unsigned long long ball = __ballot(carry[i] + incl[i] > target);
            if (ball) {
                const int owner = __ffsll((long long)ball) - 1;
                int mine_pick = -1;
                if (lane == owner) {
                    const double w4[4] = {(double)v[i].x, (double)v[i].y, (double)v[i].z, (double)v[i].w};
                    double cum = carry[i] + incl[i] - ((((double)v[i].x + (double)v[i].y) + (double)v[i].z) + (double)v[i].w);
                    mine_pick = 4 * (i * kWave + lane) + 3;
#pragma unroll
                    for (int e = 3; e >= 0; --e) {   // first slot of the four whose cumulative weight exceeds the target
                        double upto = cum;
#pragma unroll
                        for (int f = 0; f <= e; ++f) upto += w4[f];
                        if (upto > target) mine_pick = 4 * (i * kWave + lane) + e;
                    }
                }
                pick = __shfl(mine_pick, owner, kWave);
            }
        }
    }
    if (pick < 0 || pick >= cnt) {            // rounding: the last slot with weight
        if (lane == 0) { pick = cnt - 1; while (pick > 0 && !(p[pick] > 0.f)) --pick; }
        pick = __shfl(pick, 0, kWave);
    }
    if (lane == 0) {
        tok[row] = idx[row * k + pick];
        if (q_scalar) q_scalar[row] = p[pick] / mass[row];
    }
}

}  // namespace

// The small variant (three workgroups per CU) serves records of up to kMaxK / 2 entries on rows long enough that the
// optimistic pass applies and its expected candidates fit the smaller buffer with room to spare (the kernel evaluates
// the same function with a slightly smaller allowance, so it agrees).
static bool small_variant_serves(int k, int V)
{
    return k <= CompressShared<kCapSmall>::kRecMax && V >= 4 * kCompressSample &&
           optimistic_rank(k, V, kCompressSample, kCapSmall, 4.5f) > 0;
}

hipError_t launch_compress(const void* logits, int dtype, int64_t ld, int n_rows, int V, float temperature,
                           int k, float top_p, int32_t* idx, float* prob, int32_t* count, float* mass,
                           float* lse, const int32_t* seq_off, const int32_t* n_accept, hipStream_t stream)
{
    static DeviceFlags limit_raised[8] = {};
    static std::atomic<int> cu_count[kMaxDevices] = {};
    const int bf = dtype == 1 ? 1 : 0;
    // general (both passes in one kernel) / fast (optimistic pass only, rows it gives up marked for the retry kernel),
    // the latter with the large or the small candidate buffer
    const void* const kernels[8] = {(const void*)compress_kernel<false, false, false>, (const void*)compress_kernel<true, false, false>,
                                    (const void*)compress_kernel<false, false, true>, (const void*)compress_kernel<true, false, true>,
                                    nullptr /* (the small buffer serves bf16 rows only) */, (const void*)compress_kernel<true, true, true>,
                                    (const void*)compress_retry_kernel<false>, (const void*)compress_retry_kernel<true>};
    const size_t smem_big = sizeof(CompressShared<kCapBig>), smem_small = sizeof(CompressShared<kCapSmall>);
    int dev = 0;
    {   // (every variant of the dtype: which of them a call takes depends on its sizes)
        hipError_t e = hipSuccess;
        for (int v = 0; v < 4 && e == hipSuccess; ++v)
            if (kernels[2 * v + bf]) e = raise_lds_limit_once(kernels[2 * v + bf], v == 2 ? smem_small : smem_big, limit_raised[2 * v + bf], dev);
        if (e != hipSuccess) return e;
    }
    if (n_rows == 0) return hipSuccess;
    int cus = cu_count[dev].load(std::memory_order_relaxed);
    if (cus == 0) {                              // (first use on this device; a second thread here computes the same value)
        cus = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && cus > 0 ? cus : -1;
        cu_count[dev].store(cus, std::memory_order_relaxed);
    }
    // Calls of more rows than the chip holds at a time take the fast kernels (fewer registers: the careful pass is
    // not in them) and pay one small launch more; smaller calls are bound by that launch and take the general kernel.
    const bool fast = cus > 0 && n_rows > 2 * cus && V > kCompressSample;
    // (fp32 rows stream faster from two workgroups per CU with the large buffer than from three with the small one,
    //  measured at every record length; bf16 rows, which cost twice the arithmetic per byte, gain from the third)
    const bool small = fast && bf && small_variant_serves(k, V);
    // rows resident at a time (2 workgroups per CU, 3 of the small variant): the distance of the look-ahead loads
    // (no look-ahead with a row map: the next row is not known from the row number)
    const int ahead = (!seq_off && cus > 0) ? (small ? 3 : 2) * cus : 0;
    const float inv_T = 1.0f / temperature;
#define PICOSPEC_COMPRESS(BF, SM, FA, SMEM) \
    hipLaunchKernelGGL((compress_kernel<BF, SM, FA>), dim3(n_rows), dim3(kT), SMEM, stream, logits, ld, V, inv_T, k, top_p, idx, prob, count, mass, lse, seq_off, n_accept, ahead)
#define PICOSPEC_RETRY(BF) \
    hipLaunchKernelGGL((compress_retry_kernel<BF>), dim3(min(64, (n_rows + kT - 1) / kT)), dim3(kT), smem_big, stream, logits, ld, n_rows, V, inv_T, k, top_p, idx, prob, count, mass, lse, seq_off, n_accept)
    if (small) {
        PICOSPEC_COMPRESS(true, true, true, smem_small);
    } else if (fast) {
        if (bf) PICOSPEC_COMPRESS(true, false, true, smem_big); else PICOSPEC_COMPRESS(false, false, true, smem_big);
    } else {
        if (bf) PICOSPEC_COMPRESS(true, false, false, smem_big); else PICOSPEC_COMPRESS(false, false, false, smem_big);
    }
    if (fast) {
        if (hipError_t e = hipGetLastError()) return e;
        if (bf) PICOSPEC_RETRY(true); else PICOSPEC_RETRY(false);
    }
#undef PICOSPEC_RETRY
#undef PICOSPEC_COMPRESS
    return hipGetLastError();
}

hipError_t launch_round_stream(const void* draft_logits, int dtype, int64_t ld_d, int n_draft, int V, float temperature,
                               int k, float top_p, int32_t* idx, float* prob, int32_t* count, float* mass, float* lse,
                               const void* tgt_logits, int64_t ld_t, int n_target,
                               float* tgt_max, float* tgt_sum, float* tgt_lse, void* seg_table, hipStream_t stream)
{
    static DeviceFlags limit_raised[2] = {};
    const size_t smem = sizeof(CompressShared<kCapBig>);
    auto f32 = round_stream_kernel<false>;
    auto b16 = round_stream_kernel<true>;
    const int which = dtype == 1;
    {
        int dev = 0;
        hipError_t e = raise_lds_limit_once(which ? (const void*)b16 : (const void*)f32, smem, limit_raised[which], dev);
        if (e != hipSuccess) return e;
    }
    if (n_draft + n_target == 0) return hipSuccess;
    const float inv_T = 1.0f / temperature;
    if (n_target == 0) seg_table = nullptr;
    SegHeader* const header = (SegHeader*)seg_table;
    const int stride = round_stats_shape(dtype, V).stride;
    if (which) hipLaunchKernelGGL(b16, dim3(n_draft + n_target), dim3(kT), smem, stream, draft_logits, ld_d, n_draft, V, inv_T, k, top_p, idx, prob, count, mass, lse, tgt_logits, ld_t, tgt_max, tgt_sum, tgt_lse, header, stride);
    else       hipLaunchKernelGGL(f32, dim3(n_draft + n_target), dim3(kT), smem, stream, draft_logits, ld_d, n_draft, V, inv_T, k, top_p, idx, prob, count, mass, lse, tgt_logits, ld_t, tgt_max, tgt_sum, tgt_lse, header, stride);
    return hipGetLastError();
}

hipError_t launch_sample_draft(const int32_t* idx, const float* prob, const int32_t* count, const float* mass,
                               int k, int n_rows, const float* uniforms, int32_t* tok, float* q_scalar,
                               hipStream_t stream)
{
    if (n_rows == 0) return hipSuccess;
    const int rows_per_block = 256 / kWave;
    const dim3 grid((n_rows + rows_per_block - 1) / rows_per_block);
    if ((k & 3) == 0 && k <= 16 * 256 && (((uintptr_t)prob) & 15u) == 0) {
        // rows on 16-byte boundaries: the row in registers, as many 256-slot chunks as k needs
#define PICOSPEC_SAMPLE_DRAFT(C) \
        hipLaunchKernelGGL(sample_draft_vec_kernel<C>, grid, dim3(256), 0, stream, idx, prob, count, mass, k, n_rows, uniforms, tok, q_scalar)
        if (k <= 256)       PICOSPEC_SAMPLE_DRAFT(1);
        else if (k <= 1024) PICOSPEC_SAMPLE_DRAFT(4);
        else if (k <= 2048) PICOSPEC_SAMPLE_DRAFT(8);
        else                PICOSPEC_SAMPLE_DRAFT(16);
#undef PICOSPEC_SAMPLE_DRAFT
        static_assert(kMaxK <= 16 * 256, "sixteen chunks hold the longest record");
        return hipGetLastError();
    }
    hipLaunchKernelGGL(sample_draft_kernel, grid, dim3(256), 0, stream,
                       idx, prob, count, mass, k, n_rows, uniforms, tok, q_scalar);
    return hipGetLastError();
}

}  // namespace picospec
