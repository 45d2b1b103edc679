// Wire messages of a speculative round (paper Section 3.3): the uplink carries the drafted tokens
// and only their own probabilities q_1..q_gamma, the downlink carries, for a sequence with a
// rejection, the Top-K record of Eq. 4 (8 bytes per entry with fp32 probabilities).  Every block of a
// message is naturally aligned behind a fixed-size header, so the receiver addresses the arrays in
// place; these kernels gather the ragged per-sequence records into one contiguous buffer (one DMA
// to the NIC or host) and spread a received message back into the record layout the local
// resampling takes.  The byte layout is stated in include/picospec.h.
#include "common.hpp"
#include "kernels.hpp"

namespace picospec {

namespace {

constexpr int kWT = 256;                      // threads per workgroup
constexpr int kWW = kWT / kWave;
constexpr uint32_t kMagicDown = 0x5350u, kMagicUp = 0x5351u, kVersion = 1u;
constexpr uint32_t kBadHeader = 1u, kBadBatch = 2u, kClamped = 4u, kTruncated = 8u;

__device__ __forceinline__ int prob_width(int fmt) { return fmt == 0 ? 4 : 2; }
__host__ __device__ __forceinline__ int64_t round_up4(int64_t n) { return (n + 3) & ~(int64_t)3; }

// fp32 -> binary16 bits, round to nearest even (the conversion instruction under the default mode:
// nearest-even, fp16 subnormals kept)
__device__ __forceinline__ uint32_t half_bits(float v) {
    const _Float16 h = (_Float16)v;
    unsigned short b;
    __builtin_memcpy(&b, &h, sizeof b);
    return b;
}
__device__ __forceinline__ float half_value(uint32_t b) {
    const unsigned short s = (unsigned short)b;
    _Float16 h;
    __builtin_memcpy(&h, &s, sizeof h);
    return (float)h;
}
// fp32 -> bfloat16 bits, round to nearest even
__device__ __forceinline__ uint32_t bf16_bits(float v) {
    const uint32_t x = __float_as_uint(v);
    if ((x & 0x7FFFFFFFu) > 0x7F800000u) return (x >> 16) | 0x40u;
    return (x + 0x7FFFu + ((x >> 16) & 1u)) >> 16;
}

__device__ __forceinline__ void store_prob(unsigned char* probs, int fmt, int64_t i, float v) {
    if (fmt == 0) reinterpret_cast<float*>(probs)[i] = v;
    else reinterpret_cast<unsigned short*>(probs)[i] = (unsigned short)(fmt == 1 ? half_bits(v) : bf16_bits(v));
}
__device__ __forceinline__ float load_prob(const unsigned char* probs, int fmt, int64_t i) {
    if (fmt == 0) return reinterpret_cast<const float*>(probs)[i];
    const uint32_t b = reinterpret_cast<const unsigned short*>(probs)[i];
    return fmt == 1 ? half_value(b) : __uint_as_float(b << 16);
}

// sum over the workgroup of two 64-bit counts, result in every thread
__device__ __forceinline__ void block_sum2(long long& a, long long& b, long long* sh) {
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
    const long long wa = wave_sum(a), wb = wave_sum(b);
    __syncthreads();
    if (lane == 0) { sh[wave] = wa; sh[kWW + wave] = wb; }
    __syncthreads();
    a = 0; b = 0;
#pragma unroll
    for (int w = 0; w < kWW; ++w) { a += sh[w]; b += sh[kWW + w]; }
}

// entries the downlink carries for sequence i: its record's, if one of its draft tokens was rejected
__device__ __forceinline__ int downlink_count(int i, const int32_t* seq_off, const int32_t* n_accept,
                                              const int32_t* count, int k) {
    if (!count) return 0;
    const int g = seq_off[i + 1] - seq_off[i];
    if (n_accept[i] >= g) return 0;
    const int c = count[i];
    return c < 0 ? 0 : (c > k ? k : c);
}

// One workgroup per sequence.  The message has no offset table (the receiver sums the counts), so
// each workgroup sums the counts in front of its sequence itself: B is a batch size, the O(B) loop
// per workgroup is small change next to the record it copies.
__global__ __launch_bounds__(kWT) void pack_downlink_kernel(
    int B, const int32_t* __restrict__ seq_off, const int32_t* __restrict__ n_accept,
    const int32_t* __restrict__ token, const int32_t* __restrict__ idx, const float* __restrict__ prob,
    const int32_t* __restrict__ count, int k, int fmt,
    unsigned char* __restrict__ wire, int64_t capacity, int64_t* __restrict__ wire_bytes, uint32_t* __restrict__ status)
{
    __shared__ long long sh[2 * kWW];
    const int tid = threadIdx.x, b = blockIdx.x;
    long long before = 0, total = 0;
    for (int i = tid; i < B; i += kWT) {
        const int c = downlink_count(i, seq_off, n_accept, count, k);
        total += c;
        if (i < b) before += c;
    }
    block_sum2(before, total, sh);
    const int64_t ids_at = 8 + 8 * (int64_t)B, probs_at = ids_at + 4 * total;
    const int64_t end = probs_at + prob_width(fmt) * total, bytes = round_up4(end);
    const bool fits = bytes <= capacity;
    if (b == 0 && tid == 0) {
        *wire_bytes = bytes;
        *status = fits ? 0u : kTruncated;
        if (fits) {
            reinterpret_cast<uint32_t*>(wire)[0] = kMagicDown | (kVersion << 16) | ((uint32_t)fmt << 24);
            reinterpret_cast<uint32_t*>(wire)[1] = (uint32_t)B;
            for (int64_t p = end; p < bytes; ++p) wire[p] = 0;
        }
    }
    if (!fits || b >= B) return;
    const int c = downlink_count(b, seq_off, n_accept, count, k);
    if (tid == 0) {
        const int g = seq_off[b + 1] - seq_off[b];
        int na = n_accept[b];
        na = na < 0 ? 0 : (na > g ? g : na);
        na = na > 65535 ? 65535 : na;
        uint32_t* e = reinterpret_cast<uint32_t*>(wire + 8 + 8 * (int64_t)b);
        e[0] = (uint32_t)na | ((uint32_t)c << 16);
        e[1] = (uint32_t)((c == 0 && token) ? token[b] : -1);
    }
    int32_t* ids = reinterpret_cast<int32_t*>(wire + ids_at);
    unsigned char* probs = wire + probs_at;
    for (int j = tid; j < c; j += kWT) {
        ids[before + j] = idx[(int64_t)b * k + j];
        store_prob(probs, fmt, before + j, prob[(int64_t)b * k + j]);
    }
}

// One workgroup per sequence: checks the header, sums the counts in front of its sequence, fills
// the sequence's slots (unused ones with id -1, probability 0) and sums the mass in fp64.
__global__ __launch_bounds__(kWT) void unpack_downlink_kernel(
    const unsigned char* __restrict__ wire, int64_t wire_bytes, int B, int k,
    int32_t* __restrict__ n_accept, int32_t* __restrict__ token, int32_t* __restrict__ idx,
    float* __restrict__ prob, int32_t* __restrict__ count, float* __restrict__ mass, uint32_t* __restrict__ status)
{
    __shared__ long long sh[2 * kWW];
    __shared__ double shd[kWW];
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave, b = blockIdx.x;
    uint32_t st = 0;
    int fmt = 0;
    if (wire_bytes < 8) st = kBadHeader;
    else {
        const uint32_t h = reinterpret_cast<const uint32_t*>(wire)[0];
        fmt = (int)(h >> 24);
        if ((h & 0xFFFFu) != kMagicDown || ((h >> 16) & 0xFFu) != kVersion || fmt > 2) st = kBadHeader;
        else if (reinterpret_cast<const uint32_t*>(wire)[1] != (uint32_t)B) st = kBadBatch;
        else if (wire_bytes < 8 + 8 * (int64_t)B) st = kTruncated;
    }
    long long before = 0, total = 0;
    int over = 0;
    if (!st) {
        for (int i = tid; i < B; i += kWT) {
            const int c = (int)(reinterpret_cast<const uint32_t*>(wire + 8 + 8 * (int64_t)i)[0] >> 16);
            total += c;
            if (i < b) before += c;
            over |= c > k;
        }
        long long any_over = over;
        block_sum2(before, total, sh);
        long long dummy = 0;
        block_sum2(any_over, dummy, sh);
        over = any_over != 0;
    }
    const int64_t ids_at = 8 + 8 * (int64_t)B, probs_at = ids_at + 4 * total;
    if (!st && wire_bytes < round_up4(probs_at + prob_width(fmt) * total)) st = kTruncated;
    if (b == 0 && tid == 0) *status = st ? st : (over ? kClamped : 0u);
    if (st || b >= B) return;
    const uint32_t* e = reinterpret_cast<const uint32_t*>(wire + 8 + 8 * (int64_t)b);
    const int c = min((int)(e[0] >> 16), k);
    const int32_t* ids = reinterpret_cast<const int32_t*>(wire + ids_at);
    const unsigned char* probs = wire + probs_at;
    double mine = 0.0;
    for (int j = tid; j < k; j += kWT) {
        int id = -1;
        float p = 0.f;
        if (j < c) { id = ids[before + j]; p = load_prob(probs, fmt, before + j); }
        idx[(int64_t)b * k + j] = id;
        prob[(int64_t)b * k + j] = p;
        mine += (double)p;
    }
    const double ws = wave_sum(mine);
    if (lane == 0) shd[wave] = ws;
    __syncthreads();
    if (tid == 0) {
        double m = 0.0;
        for (int w = 0; w < kWW; ++w) m += shd[w];
        mass[b] = (float)m;
        count[b] = c;
        n_accept[b] = (int)(e[0] & 0xFFFFu);
        token[b] = (int32_t)e[1];
    }
}

// Elementwise over max(N, B): position i copies its token and converts its probability, sequence i
// writes its gamma; thread 0 of the grid writes the header and the padding.
__global__ __launch_bounds__(kWT) void pack_uplink_kernel(
    int B, int N, const int32_t* __restrict__ seq_off, const int32_t* __restrict__ draft_tok,
    const float* __restrict__ q_scalar, int fmt, unsigned char* __restrict__ wire, int64_t* __restrict__ wire_bytes)
{
    const int64_t i = (int64_t)blockIdx.x * kWT + threadIdx.x;
    const int64_t tok_at = 8 + round_up4(2 * (int64_t)B), q_at = tok_at + 4 * (int64_t)N;
    const int64_t end = q_at + prob_width(fmt) * (int64_t)N, bytes = round_up4(end);
    if (i == 0) {
        *wire_bytes = bytes;
        reinterpret_cast<uint32_t*>(wire)[0] = kMagicUp | (kVersion << 16) | ((uint32_t)fmt << 24);
        reinterpret_cast<uint32_t*>(wire)[1] = (uint32_t)B;
        for (int64_t p = 8 + 2 * (int64_t)B; p < tok_at; ++p) wire[p] = 0;
        for (int64_t p = end; p < bytes; ++p) wire[p] = 0;
    }
    if (i < B) reinterpret_cast<unsigned short*>(wire + 8)[i] = (unsigned short)(seq_off[i + 1] - seq_off[i]);
    if (i < N) {
        reinterpret_cast<int32_t*>(wire + tok_at)[i] = draft_tok[i];
        store_prob(wire + q_at, fmt, i, q_scalar[i]);
    }
}

// First kernel of the uplink's unpacking, one workgroup: header check and the prefix sum of the
// gammas into seq_off.  Sequences are kept whole: the first one that does not fit n_max positions,
// and all behind it, come out empty, so seq_off[B] is also the number of positions to copy.
__global__ __launch_bounds__(kWT) void unpack_uplink_offsets_kernel(
    const unsigned char* __restrict__ wire, int64_t wire_bytes, int B, int n_max,
    int32_t* __restrict__ seq_off, uint32_t* __restrict__ status)
{
    __shared__ long long sh[2 * kWW];
    __shared__ long long s_wave[kWW];
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
    uint32_t st = 0;
    int fmt = 0;
    const int64_t tok_at = 8 + round_up4(2 * (int64_t)B);
    if (wire_bytes < 8) st = kBadHeader;
    else {
        const uint32_t h = reinterpret_cast<const uint32_t*>(wire)[0];
        fmt = (int)(h >> 24);
        if ((h & 0xFFFFu) != kMagicUp || ((h >> 16) & 0xFFu) != kVersion || fmt > 2) st = kBadHeader;
        else if (reinterpret_cast<const uint32_t*>(wire)[1] != (uint32_t)B) st = kBadBatch;
        else if (wire_bytes < tok_at) st = kTruncated;
    }
    const unsigned short* gam = reinterpret_cast<const unsigned short*>(wire + 8);
    long long N = 0, dummy = 0;
    if (!st) {
        for (int i = tid; i < B; i += kWT) N += gam[i];
        block_sum2(N, dummy, sh);
        if (wire_bytes < round_up4(tok_at + (4 + prob_width(fmt)) * N)) st = kTruncated;
    }
    if (st) {
        if (tid == 0) *status = st;
        return;
    }
    // inclusive prefix sums, kWT sequences per trip.  Prefix sums only grow, so the sequences that fit
    // n_max are a prefix and the last fitting sum is the number of positions kept.
    __shared__ unsigned long long s_kept;
    if (tid == 0) s_kept = 0;
    long long carry = 0, my_fit = 0;
    for (int base = 0; base < B; base += kWT) {
        const int i = base + tid;
        const long long g = i < B ? (long long)gam[i] : 0;
        long long incl = wave_scan_incl(g);
        __syncthreads();
        if (lane == kWave - 1) s_wave[wave] = incl;
        __syncthreads();
        long long tot = 0;
#pragma unroll
        for (int w = 0; w < kWW; ++w) { const long long t = s_wave[w]; if (w < wave) incl += t; tot += t; }
        incl += carry;
        if (i < B) {
            const bool fits = incl <= (long long)n_max;
            if (fits) my_fit = incl;
            seq_off[i + 1] = fits ? (int32_t)incl : -1;      // (-1: patched below, by this same thread)
        }
        carry += tot;
    }
    atomicMax(&s_kept, (unsigned long long)my_fit);
    __syncthreads();
    const long long kept = (long long)s_kept;
    if (tid == 0) { seq_off[0] = 0; *status = carry > kept ? kClamped : 0u; }
    for (int i = tid; i < B; i += kWT)
        if (seq_off[i + 1] < 0) seq_off[i + 1] = (int32_t)kept;
}

// Second kernel: copies the seq_off[B] kept positions.
__global__ __launch_bounds__(kWT) void unpack_uplink_copy_kernel(
    const unsigned char* __restrict__ wire, int B, int n_max, const int32_t* __restrict__ seq_off,
    const uint32_t* __restrict__ status, int32_t* __restrict__ draft_tok, float* __restrict__ q_scalar)
{
    const uint32_t st = *status;
    if (st & (kBadHeader | kBadBatch | kTruncated)) return;
    const int64_t i = (int64_t)blockIdx.x * kWT + threadIdx.x;
    const int kept = min(seq_off[B], n_max);
    if (i >= kept) return;
    const int fmt = (int)(reinterpret_cast<const uint32_t*>(wire)[0] >> 24);
    const int64_t tok_at = 8 + round_up4(2 * (int64_t)B);
    // the q block starts behind ALL tokens of the message, kept or not
    long long N = 0;
    const unsigned short* gam = reinterpret_cast<const unsigned short*>(wire + 8);
    if (st & kClamped) { for (int s = 0; s < B; ++s) N += gam[s]; } else N = kept;
    draft_tok[i] = reinterpret_cast<const int32_t*>(wire + tok_at)[i];
    q_scalar[i] = load_prob(wire + tok_at + 4 * N, fmt, i);
}

}  // namespace

int64_t downlink_bytes_max(int B, int k, int fmt) {
    return round_up4(8 + 8 * (int64_t)B + (int64_t)(4 + (fmt == 0 ? 4 : 2)) * B * k);
}

int64_t uplink_bytes(int B, int n_draft, int fmt) {
    return round_up4(8 + round_up4(2 * (int64_t)B) + (int64_t)(4 + (fmt == 0 ? 4 : 2)) * n_draft);
}

hipError_t launch_pack_downlink(int B, const int32_t* seq_off, const int32_t* n_accept, const int32_t* token,
                                const int32_t* idx, const float* prob, const int32_t* count, int k, int fmt,
                                void* wire, int64_t capacity, int64_t* wire_bytes, uint32_t* status, hipStream_t stream)
{
    // (B = 0 still writes the 8-byte header)
    hipLaunchKernelGGL(pack_downlink_kernel, dim3(B > 0 ? B : 1), dim3(kWT), 0, stream, B, seq_off, n_accept, token,
                       idx, prob, count, k, fmt, (unsigned char*)wire, capacity, wire_bytes, status);
    return hipGetLastError();
}

hipError_t launch_unpack_downlink(const void* wire, int64_t wire_bytes, int B, int k, int32_t* n_accept,
                                  int32_t* token, int32_t* idx, float* prob, int32_t* count, float* mass,
                                  uint32_t* status, hipStream_t stream)
{
    hipLaunchKernelGGL(unpack_downlink_kernel, dim3(B > 0 ? B : 1), dim3(kWT), 0, stream, (const unsigned char*)wire,
                       wire_bytes, B, k, n_accept, token, idx, prob, count, mass, status);
    return hipGetLastError();
}

hipError_t launch_pack_uplink(int B, int n_draft, const int32_t* seq_off, const int32_t* draft_tok,
                              const float* q_scalar, int fmt, void* wire, int64_t* wire_bytes, hipStream_t stream)
{
    const int64_t n = n_draft > B ? n_draft : B;
    hipLaunchKernelGGL(pack_uplink_kernel, dim3((unsigned)((n + kWT - 1) / kWT > 0 ? (n + kWT - 1) / kWT : 1)), dim3(kWT), 0,
                       stream, B, n_draft, seq_off, draft_tok, q_scalar, fmt, (unsigned char*)wire, wire_bytes);
    return hipGetLastError();
}

hipError_t launch_unpack_uplink(const void* wire, int64_t wire_bytes, int B, int n_max, int32_t* seq_off,
                                int32_t* draft_tok, float* q_scalar, uint32_t* status, hipStream_t stream)
{
    hipLaunchKernelGGL(unpack_uplink_offsets_kernel, dim3(1), dim3(kWT), 0, stream, (const unsigned char*)wire,
                       wire_bytes, B, n_max, seq_off, status);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || n_max == 0) return e;
    hipLaunchKernelGGL(unpack_uplink_copy_kernel, dim3((unsigned)(((int64_t)n_max + kWT - 1) / kWT)), dim3(kWT), 0, stream,
                       (const unsigned char*)wire, B, n_max, seq_off, status, draft_tok, q_scalar);
    return hipGetLastError();
}

}  // namespace picospec
