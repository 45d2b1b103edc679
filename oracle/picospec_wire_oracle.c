/*
 * PicoSpec wire messages -- CPU oracle (byte-exact definition of the formats).
 *
 * TEST INFRASTRUCTURE ONLY.  Plain C; shares no code, header, table or helper
 * with the HIP library and must never be called from the product path.
 *
 * What it follows (paper Section 3.3):
 *   - Uplink: per round the edge sends the drafted tokens and only their own
 *     probabilities q_1..q_gamma (8 bytes per drafted token with fp32
 *     probabilities: 48 bytes at gamma = 6, the "less than 50 bytes per round").
 *   - Downlink: only for a sequence with a rejection, the Top-K record of the
 *     target distribution at the rejected position, Eq. 4: (id, prob) pairs,
 *     8 bytes per entry (80 bytes at K = 10: "less than 100 bytes").
 *   - The messages are laid out so that the receiver addresses the arrays in
 *     place (naturally aligned blocks behind a fixed-size header): the paper's
 *     zero-copy serialisation.  The paper does not print its byte layout; the
 *     one below is this project's (see the public header for the same text).
 *
 * All fields little-endian.
 *
 * Downlink message (cloud -> edge), one per round and batch:
 *   0   u16 magic 0x5350   2  u8 version (1)   3  u8 prob_format   4  u32 B
 *   8   B entries of 8 bytes: u16 n_accept, u16 count, i32 token
 *       count = entries of the sequence's record that follow (0 when every
 *       draft token was accepted, or when the cloud sends a token instead);
 *       token = the token the cloud decided itself (bonus or correction), -1 if none
 *   ... int32 ids[total]            total = sum of count, sequences in order
 *   ... prob[total] in prob_format  0: fp32, 1: fp16, 2: bf16 (round to nearest even)
 *   ... zero bytes up to a multiple of 4
 *
 * Uplink message (edge -> cloud), one per round and batch:
 *   0   u16 magic 0x5351   2  u8 version (1)   3  u8 prob_format   4  u32 B
 *   8   u16 gamma[B], zero bytes up to a multiple of 4
 *   ... int32 tok[N]   N = sum of gamma
 *   ... q[N] in prob_format, zero bytes up to a multiple of 4
 *
 * Pins live in tests/test_oracle_wire.py: bytes of a hand-written message
 * (tests/golden/wire_small.txt), the paper's payload sizes, fp16/bf16 rounding
 * against numpy's and torch's converters, round trips.
 */
#include <math.h>
#include <stdint.h>
#include <string.h>

enum { WIRE_FP32 = 0, WIRE_FP16 = 1, WIRE_BF16 = 2 };
enum { WIRE_MAGIC_DOWN = 0x5350, WIRE_MAGIC_UP = 0x5351, WIRE_VERSION = 1 };
enum {
    WIRE_BAD_HEADER = 1u,   /* magic, version or prob_format not as expected */
    WIRE_BAD_BATCH = 2u,    /* B in the message differs from the caller's */
    WIRE_CLAMPED = 4u,      /* a count exceeded the receiver's k (or N its capacity): surplus dropped */
    WIRE_TRUNCATED = 8u     /* the buffer is shorter than the message it starts */
};

static void put_u16(uint8_t *p, uint32_t v) { p[0] = (uint8_t)(v & 0xFF); p[1] = (uint8_t)((v >> 8) & 0xFF); }
static void put_u32(uint8_t *p, uint32_t v) { put_u16(p, v & 0xFFFF); put_u16(p + 2, v >> 16); }
static uint32_t get_u16(const uint8_t *p) { return (uint32_t)p[0] | ((uint32_t)p[1] << 8); }
static uint32_t get_u32(const uint8_t *p) { return get_u16(p) | (get_u16(p + 2) << 16); }

/* fp32 -> IEEE binary16, round to nearest, ties to even; overflow -> inf; subnormals kept */
static uint32_t half_bits_of(float f)
{
    uint32_t x;
    memcpy(&x, &f, sizeof x);
    const uint32_t sign = (x >> 16) & 0x8000u;
    const uint32_t e = (x >> 23) & 0xFFu;
    uint32_t m = x & 0x7FFFFFu;
    if (e == 0xFFu) return sign | 0x7C00u | (m ? (0x200u | (m >> 13)) : 0u);
    const int32_t E = (int32_t)e - 127 + 15;   /* exponent field of the half */
    if (E >= 31) return sign | 0x7C00u;
    if (E <= 0) {
        /* below the smallest normal half (2^-14): the result is an integer count of 2^-24 */
        if (E < -10) return sign;              /* below 2^-25: nearest is zero */
        m |= 0x800000u;
        const int shift = 14 - E;              /* 14..24 */
        uint32_t q = m >> shift;
        const uint32_t rem = m & ((1u << shift) - 1u), halfway = 1u << (shift - 1);
        if (rem > halfway || (rem == halfway && (q & 1u))) ++q;
        return sign | q;
    }
    uint32_t h = ((uint32_t)E << 10) | (m >> 13);
    const uint32_t rem = m & 0x1FFFu;
    if (rem > 0x1000u || (rem == 0x1000u && (h & 1u))) ++h;   /* a carry into the exponent is the right result */
    return sign | h;
}

static double value_of_half(uint32_t h)
{
    const double sign = (h & 0x8000u) ? -1.0 : 1.0;
    const int e = (int)((h >> 10) & 0x1Fu);
    const uint32_t m = h & 0x3FFu;
    if (e == 31) return m ? NAN : sign * INFINITY;
    if (e == 0) return sign * ldexp((double)m, -24);
    return sign * ldexp((double)(m | 0x400u), e - 25);
}

/* fp32 -> bfloat16 (the top 16 bits of an fp32), round to nearest, ties to even */
static uint32_t bf16_bits_of(float f)
{
    uint32_t x;
    memcpy(&x, &f, sizeof x);
    if (((x >> 23) & 0xFFu) == 0xFFu && (x & 0x7FFFFFu)) return (x >> 16) | 0x40u;   /* NaN stays NaN */
    const uint32_t low = x & 0xFFFFu;
    uint32_t top = x >> 16;
    if (low > 0x8000u || (low == 0x8000u && (top & 1u))) ++top;
    return top & 0xFFFFu;
}

static double value_of_bf16(uint32_t b)
{
    const uint32_t x = b << 16;
    float f;
    memcpy(&f, &x, sizeof f);
    return (double)f;
}

static int prob_width(int fmt) { return fmt == WIRE_FP32 ? 4 : 2; }

static void put_prob(uint8_t *p, int fmt, float v)
{
    if (fmt == WIRE_FP32) {
        uint32_t x;
        memcpy(&x, &v, sizeof x);
        put_u32(p, x);
    } else if (fmt == WIRE_FP16) {
        put_u16(p, half_bits_of(v));
    } else {
        put_u16(p, bf16_bits_of(v));
    }
}

static double get_prob(const uint8_t *p, int fmt)
{
    if (fmt == WIRE_FP32) {
        const uint32_t x = get_u32(p);
        float f;
        memcpy(&f, &x, sizeof f);
        return (double)f;
    }
    return fmt == WIRE_FP16 ? value_of_half(get_u16(p)) : value_of_bf16(get_u16(p));
}

static int64_t round_up4(int64_t n) { return (n + 3) / 4 * 4; }

/* exposed for the rounding pins */
int oracle_wire_quantise(const float *in, int32_t n, int fmt, uint16_t *bits, double *back)
{
    if (fmt != WIRE_FP16 && fmt != WIRE_BF16) return -1;
    for (int32_t i = 0; i < n; ++i) {
        const uint32_t b = fmt == WIRE_FP16 ? half_bits_of(in[i]) : bf16_bits_of(in[i]);
        bits[i] = (uint16_t)b;
        back[i] = fmt == WIRE_FP16 ? value_of_half(b) : value_of_bf16(b);
    }
    return 0;
}

/* entries the downlink carries for sequence b: the record's, if a draft token was rejected */
static int32_t downlink_count(int32_t b, const int32_t *seq_off, const int32_t *n_accept,
                              const int32_t *idx, const int32_t *count, int32_t k)
{
    if (!idx) return 0;
    const int32_t gamma = seq_off[b + 1] - seq_off[b];
    if (n_accept[b] >= gamma) return 0;
    int32_t c = count[b];
    if (c < 0) c = 0;
    if (c > k) c = k;
    return c;
}

/* Packs one downlink message.  idx/prob/count: the records of the rejected positions, [B,k] (idx may be
 * NULL: no records, tokens only).  token: nullable [B], sent for the sequences that carry no record.
 * *wire_bytes = size of the message; nothing is written if it exceeds capacity (returns 1). */
int oracle_pack_downlink(int32_t B, const int32_t *seq_off, const int32_t *n_accept, const int32_t *token,
                         const int32_t *idx, const float *prob, const int32_t *count, int32_t k, int fmt,
                         uint8_t *wire, int64_t capacity, int64_t *wire_bytes)
{
    if (B < 0 || k < 0 || fmt < 0 || fmt > 2) return -1;
    int64_t total = 0;
    for (int32_t b = 0; b < B; ++b) total += downlink_count(b, seq_off, n_accept, idx, count, k);
    const int64_t ids_at = 8 + 8 * (int64_t)B, probs_at = ids_at + 4 * total;
    const int64_t bytes = round_up4(probs_at + prob_width(fmt) * total);
    *wire_bytes = bytes;
    if (bytes > capacity) return 1;
    memset(wire, 0, (size_t)bytes);
    put_u16(wire, WIRE_MAGIC_DOWN);
    wire[2] = WIRE_VERSION;
    wire[3] = (uint8_t)fmt;
    put_u32(wire + 4, (uint32_t)B);
    int64_t at = 0;
    for (int32_t b = 0; b < B; ++b) {
        const int32_t c = downlink_count(b, seq_off, n_accept, idx, count, k);
        const int32_t gamma = seq_off[b + 1] - seq_off[b];
        int32_t na = n_accept[b];
        if (na < 0) na = 0;
        if (na > gamma) na = gamma;
        if (na > 65535) na = 65535;
        uint8_t *e = wire + 8 + 8 * (int64_t)b;
        put_u16(e, (uint32_t)na);
        put_u16(e + 2, (uint32_t)c);
        put_u32(e + 4, (uint32_t)((c == 0 && token) ? token[b] : -1));
        for (int32_t j = 0; j < c; ++j) {
            put_u32(wire + ids_at + 4 * (at + j), (uint32_t)idx[(int64_t)b * k + j]);
            put_prob(wire + probs_at + prob_width(fmt) * (at + j), fmt, prob[(int64_t)b * k + j]);
        }
        at += c;
    }
    return 0;
}

/* Unpacks a downlink message into the record layout the local resampling takes: idx/prob [B,k]
 * (unused slots idx = -1, prob = 0), count, mass = sum of the probabilities as received, in slot order.
 * status: bit set of WIRE_*; with WIRE_BAD_HEADER, WIRE_BAD_BATCH or WIRE_TRUNCATED nothing else is written. */
int oracle_unpack_downlink(const uint8_t *wire, int64_t wire_bytes, int32_t B, int32_t k,
                           int32_t *n_accept, int32_t *token, int32_t *idx, double *prob, int32_t *count,
                           double *mass, uint32_t *status)
{
    *status = 0;
    if (wire_bytes < 8 || get_u16(wire) != WIRE_MAGIC_DOWN || wire[2] != WIRE_VERSION || wire[3] > 2) {
        *status = WIRE_BAD_HEADER;
        return 0;
    }
    if (get_u32(wire + 4) != (uint32_t)B) { *status = WIRE_BAD_BATCH; return 0; }
    const int fmt = wire[3];
    if (wire_bytes < 8 + 8 * (int64_t)B) { *status = WIRE_TRUNCATED; return 0; }
    int64_t total = 0;
    for (int32_t b = 0; b < B; ++b) total += get_u16(wire + 8 + 8 * (int64_t)b + 2);
    const int64_t ids_at = 8 + 8 * (int64_t)B, probs_at = ids_at + 4 * total;
    if (wire_bytes < round_up4(probs_at + prob_width(fmt) * total)) { *status = WIRE_TRUNCATED; return 0; }
    int64_t at = 0;
    for (int32_t b = 0; b < B; ++b) {
        const uint8_t *e = wire + 8 + 8 * (int64_t)b;
        const int32_t c_sent = (int32_t)get_u16(e + 2);
        int32_t c = c_sent;
        if (c > k) { c = k; *status |= WIRE_CLAMPED; }
        n_accept[b] = (int32_t)get_u16(e);
        token[b] = (int32_t)get_u32(e + 4);
        count[b] = c;
        double m = 0.0;
        for (int32_t j = 0; j < k; ++j) {
            if (j < c) {
                idx[(int64_t)b * k + j] = (int32_t)get_u32(wire + ids_at + 4 * (at + j));
                prob[(int64_t)b * k + j] = get_prob(wire + probs_at + prob_width(fmt) * (at + j), fmt);
                m += prob[(int64_t)b * k + j];
            } else {
                idx[(int64_t)b * k + j] = -1;
                prob[(int64_t)b * k + j] = 0.0;
            }
        }
        mass[b] = m;
        at += c_sent;
    }
    return 0;
}

/* Packs one uplink message: the drafted tokens of every sequence and their own probabilities. */
int oracle_pack_uplink(int32_t B, const int32_t *seq_off, const int32_t *draft_tok, const float *q_scalar,
                       int fmt, uint8_t *wire, int64_t capacity, int64_t *wire_bytes)
{
    if (B < 0 || fmt < 0 || fmt > 2) return -1;
    const int64_t N = seq_off[B] - seq_off[0];
    const int64_t tok_at = 8 + round_up4(2 * (int64_t)B), q_at = tok_at + 4 * N;
    const int64_t bytes = round_up4(q_at + prob_width(fmt) * N);
    *wire_bytes = bytes;
    if (bytes > capacity) return 1;
    memset(wire, 0, (size_t)bytes);
    put_u16(wire, WIRE_MAGIC_UP);
    wire[2] = WIRE_VERSION;
    wire[3] = (uint8_t)fmt;
    put_u32(wire + 4, (uint32_t)B);
    for (int32_t b = 0; b < B; ++b) {
        int32_t g = seq_off[b + 1] - seq_off[b];
        if (g < 0 || g > 65535) return -1;
        put_u16(wire + 8 + 2 * (int64_t)b, (uint32_t)g);
    }
    for (int64_t i = 0; i < N; ++i) {
        put_u32(wire + tok_at + 4 * i, (uint32_t)draft_tok[seq_off[0] + i]);
        put_prob(wire + q_at + prob_width(fmt) * i, fmt, q_scalar[seq_off[0] + i]);
    }
    return 0;
}

/* Unpacks an uplink message: seq_off[B+1] (from 0), draft_tok and q_scalar for at most n_max positions. */
int oracle_unpack_uplink(const uint8_t *wire, int64_t wire_bytes, int32_t B, int32_t n_max,
                         int32_t *seq_off, int32_t *draft_tok, double *q_scalar, uint32_t *status)
{
    *status = 0;
    if (wire_bytes < 8 || get_u16(wire) != WIRE_MAGIC_UP || wire[2] != WIRE_VERSION || wire[3] > 2) {
        *status = WIRE_BAD_HEADER;
        return 0;
    }
    if (get_u32(wire + 4) != (uint32_t)B) { *status = WIRE_BAD_BATCH; return 0; }
    const int fmt = wire[3];
    const int64_t tok_at = 8 + round_up4(2 * (int64_t)B);
    if (wire_bytes < tok_at) { *status = WIRE_TRUNCATED; return 0; }
    int64_t N = 0;
    for (int32_t b = 0; b < B; ++b) N += get_u16(wire + 8 + 2 * (int64_t)b);
    const int64_t q_at = tok_at + 4 * N;
    if (wire_bytes < round_up4(q_at + prob_width(fmt) * N)) { *status = WIRE_TRUNCATED; return 0; }
    /* sequences are kept whole: the first one that does not fit n_max, and all behind it, come out empty */
    int64_t at = 0;
    int fits = 1;
    seq_off[0] = 0;
    for (int32_t b = 0; b < B; ++b) {
        const int64_t g = get_u16(wire + 8 + 2 * (int64_t)b);
        if (fits && seq_off[b] + g > n_max) { fits = 0; *status |= WIRE_CLAMPED; }
        const int64_t keep = fits ? g : 0;
        for (int64_t i = 0; i < keep; ++i) {
            draft_tok[seq_off[b] + i] = (int32_t)get_u32(wire + tok_at + 4 * (at + i));
            q_scalar[seq_off[b] + i] = get_prob(wire + q_at + prob_width(fmt) * (at + i), fmt);
        }
        seq_off[b + 1] = seq_off[b] + (int32_t)keep;
        at += g;
    }
    return 0;
}
