/*
 * picospec.h -- C ABI of the MI355X (gfx950) implementation of PicoSpec's separate rejection
 * sampling with sparse compression (paper Section 3.3).
 *
 * One speculative round over B sequences, sequence b having gamma_b drafted positions:
 *
 *   picospec_compress        sparse Top-K record of every draft distribution        (Eq. 4)
 *   picospec_sample_draft    the drafter's token draw from that record (edge side, Section 3.3)
 *   picospec_verify          parallel verification: acceptance test, first rejection (Section 3.3)
 *   picospec_verify_range    the same for a range of each draft's positions (Section 3.2, Fast Verification)
 *   picospec_sample_residual correction token ~ norm(max(0, P_j - Q_j)), or the bonus token
 *   picospec_round           the three calls above as one (two launches for small rounds)
 *   picospec_row_stats / picospec_compress_rejected / picospec_resample_sparse
 *                            the paper's own downlink: Top-K record of the target row at the
 *                            rejected position, local resampling at the edge (Section 3.3, Eq. 4)
 *   picospec_pack_uplink / picospec_unpack_uplink / picospec_pack_downlink / picospec_unpack_downlink
 *                            the two messages of a round as contiguous, in-place addressable buffers
 *
 * Conventions shared by all calls
 *   - Every data pointer is a DEVICE pointer (HBM) unless marked "host".  The caller owns all
 *     buffers; the library neither allocates nor frees nor synchronises.  Work is enqueued on
 *     `stream` (a hipStream_t passed as void*, NULL = the default stream) of the current device
 *     and the call returns at once; outputs are valid once the stream reaches that point.
 *   - Logits are row-major [rows, ld] with ld >= V elements between row starts, dtype
 *     PICOSPEC_F32 or PICOSPEC_BF16; the base pointer must be element-aligned.  Rows need not be
 *     16-byte aligned (aligned rows stream fastest).  Softmax is taken at `temperature` > 0:
 *     P(x) = exp(z_x / T - lse).  -inf logits are legal (P = 0: a masked vocabulary entry).  NaN or +inf
 *     logits, and rows without any finite logit (no distribution exists), give unspecified (but
 *     memory-safe) results.
 *   - Ragged batch: seq_off[B+1] (int32, device) is the CSR over draft rows, gamma_b =
 *     seq_off[b+1] - seq_off[b] >= 0, N = seq_off[B] is also passed from the host as n_draft.
 *     Target rows are packed with one extra (bonus) row per sequence: position t in 0..gamma_b
 *     of sequence b is target row seq_off[b] + b + t.  `uniforms` ([N+B] fp32 in [0,1)) is
 *     indexed like target rows: entry (b, t < gamma_b) drives the acceptance of draft position t,
 *     entry (b, gamma_b) drives the correction / bonus draw whatever n_accept[b] turns out to be.
 *   - Sparse record of one row: k slots; idx[slot] (int32 vocabulary id) and prob[slot] (fp32,
 *     the raw probability P(id), not renormalised), ordered by (logit descending, id ascending);
 *     count used slots, the rest hold idx = -1, prob = 0; mass = sum of the kept prob.
 *     8 bytes per kept component, as in the paper's payload arithmetic.
 *   - Workspace: optional everywhere (NULL: the call works without it).  picospec_verify, picospec_verify_sample and
 *     picospec_round can keep the target rows' SEGMENT TABLE in it: the sum of exp((z - M)/T) over every 2 or 4 KB of
 *     every target row, which the statistics pass has at hand anyway.  With it the correction / bonus draw
 *     (picospec_sample_residual given the SAME workspace that picospec_verify filled for the same rows, or the draw
 *     inside the fused calls) does not stream its target row a second time: it gathers one logit per record entry
 *     and reads the one segment in which the draw falls.  Size: picospec_workspace_bytes(call, dtype, n_draft + B, V, k)
 *     bytes on a 16-byte boundary (about 1.2 KB per target row at V = 152 K); its content is the library's business.
 *   - Return value: PICOSPEC_OK or a negative PICOSPEC_E* code.  Misuse that the host can see
 *     (null pointers, sizes, dtype, workspace) is rejected BEFORE anything is launched.
 *     Data-dependent conditions never fail a call; they set bits in `flags`.
 *   - Thread safety: no global mutable state besides per-device kernel attributes set on first
 *     use; concurrent calls on different streams are independent.
 *   - Stream capture: a call only enqueues kernels (no memset, no copy, no allocation, no
 *     synchronisation), so a stream that is being captured into a HIP graph records it like any
 *     other launch.  The kernel attributes are set the first time a kernel is used on a device:
 *     make each call once outside a capture first.
 */
#ifndef PICOSPEC_H
#define PICOSPEC_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum { PICOSPEC_F32 = 0, PICOSPEC_BF16 = 1 };

enum {
    PICOSPEC_OK = 0,
    PICOSPEC_EINVAL = -1,      /* null pointer, size out of range, bad temperature ... */
    PICOSPEC_EWORKSPACE = -2,  /* a workspace was given that is smaller than picospec_workspace_bytes() says, or misaligned */
    PICOSPEC_EDTYPE = -3,      /* dtype is neither PICOSPEC_F32 nor PICOSPEC_BF16 */
    PICOSPEC_EHIP = -4,        /* a HIP runtime call (launch, attribute) failed */
    PICOSPEC_EUNSUPPORTED = -5,/* k or V beyond the limits reported by picospec_limit() */
    PICOSPEC_ESCRATCH = -6     /* picospec_verify_sample_static: the rows' segment table exceeds the library's fixed array */
};

/* bits of flags[b] */
enum {
    PICOSPEC_FLAG_TOKEN_NOT_IN_SUPPORT = 1u, /* a drafted token was absent from its compressed row: treated as q = 0 (accepted) */
    PICOSPEC_FLAG_NONFINITE = 2u,            /* a target row's log-sum-exp is not finite */
    PICOSPEC_FLAG_RESIDUAL_EMPTY = 4u,       /* residual mass <= 0: the token was drawn from P itself */
    PICOSPEC_FLAG_BAD_INPUT = 8u             /* token id outside [0,V) (p = 0: rejected, with or without q_scalar), negative gamma_b,
                                                n_accept outside [0,gamma_b] (clamped) */
};

enum { PICOSPEC_CALL_COMPRESS = 0, PICOSPEC_CALL_SAMPLE_DRAFT = 1, PICOSPEC_CALL_VERIFY = 2, PICOSPEC_CALL_SAMPLE_RESIDUAL = 3,
       PICOSPEC_CALL_COMPRESS_REJECTED = 4, PICOSPEC_CALL_RESAMPLE_SPARSE = 5, PICOSPEC_CALL_ROUND = 6,
       PICOSPEC_CALL_VERIFY_SAMPLE = 7 };
enum { PICOSPEC_LIMIT_MAX_K = 0, PICOSPEC_LIMIT_MAX_V = 1 };

/*
 * Sparse compression (Section 3.3, Eq. 4): for each of n_rows distributions keep the k
 * highest-probability components and their indices.  One streaming pass per row computes the
 * softmax statistics and selects on the stored logits (exact integer order; equal logits -> lower
 * id first; -0.0 ties with +0.0).
 *   logits [n_rows, ld]           in
 *   k      1..min(V, picospec_limit(MAX_K)) slots per row
 *   top_p  <= 0 or >= 1: plain Top-K.  Otherwise count = the smallest prefix of the descending
 *          order whose probability sum reaches top_p, capped at k (a workload setting, not in the paper)
 *   idx [n_rows,k] int32, prob [n_rows,k] fp32, count [n_rows] int32, mass [n_rows] fp32,
 *   lse [n_rows] fp32             out
 *   workspace: unused (picospec_workspace_bytes(PICOSPEC_CALL_COMPRESS, ...) is 0); pass NULL.
 */
int picospec_compress(const void* logits, int dtype, int64_t ld, int32_t n_rows, int32_t V,
                      float temperature, int32_t k, float top_p,
                      int32_t* idx, float* prob, int32_t* count, float* mass, float* lse,
                      void* workspace, size_t workspace_bytes, void* stream);

/*
 * The drafter's draw (Section 3.3: the edge drafts a token and records its probability q_i):
 * inverse CDF over the used slots of each row in slot order with weights prob[slot]:
 * tok = idx[first slot whose inclusive cumulative weight exceeds u * sum of weights].
 *   uniforms [n_rows] fp32 in [0,1)   in
 *   tok [n_rows] int32, q_scalar [n_rows] fp32 (nullable) = prob/mass of the drawn slot   out
 */
int picospec_sample_draft(const int32_t* idx, const float* prob, const int32_t* count, const float* mass,
                          int32_t k, int32_t n_rows, const float* uniforms,
                          int32_t* tok, float* q_scalar, void* stream);

/*
 * Parallel verification (Section 3.3; acceptance rule of standard speculative sampling, cited
 * there from Chen et al.): for every target row its softmax statistics; for every draft position
 * p_i = P_i(x_i) and qhat_i; accept_i <=> u_i < min(1, p_i / qhat_i); n_accept[b] = index of the
 * first position not accepted, gamma_b if none.
 *   tgt_logits [n_draft + B, ld]; seq_off [B+1]; draft_tok [n_draft]                         in
 *   q_idx/q_prob [n_draft,k], q_count/q_mass [n_draft]: records from picospec_compress       in
 *   renorm   1: qhat = prob/mass (the distribution picospec_sample_draft draws from; keeps the
 *            emitted tokens distributed exactly as the target for any k)   0: qhat = prob
 *   q_scalar nullable [n_draft]: the scalar q_i the edge recorded and uplinks (Section 3.3); when
 *            given it replaces the sparse lookup and q_idx/q_prob/q_count/q_mass may be NULL
 *   uniforms [n_draft + B]                                                                    in
 *   n_accept [B]; p_tok, q_tok [n_draft] (nullable); flags [B]                                out
 *   tgt_max, tgt_sum, tgt_lse [n_draft + B] fp32: row maximum M of the raw logits,
 *            S = sum exp((z - M)/T), and lse = M/T + ln S (tgt_lse nullable)                  out
 */
int picospec_verify(const void* tgt_logits, int dtype, int64_t ld, int32_t V, float temperature,
                    int32_t B, int32_t n_draft, const int32_t* seq_off, const int32_t* draft_tok,
                    const int32_t* q_idx, const float* q_prob, const int32_t* q_count, const float* q_mass,
                    int32_t k, int renorm, const float* q_scalar, const float* uniforms,
                    int32_t* n_accept, float* p_tok, float* q_tok,
                    float* tgt_max, float* tgt_sum, float* tgt_lse, uint32_t* flags,
                    void* workspace, size_t workspace_bytes, void* stream);

/*
 * Verification of a part of the draft (Section 3.2, Fast Verification: the cloud starts on the
 * positions of a draft that are known and goes on when the rest arrives; Section 3.3 for the test).
 * picospec_verify restricted, per sequence, to the draft positions begin_b <= t < end_b with
 * begin_b = pos_begin[b] and end_b = pos_end[b] (either may be NULL: 0 and gamma_b), in the same row
 * layout: target rows begin_b..end_b are read (row end_b is the one behind the last known position)
 * and their entries of tgt_max, tgt_sum, tgt_lse written; p_tok, q_tok are written for the
 * positions of the range; everything else in those arrays keeps what an earlier call left there.
 *   n_accept[b] = first rejected position of the range, else end_b
 *   flags[b]    = the conditions met in this range (BAD_INPUT also for a range outside
 *                 0 <= begin_b <= end_b <= gamma_b, which is clamped)
 * Consecutive ranges compose: with n' from an earlier call over [begin', end') and n from this one
 * over [end', end), the sequence's first rejection is n' if n' < end', else n.
 *   gamma_max  host value >= every gamma_b (<= n_draft): the launch is (gamma_max + 1) x B workgroups,
 *              B <= 65535
 */
int picospec_verify_range(const void* tgt_logits, int dtype, int64_t ld, int32_t V, float temperature,
                          int32_t B, int32_t n_draft, const int32_t* seq_off, const int32_t* draft_tok,
                          const int32_t* q_idx, const float* q_prob, const int32_t* q_count, const float* q_mass,
                          int32_t k, int renorm, const float* q_scalar, const float* uniforms,
                          const int32_t* pos_begin, const int32_t* pos_end, int32_t gamma_max,
                          int32_t* n_accept, float* p_tok, float* q_tok,
                          float* tgt_max, float* tgt_sum, float* tgt_lse, uint32_t* flags,
                          void* workspace, size_t workspace_bytes, void* stream);

/*
 * Correction / bonus token (Section 3.3: norm(max(0, P_j(x) - Q_j(x)))): for sequence b with
 * j = n_accept[b], r(x) = max(0, P_j(x) - qhat_j(x)) with qhat = 0 off the record's support, and
 * the empty record when j = gamma_b (bonus token ~ P).  R = sum_x r(x);
 * out_tok[b] = first x (ascending id) whose inclusive cumulative r exceeds u*R.
 *   tgt_max, tgt_sum [n_draft + B]: from picospec_verify                                      in
 *   out_tok [B] int32, resid_mass [B] fp32 (= R; 0 with PICOSPEC_FLAG_RESIDUAL_EMPTY), flags [B]   out
 */
int picospec_sample_residual(const void* tgt_logits, int dtype, int64_t ld, int32_t V, float temperature,
                             int32_t B, int32_t n_draft, const int32_t* seq_off, const int32_t* n_accept,
                             const float* tgt_max, const float* tgt_sum,
                             const int32_t* q_idx, const float* q_prob, const int32_t* q_count, const float* q_mass,
                             int32_t k, int renorm, const float* uniforms,
                             int32_t* out_tok, float* resid_mass, uint32_t* flags,
                             void* workspace, size_t workspace_bytes, void* stream);

/*
 * ---- The paper's own direction of the sparse record (Section 3.3, last part) -------------------
 * The edge uplinks the scalars q_1..q_gamma (picospec_verify with q_scalar), the cloud verifies,
 * and only on a rejection at position j it sends the Top-K record of the TARGET distribution P_j
 * (Eq. 4); the edge then resamples locally from norm(max(0, P_j - Q_j)) with its own dense Q_j.
 * The three calls below are that downlink; the calls above compress the draft side instead.
 */

/*
 * Softmax statistics of n_rows rows (max, sum of exp((z - max)/T), log-sum-exp): what
 * picospec_verify computes for the target rows, offered for the edge's dense draft rows.
 *   row_max, row_sum [n_rows] out; row_lse [n_rows] out, may be NULL.
 */
int picospec_row_stats(const void* logits, int dtype, int64_t ld, int32_t n_rows, int32_t V, float temperature,
                       float* row_max, float* row_sum, float* row_lse, void* stream);

/*
 * The downlink record (Eq. 4): picospec_compress of ONE target row per sequence, the row of its
 * first rejected position (or of the bonus position when every draft token was accepted):
 * target row seq_off[b] + b + n_accept[b], with n_accept[b] clamped to 0..gamma_b.
 *   tgt_logits [n_draft + B, ld] in;  seq_off [B+1], n_accept [B] in
 *   idx, prob [B,k], count, mass, lse [B] out (record b belongs to sequence b)
 */
int picospec_compress_rejected(const void* tgt_logits, int dtype, int64_t ld, int32_t V, float temperature,
                               int32_t B, int32_t n_draft, const int32_t* seq_off, const int32_t* n_accept,
                               int32_t k, float top_p,
                               int32_t* idx, float* prob, int32_t* count, float* mass, float* lse,
                               void* workspace, size_t workspace_bytes, void* stream);

/*
 * Local resampling at the edge (Section 3.3: norm(max(0, P_j - Q_j))) from the downlink record.
 * The target is known only through the record: Pt(id_s) = p_prob[s] (renorm 0, the values as
 * sent) or p_prob[s] / p_mass (renorm 1), 0 elsewhere, so the residual lives on the record's slots:
 *   r_s = max(0, Pt(id_s) - Q_j(id_s)),  Q_j(x) = exp((z_d[x] - draft_max) / T) / draft_sum of dense
 *   draft row seq_off[b] + j, j = n_accept[b];  j = gamma_b: r_s = Pt(id_s) (bonus token).
 * out_tok[b] = id of the first slot, in slot order, whose inclusive cumulative r exceeds u * R,
 * R = sum r_s, u = uniforms[seq_off[b] + b + gamma_b]; resid_mass[b] = R.  R <= 0: the draw comes
 * from Pt itself, resid_mass = 0, flag RESIDUAL_EMPTY.  An empty record gives out_tok = -1.
 * With k < V this draw is biased against the exact residual by exactly the residual mass that
 * lies off the record (total variation 1 - R_K / R for renorm 0); with k = V it is exact.
 *   draft_logits [n_draft, ld] in; draft_max, draft_sum [n_draft] in (picospec_row_stats)
 *   p_idx, p_prob [B,k], p_count, p_mass [B] in (picospec_compress_rejected); uniforms [n_draft + B] in
 *   out_tok, resid_mass, flags [B] out (BAD_INPUT: n_accept outside 0..gamma_b, an id outside [0,V))
 */
int picospec_resample_sparse(const void* draft_logits, int dtype, int64_t ld, int32_t V, float temperature,
                             int32_t B, int32_t n_draft, const int32_t* seq_off, const int32_t* n_accept,
                             const float* draft_max, const float* draft_sum,
                             const int32_t* p_idx, const float* p_prob, const int32_t* p_count, const float* p_mass,
                             int32_t k, int renorm, const float* uniforms,
                             int32_t* out_tok, float* resid_mass, uint32_t* flags,
                             void* workspace, size_t workspace_bytes, void* stream);

/*
 * One call for a whole round with the draft side compressed (Section 3.3): picospec_compress of the draft
 * rows, picospec_verify with the records, picospec_sample_residual, with the same arguments, outputs and
 * flags as the three calls (verify_flags as picospec_verify's, residual_flags as picospec_sample_residual's).
 * The drafted tokens must be known beforehand (in a deployment they come from picospec_sample_draft on an
 * earlier compress of the same rows; the records written here are then the same ones).
 * Acceptance and residual draw of a sequence run in one workgroup (one launch, the rejected position never
 * leaves it).  Rounds of up to 512 rows (draft + target) also stream the draft and the target rows in one
 * launch (two launches in all instead of four): such rounds are bound by the launches' serial parts, not by
 * bandwidth.  Larger rounds keep the two streaming launches of the separate calls (three in all).
 * The records are the same bit for bit in both schedules; the target statistics of the two-launch schedule are
 * summed in another order, so what depends on them agrees with the separate calls to rounding.
 * workspace (optional): picospec_workspace_bytes(PICOSPEC_CALL_ROUND, ...) bytes; either schedule then leaves the
 * target rows' segment table there (in a layout of its own: the table of one call of picospec_round serves that call
 * only) and draws from it without a second pass over the target row.
 */
int picospec_round(const void* draft_logits, const void* tgt_logits, int dtype, int64_t ld_draft, int64_t ld_tgt,
                   int32_t V, float temperature, int32_t B, int32_t n_draft, const int32_t* seq_off,
                   const int32_t* draft_tok, int32_t k, float top_p, int renorm, const float* uniforms,
                   int32_t* q_idx, float* q_prob, int32_t* q_count, float* q_mass, float* q_lse,
                   int32_t* n_accept, float* p_tok, float* q_tok,
                   float* tgt_max, float* tgt_sum, float* tgt_lse, uint32_t* verify_flags,
                   int32_t* out_tok, float* resid_mass, uint32_t* residual_flags,
                   void* workspace, size_t workspace_bytes, void* stream);

/*
 * Verification and draw in one call on records that exist (Section 3.3: the cloud's part of a round when the drafter
 * has compressed its distributions, drawn from them and sent records and tokens): picospec_verify followed by
 * picospec_sample_residual, with the same arguments, outputs and flags, as two launches (the statistics of the target
 * rows; acceptance and draw of a sequence in one workgroup, so the rejected position never leaves it).  Nothing is
 * compressed here: unlike picospec_round the call takes the records the drafted tokens were drawn from.
 */
int picospec_verify_sample(const void* tgt_logits, int dtype, int64_t ld, int32_t V, float temperature,
                           int32_t B, int32_t n_draft, const int32_t* seq_off, const int32_t* draft_tok,
                           const int32_t* q_idx, const float* q_prob, const int32_t* q_count, const float* q_mass,
                           int32_t k, int renorm, const float* uniforms,
                           int32_t* n_accept, float* p_tok, float* q_tok,
                           float* tgt_max, float* tgt_sum, float* tgt_lse, uint32_t* verify_flags,
                           int32_t* out_tok, float* resid_mass, uint32_t* residual_flags,
                           void* workspace, size_t workspace_bytes, void* stream);

/*
 * picospec_verify_sample for callers that cannot allocate device memory and have none to spare for a workspace: code
 * under HIP graph capture, tight serving loops, harnesses that forbid allocation.  Same arguments (without the
 * workspace), same kernels, same outputs bit for bit as picospec_verify_sample with a workspace; the target rows'
 * segment table lives in a fixed array of picospec_static_scratch_bytes() bytes (8 MiB) inside the library's device
 * image, one copy per GPU, held until the process ends.  The call allocates and frees nothing.
 *   - Sizes: picospec_workspace_bytes(PICOSPEC_CALL_VERIFY_SAMPLE, dtype, n_draft + B, V, k) must not exceed the array
 *     (about 6,500 target rows at V = 152 K fp32, 13,000 bf16), else PICOSPEC_ESCRATCH and nothing is launched.
 *   - Every call on a GPU uses that GPU's one array: calls that overlap in time on one GPU (different streams, or
 *     different threads) race on it; calls on one stream are ordered and safe.  The array keeps the last call's table;
 *     nothing in it has to be cleared (every entry that is read is written first by the same call).
 *   - The first call on a device asks the runtime for the array's address there (no allocation), with that device current.
 */
int picospec_verify_sample_static(const void* tgt_logits, int dtype, int64_t ld, int32_t V, float temperature,
                                  int32_t B, int32_t n_draft, const int32_t* seq_off, const int32_t* draft_tok,
                                  const int32_t* q_idx, const float* q_prob, const int32_t* q_count, const float* q_mass,
                                  int32_t k, int renorm, const float* uniforms,
                                  int32_t* n_accept, float* p_tok, float* q_tok,
                                  float* tgt_max, float* tgt_sum, float* tgt_lse, uint32_t* verify_flags,
                                  int32_t* out_tok, float* resid_mass, uint32_t* residual_flags, void* stream);

/* host: size of the fixed array behind picospec_verify_sample_static, in bytes. */
int64_t picospec_static_scratch_bytes(void);

/*
 * ---- Wire messages of a round (Section 3.3) ----------------------------------------------------
 * Uplink (edge -> cloud): the drafted tokens and only their own probabilities q_1..q_gamma, 8 bytes
 * per drafted token with fp32 probabilities (48 bytes at gamma = 6).  Downlink (cloud -> edge): per
 * sequence the number of accepted tokens and, only if a draft token was rejected, the Top-K record
 * of Eq. 4 (8 bytes per entry; 80 bytes at K = 10), else the token the cloud decided itself.
 * The paper names a zero-copy serialisation but prints no byte layout; this is the library's.  Every
 * block is naturally aligned behind a fixed header, so a receiver addresses the arrays in place.
 * All fields little-endian; probabilities fp32, or fp16 / bf16 rounded to nearest even:
 *
 *   downlink   0  u16 magic 0x5350   2  u8 version (1)   3  u8 prob_format   4  u32 B
 *              8  B entries of 8 bytes: u16 n_accept, u16 count, i32 token
 *                 (count entries of this sequence follow below; token = -1 unless count = 0)
 *              .. int32 ids[total], total = sum of count, sequences in order
 *              .. prob[total] in prob_format, then zero bytes up to a multiple of 4
 *   uplink     0  u16 magic 0x5351   2  u8 version (1)   3  u8 prob_format   4  u32 B
 *              8  u16 gamma[B], zero bytes up to a multiple of 4
 *              .. int32 tok[N], N = sum of gamma;  q[N] in prob_format, zero bytes up to a multiple of 4
 *
 * `wire` is a DEVICE buffer, 4-byte aligned (the caller moves it to and from the NIC or host).
 * status (device, one uint32) receives a bit set of PICOSPEC_WIRE_*; with BAD_HEADER, BAD_BATCH or
 * TRUNCATED an unpacking call writes nothing else.
 */
enum { PICOSPEC_WIRE_FP32 = 0, PICOSPEC_WIRE_FP16 = 1, PICOSPEC_WIRE_BF16 = 2 };
enum {
    PICOSPEC_WIRE_BAD_HEADER = 1u, /* magic, version or prob_format not as expected */
    PICOSPEC_WIRE_BAD_BATCH = 2u,  /* B in the message differs from the caller's */
    PICOSPEC_WIRE_CLAMPED = 4u,    /* a record longer than the receiver's k (front kept), or more positions than n_max */
    PICOSPEC_WIRE_TRUNCATED = 8u   /* the buffer is shorter than the message (unpack) or than the message needs (pack) */
};

/* host: size of the largest downlink message for B sequences with records of k slots / exact size of
 * the uplink message for B sequences and n_draft positions; -1 for arguments out of range. */
int64_t picospec_downlink_bytes_max(int32_t B, int32_t k, int prob_format);
int64_t picospec_uplink_bytes(int32_t B, int32_t n_draft, int prob_format);

/*
 * Packs the downlink message of a round.  Sequence b carries its record (idx/prob/count row b, as
 * picospec_compress_rejected wrote it) iff n_accept[b] < gamma_b; every other sequence carries
 * token[b] (the bonus token, or a correction the cloud drew itself), -1 if token is NULL.
 * idx, prob and count may all be NULL: tokens only, 8 bytes per sequence.
 *   seq_off [B+1], n_accept [B] in; token [B] in, nullable; idx, prob [B,k], count [B] in, nullable together
 *   wire out, wire_capacity bytes; *wire_bytes (device int64) = size of the message;
 *   *status = 0, or TRUNCATED when the message exceeds wire_capacity (then only wire_bytes and status are written)
 * Each workgroup sums the counts in front of its sequence: O(B) per sequence, meant for batch sizes.
 */
int picospec_pack_downlink(int32_t B, const int32_t* seq_off, const int32_t* n_accept, const int32_t* token,
                           const int32_t* idx, const float* prob, const int32_t* count, int32_t k,
                           int prob_format, void* wire, int64_t wire_capacity,
                           int64_t* wire_bytes, uint32_t* status, void* stream);

/*
 * Unpacks a downlink message of wire_bytes bytes (host value: the received length) into the record
 * layout picospec_resample_sparse takes: idx/prob [B,k] (unused slots -1 / 0, probabilities widened
 * to fp32 exactly), count, mass = sum of the received probabilities; n_accept and token [B].
 */
int picospec_unpack_downlink(const void* wire, int64_t wire_bytes, int32_t B, int32_t k,
                             int32_t* n_accept, int32_t* token, int32_t* idx, float* prob, int32_t* count,
                             float* mass, uint32_t* status, void* stream);

/*
 * Packs the uplink message: gamma_b = seq_off[b+1] - seq_off[b] (<= 65535), the drafted tokens and
 * their probabilities (q_scalar of picospec_sample_draft).  wire_capacity >= picospec_uplink_bytes().
 */
int picospec_pack_uplink(int32_t B, int32_t n_draft, const int32_t* seq_off, const int32_t* draft_tok,
                         const float* q_scalar, int prob_format, void* wire, int64_t wire_capacity,
                         int64_t* wire_bytes, void* stream);

/*
 * Unpacks an uplink message: seq_off [B+1] (from 0), draft_tok and q_scalar (fp32) for at most n_max
 * positions.  Sequences are kept whole: the first that does not fit n_max, and all behind it, come
 * out empty (CLAMPED).  seq_off, draft_tok, q_scalar then feed picospec_verify.
 */
int picospec_unpack_uplink(const void* wire, int64_t wire_bytes, int32_t B, int32_t n_max,
                           int32_t* seq_off, int32_t* draft_tok, float* q_scalar, uint32_t* status, void* stream);

/*
 * host: memory-safety check of the streaming row loads.  For a row of V elements whose first byte lies
 * misalign_bytes (0..15, a multiple of the element size) above a 16-byte boundary, the end (exclusive), in bytes
 * from the row's first byte, of the highest byte that the row loads of picospec_compress (which_call =
 * PICOSPEC_CALL_COMPRESS; also picospec_compress_rejected and picospec_round) or of picospec_sample_residual
 * (PICOSPEC_CALL_SAMPLE_RESIDUAL) can address, look-ahead loads behind the row included.  The library guarantees
 * that this lies inside the aligned 16-byte block that holds the row's last byte (a block that holds a valid byte
 * cannot leave that byte's page); the function evaluates the kernels' own addressing rule over every lane, so a test
 * can hold the library to it without a GPU.  The rule rests on one property of the device's buffer loads, which
 * picospec_check_device() tests.  -1 for arguments out of range.
 */
int64_t picospec_max_load_byte(int which_call, int dtype, int32_t V, int32_t misalign_bytes);

/*
 * Device self-check (enqueues two small kernels): does a raw buffer load of the current device range-check the
 * way the row kernels assume (scalar offset + per-lane offset + 16 <= descriptor size, else the lane reads zero and
 * touches no memory)?  *status (device uint32) = 0 if so, else one bit per failed probe.  workspace: >= 64 KiB of
 * device memory on a 16-byte boundary, overwritten; every address the probes form lies inside it.
 */
int picospec_check_device(void* workspace, size_t workspace_bytes, uint32_t* status, void* stream);

/*
 * Measurement aid (enqueues one single-wave kernel of about 10 microseconds): ticks[0] = shader-clock cycles and
 * ticks[1] = ticks of the constant 100 MHz wall clock over the same fixed loop, so that 100 * ticks[0] / ticks[1] is the
 * shader clock in MHz that the device runs at when the stream reaches this point.  The kernels of the hot path that are
 * bound by the vector ALU follow that clock; after a pause in the work it dips for some tens of milliseconds.
 *   ticks  device, two uint64 on an 8-byte boundary   out
 */
int picospec_probe_clock(uint64_t* ticks, void* stream);

/* host: bytes of the optional device workspace of the given call for (dtype, rows, V, k), rows = n_draft + B for the
 * calls that take target rows; 0 if the call has no use for one. */
size_t picospec_workspace_bytes(int which_call, int dtype, int32_t rows, int32_t V, int32_t k);

/* host: largest supported k (PICOSPEC_LIMIT_MAX_K) or V (PICOSPEC_LIMIT_MAX_V); -1 for an unknown id. */
int64_t picospec_limit(int which);

/* host: static string for a return code. */
const char* picospec_strerror(int code);

/* host: ABI version, major*1000 + minor. */
int picospec_version(void);

#ifdef __cplusplus
}
#endif
#endif /* PICOSPEC_H */
