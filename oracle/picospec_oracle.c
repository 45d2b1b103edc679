/*
 * PicoSpec separate rejection sampling with sparse compression -- CPU oracle.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain, fp64 definition of
 * what the GPU path has to compute.  It shares no code, header, table or
 * helper with the HIP library and must never be called from the product path.
 *
 * What it follows (paper sections, by name):
 *   - Sparse Top-K compression of a vocabulary distribution: Section 3.3,
 *     Eq. 4 (keep the K largest-probability components with their indices;
 *     8 bytes per record = int32 id + fp32 prob).
 *   - Parallel verification with the acceptance test min(1, p/q) of standard
 *     speculative sampling: Section 3.3 (second paragraph) and the rule of
 *     Chen et al. cited in Section 2.1.
 *   - Correction token drawn from norm(max(0, P_j - Q_j)): Section 3.3; both
 *     with the draft side compressed (dense target on the verifier) and, as the
 *     paper ships it, with the target's Top-K record sent to the edge, which
 *     resamples locally against its dense draft distribution.
 *   - Bonus token when every draft token is accepted: implied by Table 1's
 *     accepted lengths exceeding the draft length (Section 4.1 / 4.2).
 *
 * Arithmetic: stored logits (fp32 or bf16) are widened exactly to double; all
 * sums run in vocabulary-index (or slot) order with plain loops; libm exp/log.
 * There is no blocking, fusion or reordering.  The only library primitive is
 * qsort for the ordering step.
 *
 * Parity pins live in tests/test_oracle_*.py (library log-sum-exp, lexsort
 * top-k, dense textbook speculative sampling for k = V, accept-all for equal
 * distributions, V = 8 chi-square, closed-form residual mass, brute force).
 * The cumulative-probability ("top-p") count rule is not in the paper (it is
 * a workload setting); it is pinned against a numpy cumsum only.
 *
 * The one OpenMP pragma per entry point spreads independent rows/sequences
 * over host threads for the timed baseline; it does not change any result.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { ORACLE_F32 = 0, ORACLE_BF16 = 1 };

enum {
    ORACLE_FLAG_TOKEN_NOT_IN_SUPPORT = 1u, /* drafted token absent from the compressed draft row */
    ORACLE_FLAG_NONFINITE = 2u,            /* a log-sum-exp came out non-finite */
    ORACLE_FLAG_RESIDUAL_EMPTY = 4u        /* residual mass <= 0: fell back to the target itself */
};

static double logit_at(const void *base, int dtype, int64_t i)
{
    if (dtype == ORACLE_F32) {
        return (double)((const float *)base)[i];
    } else {
        uint32_t bits = (uint32_t)((const uint16_t *)base)[i] << 16; /* bf16 = top half of fp32 */
        float f;
        memcpy(&f, &bits, sizeof f);
        return (double)f;
    }
}

/* log-sum-exp of one row of logits at temperature T: y = z/T, m = max y,
 * s = sum exp(y - m), lse = m + ln s.  P(x) = exp(y_x - lse). */
static double row_lse(const void *row, int dtype, int32_t V, double T)
{
    double m = -INFINITY;
    for (int32_t x = 0; x < V; ++x) {
        double y = logit_at(row, dtype, x) / T;
        if (y > m) m = y;
    }
    double s = 0.0;
    for (int32_t x = 0; x < V; ++x) s += exp(logit_at(row, dtype, x) / T - m);
    return m + log(s);
}

typedef struct {
    double z;
    int32_t x;
} ranked_t;

/* value descending (compared as numbers, so -0.0 ties with +0.0), index ascending */
static int ranked_cmp(const void *a, const void *b)
{
    const ranked_t *p = (const ranked_t *)a, *q = (const ranked_t *)b;
    if (p->z > q->z) return -1;
    if (p->z < q->z) return 1;
    return (p->x > q->x) - (p->x < q->x);
}

/*
 * Sparse compression of n_rows distributions (Section 3.3, Eq. 4).
 *   logits   [n_rows, ld]  stored dtype; row r starts at element r*ld
 *   k        slots per row (1..V); top_p in (0,1) switches to "smallest prefix of the
 *            descending order whose probability reaches top_p, capped at k"
 *   idx      [n_rows,k]  vocabulary ids in (value desc, id asc) order, -1 in unused slots
 *   prob     [n_rows,k]  P(id) itself (raw, not renormalised), 0 in unused slots
 *   count    [n_rows]    used slots
 *   mass     [n_rows]    sum of the kept prob, slot order
 *   lse      [n_rows]
 *   topp_margin [n_rows] nullable: distance of the top-p threshold from the two
 *            cumulative sums that decide count (infinity in plain top-k mode)
 * Selection compares the stored logits, never computed probabilities.
 */
int oracle_compress(const void *logits, int dtype, int64_t ld, int32_t n_rows, int32_t V,
                    double T, int32_t k, double top_p,
                    int32_t *idx, double *prob, int32_t *count, double *mass, double *lse,
                    double *topp_margin)
{
    if (!logits || V < 1 || k < 1 || k > V || !(T > 0.0) || ld < V) return -1;
    const size_t esz = dtype == ORACLE_F32 ? 4 : 2;
    int failed = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int32_t r = 0; r < n_rows; ++r) {
        const void *row = (const char *)logits + (size_t)r * (size_t)ld * esz;
        ranked_t *order = (ranked_t *)malloc((size_t)V * sizeof *order);
        if (!order) { failed = 1; continue; }
        double l = row_lse(row, dtype, V, T);
        for (int32_t x = 0; x < V; ++x) {
            order[x].z = logit_at(row, dtype, x);
            order[x].x = x;
        }
        qsort(order, (size_t)V, sizeof *order, ranked_cmp);
        int32_t c = k;
        double margin = INFINITY;
        if (top_p > 0.0 && top_p < 1.0) {
            double cum = 0.0, prev = 0.0;
            c = k;
            for (int32_t j = 0; j < k; ++j) {
                prev = cum;
                cum += exp(order[j].z / T - l);
                if (cum >= top_p) { c = j + 1; break; }
            }
            margin = fmin(fabs(cum - top_p), fabs(prev - top_p));
        }
        double ms = 0.0;
        for (int32_t j = 0; j < k; ++j) {
            if (j < c) {
                idx[(size_t)r * k + j] = order[j].x;
                prob[(size_t)r * k + j] = exp(order[j].z / T - l);
                ms += prob[(size_t)r * k + j];
            } else {
                idx[(size_t)r * k + j] = -1;
                prob[(size_t)r * k + j] = 0.0;
            }
        }
        count[r] = c;
        mass[r] = ms;
        lse[r] = l;
        if (topp_margin) topp_margin[r] = margin;
        free(order);
    }
    return failed ? -2 : 0;
}

/* Draft probability as used by the test: prob/mass (renorm) or prob itself. */
static double qhat_of_slot(const double *prob, double mass, int renorm, int32_t s)
{
    return renorm ? prob[s] / mass : prob[s];
}

/*
 * Edge-side draw of the drafted token from the compressed draft distribution
 * (Section 3.3: the edge drafts and records q_i).  Inverse CDF over the used
 * slots in slot order with weights prob[s]: token = first slot whose inclusive
 * cumulative weight exceeds u * (sum of weights).  (Identical for renorm 0/1.)
 *   tok [n_rows], slot [n_rows] (nullable), cdf_margin [n_rows] (nullable):
 *   relative distance of u*total from the nearer edge of the chosen slot's interval.
 */
int oracle_sample_draft(const int32_t *idx, const double *prob, const int32_t *count, int32_t k,
                        int32_t n_rows, const float *uniforms,
                        int32_t *tok, int32_t *slot, double *cdf_margin)
{
    for (int32_t r = 0; r < n_rows; ++r) {
        const double *p = prob + (size_t)r * k;
        int32_t c = count[r];
        double total = 0.0;
        for (int32_t s = 0; s < c; ++s) total += p[s];
        double target = (double)uniforms[r] * total;
        double cum = 0.0, prev = 0.0;
        int32_t pick = -1;
        for (int32_t s = 0; s < c; ++s) {
            prev = cum;
            cum += p[s];
            if (cum > target) { pick = s; break; }
        }
        if (pick < 0) { /* rounding: take the last slot with weight */
            pick = c - 1;
            while (pick > 0 && !(p[pick] > 0.0)) --pick;
            prev = cum;
        }
        tok[r] = idx[(size_t)r * k + pick];
        if (slot) slot[r] = pick;
        if (cdf_margin) cdf_margin[r] = fmin(fabs(target - prev), fabs(cum - target)) / total;
    }
    return 0;
}

/*
 * Verification of B sequences (Section 3.3; rule of standard speculative sampling).
 * Sequence b owns draft rows seq_off[b]..seq_off[b+1]-1 (gamma_b of them) and the
 * gamma_b+1 target rows seq_off[b]+b .. seq_off[b+1]+b (last = bonus position).
 * uniforms are indexed like target rows.
 *   accept_i  <=>  u_i < min(1, p_i / qhat_i);   n_accept[b] = first i not accepted, else gamma_b
 *   q_scalar  nullable [N]: the edge's recorded scalar q_i; overrides the sparse lookup
 *   p_tok, q_tok [N]; tgt_lse [N+B]; flags [B]; margin [N] = |u - p/q| / (p/q)
 * Verification of a part of the draft (Section 3.2, Fast Verification: the cloud starts on the
 * positions that are known and goes on when the rest arrives): pos_begin / pos_end, nullable [B],
 * restrict sequence b to its positions begin_b <= t < end_b (defaults 0 and gamma_b; clamped to
 * that range).  Target rows begin_b..end_b are read (row end_b is the one behind the last known
 * position); entries of the outputs for other rows and positions are left as they are;
 * n_accept[b] = first rejected position in the range, else end_b.
 */
int oracle_verify(const void *tgt_logits, int dtype, int64_t ld, int32_t V, double T,
                  int32_t B, const int32_t *seq_off, const int32_t *draft_tok,
                  const int32_t *q_idx, const double *q_prob, const int32_t *q_count,
                  const double *q_mass, int32_t k, int renorm,
                  const double *q_scalar, const float *uniforms,
                  int32_t *n_accept, double *p_tok, double *q_tok, double *tgt_lse,
                  uint32_t *flags, double *margin,
                  const int32_t *pos_begin, const int32_t *pos_end)
{
    if (!tgt_logits || V < 1 || !(T > 0.0) || ld < V || B < 0) return -1;
    const size_t esz = dtype == ORACLE_F32 ? 4 : 2;
#pragma omp parallel for schedule(dynamic, 1)
    for (int32_t b = 0; b < B; ++b) {
        int32_t d0 = seq_off[b], gamma = seq_off[b + 1] - seq_off[b];
        int64_t t0 = (int64_t)d0 + b;
        uint32_t fl = 0;
        int32_t begin = pos_begin ? pos_begin[b] : 0, end = pos_end ? pos_end[b] : gamma;
        if (end < 0) end = 0;
        if (end > gamma) end = gamma;
        if (begin < 0) begin = 0;
        if (begin > end) begin = end;
        int32_t first_reject = end;
        for (int32_t t = begin; t <= end; ++t) {
            const void *row = (const char *)tgt_logits + (size_t)(t0 + t) * (size_t)ld * esz;
            double l = row_lse(row, dtype, V, T);
            tgt_lse[t0 + t] = l;
            if (!isfinite(l)) fl |= ORACLE_FLAG_NONFINITE;
            if (t == end) break; /* the row behind the last position (the bonus row when end = gamma): statistics only */
            int32_t i = d0 + t, x = draft_tok[i];
            double p = exp(logit_at(row, dtype, x) / T - l);
            double q;
            if (q_scalar) {
                q = q_scalar[i];
            } else {
                q = 0.0;
                int found = 0;
                for (int32_t s = 0; s < q_count[i]; ++s) {
                    if (q_idx[(size_t)i * k + s] == x) {
                        q = qhat_of_slot(q_prob + (size_t)i * k, q_mass[i], renorm, s);
                        found = 1;
                        break;
                    }
                }
                if (!found) fl |= ORACLE_FLAG_TOKEN_NOT_IN_SUPPORT;
            }
            double ratio = q > 0.0 ? p / q : INFINITY;
            double u = (double)uniforms[t0 + t];
            int accept = u < fmin(1.0, ratio);
            if (!accept && t < first_reject) first_reject = t;
            if (p_tok) p_tok[i] = p;
            if (q_tok) q_tok[i] = q;
            if (margin) margin[i] = isfinite(ratio) && ratio > 0.0 ? fabs(u - ratio) / ratio : INFINITY;
        }
        n_accept[b] = first_reject;
        if (flags) flags[b] = fl;
    }
    return 0;
}

/*
 * Correction / bonus token (Section 3.3: norm(max(0, P_j - Q_j))).
 * For sequence b: j = n_accept[b]; target row t = seq_off[b]+b+j; the draft row
 * seq_off[b]+j supplies qhat on its sparse support (empty when j = gamma_b, which
 * makes the draw the bonus token from P).  r(x) = max(0, P(x) - qhat(x)),
 * R = sum r;  token = first x whose inclusive cumulative r exceeds u*R with
 * u = uniforms[seq_off[b]+b+gamma_b] (the sequence's last target-row slot).
 *   out_tok, resid_mass, flags [B]; cdf_margin [B] nullable, relative to R.
 */
int oracle_sample_residual(const void *tgt_logits, int dtype, int64_t ld, int32_t V, double T,
                           int32_t B, const int32_t *seq_off, const int32_t *n_accept,
                           const double *tgt_lse,
                           const int32_t *q_idx, const double *q_prob, const int32_t *q_count,
                           const double *q_mass, int32_t k, int renorm,
                           const float *uniforms,
                           int32_t *out_tok, double *resid_mass, uint32_t *flags,
                           double *cdf_margin)
{
    if (!tgt_logits || V < 1 || !(T > 0.0) || ld < V || B < 0) return -1;
    const size_t esz = dtype == ORACLE_F32 ? 4 : 2;
    int failed = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int32_t b = 0; b < B; ++b) {
        int32_t d0 = seq_off[b], gamma = seq_off[b + 1] - seq_off[b];
        int32_t j = n_accept[b];
        int64_t t = (int64_t)d0 + b + j;
        const void *row = (const char *)tgt_logits + (size_t)t * (size_t)ld * esz;
        double l = tgt_lse[t];
        double *r = (double *)malloc((size_t)V * sizeof *r);
        if (!r) { failed = 1; continue; }
        for (int32_t x = 0; x < V; ++x) r[x] = exp(logit_at(row, dtype, x) / T - l); /* P(x) */
        uint32_t fl = 0;
        if (j < gamma) {
            int32_t i = d0 + j;
            for (int32_t s = 0; s < q_count[i]; ++s) {
                int32_t x = q_idx[(size_t)i * k + s];
                double q = qhat_of_slot(q_prob + (size_t)i * k, q_mass[i], renorm, s);
                double d = r[x] - q;
                r[x] = d > 0.0 ? d : 0.0;
            }
        }
        double R = 0.0;
        for (int32_t x = 0; x < V; ++x) R += r[x];
        if (!(R > 0.0)) { /* P == qhat numerically: draw from P */
            fl |= ORACLE_FLAG_RESIDUAL_EMPTY;
            for (int32_t x = 0; x < V; ++x) r[x] = exp(logit_at(row, dtype, x) / T - l);
            R = 0.0;
            for (int32_t x = 0; x < V; ++x) R += r[x];
        }
        double target = (double)uniforms[(int64_t)d0 + b + gamma] * R;
        double cum = 0.0, prev = 0.0;
        int32_t pick = -1;
        for (int32_t x = 0; x < V; ++x) {
            prev = cum;
            cum += r[x];
            if (cum > target) { pick = x; break; }
        }
        if (pick < 0) { /* rounding: last x with r(x) > 0 */
            pick = V - 1;
            while (pick > 0 && !(r[pick] > 0.0)) --pick;
            prev = cum;
        }
        out_tok[b] = pick;
        resid_mass[b] = (fl & ORACLE_FLAG_RESIDUAL_EMPTY) ? 0.0 : R;
        if (flags) flags[b] = fl;
        if (cdf_margin) cdf_margin[b] = fmin(fabs(target - prev), fabs(cum - target)) / R;
        free(r);
    }
    return failed ? -2 : 0;
}

/*
 * Edge-side local resampling on the sparse downlink (Section 3.3, last part: on a rejection at
 * position j the cloud sends only the Top-K components of the target distribution, Eq. 4, and the
 * edge draws the corrected token from norm(max(0, P_j - Q_j)) with its own, dense, Q_j).
 * For sequence b: j = n_accept[b]; record b holds (id_s, prob_s), s < count[b], of target row
 * seq_off[b]+b+j.  The edge knows the target only through the record: Pt(id_s) = prob_s
 * (renorm 0, the values as sent) or prob_s/mass (renorm 1), Pt = 0 elsewhere, so the residual
 * lives on the record's slots:
 *     r_s = max(0, Pt(id_s) - Q_j(id_s)),   Q_j(x) = exp(z_d[x]/T - lse_d) of dense draft row seq_off[b]+j;
 *     j = gamma_b (every draft token accepted): no Q, r_s = Pt(id_s) (the bonus token).
 * R = sum r_s; token = id of the first slot, in slot order, whose inclusive cumulative r exceeds u*R,
 * u = uniforms[seq_off[b]+b+gamma_b].  R <= 0: draw from Pt itself and flag it.
 *   out_tok, resid_mass, flags [B]; cdf_margin [B] nullable (relative to the total weight);
 *   weights [B,k] nullable: the r_s actually drawn from (0 in unused slots).
 */
int oracle_resample_sparse(const void *draft_logits, int dtype, int64_t ld, int32_t V, double T,
                           int32_t B, const int32_t *seq_off, const int32_t *n_accept,
                           const int32_t *p_idx, const double *p_prob, const int32_t *p_count,
                           const double *p_mass, int32_t k, int renorm,
                           const float *uniforms,
                           int32_t *out_tok, double *resid_mass, uint32_t *flags,
                           double *cdf_margin, double *weights)
{
    if (V < 1 || !(T > 0.0) || ld < V || B < 0 || k < 1) return -1;
    const size_t esz = dtype == ORACLE_F32 ? 4 : 2;
    int failed = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int32_t b = 0; b < B; ++b) {
        int32_t d0 = seq_off[b], gamma = seq_off[b + 1] - seq_off[b];
        int32_t j = n_accept[b], c = p_count[b];
        const int32_t *ids = p_idx + (size_t)b * k;
        const double *pp = p_prob + (size_t)b * k;
        double *r = (double *)malloc((size_t)k * sizeof *r);
        if (!r) { failed = 1; continue; }
        uint32_t fl = 0;
        for (int32_t s = 0; s < c; ++s) r[s] = renorm ? pp[s] / p_mass[b] : pp[s]; /* Pt(id_s) */
        if (j < gamma) {
            const void *row = (const char *)draft_logits + (size_t)(d0 + j) * (size_t)ld * esz;
            double l = row_lse(row, dtype, V, T);
            for (int32_t s = 0; s < c; ++s) {
                double q = exp(logit_at(row, dtype, ids[s]) / T - l);
                double d = r[s] - q;
                r[s] = d > 0.0 ? d : 0.0;
            }
        }
        double R = 0.0;
        for (int32_t s = 0; s < c; ++s) R += r[s];
        if (!(R > 0.0)) { /* nothing of the record exceeds Q: draw from the record itself */
            fl |= ORACLE_FLAG_RESIDUAL_EMPTY;
            R = 0.0;
            for (int32_t s = 0; s < c; ++s) { r[s] = renorm ? pp[s] / p_mass[b] : pp[s]; R += r[s]; }
        }
        double target = (double)uniforms[(int64_t)d0 + b + gamma] * R;
        double cum = 0.0, prev = 0.0;
        int32_t pick = -1;
        for (int32_t s = 0; s < c; ++s) {
            prev = cum;
            cum += r[s];
            if (cum > target) { pick = s; break; }
        }
        if (pick < 0) { /* rounding: last slot with weight */
            pick = c - 1;
            while (pick > 0 && !(r[pick] > 0.0)) --pick;
            prev = cum;
        }
        out_tok[b] = c > 0 ? ids[pick] : -1;
        resid_mass[b] = (fl & ORACLE_FLAG_RESIDUAL_EMPTY) ? 0.0 : R;
        if (flags) flags[b] = fl;
        if (cdf_margin) cdf_margin[b] = fmin(fabs(target - prev), fabs(cum - target)) / R;
        if (weights) {
            for (int32_t s = 0; s < k; ++s) weights[(size_t)b * k + s] = s < c ? r[s] : 0.0;
        }
        free(r);
    }
    return failed ? -2 : 0;
}

int oracle_record_bytes(void) { return (int)(sizeof(int32_t) + sizeof(float)); }
