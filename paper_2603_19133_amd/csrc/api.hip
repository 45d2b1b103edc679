// C ABI of the library (include/picospec.h): host-side validation and the ragged-batch dispatch
// onto the gfx950 kernels.  Nothing is launched unless every host-checkable argument is valid.
#include "../../include/picospec.h"

#include <algorithm>
#include <cmath>

#include "kernels.hpp"
#include "rowspan.hpp"

using namespace picospec;

namespace {

bool finite_pos(float t) { return std::isfinite(t) && t > 0.f; }

int check_logits(const void* logits, int dtype, int64_t ld, int64_t rows, int32_t V, float temperature)
{
    if (dtype != PICOSPEC_F32 && dtype != PICOSPEC_BF16) return PICOSPEC_EDTYPE;
    if (rows < 0 || V < 1 || ld < V || !finite_pos(temperature)) return PICOSPEC_EINVAL;
    if (V > kMaxV) return PICOSPEC_EUNSUPPORTED;
    if (rows > 0 && !logits) return PICOSPEC_EINVAL;
    const uintptr_t esz = dtype == PICOSPEC_F32 ? 4 : 2;
    if ((uintptr_t)logits % esz) return PICOSPEC_EINVAL;
    return PICOSPEC_OK;
}

// The workspace is optional: a call that is given none works without it.  One that is too small is an error.
int check_workspace(int which, int dtype, int64_t rows, int32_t V, int32_t k, const void* ws, size_t ws_bytes)
{
    if (!ws) return PICOSPEC_OK;
    if (((uintptr_t)ws & 15u) || ws_bytes < picospec_workspace_bytes(which, dtype, (int32_t)rows, V, k)) return PICOSPEC_EWORKSPACE;
    return PICOSPEC_OK;
}

int hip_status(hipError_t e) { return e == hipSuccess ? PICOSPEC_OK : PICOSPEC_EHIP; }

}  // namespace

namespace {

template <bool BF16>
int64_t max_load_end(int which, int V, int o)
{
    const int N = BF16 ? 8 : 4;
    const int L = o + V, nq = (L + N - 1) / N;
    const int64_t size = (int64_t)nq * 16;                                  // the row's descriptor
    int64_t end = 0;
    if (which == PICOSPEC_CALL_COMPRESS) {
        auto sweep = [&](auto geom) {                                       // both variants of the kernel
            using G = decltype(geom);
            const int sub_elems = G::SUB_VECS * N, n_sub = (L + sub_elems - 1) / sub_elems;
            for (int sub = 0; sub < n_sub + 2 * G::RING; ++sub)           // every sub-tile and every look-ahead position behind the row
                for (int j = 0; j < G::SV; ++j)
                    for (int tid = 0; tid < kCompressThreads; ++tid)
                        end = std::max(end, buffer_lane_read_end(size, (int64_t)G::group_first(sub, j) * 16, (int64_t)tid * 16));
        };
        sweep(CompressGeom<BF16, false>{});
        sweep(CompressGeom<BF16, true>{});
    } else {
        using G = ResidualGeom<BF16>;
        const int n_tiles = (L + kResidualTile - 1) / kResidualTile;
        for (int it = 0; it < n_tiles + 2 * G::AHEAD; ++it)
            for (int w = 0; w < kResidualThreads / 64; ++w)
                for (int jv = 0; jv < G::NV; ++jv)
                    for (int lane = 0; lane < 64; ++lane)
                        end = std::max(end, buffer_lane_read_end(size, (int64_t)G::group_first(it, w, jv) * 16, (int64_t)lane * 16));
    }
    return end;
}

}  // namespace

extern "C" {

int picospec_compress(const void* logits, int dtype, int64_t ld, int32_t n_rows, int32_t V,
                      float temperature, int32_t k, float top_p,
                      int32_t* idx, float* prob, int32_t* count, float* mass, float* lse,
                      void* workspace, size_t workspace_bytes, void* stream)
{
    if (int rc = check_logits(logits, dtype, ld, n_rows, V, temperature)) return rc;
    if (k < 1 || k > V || std::isnan(top_p)) return PICOSPEC_EINVAL;
    if (k > kMaxK) return PICOSPEC_EUNSUPPORTED;
    if (n_rows > 0 && (!idx || !prob || !count || !mass || !lse)) return PICOSPEC_EINVAL;
    if (int rc = check_workspace(PICOSPEC_CALL_COMPRESS, dtype, n_rows, V, k, workspace, workspace_bytes)) return rc;
    return hip_status(launch_compress(logits, dtype, ld, n_rows, V, temperature, k, top_p, idx, prob, count,
                                      mass, lse, nullptr, nullptr, (hipStream_t)stream));
}

int picospec_row_stats(const void* logits, int dtype, int64_t ld, int32_t n_rows, int32_t V, float temperature,
                       float* row_max, float* row_sum, float* row_lse, void* stream)
{
    if (int rc = check_logits(logits, dtype, ld, n_rows, V, temperature)) return rc;
    if (n_rows > 0 && (!row_max || !row_sum)) return PICOSPEC_EINVAL;
    return hip_status(launch_row_stats(logits, dtype, ld, n_rows, V, temperature, row_max, row_sum, row_lse,
                                       nullptr, (hipStream_t)stream));
}

int picospec_compress_rejected(const void* tgt_logits, int dtype, int64_t ld, int32_t V, float temperature,
                               int32_t B, int32_t n_draft, const int32_t* seq_off, const int32_t* n_accept,
                               int32_t k, float top_p,
                               int32_t* idx, float* prob, int32_t* count, float* mass, float* lse,
                               void* workspace, size_t workspace_bytes, void* stream)
{
    if (B < 0 || n_draft < 0) return PICOSPEC_EINVAL;
    const int64_t rows = (int64_t)n_draft + B;
    if (rows > INT32_MAX) return PICOSPEC_EINVAL;
    if (int rc = check_logits(tgt_logits, dtype, ld, rows, V, temperature)) return rc;
    if (k < 1 || k > V || std::isnan(top_p)) return PICOSPEC_EINVAL;
    if (k > kMaxK) return PICOSPEC_EUNSUPPORTED;
    if (B > 0 && (!seq_off || !n_accept || !idx || !prob || !count || !mass || !lse)) return PICOSPEC_EINVAL;
    if (int rc = check_workspace(PICOSPEC_CALL_COMPRESS_REJECTED, dtype, B, V, k, workspace, workspace_bytes)) return rc;
    return hip_status(launch_compress(tgt_logits, dtype, ld, B, V, temperature, k, top_p, idx, prob, count,
                                      mass, lse, seq_off, n_accept, (hipStream_t)stream));
}

int picospec_resample_sparse(const void* draft_logits, int dtype, int64_t ld, int32_t V, float temperature,
                             int32_t B, int32_t n_draft, const int32_t* seq_off, const int32_t* n_accept,
                             const float* draft_max, const float* draft_sum,
                             const int32_t* p_idx, const float* p_prob, const int32_t* p_count, const float* p_mass,
                             int32_t k, int renorm, const float* uniforms,
                             int32_t* out_tok, float* resid_mass, uint32_t* flags,
                             void* workspace, size_t workspace_bytes, void* stream)
{
    if (B < 0 || n_draft < 0) return PICOSPEC_EINVAL;
    if (int rc = check_logits(draft_logits, dtype, ld, n_draft, V, temperature)) return rc;
    if (renorm != 0 && renorm != 1) return PICOSPEC_EINVAL;
    if (k < 1) return PICOSPEC_EINVAL;
    if (k > kMaxK) return PICOSPEC_EUNSUPPORTED;
    if (B > 0 && (!seq_off || !n_accept || !p_idx || !p_prob || !p_count || !p_mass || !uniforms ||
                  !out_tok || !resid_mass || !flags)) return PICOSPEC_EINVAL;
    if (n_draft > 0 && (!draft_max || !draft_sum)) return PICOSPEC_EINVAL;
    if (int rc = check_workspace(PICOSPEC_CALL_RESAMPLE_SPARSE, dtype, n_draft, V, k, workspace, workspace_bytes)) return rc;
    return hip_status(launch_resample_sparse(draft_logits, dtype, ld, V, temperature, B, seq_off, n_accept,
                                             draft_max, draft_sum, p_idx, p_prob, p_count, p_mass, k, renorm,
                                             uniforms, out_tok, resid_mass, flags, (hipStream_t)stream));
}

// ---- one call for a whole round

int picospec_round(const void* draft_logits, const void* tgt_logits, int dtype, int64_t ld_draft, int64_t ld_tgt,
                   int32_t V, float temperature, int32_t B, int32_t n_draft, const int32_t* seq_off,
                   const int32_t* draft_tok, int32_t k, float top_p, int renorm, const float* uniforms,
                   int32_t* q_idx, float* q_prob, int32_t* q_count, float* q_mass, float* q_lse,
                   int32_t* n_accept, float* p_tok, float* q_tok,
                   float* tgt_max, float* tgt_sum, float* tgt_lse, uint32_t* verify_flags,
                   int32_t* out_tok, float* resid_mass, uint32_t* residual_flags,
                   void* workspace, size_t workspace_bytes, void* stream)
{
    if (B < 0 || n_draft < 0) return PICOSPEC_EINVAL;
    const int64_t rows = (int64_t)n_draft + B;
    if (rows > INT32_MAX) return PICOSPEC_EINVAL;
    if (int rc = check_logits(draft_logits, dtype, ld_draft, n_draft, V, temperature)) return rc;
    if (int rc = check_logits(tgt_logits, dtype, ld_tgt, rows, V, temperature)) return rc;
    if (k < 1 || k > V || std::isnan(top_p) || (renorm != 0 && renorm != 1)) return PICOSPEC_EINVAL;
    if (k > kMaxK) return PICOSPEC_EUNSUPPORTED;
    if (n_draft > 0 && (!draft_tok || !q_idx || !q_prob || !q_count || !q_mass || !q_lse)) return PICOSPEC_EINVAL;
    if (B > 0 && (!seq_off || !uniforms || !n_accept || !verify_flags || !tgt_max || !tgt_sum || !out_tok ||
                  !resid_mass || !residual_flags)) return PICOSPEC_EINVAL;
    if (int rc = check_workspace(PICOSPEC_CALL_ROUND, dtype, rows, V, k, workspace, workspace_bytes)) return rc;
    hipStream_t s = (hipStream_t)stream;
    // The two per-sequence kernels always go out as one (the position found by the acceptance test never leaves
    // the workgroup).  A round that leaves most of the chip idle is bound by the serial part of each launch, so
    // its two streaming kernels go out as one as well; a round that fills the chip streams faster with each
    // kernel in its own launch shape.
    const bool small_round = rows + n_draft <= kRoundSmallRows;     // (bound by its launches: two of them)
    if (small_round) {
        if (hipError_t e = launch_round_stream(draft_logits, dtype, ld_draft, n_draft, V, temperature, k, top_p, q_idx,
                                               q_prob, q_count, q_mass, q_lse, tgt_logits, ld_tgt, (int)rows,
                                               tgt_max, tgt_sum, tgt_lse, workspace, s))
            return hip_status(e);
    } else {
        if (hipError_t e = launch_compress(draft_logits, dtype, ld_draft, n_draft, V, temperature, k, top_p, q_idx, q_prob,
                                           q_count, q_mass, q_lse, nullptr, nullptr, s))
            return hip_status(e);
        if (hipError_t e = launch_row_stats(tgt_logits, dtype, ld_tgt, (int)rows, V, temperature, tgt_max, tgt_sum, tgt_lse, workspace, s))
            return hip_status(e);
    }
    return hip_status(launch_decide(tgt_logits, dtype, ld_tgt, V, temperature, B, seq_off, draft_tok, q_idx, q_prob,
                                    q_count, q_mass, k, renorm, uniforms, tgt_max, tgt_sum, n_accept, p_tok, q_tok,
                                    verify_flags, out_tok, resid_mass, residual_flags, workspace, rows, small_round, s));
}

// ---- verification and draw on records that exist

int picospec_verify_sample(const void* tgt_logits, int dtype, int64_t ld, int32_t V, float temperature,
                           int32_t B, int32_t n_draft, const int32_t* seq_off, const int32_t* draft_tok,
                           const int32_t* q_idx, const float* q_prob, const int32_t* q_count, const float* q_mass,
                           int32_t k, int renorm, const float* uniforms,
                           int32_t* n_accept, float* p_tok, float* q_tok,
                           float* tgt_max, float* tgt_sum, float* tgt_lse, uint32_t* verify_flags,
                           int32_t* out_tok, float* resid_mass, uint32_t* residual_flags,
                           void* workspace, size_t workspace_bytes, void* stream)
{
    if (B < 0 || n_draft < 0) return PICOSPEC_EINVAL;
    const int64_t rows = (int64_t)n_draft + B;
    if (rows > INT32_MAX) return PICOSPEC_EINVAL;
    if (int rc = check_logits(tgt_logits, dtype, ld, rows, V, temperature)) return rc;
    if (renorm != 0 && renorm != 1) return PICOSPEC_EINVAL;
    if (n_draft > 0 && (k < 1 || !draft_tok || !q_idx || !q_prob || !q_count || !q_mass)) return PICOSPEC_EINVAL;
    if (n_draft > 0 && k > kMaxK) return PICOSPEC_EUNSUPPORTED;
    if (B > 0 && (!seq_off || !uniforms || !n_accept || !verify_flags || !tgt_max || !tgt_sum || !out_tok ||
                  !resid_mass || !residual_flags)) return PICOSPEC_EINVAL;
    if (int rc = check_workspace(PICOSPEC_CALL_VERIFY_SAMPLE, dtype, rows, V, k, workspace, workspace_bytes)) return rc;
    hipStream_t s = (hipStream_t)stream;
    if (hipError_t e = launch_row_stats(tgt_logits, dtype, ld, (int)rows, V, temperature, tgt_max, tgt_sum, tgt_lse, workspace, s))
        return hip_status(e);
    return hip_status(launch_decide(tgt_logits, dtype, ld, V, temperature, B, seq_off, draft_tok, q_idx, q_prob,
                                    q_count, q_mass, k, renorm, uniforms, tgt_max, tgt_sum, n_accept, p_tok, q_tok,
                                    verify_flags, out_tok, resid_mass, residual_flags, workspace, rows, false, s));
}

// ---- wire messages

namespace {
bool wire_format_ok(int f) { return f == PICOSPEC_WIRE_FP32 || f == PICOSPEC_WIRE_FP16 || f == PICOSPEC_WIRE_BF16; }
bool aligned4(const void* p) { return ((uintptr_t)p & 3u) == 0; }
}  // namespace

int64_t picospec_downlink_bytes_max(int32_t B, int32_t k, int prob_format)
{
    if (B < 0 || k < 0 || k > kMaxK || !wire_format_ok(prob_format)) return -1;
    return downlink_bytes_max(B, k, prob_format);
}

int64_t picospec_uplink_bytes(int32_t B, int32_t n_draft, int prob_format)
{
    if (B < 0 || n_draft < 0 || !wire_format_ok(prob_format)) return -1;
    return uplink_bytes(B, n_draft, prob_format);
}

int picospec_pack_downlink(int32_t B, const int32_t* seq_off, const int32_t* n_accept, const int32_t* token,
                           const int32_t* idx, const float* prob, const int32_t* count, int32_t k,
                           int prob_format, void* wire, int64_t wire_capacity,
                           int64_t* wire_bytes, uint32_t* status, void* stream)
{
    if (B < 0 || !wire_format_ok(prob_format)) return PICOSPEC_EINVAL;
    const bool records = idx || prob || count;
    if (records && (!idx || !prob || !count || k < 1)) return PICOSPEC_EINVAL;
    if (records && k > kMaxK) return PICOSPEC_EUNSUPPORTED;
    if (!wire || !aligned4(wire) || wire_capacity < 8 || !wire_bytes || !status) return PICOSPEC_EINVAL;
    if (B > 0 && (!seq_off || !n_accept)) return PICOSPEC_EINVAL;
    return hip_status(launch_pack_downlink(B, seq_off, n_accept, token, idx, prob, count, records ? k : 0, prob_format,
                                           wire, wire_capacity, wire_bytes, status, (hipStream_t)stream));
}

int picospec_unpack_downlink(const void* wire, int64_t wire_bytes, int32_t B, int32_t k,
                             int32_t* n_accept, int32_t* token, int32_t* idx, float* prob, int32_t* count,
                             float* mass, uint32_t* status, void* stream)
{
    if (B < 0 || k < 1 || wire_bytes < 0) return PICOSPEC_EINVAL;
    if (k > kMaxK) return PICOSPEC_EUNSUPPORTED;
    if (!status || (wire_bytes > 0 && (!wire || !aligned4(wire)))) return PICOSPEC_EINVAL;
    if (B > 0 && (!n_accept || !token || !idx || !prob || !count || !mass)) return PICOSPEC_EINVAL;
    return hip_status(launch_unpack_downlink(wire, wire_bytes, B, k, n_accept, token, idx, prob, count, mass, status,
                                             (hipStream_t)stream));
}

int picospec_pack_uplink(int32_t B, int32_t n_draft, const int32_t* seq_off, const int32_t* draft_tok,
                         const float* q_scalar, int prob_format, void* wire, int64_t wire_capacity,
                         int64_t* wire_bytes, void* stream)
{
    if (B < 0 || n_draft < 0 || !wire_format_ok(prob_format)) return PICOSPEC_EINVAL;
    if (!wire || !aligned4(wire) || !wire_bytes) return PICOSPEC_EINVAL;
    if (wire_capacity < uplink_bytes(B, n_draft, prob_format)) return PICOSPEC_EINVAL;
    if (B > 0 && !seq_off) return PICOSPEC_EINVAL;
    if (n_draft > 0 && (!draft_tok || !q_scalar)) return PICOSPEC_EINVAL;
    return hip_status(launch_pack_uplink(B, n_draft, seq_off, draft_tok, q_scalar, prob_format, wire, wire_bytes,
                                         (hipStream_t)stream));
}

int picospec_unpack_uplink(const void* wire, int64_t wire_bytes, int32_t B, int32_t n_max,
                           int32_t* seq_off, int32_t* draft_tok, float* q_scalar, uint32_t* status, void* stream)
{
    if (B < 0 || n_max < 0 || wire_bytes < 0) return PICOSPEC_EINVAL;
    if (!status || !seq_off || (wire_bytes > 0 && (!wire || !aligned4(wire)))) return PICOSPEC_EINVAL;
    if (n_max > 0 && (!draft_tok || !q_scalar)) return PICOSPEC_EINVAL;
    return hip_status(launch_unpack_uplink(wire, wire_bytes, B, n_max, seq_off, draft_tok, q_scalar, status,
                                           (hipStream_t)stream));
}

int picospec_sample_draft(const int32_t* idx, const float* prob, const int32_t* count, const float* mass,
                          int32_t k, int32_t n_rows, const float* uniforms,
                          int32_t* tok, float* q_scalar, void* stream)
{
    if (n_rows < 0 || k < 1) return PICOSPEC_EINVAL;
    if (n_rows > 0 && (!idx || !prob || !count || !mass || !uniforms || !tok)) return PICOSPEC_EINVAL;
    return hip_status(launch_sample_draft(idx, prob, count, mass, k, n_rows, uniforms, tok, q_scalar,
                                          (hipStream_t)stream));
}

namespace {

// picospec_verify and picospec_verify_range share everything but the rows the statistics pass visits.
int verify_impl(const void* tgt_logits, int dtype, int64_t ld, int32_t V, float temperature,
                int32_t B, int32_t n_draft, const int32_t* seq_off, const int32_t* draft_tok,
                const int32_t* q_idx, const float* q_prob, const int32_t* q_count, const float* q_mass,
                int32_t k, int renorm, const float* q_scalar, const float* uniforms,
                int32_t* n_accept, float* p_tok, float* q_tok,
                float* tgt_max, float* tgt_sum, float* tgt_lse, uint32_t* flags,
                bool ranged, const int32_t* pos_begin, const int32_t* pos_end, int32_t gamma_max,
                void* workspace, size_t workspace_bytes, void* stream)
{
    if (B < 0 || n_draft < 0) return PICOSPEC_EINVAL;
    const int64_t rows = (int64_t)n_draft + B;
    if (rows > INT32_MAX) return PICOSPEC_EINVAL;
    if (int rc = check_logits(tgt_logits, dtype, ld, rows, V, temperature)) return rc;
    if (renorm != 0 && renorm != 1) return PICOSPEC_EINVAL;
    if (B > 0 && (!seq_off || !uniforms || !n_accept || !flags || !tgt_max || !tgt_sum)) return PICOSPEC_EINVAL;
    if (n_draft > 0) {
        if (!draft_tok) return PICOSPEC_EINVAL;
        if (!q_scalar && (k < 1 || !q_idx || !q_prob || !q_count || !q_mass)) return PICOSPEC_EINVAL;
    }
    if (ranged) {
        if (gamma_max < 0 || gamma_max > n_draft) return PICOSPEC_EINVAL;
        if (B > 65535 || gamma_max >= (1 << 20)) return PICOSPEC_EUNSUPPORTED;   // a (gamma_max + 1) x B launch
    }
    if (int rc = check_workspace(PICOSPEC_CALL_VERIFY, dtype, rows, V, k, workspace, workspace_bytes)) return rc;
    hipStream_t s = (hipStream_t)stream;
    const hipError_t e = ranged
        ? launch_row_stats_range(tgt_logits, dtype, ld, V, temperature, B, gamma_max, seq_off, pos_begin, pos_end,
                                 tgt_max, tgt_sum, tgt_lse, s)
        : launch_row_stats(tgt_logits, dtype, ld, (int)rows, V, temperature, tgt_max, tgt_sum, tgt_lse, workspace, s);
    if (e != hipSuccess) return hip_status(e);
    return hip_status(launch_accept(tgt_logits, dtype, ld, V, temperature, B, seq_off, draft_tok, q_idx, q_prob,
                                    q_count, q_mass, k, renorm, q_scalar, uniforms, tgt_max, tgt_sum,
                                    n_accept, p_tok, q_tok, flags, ranged ? pos_begin : nullptr,
                                    ranged ? pos_end : nullptr, s));
}

}  // namespace

int picospec_verify(const void* tgt_logits, int dtype, int64_t ld, int32_t V, float temperature,
                    int32_t B, int32_t n_draft, const int32_t* seq_off, const int32_t* draft_tok,
                    const int32_t* q_idx, const float* q_prob, const int32_t* q_count, const float* q_mass,
                    int32_t k, int renorm, const float* q_scalar, const float* uniforms,
                    int32_t* n_accept, float* p_tok, float* q_tok,
                    float* tgt_max, float* tgt_sum, float* tgt_lse, uint32_t* flags,
                    void* workspace, size_t workspace_bytes, void* stream)
{
    return verify_impl(tgt_logits, dtype, ld, V, temperature, B, n_draft, seq_off, draft_tok, q_idx, q_prob, q_count,
                       q_mass, k, renorm, q_scalar, uniforms, n_accept, p_tok, q_tok, tgt_max, tgt_sum, tgt_lse, flags,
                       false, nullptr, nullptr, 0, workspace, workspace_bytes, stream);
}

int picospec_verify_range(const void* tgt_logits, int dtype, int64_t ld, int32_t V, float temperature,
                          int32_t B, int32_t n_draft, const int32_t* seq_off, const int32_t* draft_tok,
                          const int32_t* q_idx, const float* q_prob, const int32_t* q_count, const float* q_mass,
                          int32_t k, int renorm, const float* q_scalar, const float* uniforms,
                          const int32_t* pos_begin, const int32_t* pos_end, int32_t gamma_max,
                          int32_t* n_accept, float* p_tok, float* q_tok,
                          float* tgt_max, float* tgt_sum, float* tgt_lse, uint32_t* flags,
                          void* workspace, size_t workspace_bytes, void* stream)
{
    return verify_impl(tgt_logits, dtype, ld, V, temperature, B, n_draft, seq_off, draft_tok, q_idx, q_prob, q_count,
                       q_mass, k, renorm, q_scalar, uniforms, n_accept, p_tok, q_tok, tgt_max, tgt_sum, tgt_lse, flags,
                       true, pos_begin, pos_end, gamma_max, workspace, workspace_bytes, stream);
}

int picospec_sample_residual(const void* tgt_logits, int dtype, int64_t ld, int32_t V, float temperature,
                             int32_t B, int32_t n_draft, const int32_t* seq_off, const int32_t* n_accept,
                             const float* tgt_max, const float* tgt_sum,
                             const int32_t* q_idx, const float* q_prob, const int32_t* q_count, const float* q_mass,
                             int32_t k, int renorm, const float* uniforms,
                             int32_t* out_tok, float* resid_mass, uint32_t* flags,
                             void* workspace, size_t workspace_bytes, void* stream)
{
    if (B < 0 || n_draft < 0) return PICOSPEC_EINVAL;
    const int64_t rows = (int64_t)n_draft + B;
    if (rows > INT32_MAX) return PICOSPEC_EINVAL;
    if (int rc = check_logits(tgt_logits, dtype, ld, rows, V, temperature)) return rc;
    if (renorm != 0 && renorm != 1) return PICOSPEC_EINVAL;
    if (B > 0 && (!seq_off || !n_accept || !tgt_max || !tgt_sum || !uniforms || !out_tok || !resid_mass || !flags))
        return PICOSPEC_EINVAL;
    if (n_draft > 0 && (k < 1 || !q_idx || !q_prob || !q_count || !q_mass)) return PICOSPEC_EINVAL;
    if (n_draft > 0 && k > kMaxK) return PICOSPEC_EUNSUPPORTED;   // records come from picospec_compress
    if (int rc = check_workspace(PICOSPEC_CALL_SAMPLE_RESIDUAL, dtype, rows, V, k, workspace, workspace_bytes)) return rc;
    return hip_status(launch_residual(tgt_logits, dtype, ld, V, temperature, B, seq_off, n_accept, tgt_max, tgt_sum,
                                      q_idx, q_prob, q_count, q_mass, k, renorm, uniforms, out_tok, resid_mass,
                                      flags, workspace, rows, (hipStream_t)stream));
}

size_t picospec_workspace_bytes(int which_call, int dtype, int32_t rows, int32_t V, int32_t k)
{
    (void)k;
    if (rows < 0 || V < 1 || V > kMaxV) return 0;
    switch (which_call) {                       // the calls that can keep the target rows' segment table
        case PICOSPEC_CALL_VERIFY: case PICOSPEC_CALL_SAMPLE_RESIDUAL: case PICOSPEC_CALL_VERIFY_SAMPLE:
            return seg_table_bytes(dtype, rows, V);
        case PICOSPEC_CALL_ROUND:               // (a small round lays the table out for its own launch shape)
            return round_seg_table_bytes(dtype, rows, V);
        default:
            return 0;                           // every other kernel keeps its intermediate state in LDS
    }
}

int64_t picospec_max_load_byte(int which_call, int dtype, int32_t V, int32_t misalign_bytes)
{
    if (which_call != PICOSPEC_CALL_COMPRESS && which_call != PICOSPEC_CALL_SAMPLE_RESIDUAL) return -1;
    if (dtype != PICOSPEC_F32 && dtype != PICOSPEC_BF16) return -1;
    const int esz = dtype == PICOSPEC_F32 ? 4 : 2;
    if (V < 1 || V > kMaxV || misalign_bytes < 0 || misalign_bytes > 15 || misalign_bytes % esz) return -1;
    const int o = misalign_bytes / esz;
    const int64_t end = dtype == PICOSPEC_BF16 ? max_load_end<true>(which_call, V, o) : max_load_end<false>(which_call, V, o);
    return end - misalign_bytes;
}

int picospec_check_device(void* workspace, size_t workspace_bytes, uint32_t* status, void* stream)
{
    if (!workspace || !status || workspace_bytes < (size_t)kCheckBytes || ((uintptr_t)workspace & 15u)) return PICOSPEC_EINVAL;
    return hip_status(launch_check_device(workspace, status, (hipStream_t)stream));
}

int picospec_probe_clock(uint64_t* ticks, void* stream)
{
    if (!ticks || ((uintptr_t)ticks & 7u)) return PICOSPEC_EINVAL;
    return hip_status(launch_probe_clock(ticks, (hipStream_t)stream));
}

int64_t picospec_limit(int which)
{
    switch (which) {
        case PICOSPEC_LIMIT_MAX_K: return kMaxK;
        case PICOSPEC_LIMIT_MAX_V: return kMaxV;
        default: return -1;
    }
}

const char* picospec_strerror(int code)
{
    switch (code) {
        case PICOSPEC_OK: return "ok";
        case PICOSPEC_EINVAL: return "invalid argument (null pointer, size out of range, temperature <= 0, misaligned base)";
        case PICOSPEC_EWORKSPACE: return "workspace smaller than picospec_workspace_bytes() or not on a 16-byte boundary";
        case PICOSPEC_EDTYPE: return "dtype must be PICOSPEC_F32 or PICOSPEC_BF16";
        case PICOSPEC_EHIP: return "HIP runtime call failed";
        case PICOSPEC_EUNSUPPORTED: return "k or V exceeds picospec_limit()";
        case PICOSPEC_ESCRATCH: return "the target rows' segment table exceeds the fixed array of picospec_verify_sample_static (picospec_static_scratch_bytes())";
        default: return "unknown picospec error code";
    }
}

int picospec_version(void) { return 1000; }

}  // extern "C"
