// picospec_verify_sample for callers that cannot allocate: the target rows' segment table, which the other entry
// points keep in a workspace the caller brings, lives here in a fixed array in device memory.
#include "../../include/picospec.h"

#include <atomic>
#include <cmath>

#include "kernels.hpp"

using namespace picospec;

namespace {

constexpr size_t kScratchBytes = 8u << 20;      // what picospec_limit(PICOSPEC_LIMIT_STATIC_SCRATCH_BYTES) reports

// Each GPU that the library runs on holds its own copy of this array, at its own address, until the process ends.
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

// The array's address on each device, asked for once per device with that device current.  (In host code the array's
// name is only a handle for that question, not an address a kernel could use.)
std::atomic<void*> scratch_ptr[kMaxDevices] = {};

hipError_t scratch_of_current_device(void** out)
{
    int dev = 0;
    if (hipError_t e = hipGetDevice(&dev)) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    void* p = scratch_ptr[dev].load(std::memory_order_acquire);
    if (!p) {                                    // (two threads that meet here get the same answer)
        if (hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch))) return e;
        if (!p) return hipErrorInvalidSymbol;
        scratch_ptr[dev].store(p, std::memory_order_release);
    }
    *out = p;
    return hipSuccess;
}

}  // namespace

extern "C" {

int64_t picospec_static_scratch_bytes(void) { return (int64_t)kScratchBytes; }

int picospec_verify_sample_static(const void* tgt_logits, int dtype, int64_t ld, int32_t V, float temperature,
                                  int32_t B, int32_t n_draft, const int32_t* seq_off, const int32_t* draft_tok,
                                  const int32_t* q_idx, const float* q_prob, const int32_t* q_count, const float* q_mass,
                                  int32_t k, int renorm, const float* uniforms,
                                  int32_t* n_accept, float* p_tok, float* q_tok,
                                  float* tgt_max, float* tgt_sum, float* tgt_lse, uint32_t* verify_flags,
                                  int32_t* out_tok, float* resid_mass, uint32_t* residual_flags, void* stream)
{
    // the same checks as picospec_verify_sample
    if (dtype != PICOSPEC_F32 && dtype != PICOSPEC_BF16) return PICOSPEC_EDTYPE;
    if (B < 0 || n_draft < 0) return PICOSPEC_EINVAL;
    const int64_t rows = (int64_t)n_draft + B;
    if (rows > INT32_MAX || V < 1 || ld < V || !(std::isfinite(temperature) && temperature > 0.f)) return PICOSPEC_EINVAL;
    if (V > kMaxV) return PICOSPEC_EUNSUPPORTED;
    if (rows > 0 && (!tgt_logits || (uintptr_t)tgt_logits % (dtype == PICOSPEC_F32 ? 4 : 2))) return PICOSPEC_EINVAL;
    if (renorm != 0 && renorm != 1) return PICOSPEC_EINVAL;
    if (n_draft > 0 && (k < 1 || !draft_tok || !q_idx || !q_prob || !q_count || !q_mass)) return PICOSPEC_EINVAL;
    if (n_draft > 0 && k > kMaxK) return PICOSPEC_EUNSUPPORTED;
    if (B > 0 && (!seq_off || !uniforms || !n_accept || !verify_flags || !tgt_max || !tgt_sum || !out_tok ||
                  !resid_mass || !residual_flags)) return PICOSPEC_EINVAL;
    // the table of these rows must fit the fixed array
    if (seg_table_bytes(dtype, rows, V) > kScratchBytes) return PICOSPEC_ESCRATCH;
    void* table = nullptr;
    if (scratch_of_current_device(&table) != hipSuccess) return PICOSPEC_EHIP;
    hipStream_t s = (hipStream_t)stream;
    // (every entry of the table that the second launch reads is written by the first: nothing has to start at zero)
    if (launch_row_stats(tgt_logits, dtype, ld, (int)rows, V, temperature, tgt_max, tgt_sum, tgt_lse, table, s) != hipSuccess)
        return PICOSPEC_EHIP;
    return launch_decide(tgt_logits, dtype, ld, V, temperature, B, seq_off, draft_tok, q_idx, q_prob, q_count, q_mass,
                         k, renorm, uniforms, tgt_max, tgt_sum, n_accept, p_tok, q_tok, verify_flags, out_tok, resid_mass,
                         residual_flags, table, rows, false, s) == hipSuccess ? PICOSPEC_OK : PICOSPEC_EHIP;
}

}  // extern "C"
