// Greedy (temperature 0) mode of fsr_spec_accept; implemented in greedy_accept.hip.
#pragma once
#include <hip/hip_runtime.h>

#include "../../include/faser_verify.h"

namespace fsr {

size_t greedy_workspace_bytes(const fsr_accept_params& p);

// Enqueues the greedy verification of one call on `s`; `workspace` holds greedy_workspace_bytes(p).
int greedy_accept_launch(const float* target, const int32_t* draft_tokens, const int32_t* cu_t, const int32_t* cu_d,
                         const int32_t* t_rows, const int32_t* d_rows, int32_t* accepted_len, int32_t* n_emitted,
                         int32_t* emitted, const fsr_accept_params& p, void* workspace, hipStream_t s);

}  // namespace fsr
