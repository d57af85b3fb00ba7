// Pieces of the host side of the C ABI (zo_abi.cpp) that other translation units of the library use.
#pragma once
#include "../../include/zo.h"

namespace zo {

// Everything zo_score checks before it looks at its workspace (no HIP call); sets the thread's error
// message and returns the status.
int32_t score_validate(const zo_batch* batch, const void* H, int64_t ldh, const void* W_head, int64_t ldw,
                       int32_t vocab, int32_t d, zo_dtype dtype, const int32_t* targets, const float* seq_nll,
                       const float* cand_sum, const int32_t* cand_cnt);
// Records `message` as the thread's last error and returns `status`.
int32_t fail_status(int32_t status, const char* message);

}  // namespace zo
