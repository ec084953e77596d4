// Shared host-side helpers of the HIP entry points (error mapping, launch checks, options).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "agentsam.h"

#define AGENTSAM_LAUNCH_CHECK()                                  \
    do {                                                         \
        if (hipGetLastError() != hipSuccess) return AGENTSAM_ERR_HIP; \
    } while (0)

namespace agentsam {
// value of the "attn_kv_chunk" option (0 = automatic)
int64_t option_attn_kv_chunk();
constexpr int kWave = 64;
}  // namespace agentsam
