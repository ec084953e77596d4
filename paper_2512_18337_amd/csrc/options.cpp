// Run-time tuning knobs (see agentsam_set_option in the header).
#include <atomic>
#include <cstring>

#include "common.h"

namespace agentsam {
static std::atomic<int64_t> g_attn_kv_chunk{0};
static std::atomic<int64_t> g_attn_v_mode{1};
static std::atomic<int64_t> g_attn_schedule{0};
static std::atomic<int64_t> g_attn_cascade{0};
int64_t option_attn_kv_chunk() { return g_attn_kv_chunk.load(std::memory_order_relaxed); }
int64_t option_attn_v_mode() { return g_attn_v_mode.load(std::memory_order_relaxed); }
int64_t option_attn_schedule() { return g_attn_schedule.load(std::memory_order_relaxed); }
int64_t option_attn_cascade() { return g_attn_cascade.load(std::memory_order_relaxed); }
}  // namespace agentsam

extern "C" int agentsam_set_option(const char *key, int64_t value) {
    if (!key) return AGENTSAM_ERR_NULL;
    if (std::strcmp(key, "attn_kv_chunk") == 0) {
        if (value != 0 && (value < 128 || value % 128 != 0 || value > (1ll << 30))) return AGENTSAM_ERR_ARG;
        agentsam::g_attn_kv_chunk.store(value, std::memory_order_relaxed);
        return AGENTSAM_OK;
    }
    if (std::strcmp(key, "attn_v_mode") == 0) {
        if (value != 0 && value != 1) return AGENTSAM_ERR_ARG;
        agentsam::g_attn_v_mode.store(value, std::memory_order_relaxed);
        return AGENTSAM_OK;
    }
    if (std::strcmp(key, "attn_cascade") == 0) {
        if (value < 0 || value > 2) return AGENTSAM_ERR_ARG;
        agentsam::g_attn_cascade.store(value, std::memory_order_relaxed);
        return AGENTSAM_OK;
    }
    if (std::strcmp(key, "attn_schedule") == 0) {
        if (value < 0 || value > 2) return AGENTSAM_ERR_ARG;
        agentsam::g_attn_schedule.store(value, std::memory_order_relaxed);
        return AGENTSAM_OK;
    }
    return AGENTSAM_ERR_ARG;
}
