// Rail health monitor (Section 4.3, "Health Monitoring"): host-side state machine over at most
// TENT_MAX_RAILS records, stepped once per measurement window.  No device work: the inputs are
// the per-rail error counts and bandwidth probes the device passes already reduced.
#include "tent_internal.h"

namespace {

enum : uint32_t { kHealthy = 0, kDegraded = 1, kPaused = 2 };
constexpr uint32_t kCooldownCap = 1u << 31;

// One window of one rail.  `errors` is the weighted error count of the window (a hard error weighs
// two congestion errors), `slow` says whether telemetry saw a degradation event.
void step_rail(const tent_monitor_params& mp, tent_rail_monitor& m, uint64_t errors, bool slow)
{
    switch (m.state) {
    case kPaused:
        // excluded: nothing the rail reports counts; the cooldown runs down and the rail comes
        // back with half weight
        if (m.cooldown_left) --m.cooldown_left;
        if (m.cooldown_left == 0) {
            m.state = kDegraded;
            m.clean = 0;
            m.score = 0;
        }
        return;
    default:
        break;
    }
    const uint64_t score = errors ? (uint64_t)m.score + errors : 0;
    m.score = score > 0xFFFFFFFFull ? 0xFFFFFFFFu : (uint32_t)score;
    const uint64_t pause_above = 2ull * mp.err_threshold;
    if (m.score > pause_above) {
        const uint32_t length = m.cooldown_next;
        m.cooldown_next = length >= (kCooldownCap >> 1) ? kCooldownCap : length << 1;
        m.score = 0;
        m.clean = 0;
        m.cooldown_left = length;
        m.state = length ? kPaused : kDegraded;
        return;
    }
    if (errors || slow) {
        m.state = kDegraded;
        m.clean = 0;
        return;
    }
    if (m.state == kDegraded && ++m.clean >= mp.recover_windows) {
        m.state = kHealthy;
        m.clean = 0;
        m.cooldown_next = mp.cooldown_windows;
    }
}

}  // namespace

extern "C" {

int tent_monitor_init(const tent_monitor_params* params, tent_rail_monitor* mon, uint32_t n_rails)
{
    if (!params || !mon) return TENT_ERR_INVALID;
    if (n_rails == 0 || n_rails > TENT_MAX_RAILS) return TENT_ERR_RANGE;
    for (uint32_t d = 0; d < n_rails; ++d)
        mon[d] = tent_rail_monitor{kHealthy, 0, 0, 0, params->cooldown_windows};
    return TENT_OK;
}

int tent_monitor_update(const tent_monitor_params* params, tent_rail_monitor* mon, tent_rail_state* rails,
                        uint32_t n_rails, const uint32_t* hard_errors, const uint32_t* congestion_errors,
                        const uint32_t* probe_MBps, const uint32_t* bw_before_MBps)
{
    if (!params || !mon || !rails || !hard_errors || !congestion_errors || !probe_MBps || !bw_before_MBps)
        return TENT_ERR_INVALID;
    if (n_rails == 0 || n_rails > TENT_MAX_RAILS) return TENT_ERR_RANGE;
    for (uint32_t d = 0; d < n_rails; ++d)
        if (mon[d].state > kPaused) return TENT_ERR_INVALID;
    for (uint32_t d = 0; d < n_rails; ++d) {
        const uint64_t errors = 2ull * hard_errors[d] + congestion_errors[d];
        const bool slow = probe_MBps[d] != 0 &&
                          256ull * probe_MBps[d] < (uint64_t)params->degrade_q8 * bw_before_MBps[d];
        step_rail(*params, mon[d], errors, slow);
        rails[d].health = (uint8_t)mon[d].state;
    }
    return TENT_OK;
}

}  // extern "C"
