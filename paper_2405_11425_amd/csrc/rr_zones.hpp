// The "pair rates -> memory zones" rule as the library's own translation units see it (rr_zones.cpp implements
// it, rr_api.hip feeds it with measured rates).  Nothing here is part of the C ABI.
#pragma once
#include "../../include/randline.h"

namespace rr {

int fail(int code, const char *fmt, ...);  // rr_state.hip: records the message for rr_last_error

// Argument checks shared by rr_zones_from_pair_rates and rr_detect_zones.
int check_zone_rule_args(uint32_t n, double min_gap, uint32_t max_zones, const void *zone_out);

// The rule itself; arguments already checked.  zone_out[n] and *details (may be NULL) are written on success.
int zones_rule(rr_pair_rate_fn rate, void *user, uint32_t n, double min_gap, uint32_t max_zones, uint8_t *zone_out,
               rr_zone_probe_t *details);

}  // namespace rr
