// What the persistent prefill kernel assumes about the device, as a pure host function (no HIP types), so
// that the rule can be compiled and tested without a GPU.
#pragma once

namespace bm {

constexpr int K64_CUS = 256;     // compute units: one persistent workgroup each (a workgroup takes a unit's whole LDS)
constexpr int K64_XCDS = 8;      // workgroups are dealt round-robin to the XCDs: blockIdx.x % 8 names the XCD

// The XCD-aware persistent schedule (and the split-tail scratch, one 256 x 256 fp32 tile per workgroup of
// a launch of at most K64_CUS workgroups) is laid out for exactly this part.  On anything else - a
// partitioned device, another chip, an attribute query that failed (0) - the launchers take the
// non-persistent kernels, which assume nothing about the device.
inline bool persistent_schedule_fits(int n_compute_units, int n_xcds) {
    return n_compute_units == K64_CUS && n_xcds == K64_XCDS;
}

}  // namespace bm
