// Which row pointers one key of a sorted key list fills (coordinate lists and doubly compressed rows).
// Plain integer arithmetic with no HIP dependency, so that the host tests can compile and check it on the CPU.
//
// Key p (0 <= p <= count; p == count is the sentinel, whose key is m) closes the rows between its predecessor's
// key and its own: rowptr[r] = position of p for prev < r <= cur.  The fill may only run when BOTH ends are valid,
// otherwise a bad predecessor (say -5 followed by 3) would start it below rowptr[0].
#pragma once

#include <stdint.h>

#if defined(__HIPCC__)
#define SCORCH_KEYS_HOST_DEVICE __host__ __device__
#else
#define SCORCH_KEYS_HOST_DEVICE
#endif

namespace scorch {

// prev: key p-1 (ignored for p == 0), cur: key p (ignored for p == count).  Returns false when the list is not
// sorted or a key lies outside [0, m): nothing may be written then.  Otherwise [lo, hi] is the range of row
// pointers to fill, always inside [0, m] (it is empty, lo > hi, for a repeated key).
SCORCH_KEYS_HOST_DEVICE inline bool rowptr_fill_range(int64_t p, int64_t count, int32_t prev, int32_t cur, int32_t m,
                                                      bool strictly_increasing, int32_t &lo, int32_t &hi) {
    const bool first = p == 0, sentinel = p == count;
    const int64_t kp = first ? -1 : (int64_t)prev;
    const int64_t kc = sentinel ? (int64_t)m : (int64_t)cur;
    if (!first && (kp < 0 || kp >= m)) return false;
    if (!sentinel && (kc < 0 || kc >= m)) return false;
    if (!first && !sentinel && (strictly_increasing ? kc <= kp : kc < kp)) return false;
    lo = (int32_t)(kp + 1);
    hi = (int32_t)kc;
    return true;
}

}  // namespace scorch
