// CPU check of the index arithmetic behind scorch_coo_to_csr_rowptr / scorch_dcsr_to_csr_rowptr.
// Replays the kernel's per-key loop on the host over every key list of length 0..4 with keys drawn from
// {INT_MIN, -3..m+2, INT_MAX}, for m = 0..4, in both orders of strictness, into a guarded array, and verifies
//   * nothing outside rowptr[0..m] is ever written, whatever the keys (the fill range is inside [0, m]),
//   * a list with an out-of-range or out-of-order key raises the flag,
//   * a valid list raises no flag and gives rowptr[r] = number of keys below r (coordinate list), every pointer
//     written exactly once.
// Prints "ok <cases>" or the first failure.
#include <climits>
#include <cstdio>
#include <vector>

#include "rowptr_keys.h"

using namespace scorch;

static long cases = 0;

static bool check(const std::vector<int32_t> &keys, int32_t m, bool strict) {
    const int guard = 8;
    std::vector<int32_t> buf(guard + m + 1 + guard, -77), writes(m + 1, 0);
    int32_t *rowptr = buf.data() + guard;
    const int64_t count = (int64_t)keys.size();
    bool flag = false;
    for (int64_t p = 0; p <= count; ++p) {
        const int32_t prev = p > 0 ? keys[p - 1] : -1;
        const int32_t cur = p < count ? keys[p] : m;
        int32_t lo = 0, hi = -1;
        if (!rowptr_fill_range(p, count, prev, cur, m, strict, lo, hi)) {
            flag = true;
            continue;
        }
        if (lo < 0 || hi > m) {
            std::printf("fill range [%d, %d] outside [0, %d]\n", lo, hi, m);
            return false;
        }
        for (int r = lo; r <= hi; ++r) {
            rowptr[r] = (int32_t)p;
            writes[r]++;
        }
    }
    for (int i = 0; i < guard; ++i)
        if (buf[i] != -77 || buf[guard + m + 1 + i] != -77) {
            std::printf("write outside rowptr\n");
            return false;
        }
    bool valid = true;
    for (int64_t p = 0; p < count; ++p) {
        if (keys[p] < 0 || keys[p] >= m) valid = false;
        if (p > 0 && (strict ? keys[p] <= keys[p - 1] : keys[p] < keys[p - 1])) valid = false;
    }
    if (valid == flag) {
        std::printf("flag %d for a %s list (m=%d, %lld keys, strict=%d)\n", (int)flag, valid ? "valid" : "bad", m,
                    (long long)count, (int)strict);
        return false;
    }
    if (valid)
        for (int r = 0; r <= m; ++r) {
            int below = 0;
            for (int32_t k : keys) below += k < r;
            if (writes[r] != 1 || rowptr[r] != below) {
                std::printf("rowptr[%d] = %d written %d times, expected %d once\n", r, rowptr[r], writes[r], below);
                return false;
            }
        }
    ++cases;
    return true;
}

int main() {
    for (int32_t m = 0; m <= 4; ++m) {
        std::vector<int32_t> alphabet = {INT_MIN, INT_MAX};
        for (int32_t v = -3; v <= m + 2; ++v) alphabet.push_back(v);
        const size_t A = alphabet.size();
        for (int strict = 0; strict <= 1; ++strict)
            for (int len = 0; len <= 4; ++len) {
                size_t total = 1;
                for (int i = 0; i < len; ++i) total *= A;
                for (size_t code = 0; code < total; ++code) {
                    std::vector<int32_t> keys(len);
                    size_t c = code;
                    for (int i = 0; i < len; ++i) {
                        keys[i] = alphabet[c % A];
                        c /= A;
                    }
                    if (!check(keys, m, strict != 0)) return 1;
                }
            }
    }
    std::printf("ok %ld\n", cases);
    return 0;
}
