// Experiment overrides of the planner's parameter choice: "key=value,key=value,..." (the SCORCH_SPMM_TUNE
// environment variable).  The text is parsed ONCE, when a plan is made, and the result is kept in the plan; no
// execution call looks at the environment.  The parser keeps no state between calls (no strtok), so plans may be
// made from several host threads at once.  No HIP dependency: the host tests compile and check it on the CPU.
#pragma once

#include <stdint.h>

namespace scorch {

struct Tuning {
    int32_t bn = 0, alpha = 0, lw = 0, ch = 0, bch = 0, u = 0, nt = -1, sliced = -1, pack = -1, panel = -1, hot = -1,
            sdblk = -1, fix = -1, cold = 0;
};

// Unknown keys, items without '=', and values that are not decimal integers are skipped; a value is clamped to the
// int32 range; blanks around keys and values are ignored.  nullptr or "" gives the defaults.
inline Tuning parse_tuning(const char *s) {
    Tuning t;
    if (!s) return t;
    struct Key { const char *name; int32_t Tuning::*field; };
    static const Key keys[] = {{"bn", &Tuning::bn}, {"alpha", &Tuning::alpha}, {"lw", &Tuning::lw}, {"ch", &Tuning::ch},
                               {"bch", &Tuning::bch}, {"u", &Tuning::u}, {"nt", &Tuning::nt}, {"sliced", &Tuning::sliced},
                               {"pack", &Tuning::pack}, {"panel", &Tuning::panel}, {"hot", &Tuning::hot},
                               {"sdblk", &Tuning::sdblk}, {"fix", &Tuning::fix}, {"cold", &Tuning::cold}};
    const char *p = s;
    while (*p) {
        const char *item = p;
        while (*p && *p != ',') ++p;
        const char *end = p;  // one past the item
        if (*p == ',') ++p;
        while (item < end && (*item == ' ' || *item == '\t')) ++item;
        const char *eq = item;
        while (eq < end && *eq != '=') ++eq;
        if (eq == end) continue;
        const char *kend = eq;
        while (kend > item && (kend[-1] == ' ' || kend[-1] == '\t')) --kend;
        const char *v = eq + 1;
        while (v < end && (*v == ' ' || *v == '\t')) ++v;
        bool neg = false;
        if (v < end && (*v == '-' || *v == '+')) neg = *v++ == '-';
        if (v == end || *v < '0' || *v > '9') continue;
        int64_t val = 0;
        while (v < end && *v >= '0' && *v <= '9') {
            val = val * 10 + (*v++ - '0');
            if (val > 0x7fffffffLL) val = 0x7fffffffLL;
        }
        while (v < end && (*v == ' ' || *v == '\t')) ++v;
        if (v != end) continue;  // trailing garbage: not a number
        if (neg) val = -val;
        for (const Key &k : keys) {
            const char *a = item, *b = k.name;
            while (a < kend && *b && *a == *b) ++a, ++b;
            if (a == kend && !*b) {
                t.*(k.field) = (int32_t)val;
                break;
            }
        }
    }
    return t;
}

}  // namespace scorch
