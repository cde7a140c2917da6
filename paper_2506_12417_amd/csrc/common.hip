// Error text, version, workspace sizes and the threshold q (section 4.4, Eq. 4).
#include "common.h"
#include <cstdarg>
#include <cstdio>
#include <cmath>

static thread_local char g_err[512] = "";

int moe_fail(int code, const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return code;
}

extern "C" const char* moe_last_error(void) { return g_err; }
extern "C" const char* moe_version(void) { return "libmoe 0.1 (gfx950)"; }

// Eq. 4: q > phi * d_type / (2 * beta)
extern "C" int moe_token_threshold(double phi, int d_type, double beta) {
    if (!(phi > 0.0) || !(beta > 0.0) || d_type < 1) return 1;
    double q = phi * (double)d_type / (2.0 * beta);
    if (q > 1e9) q = 1e9;
    int qi = (int)std::ceil(q);
    return qi < 1 ? 1 : qi;
}

// permute scratch: one histogram of E counters per block of PERMUTE_BLOCK_ITEMS assignments
extern "C" size_t moe_workspace_bytes(int op, int T, int d, int F, int E, int k, moe_dtype dt) {
    (void)d; (void)F; (void)dt;
    if (op == MOE_OP_PERMUTE) {
        if (T < 0 || k < 1 || E < 1) return 0;
        size_t A = (size_t)T * (size_t)k;
        size_t nb = (A + 1023) / 1024;
        if (nb == 0) nb = 1;
        return nb * (size_t)E * sizeof(int32_t);
    }
    return 0;
}
