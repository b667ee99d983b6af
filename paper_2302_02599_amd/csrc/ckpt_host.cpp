// Host-only part of the C ABI: table layout helpers, the planner's budget list and error
// strings.  No HIP in this file, so that it can also be built and run under host sanitizers.
#include <cstddef>
#include <cstdint>

#include "ckpt_dp.h"

extern "C" {

size_t ckpt_row_pitch(int M) { return M < 0 ? 0 : (size_t(M) + 1 + 63) & ~size_t(63); }

size_t ckpt_table_rows(int L) { return L < 1 ? 0 : size_t(L) * (size_t(L) + 1) / 2; }

long ckpt_row_index(int L, int s, int t) {
    if (L < 1 || s < 1 || t < s || t > L) return -1;
    return long(s - 1) * L - long(s - 1) * (s - 2) / 2 + (t - s);
}

size_t ckpt_table_elems(int L, int M, int B) {
    if (L < 1 || M < 0 || B < 1) return 0;
    return size_t(B) * ckpt_table_rows(L) * ckpt_row_pitch(M);
}

int ckpt_budget_sweep(int64_t base_budget, int alpha_num, int alpha_den, int count, int64_t* budgets) {
    if (base_budget <= 0 || alpha_num < 0 || alpha_den <= 0 || count < 1 || !budgets) return CKPT_E_ARG;
    if (count > CKPT_MAX_SWEEP) return CKPT_E_LIMIT;
    // budget_n = floor(base * (den + num)^n / den^n), kept exact in 128 bits
    const unsigned __int128 limit = ~static_cast<unsigned __int128>(0);
    const unsigned __int128 grow = static_cast<unsigned __int128>(alpha_num) + static_cast<unsigned>(alpha_den);
    unsigned __int128 top = static_cast<unsigned __int128>(base_budget), bottom = 1;
    for (int n = 0; n < count; ++n) {
        const unsigned __int128 b = top / bottom;
        if (b > static_cast<unsigned __int128>(INT64_MAX)) return CKPT_E_LIMIT;
        budgets[n] = static_cast<int64_t>(b);
        if (n + 1 == count) break;
        if (top > limit / grow || bottom > limit / static_cast<unsigned>(alpha_den)) return CKPT_E_LIMIT;
        top *= grow;
        bottom *= static_cast<unsigned>(alpha_den);
    }
    return CKPT_OK;
}

const char* ckpt_strerror(int code) {
    switch (code) {
        case CKPT_OK: return "ok";
        case CKPT_E_ARG: return "bad argument";
        case CKPT_E_LIMIT: return "size limit exceeded";
        case CKPT_E_INFEASIBLE: return "requested cell is infeasible";
        case CKPT_E_SMALLBUF: return "output buffer too small";
        case CKPT_E_HIP: return "HIP call failed";
        case CKPT_E_INPUT: return "chain values violate the preconditions";
        case CKPT_E_CORRUPT: return "arg table or operation list is inconsistent";
        case CKPT_E_NOTREADY: return "helper streams do not exist yet and cannot be created now: call ckpt_init first";
        case CKPT_E_INTERNAL: return "a wait between work-groups of the fill expired; the tables are incomplete";
        default: return "unknown error";
    }
}

}  // extern "C"
