// Host-side schedule reconstruction: walks one chain's recorded candidates back
// into the operation sequence of Table 1 (C_all / C_ck of the Theorem, Section
// "Activation Checkpoint Solver / Modeling", read from the root cell downwards).
#include <cstdint>

#include "ckpt_dp.h"

namespace {

struct Walker {
    const uint8_t* arg;
    const int32_t* wa;
    const int32_t* wabar;
    int L;
    int M;
    size_t pitch;
    ckpt_op_t* out;
    int cap;
    int n = 0;
    int err = CKPT_OK;

    bool emit(int kind, int stage) {
        if (n >= cap) {
            err = CKPT_E_SMALLBUF;
            return false;
        }
        out[n].kind = static_cast<uint8_t>(kind);
        out[n].stage = static_cast<uint8_t>(stage);
        ++n;
        return true;
    }

    // Emits the schedule of cell (s, t, m).  Depth of the recursion is at most t - s + 1.
    bool walk(int s, int t, long m, bool root) {
        if (m < 0 || m > M) {
            err = root ? CKPT_E_ARG : CKPT_E_CORRUPT;
            return false;
        }
        const int k = arg[size_t(ckpt_row_index(L, s, t)) * pitch + size_t(m)];
        if (k == 0) {
            // An infeasible cell below a feasible one cannot come from a table this library wrote.
            err = root ? CKPT_E_INFEASIBLE : CKPT_E_CORRUPT;
            return false;
        }
        if (k < s || k > t) {
            err = CKPT_E_CORRUPT;
            return false;
        }
        if (s == t) return emit(CKPT_OP_F_ALL, s) && emit(CKPT_OP_B, s);
        if (k == s) {  // C_all: F_all^s, schedule of (s+1, t, m - omega_abar^s), B^s
            return emit(CKPT_OP_F_ALL, s) && walk(s + 1, t, m - long(wabar[s - 1]), false) &&
                   emit(CKPT_OP_B, s);
        }
        // C_ck at s' = k: F_ck^s, F_null^{s+1..k-1}, schedule of (k, t, m - omega_a^{k-1}), schedule of (s, k-1, m)
        if (!emit(CKPT_OP_F_CK, s)) return false;
        for (int j = s + 1; j < k; ++j)
            if (!emit(CKPT_OP_F_NULL, j)) return false;
        return walk(k, t, m - long(wa[k - 1]), false) && walk(s, k - 1, m, false);
    }
};

}  // namespace

extern "C" int ckpt_schedule(const uint8_t* arg_host, const int32_t* wa, const int32_t* wabar, int L, int M,
                             int s, int t, int m_budget, ckpt_op_t* ops_out, int ops_cap) {
    if (!arg_host || !wa || !wabar || !ops_out || ops_cap < 0) return CKPT_E_ARG;
    if (L < 1 || M < 0 || s < 1 || t < s || t > L || m_budget < 0) return CKPT_E_ARG;
    if (L > CKPT_MAX_L) return CKPT_E_LIMIT;
    Walker w{arg_host, wa, wabar, L, M, ckpt_row_pitch(M), ops_out, ops_cap};
    if (!w.walk(s, t, m_budget > M ? M : m_budget, true)) return w.err;  // the table ends at M
    return w.n;
}

// Checkpoint block index of every stage from an operation list over stages 1..L (Section "Code
// generation").  The annotation of a stage comes from its first forward operation; the
// operations before the first B are exactly the first forwards of stages 1..L, in order.
extern "C" int ckpt_block_indices(const ckpt_op_t* ops, int n_ops, int L, int32_t* block_of_stage) {
    if (!ops || !block_of_stage || L < 1 || n_ops < 0) return CKPT_E_ARG;
    if (L > CKPT_MAX_L) return CKPT_E_LIMIT;
    if (n_ops < L + 1) return CKPT_E_CORRUPT;
    int blocks = 0;
    for (int k = 0; k < L; ++k) {
        const int kind = ops[k].kind;
        if (ops[k].stage != k + 1) return CKPT_E_CORRUPT;
        if (kind == CKPT_OP_F_ALL) {
            block_of_stage[k] = -1;
        } else if (kind == CKPT_OP_F_CK) {
            block_of_stage[k] = blocks++;
        } else if (kind == CKPT_OP_F_NULL && k > 0 && block_of_stage[k - 1] >= 0) {
            block_of_stage[k] = block_of_stage[k - 1];
        } else {
            return CKPT_E_CORRUPT;
        }
    }
    if (ops[L].kind != CKPT_OP_B || ops[L].stage != L) return CKPT_E_CORRUPT;
    return blocks;
}
