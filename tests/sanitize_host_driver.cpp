// Driver for the host sanitizer job (tests/test_host_sanitizers.py).  It is compiled together with
// oracle/ckpt_oracle.c and the host-only sources of the library under
// -fsanitize=address,undefined, reads commands from stdin and prints what the functions return;
// the test compares the output with the results of the ordinary builds.  Any sanitizer report
// aborts the process.
//
//   chain L M uf.. ub.. wa.. wabar.. wdelta.. of.. ob..   solve with the oracle, keep the tables
//   dump PATH_COST PATH_CHOICE                            write them (int32 / int16, [L][L][M+1])
//   thresholds s t                                        -> m_all m_null
//   schedule s t m cap                                    -> rc k:stage ... | blocks rc i i i
//   blocks n k:stage ...                                  -> rc i i i (ckpt_block_indices on a given list)
//   linearize n  deg.. (children of every node)  flags..  -> groups g.. common c..
//   sweep base num den count                              -> rc b..
//   layout L M                                            -> pitch rows elems index-of-(s,t)..
#include <cstdint>
#include <cstdio>
#include <iostream>
#include <string>
#include <vector>

#include "ckpt_dp.h"

extern "C" {
int oracle_solve_chain(int L, int M, const int32_t* uf, const int32_t* ub, const int32_t* wa, const int32_t* wab,
                       const int32_t* wd, const int32_t* of, const int32_t* ob, int32_t* cost, int16_t* choice,
                       int nthreads);
int64_t oracle_m_all(int L, const int32_t* wa, const int32_t* wab, const int32_t* wd, const int32_t* of,
                     const int32_t* ob, int s, int t);
int64_t oracle_m_null(int L, const int32_t* wa, const int32_t* wab, const int32_t* wd, const int32_t* of,
                      const int32_t* ob, int s, int t);
}

namespace {

std::vector<int32_t> read_ints(int n) {
    std::vector<int32_t> v(n);
    for (int& x : v) std::cin >> x;
    return v;
}

struct Chain {
    int L = 0, M = 0;
    std::vector<int32_t> uf, ub, wa, wab, wd, of, ob, cost;
    std::vector<int16_t> choice;
    std::vector<uint8_t> arg;  // the library's layout: [rows][pitch]
};

void print_blocks(const ckpt_op_t* ops, int n, int L) {
    std::vector<int32_t> blocks(L, -9);
    const int rc = ckpt_block_indices(ops, n, L, blocks.data());
    std::printf("blocks %d", rc);
    if (rc >= 0)
        for (int v : blocks) std::printf(" %d", v);
    std::printf("\n");
}

}  // namespace

int main() {
    Chain c;
    std::string cmd;
    while (std::cin >> cmd) {
        if (cmd == "chain") {
            std::cin >> c.L >> c.M;
            c.uf = read_ints(c.L); c.ub = read_ints(c.L); c.wa = read_ints(c.L + 1); c.wab = read_ints(c.L);
            c.wd = read_ints(c.L + 1); c.of = read_ints(c.L); c.ob = read_ints(c.L);
            const size_t cells = size_t(c.L) * c.L * (c.M + 1);
            c.cost.assign(cells, -1);
            c.choice.assign(cells, -1);
            const int rc = oracle_solve_chain(c.L, c.M, c.uf.data(), c.ub.data(), c.wa.data(), c.wab.data(),
                                              c.wd.data(), c.of.data(), c.ob.data(), c.cost.data(), c.choice.data(), 2);
            const size_t pitch = ckpt_row_pitch(c.M);
            c.arg.assign(ckpt_table_rows(c.L) * pitch, 0xEE);
            for (int s = 1; s <= c.L; ++s)
                for (int t = s; t <= c.L; ++t)
                    for (int m = 0; m <= c.M; ++m)
                        c.arg[size_t(ckpt_row_index(c.L, s, t)) * pitch + m] =
                            uint8_t(c.choice[(size_t(s - 1) * c.L + (t - 1)) * (c.M + 1) + m]);
            std::printf("chain %d\n", rc);
        } else if (cmd == "dump") {
            std::string pc, pk;
            std::cin >> pc >> pk;
            FILE* f = std::fopen(pc.c_str(), "wb");
            std::fwrite(c.cost.data(), sizeof(int32_t), c.cost.size(), f);
            std::fclose(f);
            f = std::fopen(pk.c_str(), "wb");
            std::fwrite(c.choice.data(), sizeof(int16_t), c.choice.size(), f);
            std::fclose(f);
            std::printf("dump %zu\n", c.cost.size());
        } else if (cmd == "thresholds") {
            int s, t;
            std::cin >> s >> t;
            std::printf("thresholds %lld %lld\n",
                        (long long)oracle_m_all(c.L, c.wa.data(), c.wab.data(), c.wd.data(), c.of.data(), c.ob.data(), s, t),
                        (long long)oracle_m_null(c.L, c.wa.data(), c.wab.data(), c.wd.data(), c.of.data(), c.ob.data(), s, t));
        } else if (cmd == "schedule") {
            int s, t, m, cap;
            std::cin >> s >> t >> m >> cap;
            std::vector<ckpt_op_t> ops(cap > 0 ? cap : 1);  // exactly cap entries: an overrun is a heap overflow
            const int rc = ckpt_schedule(c.arg.data(), c.wa.data(), c.wab.data(), c.L, c.M, s, t, m,
                                         cap > 0 ? ops.data() : ops.data(), cap);
            std::printf("schedule %d", rc);
            for (int k = 0; k < rc; ++k) std::printf(" %d:%d", ops[k].kind, ops[k].stage);
            std::printf("\n");
            if (rc > 0 && s == 1 && t == c.L) print_blocks(ops.data(), rc, c.L);
        } else if (cmd == "blocks") {
            int n, L;
            std::cin >> L >> n;
            std::vector<ckpt_op_t> ops(n > 0 ? n : 1);
            for (int k = 0; k < n; ++k) {
                int kind, stage;
                char colon;
                std::cin >> kind >> colon >> stage;
                ops[k].kind = uint8_t(kind);
                ops[k].stage = uint8_t(stage);
            }
            print_blocks(ops.data(), n, L);
        } else if (cmd == "linearize") {
            int n;
            std::cin >> n;
            std::vector<int32_t> ptr(n + 1, 0), idx;
            for (int v = 0; v < n; ++v) {
                int deg;
                std::cin >> deg;
                for (int e = 0; e < deg; ++e) {
                    int ch;
                    std::cin >> ch;
                    idx.push_back(ch);
                }
                ptr[v + 1] = int32_t(idx.size());
            }
            std::vector<uint8_t> flags(n > 0 ? n : 1);
            for (int v = 0; v < n; ++v) {
                int f;
                std::cin >> f;
                flags[v] = uint8_t(f);
            }
            std::vector<int32_t> group(n > 0 ? n : 1, -9);
            std::vector<uint8_t> common(n > 0 ? n : 1, 9);
            const int rc = ckpt_linearize(n, ptr.data(), idx.empty() ? nullptr : idx.data(), flags.data(), group.data(),
                                          common.data());
            std::printf("linearize %d groups", rc);
            for (int v = 0; v < n && rc >= 0; ++v) std::printf(" %d", group[v]);
            std::printf(" common");
            for (int v = 0; v < n && rc >= 0; ++v) std::printf(" %d", common[v]);
            std::printf("\n");
        } else if (cmd == "sweep") {
            long long base;
            int num, den, count;
            std::cin >> base >> num >> den >> count;
            std::vector<int64_t> out(count > 0 && count <= CKPT_MAX_SWEEP ? count : 1, -1);
            const int rc = ckpt_budget_sweep(base, num, den, count, out.data());
            std::printf("sweep %d", rc);
            for (size_t k = 0; k < out.size() && rc == 0; ++k) std::printf(" %lld", (long long)out[k]);
            std::printf("\n");
        } else if (cmd == "layout") {
            int L, M;
            std::cin >> L >> M;
            std::printf("layout %zu %zu %zu", ckpt_row_pitch(M), ckpt_table_rows(L), ckpt_table_elems(L, M, 3));
            for (int s = 0; s <= L + 1; ++s)
                for (int t = 0; t <= L + 1; ++t) std::printf(" %ld", ckpt_row_index(L, s, t));
            std::printf(" %s\n", ckpt_strerror(-7));
        } else {
            std::fprintf(stderr, "unknown command %s\n", cmd.c_str());
            return 2;
        }
    }
    return 0;
}
