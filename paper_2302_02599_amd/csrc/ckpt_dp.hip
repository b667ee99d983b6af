// Batched activation-checkpoint dynamic program on gfx950: kernels and C ABI.
//
// Computes C_BP(s, t, m) of the paper's Theorem (Section "Activation Checkpoint
// Solver / Modeling") for B chains at once.  See include/ckpt_dp.h for the
// conventions (candidate numbering, saturation at 2^30, table layout).
#include <hip/hip_runtime.h>

#include <array>
#include <atomic>
#include <utility>
#include <cstdint>
#include <cstring>
#include <vector>

#include "ckpt_dp.h"

namespace {

constexpr uint32_t kInf = 1u << 30;
std::atomic<int> g_last_hip_error{0};

inline bool hip_ok(hipError_t e) {
    if (e != hipSuccess) {
        g_last_hip_error.store(static_cast<int>(e));
        return false;
    }
    return true;
}

// ---------------------------------------------------------------------------
// How the table is filled
//
// Stages are 0-based inside this file: cell (i, j), 0 <= i <= j < L, is the paper's
// (s, t) = (i + 1, j + 1).  A checkpoint split q in i+1..j is the paper's s' = q + 1:
// left operand cell (i, q-1) at the same m, right operand cell (q, j) at m - omega_a^q,
// plus the forward sweep P[q] - P[i] (C_ck of the Theorem).  Its candidate number is q + 1.
//
// Stages are grouped in blocks of T.  Tile (I, J) holds the cells with i in block I and
// j in block J.  Tiles are processed by block diagonal D = J - I; within one D every
// tile is independent.  The splits of a cell of tile (I, J), D >= 2, fall in three groups:
//   middle   q in [(I+1)T, JT]: both operands lie in tiles of a smaller D.  This is a
//            min-plus product of an 8x8 register tile per lane (gemm_kernel), where each
//            loaded operand row is reused by 8 cells.
//   near-i   q in block I: the right operand (q, j) is a lower row of the SAME tile, read
//            at a shifted m, so rows must be finished bottom-up across launches.
//   near-j   q in block J: the left operand (i, q-1) is an earlier cell of the same row at
//            the same m, kept in registers.
// row_kernel finishes one row r of every tile of the diagonal: near-i splits, then the
// partial minimum of gemm_kernel, then near-j splits, then C_all and the two gates.
// Launch order per D: gemm (D >= 2), then rows r = T-1 .. 0.
//
// Reads at m - shift are not bounds-checked against m < shift: a lane whose m is below
// a shift of one of its splits is below m_null (m_all for C_all) of that cell, because
// both thresholds contain every shift of the cell, so the gate discards whatever it
// read.  Shifts are clamped to one row pitch, which keeps such reads inside the table.
// ---------------------------------------------------------------------------

// Workspace layout, all per chain b:
//   P     [B][L+1] int32   P[i] = sum of u_f of stages 1..i
//   fb    [B][L]   int32   min(2^30, u_f + u_b) of stage i+1
//   wsh   [B][L]   int32   shift of split q: omega_a^q clamped to [0, pitch]
//   wabs  [B][L]   int32   shift of C_all at row i: omega_abar^{i+1} clamped to [0, pitch]
//   mall  [B][L][L] int32  m_all^{s,t}  at [i*L + j]
//   mnull [B][L][L] int32  m_null^{s,t}
//   flags [B]      int32   input precondition flags
//   kq    [B][L]   double  P[q] + (q + 1) / 256: forward sweep up to split q, candidate number
//                          in the fraction bits
struct Workspace {
    int32_t* P;
    int32_t* fb;
    int32_t* wsh;
    int32_t* wabs;
    int32_t* mall;
    int32_t* mnull;
    int32_t* flags;
    double* kq;
};

inline size_t align64(size_t n) { return (n + 63) & ~size_t(63); }

inline size_t ws_ints(int L, int B) {
    return align64(size_t(B) * (L + 1)) + 3 * align64(size_t(B) * L) + 2 * align64(size_t(B) * L * L) +
           align64(size_t(B)) + 2 * align64(size_t(B) * L);
}

inline Workspace carve(void* base, int L, int B) {
    int32_t* p = static_cast<int32_t*>(base);
    Workspace w;
    w.P = p;      p += align64(size_t(B) * (L + 1));
    w.fb = p;     p += align64(size_t(B) * L);
    w.wsh = p;    p += align64(size_t(B) * L);
    w.wabs = p;   p += align64(size_t(B) * L);
    w.mall = p;   p += align64(size_t(B) * L * L);
    w.mnull = p;  p += align64(size_t(B) * L * L);
    w.flags = p;  p += align64(size_t(B));
    w.kq = reinterpret_cast<double*>(p);
    return w;
}

struct Ctx {
    int L, M, pitch, rows;
    Workspace ws;
    int32_t* cost;
    uint8_t* arg;
};

__host__ __device__ inline int tri_row(int L, int i, int j) {  // 0-based i <= j
    return i * L - (i * (i - 1)) / 2 + (j - i);
}

// One block per chain.  Thread 0 builds the prefix sums and the flags; thread i builds
// row i of both threshold tables with a running maximum over t (last display of the
// Theorem).
__global__ void precompute_kernel(ckpt_chains_t ch, int L, int pitch, Workspace ws) {
    const int b = blockIdx.x;
    const int32_t* uf = ch.uf + size_t(b) * L;
    const int32_t* ub = ch.ub + size_t(b) * L;
    const int32_t* wa = ch.wa + size_t(b) * (L + 1);
    const int32_t* wab = ch.wabar + size_t(b) * L;
    const int32_t* wd = ch.wdelta ? ch.wdelta + size_t(b) * (L + 1) : wa;
    const int32_t* of = ch.of ? ch.of + size_t(b) * L : nullptr;
    const int32_t* ob = ch.ob ? ch.ob + size_t(b) * L : nullptr;

    if (threadIdx.x == 0) {
        int flags = 0;
        long long acc = 0;
        int32_t* P = ws.P + size_t(b) * (L + 1);
        P[0] = 0;
        for (int k = 0; k < L; ++k) {
            const int f = uf[k], bw = ub[k];
            if (f < 0 || bw < 0) flags |= 1;
            if (bw >= (1 << 30)) flags |= 2;
            ws.kq[size_t(b) * L + k] = double(acc) + double(k + 1) * (1.0 / 256.0);
            acc += f > 0 ? f : 0;
            if (acc >= (1ll << 30)) { flags |= 2; acc = (1ll << 30) - 1; }
            P[k + 1] = static_cast<int32_t>(acc);
            ws.fb[size_t(b) * L + k] = static_cast<int32_t>(
                min(static_cast<long long>(kInf), static_cast<long long>(f > 0 ? f : 0) + (bw > 0 ? bw : 0)));
            ws.wsh[size_t(b) * L + k] = min(max(wa[k], 0), pitch);
            ws.wabs[size_t(b) * L + k] = min(max(wab[k], 0), pitch);
            const int sizes[5] = {wa[k + 1], wab[k], wd[k + 1], of ? of[k] : 0, ob ? ob[k] : 0};
            for (int v : sizes) {
                if (v < 0) flags |= 1;
                if (v > (1 << 28)) flags |= 4;
            }
        }
        if (wa[0] < 0 || wd[0] < 0) flags |= 1;
        if (wa[0] > (1 << 28) || wd[0] > (1 << 28)) flags |= 4;
        ws.flags[b] = flags;
    }
    // Clamp sizes into [0, 2^28] so that thresholds of a bad chain cannot overflow.
    auto sz = [](int v) { return min(max(v, 0), 1 << 28); };
    for (int s0 = threadIdx.x; s0 < L; s0 += blockDim.x) {
        const int s = s0 + 1;
        const int ofs = of ? sz(of[s0]) : 0, obs = ob ? sz(ob[s0]) : 0;
        int sweep = sz(wa[s]) + ofs;  // omega_a^s + o_f^s, then max over s+1 <= j < t
        int32_t* mall = ws.mall + (size_t(b) * L + s0) * L;
        int32_t* mnull = ws.mnull + (size_t(b) * L + s0) * L;
        for (int t = s; t <= L; ++t) {
            if (t >= s + 2) {
                const int j = t - 1;
                sweep = max(sweep, sz(wa[j - 1]) + sz(wa[j]) + (of ? sz(of[j - 1]) : 0));
            }
            mall[t - 1] = max(sz(wd[t]) + sz(wab[s0]) + ofs, sz(wd[s]) + sz(wab[s0]) + obs);
            mnull[t - 1] = sz(wd[t]) + sweep;
        }
    }
}

// Table reads go through a raw buffer descriptor of the chain's cost table: the address
// is descriptor base + per-lane byte offset (vector register, fixed for the whole kernel)
// + wave-uniform byte offset of the row (scalar register), so no vector instruction is
// spent on addressing, and a read outside the chain's table returns 0 instead of faulting.
// The scalar offset is 32-bit: a chain's table must stay below 4 GiB (checked on the host).
using rsrc_t = __amdgpu_buffer_rsrc_t;

__device__ __forceinline__ rsrc_t table_rsrc(const int32_t* tab, uint32_t bytes) {
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<int32_t*>(tab), 0, int(bytes), 0x00020000);
}

__device__ __forceinline__ uint32_t ld32(rsrc_t tab, uint32_t elem, uint32_t off) {
    return uint32_t(__builtin_amdgcn_raw_buffer_load_b32(tab, int(off), int(elem << 2), 0));
}

// Middle splits of every tile of block diagonal D >= 2 (also correct for D = 1).
// One wave owns an 8x8 sub-tile of cells for 64 consecutive m; lane = m.  For T = 16 the
// four waves of a work-group cover the 16x16 tile and share operand rows through L1/L2.
// Candidates are compared as float64 keys  cost + (q+1)/256 : one add and one min per
// candidate give the minimum cost and, among equal costs, the smallest candidate number
// (all values are integers below 2^34 scaled by 2^-8, exact in float64).
// Output: cost[] <- unsaturated partial minimum, arg[] <- its candidate number.
template <int T, int NB, int UNR>
__global__ void __launch_bounds__(64 * (T / 8) * (T / 8), 2) gemm_kernel(Ctx c, int D) {
    constexpr bool XCD = false;
    constexpr int W = T / 8;
    // NB operand buffers in flight: loads run NB-1 splits ahead
    const int wave = __builtin_amdgcn_readfirstlane(int(threadIdx.x >> 6));
    const int rw = wave / W, cw = wave % W;
    int bx = blockIdx.x, by = blockIdx.y, bz = blockIdx.z;
    if (XCD) {
        // Work-groups go round-robin to the 8 XCDs in dispatch order.  Renumber them so that
        // each XCD works on a contiguous range of (chain, tile, m-chunk).
        const uint32_t n = gridDim.x * gridDim.y * gridDim.z;
        const uint32_t id = blockIdx.x + gridDim.x * (blockIdx.y + gridDim.y * blockIdx.z);
        const uint32_t per = n / 8, main = per * 8;
        const uint32_t lid = id < main ? (id % 8) * per + id / 8 : id;
        bx = lid % gridDim.x;
        by = (lid / gridDim.x) % gridDim.y;
        bz = lid / (gridDim.x * gridDim.y);
    }
    const int b = bz, I = by, J = I + D;
    const int L = c.L, pitch = c.pitch;
    const int qlo = (I + 1) * T, qhi = J * T;

    // Per-split constants (shift, key offset) go through LDS once: a scalar memory load per
    // split would put its full latency on the critical path of every pipeline step.
    __shared__ double s_kq[CKPT_MAX_L + 2];
    __shared__ int32_t s_sh[CKPT_MAX_L + 2];
    for (int k = threadIdx.x; k <= qhi - qlo; k += blockDim.x) {
        s_kq[k] = c.ws.kq[size_t(b) * L + qlo + k];
        s_sh[k] = c.ws.wsh[size_t(b) * L + qlo + k];
    }
    __syncthreads();

    const int j0 = J * T + cw * 8;
    if (j0 >= L) return;  // ragged last block: this sub-tile has no column
    const int i0 = I * T + rw * 8;
    const uint32_t m = bx * 64 + (threadIdx.x & 63);
    const uint32_t moff = m * 4;
    const size_t chain = size_t(b) * c.rows * pitch;
    const rsrc_t tab = table_rsrc(c.cost + chain, uint32_t(c.rows) * uint32_t(pitch) * 4u);

    int lrow0[8], jcol[8];
#pragma unroll
    for (int r = 0; r < 8; ++r) lrow0[r] = tri_row(L, i0 + r, i0 + r) - (i0 + r) - 1;  // + q = row of (i, q-1)
#pragma unroll
    for (int cc = 0; cc < 8; ++cc) jcol[cc] = min(j0 + cc, L - 1);

    double key[8][8];
#pragma unroll
    for (int r = 0; r < 8; ++r)
#pragma unroll
        for (int cc = 0; cc < 8; ++cc) key[r][cc] = 0x1p60;

    uint32_t buf[NB][16];
    auto load = [&](uint32_t(&v)[16], int q) {
        const int rq = q * L - (q * (q - 1)) / 2 - q;  // + j = row of (q, j)
        const int sh = __builtin_amdgcn_readfirstlane(s_sh[q - qlo]);
#pragma unroll
        for (int r = 0; r < 8; ++r) v[r] = ld32(tab, uint32_t(lrow0[r] + q) * uint32_t(pitch), moff);
#pragma unroll
        for (int cc = 0; cc < 8; ++cc)
            v[8 + cc] = ld32(tab, uint32_t(rq + jcol[cc]) * uint32_t(pitch) - uint32_t(sh), moff);
    };
    auto compute = [&](const uint32_t(&v)[16], int q) {
        const double cq = s_kq[q - qlo];
        double lk[8], rk[8];
#pragma unroll
        for (int r = 0; r < 8; ++r) lk[r] = double(v[r]);
#pragma unroll
        for (int cc = 0; cc < 8; ++cc) rk[cc] = double(v[8 + cc]) + cq;
#pragma unroll
        for (int r = 0; r < 8; ++r)
#pragma unroll
            for (int cc = 0; cc < 8; ++cc) key[r][cc] = fmin(key[r][cc], lk[r] + rk[cc]);
    };

    // Straight-line pipeline: the split list is padded to a multiple of NB by repeating the
    // last split (a repeated candidate cannot change a minimum), so the loop body has no
    // branches and the loads of split q + 2 are in flight while split q is evaluated.
#pragma unroll
    for (int u = 0; u < NB - 1; ++u) load(buf[u], min(qlo + u, qhi));
    constexpr int STEPS = NB * UNR;  // pipeline steps per loop iteration
    const int iters = (qhi - qlo + STEPS) / STEPS;
    int q = qlo;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int u = 0; u < STEPS; ++u) {
            load(buf[(u + NB - 1) % NB], min(q + NB - 1, qhi));
            __builtin_amdgcn_sched_barrier(0);  // keep the loads of split q+NB-1 ahead of the math of split q
            compute(buf[u % NB], min(q, qhi));
            __builtin_amdgcn_sched_barrier(0);
            ++q;
        }
    }

    const int32_t* P = c.ws.P + size_t(b) * (L + 1);
#pragma unroll
    for (int r = 0; r < 8; ++r) {
        const uint32_t Pi = P[i0 + r];
        const size_t row = chain + size_t(tri_row(L, i0 + r, j0)) * pitch + m;
#pragma unroll
        for (int cc = 0; cc < 8; ++cc) {
            if (j0 + cc < L) {
                const double k = fmin(key[r][cc], 0x1p33);
                const double fl = floor(k);
                c.cost[row + size_t(cc) * pitch] = int32_t(uint32_t(fl) - Pi);
                c.arg[row + size_t(cc) * pitch] = uint8_t(uint32_t((k - fl) * 256.0));
            }
        }
    }
}

// Finishes row R of every tile of block diagonal D: cells (i, j), i = I*T + R, j in block
// J = I + D.  One lane per m.  Candidate order = candidate number order, strict '<' keeps
// the smallest number among equal costs: near-i splits, gemm partial, near-j splits; C_all
// (number i + 1, the smallest) wins ties at the end.
// R and the diagonal class DC (0: D = 0, 1: D = 1, 2: D >= 2) are compile-time so that every
// trip count is static: all operand addresses are known up front, the loads are issued
// together and the kernel pays the memory latency once instead of once per split.
template <int T, int R, int DC>
__global__ void __launch_bounds__(256) row_kernel(Ctx c, int D) {
    constexpr int CF = (DC == 0) ? R : 0;                              // first column with j >= i
    constexpr int NQ = (DC == 0) ? 0 : (DC == 1 ? T - R : T - 1 - R);  // near-i splits (D = 1: and q = jb)
    constexpr int NQA = NQ > 0 ? NQ : 1;
    const int b = blockIdx.z, I = blockIdx.y, J = I + D;
    const int L = c.L, pitch = c.pitch;
    const int i = I * T + R;
    if (i >= L) return;
    const uint32_t m = blockIdx.x * 256 + threadIdx.x;
    if (m >= uint32_t(pitch)) return;
    const uint32_t moff = m * 4;
    const size_t chain = size_t(b) * c.rows * pitch;
    const rsrc_t tab = table_rsrc(c.cost + chain, uint32_t(c.rows) * uint32_t(pitch) * 4u);
    const int32_t* P = c.ws.P + size_t(b) * (L + 1);
    const int32_t* wsh = c.ws.wsh + size_t(b) * L;
    const int32_t* mall = c.ws.mall + (size_t(b) * L + i) * L;
    const int32_t* mnull = c.ws.mnull + (size_t(b) * L + i) * L;
    const int jb = J * T;
    const int cend = min(T, L - jb);  // columns of this tile that exist
    const uint32_t Pi = P[i];
    const uint32_t fbi = c.ws.fb[size_t(b) * L + i];
    const uint32_t wabi = c.ws.wabs[size_t(b) * L + i];
    const int rowi = tri_row(L, i, i) - i;  // + j = row of (i, j)
    auto rowq = [&](int q) { return q * L - (q * (q - 1)) / 2 - q; };  // + j = row of (q, j)

    // Columns past the end of a ragged last block are computed on a clamped j and not stored.
    int jc[T];
#pragma unroll
    for (int cc = 0; cc < T; ++cc) jc[cc] = min(jb + cc, L - 1);

    // ---- every load of this row, issued before anything is consumed ----
    uint32_t nl[NQA], nr[NQA][T];   // near-i: left (i, q-1) and right (q, j) at m - omega_a^q
#pragma unroll
    for (int u = 0; u < NQ; ++u) {
        const int q = i + 1 + u;
        const uint32_t rq = uint32_t(rowq(q)), sh = uint32_t(wsh[q]);
        nl[u] = ld32(tab, uint32_t(rowi + q - 1) * uint32_t(pitch), moff);
#pragma unroll
        for (int cc = 0; cc < T; ++cc) nr[u][cc] = ld32(tab, (rq + jc[cc]) * uint32_t(pitch) - sh, moff);
    }
    uint32_t pc[T], pp[T];  // gemm partial
    if (DC == 2) {
#pragma unroll
        for (int cc = 0; cc < T; ++cc) {
            const size_t o = chain + size_t(rowi + jc[cc]) * pitch + m;
            pc[cc] = uint32_t(c.cost[o]);
            pp[cc] = c.arg[o];
        }
    }
    uint32_t tj[T][T];  // near-j: right (jb + c2 + 1, j) at its shift, for CF <= c2 < cc
#pragma unroll
    for (int cc = CF + 1; cc < T; ++cc)
#pragma unroll
        for (int c2 = CF; c2 < cc; ++c2) {
            const int q = min(jb + c2 + 1, L - 1);
            tj[c2][cc] = ld32(tab, uint32_t(rowq(q) + jc[cc]) * uint32_t(pitch) - uint32_t(wsh[q]), moff);
        }
    uint32_t al[T];  // C_all: right (i + 1, j) at m - omega_abar^{i+1}
#pragma unroll
    for (int cc = CF; cc < T; ++cc) {
        const int i1 = min(i + 1, L - 1);
        al[cc] = ld32(tab, uint32_t(rowq(i1) + max(jc[cc], i1)) * uint32_t(pitch) - wabi, moff);
    }

    // ---- evaluation ----
    uint32_t best[T], pick[T], val[T];
#pragma unroll
    for (int cc = 0; cc < T; ++cc) best[cc] = 0xffffffffu, pick[cc] = 0, val[cc] = kInf;
#pragma unroll
    for (int u = 0; u < NQ; ++u) {
        const int q = i + 1 + u;
        const uint32_t lb = nl[u] + (uint32_t(P[q]) - Pi);
#pragma unroll
        for (int cc = 0; cc < T; ++cc) {
            const uint32_t v = lb + nr[u][cc];
            if (v < best[cc]) best[cc] = v, pick[cc] = q + 1;
        }
    }
    if (DC == 2) {
#pragma unroll
        for (int cc = 0; cc < T; ++cc)
            if (pc[cc] < best[cc]) best[cc] = pc[cc], pick[cc] = pp[cc];
    }
#pragma unroll
    for (int cc = CF; cc < T; ++cc) {
        const int j = jc[cc];
#pragma unroll
        for (int c2 = CF; c2 < cc; ++c2) {
            const int q = min(jb + c2 + 1, L - 1);  // left operand (i, q-1) = val[c2]
            const uint32_t v = val[c2] + (uint32_t(P[q]) - Pi) + tj[c2][cc];
            if (v < best[cc]) best[cc] = v, pick[cc] = q + 1;
        }
        const uint32_t ck = (m >= uint32_t(mnull[j])) ? min(best[cc], kInf) : kInf;
        uint32_t all = fbi;
        if (DC != 0 || cc > CF) all += al[cc];  // j > i
        all = (m >= uint32_t(mall[j])) ? min(all, kInf) : kInf;
        const bool take_all = all < kInf && all <= ck;
        const uint32_t fin = take_all ? all : ck;
        const uint32_t fpk = take_all ? uint32_t(i + 1) : (ck < kInf ? pick[cc] : 0u);
        val[cc] = fin;
        if (cc < cend) {
            const size_t o = chain + size_t(rowi + j) * pitch + m;
            c.cost[o] = int32_t(fin);
            c.arg[o] = uint8_t(fpk);
        }
    }
}

using RowFn = void (*)(Ctx, int);
template <int T, int DC, int... Rs>
constexpr std::array<RowFn, sizeof...(Rs)> row_table(std::integer_sequence<int, Rs...>) {
    return {{row_kernel<T, Rs, DC>...}};
}
constexpr int kT = 8;  // stage-block size
const std::array<RowFn, kT> kRow0 = row_table<kT, 0>(std::make_integer_sequence<int, kT>{});
const std::array<RowFn, kT> kRow1 = row_table<kT, 1>(std::make_integer_sequence<int, kT>{});
const std::array<RowFn, kT> kRow2 = row_table<kT, 2>(std::make_integer_sequence<int, kT>{});

std::atomic<int> g_tile{0};  // 0 = choose automatically

int check_dims(int L, int M, int B) {
    if (L < 1 || M < 0 || B < 1) return CKPT_E_ARG;
    if (L > CKPT_MAX_L) return CKPT_E_LIMIT;
    const unsigned long long per_chain = (unsigned long long)ckpt_table_rows(L) * ckpt_row_pitch(M);
    if (per_chain >= (1ull << 30)) return CKPT_E_LIMIT;  // 4 GiB of int32 per chain
    return CKPT_OK;
}

// Optional per-launch event trail of ckpt_solve_profiled.
struct Profile {
    hipStream_t stream = nullptr;
    std::vector<hipEvent_t> events;
    std::vector<int> kinds;
    bool mark(int kind) {
        hipEvent_t e;
        if (!hip_ok(hipEventCreate(&e))) return false;
        events.push_back(e);
        kinds.push_back(kind);
        return hip_ok(hipEventRecord(e, stream));
    }
};

#define CKPT_AFTER_LAUNCH(kind)                                   \
    do {                                                          \
        if (!hip_ok(hipGetLastError())) return CKPT_E_HIP;        \
        if (prof && !prof->mark(kind)) return CKPT_E_HIP;         \
    } while (0)

int solve_impl(const ckpt_chains_t* chains, int L, int M, int B, void* stream, int32_t* cost, uint8_t* arg,
               void* workspace, Profile* prof) {
    if (!chains || !cost || !arg || !workspace) return CKPT_E_ARG;
    if (int rc = check_dims(L, M, B)) return rc;
    if (!chains->uf || !chains->ub || !chains->wa || !chains->wabar) return CKPT_E_ARG;
    if ((reinterpret_cast<uintptr_t>(cost) | reinterpret_cast<uintptr_t>(arg) |
         reinterpret_cast<uintptr_t>(workspace)) & 255)
        return CKPT_E_ARG;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int pitch = int(ckpt_row_pitch(M));
    const int rows = int(ckpt_table_rows(L));
    const Workspace ws = carve(workspace, L, B);

    hipLaunchKernelGGL(precompute_kernel, dim3(B), dim3(64), 0, st, *chains, L, pitch, ws);
    CKPT_AFTER_LAUNCH(CKPT_K_PRECOMPUTE);
    const Ctx ctx{L, M, pitch, rows, ws, cost, arg};
    constexpr int T = kT;
    const int nblk = (L + T - 1) / T;
    const int gx_gemm = pitch / 64, gx_row = (pitch + 255) / 256;
    for (int D = 0; D < nblk; ++D) {
        const dim3 tiles_gemm(gx_gemm, nblk - D, B), tiles_row(gx_row, nblk - D, B);
        if (D >= 2) {
            switch (g_tile.load()) {  // experiment selector
                case 1: hipLaunchKernelGGL((gemm_kernel<T, 3, 2>), tiles_gemm, dim3(64), 0, st, ctx, D); break;
                case 2: hipLaunchKernelGGL((gemm_kernel<T, 3, 3>), tiles_gemm, dim3(64), 0, st, ctx, D); break;
                case 3: hipLaunchKernelGGL((gemm_kernel<T, 2, 4>), tiles_gemm, dim3(64), 0, st, ctx, D); break;
                default: hipLaunchKernelGGL((gemm_kernel<T, 3, 1>), tiles_gemm, dim3(64), 0, st, ctx, D); break;
            }
            CKPT_AFTER_LAUNCH(CKPT_K_GEMM);
        }
        const auto& rowfn = D == 0 ? kRow0 : (D == 1 ? kRow1 : kRow2);
        for (int r = T - 1; r >= 0; --r) {
            hipLaunchKernelGGL(rowfn[r], tiles_row, dim3(256), 0, st, ctx, D);
            CKPT_AFTER_LAUNCH(CKPT_K_ROW);
        }
    }
    return CKPT_OK;
}

}  // namespace

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

size_t ckpt_workspace_bytes(int L, int M, int B) {
    if (L < 1 || M < 0 || B < 1) return 0;
    return ws_ints(L, B) * sizeof(int32_t);
}

int ckpt_solve_batched(const ckpt_chains_t* chains, int L, int M, int B, void* stream, int32_t* cost,
                       uint8_t* arg, void* workspace) {
    return solve_impl(chains, L, M, B, stream, cost, arg, workspace, nullptr);
}

int ckpt_solve_profiled(const ckpt_chains_t* chains, int L, int M, int B, void* stream, int32_t* cost,
                        uint8_t* arg, void* workspace, float* kind_ms, int* kind_launches) {
    if (!kind_ms || !kind_launches) return CKPT_E_ARG;
    hipStream_t st = static_cast<hipStream_t>(stream);
    Profile prof;
    prof.stream = st;
    for (int k = 0; k < CKPT_N_KERNEL_KINDS; ++k) kind_ms[k] = 0.f, kind_launches[k] = 0;
    int rc = CKPT_OK;
    if (!prof.mark(-1)) rc = CKPT_E_HIP;
    if (rc == CKPT_OK) rc = solve_impl(chains, L, M, B, stream, cost, arg, workspace, &prof);
    if (!hip_ok(hipStreamSynchronize(st)) && rc == CKPT_OK) rc = CKPT_E_HIP;
    for (size_t i = 1; i < prof.events.size() && rc == CKPT_OK; ++i) {
        float ms = 0.f;
        if (!hip_ok(hipEventElapsedTime(&ms, prof.events[i - 1], prof.events[i]))) rc = CKPT_E_HIP;
        kind_ms[prof.kinds[i]] += ms;
        kind_launches[prof.kinds[i]] += 1;
    }
    for (hipEvent_t e : prof.events) (void)hipEventDestroy(e);
    return rc;
}

const char* ckpt_kernel_name(int kind) {
    switch (kind) {
        case CKPT_K_PRECOMPUTE: return "precompute_kernel";
        case CKPT_K_GEMM: return "gemm_kernel";
        case CKPT_K_ROW: return "row_kernel";
        default: return nullptr;
    }
}

int ckpt_check_inputs(const void* workspace, int L, int M, int B, void* stream, int32_t* flags_host) {
    if (!workspace || !flags_host) return CKPT_E_ARG;
    if (int rc = check_dims(L, M, B)) return rc;
    const Workspace ws = carve(const_cast<void*>(workspace), L, B);
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (!hip_ok(hipMemcpyAsync(flags_host, ws.flags, size_t(B) * sizeof(int32_t), hipMemcpyDeviceToHost, st)))
        return CKPT_E_HIP;
    if (!hip_ok(hipStreamSynchronize(st))) return CKPT_E_HIP;
    for (int b = 0; b < B; ++b)
        if (flags_host[b]) return CKPT_E_INPUT;
    return CKPT_OK;
}

int ckpt_last_hip_error(void) { return g_last_hip_error.load(); }

int ckpt_set_tile(int T) {
    if (T < 0 || T > 16) return CKPT_E_ARG;
    return g_tile.exchange(T);
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
        case CKPT_E_CORRUPT: return "arg table is inconsistent";
        default: return "unknown error";
    }
}

}  // extern "C"
