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
#include <algorithm>
#include <mutex>
#include <type_traits>
#include <vector>

#include "ckpt_dp.h"

namespace {

constexpr uint32_t kInf = 1u << 30;
constexpr int kT = 8;  // stage-block size of the fill
constexpr int kCH = 4;  // 64-column chunks of m per gemm work-group
constexpr int kRowWG = 256;  // threads (columns of m) per work-group of the row kernels
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
//   need  [B][L][L] int32  feasibility frontier: smallest m at which cell (i, j) can be finite
//   kq    [B][L]   double  P[q] + (q + 1) / 256: forward sweep up to split q, candidate number
//                          in the fraction bits
//   prog  [B][tiles][chunks] int32  rows of tile (I, J) finished by tile_rows_kernel for the chunk
//                          of 64 columns; tiles = nblk (nblk + 1) / 2, chunks = pitch / 64
//   tick  [nblk][4] int32  ticket counter of the tile_rows_kernel launch of diagonal D, group g
//   fault [1]      int32   set when a bounded wait inside tile_rows_kernel expired
// prog, tick and fault are cleared by precompute_kernel at the start of every solve.
struct Workspace {
    int32_t* P;
    int32_t* fb;
    int32_t* wsh;
    int32_t* wabs;
    int32_t* mall;
    int32_t* mnull;
    int32_t* flags;
    int32_t* need;
    double* kq;
    int32_t* prog;
    int32_t* tick;
    int32_t* fault;
};

constexpr int kBand = kRowWG;  // columns of m per work-group of the row kernels
constexpr int kTickGroups = 4;

inline size_t align64(size_t n) { return (n + 63) & ~size_t(63); }
__host__ __device__ inline int blocks_of(int L) { return (L + kT - 1) / kT; }
__host__ __device__ inline size_t tiles_of(int L) { return size_t(blocks_of(L)) * (blocks_of(L) + 1) / 2; }
__host__ __device__ inline int bands_of(int pitch) { return (pitch + kBand - 1) / kBand; }
// index of tile (I, J), I <= J, in the row-major packed block triangle
__host__ __device__ inline int tile_index(int nblk, int I, int J) { return I * nblk - (I * (I - 1)) / 2 + (J - I); }

inline size_t ws_ints(int L, int pitch, int B) {
    return align64(size_t(B) * (L + 1)) + 3 * align64(size_t(B) * L) + 3 * align64(size_t(B) * L * L) +
           align64(size_t(B)) + 2 * align64(size_t(B) * L) + align64(size_t(B) * tiles_of(L) * (pitch / 64)) +
           align64(size_t(blocks_of(L)) * kTickGroups) + 64;
}

inline Workspace carve(void* base, int L, int pitch, int B) {
    int32_t* p = static_cast<int32_t*>(base);
    Workspace w;
    w.P = p;      p += align64(size_t(B) * (L + 1));
    w.fb = p;     p += align64(size_t(B) * L);
    w.wsh = p;    p += align64(size_t(B) * L);
    w.wabs = p;   p += align64(size_t(B) * L);
    w.mall = p;   p += align64(size_t(B) * L * L);
    w.mnull = p;  p += align64(size_t(B) * L * L);
    w.flags = p;  p += align64(size_t(B));
    w.need = p;   p += align64(size_t(B) * L * L);
    w.kq = reinterpret_cast<double*>(p);  p += 2 * align64(size_t(B) * L);
    w.prog = p;   p += align64(size_t(B) * tiles_of(L) * (pitch / 64));
    w.tick = p;   p += align64(size_t(blocks_of(L)) * kTickGroups);
    w.fault = p;
    return w;
}

struct Ctx {
    int L, M, pitch, rows;
    int b0;  // first chain of this launch; blockIdx.z counts from it
    int spin_limit;  // polls before a wait between work-groups gives up; < 0: every such wait gives up at once
    Workspace ws;
    int32_t* cost;
    uint8_t* arg;
    // measurement only (ckpt_solve_profiled), else null: kWorkSets sets of four counters, [0] bytes
    // of table loads the gemm's waves asked for, [1] bytes they stored, [2], [3] the same for the
    // row kernel; a wave adds to the set its position selects, the host sums the sets
    unsigned long long* work;
};
constexpr int kWorkSets = 256;

// One lane per wave adds the wave's byte counts (per lane 4 bytes a load, 5 a stored cell).
template <bool CNT>
__device__ __forceinline__ void count_work(unsigned long long* work, int slot, unsigned loads, unsigned cells) {
    if constexpr (!CNT) return;  // the counting variants are separate instantiations: no cost otherwise
    if (work && (threadIdx.x & 63) == 0) {
        const unsigned set = (blockIdx.x * 7u + blockIdx.y * 13u + blockIdx.z * 29u + (threadIdx.x >> 6)) % kWorkSets;
        atomicAdd(work + set * 4 + slot, 256ull * loads);
        atomicAdd(work + set * 4 + slot + 1, 320ull * cells);
    }
}

__host__ __device__ inline int tri_row(int L, int i, int j) {  // 0-based i <= j
    return i * L - (i * (i - 1)) / 2 + (j - i);
}

// One block per chain: input checks, prefix sums, shifts and both threshold tables (last
// display of the Theorem).
__global__ void __launch_bounds__(256) precompute_kernel(ckpt_chains_t ch, int L, int pitch, Workspace ws) {
    const int b = blockIdx.x;
    const int tid = threadIdx.x;
    const int32_t* uf = ch.uf + size_t(b) * L;
    const int32_t* ub = ch.ub + size_t(b) * L;
    const int32_t* wa = ch.wa + size_t(b) * (L + 1);
    const int32_t* wab = ch.wabar + size_t(b) * L;
    const int32_t* wd = ch.wdelta ? ch.wdelta + size_t(b) * (L + 1) : wa;
    const int32_t* of = ch.of ? ch.of + size_t(b) * L : nullptr;
    const int32_t* ob = ch.ob ? ch.ob + size_t(b) * L : nullptr;
    __shared__ int s_flags;
    __shared__ int32_t s_uf[CKPT_MAX_L + 2];
    if (tid == 0) s_flags = 0;
    {   // progress flags of this chain's tiles, and (first block) the ticket counters and the fault word
        const size_t n = tiles_of(L) * (pitch / 64);
        for (size_t k = tid; k < n; k += blockDim.x) ws.prog[size_t(b) * n + k] = 0;
        if (b == 0) {
            for (int k = tid; k < blocks_of(L) * kTickGroups; k += blockDim.x) ws.tick[k] = 0;
            if (tid == 0) ws.fault[0] = 0;
        }
    }
    __syncthreads();

    // Sizes are clamped into [0, 2^28] so that thresholds of a bad chain cannot overflow.
    auto sz = [](int v) { return min(max(v, 0), 1 << 28); };
    for (int k = tid; k < L; k += blockDim.x) {
        const int f = uf[k], bw = ub[k];
        int flags = 0;
        if (f < 0 || bw < 0) flags |= 1;
        if (f >= (1 << 30) || bw >= (1 << 30)) flags |= 2;
        const int fc = min(max(f, 0), (1 << 30) - 1), bc = min(max(bw, 0), 1 << 30);
        s_uf[k] = fc;
        ws.fb[size_t(b) * L + k] = int32_t(min(kInf, uint32_t(fc) + uint32_t(bc)));
        ws.wsh[size_t(b) * L + k] = min(max(wa[k], 0), pitch);
        ws.wabs[size_t(b) * L + k] = min(max(wab[k], 0), pitch);
        const int sizes[5] = {wa[k + 1], wab[k], wd[k + 1], of ? of[k] : 0, ob ? ob[k] : 0};
        for (int v : sizes) {
            if (v < 0) flags |= 1;
            if (v > (1 << 28)) flags |= 4;
        }
        if (wab[k] < wa[k + 1]) flags |= 8;  // abar^k must contain a^k: outside the Theorem's model
        if (k == 0) {
            if (wa[0] < 0 || wd[0] < 0) flags |= 1;
            if (wa[0] > (1 << 28) || wd[0] > (1 << 28)) flags |= 4;
        }
        if (flags) atomicOr(&s_flags, flags);
    }
    __syncthreads();
    if (tid == 0) {
        int flags = s_flags;
        long long acc = 0;
        int32_t* P = ws.P + size_t(b) * (L + 1);
        P[0] = 0;
        for (int k = 0; k < L; ++k) {
            ws.kq[size_t(b) * L + k] = double(acc) + double(k + 1) * (1.0 / 256.0);
            acc += s_uf[k];
            if (acc >= (1ll << 30)) { flags |= 2; acc = (1ll << 30) - 1; }
            P[k + 1] = int32_t(acc);
        }
        ws.flags[b] = flags;
    }
    // thresholds: sizes staged in LDS, thread s builds row s with a running maximum over t
    __shared__ int32_t s_wa[CKPT_MAX_L + 2], s_wd[CKPT_MAX_L + 2], s_of[CKPT_MAX_L + 2];
    for (int k = tid; k <= L; k += blockDim.x) {
        s_wa[k] = sz(wa[k]);
        s_wd[k] = sz(wd[k]);
        s_of[k] = (of && k < L) ? sz(of[k]) : 0;
    }
    __syncthreads();
    for (int s0 = tid; s0 < L; s0 += blockDim.x) {
        const int s = s0 + 1;
        const int ofs = s_of[s0], obs = ob ? sz(ob[s0]) : 0, abar = sz(wab[s0]);
        int sweep = s_wa[s] + ofs;  // omega_a^s + o_f^s, then max over s+1 <= j < t
        int32_t* mall = ws.mall + (size_t(b) * L + s0) * L;
        int32_t* mnull = ws.mnull + (size_t(b) * L + s0) * L;
        int32_t* need = ws.need + (size_t(b) * L + s0) * L;
        for (int t = s; t <= L; ++t) {
            if (t >= s + 2) {
                const int j = t - 1;
                sweep = max(sweep, s_wa[j - 1] + s_wa[j] + s_of[j - 1]);
            }
            const int keep = max(s_wd[t] + abar + ofs, s_wd[s] + abar + obs), ck = s_wd[t] + sweep;
            mall[t - 1] = keep;
            mnull[t - 1] = ck;
            // A first, weak feasibility frontier: a finite cell passes at least one of its two gates.
            // The frontier kernel overwrites it with the exact one while the fill already runs;
            // whichever value a reader sees is a valid lower bound.
            need[t - 1] = min(keep, ck);
        }
    }
}

// Feasibility frontier need[i][j] = smallest m at which cell (i, j) can be finite: the
// recurrence with costs dropped.  A leaf needs m_all; keeping abar^s needs
// max(m_all, omega_abar^s + need(s+1, t)); a checkpoint split at q needs
// max(m_null, omega_a^q + need(q, t), need(s, q-1)).  A cell below its frontier is infeasible
// whatever the times are, so the fill kernels skip work there.  Values saturate at 2^30,
// above any admissible M.  One block per chain, one segment length at a time; the triangle
// lives in LDS (row-major packed, L(L+1)/2 ints <= 127 KiB); 16 lanes share the splits of a cell.
__global__ void __launch_bounds__(1024) frontier_kernel(ckpt_chains_t ch, int L, Workspace ws) {
    const int b = blockIdx.x;
    const int tid = threadIdx.x;
    const int32_t* wa = ch.wa + size_t(b) * (L + 1);
    const int32_t* wab = ch.wabar + size_t(b) * L;
    auto sz = [](int v) { return min(max(v, 0), 1 << 28); };
    extern __shared__ int32_t s_need[];
    __shared__ int32_t s_wa[CKPT_MAX_L + 2];
    __shared__ int32_t s_wab[CKPT_MAX_L + 2];
    for (int k = tid; k <= L; k += blockDim.x) s_wa[k] = sz(wa[k]);
    for (int k = tid; k < L; k += blockDim.x) s_wab[k] = sz(wab[k]);
    int32_t* need = ws.need + size_t(b) * L * L;
    const int32_t* mallb = ws.mall + size_t(b) * L * L;
    const int32_t* mnullb = ws.mnull + size_t(b) * L * L;
    constexpr int kSat = 1 << 30;
    const int g = tid & 15, cells_per_pass = blockDim.x >> 4;
    __syncthreads();
    for (int d = 0; d < L; ++d) {
        for (int base = 0; base + d < L; base += cells_per_pass) {
            const int i = base + (tid >> 4), j = i + d;
            const bool valid = j < L;
            int split = kSat;
            int keep = 0, sweep = 0;
            if (valid && g == 0) keep = mallb[i * L + j], sweep = mnullb[i * L + j];  // in flight during the loop
            if (valid) {
                const int rowi = tri_row(L, i, i) - i;  // + j' = index of (i, j')
                for (int q = i + 1 + g; q <= j; q += 16)
                    split = min(split, max(min(kSat, s_wa[q] + s_need[tri_row(L, q, j)]), s_need[rowi + q - 1]));
            }
#pragma unroll
            for (int o = 8; o > 0; o >>= 1) split = min(split, __shfl_xor(split, o));
            if (valid && g == 0) {
                int nd = keep;
                if (d > 0) {
                    const int opt_all = max(keep, min(kSat, s_wab[i] + s_need[tri_row(L, i + 1, j)]));
                    nd = min(opt_all, max(sweep, split));
                }
                nd = min(nd, kSat);
                s_need[tri_row(L, i, j)] = nd;
                need[i * L + j] = nd;
            }
        }
        __syncthreads();
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

// Which (chunk of m, tile, chain) a work-group takes.  The hardware hands work-groups out in
// linear order and to the 8 XCDs round-robin, and the cost of a chunk grows with m (low budgets
// are infeasible and skipped).  The linear index is therefore re-read as (tile and chain)
// fastest, chunk slowest and descending: the expensive chunks of all tiles start first and
// the cheap ones fill the tail of the launch, and at every chunk level the tiles and chains
// spread evenly over the XCDs.
struct Work { int chunk, tile, chain; };
__device__ __forceinline__ Work work_of_block() {
    const uint32_t nt = gridDim.y * gridDim.z;
    const uint32_t lin = blockIdx.x + gridDim.x * (blockIdx.y + gridDim.y * blockIdx.z);
    const uint32_t level = lin / nt, t = lin - level * nt;
    return {int(gridDim.x - 1 - level), int(t % gridDim.y), int(t / gridDim.y)};
}

// + j = table row of cell (q, j)
__device__ __forceinline__ int row_base(int L, int q) { return q * L - (q * (q - 1)) / 2 - q; }

// Operands of the part of a row that does not depend on the row block: the splits in the
// column block (right operand (jb + c2 + 1, j) at its shift, for CF <= c2 < cc) and C_all (right
// operand (i + 1, j) at m - omega_abar^{i+1}).
template <int T, int CF>
__device__ __forceinline__ void load_row_tail(rsrc_t tab, const int32_t* __restrict__ wsh, int L, int pitch, int i,
                                              int jb, const int (&jc)[T], uint32_t wabi, uint32_t moff,
                                              uint32_t (&tj)[T][T], uint32_t (&al)[T]) {
#pragma unroll
    for (int cc = CF + 1; cc < T; ++cc)
#pragma unroll
        for (int c2 = CF; c2 < cc; ++c2) {
            const int q = min(jb + c2 + 1, L - 1);
            tj[c2][cc] = ld32(tab, uint32_t(row_base(L, q) + jc[cc]) * uint32_t(pitch) - uint32_t(wsh[q]), moff);
        }
#pragma unroll
    for (int cc = CF; cc < T; ++cc) {
        const int i1 = min(i + 1, L - 1);
        al[cc] = ld32(tab, uint32_t(row_base(L, i1) + max(jc[cc], i1)) * uint32_t(pitch) - wabi, moff);
    }
}

// Finishes the cells of row i in column block jb from the best candidate so far (splits in the
// row block, gemm partial): splits in the column block with the left operand (i, q-1) = the
// cell just finished, then the m_null gate, C_all with the m_all gate (smallest candidate
// number: wins ties), saturation, store.
template <int T, int CF, int DC>
__device__ __forceinline__ void finish_row(const Ctx& c, size_t chain, const int32_t* __restrict__ P,
                                           const int32_t* __restrict__ mall, const int32_t* __restrict__ mnull,
                                           int L, int pitch, int i, int jb, int cend, const int (&jc)[T],
                                           uint32_t fbi, uint32_t m, uint32_t (&best)[T], uint32_t (&pick)[T],
                                           const uint32_t (&tj)[T][T], const uint32_t (&al)[T]) {
    const uint32_t Pi = P[i];
    const int rowi = tri_row(L, i, i) - i;  // + j = row of (i, j)
    uint32_t val[T];
#pragma unroll
    for (int cc = 0; cc < T; ++cc) val[cc] = kInf;
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

// Middle splits of every tile of block diagonal D >= 2.
// One wave owns the 8x8 tile of cells for 64 consecutive m; lane = m.  Each loaded operand
// row is used by 8 cells (1 byte of table traffic per candidate instead of 8).  The CH waves of
// a work-group take adjacent chunks of m of the same tile: the cache lines that a shifted
// operand read straddles are fetched once for two waves.
// Candidates are compared as float64 keys  cost + (q+1)/256 : one add and one min per
// candidate give the minimum cost and, among equal costs, the smallest candidate number
// (all values are integers below 2^34 scaled by 2^-8, exact in float64).
// Splits whose operands are infeasible for the whole chunk (frontier test) are dropped
// from the work list before the pipeline starts.
// Output, rows 0..6 of the tile: cost[] <- partial minimum clamped to 2^31 - 1, with bit 31 set as
// the mark "not finished", arg[] <- its number; the row kernels finish them.  Row 7 has no split
// in its own row block, so its partial minimum stays in registers and the wave finishes the row
// itself.
// KS > 1 (launches with too few tiles to fill the chip): KS waves share one chunk, each takes
// every KS-th entry of the work list, and their key tiles are merged through LDS at the end.
template <int NB, int UNR, int CH, int KS, bool CNT>
__global__ void __launch_bounds__(64 * CH * KS, 2) gemm_kernel(Ctx c, int D) {
    constexpr int T = kT;
    static_assert(T == 8, "one wave per 8x8 tile");
    const Work w = work_of_block();
    const int b = c.b0 + w.chain, I = w.tile, J = I + D;
    const int L = c.L, pitch = c.pitch;
    const int qlo = (I + 1) * T, qhi = J * T;
    const int j0 = J * T, i0 = I * T;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(int(threadIdx.x >> 6));
    const int bx = w.chunk;
    const int cw = wave / KS, slice = wave % KS;  // chunk within the work-group, slice of the list
    const int chunk = bx * CH + cw;  // this wave's 64 columns of m
    const uint32_t m = chunk * 64 + lane;
    const uint32_t moff = m * 4;
    const size_t chain = size_t(b) * c.rows * pitch;
    const rsrc_t tab = table_rsrc(c.cost + chain, uint32_t(c.rows) * uint32_t(pitch) * 4u);
    const int32_t* need = c.ws.need + size_t(b) * L * L;

    int lrow0[8], jcol[8];
#pragma unroll
    for (int r = 0; r < 8; ++r) lrow0[r] = tri_row(L, i0 + r, i0 + r) - (i0 + r) - 1;  // + q = row of (i, q-1)
#pragma unroll
    for (int cc = 0; cc < 8; ++cc) jcol[cc] = min(j0 + cc, L - 1);

    // Work list of the chunk: the splits q for which some cell of the tile can have both operands
    // feasible somewhere in these 64 columns.  Per-split constants (shift, key offset) travel
    // with the list through LDS, so the pipeline never waits on scalar memory.  Every chunk of
    // the work-group has a list of its own, built by its (first) wave: the lower chunks of a
    // work-group drop splits that only its highest chunk can use.
    __shared__ double s_kq[CKPT_MAX_L + 2][CH];
    __shared__ int2 s_qs[CKPT_MAX_L + 2][CH];  // .x = q, .y = its shift: one LDS read per entry
    __shared__ int32_t s_n[CH];
    const bool active = chunk * 64 < pitch;
    if (slice == 0) {
        const int m_hi = min(chunk * 64 + 63, pitch - 1);  // largest m of the chunk
        int n = 0;
        int out_need = need[(i0 + (lane >> 3)) * L + min(j0 + (lane & 7), L - 1)];
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) out_need = min(out_need, __shfl_xor(out_need, o));
        if (active && m_hi >= out_need) {
            for (int base = qlo; base <= qhi; base += 64) {
                const int q = base + lane;
                bool on = false;
                int sh = 0;
                if (q <= qhi) {
                    sh = c.ws.wsh[size_t(b) * L + q];
                    int tl = 1 << 30, tr = 1 << 30;
#pragma unroll
                    for (int r = 0; r < 8; ++r) tl = min(tl, need[(i0 + r) * L + q - 1]);
#pragma unroll
                    for (int cc = 0; cc < 8; ++cc) tr = min(tr, need[q * L + jcol[cc]]);
                    on = m_hi >= max(tl, tr + sh);
                }
                const unsigned long long mask = __ballot(on);
                if (on) {
                    const int pos = n + __popcll(mask & ((1ull << lane) - 1ull));
                    s_qs[pos][cw] = make_int2(q, sh);
                    s_kq[pos][cw] = c.ws.kq[size_t(b) * L + q];
                }
                n += __popcll(mask);
            }
        }
        if (lane == 0) s_n[cw] = n;
    }
    if constexpr (KS > 1) {
        __syncthreads();  // the other slices of the chunk read the list
    } else {
        if (!active) return;  // KS > 1: every wave stays for the barriers of the merge
        __builtin_amdgcn_wave_barrier();  // the wave reads what its own lanes wrote: LDS keeps a wave's order
        __builtin_amdgcn_sched_barrier(0);
    }
    // this wave's entries: slice, slice + KS, ...
    const int n_all = __builtin_amdgcn_readfirstlane(s_n[cw]);
    const int n = active && n_all > slice ? (n_all - slice + KS - 1) / KS : 0;
    auto entry = [&](int t) { return slice + KS * t; };

    double key[8][8];
#pragma unroll
    for (int r = 0; r < 8; ++r)
#pragma unroll
        for (int cc = 0; cc < 8; ++cc) key[r][cc] = 0x1p60;

    if (n > 0) {
        uint32_t buf[NB][16];
        auto load = [&](uint32_t(&v)[16], int t) {
            const int k = entry(t);
            const int2 qs = s_qs[k][cw];
            const int q = __builtin_amdgcn_readfirstlane(qs.x);
            const int sh = __builtin_amdgcn_readfirstlane(qs.y);
            const int rq = q * L - (q * (q - 1)) / 2 - q;  // + j = row of (q, j)
#pragma unroll
            for (int r = 0; r < 8; ++r) v[r] = ld32(tab, uint32_t(lrow0[r] + q) * uint32_t(pitch), moff);
#pragma unroll
            for (int cc = 0; cc < 8; ++cc)
                v[8 + cc] = ld32(tab, uint32_t(rq + jcol[cc]) * uint32_t(pitch) - uint32_t(sh), moff);
        };
        auto compute = [&](const uint32_t(&v)[16], int t) {
            const double cq = s_kq[entry(t)][cw];
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

        // Straight-line pipeline: the list is padded to a multiple of the unroll by repeating
        // its last entry (a repeated candidate cannot change a minimum), so the loop body has
        // no branches and the loads of entry k + NB - 1 are in flight while entry k is evaluated.
#pragma unroll
        for (int u = 0; u < NB - 1; ++u) load(buf[u], min(u, n - 1));
        constexpr int STEPS = NB * UNR;
        auto steps = [&](auto count, int& k) {  // count.value pipeline steps, straight-line
#pragma unroll
            for (int u = 0; u < decltype(count)::value; ++u) {
                load(buf[(u + NB - 1) % NB], min(k + NB - 1, n - 1));
                __builtin_amdgcn_sched_barrier(0);  // keep these loads ahead of the math of entry k
                compute(buf[u % NB], min(k, n - 1));
                __builtin_amdgcn_sched_barrier(0);
                ++k;
            }
        };
        // long body for the bulk (the compiler's wait at a loop header is conservative, so few
        // headers), then the remainder in bodies of NB steps: at most NB - 1 padded entries
        int k = 0;
        const int bulk = n / STEPS, tail = (n - bulk * STEPS + NB - 1) / NB;
        for (int it = 0; it < bulk; ++it) steps(std::integral_constant<int, STEPS>{}, k);
        for (int it = 0; it < tail; ++it) steps(std::integral_constant<int, NB>{}, k);
        count_work<CNT>(c.work, 0, 16u * unsigned(NB - 1 + bulk * STEPS + tail * NB), 0);
    }

    if constexpr (KS > 1) {
        // Merge: row by row of the tile, the waves of slices 1.. hand their keys to the wave of
        // slice 0 through LDS.  Every wave of the work-group passes all sixteen barriers.
        __shared__ double s_red[CH][KS - 1][8][64];
#pragma unroll
        for (int r = 0; r < 8; ++r) {
            if (slice > 0) {
#pragma unroll
                for (int cc = 0; cc < 8; ++cc) s_red[cw][slice - 1][cc][lane] = key[r][cc];
            }
            __syncthreads();
            if (slice == 0) {
#pragma unroll
                for (int o = 0; o < KS - 1; ++o)
#pragma unroll
                    for (int cc = 0; cc < 8; ++cc) key[r][cc] = fmin(key[r][cc], s_red[cw][o][cc][lane]);
            }
            __syncthreads();
        }
        if (slice != 0 || !active) return;
    }

    const int32_t* P = c.ws.P + size_t(b) * (L + 1);
    // Row 7: operands of its column-block splits and of C_all are requested before the other rows
    // are converted and stored -- unless the whole chunk lies below the frontier of its cells.
    const int i7 = i0 + 7;
    const int cend = min(8, L - j0);
    int need7 = 1 << 30;
#pragma unroll
    for (int cc = 0; cc < 8; ++cc) need7 = min(need7, need[i7 * L + jcol[cc]]);
    const bool live7 = int(m | 63u) >= need7;  // wave-uniform
    uint32_t tj[8][8], al[8];
    if (live7)
        load_row_tail<8, 0>(tab, c.ws.wsh + size_t(b) * L, L, pitch, i7, j0, jcol, c.ws.wabs[size_t(b) * L + i7],
                            moff, tj, al);
    auto partial = [&](int r, int cc, uint32_t Pi, uint32_t& cst, uint32_t& num) {
        const double k = key[r][cc];
        const double fl = floor(fmin(k, 0x1p33));
        cst = k < 0x1p32 ? uint32_t(fl) - Pi : 0xffffffffu;
        num = uint32_t((fmin(k, 0x1p33) - fl) * 256.0);
    };
    // A partial minimum is stored with bit 31 set: a finished cell never exceeds 2^30, so whoever
    // reads the table can tell a cell that still waits for its row kernel from a finished one.
    // Partial minima of 2^31 - 1 and more are infeasible whatever they were and are clamped.
    auto tagged = [](uint32_t cst) { return min(cst, 0x7fffffffu) | 0x80000000u; };
#pragma unroll
    for (int r = 0; r < 7; ++r) {
        const uint32_t Pi = P[i0 + r];
        const size_t row = chain + size_t(tri_row(L, i0 + r, j0)) * pitch + m;
#pragma unroll
        for (int cc = 0; cc < 8; ++cc) {
            if (cc < cend) {
                uint32_t cst, num;
                partial(r, cc, Pi, cst, num);
                c.cost[row + size_t(cc) * pitch] = int32_t(tagged(cst));
                c.arg[row + size_t(cc) * pitch] = uint8_t(num);
            }
        }
    }
    count_work<CNT>(c.work, 0, live7 ? 36u : 0u, 8u * unsigned(cend));
    if (live7) {
        uint32_t best[8], pick[8];
#pragma unroll
        for (int cc = 0; cc < 8; ++cc) partial(7, cc, uint32_t(P[i7]), best[cc], pick[cc]);
        finish_row<8, 0, 2>(c, chain, P, c.ws.mall + (size_t(b) * L + i7) * L, c.ws.mnull + (size_t(b) * L + i7) * L, L,
                            pitch, i7, j0, cend, jcol, c.ws.fb[size_t(b) * L + i7], m, best, pick, tj, al);
    } else {
        const size_t row = chain + size_t(tri_row(L, i7, j0)) * pitch + m;
#pragma unroll
        for (int cc = 0; cc < 8; ++cc) {
            if (cc < cend) {
                c.cost[row + size_t(cc) * pitch] = int32_t(kInf);
                c.arg[row + size_t(cc) * pitch] = 0;
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
__global__ void __launch_bounds__(kRowWG) row_kernel(Ctx c, int D) {
    constexpr int CF = (DC == 0) ? R : 0;                              // first column with j >= i
    constexpr int NQ = (DC == 0) ? 0 : (DC == 1 ? T - R : T - 1 - R);  // near-i splits (D = 1: and q = jb)
    constexpr int NQA = NQ > 0 ? NQ : 1;
    const Work w = work_of_block();
    const int b = c.b0 + w.chain, I = w.tile, J = I + D;
    const int L = c.L, pitch = c.pitch;
    const int i = I * T + R;
    if (i >= L) return;
    const uint32_t m = uint32_t(w.chunk) * kRowWG + threadIdx.x;
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
    auto rowq = [&](int q) { return row_base(L, q); };

    // Columns past the end of a ragged last block are computed on a clamped j and not stored.
    int jc[T];
#pragma unroll
    for (int cc = 0; cc < T; ++cc) jc[cc] = min(jb + cc, L - 1);

    // A wave whose whole chunk lies below the feasibility frontier of every cell of the row
    // stores "infeasible" and reads nothing.
    {
        // the frontier as far as it is known: the weak one of the precompute kernel (a finite cell
        // passes at least one of its two gates) until the frontier kernel has written the exact one
        const int32_t* need = c.ws.need + (size_t(b) * L + i) * L;
        int row_need = 1 << 30;
#pragma unroll
        for (int cc = CF; cc < T; ++cc)
            row_need = min(row_need, need[jc[cc]]);
        const int m_hi = __builtin_amdgcn_readfirstlane(int(m)) | 63;
        if (m_hi < row_need) {
#pragma unroll
            for (int cc = CF; cc < T; ++cc) {
                if (cc < cend) {
                    const size_t o = chain + size_t(rowi + jc[cc]) * pitch + m;
                    c.cost[o] = int32_t(kInf);
                    c.arg[o] = 0;
                }
            }
            return;
        }
    }

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
            pc[cc] = uint32_t(c.cost[o]) & 0x7fffffffu;  // bit 31 marks the gemm's partial minima
            pp[cc] = c.arg[o];
        }
    }
    uint32_t tj[T][T], al[T];
    load_row_tail<T, CF>(tab, wsh, L, pitch, i, jb, jc, wabi, moff, tj, al);

    // ---- evaluation ----
    uint32_t best[T], pick[T];
#pragma unroll
    for (int cc = 0; cc < T; ++cc) best[cc] = 0xffffffffu, pick[cc] = 0;
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
    finish_row<T, CF, DC>(c, chain, P, mall, mnull, L, pitch, i, jb, cend, jc, fbi, m, best, pick, tj, al);
}

// ---------------------------------------------------------------------------
// All rows of every tile of one block diagonal in ONE launch.
//
// A work-group owns one band of kBand columns of m of one tile and finishes its rows bottom-up.
// Row r needs the row below it in the same tile at m - shift: from its own band, and from lower
// bands that other work-groups finish in the same launch.
//   - Inside the band the row below travels through LDS (two buffers, one barrier per row).
//   - Between bands it travels through memory.  Work-groups take their work by ticket (an atomic
//     counter), bands in ascending order, so whatever a wave waits for belongs to a work-group
//     that already runs -- no deadlock, whatever order the hardware starts work-groups in.
//     D >= 2: before its row is finished a cell holds the gemm's partial minimum, marked by bit 31
//     (finished cells never exceed 2^30), so a reader needs no flag and a writer never waits for
//     its stores: a lane that finds the mark simply reads again.  D < 2: the cells hold whatever
//     the caller's buffer held, so every wave publishes "rows finished" for its chunk of 64
//     columns once its stores of the row have completed, and readers wait for those flags
//     (looked at one row ahead of the need, while the wave waits for its own stores).
//     Every wait is bounded: when it expires the kernel sets the fault word and all work-groups
//     drain (ckpt_check_inputs then reports CKPT_E_INTERNAL).
// Coherence between compute units and between the L2 caches of the eight dies, without cache
// flushes: a cell of the table is written once per solve and only read after it was published.
// Finished rows are stored with device-scope stores (written through to memory before the
// store counts as complete) and rows of the same launch are read with device-scope loads
// (never served from a compute unit's L1 or from a stale line of another die's L2).  Lanes whose
// shifted column would be negative read nothing (an out-of-range buffer offset returns 0), so
// no line of the table is touched before its owner has written it.
// Each loaded operand of a split is kept in registers for all rows that use it: per tile and
// lane 7 x 8 + 28 + 64 operand loads instead of the 252 + 224 + 64 of one launch per row.
// ---------------------------------------------------------------------------
constexpr uint32_t kNoRead = 0xfffffff0u;  // buffer offset beyond any table: the load returns 0, no access
constexpr int kSpinLimit = 1 << 20;        // default polls of a wait before it gives up (seconds, never reached)


// Per-tile parameters of the row kernel, fetched once into LDS by the whole work-group: the
// rows' thresholds and frontier, prefix sums, shifts, and the byte offsets of the table rows the
// tile touches.  Inside the row steps nothing but table cells comes from memory, so a step
// costs one memory round trip, and an address is one add: every access is
// descriptor base + per-lane offset (row offset from here + 4 m - 4 shift) + cc * row pitch.
struct TilePar {
    int32_t mall[kT][kT], mnull[kT][kT], need[kT][kT];  // [r][cc]: cell (i0 + r, j_cc)
    int32_t Pi[kT + 1];       // P[i0 + u], u = 0..8
    int32_t Pj[kT];           // P[min(jb + c2 + 1, L - 1)]
    int32_t wsh[kT + 1];      // shift of split q = i0 + u
    int32_t wabs[kT], fb[kT];
    uint32_t rowoff[kT + 1];  // byte offset of cell (i0 + u, jb) in the chain's cost table, u = 0..8
    uint32_t diagoff[kT];     // byte offset of cell (i0 + r, i0 + r)
};

template <int DC>
struct TileCtx {
    Ctx c;
    const TilePar* par;
    int b, I, J, L, pitch, i0, jb, cend, band;
    rsrc_t tab, atab;  // the chain's cost table (bytes) and candidate table
    uint32_t m, moff;
    uint32_t col4[kT];  // cc * pitch * 4: the scalar part of every address
    int32_t* prog;    // progress of this tile: [chunks of 64 columns]
    int chunk0;       // first chunk of this band
    int nwait;        // chunks below the band that this wave's shifted reads can reach
    int seen;         // lane k < nwait: progress of chunk chunk0 - 1 - k as last looked at
    bool dead;        // a wait expired: stop working, keep meeting the barriers (per wave)
    bool idle;        // this wave's columns lie past the end of the rows (wave-uniform)
    // right operands kept for all rows: ri[u][cc] = cell (i0 + u, j_cc) at m - omega_a^{i0+u}, u = 1..8
    // (rows of this tile; u = 8 is the first stage of the column block, D = 1 only);
    // rj[c2][cc] = cell (jb + c2 + 1, j_cc) at its shift, c2 < cc (column block, D >= 1)
    uint32_t ri[kT + 1][kT];
    uint32_t rj[kT][kT];
};

// Table accesses of the row kernel: voff = per-lane byte offset (kNoRead: nothing is read, the
// result is 0), soff = wave-uniform byte offset.  dev = device scope.
__device__ __forceinline__ uint32_t tld(rsrc_t tab, uint32_t voff, uint32_t soff) {
    return uint32_t(__builtin_amdgcn_raw_buffer_load_b32(tab, int(voff), int(soff), 0));
}
__device__ __forceinline__ uint32_t tld_dev(rsrc_t tab, uint32_t voff, uint32_t soff) {
    return uint32_t(__builtin_amdgcn_raw_buffer_load_b32(tab, int(voff), int(soff), 16));
}

// Requests the progress of the chunks below the band (lane k looks at chunk chunk0 - 1 - k);
// consumed by the next wait_rows_below, by which time the load has long returned.
template <int DC>
__device__ __forceinline__ void look_below(TileCtx<DC>& x) {
    const int k = threadIdx.x & 63;
    if (k < x.nwait) x.seen = __hip_atomic_load(x.prog + x.chunk0 - 1 - k, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Every wave for itself: until each of the nwait chunks below the band has finished `rows` rows.
template <int DC>
__device__ __forceinline__ void wait_rows_below(TileCtx<DC>& x, int rows) {
    if (x.nwait == 0 || x.dead) return;
    const int lane = threadIdx.x & 63;
    bool ok = __all(lane >= x.nwait || x.seen >= rows) && x.nwait <= 64 && x.c.spin_limit >= 0;
    for (int spin = 0; !ok && spin < x.c.spin_limit; ++spin) {
        ok = true;
        for (int k = lane; k < x.nwait; k += 64)
            ok = ok && __hip_atomic_load(x.prog + x.chunk0 - 1 - k, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) >= rows;
        ok = __all(ok);
        if (ok) break;
        if ((spin & 63) == 63 && __hip_atomic_load(x.c.ws.fault, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0)
            break;
        __builtin_amdgcn_s_sleep(2);
    }
    if (!ok) {
        x.dead = true;
        if (lane == 0) __hip_atomic_store(x.c.ws.fault, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
}

// Cells (i0 + u, jb + cc), cc = first_cc .. cend - 1, of a row finished in THIS launch, at column
// m - sh: from LDS if that column lies in this band (`below` = the row's buffer), else from the
// table with a device-scope load.
// D >= 2: the cells of the tile hold the gemm's partial minima, marked by bit 31, until their
// row is finished, so the read needs no flag: a lane that finds the mark reads again (bounded).
// D < 2: the caller has waited for the progress flags of the chunks that are read.
template <int DC, bool FULL, bool CNT>
__device__ __forceinline__ void read_row_below(TileCtx<DC>& x, const uint32_t (*below)[kBand], uint32_t rowoff,
                                               uint32_t sh, int first_cc, uint32_t (&out)[kT]) {
    const int cend = FULL ? kT : x.cend;
    const int t = int(threadIdx.x) - int(sh);  // column inside the band
    const bool in_band = t >= 0;
    const uint32_t voff = (!in_band && x.m >= sh) ? x.moff + rowoff - 4 * sh : kNoRead;
    if (CNT && __any(voff != kNoRead)) count_work<CNT>(x.c.work, 2, unsigned(max(0, cend - first_cc)), 0);
    uint32_t mem[kT];
    auto fetch = [&]() {
        uint32_t marks = 0;
#pragma unroll
        for (int cc = 0; cc < kT; ++cc) {
            mem[cc] = 0;
            if (cc >= first_cc && cc < cend) mem[cc] = tld_dev(x.tab, voff, x.col4[cc]);  // only cells that exist
            marks |= mem[cc];
        }
        return (marks >> 31) != 0;
    };
    bool again = fetch();
    if (DC == 2) {
        int spin = 0;
        if (x.c.spin_limit < 0) again = !in_band && x.m >= sh;  // forced: every read from another band gives up
        while (__any(again)) {  // some lane met a cell that its owner has not finished yet
            if (++spin > x.c.spin_limit ||
                ((spin & 63) == 0 && __hip_atomic_load(x.c.ws.fault, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0)) {
                x.dead = true;
                if ((threadIdx.x & 63) == 0)
                    __hip_atomic_store(x.c.ws.fault, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                break;
            }
            __builtin_amdgcn_s_sleep(2);
            if (again) again = fetch();
        }
    }
#pragma unroll
    for (int cc = 0; cc < kT; ++cc) {
        if (cc >= first_cc && cc < cend) {
            const uint32_t lds = below[cc][in_band ? t : 0];
            out[cc] = in_band ? lds : mem[cc];
        }
    }
}

// FULL: the tile has all eight columns (always, except in the last column block of a chain whose
// length is not a multiple of eight); the tests for columns that do not exist then vanish.
template <int DC, int R, bool CNT, bool FULL>
__device__ __forceinline__ void tile_row(TileCtx<DC>& x, uint32_t (*s_row)[kT][kBand]) {
    constexpr int T = kT;
    constexpr int RF = (DC == 2) ? T - 2 : T - 1;                      // first row this kernel finishes
    constexpr int CF = (DC == 0) ? R : 0;                              // first column with j >= i
    constexpr int NQ = (DC == 0) ? 0 : (DC == 1 ? T - R : T - 1 - R);  // splits in the row block (D = 1: and q = jb)
    constexpr int NQA = NQ > 0 ? NQ : 1;
    constexpr int U = R + 1;                                           // the row below
    const int L = x.L;
    const int cend = FULL ? T : x.cend;
    const int i = x.i0 + R;
    if (i >= L) return;  // ragged last block: uniform over the work-group
    const bool below_here = R < RF && i + 1 < L;  // the row below exists and belongs to this launch
    const uint32_t m = x.m, moff = x.moff;
    const TilePar& par = *x.par;
    const uint32_t (*below)[kBand] = s_row[U & 1];
    uint32_t (*mine)[kBand] = s_row[R & 1];
    uint32_t val[T];
#pragma unroll
    for (int cc = 0; cc < T; ++cc) val[cc] = kInf;

    if (DC < 2 && below_here) wait_rows_below(x, RF - R);
    if (!x.dead && !x.idle) {
        // ---- loads of this row, all issued together ----
        // the operands that the row below contributes to all rows above it, kept
        if ((U < T || DC == 1) && x.i0 + U < L) {
            const uint32_t sh = uint32_t(par.wsh[U]);
            if (below_here) {
                read_row_below<DC, FULL, CNT>(x, below, par.rowoff[U], sh, DC == 0 ? U : 0, x.ri[U]);
            } else {  // finished by an earlier launch
                const uint32_t voff = m >= sh ? moff + par.rowoff[U] - 4 * sh : kNoRead;
#pragma unroll
                for (int cc = (DC == 0 ? U : 0); cc < T; ++cc)
                    if (cc < cend) x.ri[U][cc] = tld(x.tab, voff, x.col4[cc]);
            }
        }
        int row_need = 1 << 30;
#pragma unroll
        for (int cc = CF; cc < T; ++cc)
            row_need = min(row_need, par.need[R][cc]);
        const int m_hi = __builtin_amdgcn_readfirstlane(int(m)) | 63;
        const bool live = m_hi >= row_need;  // else the whole chunk lies below the feasibility frontier of the row
        const unsigned cols = unsigned(max(0, cend - CF));  // cells of the row that exist
        // loads from earlier launches: the row below (first row of the kernel only), left operands, the
        // gemm's partial minima (cost + number), C_all operands (first row only); reads of rows of this
        // launch are counted where they are issued, and only for waves that reach below their band
        count_work<CNT>(x.c.work, 2, (below_here ? 0u : cols) + (live ? unsigned(NQ) + (DC == 2 ? 10u : 0u) +
                                                                          (below_here ? 0u : cols) : 0u), cols);
        const uint32_t Pi = par.Pi[R];
        const uint32_t fbi = par.fb[R];
        const uint32_t wabi = par.wabs[R];
        const uint32_t own = moff + par.rowoff[R];  // this lane's cell of the row, column block start
        uint32_t nl[NQA], pc[T], pp[T], al[T];
#pragma unroll
        for (int cc = 0; cc < T; ++cc) al[cc] = 0, pc[cc] = 0xffffffffu, pp[cc] = 0;
        if (live) {
            const uint32_t left = moff + par.diagoff[R];  // cell (i, i); (i, i + u) is u rows further
#pragma unroll
            for (int u = 0; u < NQ; ++u) nl[u] = tld(x.tab, left, x.col4[u]);
            if (DC == 2) {  // gemm partial; bit 31 marks it
#pragma unroll
                for (int cc = 0; cc < T; ++cc) {
                    if (cc < cend) {
                        pc[cc] = tld(x.tab, own, x.col4[cc]) & 0x7fffffffu;
                        pp[cc] = uint32_t(__builtin_amdgcn_raw_buffer_load_b8(x.atab, int(own >> 2), int(x.col4[cc] >> 2), 0));
                    }
                }
            }
            // C_all: cell (i + 1, j) at m - omega_abar^{i+1}, for j > i
            if (below_here) {
                read_row_below<DC, FULL, CNT>(x, below, par.rowoff[U], wabi, DC == 0 ? CF + 1 : CF, al);
            } else if (i + 1 < L) {  // row 0 of the tile below, or row 7 finished by the gemm: earlier launches
                const uint32_t voff = m >= wabi ? moff + par.rowoff[U] - 4 * wabi : kNoRead;
#pragma unroll
                for (int cc = (DC == 0 ? CF + 1 : CF); cc < T; ++cc)
                    if (cc < cend) al[cc] = tld(x.tab, voff, x.col4[cc]);
            }
            // ---- evaluation, in candidate-number order with strict '<' ----
            uint32_t best[T], pick[T];
#pragma unroll
            for (int cc = 0; cc < T; ++cc) best[cc] = 0xffffffffu, pick[cc] = 0;
#pragma unroll
            for (int u = 0; u < NQ; ++u) {
                const int q = i + 1 + u;
                const uint32_t lb = nl[u] + (uint32_t(par.Pi[R + 1 + u]) - Pi);
#pragma unroll
                for (int cc = 0; cc < T; ++cc) {
                    const uint32_t v = lb + x.ri[R + 1 + u][cc];
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
#pragma unroll
                for (int c2 = CF; c2 < cc; ++c2) {  // splits in the column block: left operand (i, q-1) = val[c2]
                    const int q = min(x.jb + c2 + 1, L - 1);
                    const uint32_t r = (DC == 0) ? x.ri[c2 + 1][cc] : x.rj[c2][cc];
                    const uint32_t v = val[c2] + (uint32_t(par.Pj[c2]) - Pi) + r;
                    if (v < best[cc]) best[cc] = v, pick[cc] = q + 1;
                }
                const uint32_t ck = (m >= uint32_t(par.mnull[R][cc])) ? min(best[cc], kInf) : kInf;
                uint32_t all = fbi;
                if (DC != 0 || cc > CF) all += al[cc];  // j > i
                all = (m >= uint32_t(par.mall[R][cc])) ? min(all, kInf) : kInf;
                const bool take_all = all < kInf && all <= ck;
                val[cc] = take_all ? all : ck;
                pick[cc] = take_all ? uint32_t(i + 1) : (ck < kInf ? pick[cc] : 0u);
            }
#pragma unroll
            for (int cc = CF; cc < T; ++cc) {
                if (cc < cend) {  // cost with a device-scope store: other bands read it in this launch
                    __builtin_amdgcn_raw_buffer_store_b32(int(val[cc]), x.tab, int(own), int(x.col4[cc]), 16);
                    __builtin_amdgcn_raw_buffer_store_b8((unsigned char)(pick[cc]), x.atab, int(own >> 2),
                                                         int(x.col4[cc] >> 2), 0);
                }
            }
        } else {
#pragma unroll
            for (int cc = CF; cc < T; ++cc) {
                if (cc < cend) {
                    __builtin_amdgcn_raw_buffer_store_b32(int(kInf), x.tab, int(own), int(x.col4[cc]), 16);
                    __builtin_amdgcn_raw_buffer_store_b8((unsigned char)(0), x.atab, int(own >> 2), int(x.col4[cc] >> 2), 0);
                }
            }
        }
        if (R > 0) {
            // the rows above read this row from LDS (this band) or from memory (bands above)
#pragma unroll
            for (int cc = CF; cc < T; ++cc) mine[cc][threadIdx.x] = val[cc];
            if (DC < 2) {
                // The cells of these tiles hold whatever the caller's buffer held: readers in other
                // bands need a flag.  Publish the row for this wave's chunk as soon as its stores
                // have completed; the look at the chunks below returns together with them.
                look_below(x);
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
                __builtin_amdgcn_s_waitcnt(0);
                if ((threadIdx.x & 63) == 0)
                    __hip_atomic_store(x.prog + (x.m >> 6), RF - R + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
        }
    }
    if (R > 0) __syncthreads();  // the row is in LDS for the waves of this band
}

template <int DC, int R, bool CNT, bool FULL>
struct TileRows {
    static __device__ __forceinline__ void run(TileCtx<DC>& x, uint32_t (*s_row)[kT][kBand]) {
        tile_row<DC, R, CNT, FULL>(x, s_row);
        if constexpr (R > 0) TileRows<DC, R - 1, CNT, FULL>::run(x, s_row);
    }
};

template <int DC, bool CNT>
__global__ void __launch_bounds__(kRowWG, 3) tile_rows_kernel(Ctx c, int D, int32_t* tick) {
    constexpr int T = kT;
    constexpr int RF = (DC == 2) ? T - 2 : T - 1;
    __shared__ int s_ticket, s_fault;
    __shared__ uint32_t s_row[2][kT][kBand];  // the last two finished rows of this band
    __shared__ TilePar s_par;
    if (threadIdx.x == 0) {
        s_ticket = atomicAdd(tick, 1);
        s_fault = __hip_atomic_load(c.ws.fault, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    __syncthreads();
    const uint32_t ntile = gridDim.y, per_band = gridDim.y * gridDim.z;
    const uint32_t ticket = uint32_t(s_ticket);
    if (ticket >= gridDim.x * per_band) return;  // cannot happen: one ticket per work-group
    TileCtx<DC> x;
    x.c = c;
    x.band = int(ticket / per_band);  // bands in ascending order
    const uint32_t rest = ticket - uint32_t(x.band) * per_band;
    x.I = int(rest % ntile);
    x.J = x.I + D;
    x.b = c.b0 + int(rest / ntile);
    x.L = c.L;
    x.pitch = c.pitch;
    x.i0 = x.I * T;
    x.jb = x.J * T;
    x.cend = min(T, c.L - x.jb);
    const size_t chain = size_t(x.b) * c.rows * c.pitch;
    x.tab = table_rsrc(c.cost + chain, uint32_t(c.rows) * uint32_t(c.pitch) * 4u);
    x.atab = __builtin_amdgcn_make_buffer_rsrc(c.arg + chain, 0, int(uint32_t(c.rows) * uint32_t(c.pitch)), 0x00020000);
    x.m = uint32_t(x.band) * kBand + threadIdx.x;
    x.moff = x.m * 4;
    x.seen = 0;
    x.dead = s_fault != 0;  // an earlier work-group gave up: drain
#pragma unroll
    for (int cc = 0; cc < T; ++cc) x.col4[cc] = uint32_t(cc) * uint32_t(c.pitch) * 4u;
#pragma unroll
    for (int u = 0; u <= T; ++u)
#pragma unroll
        for (int cc = 0; cc < T; ++cc) x.ri[u][cc] = 0;
#pragma unroll
    for (int c2 = 0; c2 < T; ++c2)
#pragma unroll
        for (int cc = 0; cc < T; ++cc) x.rj[c2][cc] = 0;
    const int32_t* P = c.ws.P + size_t(x.b) * (c.L + 1);
    const int32_t* wsh = c.ws.wsh + size_t(x.b) * c.L;
    {   // parameters of the tile: one fetch by the whole work-group
        const int t = threadIdx.x, L = c.L;
        const size_t bL = size_t(x.b) * L;
        if (t < 64) {
            const int r = t >> 3, i = min(x.i0 + r, L - 1);
            const size_t at = (bL + i) * L + min(x.jb + (t & 7), L - 1);  // no dynamic index into x: it stays in registers
            s_par.mall[r][t & 7] = c.ws.mall[at];
            s_par.mnull[r][t & 7] = c.ws.mnull[at];
            s_par.need[r][t & 7] = c.ws.need[at];  // weak or exact, whichever is there: both are lower bounds
        } else if (t < 64 + T + 1) {
            const int u = t - 64, q = min(x.i0 + u, L - 1);
            s_par.Pi[u] = P[min(x.i0 + u, L)];
            s_par.wsh[u] = wsh[q];
            // cell (q, jb); on the diagonal tile only the cells with jb + cc >= q exist and are touched
            s_par.rowoff[u] = uint32_t(row_base(L, q) + x.jb) * uint32_t(c.pitch) * 4u;
        } else if (t >= 96 && t < 96 + T) {
            const int r = t - 96, q = min(x.jb + r + 1, L - 1), i = min(x.i0 + r, L - 1);
            s_par.Pj[r] = P[q];
            s_par.wabs[r] = c.ws.wabs[bL + i];
            s_par.fb[r] = c.ws.fb[bL + i];
            s_par.diagoff[r] = uint32_t(row_base(L, i) + i) * uint32_t(c.pitch) * 4u;
        }
    }
    x.par = &s_par;
    // The band may lie past the end of the rows (pitch is a multiple of 64, not of kBand): those
    // waves read and store nothing but still meet every barrier.
    x.idle = x.m >= uint32_t(c.pitch);
    __syncthreads();
    {   // A band below the feasibility frontier of every cell this kernel finishes in the tile: all of
        // them are infeasible there.  Store that and leave (the whole work-group decides alike).
        int tile_need = 1 << 30;
        {   // every wave for itself: lane = cell, then a minimum over the wave
            const int lane = threadIdx.x & 63, r = lane >> 3, cc = lane & 7;
            if (r <= RF && cc >= (DC == 0 ? r : 0) && x.i0 + r < c.L && cc < x.cend) tile_need = s_par.need[r][cc];
#pragma unroll
            for (int o = 32; o > 0; o >>= 1) tile_need = min(tile_need, __shfl_xor(tile_need, o));
        }
        if (int(min(uint32_t(x.band) * kBand + kBand - 1, uint32_t(c.pitch) - 1)) < tile_need) {
            unsigned cells = 0;
            if (!x.idle && !x.dead) {
                for (int r = 0; r <= RF; ++r) {
                    if (x.i0 + r >= c.L) continue;
                    const uint32_t own = x.moff + s_par.rowoff[r];
                    for (int cc = (DC == 0 ? r : 0); cc < x.cend; ++cc) {  // no dynamic index into x: it stays in registers
                        const uint32_t col = uint32_t(cc) * uint32_t(c.pitch);
                        __builtin_amdgcn_raw_buffer_store_b32(int(kInf), x.tab, int(own), int(col * 4u), 16);
                        __builtin_amdgcn_raw_buffer_store_b8((unsigned char)(0), x.atab, int(own >> 2), int(col), 0);
                        ++cells;
                    }
                }
                count_work<CNT>(c.work, 2, 0, cells);
                if (DC < 2) {  // readers in the bands above wait for this chunk's progress
                    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
                    __builtin_amdgcn_s_waitcnt(0);
                    if ((threadIdx.x & 63) == 0)
                        __hip_atomic_store(c.ws.prog + (size_t(x.b) * tiles_of(c.L) + tile_index(blocks_of(c.L), x.I, x.J)) *
                                                           (c.pitch / 64) + (x.m >> 6),
                                           RF + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                }
            }
            return;
        }
    }
    const int nblk = blocks_of(c.L);
    x.prog = c.ws.prog + (size_t(x.b) * tiles_of(c.L) + tile_index(nblk, x.I, x.J)) * (c.pitch / 64);
    x.chunk0 = x.band * (kBand / 64);
    {   // chunks below the band that the shifts of this tile's rows can reach from this wave's columns
        int reach = 0;
        for (int r = 0; r < T; ++r) reach = max(reach, max(s_par.wsh[r], s_par.wabs[r]));
        const int m0 = __builtin_amdgcn_readfirstlane(int(x.m));  // first column of the wave
        x.nwait = max(0, x.chunk0 - (max(0, m0 - reach) >> 6));
    }
    if (DC >= 1 && !x.dead && !x.idle) {
        // operands of the splits in the column block, finished by earlier launches
#pragma unroll
        for (int c2 = 0; c2 < T - 1; ++c2) {
            const int q = min(x.jb + c2 + 1, c.L - 1);
            const uint32_t sh = uint32_t(wsh[q]);
            const uint32_t voff =
                x.m >= sh ? x.moff + uint32_t(row_base(c.L, q) + x.jb) * uint32_t(c.pitch) * 4u - 4 * sh : kNoRead;
#pragma unroll
            for (int cc = c2 + 1; cc < T; ++cc)
                if (cc < x.cend) x.rj[c2][cc] = tld(x.tab, voff, x.col4[cc]);
        }
        count_work<CNT>(c.work, 2, 28u, 0);
    }
    if (x.cend == T)
        TileRows<DC, RF, CNT, true>::run(x, s_row);
    else
        TileRows<DC, RF, CNT, false>::run(x, s_row);
}

using RowFn = void (*)(Ctx, int);
template <int T, int DC, int... Rs>
constexpr std::array<RowFn, sizeof...(Rs)> row_table(std::integer_sequence<int, Rs...>) {
    return {{row_kernel<T, Rs, DC>...}};
}
const std::array<RowFn, kT> kRow0 = row_table<kT, 0>(std::make_integer_sequence<int, kT>{});
const std::array<RowFn, kT> kRow1 = row_table<kT, 1>(std::make_integer_sequence<int, kT>{});
const std::array<RowFn, kT> kRow2 = row_table<kT, 2>(std::make_integer_sequence<int, kT>{});


// ---------------------------------------------------------------------------
// Planner-side steps (Section "Integrate Two Solvers").
// ---------------------------------------------------------------------------

// One block: lexicographic minimum of (C_BP(1, L, m_b), b) over the chains.
__global__ void __launch_bounds__(256) select_kernel(const int32_t* __restrict__ cost, int L, int M, int pitch,
                                                      int rows, int B, const int32_t* __restrict__ m_budget,
                                                      int32_t* __restrict__ out) {
    __shared__ unsigned long long s_best[256];
    const size_t root = size_t(tri_row(L, 0, L - 1)) * pitch;
    unsigned long long best = (static_cast<unsigned long long>(kInf) << 32) | 0xffffffffull;
    for (int b = threadIdx.x; b < B; b += blockDim.x) {
        const int m = m_budget[b];
        if (m < 0) continue;
        const uint32_t v = uint32_t(cost[size_t(b) * rows * pitch + root + min(m, M)]);
        if (v < kInf) best = min(best, (static_cast<unsigned long long>(v) << 32) | uint32_t(b));
    }
    s_best[threadIdx.x] = best;
    __syncthreads();
    for (int o = blockDim.x / 2; o > 0; o >>= 1) {
        if (int(threadIdx.x) < o) s_best[threadIdx.x] = min(s_best[threadIdx.x], s_best[threadIdx.x + o]);
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        const unsigned long long r = s_best[0];
        out[0] = (r >> 32) < kInf ? int32_t(r & 0xffffffffull) : -1;
        out[1] = int32_t(r >> 32);
    }
}

// slots = min(2^31 - 1, ceil(bytes * M / budget))
__device__ inline int32_t slots_of(long long bytes, unsigned long long budget, int M) {
    const unsigned long long v = static_cast<unsigned long long>(bytes) * uint32_t(M);
    const unsigned long long q = budget ? v / budget + (v % budget != 0) : 0x7fffffffull;
    return int32_t(min(q, 0x7fffffffull));
}

// One thread per element, one chain per blockIdx.y.
__global__ void __launch_bounds__(256) discretize_kernel(const long long* __restrict__ in, int32_t* __restrict__ out,
                                                          const long long* __restrict__ budget, int per_chain, int M) {
    const int b = blockIdx.y;
    const int k = blockIdx.x * blockDim.x + threadIdx.x;
    if (k >= per_chain) return;
    out[size_t(b) * per_chain + k] =
        slots_of(in[size_t(b) * per_chain + k], static_cast<unsigned long long>(budget[b]), M);
}

// The same for one profile under every budget of a sweep: chain blockIdx.y uses budget[blockIdx.y].
struct SweepBudgets { long long v[CKPT_MAX_SWEEP]; };
__global__ void __launch_bounds__(256) discretize_sweep_kernel(const long long* __restrict__ in,
                                                                int32_t* __restrict__ out, SweepBudgets budget,
                                                                int per_chain, int M) {
    const int b = blockIdx.y;
    const int k = blockIdx.x * blockDim.x + threadIdx.x;
    if (k >= per_chain) return;
    out[size_t(b) * per_chain + k] = slots_of(in[k], static_cast<unsigned long long>(budget.v[b]), M);
}

__global__ void __launch_bounds__(64) store_budgets_kernel(SweepBudgets budget, int count,
                                                            long long* __restrict__ out) {
    if (int(threadIdx.x) < count) out[threadIdx.x] = budget.v[threadIdx.x];
}

// One thread per chain walks its recorded candidates with an explicit stack.  Pending work
// is either "walk cell (s, t, m)" or "emit B^s"; at most 2 entries per open segment.
__global__ void __launch_bounds__(64) schedule_kernel(const uint8_t* __restrict__ arg, const int32_t* __restrict__ wa,
                                                       const int32_t* __restrict__ wabar, int L, int M, int pitch,
                                                       int rows, int B, const int32_t* __restrict__ m_budget,
                                                       ckpt_op_t* __restrict__ ops, int cap,
                                                       int32_t* __restrict__ n_ops,
                                                       int4* __restrict__ stack_mem) {
    const int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= B) return;
    const uint8_t* tab = arg + size_t(b) * rows * pitch;
    const int32_t* a = wa + size_t(b) * (L + 1);
    const int32_t* ab = wabar + size_t(b) * L;
    ckpt_op_t* out = ops + size_t(b) * cap;
    int4* stack = stack_mem + size_t(b) * (2 * L + 2);  // (s, t, m, kind): kind 0 walk, 1 emit B^s
    int top = 0, n = 0, err = 0;
    auto emit = [&](int kind, int stage) {
        if (n >= cap) { err = CKPT_E_SMALLBUF; return; }
        out[n].kind = uint8_t(kind);
        out[n].stage = uint8_t(stage);
        ++n;
    };
    const int m0 = m_budget[b];
    if (m0 < 0) err = CKPT_E_ARG;
    stack[top++] = make_int4(1, L, min(m0, M), 0);
    bool root = true;
    while (top > 0 && err == 0) {
        const int4 e = stack[--top];
        const int s = e.x, t = e.y, m = e.z;
        if (e.w == 1) { emit(CKPT_OP_B, s); continue; }
        if (m < 0) { err = CKPT_E_CORRUPT; break; }
        const int k = tab[size_t(tri_row(L, s - 1, t - 1)) * pitch + m];
        if (k == 0) { err = root ? CKPT_E_INFEASIBLE : CKPT_E_CORRUPT; break; }
        root = false;
        if (k < s || k > t) { err = CKPT_E_CORRUPT; break; }
        if (s == t) {
            emit(CKPT_OP_F_ALL, s);
            emit(CKPT_OP_B, s);
        } else if (k == s) {  // C_all: F_all^s, (s+1, t, m - abar^s), B^s
            emit(CKPT_OP_F_ALL, s);
            stack[top++] = make_int4(s, s, 0, 1);
            stack[top++] = make_int4(s + 1, t, m - ab[s - 1], 0);
        } else {  // C_ck at s' = k: F_ck^s, F_null^{s+1..k-1}, (k, t, m - a^{k-1}), (s, k-1, m)
            emit(CKPT_OP_F_CK, s);
            for (int j = s + 1; j < k; ++j) emit(CKPT_OP_F_NULL, j);
            stack[top++] = make_int4(s, k - 1, m, 0);
            stack[top++] = make_int4(k, t, m - a[k - 1], 0);
        }
    }
    n_ops[b] = err ? err : n;
}

// Checkpoint block index of every stage (Section "Code generation"): one wave per chain reads the
// first forward sweep of its operation list.  In a list produced by the walk above, operation k
// (k < L) is the first forward of stage k + 1 and operation L is B^L; F_ck opens a block, F_null
// continues it, F_all lies in none.  The block number of a stage is the count of F_ck up to it,
// minus one: an inclusive prefix sum over the lanes, carried across passes of 64 stages.
__global__ void __launch_bounds__(64) block_index_kernel(const ckpt_op_t* __restrict__ ops, int cap,
                                                          const int32_t* __restrict__ n_ops, int L,
                                                          int32_t* __restrict__ block_of_stage,
                                                          int32_t* __restrict__ n_blocks) {
    const int b = blockIdx.x, lane = threadIdx.x;
    const int n = n_ops[b];
    int32_t* out = block_of_stage + size_t(b) * L;
    if (n < 0 || n > cap || n < L + 1) {  // uniform: a failed walk keeps its code, a short list is corrupt
        for (int k = lane; k < L; k += 64) out[k] = -1;
        if (lane == 0) n_blocks[b] = n < 0 ? n : (n > cap ? CKPT_E_ARG : CKPT_E_CORRUPT);
        return;
    }
    const ckpt_op_t* list = ops + size_t(b) * cap;
    int carry = 0;       // F_ck seen in earlier passes
    int prev_in = 0;     // was the last stage of the previous pass inside a block
    bool bad = false;
    for (int base = 0; base < L; base += 64) {  // L is uniform: every lane takes every pass
        const int k = base + lane;
        const bool valid = k < L;
        const int kind = valid ? list[k].kind : CKPT_OP_F_ALL;
        const int stage = valid ? list[k].stage : k + 1;
        const bool opens = valid && kind == CKPT_OP_F_CK;
        const bool inside = valid && (kind == CKPT_OP_F_CK || kind == CKPT_OP_F_NULL);
        int before = __shfl_up(int(inside), 1);
        if (lane == 0) before = prev_in;
        if (valid && (stage != k + 1 || kind > CKPT_OP_F_NULL || (kind == CKPT_OP_F_NULL && !before))) bad = true;
        int scan = int(opens);
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const int v = __shfl_up(scan, o);
            if (lane >= o) scan += v;
        }
        if (valid) out[k] = inside ? carry + scan - 1 : -1;
        carry += __shfl(scan, 63);
        prev_in = __shfl(int(inside), 63);
    }
    if (lane == 0 && (list[L].kind != CKPT_OP_B || list[L].stage != L)) bad = true;
    bad = __any(bad);
    if (bad)
        for (int k = lane; k < L; k += 64) out[k] = -1;
    if (lane == 0) n_blocks[b] = bad ? CKPT_E_CORRUPT : carry;
}

// Self-check of operation lists: one wave per chain executes its list under the memory model
// of Table 1 ("List of Operations").  The lanes stage the chain's arrays and the list through
// LDS; lane 0 carries the state: per stage j one byte with bit 0 = a^j resident on its own,
// bit 1 = abar^j resident, bit 2 = delta^j resident, and the running sum of resident sizes.
constexpr int kSimChunk = 256;  // operations staged per pass, a multiple of the wave size

__global__ void __launch_bounds__(64) simulate_kernel(ckpt_chains_t ch, int L, const ckpt_op_t* __restrict__ ops,
                                                       int cap, const int32_t* __restrict__ n_ops,
                                                       long long* __restrict__ time_out,
                                                       long long* __restrict__ peak_out, int32_t* __restrict__ status) {
    __shared__ int32_t s_uf[CKPT_MAX_L], s_ub[CKPT_MAX_L], s_wab[CKPT_MAX_L], s_of[CKPT_MAX_L], s_ob[CKPT_MAX_L];
    __shared__ int32_t s_wa[CKPT_MAX_L + 1], s_wd[CKPT_MAX_L + 1];
    __shared__ uint8_t s_state[CKPT_MAX_L + 2];
    __shared__ ckpt_op_t s_ops[kSimChunk];
    const int b = blockIdx.x, lane = threadIdx.x;
    const int n = n_ops[b];
    if (n < 0 || n > cap) {  // uniform over the wave
        if (lane == 0) {
            status[b] = n < 0 ? n : CKPT_E_ARG;
            time_out[b] = peak_out[b] = -1;
        }
        return;
    }
    const int32_t* wd = ch.wdelta ? ch.wdelta : ch.wa;
    for (int k = lane; k < L; k += 64) {
        s_uf[k] = ch.uf[size_t(b) * L + k];
        s_ub[k] = ch.ub[size_t(b) * L + k];
        s_wab[k] = ch.wabar[size_t(b) * L + k];
        s_of[k] = ch.of ? ch.of[size_t(b) * L + k] : 0;
        s_ob[k] = ch.ob ? ch.ob[size_t(b) * L + k] : 0;
    }
    for (int k = lane; k <= L; k += 64) {
        s_wa[k] = k ? ch.wa[size_t(b) * (L + 1) + k] : 0;  // the chain input a^0 is not counted
        s_wd[k] = wd[size_t(b) * (L + 1) + k];
        s_state[k] = k == 0 ? 1 : k == L ? 4 : 0;  // a^0 and delta^L are there from the start
    }
    __syncthreads();
    const ckpt_op_t* list = ops + size_t(b) * cap;
    long long time = 0, peak = 0, resident = s_wd[L];
    bool bad = false;
    for (int base = 0; base < n; base += kSimChunk) {  // n is uniform over the wave
        if (base) __syncthreads();  // lane 0 is done with the previous part of the list
        for (int k = lane; k < kSimChunk && base + k < n; k += 64) s_ops[k] = list[base + k];
        __syncthreads();
        if (lane != 0 || bad) continue;
        const int end = min(kSimChunk, n - base);
        for (int k = 0; k < end; ++k) {
            const int kind = s_ops[k].kind, j = s_ops[k].stage;
            if (j < 1 || j > L || kind > CKPT_OP_B) { bad = true; break; }
            const int in = s_state[j - 1], self = s_state[j];
            if (kind == CKPT_OP_B) {  // needs delta^j, abar^j and a^{j-1}; its output is not counted while it runs
                if (!(self & 4) || !(self & 2) || !(in & 3)) { bad = true; break; }
                peak = max(peak, resident + s_ob[j - 1]);
                resident -= (long long)s_wd[j] + s_wab[j - 1];
                if (in & 1) resident -= s_wa[j - 1];
                if (!(in & 4)) resident += s_wd[j - 1];
                s_state[j] = uint8_t(self & 1);
                s_state[j - 1] = uint8_t((in & 2) | 4);
                time += s_ub[j - 1];
            } else {  // a forward operation needs room for its output; F_null drops its input
                const int bit = kind == CKPT_OP_F_ALL ? 2 : 1;
                if (!(in & 3) || (kind == CKPT_OP_F_NULL && !(in & 1)) || (self & bit)) { bad = true; break; }
                const long long size = kind == CKPT_OP_F_ALL ? s_wab[j - 1] : s_wa[j];
                peak = max(peak, resident + size + s_of[j - 1]);
                resident += size;
                s_state[j] = uint8_t(self | bit);
                if (kind == CKPT_OP_F_NULL) {
                    resident -= s_wa[j - 1];
                    s_state[j - 1] = uint8_t(in & ~1);
                }
                time += s_uf[j - 1];
            }
        }
    }
    if (lane == 0) {
        if (!bad && !(s_state[0] & 4)) bad = true;  // the list must end with delta^0
        status[b] = bad ? CKPT_E_CORRUPT : CKPT_OK;
        time_out[b] = bad ? -1 : time;
        peak_out[b] = bad ? -1 : peak;
    }
}

int check_dims(int L, int M, int B) {
    if (L < 1 || M < 0 || B < 1) return CKPT_E_ARG;
    if (L > CKPT_MAX_L) return CKPT_E_LIMIT;
    const unsigned long long per_chain = (unsigned long long)ckpt_table_rows(L) * ckpt_row_pitch(M);
    if (per_chain >= (1ull << 30)) return CKPT_E_LIMIT;  // 4 GiB of int32 per chain
    if (B > 65535) return CKPT_E_LIMIT;                   // chains are the z dimension of the grids
    return CKPT_OK;
}

// Optional per-launch event trail of ckpt_solve_profiled.
struct Profile {
    hipStream_t stream = nullptr;
    std::vector<hipEvent_t> events;
    std::vector<int> kinds;
    unsigned long long* work = nullptr;  // device, 4 counters
    bool trail = true;                   // record an event after every launch
    bool mark(int kind) {
        if (!trail) return true;
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

// Per-device state of the library, kept for the life of the process:
//   helpers  three streams (default priority, non-blocking) and five events for the batch split;
//            with the caller's stream they make four, the number of hardware queues a process
//            gets by default (more streams than that share queues and serialise: six or eight
//            groups measured slower than one).  Created by ckpt_init or by the first solve
//            that wants to split, never while that solve's stream is being captured.
//   scratch  the device address of this GPU's copy of the static workspace below.
constexpr int kSideStreams = 3;
struct Device {
    hipStream_t stream[kSideStreams] = {};
    hipEvent_t join[kSideStreams] = {};
    hipEvent_t fork = nullptr;
    hipEvent_t stagger = nullptr;
    bool helpers_tried = false, helpers_ok = false;
    void* scratch = nullptr;
    std::mutex busy;  // one fork/join sequence at a time per device
};

// Workspace of ckpt_solve_batched_noalloc, for callers that cannot allocate: a fixed array in
// every GPU's copy of the code object, held until the process ends.  In host code the array's
// name is only a handle for hipGetSymbolAddress; kernels are given the resolved address.
static __device__ __align__(256) unsigned char g_scratch[CKPT_NOALLOC_MAX_WORKSPACE];

std::mutex g_devices_lock;
Device g_devices[64];

Device* current_device() {
    int dev = 0;
    if (!hip_ok(hipGetDevice(&dev)) || dev < 0 || dev >= 64) return nullptr;
    return &g_devices[dev];
}

// Both set-up steps run with the device current and under g_devices_lock.
bool ensure_helpers(Device& d) {
    std::lock_guard<std::mutex> guard(g_devices_lock);
    if (!d.helpers_tried) {
        d.helpers_tried = true;
        bool ok = hip_ok(hipEventCreateWithFlags(&d.fork, hipEventDisableTiming)) &&
                  hip_ok(hipEventCreateWithFlags(&d.stagger, hipEventDisableTiming));
        for (int k = 0; k < kSideStreams && ok; ++k)
            ok = hip_ok(hipStreamCreateWithFlags(&d.stream[k], hipStreamNonBlocking)) &&
                 hip_ok(hipEventCreateWithFlags(&d.join[k], hipEventDisableTiming));
        d.helpers_ok = ok;
    }
    return d.helpers_ok;
}

// Resolves this device's address of g_scratch once (the device must be current).
void* ensure_scratch(Device& d) {
    std::lock_guard<std::mutex> guard(g_devices_lock);
    if (!d.scratch) {
        void* p = nullptr;
        if (!hip_ok(hipGetSymbolAddress(&p, HIP_SYMBOL(g_scratch))) || !p) return nullptr;
        d.scratch = p;
    }
    return d.scratch;
}

bool helpers_ready(Device& d) {
    std::lock_guard<std::mutex> guard(g_devices_lock);
    return d.helpers_ok;
}

// The frontier kernel keeps its triangle in LDS; above the default per-block limit it has to be
// allowed the size.  Set once (to the largest size any L can need); allocates nothing.
bool allow_frontier_lds() {
    static std::once_flag once;
    static bool ok = false;
    std::call_once(once, [] {
        ok = hip_ok(hipFuncSetAttribute(reinterpret_cast<const void*>(frontier_kernel),
                                        hipFuncAttributeMaxDynamicSharedMemorySize,
                                        int(ckpt_table_rows(CKPT_MAX_L) * sizeof(int32_t))));
    });
    return ok;
}

int solve_impl(const ckpt_chains_t* chains, int L, int M, int B, void* stream, int32_t* cost, uint8_t* arg,
               void* workspace, Profile* prof, const ckpt_solve_opts_t* opts, bool may_create_helpers) {
    if (!chains || !cost || !arg || !workspace) return CKPT_E_ARG;
    if (int rc = check_dims(L, M, B)) return rc;
    if (!chains->uf || !chains->ub || !chains->wa || !chains->wabar) return CKPT_E_ARG;
    if ((reinterpret_cast<uintptr_t>(cost) | reinterpret_cast<uintptr_t>(arg) |
         reinterpret_cast<uintptr_t>(workspace)) & 255)
        return CKPT_E_ARG;
    const int want_groups = opts ? opts->groups : 0, want_ks = opts ? opts->list_split : 0;
    const int row_mode = opts ? opts->row_launches : 0;
    if (row_mode != 0 && row_mode != 1) return CKPT_E_ARG;
    const bool fused_rows = row_mode == 0;
    const int stagger = opts ? opts->stagger : 0;
    const int frontier_mode = opts ? opts->frontier : 0;
    const int spin_limit = opts && opts->spin_limit ? opts->spin_limit : kSpinLimit;
    if (frontier_mode < 0 || frontier_mode > 2) return CKPT_E_ARG;
    unsigned long long* work = prof ? prof->work : nullptr;
    if (want_groups < 0 || want_groups > kSideStreams + 1) return CKPT_E_ARG;
    if (want_ks != 0 && want_ks != 1 && want_ks != 2 && want_ks != 4) return CKPT_E_ARG;
    bool own_side = false;
    if (opts) {
        for (int k = 0; k < kSideStreams; ++k) own_side = own_side || opts->side_streams[k];
        for (int k = 0; k < kSideStreams && own_side; ++k)
            if (!opts->side_streams[k] && k + 2 <= (want_groups ? want_groups : kSideStreams + 1)) return CKPT_E_ARG;
    }
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int pitch = int(ckpt_row_pitch(M));
    const int rows = int(ckpt_table_rows(L));
    const Workspace ws = carve(workspace, L, pitch, B);

    const size_t frontier_lds = ckpt_table_rows(L) * sizeof(int32_t);
    if (frontier_lds > 48 * 1024 && !allow_frontier_lds()) return CKPT_E_HIP;
    constexpr int T = kT;
    const int nblk = (L + T - 1) / T;
    const int gx_row = (pitch + kRowWG - 1) / kRowWG;

    // Several streams.  Chains are independent, so from D = 2 on the batch is split in up to four
    // groups that run the same launch sequence on as many streams: the many short row launches
    // of one group overlap with work of the others instead of leaving the machine idle between
    // dependent launches.  The frontier kernel (a few busy CUs for a long time) runs on the first
    // side stream beside everything else: the fill prunes with whatever frontier is in memory,
    // the weak one of the precompute kernel or the exact one.  The side streams are forked from
    // and joined back into the caller's stream with events.  Small problems are bound by launch
    // latency, where more streams only add launches.
    // Automatic choice: split when the batch is large enough to be bound by the GPU and not by
    // launch latency (where more streams only add launches).  The caller can force either way.
    const bool large = B >= 2 && size_t(B) * nblk * pitch >= (size_t(1) << 19);

    int groups = want_groups ? want_groups : (large ? kSideStreams + 1 : 1);
    groups = std::min(groups, B);
    if (prof || nblk < 3) groups = 1;  // the event trail times one stream; no diagonal to split
    Device* dev = nullptr;
    if (groups > 1) {
        dev = current_device();
        if (!dev) return CKPT_E_HIP;
        if (!helpers_ready(*dev)) {
            // Streams and events are not created behind a capture: a captured stream must only see
            // enqueued work.  ckpt_init beforehand makes the split available to captured solves.
            hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
            if (!hip_ok(hipStreamIsCapturing(st, &cap))) return CKPT_E_HIP;
            if (cap != hipStreamCaptureStatusNone || !may_create_helpers) {
                if (want_groups > 1) return CKPT_E_NOTREADY;
                groups = 1;
            } else if (!ensure_helpers(*dev)) {
                return CKPT_E_HIP;
            }
        }
    }
    Device* side = groups > 1 ? dev : nullptr;
    // The exact frontier costs one long single-block launch per chain (about 2 us per stage).  On
    // a side stream it runs beside the fill for free; on the caller's stream it pays only when
    // the pruning it adds (about a third of the block products) saves more than it costs.
    const bool want_frontier =
        frontier_mode == 1 || (frontier_mode == 0 && (groups > 1 || size_t(B) * pitch * nblk * nblk >= 6000000));
    std::unique_lock<std::mutex> lock;
    if (side) lock = std::unique_lock<std::mutex>(side->busy);  // one fork/join at a time per device
    hipStream_t gs[kSideStreams + 1] = {st, st, st, st};  // stream of group g
    hipStream_t side_stream[kSideStreams] = {};
    for (int g = 1; g < groups; ++g)
        gs[g] = side_stream[g - 1] = own_side ? static_cast<hipStream_t>(opts->side_streams[g - 1]) : side->stream[g - 1];
    int first[kSideStreams + 2];  // group g holds chains first[g] .. first[g + 1] - 1
    for (int g = 0; g <= groups; ++g) first[g] = int((long long)B * g / groups);

    int forked = 0;  // side streams that wait on the caller's stream and have to be joined back
    auto join_side = [&](int k) {  // the caller's stream waits for side stream k
        return hip_ok(hipEventRecord(side->join[k], side_stream[k])) &&
               hip_ok(hipStreamWaitEvent(st, side->join[k], 0));
    };
    auto enqueue = [&]() -> int {
        hipLaunchKernelGGL(precompute_kernel, dim3(B), dim3(256), 0, st, *chains, L, pitch, ws);
        CKPT_AFTER_LAUNCH(CKPT_K_PRECOMPUTE);
        if (side) {
            if (!hip_ok(hipEventRecord(side->fork, st)) || !hip_ok(hipStreamWaitEvent(gs[1], side->fork, 0)))
                return CKPT_E_HIP;
            forked = 1;
        }
        if (want_frontier) {
            hipLaunchKernelGGL(frontier_kernel, dim3(B), dim3(1024), frontier_lds, gs[1], *chains, L, ws);
            CKPT_AFTER_LAUNCH(CKPT_K_FRONTIER);
        }

        const int nbands = bands_of(pitch);
        for (int D = 0; D < 2 && D < nblk; ++D) {
            const Ctx ctx{L, M, pitch, rows, 0, spin_limit, ws, cost, arg, work};
            if (fused_rows) {
                const dim3 grid(nbands, nblk - D, B);
                int32_t* tick = ws.tick + D * kTickGroups;
                const auto fn = D == 0 ? (work ? tile_rows_kernel<0, true> : tile_rows_kernel<0, false>)
                                       : (work ? tile_rows_kernel<1, true> : tile_rows_kernel<1, false>);
                hipLaunchKernelGGL(fn, grid, dim3(kRowWG), 0, st, ctx, D, tick);
                CKPT_AFTER_LAUNCH(CKPT_K_ROW);
                continue;
            }
            const auto& rowfn = D == 0 ? kRow0 : kRow1;
            for (int r = T - 1; r >= 0; --r) {
                hipLaunchKernelGGL(rowfn[r], dim3(gx_row, nblk - D, B), dim3(kRowWG), 0, st, ctx, D);
                CKPT_AFTER_LAUNCH(CKPT_K_ROW);
            }
        }
        if (side) {
            // every side stream waits for the D < 2 rows.  Nobody waits for the frontier kernel: the
            // fill uses whatever frontier is in memory, and the group on its stream follows it anyway.
            if (!hip_ok(hipEventRecord(side->fork, st))) return CKPT_E_HIP;
            for (int g = 1; g < groups; ++g) {
                if (!hip_ok(hipStreamWaitEvent(gs[g], side->fork, 0))) return CKPT_E_HIP;
                forked = g;
            }
        }
        for (int D = 2; D < nblk; ++D) {
            // Later diagonals have fewer tiles and longer work lists.  The chip holds 2048 of these
            // waves; once a launch brings fewer than about three and a half times that, whole-list
            // waves leave the machine half empty while the last ones finish, so 2 waves share each
            // chunk and split its list (measured: a gain from there on, a loss with more tiles,
            // where the lists are short); with fewer waves than a quarter of the chip, 4 do.
            const long long waves = (long long)(nblk - D) * (pitch / 64) * B;
            const int ks = want_ks ? want_ks : (waves <= 600 ? 4 : (waves <= 7000 ? 2 : 1));
            const int gx = (pitch / 64 + kCH / ks - 1) / (kCH / ks);
            for (int g = 0; g < groups; ++g) {
                const Ctx ctx{L, M, pitch, rows, first[g], spin_limit, ws, cost, arg, work};
                const dim3 grid(gx, nblk - D, first[g + 1] - first[g]), block(64 * kCH);
                const auto fn = ks == 4 ? (work ? gemm_kernel<3, 3, kCH / 4, 4, true> : gemm_kernel<3, 3, kCH / 4, 4, false>)
                              : ks == 2 ? (work ? gemm_kernel<3, 3, kCH / 2, 2, true> : gemm_kernel<3, 3, kCH / 2, 2, false>)
                                        : (work ? gemm_kernel<3, 3, kCH, 1, true> : gemm_kernel<3, 3, kCH, 1, false>);
                hipLaunchKernelGGL(fn, grid, block, 0, gs[g], ctx, D);
                CKPT_AFTER_LAUNCH(CKPT_K_GEMM);
                if (D == 2 && g == 0 && side && stagger && groups >= 3) {
                    // the second half of the groups starts when the first group's block product is
                    // done: from then on their bandwidth-bound and latency-bound phases alternate
                    if (!hip_ok(hipEventRecord(side->stagger, gs[0]))) return CKPT_E_HIP;
                    for (int h = (groups + 1) / 2; h < groups; ++h)
                        if (!hip_ok(hipStreamWaitEvent(gs[h], side->stagger, 0))) return CKPT_E_HIP;
                }
            }
            if (fused_rows) {  // rows 6..0 of every tile of the diagonal in one launch per group
                for (int g = 0; g < groups; ++g) {
                    const Ctx ctx{L, M, pitch, rows, first[g], spin_limit, ws, cost, arg, work};
                    const auto fn = work ? tile_rows_kernel<2, true> : tile_rows_kernel<2, false>;
                    hipLaunchKernelGGL(fn, dim3(nbands, nblk - D, first[g + 1] - first[g]), dim3(kRowWG), 0, gs[g], ctx,
                                       D, ws.tick + D * kTickGroups + g);
                    CKPT_AFTER_LAUNCH(CKPT_K_ROW);
                }
                continue;
            }
            // rows of the groups are issued in turn so that every queue stays fed; row 7 was
            // finished by the gemm
            for (int r = T - 2; r >= 0; --r) {
                for (int g = 0; g < groups; ++g) {
                    const Ctx ctx{L, M, pitch, rows, first[g], spin_limit, ws, cost, arg, work};
                    hipLaunchKernelGGL(kRow2[r], dim3(gx_row, nblk - D, first[g + 1] - first[g]), dim3(kRowWG), 0,
                                       gs[g], ctx, D);
                    CKPT_AFTER_LAUNCH(CKPT_K_ROW);
                }
            }
        }
        return CKPT_OK;
    };
    int rc = enqueue();
    // Every forked side stream rejoins the caller's stream, also after a failed launch, so that
    // the caller's stream (or a capture in progress) is never left with an open fork.
    for (int k = 0; k < forked; ++k)
        if (!join_side(k) && rc == CKPT_OK) rc = CKPT_E_HIP;
    return rc;
}

}  // namespace

extern "C" {

size_t ckpt_workspace_bytes(int L, int M, int B) {
    if (L < 1 || M < 0 || B < 1) return 0;
    return ws_ints(L, int(ckpt_row_pitch(M)), B) * sizeof(int32_t);
}

int ckpt_init(int device) {
    if (device >= 64) return CKPT_E_LIMIT;
    int prev = 0;
    if (!hip_ok(hipGetDevice(&prev))) return CKPT_E_HIP;
    if (device < 0) device = prev;
    if (device >= 64) return CKPT_E_LIMIT;
    if (device != prev && !hip_ok(hipSetDevice(device))) return CKPT_E_HIP;
    Device& d = g_devices[device];
    const bool ok = ensure_helpers(d) && ensure_scratch(d) != nullptr && allow_frontier_lds();
    if (device != prev && !hip_ok(hipSetDevice(prev))) return CKPT_E_HIP;
    return ok ? CKPT_OK : CKPT_E_HIP;
}

int ckpt_solve_batched(const ckpt_chains_t* chains, int L, int M, int B, void* stream, int32_t* cost,
                       uint8_t* arg, void* workspace) {
    return solve_impl(chains, L, M, B, stream, cost, arg, workspace, nullptr, nullptr, true);
}

int ckpt_solve_batched_noalloc(const ckpt_chains_t* chains, int L, int M, int B, void* stream, int32_t* cost,
                               uint8_t* arg) {
    if (int rc = check_dims(L, M, B)) return rc;
    if (ckpt_workspace_bytes(L, M, B) > CKPT_NOALLOC_MAX_WORKSPACE) return CKPT_E_LIMIT;
    Device* dev = current_device();
    if (!dev) return CKPT_E_HIP;
    void* scratch = ensure_scratch(*dev);
    if (!scratch) return CKPT_E_HIP;
    // creates nothing: the batch is split only if the helper streams exist already
    return solve_impl(chains, L, M, B, stream, cost, arg, scratch, nullptr, nullptr, false);
}

int ckpt_solve_batched_opts(const ckpt_chains_t* chains, int L, int M, int B, void* stream, int32_t* cost,
                            uint8_t* arg, void* workspace, const ckpt_solve_opts_t* opts) {
    return solve_impl(chains, L, M, B, stream, cost, arg, workspace, nullptr, opts, true);
}

int ckpt_solve_profiled(const ckpt_chains_t* chains, int L, int M, int B, void* stream, int32_t* cost,
                        uint8_t* arg, void* workspace, float* kind_ms, int* kind_launches, double* kind_bytes) {
    if (!kind_ms || !kind_launches) return CKPT_E_ARG;
    hipStream_t st = static_cast<hipStream_t>(stream);
    Profile prof;
    prof.stream = st;
    for (int k = 0; k < CKPT_N_KERNEL_KINDS; ++k) kind_ms[k] = 0.f, kind_launches[k] = 0;
    int rc = CKPT_OK;
    if (!prof.mark(-1)) rc = CKPT_E_HIP;
    if (rc == CKPT_OK) rc = solve_impl(chains, L, M, B, stream, cost, arg, workspace, &prof, nullptr, false);
    if (!hip_ok(hipStreamSynchronize(st)) && rc == CKPT_OK) rc = CKPT_E_HIP;
    for (size_t i = 1; i < prof.events.size() && rc == CKPT_OK; ++i) {
        float ms = 0.f;
        if (!hip_ok(hipEventElapsedTime(&ms, prof.events[i - 1], prof.events[i]))) rc = CKPT_E_HIP;
        kind_ms[prof.kinds[i]] += ms;
        kind_launches[prof.kinds[i]] += 1;
    }
    for (hipEvent_t e : prof.events) (void)hipEventDestroy(e);
    if (kind_bytes && rc == CKPT_OK) {
        // a second, untimed pass in which every wave adds up the bytes it asks for
        for (int k = 0; k < 2 * CKPT_N_KERNEL_KINDS; ++k) kind_bytes[k] = 0.0;
        Profile count;
        count.stream = st;
        count.trail = false;
        std::vector<unsigned long long> host(size_t(kWorkSets) * 4, 0);
        const size_t bytes = host.size() * sizeof(unsigned long long);
        if (!hip_ok(hipMalloc(reinterpret_cast<void**>(&count.work), bytes))) return CKPT_E_HIP;
        if (!hip_ok(hipMemsetAsync(count.work, 0, bytes, st))) rc = CKPT_E_HIP;
        if (rc == CKPT_OK) rc = solve_impl(chains, L, M, B, stream, cost, arg, workspace, &count, nullptr, false);
        if (rc == CKPT_OK && !hip_ok(hipMemcpyAsync(host.data(), count.work, bytes, hipMemcpyDeviceToHost, st)))
            rc = CKPT_E_HIP;
        if (!hip_ok(hipStreamSynchronize(st)) && rc == CKPT_OK) rc = CKPT_E_HIP;
        (void)hipFree(count.work);
        for (int set = 0; set < kWorkSets; ++set) {
            kind_bytes[2 * CKPT_K_GEMM] += double(host[set * 4]);
            kind_bytes[2 * CKPT_K_GEMM + 1] += double(host[set * 4 + 1]);
            kind_bytes[2 * CKPT_K_ROW] += double(host[set * 4 + 2]);
            kind_bytes[2 * CKPT_K_ROW + 1] += double(host[set * 4 + 3]);
        }
    }
    return rc;
}

const char* ckpt_kernel_name(int kind) {
    switch (kind) {
        case CKPT_K_PRECOMPUTE: return "precompute_kernel";
        case CKPT_K_FRONTIER: return "frontier_kernel";
        case CKPT_K_GEMM: return "gemm_kernel";
        case CKPT_K_ROW: return "tile_rows_kernel";
        default: return nullptr;
    }
}

int ckpt_check_inputs(const void* workspace, int L, int M, int B, void* stream, int32_t* flags_host) {
    if (!flags_host) return CKPT_E_ARG;
    if (int rc = check_dims(L, M, B)) return rc;
    if (!workspace) {  // the static workspace of ckpt_solve_batched_noalloc on the current device
        if (ckpt_workspace_bytes(L, M, B) > CKPT_NOALLOC_MAX_WORKSPACE) return CKPT_E_LIMIT;
        Device* dev = current_device();
        workspace = dev ? ensure_scratch(*dev) : nullptr;
        if (!workspace) return CKPT_E_HIP;
    }
    const Workspace ws = carve(const_cast<void*>(workspace), L, int(ckpt_row_pitch(M)), B);
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (!hip_ok(hipMemcpyAsync(flags_host, ws.flags, size_t(B) * sizeof(int32_t), hipMemcpyDeviceToHost, st)))
        return CKPT_E_HIP;
    int32_t fault = 0;
    if (!hip_ok(hipMemcpyAsync(&fault, ws.fault, sizeof(int32_t), hipMemcpyDeviceToHost, st))) return CKPT_E_HIP;
    if (!hip_ok(hipStreamSynchronize(st))) return CKPT_E_HIP;
    if (fault) return CKPT_E_INTERNAL;
    for (int b = 0; b < B; ++b)
        if (flags_host[b]) return CKPT_E_INPUT;
    return CKPT_OK;
}

int ckpt_select_plan(const int32_t* cost, int L, int M, int B, const int32_t* m_budget, void* stream,
                     int32_t* out) {
    if (!cost || !m_budget || !out) return CKPT_E_ARG;
    if (int rc = check_dims(L, M, B)) return rc;
    hipLaunchKernelGGL(select_kernel, dim3(1), dim3(256), 0, static_cast<hipStream_t>(stream), cost, L, M,
                       int(ckpt_row_pitch(M)), int(ckpt_table_rows(L)), B, m_budget, out);
    return hip_ok(hipGetLastError()) ? CKPT_OK : CKPT_E_HIP;
}

int ckpt_discretize(const int64_t* bytes_wa, const int64_t* bytes_wabar, const int64_t* bytes_wdelta,
                    const int64_t* bytes_of, const int64_t* bytes_ob, const int64_t* budget_bytes, int L,
                    int M, int B, void* stream, const ckpt_chains_t* out) {
    if (!bytes_wa || !bytes_wabar || !budget_bytes || !out || !out->wa || !out->wabar) return CKPT_E_ARG;
    if ((bytes_wdelta && !out->wdelta) || (bytes_of && !out->of) || (bytes_ob && !out->ob)) return CKPT_E_ARG;
    if (int rc = check_dims(L, M, B)) return rc;
    if (M > (1 << 20)) return CKPT_E_LIMIT;
    hipStream_t st = static_cast<hipStream_t>(stream);
    struct Job { const int64_t* in; const int32_t* out; int n; };
    const Job jobs[5] = {{bytes_wa, out->wa, L + 1}, {bytes_wabar, out->wabar, L}, {bytes_wdelta, out->wdelta, L + 1},
                         {bytes_of, out->of, L}, {bytes_ob, out->ob, L}};
    for (const Job& j : jobs) {
        if (!j.in) continue;
        hipLaunchKernelGGL(discretize_kernel, dim3((j.n + 255) / 256, B), dim3(256), 0, st,
                           reinterpret_cast<const long long*>(j.in), const_cast<int32_t*>(j.out),
                           reinterpret_cast<const long long*>(budget_bytes), j.n, M);
        if (!hip_ok(hipGetLastError())) return CKPT_E_HIP;
    }
    return CKPT_OK;
}

int ckpt_discretize_sweep(const int64_t* bytes_wa, const int64_t* bytes_wabar, const int64_t* bytes_wdelta,
                          const int64_t* bytes_of, const int64_t* bytes_ob, int64_t base_budget, int alpha_num,
                          int alpha_den, int count, int L, int M, void* stream, int64_t* budgets_out,
                          const ckpt_chains_t* out) {
    if (!bytes_wa || !bytes_wabar || !out || !out->wa || !out->wabar) return CKPT_E_ARG;
    if ((bytes_wdelta && !out->wdelta) || (bytes_of && !out->of) || (bytes_ob && !out->ob)) return CKPT_E_ARG;
    SweepBudgets budget{};
    static_assert(sizeof(long long) == sizeof(int64_t), "budget words");
    if (int rc = ckpt_budget_sweep(base_budget, alpha_num, alpha_den, count, reinterpret_cast<int64_t*>(budget.v)))
        return rc;
    if (int rc = check_dims(L, M, count)) return rc;
    if (M > (1 << 20)) return CKPT_E_LIMIT;
    hipStream_t st = static_cast<hipStream_t>(stream);
    struct Job { const int64_t* in; const int32_t* out; int n; };
    const Job jobs[5] = {{bytes_wa, out->wa, L + 1}, {bytes_wabar, out->wabar, L}, {bytes_wdelta, out->wdelta, L + 1},
                         {bytes_of, out->of, L}, {bytes_ob, out->ob, L}};
    for (const Job& j : jobs) {
        if (!j.in) continue;
        hipLaunchKernelGGL(discretize_sweep_kernel, dim3((j.n + 255) / 256, count), dim3(256), 0, st,
                           reinterpret_cast<const long long*>(j.in), const_cast<int32_t*>(j.out), budget, j.n, M);
        if (!hip_ok(hipGetLastError())) return CKPT_E_HIP;
    }
    if (budgets_out) {
        hipLaunchKernelGGL(store_budgets_kernel, dim3(1), dim3(64), 0, st, budget, count,
                           reinterpret_cast<long long*>(budgets_out));
        if (!hip_ok(hipGetLastError())) return CKPT_E_HIP;
    }
    return CKPT_OK;
}

size_t ckpt_schedule_workspace_bytes(int L, int B) {
    if (L < 1 || B < 1) return 0;
    return size_t(B) * (2 * size_t(L) + 2) * sizeof(int4);
}

int ckpt_schedule_batched(const uint8_t* arg, const int32_t* wa, const int32_t* wabar, int L, int M, int B,
                          const int32_t* m_budget, void* stream, ckpt_op_t* ops, int ops_cap, int32_t* n_ops,
                          void* workspace) {
    if (!arg || !wa || !wabar || !m_budget || !ops || !n_ops || !workspace || ops_cap < 0) return CKPT_E_ARG;
    if (reinterpret_cast<uintptr_t>(workspace) & 15) return CKPT_E_ARG;
    if (int rc = check_dims(L, M, B)) return rc;
    hipLaunchKernelGGL(schedule_kernel, dim3((B + 63) / 64), dim3(64), 0, static_cast<hipStream_t>(stream), arg, wa,
                       wabar, L, M, int(ckpt_row_pitch(M)), int(ckpt_table_rows(L)), B, m_budget, ops, ops_cap,
                       n_ops, static_cast<int4*>(workspace));
    return hip_ok(hipGetLastError()) ? CKPT_OK : CKPT_E_HIP;
}

int ckpt_block_indices_batched(const ckpt_op_t* ops, int ops_cap, const int32_t* n_ops, int L, int B, void* stream,
                               int32_t* block_of_stage, int32_t* n_blocks) {
    if (!ops || !n_ops || !block_of_stage || !n_blocks || ops_cap < 0 || L < 1 || B < 1) return CKPT_E_ARG;
    if (L > CKPT_MAX_L) return CKPT_E_LIMIT;
    hipLaunchKernelGGL(block_index_kernel, dim3(B), dim3(64), 0, static_cast<hipStream_t>(stream), ops, ops_cap, n_ops,
                       L, block_of_stage, n_blocks);
    return hip_ok(hipGetLastError()) ? CKPT_OK : CKPT_E_HIP;
}

int ckpt_simulate_batched(const ckpt_chains_t* chains, int L, int B, const ckpt_op_t* ops, int ops_cap,
                          const int32_t* n_ops, void* stream, int64_t* time_out, int64_t* peak_out,
                          int32_t* status) {
    if (!chains || !chains->uf || !chains->ub || !chains->wa || !chains->wabar || !ops || !n_ops || !time_out ||
        !peak_out || !status || ops_cap < 0 || L < 1 || B < 1)
        return CKPT_E_ARG;
    if (L > CKPT_MAX_L) return CKPT_E_LIMIT;
    hipLaunchKernelGGL(simulate_kernel, dim3(B), dim3(64), 0, static_cast<hipStream_t>(stream), *chains, L, ops,
                       ops_cap, n_ops, reinterpret_cast<long long*>(time_out), reinterpret_cast<long long*>(peak_out),
                       status);
    return hip_ok(hipGetLastError()) ? CKPT_OK : CKPT_E_HIP;
}

int ckpt_last_hip_error(void) { return g_last_hip_error.load(); }


}  // extern "C"
