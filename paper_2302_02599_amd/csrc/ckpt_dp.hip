// Batched activation-checkpoint dynamic program on gfx950: kernels and C ABI.
//
// Computes C_BP(s, t, m) of the paper's Theorem (Section "Activation Checkpoint
// Solver / Modeling") for B chains at once.  See include/ckpt_dp.h for the
// conventions (candidate numbering, saturation at 2^30, table layout).
#include <hip/hip_runtime.h>

#include <atomic>
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
// Workspace layout (int32 units), all per chain b:
//   P     [B][L+1]   P[i] = sum of u_f of stages 1..i
//   fb    [B][L]     u_f^s + u_b^s
//   mall  [B][L][L]  m_all^{s,t}  at [(s-1)*L + (t-1)]
//   mnull [B][L][L]  m_null^{s,t}
//   flags [B]        input precondition flags
// ---------------------------------------------------------------------------
struct Workspace {
    int32_t* P;
    int32_t* fb;
    int32_t* mall;
    int32_t* mnull;
    int32_t* flags;
};

inline size_t align64(size_t n) { return (n + 63) & ~size_t(63); }

inline size_t ws_ints(int L, int B) {
    return align64(size_t(B) * (L + 1)) + align64(size_t(B) * L) + 2 * align64(size_t(B) * L * L) +
           align64(size_t(B));
}

inline Workspace carve(void* base, int L, int B) {
    int32_t* p = static_cast<int32_t*>(base);
    Workspace w;
    w.P = p;      p += align64(size_t(B) * (L + 1));
    w.fb = p;     p += align64(size_t(B) * L);
    w.mall = p;   p += align64(size_t(B) * L * L);
    w.mnull = p;  p += align64(size_t(B) * L * L);
    w.flags = p;
    return w;
}

__host__ __device__ inline int tri_row(int L, int s0, int t0) {  // 0-based s0 <= t0
    return s0 * L - (s0 * (s0 - 1)) / 2 + (t0 - s0);
}

// One block per chain.  Thread 0 builds the prefix sums and the flags; thread s0
// builds row s of both threshold tables with a running maximum over t (last display
// of the Theorem).
__global__ void precompute_kernel(ckpt_chains_t ch, int L, Workspace ws) {
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
            acc += f > 0 ? f : 0;
            if (acc >= (1ll << 30)) { flags |= 2; acc = (1ll << 30) - 1; }
            P[k + 1] = static_cast<int32_t>(acc);
            ws.fb[size_t(b) * L + k] = static_cast<int32_t>(
                min(static_cast<long long>(kInf), static_cast<long long>(f > 0 ? f : 0) + (bw > 0 ? bw : 0)));
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
        int sweep = sz(wa[s]) + ofs;  // wa^s + o_f^s, then max over s+1 <= j < t
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

// Reference-shaped fill of one anti-diagonal d = t - s: one thread per (chain, s, m),
// serial loop over the split point.  Operands come straight from global memory.
__global__ void __launch_bounds__(256)
diag_kernel(ckpt_chains_t ch, int L, int M, int pitch, int rows, int d, Workspace ws,
            int32_t* __restrict__ cost, uint8_t* __restrict__ arg) {
    const int b = blockIdx.z;
    const int s0 = blockIdx.y;  // 0-based stage s-1
    const int t0 = s0 + d;
    const int m = blockIdx.x * blockDim.x + threadIdx.x;
    if (m > M) return;
    const int32_t* wa = ch.wa + size_t(b) * (L + 1);
    const int32_t* wab = ch.wabar + size_t(b) * L;
    const int32_t* P = ws.P + size_t(b) * (L + 1);
    const int32_t* tab = cost + size_t(b) * rows * pitch;
    const uint32_t mall = ws.mall[(size_t(b) * L + s0) * L + t0];
    const uint32_t mnull = ws.mnull[(size_t(b) * L + s0) * L + t0];
    const uint32_t fb = ws.fb[size_t(b) * L + s0];

    uint32_t best = kInf;
    uint32_t pick = 0;
    if (uint32_t(m) >= mall) {
        uint32_t v = fb;
        if (d > 0) {
            const int mm = m - min(max(wab[s0], 0), pitch);
            v += (mm >= 0) ? uint32_t(tab[size_t(tri_row(L, s0 + 1, t0)) * pitch + mm]) : kInf;
        }
        v = min(v, kInf);
        if (v < best) { best = v; pick = s0 + 1; }
    }
    if (d > 0 && uint32_t(m) >= mnull) {
        const int32_t* left = tab + size_t(tri_row(L, s0, s0)) * pitch + m;  // rows (s, s..t-1)
        const uint32_t Ps = P[s0];
        for (int q0 = s0 + 1; q0 <= t0; ++q0) {  // q0 = 0-based s'-1 ... candidate stage s' = q0 + 1
            const int mm = m - min(max(wa[q0], 0), pitch);
            const uint32_t r = (mm >= 0) ? uint32_t(tab[size_t(tri_row(L, q0, t0)) * pitch + mm]) : kInf;
            const uint32_t l = uint32_t(left[size_t(q0 - 1 - s0) * pitch]);
            const uint32_t v = min(uint32_t(P[q0]) - Ps + r + l, kInf);
            if (v < best) { best = v; pick = q0 + 1; }
        }
    }
    const size_t o = (size_t(b) * rows + tri_row(L, s0, t0)) * pitch + m;
    cost[o] = int32_t(best);
    arg[o] = uint8_t(pick);
}

int check_dims(int L, int M, int B) {
    if (L < 1 || M < 0 || B < 1) return CKPT_E_ARG;
    if (L > CKPT_MAX_L) return CKPT_E_LIMIT;
    const unsigned long long per_chain = (unsigned long long)ckpt_table_rows(L) * ckpt_row_pitch(M);
    if (per_chain > 0x7fffffffull) return CKPT_E_LIMIT;
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

    hipLaunchKernelGGL(precompute_kernel, dim3(B), dim3(64), 0, st, *chains, L, ws);
    CKPT_AFTER_LAUNCH(CKPT_K_PRECOMPUTE);
    const int mblocks = (M + 1 + 255) / 256;
    for (int d = 0; d < L; ++d) {
        hipLaunchKernelGGL(diag_kernel, dim3(mblocks, L - d, B), dim3(256), 0, st, *chains, L, M, pitch, rows,
                           d, ws, cost, arg);
        CKPT_AFTER_LAUNCH(CKPT_K_DIAG);
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
        case CKPT_K_DIAG: return "diag_kernel";
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
