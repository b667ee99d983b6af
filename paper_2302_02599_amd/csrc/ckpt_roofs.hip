// Measured roofs of one MI355X for the benchmark harness (bench.py --roofs).  Not part of the
// solver: a separate small library (libckpt_roofs.so) with its own C ABI, so that the figures
// the roofline is judged against can be reproduced from committed code.
//
//   ckpt_roof_copy       plain device copy, 16 bytes per lane: what the box streams at best
//   ckpt_roof_read       read-only stream over a buffer, one launch per pass: with a buffer that
//                        fits the 256 MB Infinity Cache the later passes are served from it
//   ckpt_roof_read_rows  the block-product kernel's access pattern without its arithmetic: a
//                        wave reads 16 table rows of 256 bytes per step (8 at the same columns,
//                        8 at a shifted, unaligned column), loads two steps ahead
//   ckpt_roof_alu        register-only 8x8 candidate tile per lane: float64 key add + min;
//                        32-bit add, compare and two selects; 32-bit add + min
// Every call records two events around its launches on `stream`, waits, and returns the time.
#include <hip/hip_runtime.h>

#include <cstddef>
#include <cstdint>

namespace {

__global__ void __launch_bounds__(256) copy_kernel(uint4* __restrict__ dst, const uint4* __restrict__ src, size_t n) {
    size_t i = blockIdx.x * size_t(blockDim.x) + threadIdx.x;
    const size_t stride = size_t(gridDim.x) * blockDim.x;
    for (; i < n; i += stride) dst[i] = src[i];
}

__global__ void __launch_bounds__(256) read_kernel(const uint4* __restrict__ src, size_t n, uint32_t* sink) {
    size_t i = blockIdx.x * size_t(blockDim.x) + threadIdx.x;
    const size_t stride = size_t(gridDim.x) * blockDim.x;
    uint32_t acc = 0;
    for (; i < n; i += stride) {
        const uint4 v = src[i];
        acc += v.x ^ v.y ^ v.z ^ v.w;
    }
    if (acc == 0x12345u) sink[0] = acc;  // keeps the loads alive; the buffer is zero-filled
}

// One wave per (tile, chunk of 64 columns); step q reads rows base + r*nq + q, r = 0..15, rows 8..15
// at column m - shift.  Three operand buffers: the loads of step q + 2 are issued before step q
// is consumed, as in the solver's kernel.
__global__ void __launch_bounds__(256) read_rows_kernel(const uint32_t* __restrict__ tab, int pitch, int nq, int shift,
                                                        uint32_t* sink) {
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int chunk = blockIdx.x * 4 + wave;
    if (chunk * 64 >= pitch) return;  // wave-uniform
    const uint32_t m = chunk * 64 + lane;
    const size_t base = size_t(blockIdx.y) * 16 * nq + 1;  // +1: the shifted read of the first row stays inside
    uint32_t buf[3][16];
    auto load = [&](uint32_t(&v)[16], int q) {
#pragma unroll
        for (int r = 0; r < 8; ++r) v[r] = tab[(base + size_t(r) * nq + q) * pitch + m];
#pragma unroll
        for (int r = 8; r < 16; ++r) v[r] = tab[(base + size_t(r) * nq + q) * pitch + m - shift];
    };
    uint32_t acc = 0;
    load(buf[0], 0);
    load(buf[1], min(1, nq - 1));
    for (int q = 0; q < nq; q += 3) {
#pragma unroll
        for (int u = 0; u < 3; ++u) {
            load(buf[(u + 2) % 3], min(q + u + 2, nq - 1));
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int r = 0; r < 16; ++r) acc += buf[u][r];
            __builtin_amdgcn_sched_barrier(0);
        }
    }
    if (acc == 0x12345u) sink[0] = acc;
}

constexpr int R = 8, C = 8;

// kind 0: key = l + r (float64), best = min(best, key)
__global__ void __launch_bounds__(64) alu_f64_kernel(const uint32_t* __restrict__ in, uint32_t* out, int iters) {
    double best[R][C], l[R], rv[C];
    const int tid = blockIdx.x * 64 + threadIdx.x;
#pragma unroll
    for (int r = 0; r < R; ++r) l[r] = double(in[(tid + r * 64) & 4095]);
#pragma unroll
    for (int c = 0; c < C; ++c) rv[c] = double(in[(tid + 512 + c * 64) & 4095]);
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
        for (int c = 0; c < C; ++c) best[r][c] = 1e300;
    for (int q = 0; q < iters; ++q) {
#pragma unroll
        for (int r = 0; r < R; ++r)
#pragma unroll
            for (int c = 0; c < C; ++c) best[r][c] = fmin(best[r][c], l[r] + rv[c]);
#pragma unroll
        for (int r = 0; r < R; ++r) l[r] += 1.0;  // new operands every step, 16 extra operations per 128
#pragma unroll
        for (int c = 0; c < C; ++c) rv[c] += 3.0;
    }
    double acc = 0;
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
        for (int c = 0; c < C; ++c) acc += best[r][c];
    out[tid] = uint32_t(acc);
}

// kind 1: v = l + r; if (v < best) best = v, pick = q.   kind 2: best = min(best, l + r)
template <bool PICK>
__global__ void __launch_bounds__(64) alu_u32_kernel(const uint32_t* __restrict__ in, uint32_t* out, int iters) {
    uint32_t best[R][C], pick[R][C], l[R], rv[C];
    const int tid = blockIdx.x * 64 + threadIdx.x;
#pragma unroll
    for (int r = 0; r < R; ++r) l[r] = in[(tid + r * 64) & 4095];
#pragma unroll
    for (int c = 0; c < C; ++c) rv[c] = in[(tid + 512 + c * 64) & 4095];
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
        for (int c = 0; c < C; ++c) best[r][c] = 0x7fffffffu, pick[r][c] = 0;
    for (int q = 0; q < iters; ++q) {
#pragma unroll
        for (int r = 0; r < R; ++r)
#pragma unroll
            for (int c = 0; c < C; ++c) {
                const uint32_t v = l[r] + rv[c];
                if (PICK) {
                    if (v < best[r][c]) best[r][c] = v, pick[r][c] = q;
                } else {
                    best[r][c] = min(best[r][c], v);
                }
            }
#pragma unroll
        for (int r = 0; r < R; ++r) l[r] = l[r] * 3u + 1u;
#pragma unroll
        for (int c = 0; c < C; ++c) rv[c] ^= rv[c] >> 3;
    }
    uint32_t acc = 0;
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
        for (int c = 0; c < C; ++c) acc += best[r][c] ^ pick[r][c];
    out[tid] = acc;
}

struct Timer {
    hipStream_t st;
    hipEvent_t a = nullptr, b = nullptr;
    bool ok;
    explicit Timer(void* stream) : st(static_cast<hipStream_t>(stream)) {
        ok = hipEventCreate(&a) == hipSuccess && hipEventCreate(&b) == hipSuccess;
    }
    bool start() { return ok && hipEventRecord(a, st) == hipSuccess; }
    bool stop(float* ms) {
        bool good = ok && hipGetLastError() == hipSuccess && hipEventRecord(b, st) == hipSuccess &&
                    hipEventSynchronize(b) == hipSuccess && hipEventElapsedTime(ms, a, b) == hipSuccess;
        return good;
    }
    ~Timer() {
        if (a) (void)hipEventDestroy(a);
        if (b) (void)hipEventDestroy(b);
    }
};

constexpr int kGrid = 256 * 8;  // work-groups of the streaming kernels: eight per compute unit

}  // namespace

extern "C" {

// dst, src: DEVICE buffers of `bytes` (a multiple of 16); reps launches are timed together.
// Returns 0 and the elapsed milliseconds, or -1.
int ckpt_roof_copy(void* dst, const void* src, size_t bytes, int reps, void* stream, float* ms) {
    if (!dst || !src || bytes % 16 || reps < 1 || !ms) return -1;
    Timer t(stream);
    hipLaunchKernelGGL(copy_kernel, dim3(kGrid), dim3(256), 0, t.st, static_cast<uint4*>(dst),
                       static_cast<const uint4*>(src), bytes / 16);  // untimed first pass
    if (!t.start()) return -1;
    for (int r = 0; r < reps; ++r)
        hipLaunchKernelGGL(copy_kernel, dim3(kGrid), dim3(256), 0, t.st, static_cast<uint4*>(dst),
                           static_cast<const uint4*>(src), bytes / 16);
    return t.stop(ms) ? 0 : -1;
}

// src: DEVICE buffer of `bytes`, zero-filled; sink: DEVICE, 4 bytes.  One untimed pass, then reps
// timed passes, one launch each.
int ckpt_roof_read(const void* src, size_t bytes, int reps, void* sink, void* stream, float* ms) {
    if (!src || !sink || bytes % 16 || reps < 1 || !ms) return -1;
    Timer t(stream);
    hipLaunchKernelGGL(read_kernel, dim3(kGrid), dim3(256), 0, t.st, static_cast<const uint4*>(src), bytes / 16,
                       static_cast<uint32_t*>(sink));
    if (!t.start()) return -1;
    for (int r = 0; r < reps; ++r)
        hipLaunchKernelGGL(read_kernel, dim3(kGrid), dim3(256), 0, t.st, static_cast<const uint4*>(src), bytes / 16,
                           static_cast<uint32_t*>(sink));
    return t.stop(ms) ? 0 : -1;
}

// tab: DEVICE int32 table of (tiles * 16 * nq + 2) rows of `pitch` elements (pitch a multiple of
// 64), zero-filled; 0 <= shift < pitch.  *bytes_read <- bytes the timed launch asked for.
int ckpt_roof_read_rows(const void* tab, int pitch, int nq, int tiles, int shift, void* sink, void* stream,
                        float* ms, double* bytes_read) {
    if (!tab || !sink || pitch < 64 || pitch % 64 || nq < 1 || tiles < 1 || shift < 0 || shift >= pitch || !ms ||
        !bytes_read)
        return -1;
    Timer t(stream);
    const dim3 grid((pitch / 64 + 3) / 4, tiles);
    hipLaunchKernelGGL(read_rows_kernel, grid, dim3(256), 0, t.st, static_cast<const uint32_t*>(tab), pitch, nq,
                       shift, static_cast<uint32_t*>(sink));
    if (!t.start()) return -1;
    hipLaunchKernelGGL(read_rows_kernel, grid, dim3(256), 0, t.st, static_cast<const uint32_t*>(tab), pitch, nq,
                       shift, static_cast<uint32_t*>(sink));
    const int steps = (nq + 2) / 3 * 3;
    *bytes_read = double(pitch / 64) * tiles * steps * 16 * 256;
    return t.stop(ms) ? 0 : -1;
}

// kind 0 float64 add + min, 1 32-bit add / compare / two selects, 2 32-bit add + min.
// in: DEVICE 4096 uint32; out: DEVICE blocks * 64 uint32.  *evals <- candidates of the timed launch.
int ckpt_roof_alu(int kind, int blocks, int iters, const void* in, void* out, void* stream, float* ms,
                  double* evals) {
    if (kind < 0 || kind > 2 || blocks < 1 || iters < 1 || !in || !out || !ms || !evals) return -1;
    Timer t(stream);
    auto launch = [&]() {
        const uint32_t* i = static_cast<const uint32_t*>(in);
        uint32_t* o = static_cast<uint32_t*>(out);
        if (kind == 0)
            hipLaunchKernelGGL(alu_f64_kernel, dim3(blocks), dim3(64), 0, t.st, i, o, iters);
        else if (kind == 1)
            hipLaunchKernelGGL(alu_u32_kernel<true>, dim3(blocks), dim3(64), 0, t.st, i, o, iters);
        else
            hipLaunchKernelGGL(alu_u32_kernel<false>, dim3(blocks), dim3(64), 0, t.st, i, o, iters);
    };
    launch();
    if (!t.start()) return -1;
    launch();
    *evals = double(blocks) * 64 * iters * R * C;
    return t.stop(ms) ? 0 : -1;
}

}  // extern "C"
