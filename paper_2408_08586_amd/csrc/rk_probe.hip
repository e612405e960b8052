// Measurement helpers, no part of the method: what the memory system gives a
// kernel that only reads, or only writes, a buffer of the size the evaluation
// kernels move.  The benchmark runs them beside k_eval and k_best_plan so that
// a profile shows the three under the same counters.
#include "rk_internal.h"

namespace {

typedef float v4f __attribute__((ext_vector_type(4)));

constexpr int PROBE_THREADS = 256;
constexpr int PROBE_UNROLL = 4;
constexpr uint64_t PROBE_TILE = (uint64_t)PROBE_THREADS * PROBE_UNROLL * 4;     // 16-byte elements per workgroup

// every workgroup streams one contiguous tile with 16-byte streaming loads, four in flight per lane, and compares the
// sum of what it read with a value it practically never has (so the loads cannot be dropped; *out is only touched in
// that case).  TAG only gives the kernel two names, so that a profile tells the read that follows a fill of the same
// buffer (0) from the read that follows another read (1).
template <int TAG>
__global__ __launch_bounds__(PROBE_THREADS) void k_probe_read(const v4f *__restrict__ buf, uint64_t n_vec,
                                                              float *__restrict__ out) {
    const uint64_t base = (uint64_t)blockIdx.x * PROBE_TILE;
    float acc = 0.f;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        v4f v[PROBE_UNROLL];
#pragma unroll
        for (int u = 0; u < PROBE_UNROLL; ++u) {
            const uint64_t i = base + (uint64_t)(r * PROBE_UNROLL + u) * PROBE_THREADS + threadIdx.x;
            v[u] = __builtin_nontemporal_load(buf + (i < n_vec ? i : n_vec - 1));
        }
#pragma unroll
        for (int u = 0; u < PROBE_UNROLL; ++u) acc += (v[u].x + v[u].y) + (v[u].z + v[u].w);
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) acc += __shfl_xor(acc, off, 64);
    if ((threadIdx.x & 63) == 0 && acc == 12345.678f) atomicAdd(out, acc);
}

// the same read by a fixed number of workgroups that stride through the buffer together, 16 KiB per workgroup and
// round: at any moment the loads in flight cover one compact stretch of the buffer
__global__ __launch_bounds__(PROBE_THREADS) void k_probe_read_strided(const v4f *__restrict__ buf, uint64_t n_vec,
                                                                      float *__restrict__ out) {
    const uint64_t step = (uint64_t)gridDim.x * PROBE_THREADS * PROBE_UNROLL;
    float acc = 0.f;
    for (uint64_t base = (uint64_t)blockIdx.x * PROBE_THREADS * PROBE_UNROLL; base < n_vec; base += step) {
        v4f v[PROBE_UNROLL];
#pragma unroll
        for (int u = 0; u < PROBE_UNROLL; ++u) {
            const uint64_t i = base + (uint64_t)u * PROBE_THREADS + threadIdx.x;
            v[u] = __builtin_nontemporal_load(buf + (i < n_vec ? i : n_vec - 1));
        }
#pragma unroll
        for (int u = 0; u < PROBE_UNROLL; ++u) acc += (v[u].x + v[u].y) + (v[u].z + v[u].w);
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) acc += __shfl_xor(acc, off, 64);
    if ((threadIdx.x & 63) == 0 && acc == 12345.678f) atomicAdd(out, acc);
}

// TAG as for k_probe_read: 0 = the fill that follows a read, 1 = the fill that follows another fill
template <int TAG>
__global__ __launch_bounds__(PROBE_THREADS) void k_probe_fill(v4f *__restrict__ buf, uint64_t n_vec, float value) {
    const uint64_t base = (uint64_t)blockIdx.x * PROBE_TILE;
    const v4f v = {value, value, value, value};
#pragma unroll
    for (int r = 0; r < 4 * PROBE_UNROLL; ++r) {
        const uint64_t i = base + (uint64_t)r * PROBE_THREADS + threadIdx.x;
        if (i < n_vec) buf[i] = v;
    }
}

}  // namespace

extern "C" int32_t rk_probe_stream(rk_ctx *ctx, float *buf, uint64_t n_floats, int32_t mode, float value, float *out) {
    if (!ctx) return RK_ERR_INVALID_ARG;
    if (!buf || n_floats < 4 || ((uintptr_t)buf & 15u) || ((mode == 0 || mode == 2 || mode == 3) && !out) || mode < 0 || mode > 4)
        return rk_fail(ctx, RK_ERR_INVALID_ARG, "rk_probe_stream: bad argument");
    RK_HIP(ctx, hipSetDevice(ctx->device));
    const uint64_t n_vec = n_floats / 4;
    const uint64_t blocks = (n_vec + PROBE_TILE - 1) / PROBE_TILE;
    if (blocks > 0x7FFFFFFFull) return rk_fail(ctx, RK_ERR_UNSUPPORTED, "buffer too large");
    if (mode == 0)
        k_probe_read<0><<<(uint32_t)blocks, PROBE_THREADS, 0, ctx->stream>>>(reinterpret_cast<const v4f *>(buf), n_vec, out);
    else if (mode == 3)
        k_probe_read<1><<<(uint32_t)blocks, PROBE_THREADS, 0, ctx->stream>>>(reinterpret_cast<const v4f *>(buf), n_vec, out);
    else if (mode == 2)
        k_probe_read_strided<<<4096, PROBE_THREADS, 0, ctx->stream>>>(reinterpret_cast<const v4f *>(buf), n_vec, out);
    else if (mode == 4)
        k_probe_fill<1><<<(uint32_t)blocks, PROBE_THREADS, 0, ctx->stream>>>(reinterpret_cast<v4f *>(buf), n_vec, value);
    else
        k_probe_fill<0><<<(uint32_t)blocks, PROBE_THREADS, 0, ctx->stream>>>(reinterpret_cast<v4f *>(buf), n_vec, value);
    RK_CHECK_LAUNCH(ctx, "k_probe");
    return RK_OK;
}
