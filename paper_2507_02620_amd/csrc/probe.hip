// Achievable-peak probes (measurement aids, not part of the method): what one launch can reach on this machine for a
// pure one-pass HBM read and for a register-resident bf16 MFMA loop.  bench.py reports kernel figures against the
// datasheet peaks and against these.
#include <hip/hip_runtime.h>

#include "../../include/flowspec.h"
#include "common.hpp"

extern thread_local int g_last_hip;

namespace {

// each wave streams a contiguous chunk of per_wave_kib KiB, 16 bytes per lane and load, 8 loads in flight, non-temporal
// (the access pattern of the projection kernels' weight stream)
__global__ void __launch_bounds__(512) probe_stream_kernel(const f32x4* __restrict__ src, int per_wave_kib, float* sink) {
    constexpr int DEPTH = 8;
    const int lane = threadIdx.x & 63;
    const size_t wave = (size_t)blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
    const f32x4* p = src + wave * (size_t)per_wave_kib * 64 + lane;
    f32x4 acc = {0.f, 0.f, 0.f, 0.f}, buf[DEPTH];
    const int n = per_wave_kib;
#pragma unroll
    for (int s = 0; s < DEPTH; ++s) buf[s] = __builtin_nontemporal_load(p + (size_t)min(s, n - 1) * 64);
    for (int i = 0; i < n; i += DEPTH) {
#pragma unroll
        for (int s = 0; s < DEPTH; ++s) {
            if (i + s < n) acc += buf[s];
            buf[s] = __builtin_nontemporal_load(p + (size_t)min(i + s + DEPTH, n - 1) * 64);
            __builtin_amdgcn_sched_barrier(0);
        }
    }
    if (acc[0] + acc[1] + acc[2] + acc[3] == 12345.678f) sink[0] = acc[0];  // keeps the loads alive; the sink is the caller's own buffer
}

// 16 independent 16x16x32 bf16 MFMAs per iteration, operands and accumulators in registers
__global__ void __launch_bounds__(256) probe_mfma_kernel(int iters, float* sink) {
    bf16x8 a, b;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        a[e] = (bf16_t)(float)((threadIdx.x + e) & 3);
        b[e] = (bf16_t)(float)((threadIdx.x * 3 + e) & 1);
    }
    f32x4 acc[16];
#pragma unroll
    for (int j = 0; j < 16; ++j) acc[j] = f32x4{0.f, 0.f, 0.f, 0.f};
    for (int i = 0; i < iters; ++i) {
#pragma unroll
        for (int j = 0; j < 16; ++j) acc[j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, acc[j], 0, 0, 0);
    }
    f32x4 t = acc[0];
#pragma unroll
    for (int j = 1; j < 16; ++j) t += acc[j];
    if (t[0] + t[1] + t[2] + t[3] == -1.f) sink[0] = t[0];
}

// Fill-rate probe: every workgroup streams `iters` x (waves x 4 KiB) from its region of `region_kib` KiB (re-read cyclically, so
// a small region stays in the caches) with 16-byte-per-lane loads, three iterations in flight; TO_LDS: direct-to-LDS loads into
// an LDS landing area, else loads into registers.  Workgroups `share` slots apart on one XCD read the same region.
template <bool TO_LDS>
__global__ void __launch_bounds__(1024) probe_fill_kernel(const unsigned char* __restrict__ src, int region_kib, int iters, int share, float* sink) {
    __shared__ __align__(1024) unsigned char sb[2][8 * 4096];  // landing area only: nothing reads it, waves 8.. share the slots of 0..
    const int lane = threadIdx.x & 63, w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), nw = blockDim.x >> 6;
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
    const size_t region = (size_t)((slot / share) * 8 + xcd) * region_kib * 1024;
    const unsigned char* base = src + region + (size_t)lane * 16;
    const unsigned per_iter = (unsigned)nw * 4096u, wrap = (unsigned)region_kib * 1024u;
    unsigned off = (unsigned)w * 4096u;
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
    for (int it = 0; it < iters; ++it) {
        if (TO_LDS) {
#pragma unroll
            for (int i = 0; i < 4; ++i)
                __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(base + off + i * 1024),
                                                 (__attribute__((address_space(3))) void*)(sb[it & 1] + (w & 7) * 4096 + i * 1024), 16, 0, 0);
            __builtin_amdgcn_s_waitcnt(0x0F70 | 8);  // vmcnt(8): two iterations stay in flight
        } else {
            f32x4 v[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) v[i] = *(const f32x4*)(base + off + i * 1024);
            __builtin_amdgcn_sched_barrier(0);
            acc += v[0] + v[1] + v[2] + v[3];
        }
        off += per_iter;
        if (off >= wrap) off -= wrap;
    }
    __builtin_amdgcn_s_waitcnt(0x0F70);
    if (TO_LDS) acc[0] = *(const float*)(sb[0] + threadIdx.x * 4);
    if (acc[0] + acc[1] + acc[2] + acc[3] == 12345.678f) sink[0] = acc[0];
}

int timed(hipStream_t s, int launches, double* ms_per_launch, void (*launch)(hipStream_t, int, void*), void* ctx) {
    hipEvent_t e0, e1;
    if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) return FS_EHIP;
    for (int i = 0; i < 2; ++i) launch(s, i, ctx);  // warm-up
    hipError_t e = hipEventRecord(e0, s);
    for (int i = 0; i < launches; ++i) launch(s, i + 2, ctx);
    if (e == hipSuccess) e = hipEventRecord(e1, s);
    if (e == hipSuccess) e = hipEventSynchronize(e1);
    float ms = 0.f;
    if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
    if (e == hipSuccess) e = hipGetLastError();
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (e != hipSuccess) {
        g_last_hip = (int)e;
        return FS_EHIP;
    }
    *ms_per_launch = (double)ms / launches;
    return FS_OK;
}

struct StreamCtx {
    const unsigned char* buf;
    size_t buf_bytes, bytes;
    float* sink;
};
void launch_stream(hipStream_t s, int i, void* c) {
    const StreamCtx* x = (const StreamCtx*)c;
    const size_t slots = x->buf_bytes / x->bytes;  // rotate so that a launch does not find its data in a cache
    const unsigned char* p = x->buf + (size_t)(i % slots) * x->bytes;
    const int per_wave_kib = 32, waves_per_wg = 8;
    const int grid = (int)(x->bytes / ((size_t)per_wave_kib * 1024 * waves_per_wg));
    hipLaunchKernelGGL(probe_stream_kernel, dim3(grid), dim3(waves_per_wg * 64), 0, s, (const f32x4*)p, per_wave_kib, x->sink);
}

struct MfmaCtx {
    int iters, grid;
    float* sink;
};
void launch_mfma(hipStream_t s, int, void* c) {
    const MfmaCtx* x = (const MfmaCtx*)c;
    hipLaunchKernelGGL(probe_mfma_kernel, dim3(x->grid), dim3(256), 0, s, x->iters, x->sink);
}

struct FillCtx {
    const unsigned char* buf;
    int grid, waves, region_kib, iters, share, to_lds;
    float* sink;
};
void launch_fill(hipStream_t s, int, void* c) {
    const FillCtx* x = (const FillCtx*)c;
    if (x->to_lds)
        hipLaunchKernelGGL(probe_fill_kernel<true>, dim3(x->grid), dim3(x->waves * 64), 0, s, x->buf, x->region_kib, x->iters, x->share, x->sink);
    else
        hipLaunchKernelGGL(probe_fill_kernel<false>, dim3(x->grid), dim3(x->waves * 64), 0, s, x->buf, x->region_kib, x->iters, x->share, x->sink);
}

}  // namespace

extern "C" {

int fs_probe_fill(const void* buf, size_t buf_bytes, int grid, int waves, int region_kib, int iters, int share, int to_lds, int launches,
                  void* stream, double* gb_per_s) {
    if (!buf || !gb_per_s || launches < 1 || grid < 1 || waves < 1 || waves > 16 || iters < 1 || share < 1 || ((uintptr_t)buf & 15)) return FS_EINVAL;
    if (region_kib < waves * 4 || region_kib % (waves * 4)) return FS_EINVAL;  // whole iterations per lap
    const size_t regions = (size_t)((grid / 8 + share - 1) / share + 1) * 8;
    if (regions * region_kib * 1024 + 64 > buf_bytes) return FS_EINVAL;
    FillCtx c{(const unsigned char*)buf, grid, waves, region_kib, iters, share, to_lds, (float*)((unsigned char*)buf + buf_bytes - 64)};
    double ms;
    int rc = timed((hipStream_t)stream, launches, &ms, launch_fill, &c);
    if (rc == FS_OK) *gb_per_s = (double)grid * iters * waves * 4096.0 / (ms * 1e-3) / 1e9;
    return rc;
}

int fs_probe_stream_read(const void* buf, size_t buf_bytes, size_t bytes_per_launch, int launches, void* stream, double* gb_per_s) {
    if (!buf || !gb_per_s || launches < 1 || bytes_per_launch < (1u << 20) || bytes_per_launch % (256 * 1024) || buf_bytes < bytes_per_launch + 64 ||
        ((uintptr_t)buf & 15))
        return FS_EINVAL;
    // the last 64 bytes of the buffer serve as the (never written) sink
    StreamCtx c{(const unsigned char*)buf, buf_bytes - 64, bytes_per_launch, (float*)((unsigned char*)buf + buf_bytes - 64)};
    double ms;
    int rc = timed((hipStream_t)stream, launches, &ms, launch_stream, &c);
    if (rc == FS_OK) *gb_per_s = (double)bytes_per_launch / (ms * 1e-3) / 1e9;
    return rc;
}

int fs_probe_mfma_bf16(void* scratch, int launches, void* stream, double* tflop_per_s) {
    if (!scratch || !tflop_per_s || launches < 1) return FS_EINVAL;
    MfmaCtx c{4096, 256 * 8, (float*)scratch};  // 8 workgroups of 4 waves per compute unit
    double ms;
    int rc = timed((hipStream_t)stream, launches, &ms, launch_mfma, &c);
    if (rc == FS_OK) *tflop_per_s = (double)c.grid * 4 * c.iters * 16 * (2.0 * 16 * 16 * 32) / (ms * 1e-3) / 1e12;
    return rc;
}

}  // extern "C"
