// Measurement probes (see include/gati_probe.h): a streaming read, a plain copy of known size and a chain of
// dependent near-empty launches.
// No part of the lookup runs through them.
#include <hip/hip_runtime.h>

#include "../../include/gati_probe.h"
#include "common.h"

using namespace gati;

namespace {

constexpr int kLoadsInFlight = 8;

// Grid-stride over 16-byte vectors, kLoadsInFlight independent loads per lane before the first use.
__global__ __launch_bounds__(256) void probe_stream_read_kernel(const u32x4_t* __restrict__ p, long nvec, float* sink) {
    const long tid = (long)blockIdx.x * blockDim.x + threadIdx.x;
    const long stride = (long)gridDim.x * blockDim.x;
    float acc = 0.f;
    long i = tid;
    for (; i + (kLoadsInFlight - 1) * stride < nvec; i += kLoadsInFlight * stride) {
        u32x4_t v[kLoadsInFlight];
#pragma unroll
        for (int u = 0; u < kLoadsInFlight; ++u) v[u] = load_stream(p + i + u * stride);
#pragma unroll
        for (int u = 0; u < kLoadsInFlight; ++u) acc += vec_sum<F32Tag>(v[u]);
    }
    for (; i < nvec; i += stride) acc += vec_sum<F32Tag>(load_stream(p + i));
    if (acc == 123.456f) sink[tid] = acc;      // keeps the loads alive; never true for real data
}

// The other launch shape: one wave per contiguous 8 KB chunk and no loop, so waves arrive and leave all
// the time (the shape of the fastest pooling kernel).  A tail shorter than a chunk is read by the last wave.
__global__ __launch_bounds__(256) void probe_stream_read_chunks_kernel(const u32x4_t* __restrict__ p, long nvec, float* sink) {
    constexpr long kChunk = 64L * kLoadsInFlight;
    const int lane = threadIdx.x & 63;
    const long wave = (long)blockIdx.x * 4 + (threadIdx.x >> 6);
    const long first = wave * kChunk;
    if (first >= nvec) return;
    u32x4_t v[kLoadsInFlight];
#pragma unroll
    for (int u = 0; u < kLoadsInFlight; ++u) {
        const long i = first + u * 64 + lane;
        v[u] = load_stream(p + (i < nvec ? i : nvec - 1));
    }
    float acc = 0.f;
#pragma unroll
    for (int u = 0; u < kLoadsInFlight; ++u) acc += vec_sum<F32Tag>(v[u]);
    if (acc == 123.456f) sink[threadIdx.x] = acc;
}

__global__ __launch_bounds__(256) void probe_copy_kernel(u32x4_t* __restrict__ dst, const u32x4_t* __restrict__ src, long nvec) {
    const long stride = (long)gridDim.x * blockDim.x;
    for (long i = (long)blockIdx.x * blockDim.x + threadIdx.x; i < nvec; i += stride) dst[i] = src[i];
}

// One link of a chain of launches: every lane follows `loads` dependent loads that start at a cell the
// previous link wrote (the values are always 0, so the walk stays inside the two cells), then one lane
// writes the cell for the next link.  What it costs is what any kernel pays that consumes its
// predecessor's output: dispatch, argument fetch, the dependent round trips, the end-of-kernel write-back.
__global__ __launch_bounds__(256) void probe_chain_kernel(int32_t* cell, int loads) {
    const volatile int32_t* p = cell;
    int v = 0;
    for (int d = 0; d < loads; ++d) v = p[v & 1];
    if (blockIdx.x == 0 && threadIdx.x == 0) cell[0] = v & 1;
}

int cu_count() {
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0) {
        (void)hipGetLastError();
        return 256;
    }
    return cus;
}

}  // namespace

extern "C" {

gati_status_t gati_probe_stream_read(const void* buf, size_t bytes, float* sink, int32_t blocks_per_cu, void* stream) {
    if (!buf || !sink || bytes % 16 != 0 || (reinterpret_cast<uintptr_t>(buf) & 15u) != 0) return GATI_ERR_INVALID_ARG;
    if (blocks_per_cu < 0 || blocks_per_cu > 32) return GATI_ERR_INVALID_ARG;
    if (bytes == 0) return GATI_OK;
    if (blocks_per_cu == 0) {
        const long nvec = (long)(bytes / 16), waves = (nvec + 64 * kLoadsInFlight - 1) / (64 * kLoadsInFlight);
        if ((waves + 3) / 4 > 0x7fffffffL) return GATI_ERR_UNSUPPORTED;
        probe_stream_read_chunks_kernel<<<(int)((waves + 3) / 4), 256, 0, (hipStream_t)stream>>>(static_cast<const u32x4_t*>(buf), nvec, sink);
        return hipGetLastError() == hipSuccess ? GATI_OK : GATI_ERR_DEVICE;
    }
    probe_stream_read_kernel<<<cu_count() * blocks_per_cu, 256, 0, (hipStream_t)stream>>>(static_cast<const u32x4_t*>(buf), (long)(bytes / 16), sink);
    return hipGetLastError() == hipSuccess ? GATI_OK : GATI_ERR_DEVICE;
}

gati_status_t gati_probe_copy(void* dst, const void* src, size_t bytes, void* stream) {
    if (!dst || !src || bytes % 16 != 0 || ((reinterpret_cast<uintptr_t>(dst) | reinterpret_cast<uintptr_t>(src)) & 15u) != 0)
        return GATI_ERR_INVALID_ARG;
    if (bytes == 0) return GATI_OK;
    probe_copy_kernel<<<cu_count() * 8, 256, 0, (hipStream_t)stream>>>(static_cast<u32x4_t*>(dst), static_cast<const u32x4_t*>(src), (long)(bytes / 16));
    return hipGetLastError() == hipSuccess ? GATI_OK : GATI_ERR_DEVICE;
}

gati_status_t gati_probe_launch_chain(int32_t* cell, int32_t links, int32_t workgroups, int32_t loads, void* stream) {
    if (!cell || links < 0 || links > 4096 || workgroups < 1 || workgroups > 65536 || loads < 0 || loads > 8)
        return GATI_ERR_INVALID_ARG;
    if (links == 0) return GATI_OK;
    for (int l = 0; l < links; ++l) probe_chain_kernel<<<workgroups, 256, 0, (hipStream_t)stream>>>(cell, loads);
    return hipGetLastError() == hipSuccess ? GATI_OK : GATI_ERR_DEVICE;
}

}  // extern "C"
