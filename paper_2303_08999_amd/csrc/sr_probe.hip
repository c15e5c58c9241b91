// Streaming probes (see include/sr_probe.h): the read stream and the read+write
// mix of the assembly kernel with nothing else in the way.  Measurement only.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/sr_dict.h"
#include "../../include/sr_probe.h"

namespace {

typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned u32x2 __attribute__((ext_vector_type(2)));

constexpr int UNROLL = 8;

__global__ __launch_bounds__(256) void k_probe_read(const u32x4* __restrict__ p, size_t n, unsigned* sink) {
    unsigned acc = 0;
    size_t i = (size_t)blockIdx.x * 256 * UNROLL + threadIdx.x;
    const size_t step = (size_t)gridDim.x * 256 * UNROLL;
    for (; i + 256 * (UNROLL - 1) < n; i += step) {
        u32x4 v[UNROLL];
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) v[u] = __builtin_nontemporal_load(p + i + u * 256);
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) acc ^= v[u][0] ^ v[u][1] ^ v[u][2] ^ v[u][3];
    }
    for (int u = 0; u < UNROLL && i + (size_t)u * 256 < n; ++u) {     // ragged end of the last sweep
        const u32x4 v = __builtin_nontemporal_load(p + i + u * 256);
        acc ^= v[0] ^ v[1] ^ v[2] ^ v[3];
    }
    if (acc == 0x9e3779b9u) *sink = acc;
}

// One wavefront per run of 128 pixels; lane (j, hf) reads pixels 4j..4j+3 of planes
// 2i + hf and writes pixels 4j + 2hf, +1 of every output plane.  The next run's
// loads are issued before this run's stores.
template <int L>
__global__ __launch_bounds__(256) void k_probe_mix(const char* __restrict__ p, size_t plane_b, int runs,
                                                   float* __restrict__ out, size_t pixels, int channels) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, hf = lane >> 5, j = lane & 31;
    const int stride = gridDim.x * 4;
    int u = blockIdx.x * 4 + wave;
    if (u >= runs) return;
    u32x2 v[L / 2];
    {
        const size_t off = (size_t)u * 256 + (size_t)j * 8;
#pragma unroll
        for (int i = 0; i < L / 2; ++i)
            v[i] = __builtin_nontemporal_load((const u32x2*)(p + (size_t)(2 * i + hf) * plane_b + off));
    }
    for (; u < runs; u += stride) {
        unsigned acc = 0;
#pragma unroll
        for (int i = 0; i < L / 2; ++i) acc ^= v[i][0] ^ v[i][1];
        acc ^= __shfl_xor(acc, 32, 64);
        const float f = (float)(acc & 0xffu);
        const int un = u + stride;
        if (un < runs) {
            const size_t off = (size_t)un * 256 + (size_t)j * 8;
#pragma unroll
            for (int i = 0; i < L / 2; ++i)
                v[i] = __builtin_nontemporal_load((const u32x2*)(p + (size_t)(2 * i + hf) * plane_b + off));
        }
        const size_t o = (size_t)u * 128 + 4 * j + 2 * hf;
        for (int c = 0; c < channels; ++c) *(float2*)(out + (size_t)c * pixels + o) = make_float2(f, f + (float)c);
    }
}

}  // namespace

extern "C" __attribute__((visibility("default")))
int sr_probe_read(const void* src, size_t bytes, void* sink, void* stream) {
    if (!src || !sink) return SR_ERR_NULL;
    if (bytes % 16 != 0) return SR_ERR_UNSUPPORTED;
    if ((uintptr_t)src % 16 != 0 || (uintptr_t)sink % 4 != 0) return SR_ERR_ALIGN;
    if (bytes == 0) return SR_OK;
    hipLaunchKernelGGL(k_probe_read, dim3(4096), dim3(256), 0, (hipStream_t)stream,
                       (const u32x4*)src, bytes / 16, (unsigned*)sink);
    return hipGetLastError() == hipSuccess ? SR_OK : SR_ERR_LAUNCH;
}

extern "C" __attribute__((visibility("default")))
int sr_probe_mix(const void* coeff, int planes, size_t pixels, void* out, int channels, void* stream) {
    if (!coeff || !out) return SR_ERR_NULL;
    if ((planes != 72 && planes != 128) || channels < 1 || channels > 4 || pixels % 128 != 0 ||
        pixels / 128 > 0x7fffffffull)
        return SR_ERR_UNSUPPORTED;
    if ((uintptr_t)coeff % 16 != 0 || (uintptr_t)out % 16 != 0) return SR_ERR_ALIGN;
    if (pixels == 0) return SR_OK;
    const int runs = (int)(pixels / 128);
    const int blocks = runs / 4 < 512 ? (runs + 3) / 4 : 512;
    if (planes == 72)
        hipLaunchKernelGGL(k_probe_mix<72>, dim3(blocks), dim3(256), 0, (hipStream_t)stream,
                           (const char*)coeff, pixels * 2, runs, (float*)out, pixels, channels);
    else
        hipLaunchKernelGGL(k_probe_mix<128>, dim3(blocks), dim3(256), 0, (hipStream_t)stream,
                           (const char*)coeff, pixels * 2, runs, (float*)out, pixels, channels);
    return hipGetLastError() == hipSuccess ? SR_OK : SR_ERR_LAUNCH;
}
