// Measurement probes behind kla_debug_peak_probe: what this GPU delivers for the two access patterns the rooflines
// of the hot path are quoted against, with none of the method's arithmetic in the way.
//   kind 0  in-place streaming: every 16 bytes of a buffer are read once and written once (x <- 2 x on floats), the
//           traffic pattern of the decode step (state read, state written) without its two column sums
//   kind 1  read-only streaming: the buffer is read once, a checksum per workgroup is written
//   kind 2  dense bf16 matrix pipe: every wave issues v_mfma_f32_16x16x32_bf16 back to back on eight independent
//           accumulators, operands in registers, nothing from memory
#include "kla_bf16_ops.hpp"
#include "kla_common.hpp"
#include "kla_kernels.hpp"
#include "kla_mma.hpp"

namespace kla {

namespace {

typedef float f4v __attribute__((ext_vector_type(4)));

// one workgroup per 64 KiB, 16 float4 per lane, all loads first: the decode kernel's own access order
template <bool NT>
__global__ __launch_bounds__(256) void probe_inplace_kernel(f4v* __restrict__ buf)
{
    f4v* p = buf + (size_t)blockIdx.x * 4096 + threadIdx.x;
    f4v x[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) x[i] = NT ? __builtin_nontemporal_load(p + 256 * i) : p[256 * i];
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const f4v y = x[i] * 2.0f;
        if (NT) __builtin_nontemporal_store(y, p + 256 * i); else p[256 * i] = y;
    }
}

__global__ __launch_bounds__(256) void probe_read_kernel(const f4v* __restrict__ buf, float* __restrict__ sums)
{
    const f4v* p = buf + (size_t)blockIdx.x * 4096 + threadIdx.x;
    f4v acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int i = 0; i < 16; ++i) acc += __builtin_nontemporal_load(p + 256 * i);
    float s = wave_sum(acc[0] + acc[1] + acc[2] + acc[3]);
    if ((threadIdx.x & 63) == 0) sums[(size_t)blockIdx.x * 4 + (threadIdx.x >> 6)] = s;
}

__global__ __launch_bounds__(256) void probe_mfma_kernel(float* __restrict__ out, int iters)
{
    const uint32_t seed = 0x3f803f80u + threadIdx.x;     // finite bf16 pairs, different per lane
    const u32x4 a = {seed, seed ^ 0x00010001u, seed ^ 0x00020002u, seed ^ 0x00030003u};
    const u32x2 b0 = {seed ^ 0x00040004u, seed}, b1 = {seed ^ 0x00050005u, seed};
    floatx4 acc[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) acc[j] = floatx4{0.f, 0.f, 0.f, 0.f};
    for (int i = 0; i < iters; ++i) {
#pragma unroll
        for (int j = 0; j < 8; ++j) mma_bf16(acc[j], a, b0, b1);
    }
    floatx4 s = acc[0];
#pragma unroll
    for (int j = 1; j < 8; ++j) s += acc[j];
    out[(size_t)blockIdx.x * 256 + threadIdx.x] = s[0] + s[1] + s[2] + s[3];
}

}  // namespace

// kind 0 / 1: `bytes` a positive multiple of 65536; kind 1 also writes bytes / 16384 floats to aux.  kind 2: `bytes`
// = number of workgroups of four waves, `iters` rounds of eight products each, aux holds 256 floats per workgroup.
hipError_t launch_probe(int kind, void* buf, void* aux, size_t bytes, int iters, hipStream_t st)
{
    if (kind == 2) {
        hipLaunchKernelGGL(probe_mfma_kernel, dim3((unsigned)bytes), dim3(256), 0, st, static_cast<float*>(aux), iters);
        return hipGetLastError();
    }
    const dim3 grid((unsigned)(bytes / 65536));
    if (kind == 0) {
        if (iters) hipLaunchKernelGGL(probe_inplace_kernel<true>, grid, dim3(256), 0, st, static_cast<f4v*>(buf));
        else       hipLaunchKernelGGL(probe_inplace_kernel<false>, grid, dim3(256), 0, st, static_cast<f4v*>(buf));
    } else {
        hipLaunchKernelGGL(probe_read_kernel, grid, dim3(256), 0, st, static_cast<const f4v*>(buf), static_cast<float*>(aux));
    }
    return hipGetLastError();
}

}  // namespace kla
