// Measurement probes behind kla_debug_peak_probe: what this GPU delivers for the two access patterns the rooflines
// of the hot path are quoted against, with none of the method's arithmetic in the way.
//   kind 0  in-place streaming: every 16 bytes of a buffer are read once and written once (x <- 2 x on floats), the
//           traffic pattern of the decode step (state read, state written) without its two column sums
//   kind 1  read-only streaming: the buffer is read once, a checksum per workgroup is written
//   kind 2  dense bf16 matrix pipe: every wave issues v_mfma_f32_16x16x32_bf16 back to back on eight independent
//           accumulators, operands in registers, nothing from memory
//   kind 3  the copy wave of the chunk kernels alone: one workgroup per CU, a wave that brings a given number of 1 KiB
//           LDS-DMA copies per step (rows of 256 bytes, 2 KiB apart, the K rows of one head of config 2; the four
//           workgroups that share a head in the scan kernels share the rows here) through a ring one or two steps deep,
//           and a barrier per step
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

// 64 steps; in every step wave 0 issues NI copies of 1 KiB (four 256-byte rows each) and waits until all but the last
// `depth - 1` steps' copies have landed; the other waves only keep the barrier company.
template <int NI, int DEPTH>
__global__ __launch_bounds__(256) void probe_ring_copy_kernel(const char* __restrict__ src, size_t unit_stride)
{
    static_assert(NI >= 1 && NI <= 63 && (DEPTH == 1 || DEPTH == 2), "6-bit counter; LDS holds two steps");
    __shared__ __attribute__((aligned(1024))) char lds[2 * 64 * 1024];
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    constexpr int kSteps = 64, kStride = 2048;
    const int unit = ((blockIdx.x >> 3) / 4) * 8 + (blockIdx.x & 7);                 // four sharers on one XCD
    const char* base = src + (size_t)(unit / 8) * unit_stride + (unit % 8) * 256;     // eight heads interleaved
    const int lo = (lane >> 4) * kStride + (lane & 15) * 16;
    for (int s = 0; s < kSteps; ++s) {
        if (wave == 0) {
            const char* p = base + (size_t)s * NI * 4 * kStride;
            char* l = lds + (s & 1) * 64 * 1024;
#pragma unroll
            for (int i = 0; i < NI; ++i) dma16(p + (size_t)i * 4 * kStride, lo, l + i * 1024);
            if (DEPTH == 2 && s + 1 < kSteps) wait_vmcnt<(DEPTH == 2 ? NI : 0)>(); else wait_vmcnt<0>();
        }
        __syncthreads();
    }
}

}  // namespace

// kind 0 / 1: `bytes` a positive multiple of 65536; kind 1 also writes bytes / 16384 floats to aux.  kind 2: `bytes`
// = number of workgroups of four waves, `iters` rounds of eight products each, aux holds 256 floats per workgroup.
// kind 3: `bytes` = size of buf, iters = copies per step (16, 32, 48 or 60) + 256 (ring depth - 1).
hipError_t launch_probe(int kind, void* buf, void* aux, size_t bytes, int iters, hipStream_t st)
{
    if (kind == 3) {
        // iters = copies per step + 256 * (ring depth - 1); `bytes` must cover 8 groups of 64 steps x copies x 8 KiB
        const int ni = iters & 255, depth = 1 + (iters >> 8);
        const size_t unit_stride = (size_t)64 * ni * 4 * 2048;
        if (depth < 1 || depth > 2 || bytes < 8 * unit_stride) return hipErrorInvalidValue;
        const char* b = static_cast<const char*>(buf);
#define KLA_RING(NI) \
        case NI: if (depth == 1) hipLaunchKernelGGL((probe_ring_copy_kernel<NI, 1>), dim3(256), dim3(256), 0, st, b, unit_stride); \
                 else            hipLaunchKernelGGL((probe_ring_copy_kernel<NI, 2>), dim3(256), dim3(256), 0, st, b, unit_stride); break;
        switch (ni) {
            KLA_RING(16) KLA_RING(32) KLA_RING(48) KLA_RING(60)
            default: return hipErrorInvalidValue;
        }
#undef KLA_RING
        return hipGetLastError();
    }
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
