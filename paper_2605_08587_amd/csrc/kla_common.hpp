// Shared device helpers for the gfx950 KLA kernels: element types, bf16 conversion,
// wave-level reductions.  gfx950 only (64-wide wavefronts).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace kla {

constexpr int kWave = 64;
constexpr int kChunk = 64;   // tokens per chunk (C in Algorithm 1, right panel)

// Storage type of a bf16 element: raw bits.  Arithmetic is never done in bf16; values are
// widened to fp32 exactly and rounded back with round-to-nearest-even.
struct bf16_t { uint16_t bits; };

__device__ __forceinline__ float to_float(float x) { return x; }
__device__ __forceinline__ float to_float(bf16_t x) { return __uint_as_float(((uint32_t)x.bits) << 16); }
__device__ __forceinline__ float bf16_bits_to_float(uint32_t b) { return __uint_as_float(b << 16); }

__device__ __forceinline__ uint32_t float_to_bf16_bits(float f)
{
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x40u;   // NaN stays NaN
    u += 0x7fffu + ((u >> 16) & 1u);                                    // round to nearest even
    return u >> 16;
}
// two fp32 -> packed bf16 pair, round to nearest even (one v_cvt_pk_bf16_f32 on gfx950)
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi)
{
    typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
    typedef float floatx2_t __attribute__((ext_vector_type(2)));
    const floatx2_t f = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(f, bf16x2_t));
}

template <typename T> __device__ __forceinline__ T from_float(float f);
template <> __device__ __forceinline__ float from_float<float>(float f) { return f; }
template <> __device__ __forceinline__ bf16_t from_float<bf16_t>(float f)
{
    bf16_t r; r.bits = (uint16_t)float_to_bf16_bits(f); return r;
}

// Compile-time loop: f(integral_constant<int, 0>) ... f(integral_constant<int, N-1>).  Used where a
// register array must be indexed by constants from the start (so that it never becomes a stack object).
template <int I> struct IntC { static constexpr int value = I; constexpr operator int() const { return I; } };
template <int N, int I = 0, typename F> __device__ __forceinline__ void static_for(F&& f)
{
    if constexpr (I < N) { f(IntC<I>()); static_for<N, I + 1>(f); }
}

__device__ __forceinline__ float wave_sum(float x)
{
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) x += __shfl_xor(x, off, kWave);
    return x;
}

// Where a per-chunk workgroup works: global chunk index cg (sequences in order, chunks of 64 tokens counted from each
// sequence's own first token) -> first token of the chunk and its length (64, or less for a ragged last chunk).
// cu_seqlens / chunk_off (chunk_off[s] = number of chunks before sequence s) describe a packed batch; both NULL for a
// fixed-length batch of sequences of T tokens (NT chunks each).
struct ChunkPos { long tok0; int clen; };
__device__ __forceinline__ ChunkPos chunk_pos(const int* cu_seqlens, const int* chunk_off, int n_seq, int T, int NT, int cg)
{
    ChunkPos p;
    if (cu_seqlens) {
        int lo = 0, hi = n_seq - 1;                  // last s with chunk_off[s] <= cg
        while (lo < hi) { const int mid = (lo + hi + 1) >> 1; if (chunk_off[mid] <= cg) lo = mid; else hi = mid - 1; }
        const int c = cg - chunk_off[lo];
        const int s0 = cu_seqlens[lo], s1 = cu_seqlens[lo + 1];
        p.tok0 = (long)s0 + 64L * c;
        p.clen = min(64, s1 - (int)p.tok0);
    } else {
        const int n = cg / NT, c = cg % NT;
        p.tok0 = (long)n * T + 64L * c;
        p.clen = min(64, T - 64 * c);
    }
    return p;
}

// Kaczmarz coefficient of eq. (3); a zero denominator (zero key, eps = 0) gives beta = 0
// because the write beta k e^T is then zero for every finite beta.
__device__ __forceinline__ float kaczmarz_beta(float eta, float knorm2, float eps)
{
    const float den = knorm2 + eps;
    return den == 0.0f ? 0.0f : eta / den;
}

// The same with the hardware reciprocal (1 ulp) instead of an IEEE division: for results that are rounded to
// bf16 right afterwards.
__device__ __forceinline__ float kaczmarz_beta_fast(float eta, float knorm2, float eps)
{
    const float den = knorm2 + eps;
    return den == 0.0f ? 0.0f : eta * __builtin_amdgcn_rcpf(den);
}

}  // namespace kla
