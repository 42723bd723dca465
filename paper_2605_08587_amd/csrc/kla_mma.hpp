// MFMA fragment ("quad") abstraction used by both chunk kernels.
//
// All matrix products of the chunk path are built from 16x16 output tiles accumulated in fp32.
// A lane l of the wave is addressed as (r = l % 16, g = l / 16).
//
//   accumulator tile  : lane (r, g) holds rows 4g..4g+3 of column r          (floatx4)
//   "quad" of operand : 4 consecutive contraction indices 4g..4g+3 (within a block of 16)
//                       of operand row r (A operand) or operand column r (B operand).
//
// One mma32 contracts over 32 indices = two blocks of 16.  For bf16 it is a single
// v_mfma_f32_16x16x32_bf16 whose 8 per-lane slots are filled with [block0 quad | block1 quad];
// the hardware pairs slot s of A with slot s of B, so any assignment of contraction indices to
// slots is valid as long as A and B use the same one.  For fp32 it is eight v_mfma_f32_16x16x4_f32.
//
// The point of this slot order: an accumulator tile whose ROW index is the next product's
// contraction index is, after conversion, already a B-operand quad for that product.  The state
// S, the right-hand side X and the solve result U therefore go from one product of the chunk
// recurrence to the next without leaving registers.
//
// LDS / workspace operand formats (E = element type, Quad<E> = 4 elements):
//   a "slot" is [block 2p quad | block 2p+1 quad] of one lane; a tile-pair (tile row t, pair p)
//   is 64 consecutive slots.  Slot index = (t * n_pairs + p) * 64 + lane.
//   RQ ("row quads")        : operand stored as rows;   tile row = row / 16,   contraction along the row.
//   TQ ("transposed quads") : operand stored as columns of a row-major matrix M[j][f]:
//                             tile row = f / 16, lane r = f % 16, contraction index = j.
#pragma once
#include "kla_common.hpp"

namespace kla {

typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));

template <typename E> struct QuadT;
template <> struct QuadT<bf16_t> { typedef uint2 type; };
template <> struct QuadT<float> { typedef float4 type; };

template <typename E> struct Slot { typename QuadT<E>::type q0, q1; };

template <typename E> constexpr int slot_bytes() { return 2 * (int)sizeof(typename QuadT<E>::type); }

// T' and P are lower triangular: of the 8 tile-pairs (tile row it, pair jp) of a 64x64 operand only
// the 6 with jp <= it/2 are stored, in this order.
constexpr int kTriPairs = 6;
// Workspace record of one chunk-head: [T' | P | gamma_i | gamma_C/gamma_i | gamma_i/||q_i||] (64 fp32 each; the
// last vector equals gamma_i unless the read-out is normalised)
template <typename E> constexpr int ws_half_bytes() { return kTriPairs * 64 * 8 * (int)sizeof(E); }
template <typename E> constexpr int ws_record_bytes() { return 2 * ws_half_bytes<E>() + 768; }
__host__ __device__ constexpr int tri_pair(int it, int jp) { return it < 2 ? it : 2 * it - 2 + jp; }
// The transposes (upper triangular) keep the 6 tile-pairs with jp >= it/2, in this order.
__host__ __device__ constexpr int triu_pair(int it, int jp) { return it < 2 ? 2 * it + jp : it + 2; }
// Record of one chunk-head for the backward pass:
// [T' | M^T | P^T | gamma_i | gamma_C/gamma_i | beta_i | 1/(|k_i|^2+eps) | 1/||q_i||],
// M = (I + L)^{-1}, T' = M B; three operand halves and five vectors of 64 fp32.  The last vector is 1 unless the
// read-out is normalised (then P^T carries it too).
template <typename E> constexpr int bwd_record_bytes() { return 3 * ws_half_bytes<E>() + 1280; }

// ---- conversions between accumulator tiles and quads -------------------------------------
__device__ __forceinline__ uint2 make_quad(floatx4 x, bf16_t)
{
    return make_uint2(pack_bf16x2(x[0], x[1]), pack_bf16x2(x[2], x[3]));
}
__device__ __forceinline__ float4 make_quad(floatx4 x, float) { return make_float4(x[0], x[1], x[2], x[3]); }
template <typename E> __device__ __forceinline__ typename QuadT<E>::type acc_to_quad(floatx4 x)
{
    return make_quad(x, E());
}

__device__ __forceinline__ floatx4 quad_to_acc(uint2 q)
{
    floatx4 r;
    r[0] = bf16_bits_to_float(q.x & 0xffffu); r[1] = bf16_bits_to_float(q.x >> 16);
    r[2] = bf16_bits_to_float(q.y & 0xffffu); r[3] = bf16_bits_to_float(q.y >> 16);
    return r;
}
__device__ __forceinline__ floatx4 quad_to_acc(float4 q)
{
    floatx4 r; r[0] = q.x; r[1] = q.y; r[2] = q.z; r[3] = q.w; return r;
}

// ---- the product ------------------------------------------------------------------------------
__device__ __forceinline__ void mma32(floatx4& acc, uint2 a0, uint2 a1, uint2 b0, uint2 b1)
{
    const uint4 a = make_uint4(a0.x, a0.y, a1.x, a1.y);
    const uint4 b = make_uint4(b0.x, b0.y, b1.x, b1.y);
    acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, a), __builtin_bit_cast(bf16x8_t, b),
                                                  acc, 0, 0, 0);
}
__device__ __forceinline__ void mma16(floatx4& acc, float4 a, float4 b)
{
    acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a.x, b.x, acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a.y, b.y, acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a.z, b.z, acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a.w, b.w, acc, 0, 0, 0);
}
__device__ __forceinline__ void mma32(floatx4& acc, float4 a0, float4 a1, float4 b0, float4 b1)
{
    mma16(acc, a0, b0);
    mma16(acc, a1, b1);
}
template <typename E>
__device__ __forceinline__ void mma32(floatx4& acc, const Slot<E>& a, typename QuadT<E>::type b0,
                                      typename QuadT<E>::type b1)
{
    mma32(acc, a.q0, a.q1, b0, b1);
}

// ---- slot access --------------------------------------------------------------------------------
// Padded areas (the *_pad functions): slot s sits at position s + s/8, i.e. one empty slot after every eight.
// The stores below write one 8- or 16-byte part of many slots whose indices differ by multiples of 8; unpadded,
// all of those fall into the same LDS banks.  An area of n slots needs pad_slots(n) slots of room.
__host__ __device__ constexpr int pad_slots(int n) { return n + n / 8; }
__device__ __forceinline__ size_t pad_pos(size_t slot) { return slot + (slot >> 3); }

// Read the slot (tile-pair index tp, this lane) from an operand area in LDS.
__device__ __forceinline__ Slot<bf16_t> load_slot(const bf16_t* base, int tp, int lane)
{
    const uint4 x = *reinterpret_cast<const uint4*>(reinterpret_cast<const char*>(base) + ((size_t)tp * 64 + lane) * 16);
    Slot<bf16_t> s; s.q0 = make_uint2(x.x, x.y); s.q1 = make_uint2(x.z, x.w); return s;
}
__device__ __forceinline__ Slot<float> load_slot(const float* base, int tp, int lane)
{
    const float4* p = reinterpret_cast<const float4*>(reinterpret_cast<const char*>(base) + ((size_t)tp * 64 + lane) * 32);
    Slot<float> s; s.q0 = p[0]; s.q1 = p[1]; return s;
}

// Store one 16-byte piece of an operand ROW (row index `row` within the 64-row tile stack,
// `piece` = index of the 16-byte piece inside the row) into an RQ area with n_pairs pairs per row.
__device__ __forceinline__ void store_rq_piece(bf16_t* base, int n_pairs, int row, int piece, uint4 d)
{
    // 8 elements k = 8*piece .. +7 : pair = piece/4, block = (piece%4)/2, quads g0 = 2*(piece%2), g0+1
    const int tp = (row >> 4) * n_pairs + (piece >> 2);
    const int blk = (piece >> 1) & 1, g0 = (piece & 1) * 2, r = row & 15;
    char* p = reinterpret_cast<char*>(base) + ((size_t)tp * 64 + r + 16 * g0) * 16 + blk * 8;
    *reinterpret_cast<uint2*>(p) = make_uint2(d.x, d.y);
    *reinterpret_cast<uint2*>(p + 16 * 16) = make_uint2(d.z, d.w);
}
__device__ __forceinline__ void store_rq_piece(float* base, int n_pairs, int row, int piece, uint4 d)
{
    // 4 elements k = 4*piece .. +3 : pair = piece/8, block = (piece%8)/4, quad g = piece%4
    const int tp = (row >> 4) * n_pairs + (piece >> 3);
    const int blk = (piece >> 2) & 1, g = piece & 3, r = row & 15;
    char* p = reinterpret_cast<char*>(base) + ((size_t)tp * 64 + r + 16 * g) * 32 + blk * 16;
    *reinterpret_cast<uint4*>(p) = d;
}

// Store four consecutive rows j = 4*tq .. 4*tq+3 of a row-major matrix, all at the same 16-byte
// piece, into a TQ area (contraction index = j, n_pairs = rows/32).  `ftile0` is subtracted from
// the feature tile so that a column slice can be stored from tile 0.
__device__ __forceinline__ void store_tq_rows(bf16_t* base, int n_pairs, int tq, int piece, const uint4 (&d)[4],
                                              int ftile0)
{
    const int jp = tq >> 3, blk = (tq >> 2) & 1, g = tq & 3;
    const int ft = (piece >> 1) - ftile0;
    const int r0 = (piece & 1) * 8;
    char* p = reinterpret_cast<char*>(base) + ((size_t)(ft * n_pairs + jp) * 64 + r0 + 16 * g) * 16 + blk * 8;
    const uint32_t w[4][4] = {{d[0].x, d[0].y, d[0].z, d[0].w}, {d[1].x, d[1].y, d[1].z, d[1].w},
                              {d[2].x, d[2].y, d[2].z, d[2].w}, {d[3].x, d[3].y, d[3].z, d[3].w}};
#pragma unroll
    for (int m = 0; m < 4; ++m) {
        // feature 2m (low halves) and 2m+1 (high halves) of the four rows
        const uint2 lo = make_uint2((w[0][m] & 0xffffu) | (w[1][m] << 16), (w[2][m] & 0xffffu) | (w[3][m] << 16));
        const uint2 hi = make_uint2((w[0][m] >> 16) | (w[1][m] & 0xffff0000u), (w[2][m] >> 16) | (w[3][m] & 0xffff0000u));
        *reinterpret_cast<uint2*>(p + (2 * m) * 16) = lo;
        *reinterpret_cast<uint2*>(p + (2 * m + 1) * 16) = hi;
    }
}
__device__ __forceinline__ void store_tq_rows(float* base, int n_pairs, int tq, int piece, const uint4 (&d)[4],
                                              int ftile0)
{
    const int jp = tq >> 3, blk = (tq >> 2) & 1, g = tq & 3;
    const int ft = (piece >> 2) - ftile0;
    const int r0 = (piece & 3) * 4;
    char* p = reinterpret_cast<char*>(base) + ((size_t)(ft * n_pairs + jp) * 64 + r0 + 16 * g) * 32 + blk * 16;
    *reinterpret_cast<uint4*>(p + 0 * 32) = make_uint4(d[0].x, d[1].x, d[2].x, d[3].x);
    *reinterpret_cast<uint4*>(p + 1 * 32) = make_uint4(d[0].y, d[1].y, d[2].y, d[3].y);
    *reinterpret_cast<uint4*>(p + 2 * 32) = make_uint4(d[0].z, d[1].z, d[2].z, d[3].z);
    *reinterpret_cast<uint4*>(p + 3 * 32) = make_uint4(d[0].w, d[1].w, d[2].w, d[3].w);
}

// ---- the same accessors for padded areas -----------------------------------------------------------
__device__ __forceinline__ Slot<bf16_t> load_slot_pad(const bf16_t* base, int tp, int lane)
{
    const uint4 x = *reinterpret_cast<const uint4*>(reinterpret_cast<const char*>(base) + pad_pos((size_t)tp * 64 + lane) * 16);
    Slot<bf16_t> s; s.q0 = make_uint2(x.x, x.y); s.q1 = make_uint2(x.z, x.w); return s;
}
__device__ __forceinline__ Slot<float> load_slot_pad(const float* base, int tp, int lane)
{
    const float4* p = reinterpret_cast<const float4*>(reinterpret_cast<const char*>(base) + pad_pos((size_t)tp * 64 + lane) * 32);
    Slot<float> s; s.q0 = p[0]; s.q1 = p[1]; return s;
}
__device__ __forceinline__ void store_rq_piece_pad(bf16_t* base, int n_pairs, int row, int piece, uint4 d)
{
    const int tp = (row >> 4) * n_pairs + (piece >> 2);
    const int blk = (piece >> 1) & 1, g0 = (piece & 1) * 2, r = row & 15;
    const size_t s0 = (size_t)tp * 64 + r + 16 * g0;
    char* b = reinterpret_cast<char*>(base) + blk * 8;
    *reinterpret_cast<uint2*>(b + pad_pos(s0) * 16) = make_uint2(d.x, d.y);
    *reinterpret_cast<uint2*>(b + pad_pos(s0 + 16) * 16) = make_uint2(d.z, d.w);
}
__device__ __forceinline__ void store_rq_piece_pad(float* base, int n_pairs, int row, int piece, uint4 d)
{
    const int tp = (row >> 4) * n_pairs + (piece >> 3);
    const int blk = (piece >> 2) & 1, g = piece & 3, r = row & 15;
    char* p = reinterpret_cast<char*>(base) + pad_pos((size_t)tp * 64 + r + 16 * g) * 32 + blk * 16;
    *reinterpret_cast<uint4*>(p) = d;
}
__device__ __forceinline__ void store_tq_rows_pad(bf16_t* base, int n_pairs, int tq, int piece, const uint4 (&d)[4],
                                                  int ftile0)
{
    const int jp = tq >> 3, blk = (tq >> 2) & 1, g = tq & 3;
    const int ft = (piece >> 1) - ftile0;
    const int r0 = (piece & 1) * 8;
    const size_t s0 = (size_t)(ft * n_pairs + jp) * 64 + r0 + 16 * g;       // a multiple of 8: the 8 slots are contiguous
    char* p = reinterpret_cast<char*>(base) + pad_pos(s0) * 16 + blk * 8;
    const uint32_t w[4][4] = {{d[0].x, d[0].y, d[0].z, d[0].w}, {d[1].x, d[1].y, d[1].z, d[1].w},
                              {d[2].x, d[2].y, d[2].z, d[2].w}, {d[3].x, d[3].y, d[3].z, d[3].w}};
#pragma unroll
    for (int m = 0; m < 4; ++m) {
        const uint2 lo = make_uint2((w[0][m] & 0xffffu) | (w[1][m] << 16), (w[2][m] & 0xffffu) | (w[3][m] << 16));
        const uint2 hi = make_uint2((w[0][m] >> 16) | (w[1][m] & 0xffff0000u), (w[2][m] >> 16) | (w[3][m] & 0xffff0000u));
        *reinterpret_cast<uint2*>(p + (2 * m) * 16) = lo;
        *reinterpret_cast<uint2*>(p + (2 * m + 1) * 16) = hi;
    }
}
__device__ __forceinline__ void store_tq_rows_pad(float* base, int n_pairs, int tq, int piece, const uint4 (&d)[4],
                                                  int ftile0)
{
    const int jp = tq >> 3, blk = (tq >> 2) & 1, g = tq & 3;
    const int ft = (piece >> 2) - ftile0;
    const int r0 = (piece & 3) * 4;
    const size_t s0 = (size_t)(ft * n_pairs + jp) * 64 + r0 + 16 * g;       // a multiple of 4: within one group of 8
    char* p = reinterpret_cast<char*>(base) + pad_pos(s0) * 32 + blk * 16;
    *reinterpret_cast<uint4*>(p + 0 * 32) = make_uint4(d[0].x, d[1].x, d[2].x, d[3].x);
    *reinterpret_cast<uint4*>(p + 1 * 32) = make_uint4(d[0].y, d[1].y, d[2].y, d[3].y);
    *reinterpret_cast<uint4*>(p + 2 * 32) = make_uint4(d[0].z, d[1].z, d[2].z, d[3].z);
    *reinterpret_cast<uint4*>(p + 3 * 32) = make_uint4(d[0].w, d[1].w, d[2].w, d[3].w);
}

}  // namespace kla
