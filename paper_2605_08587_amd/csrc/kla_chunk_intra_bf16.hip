// bf16 intra-chunk stage: same objects as kla_chunk_intra.hip (beta of eq. (3), g = log gamma,
// T' = (I + B(A^- o KK^T))^{-1} B of eq. (6), P = A o QK^T of eq. (7), and the decay factors the scan
// stage multiplies with), laid out for gfx950:
//
//   * K and Q go global -> LDS directly (global_load_lds_dwordx4) as token-major rows with the
//     16-byte columns XOR-swizzled by the row; every MFMA operand slot is then one conflict-free
//     128-bit LDS read of 8 consecutive features (A and B operands of both Gram products are rows of
//     K or Q, so any slot order common to both is valid).
//   * Each wave runs its five 16x16 tiles with five independent accumulators, operands one
//     contraction step ahead.
//   * (I+L)^{-1} is built IN PLACE in one fp32 64x64 LDS matrix (diagonal 16x16 blocks by forward
//     substitution with the rows read one ahead, off-diagonal blocks by two levels of fp32 MFMA block
//     products), and the fp32 image of P overlays the dead K/Q tiles: 50 KB of LDS, three workgroups
//     per CU, so that one workgroup's global-memory latency hides behind the others' arithmetic.
//   * Rows beyond a short last chunk re-read its last row; beta = 0 there zeroes their rows and columns
//     of T', and their rows of P are masked.
#include "kla_bf16_ops.hpp"
#include "kla_common.hpp"
#include "kla_kernels.hpp"
#include "kla_mma.hpp"

namespace kla {

namespace {

constexpr int kLd = 68;   // row stride (floats) of the fp32 64x64 matrices in LDS

// The 20 lower-triangular 16x16 tiles of K K^T (q = 0) and Q K^T (q = 1), five per wave, grouped so that a
// wave's tiles share operands: the A slots of tile (ti, tj) are rows 16 ti.. of K (or Q), the B slots rows
// 16 tj.. of K, and a K row block is the same registers in either role.  Waves 0..3 need 5, 4, 5, 4 distinct
// row blocks per contraction step instead of 10.
struct GramJob { int q, ti, tj; };
constexpr GramJob kJobs[4][5] = {
    {{1, 3, 0}, {1, 3, 1}, {1, 3, 2}, {1, 3, 3}, {0, 3, 3}},
    {{0, 3, 0}, {0, 3, 1}, {0, 3, 2}, {0, 2, 0}, {0, 2, 1}},
    {{1, 2, 0}, {1, 2, 1}, {1, 2, 2}, {1, 1, 0}, {1, 1, 1}},
    {{0, 0, 0}, {0, 1, 0}, {0, 1, 1}, {0, 2, 2}, {1, 0, 0}}};
constexpr bool gram_needs(int w, int blk)            // blk 0..3: K row block, 4..7: Q row block
{
    for (int j = 0; j < 5; ++j)
        if (kJobs[w][j].q * 4 + kJobs[w][j].ti == blk || kJobs[w][j].tj == blk) return true;
    return false;
}

__device__ __forceinline__ floatx4 ldf4(const float* p) { return *reinterpret_cast<const floatx4*>(p); }
// fp32 MFMA 16x16x16 = four 16x16x4 steps; quads hold contraction indices 4g..4g+3
__device__ __forceinline__ void mma16f(floatx4& acc, floatx4 a, floatx4 b)
{
    acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a[0], b[0], acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a[1], b[1], acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a[2], b[2], acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a[3], b[3], acc, 0, 0, 0);
}
// A-operand quad of a row-major fp32 matrix: columns 4g..4g+3 of row r
__device__ __forceinline__ floatx4 aq(const float* m, int row0, int col0, int r, int g)
{
    return ldf4(m + (row0 + r) * kLd + col0 + 4 * g);
}
// B-operand quad: rows 4g..4g+3 of column r
__device__ __forceinline__ floatx4 bq(const float* m, int row0, int col0, int r, int g)
{
    const float* p = m + (row0 + 4 * g) * kLd + col0 + r;
    floatx4 x; x[0] = p[0]; x[1] = p[kLd]; x[2] = p[2 * kLd]; x[3] = p[3 * kLd]; return x;
}

// The transpose of a lower-triangular fp32 64x64 matrix (row stride kLd; its strictly-upper tiles hold garbage) as
// the 6 upper-triangular tile-pairs of bf16 operand slots: pair ctp = wave (+ 4) is row tile jt, column pair ip with
// (jt, ip) = (0,0) (0,1) (1,0) (1,1) (2,1) (3,1); slot entry (row j, column i) is m[i][j].
__device__ __forceinline__ void write_transposed(char* out, const float* m, int wave, int lane)
{
    const int r = lane & 15, g = lane >> 4;
#pragma unroll
    for (int it = 0; it < 2; ++it) {
        const int ctp = wave + 4 * it;
        if (ctp < kTriPairs) {
            const int jt = ctp < 4 ? (ctp >> 1) : ctp - 2, ip = ctp < 4 ? (ctp & 1) : 1;
            const float* src = m + (32 * ip + 4 * g) * kLd + 16 * jt + r;
            const bool low = ctp == 2 || ctp == 5;        // first block of the pair lies below the diagonal of m^T: zero
            floatx4 x0, x1;
#pragma unroll
            for (int e = 0; e < 4; ++e) { x0[e] = src[e * kLd]; x1[e] = src[(16 + e) * kLd]; }
            const u32x2 q0 = low ? u32x2{0u, 0u} : to_quad(x0);
            const u32x2 q1 = to_quad(x1);
            const u32x4 v = {q0.x, q0.y, q1.x, q1.y};
            st16(out + (size_t)(ctp * 64 + lane) * 16, v);
        }
    }
}

}  // namespace

// BWD = true: the record of the backward pass,
// [T' | M^T | P^T | gamma_i | gamma_C/gamma_i | beta_i | 1/(||k_i||^2+eps) | 1/||q_i||]
// (M = (I + L)^{-1}; the transposes as the 6 upper-triangular tile-pairs, see kla_mma.hpp).  kOptGdnBeta: beta = eta
// and the fourth vector, d beta / d eta, is 1; kOptNormalizeQ: P^T carries 1/||q_i|| and the fifth vector holds it
// (1 otherwise).
template <int DK, bool BWD>
__global__ __launch_bounds__(256, 3) void intra_bf16_kernel(IntraArgs<bf16_t> a)
{
    constexpr int RB = DK * 2, PPR = DK / 8, KP = DK / 32;
    constexpr int RPB = 1024 / RB, NKB = 64 / RPB;           // rows per 1 KiB copy block, blocks per tile
    constexpr int TILE = 64 * RB;
    constexpr int REC = BWD ? bwd_record_bytes<bf16_t>() : ws_record_bytes<bf16_t>(), HALF = ws_half_bytes<bf16_t>();
    constexpr int VEC = (BWD ? 3 : 2) * HALF;                // offset of the fp32 vectors in the record
    static_assert(2 * TILE >= 64 * kLd * 4 || DK == 64, "P image overlays the K/Q tiles");

    __shared__ __attribute__((aligned(1024))) char kq[2 * TILE > 64 * kLd * 4 ? 2 * TILE : 64 * kLd * 4];
    __shared__ __attribute__((aligned(16))) float M[64 * kLd];
    __shared__ __attribute__((aligned(16))) float beta_s[64];
    __shared__ __attribute__((aligned(16))) float g_s[64];
    __shared__ __attribute__((aligned(16))) float eta_s[64];
    __shared__ __attribute__((aligned(16))) float rq_s[64];      // 1/||q_i|| when the read-out is normalised, else 1
    __shared__ __attribute__((aligned(16))) float invden_s[BWD ? 64 : 4];
    float* Pm = reinterpret_cast<float*>(kq);

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int r = lane & 15, g = lane >> 4;
    const bool norm_q = (a.opts & kOptNormalizeQ) != 0, gdn = (a.opts & kOptGdnBeta) != 0;

    // ---- which chunk of which sequence -------------------------------------------------------
    const int h = blockIdx.x % a.H;
    const int cg = blockIdx.x / a.H;
    const ChunkPos cp = chunk_pos(a.cu_seqlens, a.chunk_off, a.n_seq, a.T, a.NT, cg);
    const long tok0 = cp.tok0;
    const int clen = cp.clen;
    char* rec = reinterpret_cast<char*>(a.wsT) + (size_t)blockIdx.x * REC;

    // ---- phase 0: K, Q -> LDS by the copy engine; gates meanwhile ---------------------------------
    {
        const size_t kq_row = (size_t)a.H * DK * 2;
        const char* kb = reinterpret_cast<const char*>(a.k) + (size_t)tok0 * kq_row + (size_t)h * DK * 2;
        const char* qb = reinterpret_cast<const char*>(a.q) + (size_t)tok0 * kq_row + (size_t)h * DK * 2;
        const int lrow = lane / PPR, pcol = lane % PPR;
#pragma unroll
        for (int i = 0; i < NKB / 4; ++i) {
            const int b = wave + 4 * i;
            const int row = b * RPB + lrow;
            const int lo = min(row, clen - 1) * (int)kq_row + ((pcol ^ swz_piece<DK>(row)) * 16);
            dma16(kb, lo, kq + b * 1024);
            dma16(qb, lo, kq + TILE + b * 1024);
        }
        if (wave == 0) {
            float x = lane < clen ? a.log_alpha[(size_t)(tok0 + lane) * a.H + h] : 0.f;
#pragma unroll
            for (int off = 1; off < 64; off <<= 1) {
                const float y = __shfl_up(x, off, kWave);
                if (lane >= off) x += y;
            }
            const float x2 = x * 1.44269504088896341f;   // in units of log 2: every decay ratio is one v_exp_f32
            g_s[lane] = x2;
            eta_s[lane] = lane < clen ? a.eta[(size_t)(tok0 + lane) * a.H + h] : 0.f;
            if constexpr (!BWD) a.wsG[(size_t)blockIdx.x * 128 + lane] = x;
            rq_s[lane] = 1.f;
            const float gl2 = __shfl(x2, 63, kWave);
            float* dec = reinterpret_cast<float*>(rec + VEC);
            dec[lane] = __builtin_amdgcn_exp2f(x2);            // gamma_i
            dec[64 + lane] = __builtin_amdgcn_exp2f(gl2 - x2); // gamma_C / gamma_i
        }
        wait_vmcnt<0>();
    }
    __syncthreads();

    // ---- query norms for the normalised read-out o_t = S_t^T q_t / ||q_t|| (Sec. 3.3): wave w takes rows
    //      16 w + r, each of its four lane groups a quarter of the row
    if (norm_q) {
        const int row = 16 * wave + r;
        const char* qrow = kq + TILE + row * RB;
        float ss = 0.f;
#pragma unroll
        for (int i = 0; i < PPR / 4; ++i) {
            const u32x4 w = ld16(qrow + ((((PPR / 4) * g + i) ^ swz_piece<DK>(row)) * 16));
#pragma unroll
            for (int m = 0; m < 4; ++m) {
                const float x0 = __uint_as_float(w[m] << 16), x1 = __uint_as_float(w[m] & 0xffff0000u);
                ss += x0 * x0; ss += x1 * x1;
            }
        }
        ss += __shfl_xor(ss, 16, kWave);
        ss += __shfl_xor(ss, 32, kWave);
        if (g == 0) rq_s[row] = ss > 0.f ? 1.0f / sqrtf(ss) : 0.f;     // ordered after wave 0's default by the barrier above
    }

    // ---- phase 2a: Gram products K K^T and Q K^T on the lower-triangular tiles; five tiles per wave,
    //      five independent accumulators, shared operand row blocks read one contraction step ahead ----
    floatx4 acc[5];
#pragma unroll
    for (int jb = 0; jb < 5; ++jb) acc[jb] = floatx4{0.f, 0.f, 0.f, 0.f};
    {
        const int sw = swz_piece<DK>(r);             // the swizzle has period 8 rows
        const char* rowp = kq + r * RB;              // row r of row block 0 of K; block b: + (b & 3) 16 RB (+ TILE for Q)
        static_for<4>([&](auto wc) {
            constexpr int W = wc;
            if (wave != W) return;
            u32x4 sl[2][8];
            auto load = [&](int kp, u32x4 (&dst)[8]) {
                const int c16 = ((4 * kp + g) ^ sw) * 16;
                static_for<8>([&](auto bc) {
                    constexpr int B = bc;
                    if constexpr (gram_needs(W, B)) dst[B] = ld16(rowp + (B >> 2) * TILE + (B & 3) * 16 * RB + c16);
                });
            };
            load(0, sl[0]);
            static_for<KP>([&](auto kc) {
                constexpr int kp = kc;
                if constexpr (kp + 1 < KP) load(kp + 1, sl[(kp + 1) & 1]);
                static_for<5>([&](auto jc) {
                    constexpr int jb = jc;
                    constexpr GramJob J = kJobs[W][jb];
                    const u32x4 b = sl[kp & 1][J.tj];
                    const u32x2 b0 = {b[0], b[1]}, b1 = {b[2], b[3]};
                    mma_bf16(acc[jb], sl[kp & 1][J.q * 4 + J.ti], b0, b1);
                });
            });
            // ||k_i||^2 is the diagonal of K K^T (exact bf16 products, fp32 sums): beta of eq. (3) from the
            // four diagonal tiles, by the lane that holds element (i, i)
            static_for<5>([&](auto jc) {
                constexpr int jb = jc;
                constexpr GramJob J = kJobs[W][jb];
                if constexpr (J.q == 0 && J.ti == J.tj) {
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        if (4 * g + e == r) {
                            beta_s[16 * J.ti + r] = gdn ? eta_s[16 * J.ti + r] : kaczmarz_beta_fast(eta_s[16 * J.ti + r], acc[jb][e], a.eps);
                            if constexpr (BWD) invden_s[16 * J.ti + r] = gdn ? 1.f : kaczmarz_beta_fast(1.f, acc[jb][e], a.eps);
                        }
                }
            });
        });
    }
    __syncthreads();   // K/Q tiles are dead from here on (Pm overlays them); beta_s and rq_s are complete
    if (wave == 0) {                                     // third vector of the record (and the scale itself)
        float* dec = reinterpret_cast<float*>(rec + VEC);
        if constexpr (BWD) { dec[128 + lane] = beta_s[lane]; dec[192 + lane] = invden_s[lane]; dec[256 + lane] = rq_s[lane]; }
        else {
            dec[128 + lane] = __builtin_amdgcn_exp2f(g_s[lane]) * rq_s[lane];
            a.wsG[(size_t)blockIdx.x * 128 + 64 + lane] = rq_s[lane];
        }
    }

    // ---- phase 2b: decay, mask, beta -> L (into M) and P (into Pm) as fp32.  Tile coordinates are compile-time
    //      per wave, so only the diagonal tiles pay for the triangular mask ------------------------------
    static_for<4>([&](auto wc) {
        constexpr int W = wc;
        if (wave != W) return;
        static_for<5>([&](auto jc) {
            constexpr int jb = jc;
            constexpr GramJob J = kJobs[W][jb];
            constexpr int ti = J.ti, tj = J.tj;
            const float gj = g_s[16 * tj + r];
            const floatx4 gi = ldf4(g_s + 16 * ti + 4 * g);
            floatx4 f;                               // gamma_i / gamma_j = 2^(g_i - g_j), only used where j <= i
#pragma unroll
            for (int e = 0; e < 4; ++e) f[e] = __builtin_amdgcn_exp2f(ti == tj ? fminf(gi[e] - gj, 0.f) : gi[e] - gj);
            if constexpr (J.q == 0) {
                const floatx4 bi = ldf4(beta_s + 16 * ti + 4 * g);
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    float x = bi[e] * f[e] * acc[jb][e];
                    if (ti == tj) x = (r < 4 * g + e) ? x : 0.f;                       // strictly lower
                    M[(16 * ti + 4 * g + e) * kLd + 16 * tj + r] = x;
                }
            } else {
                floatx4 rqv = {1.f, 1.f, 1.f, 1.f};
                if (norm_q) rqv = ldf4(rq_s + 16 * ti + 4 * g);
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    float x = f[e] * acc[jb][e] * rqv[e];
                    if (ti == tj) x = (r <= 4 * g + e) ? x : 0.f;                      // lower with diagonal
                    if (clen < 64) x = (16 * ti + 4 * g + e < clen) ? x : 0.f;         // rows beyond a short chunk
                    Pm[(16 * ti + 4 * g + e) * kLd + 16 * tj + r] = x;
                }
            }
        });
    });
    // the six strictly-upper tiles are never written: every reader below knows they are zero
    __syncthreads();

    // ---- phase 3: diagonal 16x16 blocks D = (I + L_bb)^{-1} by forward substitution (wave w: block w,
    //      lane column r, the four 16-lane groups redundantly), rows read one ahead; in place ---------
    {
        const float* Lb = M + (16 * wave) * kLd + 16 * wave;
        float x[16];
        floatx4 row[4], nxt[4] = {};
#pragma unroll
        for (int c4 = 0; c4 < 4; ++c4) row[c4] = ldf4(Lb + kLd + 4 * c4);          // row 1
        x[0] = (r == 0) ? 1.f : 0.f;
#pragma unroll
        for (int i = 1; i < 16; ++i) {
            if (i + 1 < 16) {
#pragma unroll
                for (int c4 = 0; c4 < 4; ++c4)
                    if (4 * c4 <= i) nxt[c4] = ldf4(Lb + (i + 1) * kLd + 4 * c4);
            }
            float s0 = (i == r) ? 1.f : 0.f, s1 = 0.f;
#pragma unroll
            for (int rr = 0; rr < i; ++rr) {
                if (rr & 1) s1 -= row[rr >> 2][rr & 3] * x[rr];
                else        s0 -= row[rr >> 2][rr & 3] * x[rr];
            }
            x[i] = s0 + s1;
#pragma unroll
            for (int c4 = 0; c4 < 4; ++c4) row[c4] = nxt[c4];
        }
        // only this wave touches block (w, w), and its reads above precede these writes in program order
#pragma unroll
        for (int i = 0; i < 16; ++i)
            if ((i >> 2) == g) M[(16 * wave + i) * kLd + 16 * wave + r] = x[i];
    }
    // P (forward) or P^T (backward) goes out to the workspace in operand order (fp32 image -> bf16 slots).  Stored
    // tile-pair ctp = wave (+ 4): wave-uniform, so its tile coordinates are scalars; slot = ctp * 64 + lane.
    if constexpr (BWD) write_transposed(rec + 2 * HALF, Pm, wave, lane);
    else {
        char* out = rec + HALF;
#pragma unroll
        for (int it = 0; it < 2; ++it) {
            const int ctp = wave + 4 * it;
            if (ctp < kTriPairs) {
                const int ti = ctp < 2 ? ctp : 2 + ((ctp - 2) >> 1), jp = ctp < 2 ? 0 : ((ctp - 2) & 1);
                const float* src = Pm + (16 * ti + r) * kLd + 32 * jp + 4 * g;
                const bool up = ctp == 0 || ctp == 3;         // second block of the pair is an upper tile: zero
                const u32x2 q0 = to_quad(ldf4(src));
                const u32x2 q1 = up ? u32x2{0u, 0u} : to_quad(ldf4(src + 16));
                const u32x4 v = {q0.x, q0.y, q1.x, q1.y};
                st16(out + (size_t)(ctp * 64 + lane) * 16, v);
            }
        }
    }
    __syncthreads();

    // ---- phase 4: 32x32 level, in place.  Waves 0,1: block pair (a, b) = (2m, 2m+1): T_ba = -D_b (L_ba D_a)
    if (wave < 2) {
        const int ra = 32 * wave, rb = ra + 16;
        floatx4 y = {0.f, 0.f, 0.f, 0.f}, z = {0.f, 0.f, 0.f, 0.f};
        mma16f(y, aq(M, rb, ra, r, g), bq(M, ra, ra, r, g));
        mma16f(z, aq(M, rb, rb, r, g), y);           // an accumulator tile is the next product's B quad
#pragma unroll
        for (int e = 0; e < 4; ++e) M[(rb + 4 * g + e) * kLd + ra + r] = -z[e];    // only this wave read L_ba
    }
    __syncthreads();

    // ---- phase 5: 64x64 level, in place.  T[32:64, 0:32] = -T22 (L21 T11); wave = (row tile ti, col tile tj)
    {
        const int ti = wave >> 1, tj = wave & 1;
        floatx4 y0 = {0.f, 0.f, 0.f, 0.f}, y1 = {0.f, 0.f, 0.f, 0.f}, z = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int tm = 0; tm < 2; ++tm) {
            if (tm == 0 && tj == 1) continue;        // T11 tile (0, 1) is zero
            const floatx4 b = bq(M, 16 * tm, 16 * tj, r, g);
            mma16f(y0, aq(M, 32, 16 * tm, r, g), b);
            mma16f(y1, aq(M, 48, 16 * tm, r, g), b);
        }
        mma16f(z, aq(M, 32 + 16 * ti, 32, r, g), y0);
        if (ti == 1) mma16f(z, aq(M, 32 + 16 * ti, 48, r, g), y1);   // T22 tile (0, 1) is zero
        __syncthreads();                             // all waves have read L21 before it is overwritten
#pragma unroll
        for (int e = 0; e < 4; ++e) M[(32 + 16 * ti + 4 * g + e) * kLd + 16 * tj + r] = -z[e];
    }
    __syncthreads();

    // ---- phase 6: T' = T diag(beta) -> workspace in operand order ------------------------------
    {
#pragma unroll
        for (int it = 0; it < 2; ++it) {
            const int ctp = wave + 4 * it;
            if (ctp < kTriPairs) {
                const int ti = ctp < 2 ? ctp : 2 + ((ctp - 2) >> 1), jp = ctp < 2 ? 0 : ((ctp - 2) & 1);
                const int cl = 32 * jp + 4 * g;
                const float* src = M + (16 * ti + r) * kLd + cl;
                const bool up = ctp == 0 || ctp == 3;
                const u32x2 q0 = to_quad(ldf4(src) * ldf4(beta_s + cl));
                const u32x2 q1 = up ? u32x2{0u, 0u} : to_quad(ldf4(src + 16) * ldf4(beta_s + cl + 16));
                const u32x4 v = {q0.x, q0.y, q1.x, q1.y};
                st16(rec + (size_t)(ctp * 64 + lane) * 16, v);
            }
        }
        if constexpr (BWD) write_transposed(rec + HALF, M, wave, lane);      // M^T
    }
}

hipError_t launch_intra_bf16(const IntraArgs<bf16_t>& a, int dk, int n_chunks, hipStream_t st)
{
    if (n_chunks == 0) return hipSuccess;
    const dim3 grid((unsigned)n_chunks * a.H), block(256);
    if (dk == 64) hipLaunchKernelGGL((intra_bf16_kernel<64, false>), grid, block, 0, st, a);
    else          hipLaunchKernelGGL((intra_bf16_kernel<128, false>), grid, block, 0, st, a);
    return hipGetLastError();
}

// the records of the backward pass at a.wsT; a.wsP and a.wsG unused, a.opts = 0
hipError_t launch_intra_bwd_bf16(const IntraArgs<bf16_t>& a, int dk, int n_chunks, hipStream_t st)
{
    if (n_chunks == 0) return hipSuccess;
    const dim3 grid((unsigned)n_chunks * a.H), block(256);
    if (dk == 64) hipLaunchKernelGGL((intra_bf16_kernel<64, true>), grid, block, 0, st, a);
    else          hipLaunchKernelGGL((intra_bf16_kernel<128, true>), grid, block, 0, st, a);
    return hipGetLastError();
}

}  // namespace kla
