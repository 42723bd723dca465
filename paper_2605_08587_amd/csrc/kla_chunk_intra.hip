// Intra-chunk stage of the chunkwise forward (Algorithm 1 right panel, lines 1-4 and the
// matrix of eq. (6)); fully parallel over (chunk, head).
//
// Per chunk of C = 64 tokens of one head it computes
//   beta_i = eta_i / (||k_i||^2 + eps)                                   eq. (3)
//   g_i    = sum_{r<=i} log alpha_r   (log gamma_i, restarting at the chunk)
//   L      = B (A^- o K K^T),  L_ij = beta_i exp(g_i - g_j) k_i.k_j  (j < i)
//   T'     = (I + L)^{-1} B          so that eq. (6) reads  U = T' (V - D_gamma K S_0)
//   P      = A o Q K^T,  P_ij = exp(g_i - g_j) q_i.k_j  (j <= i)         eq. (7)
// and leaves T', P (in the element type, in MFMA operand order) and g in the workspace for the
// scan stage.  Every decay ratio is formed as exp of a difference of g, masked before the exp,
// because gamma itself underflows fp32 inside a chunk for fast decays.
//
// (I + L)^{-1} is built in fp32: the four 16x16 diagonal blocks by forward substitution in LDS,
// then the off-diagonal blocks by two levels of block products on fp32 MFMA,
//   [T11 0; T21 T22] with T21 = -T22 (L21 T11).
#include "kla_common.hpp"
#include "kla_kernels.hpp"
#include "kla_mma.hpp"

namespace kla {

namespace {

constexpr int kLdm = 68;   // row stride (floats) of the fp32 64x64 matrices in LDS: 16-byte aligned rows

// lower-triangular 16x16 tile enumeration of a 64x64 matrix: 10 tiles
__device__ __constant__ const int8_t kTileI[10] = {0, 1, 1, 2, 2, 2, 3, 3, 3, 3};
__device__ __constant__ const int8_t kTileJ[10] = {0, 0, 1, 0, 1, 2, 0, 1, 2, 3};

__device__ __forceinline__ float4 ld4(const float* p) { return *reinterpret_cast<const float4*>(p); }

// B-operand quad of a row-major fp32 matrix: rows 4g..4g+3 of column r
__device__ __forceinline__ float4 bquad(const float* m, int row0, int col0, int r, int g)
{
    const float* p = m + (row0 + 4 * g) * kLdm + col0 + r;
    return make_float4(p[0], p[kLdm], p[2 * kLdm], p[3 * kLdm]);
}
// A-operand quad: columns 4g..4g+3 of row r
__device__ __forceinline__ float4 aquad(const float* m, int row0, int col0, int r, int g)
{
    return ld4(m + (row0 + r) * kLdm + col0 + 4 * g);
}
__device__ __forceinline__ float4 acc_as_quad(floatx4 x) { return make_float4(x[0], x[1], x[2], x[3]); }

// A triangular 64x64 fp32 matrix m (row stride kLdm) -> 6 stored tile-pairs of operand slots at `out`.
// TRANSPOSE = false: the lower-triangular matrix itself (pairs tri_pair(it, jp), jp <= it/2), optionally with
// column j scaled by colscale[j].  TRANSPOSE = true: its transpose, which is upper triangular (pairs
// triu_pair(it, jp), jp >= it/2).  Called by all 256 threads.
template <typename E, bool TRANSPOSE, bool SCALE>
__device__ __forceinline__ void write_tri(char* out, const float* m, const float* colscale, int tid)
{
#pragma unroll
    for (int it = 0; it < 2; ++it) {
        const int sl = tid + 256 * it;           // slot index: stored tile-pair * 64 + lane
        if (sl >= kTriPairs * 64) break;
        const int ctp = sl >> 6, ln = sl & 63;
        int ti, jp;
        if constexpr (TRANSPOSE) { ti = ctp < 4 ? (ctp >> 1) : ctp - 2; jp = ctp < 4 ? (ctp & 1) : 1; }
        else                     { ti = ctp < 2 ? ctp : 2 + ((ctp - 2) >> 1); jp = ctp < 2 ? 0 : ((ctp - 2) & 1); }
        const int row = 16 * ti + (ln & 15), col = 32 * jp + 4 * (ln >> 4);
        floatx4 v0, v1;
        if constexpr (TRANSPOSE) {
#pragma unroll
            for (int e = 0; e < 4; ++e) { v0[e] = m[(col + e) * kLdm + row]; v1[e] = m[(col + 16 + e) * kLdm + row]; }
        } else {
            const float4 f0 = ld4(m + row * kLdm + col), f1 = ld4(m + row * kLdm + col + 16);
            v0[0] = f0.x; v0[1] = f0.y; v0[2] = f0.z; v0[3] = f0.w;
            v1[0] = f1.x; v1[1] = f1.y; v1[2] = f1.z; v1[3] = f1.w;
            if constexpr (SCALE) {
                const float4 b0 = ld4(colscale + col), b1 = ld4(colscale + col + 16);
                v0[0] *= b0.x; v0[1] *= b0.y; v0[2] *= b0.z; v0[3] *= b0.w;
                v1[0] *= b1.x; v1[1] *= b1.y; v1[2] *= b1.z; v1[3] *= b1.w;
            }
        }
        Slot<E> s; s.q0 = acc_to_quad<E>(v0); s.q1 = acc_to_quad<E>(v1);
        *reinterpret_cast<Slot<E>*>(out + (size_t)sl * slot_bytes<E>()) = s;
    }
}


// Phases 3-6 of the intra-chunk stage, shared by its variants: from L (strictly lower triangular, fp32, in Lm) and
// the fp32 image of P (in Pm) to the record at `rec`: T' = (I + L)^{-1} B and P (forward), or T', M^T and P^T
// (backward).  Tm receives (I + L)^{-1}; the strictly-upper tiles of Lm, Pm, Tm must be zero on entry.  Called by all
// 256 threads after a barrier; contains barriers.
template <typename E, bool BWD>
__device__ __forceinline__ void invert_and_store(const float* Lm, float* Tm, const float* Pm, const float* beta_s, char* rec,
                                                 int tid)
{
    const int lane = tid & 63, wave = tid >> 6;
    const int r = lane & 15, g = lane >> 4;
    // ---- phase 3: diagonal 16x16 blocks of (I+L)^{-1} by forward substitution (wave w: block w);
    //      meanwhile P goes out to the workspace in operand order ------------------------------
    {
        const int b0 = 16 * wave;
        float x[16];
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            float s = (i == r) ? 1.f : 0.f;
#pragma unroll
            for (int rr = 0; rr < i; ++rr) s -= Lm[(b0 + i) * kLdm + b0 + rr] * x[rr];
            x[i] = s;
        }
#pragma unroll
        for (int i = 0; i < 16; ++i)
            if ((i >> 2) == g) Tm[(b0 + i) * kLdm + b0 + r] = x[i];
    }
    if constexpr (BWD) write_tri<E, true, false>(rec + 2 * ws_half_bytes<E>(), Pm, nullptr, tid);      // P^T
    else               write_tri<E, false, false>(rec + ws_half_bytes<E>(), Pm, nullptr, tid);
    __syncthreads();

    // ---- phase 4: 32x32 level.  Waves 0,1: block pair (a, b) = (2m, 2m+1): T_ba = -D_b (L_ba D_a)
    if (wave < 2) {
        const int ra = 32 * wave, rb = ra + 16;
        floatx4 y = {0.f, 0.f, 0.f, 0.f}, z = {0.f, 0.f, 0.f, 0.f};
        mma16(y, aquad(Lm, rb, ra, r, g), bquad(Tm, ra, ra, r, g));
        mma16(z, aquad(Tm, rb, rb, r, g), acc_as_quad(y));
#pragma unroll
        for (int e = 0; e < 4; ++e) Tm[(rb + 4 * g + e) * kLdm + ra + r] = -z[e];
    }
    __syncthreads();

    // ---- phase 5: 64x64 level.  T[32:64, 0:32] = -T22 (L21 T11); wave = (row tile ti, col tile tj)
    {
        const int ti = wave >> 1, tj = wave & 1;
        floatx4 y0 = {0.f, 0.f, 0.f, 0.f}, y1 = {0.f, 0.f, 0.f, 0.f}, z = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int tm = 0; tm < 2; ++tm) {
            const float4 b = bquad(Tm, 16 * tm, 16 * tj, r, g);
            mma16(y0, aquad(Lm, 32, 16 * tm, r, g), b);
            mma16(y1, aquad(Lm, 48, 16 * tm, r, g), b);
        }
        mma16(z, aquad(Tm, 32 + 16 * ti, 32, r, g), acc_as_quad(y0));
        mma16(z, aquad(Tm, 32 + 16 * ti, 48, r, g), acc_as_quad(y1));
        // the block written below is read by no wave in this phase, so no barrier is needed here
#pragma unroll
        for (int e = 0; e < 4; ++e) Tm[(32 + 16 * ti + 4 * g + e) * kLdm + 16 * tj + r] = -z[e];
    }
    __syncthreads();

    // ---- phase 6: T' = T diag(beta) (and T^T for the backward) -> workspace in operand order ------------------
    {
        char* out = rec;
        if constexpr (BWD) {
            write_tri<E, false, true>(out, Tm, beta_s, tid);
            write_tri<E, true, false>(out + ws_half_bytes<E>(), Tm, nullptr, tid);
        } else {
            write_tri<E, false, true>(out, Tm, beta_s, tid);
        }
    }
}

}  // namespace

// BWD = false: the forward's records [T' | P | three vectors].  BWD = true: the records of the backward pass,
// [T' | M^T | P^T | gamma_i | gamma_C/gamma_i | beta_i | 1/(||k_i||^2+eps)] with M = (I + L)^{-1}, T' = M B; the transposes are stored as the
// 6 upper-triangular tile-pairs (see bwd_record_bytes in kla_mma.hpp).
template <typename E, int DK, bool BWD>
__global__ __launch_bounds__(256) void intra_kernel(IntraArgs<E> a)
{
    constexpr int REC = BWD ? bwd_record_bytes<E>() : ws_record_bytes<E>();
    constexpr int PPR = DK * (int)sizeof(E) / 16;    // 16-byte pieces per row
    constexpr int EPP = 16 / (int)sizeof(E);         // elements per piece
    constexpr int KP = DK / 32;                      // contraction pairs per row
    constexpr int OPB = 64 * DK * (int)sizeof(E);    // bytes of one operand area

    __shared__ __attribute__((aligned(16))) char op_area[2 * OPB > 64 * kLdm * 4 ? 2 * OPB : 64 * kLdm * 4];
    __shared__ __attribute__((aligned(16))) float Lm[64 * kLdm];
    __shared__ __attribute__((aligned(16))) float Tm[64 * kLdm];
    __shared__ __attribute__((aligned(16))) float beta_s[64];
    __shared__ __attribute__((aligned(16))) float rq_s[64];      // 1/||q_i|| when the read-out is normalised, else 1
    __shared__ __attribute__((aligned(16))) float g_s[64];
    __shared__ __attribute__((aligned(16))) float invden_s[BWD ? 64 : 4];   // 1/(||k_i||^2 + eps), for the backward pass
    E* Krq = reinterpret_cast<E*>(op_area);
    E* Qrq = reinterpret_cast<E*>(op_area + OPB);
    float* Pm = reinterpret_cast<float*>(op_area);   // reused after the Gram products are in registers

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int r = lane & 15, g = lane >> 4;

    // ---- which chunk of which sequence -------------------------------------------------------
    const int h = blockIdx.x % a.H;
    const int cg = blockIdx.x / a.H;                 // global chunk index
    const ChunkPos cp = chunk_pos(a.cu_seqlens, a.chunk_off, a.n_seq, a.T, a.NT, cg);
    const long tok0 = cp.tok0;
    const int clen = cp.clen;

    // ---- phase 1: K, Q -> LDS (operand order), key norms -> beta, log-decay prefix sum -> g ---
    {
        const size_t row_stride = (size_t)a.H * DK;
        const E* kb = a.k + (size_t)tok0 * row_stride + (size_t)h * DK;
        const E* qb = a.q + (size_t)tok0 * row_stride + (size_t)h * DK;
#pragma unroll
        for (int it = 0; it < 64 * PPR / 256; ++it) {
            const int pi = tid + 256 * it;
            const int row = pi / PPR, piece = pi % PPR;
            uint4 kd = make_uint4(0, 0, 0, 0), qd = make_uint4(0, 0, 0, 0);
            if (row < clen) {
                kd = *reinterpret_cast<const uint4*>(kb + (size_t)row * row_stride + piece * EPP);
                qd = *reinterpret_cast<const uint4*>(qb + (size_t)row * row_stride + piece * EPP);
            }
            store_rq_piece(Krq, KP, row, piece, kd);
            store_rq_piece(Qrq, KP, row, piece, qd);
            auto sum_squares = [](uint4 d) {
                float ss = 0.f;
                if constexpr (sizeof(E) == 2) {
                    const uint32_t w[4] = {d.x, d.y, d.z, d.w};
#pragma unroll
                    for (int m = 0; m < 4; ++m) {
                        const float x0 = bf16_bits_to_float(w[m] & 0xffffu), x1 = bf16_bits_to_float(w[m] >> 16);
                        ss += x0 * x0; ss += x1 * x1;
                    }
                } else {
                    const float x0 = __uint_as_float(d.x), x1 = __uint_as_float(d.y), x2 = __uint_as_float(d.z),
                                x3 = __uint_as_float(d.w);
                    ss = x0 * x0 + x1 * x1 + x2 * x2 + x3 * x3;
                }
                return ss;
            };
            float ss = sum_squares(kd), sq = sum_squares(qd);
#pragma unroll
            for (int off = 1; off < PPR; off <<= 1) { ss += __shfl_xor(ss, off, kWave); sq += __shfl_xor(sq, off, kWave); }
            if (piece == 0) {
                const float et = row < clen ? a.eta[(size_t)(tok0 + row) * a.H + h] : 0.f;
                beta_s[row] = (a.opts & kOptGdnBeta) ? et : kaczmarz_beta(et, ss, a.eps);
                // scale of the normalised read-out o_t = S_t^T q_t / ||q_t|| (Sec. 3.3); a zero query gives 0
                rq_s[row] = (a.opts & kOptNormalizeQ) ? (sq > 0.f ? 1.0f / sqrtf(sq) : 0.f) : 1.f;
                if constexpr (BWD) invden_s[row] = (a.opts & kOptGdnBeta) ? 1.f : ((ss + a.eps == 0.f) ? 0.f : 1.0f / (ss + a.eps));
            }
        }
        if (wave == 0) {
            float x = lane < clen ? a.log_alpha[(size_t)(tok0 + lane) * a.H + h] : 0.f;
#pragma unroll
            for (int off = 1; off < 64; off <<= 1) {
                const float y = __shfl_up(x, off, kWave);
                if (lane >= off) x += y;
            }
            g_s[lane] = x;
            if constexpr (!BWD) a.wsG[(size_t)blockIdx.x * 128 + lane] = x;
            // decay factors the scan stage multiplies with: gamma_i and gamma_C / gamma_i
            const float gl = __shfl(x, 63, kWave);
            float* dec = reinterpret_cast<float*>(reinterpret_cast<char*>(a.wsT) + (size_t)blockIdx.x * REC
                                                  + (BWD ? 3 : 2) * ws_half_bytes<E>());
            dec[lane] = expf(x);
            dec[64 + lane] = expf(gl - x);
        }
    }
    __syncthreads();
    if (wave == 0) {                                     // third vector of the record (and the scale itself)
        float* dec = reinterpret_cast<float*>(reinterpret_cast<char*>(a.wsT) + (size_t)blockIdx.x * REC
                                              + (BWD ? 3 : 2) * ws_half_bytes<E>());
        if constexpr (BWD) { dec[128 + lane] = beta_s[lane]; dec[192 + lane] = invden_s[lane]; dec[256 + lane] = rq_s[lane]; }
        else {
            dec[128 + lane] = expf(g_s[lane]) * rq_s[lane];
            a.wsG[(size_t)blockIdx.x * 128 + 64 + lane] = rq_s[lane];
        }
    }

    // ---- phase 2a: Gram products K K^T and Q K^T on the lower-triangular tiles ---------------
    floatx4 acc[5];
#pragma unroll
    for (int jb = 0; jb < 5; ++jb) {
        const int job = wave + 4 * jb;               // 0..9: K K^T tiles, 10..19: Q K^T tiles
        const int lt = job % 10;
        const int ti = kTileI[lt], tj = kTileJ[lt];
        const E* A = job < 10 ? Krq : Qrq;
        floatx4 c = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int kp = 0; kp < KP; ++kp) {
            const Slot<E> sa = load_slot(A, ti * KP + kp, lane);
            const Slot<E> sb = load_slot(Krq, tj * KP + kp, lane);
            mma32<E>(c, sa, sb.q0, sb.q1);
        }
        acc[jb] = c;
    }
    __syncthreads();   // operand areas are dead from here on; Pm overlays them

    // ---- phase 2b: decay, mask, beta -> L and P as fp32 matrices; zero the upper tiles --------
#pragma unroll
    for (int jb = 0; jb < 5; ++jb) {
        const int job = wave + 4 * jb;
        const int lt = job % 10;
        const int ti = kTileI[lt], tj = kTileJ[lt];
        const int j = 16 * tj + r;
        const float gj = g_s[j];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int i = 16 * ti + 4 * g + e;
            const float gi = g_s[i];
            if (job < 10) {
                const float val = (j < i) ? beta_s[i] * expf(gi - gj) * acc[jb][e] : 0.f;
                Lm[i * kLdm + j] = val;
            } else {
                const float val = (j <= i) ? expf(gi - gj) * acc[jb][e] * rq_s[i] : 0.f;
                Pm[i * kLdm + j] = val;
            }
        }
    }
    for (int x = tid; x < 6 * 256; x += 256) {       // the six strictly-upper tiles
        const int t = x >> 8, e = x & 255;
        const int ti = t < 3 ? 0 : (t < 5 ? 1 : 2);
        const int tj = t < 3 ? t + 1 : (t < 5 ? t - 1 : 3);
        const int idx = (16 * ti + (e >> 4)) * kLdm + 16 * tj + (e & 15);
        Lm[idx] = 0.f; Pm[idx] = 0.f; Tm[idx] = 0.f;
    }
    __syncthreads();

    invert_and_store<E, BWD>(Lm, Tm, Pm, beta_s, reinterpret_cast<char*>(a.wsT) + (size_t)blockIdx.x * REC, tid);
}

template <typename E>
hipError_t launch_intra(const IntraArgs<E>& a, int dk, int n_chunks, hipStream_t st)
{
    if (n_chunks == 0) return hipSuccess;
    const dim3 grid((unsigned)n_chunks * a.H), block(256);
    if (dk == 64) hipLaunchKernelGGL((intra_kernel<E, 64, false>), grid, block, 0, st, a);
    else          hipLaunchKernelGGL((intra_kernel<E, 128, false>), grid, block, 0, st, a);
    return hipGetLastError();
}
template hipError_t launch_intra<float>(const IntraArgs<float>&, int, int, hipStream_t);
template hipError_t launch_intra<bf16_t>(const IntraArgs<bf16_t>&, int, int, hipStream_t);

// The records of the backward pass: a.wsT points at them, a.wsP and a.wsG are not used.  kOptGdnBeta: beta = eta, and
// the record's fourth vector, d beta / d eta, is 1; kOptNormalizeQ: P^T carries 1/||q_i||, which is also the fifth vector.
template <typename E>
hipError_t launch_intra_bwd(const IntraArgs<E>& a, int dk, int n_chunks, hipStream_t st)
{
    if (n_chunks == 0) return hipSuccess;
    const dim3 grid((unsigned)n_chunks * a.H), block(256);
    if (dk == 64) hipLaunchKernelGGL((intra_kernel<E, 64, true>), grid, block, 0, st, a);
    else          hipLaunchKernelGGL((intra_kernel<E, 128, true>), grid, block, 0, st, a);
    return hipGetLastError();
}
template hipError_t launch_intra_bwd<float>(const IntraArgs<float>&, int, int, hipStream_t);
template hipError_t launch_intra_bwd<bf16_t>(const IntraArgs<bf16_t>&, int, int, hipStream_t);

// ---- diagonal gating (App. B, "Extension to diagonal gating") -----------------------------------------------
// log_alpha holds d_k values per token and head; gamma_i is a vector and every decay ratio acts inside the inner
// products:  L_ij = beta_i sum_c k_ic k_jc gamma_ic/gamma_jc (j < i),  P_ij = sum_c q_ic k_jc gamma_ic/gamma_jc (j <= i).
// Every ratio is split at a reference row e with j <= e < i, gamma_i/gamma_j = [gamma_i/gamma_e][gamma_e/gamma_j], so
// that both factors are <= 1 (gamma itself may underflow inside a chunk; nothing can overflow): the off-diagonal
// 16x16 tiles and the lower-left 8x8 block of each diagonal tile become ordinary MFMA products of rescaled rows,
// formed in registers from fp32 tables of K, Q and the running log sums; only the 8x8 blocks on the diagonal are
// summed pair by pair on the vector ALUs (there gamma_i/gamma_j <= 1 directly).  The triangular inverse and the records are those of
// the scalar kernel, with unit decay vectors: the decay travels in the operands the scan is given instead,
//     K+ = K o Gamma,  Q+ = Q o Gamma,  K~ = K o (gamma_C / Gamma)   (all factors <= 1)  and gamma_C per channel,
// which this kernel writes next to the records.  Options: kOptGdnBeta (beta = eta); kOptNormalizeQ, for which the
// rows of Q+ and of P are divided by ||q_i|| here, so that the scan needs no variant of its own.
template <typename E, int DK>
__global__ __launch_bounds__(256, 3) void intra_diag_kernel(IntraDiagArgs<E> a)
{
    // The tables hold CH = 64 channels at a time: d_k = 128 takes two passes, whose partial sums meet in the registers
    // that hold the products.  That keeps the kernel at the LDS footprint of the 64x64 fp32 matrices of the later
    // phases (52.5 KB), i.e. three workgroups per CU instead of two.
    constexpr int CH = 64, NPASS = DK / CH;
    constexpr int EPP = 16 / (int)sizeof(E), PPR = DK / EPP, PPH = CH / EPP;
    constexpr int LE = CH + EPP;                     // row stride of the K, Q tables (elements): one 16-byte piece of padding
    constexpr int LD = CH + 4;                       // row stride of the log-sum table (floats)
    constexpr int TE = 64 * LE * (int)sizeof(E), TG = 64 * LD * 4;
    constexpr int NSEG = 256 / CH, SROWS = 64 / NSEG;   // the running sums: 256 threads = CH channels x NSEG row segments
    constexpr int REC = ws_record_bytes<E>();
    __shared__ __attribute__((aligned(16))) char area[2 * TE + TG > 3 * 64 * kLdm * 4 ? 2 * TE + TG : 3 * 64 * kLdm * 4];
    __shared__ __attribute__((aligned(16))) float beta_s[64];
    __shared__ __attribute__((aligned(16))) float rq_s[64];      // 1/||q_i|| for the normalised read-out (Sec. 3.3), else 1
    __shared__ float segsum[NSEG][CH];
    const E* Kp = reinterpret_cast<const E*>(area);           // K rows (element type), later overlaid by Lm, Pm, Tm
    const E* Qp = reinterpret_cast<const E*>(area + TE);      // Q rows
    float* Gs = reinterpret_cast<float*>(area + 2 * TE);      // running sums of log2 alpha per channel
    float* Lm = reinterpret_cast<float*>(area);
    float* Pm = reinterpret_cast<float*>(area + 64 * kLdm * 4);
    float* Tm = reinterpret_cast<float*>(area + 2 * 64 * kLdm * 4);

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int h = blockIdx.x % a.H;
    const int cg = blockIdx.x / a.H;
    const ChunkPos cp = chunk_pos(a.cu_seqlens, a.chunk_off, a.n_seq, a.T, a.NT, cg);
    const long tok0 = cp.tok0;
    const int clen = cp.clen;
    const size_t row_stride = (size_t)a.H * DK;
    auto unpack = [](uint4 d, float (&f)[EPP]) {
        if constexpr (sizeof(E) == 2) {
            const uint32_t w[4] = {d.x, d.y, d.z, d.w};
#pragma unroll
            for (int m = 0; m < 4; ++m) { f[2 * m] = bf16_bits_to_float(w[m] & 0xffffu); f[2 * m + 1] = bf16_bits_to_float(w[m] >> 16); }
        } else {
            f[0] = __uint_as_float(d.x); f[1] = __uint_as_float(d.y); f[2] = __uint_as_float(d.z); f[3] = __uint_as_float(d.w);
        }
    };
    auto pack = [](const float (&f)[EPP]) {
        if constexpr (sizeof(E) == 2)
            return make_uint4(pack_bf16x2(f[0], f[1]), pack_bf16x2(f[2], f[3]), pack_bf16x2(f[4], f[5]), pack_bf16x2(f[6], f[7]));
        else
            return make_uint4(__float_as_uint(f[0]), __float_as_uint(f[1]), __float_as_uint(f[2]), __float_as_uint(f[3]));
    };

    auto ld4e = [](const E* p) {                     // 4 consecutive elements (8- resp. 16-byte aligned) as floats
        floatx4 f;
        if constexpr (sizeof(E) == 2) {
            const uint2 w = *reinterpret_cast<const uint2*>(p);
            f[0] = bf16_bits_to_float(w.x & 0xffffu); f[1] = bf16_bits_to_float(w.x >> 16);
            f[2] = bf16_bits_to_float(w.y & 0xffffu); f[3] = bf16_bits_to_float(w.y >> 16);
        } else {
            const float4 w = *reinterpret_cast<const float4*>(p);
            f[0] = w.x; f[1] = w.y; f[2] = w.z; f[3] = w.w;
        }
        return f;
    };
    auto ld4f = [](const float* p) { const float4 w = *reinterpret_cast<const float4*>(p); floatx4 f; f[0] = w.x; f[1] = w.y; f[2] = w.z; f[3] = w.w; return f; };

    const E* kb = a.k + (size_t)tok0 * row_stride + (size_t)h * DK;
    const E* qb = a.q + (size_t)tok0 * row_stride + (size_t)h * DK;
    const float* lb = a.log_alpha + (size_t)tok0 * row_stride + (size_t)h * DK;

    // ---- phase 0: the normalised read-out (Sec. 3.3) needs 1/||q_i|| over all channels before the first pass scales
    //      Q; otherwise nothing is read ahead of the passes (the key norms are summed up pass by pass)
    if (a.opts & kOptNormalizeQ) {
#pragma unroll
        for (int it = 0; it < 64 * PPR / 256; ++it) {
            const int pi = tid + 256 * it;
            const int row = pi / PPR, piece = pi % PPR;
            uint4 qd = make_uint4(0, 0, 0, 0);
            if (row < clen) qd = *reinterpret_cast<const uint4*>(qb + (size_t)row * row_stride + piece * EPP);
            float qf0[EPP];
            unpack(qd, qf0);
            float sq = 0.f;
#pragma unroll
            for (int i = 0; i < EPP; ++i) sq += qf0[i] * qf0[i];
#pragma unroll
            for (int off = 1; off < PPR; off <<= 1) sq += __shfl_xor(sq, off, kWave);
            if (piece == 0) rq_s[row] = sq > 0.f ? 1.0f / sqrtf(sq) : 0.f;
        }
    } else if (tid < 64) rq_s[tid] = 1.f;
    if (tid < 128) {                                 // unit decay vectors for the scan: g = 0, 1/||q|| = 1
        a.wsG[(size_t)blockIdx.x * 128 + tid] = tid < 64 ? 0.f : 1.f;
        float* dec = reinterpret_cast<float*>(reinterpret_cast<char*>(a.wsT) + (size_t)blockIdx.x * REC + 2 * ws_half_bytes<E>());
        dec[tid] = 1.f;
        if (tid < 64) dec[128 + tid] = 1.f;
    }

    // accumulators of phase 2a, over all passes
    const int r = lane & 15, g = lane >> 4;
    floatx4 tkk[2], tqk[2];
#pragma unroll
    for (int jb = 0; jb < 2; ++jb) { tkk[jb] = floatx4{0.f, 0.f, 0.f, 0.f}; tqk[jb] = tkk[jb]; }
    // The MFMA jobs of phase 2a, two per wave: jobs 0..5 are the off-diagonal tiles (ti, tj); jobs 6 and 7 each take the
    // lower-left 8x8 blocks of TWO diagonal tiles (2 (job - 6) and the next) in one 16x16 product - operand rows 0..7 belong
    // to the first tile, rows 8..15 to the second, and the two off-diagonal 8x8 blocks of the result are not used.
    // Per lane: the table row of its A operand row (ja), of its B operand row (jbr) and of the reference rows they are
    // split at.
    auto job_rows = [&](int job, int& ja, int& jbr, int& ea, int& eb) {
        if (job < 6) {
            const int ti = job < 1 ? 1 : (job < 3 ? 2 : 3);
            const int tj = job < 1 ? 0 : (job < 3 ? job - 1 : job - 3);
            ja = 16 * ti + r; jbr = 16 * tj + r; ea = eb = 16 * tj + 15;
        } else {
            const int t = 2 * (job - 6) + (r >> 3);      // the diagonal tile this lane's operand rows belong to
            ja = 16 * t + 8 + (r & 7); jbr = 16 * t + (r & 7); ea = eb = 16 * t + 7;
        }
    };
    float pkk = 0.f, pqk = 0.f, pdg = 0.f;
    int pi = 0, pj = 0;
    if (tid < 224) {                                 // 8 blocks x 28 pairs with j < i
        const int b8 = tid / 28, p = tid % 28;
        int ii = 1;
        while ((ii * (ii + 1)) / 2 <= p) ++ii;       // ii (ii - 1) / 2 <= p < ii (ii + 1) / 2
        pi = 8 * b8 + ii; pj = 8 * b8 + p - (ii * (ii - 1)) / 2;
    }

    float ksq[64 * PPH / 256];                       // this thread's share of ||k_row||^2, rows (tid + 256 it) / PPH
#pragma unroll
    for (int it = 0; it < 64 * PPH / 256; ++it) ksq[it] = 0.f;
    // A pass's rows of K, Q and log alpha come from memory into registers (fetch) and go on into the tables once the
    // pass before has read them; the fetch of the next pass is issued ahead of the last, long, lightly loaded phase of
    // a pass, so that a workgroup waits for memory once, not once per pass.
    constexpr int NKQ = 64 * PPH / 256, NLA = 64 * CH / 4 / 256;
    uint4 kd[NKQ], qd[NKQ];
    float4 lad[NLA];
    auto fetch = [&](int c0) {
#pragma unroll
        for (int it = 0; it < NKQ; ++it) {
            const int x = tid + 256 * it;
            const int row = x / PPH, piece = x % PPH;
            kd[it] = make_uint4(0, 0, 0, 0); qd[it] = make_uint4(0, 0, 0, 0);
            if (row < clen) {
                kd[it] = *reinterpret_cast<const uint4*>(kb + (size_t)row * row_stride + c0 + piece * EPP);
                qd[it] = *reinterpret_cast<const uint4*>(qb + (size_t)row * row_stride + c0 + piece * EPP);
            }
        }
#pragma unroll
        for (int it = 0; it < NLA; ++it) {
            const int x = tid + 256 * it, row = x / (CH / 4), c4 = x % (CH / 4);
            lad[it] = make_float4(0.f, 0.f, 0.f, 0.f);
            if (row < clen) lad[it] = *reinterpret_cast<const float4*>(lb + (size_t)row * row_stride + c0 + 4 * c4);
        }
    };
    constexpr bool AHEAD = sizeof(E) == 2;           // fp32 rows are twice the registers: fetched pass by pass
    if constexpr (AHEAD) fetch(0);
    for (int pass = 0; pass < NPASS; ++pass) {
        const int c0 = pass * CH;                    // first channel of this pass
        if (pass > 0) __syncthreads();               // the previous pass has read its tables
        if constexpr (!AHEAD) fetch(c0);
        // ---- phase 1: K, Q rows and log2 alpha of CH channels -> LDS (the squares of K summed for the key norms on the way)
#pragma unroll
        for (int it = 0; it < NKQ; ++it) {
            const int x = tid + 256 * it;
            const int row = x / PPH, piece = x % PPH;
            *reinterpret_cast<uint4*>(area + (size_t)(row * LE + piece * EPP) * sizeof(E)) = kd[it];
            *reinterpret_cast<uint4*>(area + TE + (size_t)(row * LE + piece * EPP) * sizeof(E)) = qd[it];
            float kf[EPP];
            unpack(kd[it], kf);
#pragma unroll
            for (int i = 0; i < EPP; ++i) ksq[it] += kf[i] * kf[i];
        }
#pragma unroll
        for (int it = 0; it < NLA; ++it) {
            const int x = tid + 256 * it, row = x / (CH / 4), c4 = x % (CH / 4);
            const float4 v = lad[it];
            const float s2 = 1.44269504088896341f;
            *reinterpret_cast<float4*>(Gs + row * LD + 4 * c4) = make_float4(v.x * s2, v.y * s2, v.z * s2, v.w * s2);
        }
        __syncthreads();
        {   // per channel: running sum over the tokens of the chunk, NSEG row segments side by side, then their offsets
            const int c = tid % CH, sg = tid / CH;
            float acc = 0.f;
            for (int i = sg * SROWS; i < (sg + 1) * SROWS; ++i) { acc += Gs[i * LD + c]; Gs[i * LD + c] = acc; }
            segsum[sg][c] = acc;
            __syncthreads();
            float base = 0.f;
            for (int s2 = 0; s2 < sg; ++s2) base += segsum[s2][c];
            if (sg > 0)
                for (int i = sg * SROWS; i < (sg + 1) * SROWS; ++i) Gs[i * LD + c] += base;
            if (sg == NSEG - 1) a.gc[(size_t)blockIdx.x * DK + c0 + c] = __builtin_amdgcn_exp2f(base + acc);      // gamma_C
        }
        __syncthreads();

        // ---- phase 1b: the scan's operands K+, Q+, K~ in the element type -------------------------------------
        {
            E* kpo = a.kplus + (size_t)tok0 * row_stride + (size_t)h * DK + c0;
            E* qpo = a.qplus + (size_t)tok0 * row_stride + (size_t)h * DK + c0;
            E* kto = a.ktilde + (size_t)tok0 * row_stride + (size_t)h * DK + c0;
#pragma unroll
            for (int it = 0; it < 64 * PPH / 256; ++it) {
                const int x = tid + 256 * it;
                const int row = x / PPH, piece = x % PPH;
                if (row < clen) {
                    float kf[EPP], qf[EPP], kp[EPP], qp[EPP], kt[EPP];
                    unpack(*reinterpret_cast<const uint4*>(area + (size_t)(row * LE + piece * EPP) * sizeof(E)), kf);
                    unpack(*reinterpret_cast<const uint4*>(area + TE + (size_t)(row * LE + piece * EPP) * sizeof(E)), qf);
#pragma unroll
                    for (int i = 0; i < EPP; ++i) {
                        const float gi = Gs[row * LD + piece * EPP + i], gl = Gs[63 * LD + piece * EPP + i];
                        const float up = __builtin_amdgcn_exp2f(gi);
                        kp[i] = kf[i] * up; qp[i] = qf[i] * (up * rq_s[row]); kt[i] = kf[i] * __builtin_amdgcn_exp2f(gl - gi);
                    }
                    const size_t off = (size_t)row * row_stride + piece * EPP;
                    typedef uint32_t u32x4n __attribute__((ext_vector_type(4)));
                    auto nts = [](E* p, uint4 v) { const u32x4n w = {v.x, v.y, v.z, v.w}; __builtin_nontemporal_store(w, reinterpret_cast<u32x4n*>(p)); };
                    nts(kpo + off, pack(kp));
                    nts(qpo + off, pack(qp));
                    nts(kto + off, pack(kt));
                }
            }
        }
        // (no barrier: phase 2a only reads the tables, like phase 1b)

        // ---- phase 2a: K K^T and Q K^T with the decay ratios inside the sums, the channels of this pass ---------
        // (1) MFMA jobs, operands formed in registers from the tables: the six off-diagonal 16x16 tiles (ti > tj), split at
        //     e = last row of tile tj, A row i = k_i (or q_i) o gamma_i/gamma_e, B row j = k_j o gamma_e/gamma_j; and of
        //     each diagonal tile the lower-left 8x8 block, split at e = row 7 of the tile, the other rows of both operands
        //     zero.  Every factor is <= 1.  Jobs 0..9 go to wave (job % 4).
        // (2) the 8x8 blocks on the diagonal, one (i, j) pair per thread over all channels: gamma_i/gamma_j <= 1 directly.
#pragma unroll
        for (int jb = 0; jb < 2; ++jb) {
            const int job = wave + 4 * jb;
            int ja, jbr, ea, eb;
            job_rows(job, ja, jbr, ea, eb);
            const float* gi = Gs + ja * LD;
            const float* gj = Gs + jbr * LD;
            const float* gea = Gs + ea * LD;
            const float* geb = Gs + eb * LD;
            const E* ki = Kp + ja * LE;
            const E* qi = Qp + ja * LE;
            const E* kj = Kp + jbr * LE;
            for (int kp = 0; kp < CH / 32; ++kp) {
                floatx4 ka[2], qa[2], kbv[2];
#pragma unroll
                for (int blk = 0; blk < 2; ++blk) {
                    const int c = 32 * kp + 16 * blk + 4 * g;
                    const floatx4 geav = ld4f(gea + c), gebv = ld4f(geb + c), giv = ld4f(gi + c), gjv = ld4f(gj + c);
                    const floatx4 kiv = ld4e(ki + c), qiv = ld4e(qi + c), kjv = ld4e(kj + c);
#pragma unroll
                    for (int x = 0; x < 4; ++x) {
                        const float up = __builtin_amdgcn_exp2f(giv[x] - geav[x]);      // gamma_i / gamma_e <= 1
                        const float dn = __builtin_amdgcn_exp2f(gebv[x] - gjv[x]);      // gamma_e / gamma_j <= 1
                        ka[blk][x] = kiv[x] * up; qa[blk][x] = qiv[x] * up; kbv[blk][x] = kjv[x] * dn;
                    }
                }
                Slot<E> sk, sq;
                sk.q0 = acc_to_quad<E>(ka[0]); sk.q1 = acc_to_quad<E>(ka[1]);
                sq.q0 = acc_to_quad<E>(qa[0]); sq.q1 = acc_to_quad<E>(qa[1]);
                const typename QuadT<E>::type b0 = acc_to_quad<E>(kbv[0]), b1 = acc_to_quad<E>(kbv[1]);
                mma32<E>(tkk[jb], sk, b0, b1);
                mma32<E>(tqk[jb], sq, b0, b1);
            }
        }
        if constexpr (AHEAD) { if (pass + 1 < NPASS) fetch(c0 + CH); }   // on their way during the pair sums
        if (tid < 224) {
            const float* gi = Gs + pi * LD; const float* gj = Gs + pj * LD;
            const E* ki = Kp + pi * LE; const E* qi = Qp + pi * LE; const E* kj = Kp + pj * LE;
#pragma unroll 2
            for (int c = 0; c < CH; c += 4) {
                const floatx4 giv = ld4f(gi + c), gjv = ld4f(gj + c);
                const floatx4 kiv = ld4e(ki + c), qiv = ld4e(qi + c), kjv = ld4e(kj + c);
#pragma unroll
                for (int x = 0; x < 4; ++x) {
                    const float w = kjv[x] * __builtin_amdgcn_exp2f(giv[x] - gjv[x]);
                    pkk += kiv[x] * w; pqk += qiv[x] * w;
                }
            }
        }
        if (tid < 64) {                                  // P_ii = q_i . k_i
            const E* ki = Kp + tid * LE; const E* qi = Qp + tid * LE;
            for (int c = 0; c < CH; c += 4) {
                const floatx4 kiv = ld4e(ki + c), qiv = ld4e(qi + c);
#pragma unroll
                for (int x = 0; x < 4; ++x) pdg += qiv[x] * kiv[x];
            }
        }
    }
    // ---- beta of eq. (3) from the key norms (the PPH threads of a row sit in consecutive lanes)
#pragma unroll
    for (int it = 0; it < 64 * PPH / 256; ++it) {
        const int x = tid + 256 * it;
        const int row = x / PPH;
        float ss = ksq[it];
#pragma unroll
        for (int off = 1; off < PPH; off <<= 1) ss += __shfl_xor(ss, off, kWave);
        if (x % PPH == 0) {
            const float et = row < clen ? a.eta[(size_t)(tok0 + row) * a.H + h] : 0.f;
            beta_s[row] = (a.opts & kOptGdnBeta) ? et : kaczmarz_beta(et, ss, a.eps);
        }
    }
    __syncthreads();   // the tables are dead from here on; Lm, Pm, Tm overlay them

    // ---- phase 2b: beta -> L and P, everything else zero ---------------------------------------------------------
    for (int x = tid; x < 64 * 64; x += 256) {
        const int i = x >> 6, j = x & 63;
        Lm[i * kLdm + j] = 0.f; Pm[i * kLdm + j] = 0.f; Tm[i * kLdm + j] = 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int jb = 0; jb < 2; ++jb) {
        const int job = wave + 4 * jb;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int il = 4 * g + e;                // row inside the product tile; its column is r
            int i, j; bool ok;
            if (job < 6) {
                const int ti = job < 1 ? 1 : (job < 3 ? 2 : 3);
                const int tj = job < 1 ? 0 : (job < 3 ? job - 1 : job - 3);
                i = 16 * ti + il; j = 16 * tj + r; ok = true;
            } else {                                 // the two diagonal 8x8 blocks of the product
                const int t = 2 * (job - 6) + (il >> 3);
                i = 16 * t + 8 + (il & 7); j = 16 * t + (r & 7); ok = (il >> 3) == (r >> 3);
            }
            if (ok) {
                Lm[i * kLdm + j] = beta_s[i] * tkk[jb][e];
                Pm[i * kLdm + j] = tqk[jb][e] * rq_s[i];
            }
        }
    }
    if (tid < 224) { Lm[pi * kLdm + pj] = beta_s[pi] * pkk; Pm[pi * kLdm + pj] = pqk * rq_s[pi]; }
    if (tid < 64) Pm[tid * kLdm + tid] = pdg * rq_s[tid];
    __syncthreads();
    invert_and_store<E, false>(Lm, Tm, Pm, beta_s, reinterpret_cast<char*>(a.wsT) + (size_t)blockIdx.x * REC, tid);
}

template <typename E>
hipError_t launch_intra_diag(const IntraDiagArgs<E>& a, int dk, int n_chunks, hipStream_t st)
{
    if (n_chunks == 0) return hipSuccess;
    const dim3 grid((unsigned)n_chunks * a.H), block(256);
    if (dk == 64) hipLaunchKernelGGL((intra_diag_kernel<E, 64>), grid, block, 0, st, a);
    else          hipLaunchKernelGGL((intra_diag_kernel<E, 128>), grid, block, 0, st, a);
    return hipGetLastError();
}
template hipError_t launch_intra_diag<float>(const IntraDiagArgs<float>&, int, int, hipStream_t);
template hipError_t launch_intra_diag<bf16_t>(const IntraDiagArgs<bf16_t>&, int, int, hipStream_t);

// ---- chunk offsets of a packed batch: chunk_off[s] = sum_{s'<s} ceil(len_s'/64) --------------
__global__ void chunk_offsets_kernel(const int* __restrict__ cu_seqlens, int n_seq, int* __restrict__ chunk_off)
{
    if (threadIdx.x == 0 && blockIdx.x == 0) {
        int acc = 0;
        for (int s = 0; s < n_seq; ++s) {
            chunk_off[s] = acc;
            acc += (cu_seqlens[s + 1] - cu_seqlens[s] + 63) / 64;
        }
        chunk_off[n_seq] = acc;
    }
}
hipError_t launch_chunk_offsets(const int* cu_seqlens, int n_seq, int* chunk_off, hipStream_t st)
{
    hipLaunchKernelGGL(chunk_offsets_kernel, dim3(1), dim3(64), 0, st, cu_seqlens, n_seq, chunk_off);
    return hipGetLastError();
}

// ---- test hook: unpack operand-order T', P to plain row-major fp32 ---------------------------
template <typename E>
__global__ void unpack_kernel(const E* __restrict__ wsT, const E* __restrict__ wsP, const float* __restrict__ wsG,
                              float* __restrict__ Tb, float* __restrict__ P, float* __restrict__ gout, long n_ch)
{
    const long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= n_ch * 4096) return;
    const long ch = idx >> 12;
    const int i = (int)((idx >> 6) & 63), j = (int)(idx & 63);
    const int ti = i >> 4, jp = j >> 5, ln = (i & 15) + 16 * ((j & 15) >> 2);
    const bool stored = jp <= (ti >> 1);             // only the lower-triangular tile-pairs exist
    const size_t e = (size_t)ch * (ws_record_bytes<E>() / sizeof(E)) + ((size_t)tri_pair(ti, jp) * 64 + ln) * 8 + ((j >> 4) & 1) * 4 + (j & 3);
    Tb[idx] = stored ? to_float(wsT[e]) : 0.f;
    P[idx] = stored ? to_float(wsP[e]) : 0.f;
    if (j == 0) gout[ch * 64 + i] = wsG[ch * 128 + i];
}
template <typename E>
hipError_t launch_unpack(const E* wsT, const E* wsP, const float* wsG, float* Tb, float* P, float* gout, long n_ch,
                         hipStream_t st)
{
    if (n_ch == 0) return hipSuccess;
    const long n = n_ch * 4096;
    hipLaunchKernelGGL((unpack_kernel<E>), dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, wsT, wsP, wsG, Tb, P,
                       gout, n_ch);
    return hipGetLastError();
}
template hipError_t launch_unpack<float>(const float*, const float*, const float*, float*, float*, float*, long, hipStream_t);
template hipError_t launch_unpack<bf16_t>(const bf16_t*, const bf16_t*, const float*, float*, float*, float*, long, hipStream_t);

}  // namespace kla
