// Decode step (Algorithm 1, left panel) and the stand-alone Kaczmarz coefficient (eq. (3)).
//
// Decode is pure state streaming: per (batch, head) the fp32 state S [dk, dv] is read once and
// written once (0.87 flop per byte), so the kernel is laid out for HBM: every lane owns float4
// columns of a few rows, issues all of its 128-bit loads before anything else, and the two
// reductions over d_k that the step needs (p = S^T k and r = S^T q) are taken from the same
// registers.  The read-out uses o = S_new^T q = alpha r + beta (k.q) e, which avoids a second pass.
#include "kla_common.hpp"
#include "kla_kernels.hpp"

namespace kla {

// One block = one (batch, head) and a slice of DVS state columns.
//   LPR lanes cover one row of the slice (4 columns each); the 256 threads cover RPP rows per pass.
// DIAG: diagonal gating (App. B): log_alpha holds d_k values per (batch, head) and row i of the state decays by
// exp(log_alpha[i]); the decay is folded into the copies of k and q that the two column sums use.
template <typename T, int DK, int DVS, int NT, bool DIAG>
__global__ __launch_bounds__(256) void decode_kernel(const T* __restrict__ q, const T* __restrict__ k,
                                                     const T* __restrict__ v,
                                                     const float* __restrict__ log_alpha,
                                                     const float* __restrict__ eta, float eps,
                                                     float* __restrict__ S, T* __restrict__ o, int dv,
                                                     unsigned opts)
{
    constexpr int LPR = DVS / 4;
    constexpr int RPP = 256 / LPR;
    constexpr int NP = DK / RPP;
    static_assert(LPR <= 64 && NP >= 1 && DK % RPP == 0, "slice shape");

    const int bh = blockIdx.x;
    const int tid = threadIdx.x;
    const int cl = tid % LPR;
    const int r0 = tid / LPR;
    const int col = blockIdx.y * DVS + cl * 4;

    // Every global load of the step is issued here, the small ones first: loads return in order, so
    // nothing small may queue behind the state, and nothing is fetched after a barrier.
    float kv = 0.f, qv = 0.f;
    if (tid < DK) {
        kv = to_float(k[(size_t)bh * DK + tid]);
        qv = to_float(q[(size_t)bh * DK + tid]);
    }
    float la;
    if constexpr (DIAG) la = tid < DK ? log_alpha[(size_t)bh * DK + tid] : 0.f;
    else                la = log_alpha[bh];
    const float et = eta[bh];
    float vv[4];
    {
        const T* vb = v + (size_t)bh * dv + col;
#pragma unroll
        for (int i = 0; i < 4; ++i) vv[i] = to_float(vb[i]);
    }
    float* Sb = S + (size_t)bh * DK * dv + col;
    float4 s[NP];
#pragma unroll
    for (int p = 0; p < NP; ++p) {
        typedef float f4v __attribute__((ext_vector_type(4)));
        const f4v* sp = reinterpret_cast<const f4v*>(Sb + (size_t)(r0 + p * RPP) * dv);
        f4v t;
        if constexpr ((NT & 1) != 0) t = __builtin_nontemporal_load(sp); else t = *sp;
        s[p] = make_float4(t.x, t.y, t.z, t.w);
    }

    __shared__ float ks[DK], qs[DK];
    __shared__ float ka[DIAG ? DK : 1], qa[DIAG ? DK : 1], al[DIAG ? DK : 1];     // alpha_i k_i, alpha_i q_i, alpha_i
    __shared__ float red[4][3];
    __shared__ float part[4][LPR][8];

    if (tid < DK) {
        ks[tid] = kv;
        qs[tid] = qv;
        if constexpr (DIAG) { const float ai = expf(la); al[tid] = ai; ka[tid] = ai * kv; qa[tid] = ai * qv; }
    }
    const float kk = wave_sum(kv * kv);
    const float kq = wave_sum(kv * qv);
    const float qq = wave_sum(qv * qv);
    const int wave = tid / kWave, lane = tid % kWave;
    if (lane == 0) { red[wave][0] = kk; red[wave][1] = kq; red[wave][2] = qq; }
    __syncthreads();
    const float knorm2 = red[0][0] + red[1][0] + red[2][0] + red[3][0];
    const float kdotq = red[0][1] + red[1][1] + red[2][1] + red[3][1];
    const float alpha = DIAG ? 1.f : expf(la);       // diagonal gating: the decay sits in ka, qa and al instead
    const float beta = (opts & kOptGdnBeta) ? et : kaczmarz_beta(et, knorm2, eps);
    // read-out scale: 1, or 1/||q|| (0 for a zero query) for the normalised read-out of Sec. 3.3
    float oscale = 1.f;
    if (opts & kOptNormalizeQ) {
        const float qnorm2 = red[0][2] + red[1][2] + red[2][2] + red[3][2];
        oscale = qnorm2 > 0.f ? 1.0f / sqrtf(qnorm2) : 0.f;
    }

    float pr[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};   // p[0..3], r[0..3] for this lane's 4 columns
#pragma unroll
    for (int p = 0; p < NP; ++p) {
        const float kr = DIAG ? ka[r0 + p * RPP] : ks[r0 + p * RPP], qr = DIAG ? qa[r0 + p * RPP] : qs[r0 + p * RPP];
        pr[0] += s[p].x * kr; pr[1] += s[p].y * kr; pr[2] += s[p].z * kr; pr[3] += s[p].w * kr;
        pr[4] += s[p].x * qr; pr[5] += s[p].y * qr; pr[6] += s[p].z * qr; pr[7] += s[p].w * qr;
    }
    // sum over the row groups that share this lane's columns: first inside the wave ...
#pragma unroll
    for (int off = LPR; off < kWave; off <<= 1)
#pragma unroll
        for (int i = 0; i < 8; ++i) pr[i] += __shfl_xor(pr[i], off, kWave);
    // ... then across the four waves, in a fixed order (deterministic)
    if (lane < LPR)
#pragma unroll
        for (int i = 0; i < 8; ++i) part[wave][lane][i] = pr[i];
    __syncthreads();
#pragma unroll
    for (int i = 0; i < 8; ++i) pr[i] = part[0][cl][i] + part[1][cl][i] + part[2][cl][i] + part[3][cl][i];

    float e[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) e[i] = vv[i] - alpha * pr[i];   // e = v - (alpha S)^T k
#pragma unroll
    for (int p = 0; p < NP; ++p) {
        const float bk = beta * ks[r0 + p * RPP];
        const float ar = DIAG ? al[r0 + p * RPP] : alpha;
        float4 n;
        n.x = ar * s[p].x + bk * e[0];
        n.y = ar * s[p].y + bk * e[1];
        n.z = ar * s[p].z + bk * e[2];
        n.w = ar * s[p].w + bk * e[3];
        typedef float f4v __attribute__((ext_vector_type(4)));
        const f4v t = {n.x, n.y, n.z, n.w};
        f4v* dp = reinterpret_cast<f4v*>(Sb + (size_t)(r0 + p * RPP) * dv);
        if constexpr ((NT & 2) != 0) __builtin_nontemporal_store(t, dp); else *dp = t;
    }
    if (r0 == 0) {
        T* ob = o + (size_t)bh * dv + col;
        const float bkq = beta * kdotq;
#pragma unroll
        for (int i = 0; i < 4; ++i) ob[i] = from_float<T>(oscale * (alpha * pr[4 + i] + bkq * e[i]));
    }
}

template <typename T, int DK, int NT>
static hipError_t launch_decode_nt(const T* q, const T* k, const T* v, const float* la, const float* eta,
                                   float eps, float* S, T* o, int BH, int dv, int slice, unsigned opts, hipStream_t st)
{
    dim3 grid(BH, dv / slice), block(256);
    if (opts & kOptDiagDecay) {                      // diagonal gating: one slice shape
        hipLaunchKernelGGL((decode_kernel<T, DK, 64, NT, true>), dim3(BH, dv / 64), block, 0, st, q, k, v, la, eta, eps, S, o, dv,
                           opts & (kOptNormalizeQ | kOptGdnBeta));
        return hipGetLastError();
    }
    switch (slice) {
        case 32:  hipLaunchKernelGGL((decode_kernel<T, DK, 32, NT, false>), grid, block, 0, st, q, k, v, la, eta, eps, S, o, dv, opts); break;
        case 64:  hipLaunchKernelGGL((decode_kernel<T, DK, 64, NT, false>), grid, block, 0, st, q, k, v, la, eta, eps, S, o, dv, opts); break;
        case 128: hipLaunchKernelGGL((decode_kernel<T, DK, 128, NT, false>), grid, block, 0, st, q, k, v, la, eta, eps, S, o, dv, opts); break;
        default:  hipLaunchKernelGGL((decode_kernel<T, DK, 256, NT, false>), grid, block, 0, st, q, k, v, la, eta, eps, S, o, dv, opts); break;
    }
    return hipGetLastError();
}

// Cache policy of the state accesses.  A state set that cannot stay in the 256 MB Infinity Cache between
// two steps (large batch, or many layers taking turns) is streamed with non-temporal loads and stores:
// measured 12.7 us instead of 16.8 us per 67 MB step.  A small one is left cacheable (8.7 us when it is
// resident).  nt_force = 0..3 overrides (bit 0: loads, bit 1: stores); -1 = this rule.
template <typename T, int DK>
static hipError_t launch_decode_dk(const T* q, const T* k, const T* v, const float* la, const float* eta,
                                   float eps, float* S, T* o, int BH, int dv, int slice, int nt_force, unsigned opts, hipStream_t st)
{
    int nt = ((size_t)BH * DK * dv * sizeof(float) >= ((size_t)16 << 20)) ? 3 : 0;
    if (nt_force >= 0 && nt_force <= 3) nt = nt_force;
    switch (nt) {
        case 0:  return launch_decode_nt<T, DK, 0>(q, k, v, la, eta, eps, S, o, BH, dv, slice, opts, st);
        case 1:  return launch_decode_nt<T, DK, 1>(q, k, v, la, eta, eps, S, o, BH, dv, slice, opts, st);
        case 2:  return launch_decode_nt<T, DK, 2>(q, k, v, la, eta, eps, S, o, BH, dv, slice, opts, st);
        default: return launch_decode_nt<T, DK, 3>(q, k, v, la, eta, eps, S, o, BH, dv, slice, opts, st);
    }
}

template <typename T>
hipError_t launch_decode(const T* q, const T* k, const T* v, const float* la, const float* eta, float eps,
                         float* S, T* o, int BH, int dk, int dv, int slice, int nt_force, unsigned opts, hipStream_t st)
{
    if (dk == 64) return launch_decode_dk<T, 64>(q, k, v, la, eta, eps, S, o, BH, dv, slice, nt_force, opts, st);
    return launch_decode_dk<T, 128>(q, k, v, la, eta, eps, S, o, BH, dv, slice, nt_force, opts, st);
}
template hipError_t launch_decode<float>(const float*, const float*, const float*, const float*, const float*,
                                         float, float*, float*, int, int, int, int, int, unsigned, hipStream_t);
template hipError_t launch_decode<bf16_t>(const bf16_t*, const bf16_t*, const bf16_t*, const float*, const float*,
                                          float, float*, bf16_t*, int, int, int, int, int, unsigned, hipStream_t);

// eq. (3) alone: one group of DK/8 lanes per row, each lane squares 8 consecutive elements.
template <typename T, int DK>
__global__ __launch_bounds__(256) void beta_kernel(const T* __restrict__ k, const float* __restrict__ eta,
                                                   float eps, float* __restrict__ beta, long n_rows)
{
    constexpr int LPR = DK / 8;
    const long row = ((long)blockIdx.x * 256 + threadIdx.x) / LPR;
    const int piece = threadIdx.x % LPR;
    float acc = 0.f;
    if (row < n_rows) {
        const T* p = k + row * DK + piece * 8;
#pragma unroll
        for (int i = 0; i < 8; ++i) { const float x = to_float(p[i]); acc += x * x; }
    }
#pragma unroll
    for (int off = 1; off < LPR; off <<= 1) acc += __shfl_xor(acc, off, kWave);
    if (row < n_rows && piece == 0) beta[row] = kaczmarz_beta(eta[row], acc, eps);
}

template <typename T>
hipError_t launch_beta(const T* k, const float* eta, float eps, float* beta, long n_rows, int dk, hipStream_t st)
{
    if (n_rows == 0) return hipSuccess;
    const int lpr = dk / 8;
    const long rows_per_block = 256 / lpr;
    const unsigned blocks = (unsigned)((n_rows + rows_per_block - 1) / rows_per_block);
    if (dk == 64) hipLaunchKernelGGL((beta_kernel<T, 64>), dim3(blocks), dim3(256), 0, st, k, eta, eps, beta, n_rows);
    else          hipLaunchKernelGGL((beta_kernel<T, 128>), dim3(blocks), dim3(256), 0, st, k, eta, eps, beta, n_rows);
    return hipGetLastError();
}
template hipError_t launch_beta<float>(const float*, const float*, float, float*, long, int, hipStream_t);
template hipError_t launch_beta<bf16_t>(const bf16_t*, const float*, float, float*, long, int, hipStream_t);

}  // namespace kla
