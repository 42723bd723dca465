// Backward pass of the chunkwise form: gradients of  sum <d_o, o> + sum <d_hT, hT>  with respect to q, k, v,
// log_alpha, eta and h0.  The paper states the forward map only (Algorithm 1; eqs. (6)-(8)); what follows is
// those equations differentiated per chunk, including the dependence of beta on k through eq. (3).
//
// Per chunk, with M = (I + L)^{-1}, B = diag(beta), X = V - D_gamma K S (S the incoming state), U = M B X = T' X,
// P = A o Q K^T, and dS' the gradient of the state the chunk hands on:
//     dU = P^T dO + diag(gamma_C/gamma_i) K dS'        Y = M^T dU        dV = dX = B Y
//     dS = gamma_C dS' + Q^T D_gamma dO - K^T D_gamma dX                          (gradient of the incoming state)
//     dP = tril(dO U^T)       D' = -A^- o (Y U^T)      dbeta_i = Y_i.X_i + (D' K)_i.k_i
//     dQ = D_gamma dO S^T + (A o dP) K
//     dK = [ -D_gamma dX S^T + B D' K ] + [ diag(gamma_C/gamma_i) U dS'^T + (A o dP)^T Q + (B D')^T K ]
//          - 2 beta dbeta / (|k|^2 + eps) k
//     dg_i = q_i.dQ_i + k_i.[first bracket]_i - k_i.[second bracket]_i,   dg_C += <dS', S'>   (S' the outgoing state)
//     dlog_alpha_r = sum_{i >= r in the chunk} dg_i,        deta_i = dbeta_i / (|k_i|^2 + eps)
// (g_i multiplies q_i and the k_i that reads the state, and divides the k_i that writes to it; hence the signs.)
//
// Three kernels after the intra-chunk stage has left [T' | M^T | P^T | gamma_i | gamma_C/gamma_i | beta_i | 1/(|k_i|^2+eps)]
// (T' = M B, so U = T' X):
//   bwd_states_kernel    forward over the chunks of a (sequence, head, column slice): S_c, X, U        -> workspace
//   bwd_scan_kernel      backward over the same chunks: dS'_c, Y -> workspace, dv and dh0 -> outputs
//   bwd_assemble_kernel  per chunk-head: the contractions over d_v and over the chunk -> dq, dk, dlog_alpha, deta
// The two sweeps treat state columns independently (as the forward does); everything that contracts over d_v is
// left to the third kernel, so no atomics are needed and the result is run-to-run deterministic.
#include "kla_common.hpp"
#include "kla_kernels.hpp"
#include "kla_mma.hpp"

namespace kla {

namespace {

__device__ __forceinline__ floatx4 ld_acc4(const float* p)
{
    const float4 f = *reinterpret_cast<const float4*>(p);
    floatx4 x; x[0] = f.x; x[1] = f.y; x[2] = f.z; x[3] = f.w; return x;
}

template <typename E, int DK, int NW>
struct SweepCfg {
    static constexpr int NTH = 64 * NW;
    static constexpr int KB = DK / 16, KP = DK / 32;
    static constexpr int SLW = 16 * NW;                         // state columns per workgroup
    static constexpr int PPR = DK * (int)sizeof(E) / 16;        // 16-byte pieces per K/Q row
    static constexpr int EPP = 16 / (int)sizeof(E);             // elements per piece
    static constexpr int VPP = SLW * (int)sizeof(E) / 16;       // pieces per row of a [tokens, d_v] slice
    static constexpr int SB = 2 * (int)sizeof(typename QuadT<E>::type);
    static constexpr int OPB = 64 * DK * (int)sizeof(E);        // one K/Q operand area
    static constexpr int TPB = kTriPairs * 64 * SB;             // one triangular operand area
    static constexpr int VB = NW * 2 * 64 * SB;                 // one [tokens, slice] area
    static constexpr int UK = (16 * PPR + NTH - 1) / NTH;       // (4-row group, piece) units of K/Q per thread
    static constexpr int UV = (16 * VPP + NTH - 1) / NTH;
    static constexpr int TP16 = TPB / 16;
    static constexpr int UT = (TP16 + NTH - 1) / NTH;
};

// which (sequence, head, column slice) a workgroup of a sweep works on; the same XCD-aware numbering as the forward
struct SweepPos { int chain, slice, h, nch, ch0; long t0; int len; bool valid; };
template <typename E>
__device__ __forceinline__ SweepPos sweep_pos(const BwdArgs<E>& a, int SLW)
{
    SweepPos p;
    const int nsl = a.dv_dim / SLW;
    const int n_states = a.n_seq > 0 ? a.n_seq : a.N;
    const int xcd = blockIdx.x & 7, pidx = blockIdx.x >> 3;
    p.chain = (pidx / nsl) * 8 + xcd; p.slice = pidx % nsl;
    p.valid = p.chain < n_states * a.H;
    const int s = p.valid ? p.chain / a.H : 0;
    p.h = p.chain % a.H;
    if (a.cu_seqlens) { p.t0 = a.cu_seqlens[s]; p.len = a.cu_seqlens[s + 1] - (int)p.t0; p.ch0 = a.chunk_off[s]; }
    else              { p.t0 = (long)s * a.T;   p.len = a.T;                               p.ch0 = s * a.NT; }
    p.nch = (p.len + 63) / 64;
    return p;
}

// accumulator tile (rows 16 it + 4 g + e, column col) -> a [tokens, H, d_v] tensor, rows below clen only
template <typename E>
__device__ __forceinline__ void store_rows(E* base, size_t v_stride, floatx4 x, int it, int g, int clen)
{
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const int row = 16 * it + 4 * g + e;
        if (row < clen) base[(size_t)row * v_stride] = from_float<E>(x[e]);
    }
}

}  // namespace

// =================================================================================================
// forward sweep: incoming state of every chunk, X and U
// =================================================================================================
template <typename E, int DK, int NW>
__global__ __launch_bounds__(64 * NW) void bwd_states_kernel(BwdArgs<E> a)
{
    typedef SweepCfg<E, DK, NW> C;
    constexpr int NTH = C::NTH, KB = C::KB, KP = C::KP, SLW = C::SLW, PPR = C::PPR, EPP = C::EPP, VPP = C::VPP;
    typedef typename QuadT<E>::type Quad;
    // K rows | K transposed | T' | V slice | gamma_i | gamma_C/gamma_i | beta_i
    constexpr int OFF_KT = C::OPB, OFF_T = 2 * C::OPB, OFF_V = OFF_T + C::TPB, OFF_VEC = OFF_V + C::VB, LDS = OFF_VEC + 768;
    __shared__ __attribute__((aligned(16))) char lds[LDS];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int r = lane & 15, g = lane >> 4;
    const SweepPos p = sweep_pos(a, SLW);
    if (!p.valid) return;
    const int h = p.h, col = p.slice * SLW + 16 * wave + r;
    const size_t kq_stride = (size_t)a.H * DK, v_stride = (size_t)a.H * a.dv_dim;

    floatx4 S[KB];
#pragma unroll
    for (int kt = 0; kt < KB; ++kt)
#pragma unroll
        for (int e = 0; e < 4; ++e)
            S[kt][e] = a.h0 ? a.h0[((size_t)p.chain * DK + 16 * kt + 4 * g + e) * a.dv_dim + col] : 0.f;

    uint4 pk[C::UK][4], pv[C::UV][4], pm[C::UT];
    float pvec[3];
    auto fetch = [&](int c) {
        const long tok0 = p.t0 + 64L * c;
        const int clen = min(64, p.len - 64 * c);
        const char* rec = a.rec + ((size_t)(p.ch0 + c) * a.H + h) * bwd_record_bytes<E>();
        const E* kb = a.k + (size_t)tok0 * kq_stride + (size_t)h * DK;
        const E* vb = a.v + (size_t)tok0 * v_stride + (size_t)h * a.dv_dim + p.slice * SLW;
#pragma unroll
        for (int it = 0; it < C::UK; ++it) {
            const int u = tid + NTH * it, tq = u / PPR, piece = u % PPR;
#pragma unroll
            for (int rr = 0; rr < 4; ++rr) {
                pk[it][rr] = make_uint4(0, 0, 0, 0);
                if (((16 * PPR) % NTH == 0 || u < 16 * PPR) && 4 * tq + rr < clen)
                    pk[it][rr] = *reinterpret_cast<const uint4*>(kb + (size_t)(4 * tq + rr) * kq_stride + piece * EPP);
            }
        }
#pragma unroll
        for (int it = 0; it < C::UV; ++it) {
            const int u = tid + NTH * it, tq = u / VPP, pc = u % VPP;
#pragma unroll
            for (int rr = 0; rr < 4; ++rr) {
                pv[it][rr] = make_uint4(0, 0, 0, 0);
                if (((16 * VPP) % NTH == 0 || u < 16 * VPP) && 4 * tq + rr < clen)
                    pv[it][rr] = *reinterpret_cast<const uint4*>(vb + (size_t)(4 * tq + rr) * v_stride + pc * EPP);
            }
        }
        const uint4* msrc = reinterpret_cast<const uint4*>(rec);
#pragma unroll
        for (int it = 0; it < C::UT; ++it) {
            const int i = tid + NTH * it;
            pm[it] = make_uint4(0, 0, 0, 0);
            if (C::TP16 % NTH == 0 || i < C::TP16) pm[it] = msrc[i];
        }
        const float* vec = reinterpret_cast<const float*>(rec + 3 * ws_half_bytes<E>());
#pragma unroll
        for (int x = 0; x < 3; ++x) pvec[x] = vec[64 * x + lane];
    };
    auto stash = [&]() {
        E* Krq = reinterpret_cast<E*>(lds);
        E* Ktq = reinterpret_cast<E*>(lds + OFF_KT);
        E* Vtq = reinterpret_cast<E*>(lds + OFF_V);
#pragma unroll
        for (int it = 0; it < C::UK; ++it) {
            const int u = tid + NTH * it;
            if ((16 * PPR) % NTH == 0 || u < 16 * PPR) {
                const int tq = u / PPR, piece = u % PPR;
#pragma unroll
                for (int rr = 0; rr < 4; ++rr) store_rq_piece(Krq, KP, 4 * tq + rr, piece, pk[it][rr]);
                store_tq_rows(Ktq, 2, tq, piece, pk[it], 0);
            }
        }
#pragma unroll
        for (int it = 0; it < C::UV; ++it) {
            const int u = tid + NTH * it;
            if ((16 * VPP) % NTH == 0 || u < 16 * VPP) store_tq_rows(Vtq, 2, u / VPP, u % VPP, pv[it], 0);
        }
#pragma unroll
        for (int it = 0; it < C::UT; ++it) {
            const int i = tid + NTH * it;
            if (C::TP16 % NTH == 0 || i < C::TP16) reinterpret_cast<uint4*>(lds + OFF_T)[i] = pm[it];
        }
        if (tid < 64) {
#pragma unroll
            for (int x = 0; x < 3; ++x) reinterpret_cast<float*>(lds + OFF_VEC)[64 * x + tid] = pvec[x];
        }
    };

    if (p.nch > 0) fetch(0);
    for (int c = 0; c < p.nch; ++c) {
        const long tok0 = p.t0 + 64L * c;
        const int clen = min(64, p.len - 64 * c);
        __syncthreads();                                 // the previous chunk's operands are no longer read
        stash();
        __syncthreads();
        if (c + 1 < p.nch) fetch(c + 1);                 // in flight while this chunk's products run

        const E* Krq = reinterpret_cast<const E*>(lds);
        const E* Ktq = reinterpret_cast<const E*>(lds + OFF_KT);
        const E* Trq = reinterpret_cast<const E*>(lds + OFF_T);     // T' = (I + L)^{-1} B
        const E* Vtq = reinterpret_cast<const E*>(lds + OFF_V);
        const float* eg = reinterpret_cast<const float*>(lds + OFF_VEC);
        const float* ed = eg + 64;

        // the incoming state of this chunk, transposed: column `col` is a row of d_k elements
        E* sck = a.s_chk + (((size_t)(p.ch0 + c) * a.H + h) * a.dv_dim + col) * DK;
        Quad Sq[KB];
#pragma unroll
        for (int kt = 0; kt < KB; ++kt) {
            Sq[kt] = acc_to_quad<E>(S[kt]);
            *reinterpret_cast<Quad*>(sck + 16 * kt + 4 * g) = Sq[kt];
        }
        E* xb = a.X + (size_t)tok0 * v_stride + (size_t)h * a.dv_dim + col;
        E* ub = a.U + (size_t)tok0 * v_stride + (size_t)h * a.dv_dim + col;
        Quad Xq[4];
#pragma unroll
        for (int it = 0; it < 4; ++it) {
            floatx4 ks = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int kp = 0; kp < KP; ++kp) mma32<E>(ks, load_slot(Krq, it * KP + kp, lane), Sq[2 * kp], Sq[2 * kp + 1]);
            const Slot<E> sv = load_slot(Vtq, wave * 2 + (it >> 1), lane);
            const floatx4 x = quad_to_acc((it & 1) ? sv.q1 : sv.q0) - ld_acc4(eg + 16 * it + 4 * g) * ks;   // eq. (6), right side
            store_rows<E>(xb, v_stride, x, it, g, clen);
            Xq[it] = acc_to_quad<E>(x);
        }
        Quad Udq[4];
#pragma unroll
        for (int it = 0; it < 4; ++it) {
            floatx4 u = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int jp = 0; jp <= (it >> 1); ++jp) mma32<E>(u, load_slot(Trq, tri_pair(it, jp), lane), Xq[2 * jp], Xq[2 * jp + 1]);
            store_rows<E>(ub, v_stride, u, it, g, clen);
            Udq[it] = acc_to_quad<E>(u * ld_acc4(ed + 16 * it + 4 * g));
        }
        const float gC = eg[63];
#pragma unroll
        for (int kt = 0; kt < KB; ++kt) {                // eq. (8)
            S[kt] = S[kt] * gC;
#pragma unroll
            for (int jp = 0; jp < 2; ++jp) mma32<E>(S[kt], load_slot(Ktq, kt * 2 + jp, lane), Udq[2 * jp], Udq[2 * jp + 1]);
        }
    }
}

// =================================================================================================
// backward sweep: gradient of the state, Y, dv, dh0
// =================================================================================================
template <typename E, int DK, int NW>
__global__ __launch_bounds__(64 * NW) void bwd_scan_kernel(BwdArgs<E> a)
{
    typedef SweepCfg<E, DK, NW> C;
    constexpr int NTH = C::NTH, KB = C::KB, KP = C::KP, SLW = C::SLW, PPR = C::PPR, EPP = C::EPP, VPP = C::VPP;
    typedef typename QuadT<E>::type Quad;
    // K rows | K transposed | Q transposed | M^T | P^T | dO slice | gamma_i | gamma_C/gamma_i | beta_i
    constexpr int OFF_KT = C::OPB, OFF_QT = 2 * C::OPB, OFF_MT = 3 * C::OPB, OFF_PT = OFF_MT + C::TPB,
                  OFF_DO = OFF_PT + C::TPB, OFF_VEC = OFF_DO + C::VB, LDS = OFF_VEC + 1024;
    static_assert(LDS <= 160 * 1024, "LDS budget of a gfx950 CU");
    __shared__ __attribute__((aligned(16))) char lds[LDS];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int r = lane & 15, g = lane >> 4;
    const SweepPos p = sweep_pos(a, SLW);
    if (!p.valid) return;
    const int h = p.h, col = p.slice * SLW + 16 * wave + r;
    const size_t kq_stride = (size_t)a.H * DK, v_stride = (size_t)a.H * a.dv_dim;

    floatx4 dS[KB];
#pragma unroll
    for (int kt = 0; kt < KB; ++kt)
#pragma unroll
        for (int e = 0; e < 4; ++e)
            dS[kt][e] = a.d_hT ? a.d_hT[((size_t)p.chain * DK + 16 * kt + 4 * g + e) * a.dv_dim + col] : 0.f;

    uint4 pk[C::UK][4], pq[C::UK][4], pd[C::UV][4], pm[C::UT], pp[C::UT];
    float pvec[4];                                   // gamma_i | gamma_C/gamma_i | beta_i | 1/||q_i||
    auto fetch = [&](int c) {
        const long tok0 = p.t0 + 64L * c;
        const int clen = min(64, p.len - 64 * c);
        const char* rec = a.rec + ((size_t)(p.ch0 + c) * a.H + h) * bwd_record_bytes<E>();
        const E* kb = a.k + (size_t)tok0 * kq_stride + (size_t)h * DK;
        const E* qb = a.q + (size_t)tok0 * kq_stride + (size_t)h * DK;
        const E* db = a.d_o + (size_t)tok0 * v_stride + (size_t)h * a.dv_dim + p.slice * SLW;
#pragma unroll
        for (int it = 0; it < C::UK; ++it) {
            const int u = tid + NTH * it, tq = u / PPR, piece = u % PPR;
#pragma unroll
            for (int rr = 0; rr < 4; ++rr) {
                pk[it][rr] = make_uint4(0, 0, 0, 0); pq[it][rr] = make_uint4(0, 0, 0, 0);
                if (((16 * PPR) % NTH == 0 || u < 16 * PPR) && 4 * tq + rr < clen) {
                    pk[it][rr] = *reinterpret_cast<const uint4*>(kb + (size_t)(4 * tq + rr) * kq_stride + piece * EPP);
                    pq[it][rr] = *reinterpret_cast<const uint4*>(qb + (size_t)(4 * tq + rr) * kq_stride + piece * EPP);
                }
            }
        }
#pragma unroll
        for (int it = 0; it < C::UV; ++it) {
            const int u = tid + NTH * it, tq = u / VPP, pc = u % VPP;
#pragma unroll
            for (int rr = 0; rr < 4; ++rr) {
                pd[it][rr] = make_uint4(0, 0, 0, 0);
                if (((16 * VPP) % NTH == 0 || u < 16 * VPP) && 4 * tq + rr < clen)
                    pd[it][rr] = *reinterpret_cast<const uint4*>(db + (size_t)(4 * tq + rr) * v_stride + pc * EPP);
            }
        }
        const uint4* msrc = reinterpret_cast<const uint4*>(rec + ws_half_bytes<E>());
        const uint4* psrc = reinterpret_cast<const uint4*>(rec + 2 * ws_half_bytes<E>());
#pragma unroll
        for (int it = 0; it < C::UT; ++it) {
            const int i = tid + NTH * it;
            pm[it] = make_uint4(0, 0, 0, 0); pp[it] = make_uint4(0, 0, 0, 0);
            if (C::TP16 % NTH == 0 || i < C::TP16) { pm[it] = msrc[i]; pp[it] = psrc[i]; }
        }
        const float* vec = reinterpret_cast<const float*>(rec + 3 * ws_half_bytes<E>());
#pragma unroll
        for (int x = 0; x < 3; ++x) pvec[x] = vec[64 * x + lane];
        pvec[3] = vec[256 + lane];
    };
    auto stash = [&]() {
        E* Krq = reinterpret_cast<E*>(lds);
        E* Ktq = reinterpret_cast<E*>(lds + OFF_KT);
        E* Qtq = reinterpret_cast<E*>(lds + OFF_QT);
        E* Dtq = reinterpret_cast<E*>(lds + OFF_DO);
#pragma unroll
        for (int it = 0; it < C::UK; ++it) {
            const int u = tid + NTH * it;
            if ((16 * PPR) % NTH == 0 || u < 16 * PPR) {
                const int tq = u / PPR, piece = u % PPR;
#pragma unroll
                for (int rr = 0; rr < 4; ++rr) store_rq_piece(Krq, KP, 4 * tq + rr, piece, pk[it][rr]);
                store_tq_rows(Ktq, 2, tq, piece, pk[it], 0);
                store_tq_rows(Qtq, 2, tq, piece, pq[it], 0);
            }
        }
#pragma unroll
        for (int it = 0; it < C::UV; ++it) {
            const int u = tid + NTH * it;
            if ((16 * VPP) % NTH == 0 || u < 16 * VPP) store_tq_rows(Dtq, 2, u / VPP, u % VPP, pd[it], 0);
        }
#pragma unroll
        for (int it = 0; it < C::UT; ++it) {
            const int i = tid + NTH * it;
            if (C::TP16 % NTH == 0 || i < C::TP16) {
                reinterpret_cast<uint4*>(lds + OFF_MT)[i] = pm[it];
                reinterpret_cast<uint4*>(lds + OFF_PT)[i] = pp[it];
            }
        }
        if (tid < 64) {
#pragma unroll
            for (int x = 0; x < 4; ++x) reinterpret_cast<float*>(lds + OFF_VEC)[64 * x + tid] = pvec[x];
        }
    };

    if (p.nch > 0) fetch(p.nch - 1);
    for (int c = p.nch - 1; c >= 0; --c) {
        const long tok0 = p.t0 + 64L * c;
        const int clen = min(64, p.len - 64 * c);
        __syncthreads();
        stash();
        __syncthreads();
        if (c > 0) fetch(c - 1);

        const E* Krq = reinterpret_cast<const E*>(lds);
        const E* Ktq = reinterpret_cast<const E*>(lds + OFF_KT);
        const E* Qtq = reinterpret_cast<const E*>(lds + OFF_QT);
        const E* MTr = reinterpret_cast<const E*>(lds + OFF_MT);
        const E* PTr = reinterpret_cast<const E*>(lds + OFF_PT);
        const E* Dtq = reinterpret_cast<const E*>(lds + OFF_DO);
        const float* eg = reinterpret_cast<const float*>(lds + OFF_VEC);
        const float* ed = eg + 64;
        const float* be = eg + 128;
        const float* rq = eg + 192;

        // the gradient of the state this chunk hands on (transposed, like the state checkpoints)
        E* dck = a.ds_chk + (((size_t)(p.ch0 + c) * a.H + h) * a.dv_dim + col) * DK;
        Quad dSq[KB];
#pragma unroll
        for (int kt = 0; kt < KB; ++kt) {
            dSq[kt] = acc_to_quad<E>(dS[kt]);
            *reinterpret_cast<Quad*>(dck + 16 * kt + 4 * g) = dSq[kt];
        }
        Quad dOq[4];
        floatx4 dOa[4];
#pragma unroll
        for (int it = 0; it < 4; ++it) {
            const Slot<E> sd = load_slot(Dtq, wave * 2 + (it >> 1), lane);
            dOq[it] = (it & 1) ? sd.q1 : sd.q0;
            dOa[it] = quad_to_acc(dOq[it]);
        }
        // dU = P^T dO + diag(gamma_C/gamma_i) K dS'
        Quad dUq[4];
#pragma unroll
        for (int it = 0; it < 4; ++it) {
            floatx4 kd = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int kp = 0; kp < KP; ++kp) mma32<E>(kd, load_slot(Krq, it * KP + kp, lane), dSq[2 * kp], dSq[2 * kp + 1]);
            floatx4 du = kd * ld_acc4(ed + 16 * it + 4 * g);
#pragma unroll
            for (int jp = (it >> 1); jp < 2; ++jp)       // P^T is upper triangular
                mma32<E>(du, load_slot(PTr, triu_pair(it, jp), lane), dOq[2 * jp], dOq[2 * jp + 1]);
            dUq[it] = acc_to_quad<E>(du);
        }
        // Y = M^T dU,  dX = B Y = dV
        E* yb = a.Y + (size_t)tok0 * v_stride + (size_t)h * a.dv_dim + col;
        E* vb = a.dv + (size_t)tok0 * v_stride + (size_t)h * a.dv_dim + col;
        Quad gdOq[4], gdXq[4];
#pragma unroll
        for (int it = 0; it < 4; ++it) {
            floatx4 y = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int jp = (it >> 1); jp < 2; ++jp)
                mma32<E>(y, load_slot(MTr, triu_pair(it, jp), lane), dUq[2 * jp], dUq[2 * jp + 1]);
            store_rows<E>(yb, v_stride, y, it, g, clen);
            const floatx4 dx = y * ld_acc4(be + 16 * it + 4 * g);
            store_rows<E>(vb, v_stride, dx, it, g, clen);
            const floatx4 egv = ld_acc4(eg + 16 * it + 4 * g);
            gdOq[it] = acc_to_quad<E>(egv * ld_acc4(rq + 16 * it + 4 * g) * dOa[it]);   // D_gamma dO / ||q||
            gdXq[it] = acc_to_quad<E>(-(egv * dx));
        }
        // dS = gamma_C dS' + Q^T D_gamma dO - K^T D_gamma dX
        const float gC = eg[63];
#pragma unroll
        for (int kt = 0; kt < KB; ++kt) {
            dS[kt] = dS[kt] * gC;
#pragma unroll
            for (int jp = 0; jp < 2; ++jp) {
                mma32<E>(dS[kt], load_slot(Qtq, kt * 2 + jp, lane), gdOq[2 * jp], gdOq[2 * jp + 1]);
                mma32<E>(dS[kt], load_slot(Ktq, kt * 2 + jp, lane), gdXq[2 * jp], gdXq[2 * jp + 1]);
            }
        }
    }
    if (a.dh0) {
#pragma unroll
        for (int kt = 0; kt < KB; ++kt)
#pragma unroll
            for (int e = 0; e < 4; ++e)
                a.dh0[((size_t)p.chain * DK + 16 * kt + 4 * g + e) * a.dv_dim + col] = dS[kt][e];
    }
}

// =================================================================================================
// per chunk-head: contractions over d_v, then over the chunk
// =================================================================================================
namespace {

constexpr int kLdc = 68;   // row stride (floats) of the fp32 64x64 matrices in LDS

template <typename E> struct Piece;
template <> struct Piece<bf16_t> {
    static constexpr int N = 8;
    __device__ static void unpack(uint4 d, float (&f)[8])
    {
        const uint32_t w[4] = {d.x, d.y, d.z, d.w};
#pragma unroll
        for (int m = 0; m < 4; ++m) { f[2 * m] = bf16_bits_to_float(w[m] & 0xffffu); f[2 * m + 1] = bf16_bits_to_float(w[m] >> 16); }
    }
    __device__ static uint4 pack(const float (&f)[8])
    {
        return make_uint4(pack_bf16x2(f[0], f[1]), pack_bf16x2(f[2], f[3]), pack_bf16x2(f[4], f[5]), pack_bf16x2(f[6], f[7]));
    }
};
template <> struct Piece<float> {
    static constexpr int N = 4;
    __device__ static void unpack(uint4 d, float (&f)[4])
    {
        f[0] = __uint_as_float(d.x); f[1] = __uint_as_float(d.y); f[2] = __uint_as_float(d.z); f[3] = __uint_as_float(d.w);
    }
    __device__ static uint4 pack(const float (&f)[4])
    {
        return make_uint4(__float_as_uint(f[0]), __float_as_uint(f[1]), __float_as_uint(f[2]), __float_as_uint(f[3]));
    }
};
template <typename E> __device__ __forceinline__ float dot_piece(uint4 x, uint4 y)
{
    float fx[Piece<E>::N], fy[Piece<E>::N];
    Piece<E>::unpack(x, fx); Piece<E>::unpack(y, fy);
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < Piece<E>::N; ++i) s += fx[i] * fy[i];
    return s;
}

// A-operand slot built from an fp32 64x64 matrix in LDS: row `row`, columns 32 jp + {0, 16} + 4 g .. + 3
template <typename E> __device__ __forceinline__ Slot<E> slot_from_rows(const float* m, int row, int jp, int g)
{
    Slot<E> s;
    s.q0 = acc_to_quad<E>(ld_acc4(m + row * kLdc + 32 * jp + 4 * g));
    s.q1 = acc_to_quad<E>(ld_acc4(m + row * kLdc + 32 * jp + 16 + 4 * g));
    return s;
}
// the same of the transposed matrix, entry (row, i) = m[i][row] * scale[i]
template <typename E, bool SCALE>
__device__ __forceinline__ Slot<E> slot_from_cols(const float* m, const float* scale, int row, int jp, int g)
{
    floatx4 x0, x1;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const int i0 = 32 * jp + 4 * g + e, i1 = i0 + 16;
        x0[e] = m[i0 * kLdc + row]; x1[e] = m[i1 * kLdc + row];
        if constexpr (SCALE) { x0[e] *= scale[i0]; x1[e] *= scale[i1]; }
    }
    Slot<E> s; s.q0 = acc_to_quad<E>(x0); s.q1 = acc_to_quad<E>(x1); return s;
}

__device__ __forceinline__ float row16_sum(float x)       // sum over the 16 lanes that share g
{
#pragma unroll
    for (int off = 1; off < 16; off <<= 1) x += __shfl_xor(x, off, kWave);
    return x;
}

}  // namespace

template <typename E, int DK>
__global__ __launch_bounds__(256, 2) void bwd_assemble_kernel(BwdArgs<E> a)
{
    constexpr int KB = DK / 16;
    constexpr int W = 128 / (int)sizeof(E);          // d_v columns per slab: 8 pieces of 16 bytes per row
    constexpr int NP = W / 32;                       // contraction pairs per slab
    constexpr int EPP = 16 / (int)sizeof(E);
    constexpr int PPR = DK * (int)sizeof(E) / 16;
    // operand areas are padded (one empty slot after every eight, see kla_mma.hpp): 9/8 of their contents
    constexpr int AB = 64 * W * (int)sizeof(E) / 8 * 9;      // a [64, slab] operand area
    constexpr int BB = DK * W * (int)sizeof(E) / 8 * 9;      // a [dk, slab] operand area
    constexpr int OPB = 64 * DK * (int)sizeof(E) / 8 * 9;
    constexpr int MB = 64 * kLdc * 4;
    // first phase: dO | U | Y | S^T | dS'^T
    constexpr int A_DO = 0, A_U = AB, A_Y = 2 * AB, B_S = 3 * AB, B_DS = 3 * AB + BB;
    constexpr int PH1 = 3 * AB + 2 * BB;
    // second phase: K transposed | Q transposed | A o dP | D'
    constexpr int C_KT = 0, C_QT = OPB, C_E1 = 2 * OPB, C_DP = 2 * OPB + MB;
    constexpr int PH2 = 2 * OPB + 2 * MB;
    constexpr int BIG = PH1 > PH2 ? PH1 : PH2;
    __shared__ __attribute__((aligned(16))) char lds[BIG];
    __shared__ __attribute__((aligned(16))) float eg_s[64], ed_s[64], beta_s[64], invden_s[64], rq_s[64], g_s[64], yx_s[64],
        dg_s[64], dbeta_s[64];
    __shared__ float red_s[8];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int r = lane & 15, g = lane >> 4;

    // ---- which chunk of which sequence (as in the intra-chunk stage) -------------------------------
    const int h = blockIdx.x % a.H;
    const int cg = blockIdx.x / a.H;
    const ChunkPos cp = chunk_pos(a.cu_seqlens, a.chunk_off, a.n_seq, a.T, a.NT, cg);
    const long tok0 = cp.tok0;
    const int clen = cp.clen;
    const size_t kq_stride = (size_t)a.H * DK, v_stride = (size_t)a.H * a.dv_dim;
    const char* rec = a.rec + (size_t)blockIdx.x * bwd_record_bytes<E>();
    {
        const float* vec = reinterpret_cast<const float*>(rec + 3 * ws_half_bytes<E>());
        float* dst = wave == 0 ? eg_s : (wave == 1 ? ed_s : (wave == 2 ? beta_s : invden_s));
        dst[lane] = vec[tid];
        // Normalised read-out (Sec. 3.3): the rows of dO are scaled by 1/||q_i|| wherever they meet U or S, which makes
        // dQ' = diag(1/||q||) dL/d(q/||q||); dq_i = dQ'_i - (q_i . dQ'_i) q_i / ||q_i||^2 at the end.
        if (wave == 1) rq_s[lane] = vec[256 + lane];
        if (wave == 0) g_s[lane] = lane < clen ? a.log_alpha[(size_t)(tok0 + lane) * a.H + h] : 0.f;
    }
    __syncthreads();
    if (wave == 0) {                                 // g_i = log gamma_i
        float x = g_s[lane];
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) { const float y = __shfl_up(x, off, kWave); if (lane >= off) x += y; }
        g_s[lane] = x;
    }

    floatx4 dQ[KB], dKr[KB], dKw[KB], dP[4], N1[4];
#pragma unroll
    for (int ct = 0; ct < KB; ++ct) { dQ[ct] = floatx4{0.f, 0.f, 0.f, 0.f}; dKr[ct] = dQ[ct]; dKw[ct] = dQ[ct]; }
#pragma unroll
    for (int jt = 0; jt < 4; ++jt) { dP[jt] = floatx4{0.f, 0.f, 0.f, 0.f}; N1[jt] = dP[jt]; }
    float yx[2] = {0.f, 0.f};
    float sdot = 0.f;                                // <dS', S> over this thread's share

    // ---- first phase: everything that contracts over d_v, one slab of W columns at a time -----------
    const E* Sg = a.s_chk + (size_t)blockIdx.x * DK * a.dv_dim;
    const E* dSg = a.ds_chk + (size_t)blockIdx.x * DK * a.dv_dim;
    for (int slab0 = 0; slab0 < a.dv_dim; slab0 += W) {
        __syncthreads();
#pragma unroll
        for (int it = 0; it < 2; ++it) {
            const int pi = tid + 256 * it, row = pi >> 3, piece = pi & 7;
            uint4 d_o = make_uint4(0, 0, 0, 0), du = d_o, dy = d_o, dx = d_o;
            if (row < clen) {
                const size_t off = (size_t)(tok0 + row) * v_stride + (size_t)h * a.dv_dim + slab0 + piece * EPP;
                d_o = *reinterpret_cast<const uint4*>(a.d_o + off);
                du = *reinterpret_cast<const uint4*>(a.U + off);
                dy = *reinterpret_cast<const uint4*>(a.Y + off);
                dx = *reinterpret_cast<const uint4*>(a.X + off);
            }
            store_rq_piece_pad(reinterpret_cast<E*>(lds + A_DO), NP, row, piece, d_o);
            store_rq_piece_pad(reinterpret_cast<E*>(lds + A_U), NP, row, piece, du);
            store_rq_piece_pad(reinterpret_cast<E*>(lds + A_Y), NP, row, piece, dy);
            yx[it] += dot_piece<E>(dy, dx);
        }
        // S^T and dS'^T rows slab0 .. slab0 + W - 1 (d_k elements each) -> operands contracted over d_v
#pragma unroll
        for (int it = 0; it < (W / 4 * PPR + 255) / 256; ++it) {
            const int u = tid + 256 * it, tq = u / PPR, piece = u % PPR;
            if ((W / 4 * PPR) % 256 != 0 && u >= W / 4 * PPR) break;
            uint4 sd[4], dd[4];
#pragma unroll
            for (int rr = 0; rr < 4; ++rr) {
                const size_t off = (size_t)(slab0 + 4 * tq + rr) * DK + piece * EPP;
                sd[rr] = *reinterpret_cast<const uint4*>(Sg + off);
                dd[rr] = *reinterpret_cast<const uint4*>(dSg + off);
                sdot += dot_piece<E>(sd[rr], dd[rr]);
            }
            store_tq_rows_pad(reinterpret_cast<E*>(lds + B_S), NP, tq, piece, sd, 0);
            store_tq_rows_pad(reinterpret_cast<E*>(lds + B_DS), NP, tq, piece, dd, 0);
        }
        __syncthreads();
#pragma unroll
        for (int kp = 0; kp < NP; ++kp) {
            // the row scalings D_gamma, -D_gamma B and diag(gamma_C/gamma_i) are applied to the sums afterwards
            const Slot<E> a_do = load_slot_pad(reinterpret_cast<const E*>(lds + A_DO), wave * NP + kp, lane);
            const Slot<E> a_u = load_slot_pad(reinterpret_cast<const E*>(lds + A_U), wave * NP + kp, lane);
            const Slot<E> a_y = load_slot_pad(reinterpret_cast<const E*>(lds + A_Y), wave * NP + kp, lane);
#pragma unroll
            for (int ct = 0; ct < KB; ++ct) {
                const Slot<E> b_s = load_slot_pad(reinterpret_cast<const E*>(lds + B_S), ct * NP + kp, lane);
                const Slot<E> b_ds = load_slot_pad(reinterpret_cast<const E*>(lds + B_DS), ct * NP + kp, lane);
                mma32<E>(dQ[ct], a_do, b_s.q0, b_s.q1);        // dO S^T
                mma32<E>(dKr[ct], a_y, b_s.q0, b_s.q1);        // Y S^T
                mma32<E>(dKw[ct], a_u, b_ds.q0, b_ds.q1);      // U dS'^T
            }
            static_for<4>([&](auto jt) {
                if (jt <= wave) {                              // lower-triangular tiles only
                    const Slot<E> b_u = load_slot_pad(reinterpret_cast<const E*>(lds + A_U), jt * NP + kp, lane);
                    mma32<E>(dP[jt], a_do, b_u.q0, b_u.q1);    // dO U^T
                    mma32<E>(N1[jt], a_y, b_u.q0, b_u.q1);     // Y U^T
                }
            });
        }
    }
    {   // D_gamma dO S^T,  -D_gamma dX S^T (dX = B Y),  diag(gamma_C/gamma_i) U dS'^T
        const floatx4 egv = ld_acc4(eg_s + 16 * wave + 4 * g), edv = ld_acc4(ed_s + 16 * wave + 4 * g);
        const floatx4 ngb = -(egv * ld_acc4(beta_s + 16 * wave + 4 * g));
        const floatx4 egq = egv * ld_acc4(rq_s + 16 * wave + 4 * g);
#pragma unroll
        for (int ct = 0; ct < KB; ++ct) { dQ[ct] = dQ[ct] * egq; dKr[ct] = dKr[ct] * ngb; dKw[ct] = dKw[ct] * edv; }
    }
    // Y_i . X_i: the 8 threads of a row are neighbours
#pragma unroll
    for (int it = 0; it < 2; ++it) {
        float x = yx[it];
        x += __shfl_xor(x, 1, kWave); x += __shfl_xor(x, 2, kWave); x += __shfl_xor(x, 4, kWave);
        if ((tid & 7) == 0) yx_s[(tid + 256 * it) >> 3] = x;
    }
    sdot = wave_sum(sdot);
    if (lane == 0) red_s[wave] = sdot;
    __syncthreads();                                 // the slab areas are dead from here on

    // ---- second phase: K^T, Q^T as operands; A o dP and D' = -A^- o (Y U^T) as fp32 matrices ---------
    E* Ktq = reinterpret_cast<E*>(lds + C_KT);
    E* Qtq = reinterpret_cast<E*>(lds + C_QT);
    float* E1 = reinterpret_cast<float*>(lds + C_E1);
    float* Dp = reinterpret_cast<float*>(lds + C_DP);
    {
        const E* kb = a.k + (size_t)tok0 * kq_stride + (size_t)h * DK;
        const E* qb = a.q + (size_t)tok0 * kq_stride + (size_t)h * DK;
#pragma unroll
        for (int it = 0; it < (16 * PPR + 255) / 256; ++it) {
            const int u = tid + 256 * it, tq = u / PPR, piece = u % PPR;
            if ((16 * PPR) % 256 != 0 && u >= 16 * PPR) break;
            uint4 kd[4], qd[4];
#pragma unroll
            for (int rr = 0; rr < 4; ++rr) {
                kd[rr] = make_uint4(0, 0, 0, 0); qd[rr] = make_uint4(0, 0, 0, 0);
                if (4 * tq + rr < clen) {
                    kd[rr] = *reinterpret_cast<const uint4*>(kb + (size_t)(4 * tq + rr) * kq_stride + piece * EPP);
                    qd[rr] = *reinterpret_cast<const uint4*>(qb + (size_t)(4 * tq + rr) * kq_stride + piece * EPP);
                }
            }
            store_tq_rows_pad(Ktq, 2, tq, piece, kd, 0);
            store_tq_rows_pad(Qtq, 2, tq, piece, qd, 0);
        }
        static_for<4>([&](auto jt) {
            const int j = 16 * jt + r;
            const float gj = g_s[j];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int i = 16 * wave + 4 * g + e;
                const float dec = (jt <= wave && j <= i) ? expf(g_s[i] - gj) : 0.f;
                E1[i * kLdc + j] = dec * rq_s[i] * dP[jt][e];
                Dp[i * kLdc + j] = (j < i) ? -dec * N1[jt][e] : 0.f;
            }
        });
    }
    __syncthreads();

    // K and Q of this wave's rows in accumulator layout: rows 16 wave + 4 g + e, column 16 ct + r
    auto kacc = [&](const E* base, int ct) {
        const Slot<E> s = load_slot_pad(base, ct * 2 + (wave >> 1), lane);
        return quad_to_acc((wave & 1) ? s.q1 : s.q0);
    };
    // sum_i (gamma_C/gamma_i) k_i . (dS' U_i): the third bracket term alone, before the others are added to it
    float zsum = 0.f;
#pragma unroll
    for (int ct = 0; ct < KB; ++ct) {
        const floatx4 kk = kacc(Ktq, ct);
#pragma unroll
        for (int e = 0; e < 4; ++e) zsum += dKw[ct][e] * kk[e];
    }
    zsum = wave_sum(zsum);
    if (lane == 0) red_s[4 + wave] = zsum;

    floatx4 E2[KB];
#pragma unroll
    for (int ct = 0; ct < KB; ++ct) E2[ct] = floatx4{0.f, 0.f, 0.f, 0.f};
    const int row_a = 16 * wave + r;                 // the operand row this lane feeds
    static_for<2>([&](auto jp) {
        if (jp <= (wave >> 1)) {                     // lower-triangular: columns up to this row tile
            const Slot<E> a_e1 = slot_from_rows<E>(E1, row_a, jp, g);
            const Slot<E> a_dp = slot_from_rows<E>(Dp, row_a, jp, g);
#pragma unroll
            for (int ct = 0; ct < KB; ++ct) {
                const Slot<E> b_k = load_slot_pad(Ktq, ct * 2 + jp, lane);
                mma32<E>(dQ[ct], a_e1, b_k.q0, b_k.q1);        // (A o dP) K
                mma32<E>(E2[ct], a_dp, b_k.q0, b_k.q1);        // D' K
            }
        }
        if (jp >= (wave >> 1)) {                     // the transposes are upper triangular
            const Slot<E> a_e1t = slot_from_cols<E, false>(E1, nullptr, row_a, jp, g);
            const Slot<E> a_dpt = slot_from_cols<E, true>(Dp, beta_s, row_a, jp, g);
#pragma unroll
            for (int ct = 0; ct < KB; ++ct) {
                const Slot<E> b_q = load_slot_pad(Qtq, ct * 2 + jp, lane);
                const Slot<E> b_k = load_slot_pad(Ktq, ct * 2 + jp, lane);
                mma32<E>(dKw[ct], a_e1t, b_q.q0, b_q.q1);      // (A o dP)^T Q
                mma32<E>(dKw[ct], a_dpt, b_k.q0, b_k.q1);      // (B D')^T K
            }
        }
    });

    // ---- rows: dbeta, dg, the beta term of dK; outputs ---------------------------------------------
    float dbr[4] = {0.f, 0.f, 0.f, 0.f}, dgr[4] = {0.f, 0.f, 0.f, 0.f}, dqr[4] = {0.f, 0.f, 0.f, 0.f};
    floatx4 kk[KB];
    const floatx4 bev = ld_acc4(beta_s + 16 * wave + 4 * g);
#pragma unroll
    for (int ct = 0; ct < KB; ++ct) {
        kk[ct] = kacc(Ktq, ct);
        const floatx4 qq = kacc(Qtq, ct);
        dKr[ct] = dKr[ct] + bev * E2[ct];            // + B D' K
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            dbr[e] += E2[ct][e] * kk[ct][e];
            dqr[e] += dQ[ct][e] * qq[e];
            dgr[e] += (dKr[ct][e] - dKw[ct][e]) * kk[ct][e];
        }
    }
    floatx4 c5, cq;                                  // -2 beta dbeta / (|k|^2 + eps) and -(q . dQ') / ||q||^2 per row
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const int i = 16 * wave + 4 * g + e;
        const float db = row16_sum(dbr[e]) + yx_s[i];
        const float dqv = row16_sum(dqr[e]);
        const float dgv = row16_sum(dgr[e]) + dqv;
        if (r == 0) { dbeta_s[i] = db; dg_s[i] = dgv; }
        cq[e] = -dqv * rq_s[i] * rq_s[i];
        c5[e] = (a.opts & kOptGdnBeta) ? 0.f : -2.f * beta_s[i] * db * invden_s[i];   // beta = eta does not depend on k
    }
    {
        E* qo = a.dq + (size_t)tok0 * kq_stride + (size_t)h * DK + r;
        E* ko = a.dk + (size_t)tok0 * kq_stride + (size_t)h * DK + r;
#pragma unroll
        for (int ct = 0; ct < KB; ++ct) {
            const floatx4 dkv = dKr[ct] + dKw[ct] + c5 * kk[ct];
            if (a.opts & kOptNormalizeQ) dQ[ct] = dQ[ct] + cq * kacc(Qtq, ct);
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int row = 16 * wave + 4 * g + e;
                if (row < clen) {
                    qo[(size_t)row * kq_stride + 16 * ct] = from_float<E>(dQ[ct][e]);
                    ko[(size_t)row * kq_stride + 16 * ct] = from_float<E>(dkv[e]);
                }
            }
        }
    }
    __syncthreads();
    if (wave == 0) {
        // g_C sits at row 63 (rows past the end of a ragged chunk carry log alpha = 0), and the gradient of the
        // outgoing state meets it through <dS', S'> = gamma_C <dS', S> + sum_i (gamma_C/gamma_i) k_i.(dS' U_i)
        float x = dg_s[lane];
        if (lane == 63) x += eg_s[63] * (red_s[0] + red_s[1] + red_s[2] + red_s[3]) + (red_s[4] + red_s[5] + red_s[6] + red_s[7]);
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) { const float y = __shfl_down(x, off, kWave); if (lane + off < 64) x += y; }
        if (lane < clen) {
            a.dlog_alpha[(size_t)(tok0 + lane) * a.H + h] = x;
            a.deta[(size_t)(tok0 + lane) * a.H + h] = dbeta_s[lane] * invden_s[lane];
        }
    }
}

// =================================================================================================
// launchers
// =================================================================================================
template <typename E, int DK>
static hipError_t launch_states_dk(const BwdArgs<E>& a, int waves, hipStream_t st)
{
    const int n_chains = (a.n_seq > 0 ? a.n_seq : a.N) * a.H;
    if (n_chains == 0) return hipSuccess;
    const dim3 grid((unsigned)(((n_chains + 7) / 8) * 8 * (a.dv_dim / (16 * waves))));
    if (waves == 1) hipLaunchKernelGGL((bwd_states_kernel<E, DK, 1>), grid, dim3(64), 0, st, a);
    else            hipLaunchKernelGGL((bwd_states_kernel<E, DK, 2>), grid, dim3(128), 0, st, a);
    return hipGetLastError();
}
template <typename E, int DK>
static hipError_t launch_scan_dk(const BwdArgs<E>& a, int waves, hipStream_t st)
{
    const int n_chains = (a.n_seq > 0 ? a.n_seq : a.N) * a.H;
    if (n_chains == 0) return hipSuccess;
    const dim3 grid((unsigned)(((n_chains + 7) / 8) * 8 * (a.dv_dim / (16 * waves))));
    if (waves == 1) hipLaunchKernelGGL((bwd_scan_kernel<E, DK, 1>), grid, dim3(64), 0, st, a);
    else            hipLaunchKernelGGL((bwd_scan_kernel<E, DK, 2>), grid, dim3(128), 0, st, a);
    return hipGetLastError();
}

template <typename E> hipError_t launch_bwd_states(const BwdArgs<E>& a, int dk, int waves, hipStream_t st)
{
    if (waves != 1 && waves != 2) return hipErrorInvalidValue;
    return dk == 64 ? launch_states_dk<E, 64>(a, waves, st) : launch_states_dk<E, 128>(a, waves, st);
}
template <typename E> hipError_t launch_bwd_scan(const BwdArgs<E>& a, int dk, int waves, hipStream_t st)
{
    if (waves != 1 && waves != 2) return hipErrorInvalidValue;
    return dk == 64 ? launch_scan_dk<E, 64>(a, waves, st) : launch_scan_dk<E, 128>(a, waves, st);
}
template <typename E> hipError_t launch_bwd_assemble(const BwdArgs<E>& a, int dk, long n_chunks, hipStream_t st)
{
    if (n_chunks == 0) return hipSuccess;
    const dim3 grid((unsigned)(n_chunks * a.H)), block(256);
    if (dk == 64) hipLaunchKernelGGL((bwd_assemble_kernel<E, 64>), grid, block, 0, st, a);
    else          hipLaunchKernelGGL((bwd_assemble_kernel<E, 128>), grid, block, 0, st, a);
    return hipGetLastError();
}
template hipError_t launch_bwd_states<float>(const BwdArgs<float>&, int, int, hipStream_t);
template hipError_t launch_bwd_states<bf16_t>(const BwdArgs<bf16_t>&, int, int, hipStream_t);
template hipError_t launch_bwd_scan<float>(const BwdArgs<float>&, int, int, hipStream_t);
template hipError_t launch_bwd_scan<bf16_t>(const BwdArgs<bf16_t>&, int, int, hipStream_t);
template hipError_t launch_bwd_assemble<float>(const BwdArgs<float>&, int, long, hipStream_t);
template hipError_t launch_bwd_assemble<bf16_t>(const BwdArgs<bf16_t>&, int, long, hipStream_t);

}  // namespace kla
