// Inter-chunk stage of the chunkwise forward: state propagation fused with the chunk outputs
// (Algorithm 1 right panel, lines 5-7; eqs. (6), (7), (8)).
//
// One workgroup walks one (sequence, head) through its chunks for a slice of the d_v state
// columns; inside it every WAVE owns 16 columns and is an independent recurrence, because
// eqs. (6)-(8) act on the columns of S, U and O separately.  Per chunk and wave, with the
// intra-chunk stage's T' = (I+L)^{-1} B, P = A o QK^T and g = log gamma:
//     X  = V - D_gamma (K S)                 right-hand side of eq. (6) without B
//     U  = T' X                              eq. (6)
//     O  = D_gamma (Q S) + P U               eq. (7)
//     S  = gamma_C S + K^T diag(gamma_C/gamma_i) U          eq. (8)
// The fp32 state S lives in MFMA accumulator registers for the whole sequence.  S, X and U move
// from one product to the next in registers (see kla_mma.hpp: an accumulator tile is the next
// product's B operand), so the only LDS traffic is the A operands K, Q, K^T, T', P and the V
// slice, staged once per chunk for all waves of the workgroup.  No per-chunk state, W or U ever
// goes to HBM.
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
}  // namespace

template <typename E, int DK, int NW>
__global__ __launch_bounds__(64 * NW) void scan_kernel(ScanArgs<E> a)
{
    constexpr int NTH = 64 * NW;
    constexpr int KB = DK / 16, KP = DK / 32;
    constexpr int SLW = 16 * NW;                         // state columns per workgroup
    constexpr int PPR = DK * (int)sizeof(E) / 16;        // 16-byte pieces per K/Q row
    constexpr int EPP = 16 / (int)sizeof(E);             // elements per piece
    constexpr int VPP = SLW * (int)sizeof(E) / 16;       // pieces per V/O slice row
    constexpr int SB = slot_bytes<E>();
    constexpr int OPB = 64 * DK * (int)sizeof(E);
    constexpr int OLD = SLW + EPP;                       // row stride of the output staging tile
    typedef typename QuadT<E>::type Quad;

    __shared__ __attribute__((aligned(16))) char Krq_[OPB];
    __shared__ __attribute__((aligned(16))) char Qrq_[OPB];
    __shared__ __attribute__((aligned(16))) char Ktq_[OPB];
    __shared__ __attribute__((aligned(16))) char Trq_[512 * SB];
    __shared__ __attribute__((aligned(16))) char Prq_[512 * SB];
    __shared__ __attribute__((aligned(16))) char Vtq_[NW * 2 * 64 * SB];
    __shared__ __attribute__((aligned(16))) E Ost[64 * OLD];
    __shared__ __attribute__((aligned(16))) float eg[64];
    __shared__ __attribute__((aligned(16))) float ed[64];
    E* Krq = reinterpret_cast<E*>(Krq_);
    E* Qrq = reinterpret_cast<E*>(Qrq_);
    E* Ktq = reinterpret_cast<E*>(Ktq_);
    E* Trq = reinterpret_cast<E*>(Trq_);
    E* Prq = reinterpret_cast<E*>(Prq_);
    E* Vtq = reinterpret_cast<E*>(Vtq_);

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int r = lane & 15, g = lane >> 4;

    // ---- workgroup -> (sequence, head, column slice).  Consecutive workgroup ids go to different
    //      XCDs; the slices of one (sequence, head) are given ids congruent mod 8 so that they share
    //      one XCD's L2 for the K, Q, T', P reads they have in common. ---------------------------
    const int nsl = a.dv / SLW;
    const int n_states = a.n_seq > 0 ? a.n_seq : a.N;
    const int n_chains = n_states * a.H;
    const int xcd = blockIdx.x & 7, p = blockIdx.x >> 3;
    const int chain = (p / nsl) * 8 + xcd, slice = p % nsl;
    if (chain >= n_chains) return;
    const int s = chain / a.H, h = chain % a.H;
    long t0; int len, ch0;
    if (a.cu_seqlens) { t0 = a.cu_seqlens[s]; len = a.cu_seqlens[s + 1] - (int)t0; ch0 = a.chunk_off[s]; }
    else              { t0 = (long)s * a.T;   len = a.T;                           ch0 = s * a.NT; }
    const int nch = (len + 63) / 64;
    const int col = slice * SLW + 16 * wave + r;         // this lane's state column

    floatx4 S[KB];
#pragma unroll
    for (int kt = 0; kt < KB; ++kt)
#pragma unroll
        for (int e = 0; e < 4; ++e)
            S[kt][e] = a.h0 ? a.h0[((size_t)chain * DK + 16 * kt + 4 * g + e) * a.dv + col] : 0.f;

    const size_t kq_stride = (size_t)a.H * DK, v_stride = (size_t)a.H * a.dv;

    for (int c = 0; c < nch; ++c) {
        const long tok0 = t0 + 64L * c;
        const int clen = min(64, len - 64 * c);
        const size_t ch = (size_t)(ch0 + c) * a.H + h;

        __syncthreads();   // every wave is done with the previous chunk's operands and staging tile

        // ---- stage this chunk's operands in LDS ------------------------------------------------
        {
            const E* kb = a.k + (size_t)tok0 * kq_stride + (size_t)h * DK;
            const E* qb = a.q + (size_t)tok0 * kq_stride + (size_t)h * DK;
            constexpr int UNITS = 16 * PPR;              // (4-row group, piece) units of a K/Q tile
#pragma unroll
            for (int it = 0; it < (UNITS + NTH - 1) / NTH; ++it) {
                const int u = tid + NTH * it;
                if (UNITS % NTH == 0 || u < UNITS) {
                    const int tq = u / PPR, piece = u % PPR;
                    uint4 kd[4], qd[4];
#pragma unroll
                    for (int rr = 0; rr < 4; ++rr) {
                        const int row = 4 * tq + rr;
                        kd[rr] = make_uint4(0, 0, 0, 0); qd[rr] = make_uint4(0, 0, 0, 0);
                        if (row < clen) {
                            kd[rr] = *reinterpret_cast<const uint4*>(kb + (size_t)row * kq_stride + piece * EPP);
                            qd[rr] = *reinterpret_cast<const uint4*>(qb + (size_t)row * kq_stride + piece * EPP);
                        }
                    }
#pragma unroll
                    for (int rr = 0; rr < 4; ++rr) {
                        store_rq_piece(Krq, KP, 4 * tq + rr, piece, kd[rr]);
                        store_rq_piece(Qrq, KP, 4 * tq + rr, piece, qd[rr]);
                    }
                    store_tq_rows(Ktq, 2, tq, piece, kd, 0);
                }
            }
            const E* vb = a.v + (size_t)tok0 * v_stride + (size_t)h * a.dv + slice * SLW;
            constexpr int VUNITS = 16 * VPP;
#pragma unroll
            for (int it = 0; it < (VUNITS + NTH - 1) / NTH; ++it) {
                const int u = tid + NTH * it;
                if (VUNITS % NTH == 0 || u < VUNITS) {
                    const int tq = u / VPP, pv = u % VPP;
                    uint4 vd[4];
#pragma unroll
                    for (int rr = 0; rr < 4; ++rr) {
                        const int row = 4 * tq + rr;
                        vd[rr] = make_uint4(0, 0, 0, 0);
                        if (row < clen) vd[rr] = *reinterpret_cast<const uint4*>(vb + (size_t)row * v_stride + pv * EPP);
                    }
                    store_tq_rows(Vtq, 2, tq, pv, vd, 0);
                }
            }
            const uint4* tsrc = reinterpret_cast<const uint4*>(reinterpret_cast<const char*>(a.wsT) + ch * 512 * SB);
            const uint4* psrc = reinterpret_cast<const uint4*>(reinterpret_cast<const char*>(a.wsP) + ch * 512 * SB);
            constexpr int TP16 = 512 * SB / 16;
#pragma unroll
            for (int it = 0; it < TP16 / NTH; ++it) {
                const int i = tid + NTH * it;
                reinterpret_cast<uint4*>(Trq_)[i] = tsrc[i];
                reinterpret_cast<uint4*>(Prq_)[i] = psrc[i];
            }
            if (tid < 64) {
                const float gv = a.wsG[ch * 64 + tid], gl = a.wsG[ch * 64 + 63];
                eg[tid] = expf(gv);                      // gamma_i
                ed[tid] = expf(gl - gv);                 // gamma_C / gamma_i
            }
        }
        __syncthreads();

        // ---- the chunk recurrence for this wave's 16 columns ------------------------------------
        Quad Sq[KB];
#pragma unroll
        for (int kt = 0; kt < KB; ++kt) Sq[kt] = acc_to_quad<E>(S[kt]);

        floatx4 ks[4], qs[4];
#pragma unroll
        for (int it = 0; it < 4; ++it) {
            ks[it] = floatx4{0.f, 0.f, 0.f, 0.f};
            qs[it] = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int kp = 0; kp < KP; ++kp) {
                const Slot<E> sk = load_slot(Krq, it * KP + kp, lane);
                mma32<E>(ks[it], sk, Sq[2 * kp], Sq[2 * kp + 1]);
                const Slot<E> sq = load_slot(Qrq, it * KP + kp, lane);
                mma32<E>(qs[it], sq, Sq[2 * kp], Sq[2 * kp + 1]);
            }
        }
        floatx4 egv[4];
        Quad Xq[4];
#pragma unroll
        for (int it = 0; it < 4; ++it) {
            egv[it] = ld_acc4(eg + 16 * it + 4 * g);
            const Slot<E> sv = load_slot(Vtq, wave * 2 + (it >> 1), lane);
            const floatx4 vv = quad_to_acc((it & 1) ? sv.q1 : sv.q0);
            Xq[it] = acc_to_quad<E>(vv - egv[it] * ks[it]);
        }
        floatx4 U[4];
        Quad Uq[4], Udq[4];
#pragma unroll
        for (int it = 0; it < 4; ++it) {
            U[it] = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int jp = 0; jp <= (it >> 1); ++jp) {   // T' is lower triangular
                const Slot<E> st = load_slot(Trq, it * 2 + jp, lane);
                mma32<E>(U[it], st, Xq[2 * jp], Xq[2 * jp + 1]);
            }
            Uq[it] = acc_to_quad<E>(U[it]);
            Udq[it] = acc_to_quad<E>(U[it] * ld_acc4(ed + 16 * it + 4 * g));
        }
#pragma unroll
        for (int it = 0; it < 4; ++it) {
            floatx4 o = egv[it] * qs[it];
#pragma unroll
            for (int jp = 0; jp <= (it >> 1); ++jp) {   // P is lower triangular
                const Slot<E> sp = load_slot(Prq, it * 2 + jp, lane);
                mma32<E>(o, sp, Uq[2 * jp], Uq[2 * jp + 1]);
            }
#pragma unroll
            for (int e = 0; e < 4; ++e) Ost[(16 * it + 4 * g + e) * OLD + 16 * wave + r] = from_float<E>(o[e]);
        }
        const float gC = eg[63];
#pragma unroll
        for (int kt = 0; kt < KB; ++kt) {
            S[kt] = S[kt] * gC;
#pragma unroll
            for (int jp = 0; jp < 2; ++jp) {
                const Slot<E> sk = load_slot(Ktq, kt * 2 + jp, lane);
                mma32<E>(S[kt], sk, Udq[2 * jp], Udq[2 * jp + 1]);
            }
        }
        __syncthreads();

        // ---- write the output rows of this slice, 16 bytes per lane ----------------------------
        {
            E* ob = a.o + (size_t)tok0 * v_stride + (size_t)h * a.dv + slice * SLW;
#pragma unroll
            for (int it = 0; it < (64 * VPP + NTH - 1) / NTH; ++it) {
                const int i = tid + NTH * it;
                const int row = i / VPP, pv = i % VPP;
                if (row < clen)
                    *reinterpret_cast<uint4*>(ob + (size_t)row * v_stride + pv * EPP) =
                        *reinterpret_cast<const uint4*>(Ost + row * OLD + pv * EPP);
            }
        }
    }

    if (a.hT) {
#pragma unroll
        for (int kt = 0; kt < KB; ++kt)
#pragma unroll
            for (int e = 0; e < 4; ++e)
                a.hT[((size_t)chain * DK + 16 * kt + 4 * g + e) * a.dv + col] = S[kt][e];
    }
}

template <typename E, int DK>
static hipError_t launch_scan_dk(const ScanArgs<E>& a, int waves, hipStream_t st)
{
    const int n_states = a.n_seq > 0 ? a.n_seq : a.N;
    const int n_chains = n_states * a.H;
    if (n_chains == 0) return hipSuccess;
    const int nsl = a.dv / (16 * waves);
    const dim3 grid((unsigned)(((n_chains + 7) / 8) * 8 * nsl));
    switch (waves) {
        case 1: hipLaunchKernelGGL((scan_kernel<E, DK, 1>), grid, dim3(64), 0, st, a); break;
        case 2: hipLaunchKernelGGL((scan_kernel<E, DK, 2>), grid, dim3(128), 0, st, a); break;
        default:
            if constexpr (sizeof(E) == 2) { hipLaunchKernelGGL((scan_kernel<E, DK, 4>), grid, dim3(256), 0, st, a); break; }
            else return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

template <typename E> hipError_t launch_scan(const ScanArgs<E>& a, int dk, int waves, hipStream_t st)
{
    if (dk == 64) return launch_scan_dk<E, 64>(a, waves, st);
    return launch_scan_dk<E, 128>(a, waves, st);
}
template hipError_t launch_scan<float>(const ScanArgs<float>&, int, int, hipStream_t);
template hipError_t launch_scan<bf16_t>(const ScanArgs<bf16_t>&, int, int, hipStream_t);

}  // namespace kla
