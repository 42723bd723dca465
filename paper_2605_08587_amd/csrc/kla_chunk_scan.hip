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
//
// The chunk loop is the only serial dependency of the whole forward, so its latency is what
// counts: the next chunk's operands are fetched from global memory into registers before the
// current chunk's products are issued, and (bf16) written to the other half of a double-buffered
// LDS area afterwards, leaving one barrier per chunk.
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
struct ScanCfg {
    static constexpr int NTH = 64 * NW;
    static constexpr int KB = DK / 16, KP = DK / 32;
    static constexpr int SLW = 16 * NW;                         // state columns per workgroup
    static constexpr int PPR = DK * (int)sizeof(E) / 16;        // 16-byte pieces per K/Q row
    static constexpr int EPP = 16 / (int)sizeof(E);             // elements per piece
    static constexpr int VPP = SLW * (int)sizeof(E) / 16;       // pieces per V/O slice row
    static constexpr int SB = 2 * (int)sizeof(typename QuadT<E>::type);
    static constexpr int OPB = 64 * DK * (int)sizeof(E);        // one K/Q operand area
    static constexpr int TPB = kTriPairs * 64 * SB;             // one T'/P operand area
    static constexpr int VB = NW * 2 * 64 * SB;                 // V slice area
    static constexpr int OLD = SLW + EPP;                       // row stride of the output staging tile
    static constexpr int OSB = 64 * OLD * (int)sizeof(E);
    // one stage: K rows | Q rows | K transposed | T' | P | V slice | gamma_i | gamma_C/gamma_i | gamma_i/||q_i||
    static constexpr int OFF_Q = OPB, OFF_KT = 2 * OPB, OFF_T = 3 * OPB, OFF_P = OFF_T + TPB, OFF_V = OFF_P + TPB,
                         OFF_EG = OFF_V + VB, OFF_ED = OFF_EG + 256, OFF_EQ = OFF_ED + 256, OFF_GC = OFF_EQ + 256,
                         STAGE = OFF_GC + 512;        // OFF_GC: gamma_C per channel (diagonal gating only)
    static constexpr int STAGES = sizeof(E) == 2 ? 2 : 1;      // fp32 operands take twice the LDS: single buffer
    static constexpr int LDS = STAGES * (STAGE + OSB);
    static constexpr int UK = (16 * PPR + NTH - 1) / NTH;       // (4-row group, piece) units of K/Q per thread
    static constexpr int UV = (16 * VPP + NTH - 1) / NTH;
    static constexpr int TP16 = TPB / 16;                       // 16-byte pieces of a T'/P area
    static constexpr int UT = (TP16 + NTH - 1) / NTH;
    static_assert(LDS <= 160 * 1024, "LDS budget of a gfx950 CU");
};

// The next chunk's operands on their way from global memory to LDS.
template <typename E, int DK, int NW, bool DIAG>
struct Prefetch {
    typedef ScanCfg<E, DK, NW> C;
    uint4 k[C::UK][4], q[C::UK][4], v[C::UV][4], t[C::UT], p[C::UT];
    uint4 kt[DIAG ? C::UK : 1][4];                   // diagonal gating: rows of the K operand of the state update
    float gc[(DK + C::NTH - 1) / C::NTH];           //                   gamma_C per channel
    float gv, gl, rq;
};

// DIAG: diagonal gating (App. B).  The decay then sits in the operands (a.k = K o Gamma, a.q = Q o Gamma, a.kt_src =
// K o (gamma_C/Gamma), unit decay vectors in the records) and the state decays per row by a.gc_vec.
template <typename E, int DK, int NW, bool DIAG>
__global__ __launch_bounds__(64 * NW) void scan_kernel(ScanArgs<E> a)
{
    typedef ScanCfg<E, DK, NW> C;
    constexpr int NTH = C::NTH, KB = C::KB, KP = C::KP, SLW = C::SLW, PPR = C::PPR, EPP = C::EPP, VPP = C::VPP;
    constexpr int OLD = C::OLD;
    typedef typename QuadT<E>::type Quad;

    __shared__ __attribute__((aligned(16))) char lds[C::LDS];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int r = lane & 15, g = lane >> 4;

    // ---- workgroup -> (sequence, head, column slice).  Consecutive workgroup ids go to different
    //      XCDs; the slices of one (sequence, head) are given ids congruent mod 8 so that they share
    //      one XCD's L2 for the K, Q, T', P reads they have in common. ---------------------------
    const int nsl = a.dv / SLW;
    const int n_states = a.n_seq > 0 ? a.n_seq : a.N;
    const int n_chains = n_states * a.H;
    const int xcd = blockIdx.x & 7, pidx = blockIdx.x >> 3;
    const int chain = (pidx / nsl) * 8 + xcd, slice = pidx % nsl;
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

    // ---- global -> registers: everything chunk c needs -------------------------------------------
    auto fetch = [&](int c, Prefetch<E, DK, NW, DIAG>& pf) {
        const long tok0 = t0 + 64L * c;
        const int clen = min(64, len - 64 * c);
        const size_t ch = (size_t)(ch0 + c) * a.H + h;
        const E* kb = a.k + (size_t)tok0 * kq_stride + (size_t)h * DK;
        const E* qb = a.q + (size_t)tok0 * kq_stride + (size_t)h * DK;
        const E* vb = a.v + (size_t)tok0 * v_stride + (size_t)h * a.dv + slice * SLW;
#pragma unroll
        for (int it = 0; it < C::UK; ++it) {
            const int u = tid + NTH * it;
            const int tq = u / PPR, piece = u % PPR;
#pragma unroll
            for (int rr = 0; rr < 4; ++rr) {
                const int row = 4 * tq + rr;
                pf.k[it][rr] = make_uint4(0, 0, 0, 0); pf.q[it][rr] = make_uint4(0, 0, 0, 0);
                if (((16 * PPR) % NTH == 0 || u < 16 * PPR) && row < clen) {
                    pf.k[it][rr] = *reinterpret_cast<const uint4*>(kb + (size_t)row * kq_stride + piece * EPP);
                    pf.q[it][rr] = *reinterpret_cast<const uint4*>(qb + (size_t)row * kq_stride + piece * EPP);
                }
                if constexpr (DIAG) {
                    pf.kt[it][rr] = make_uint4(0, 0, 0, 0);
                    if (((16 * PPR) % NTH == 0 || u < 16 * PPR) && row < clen)
                        pf.kt[it][rr] = *reinterpret_cast<const uint4*>(a.kt_src + (size_t)tok0 * kq_stride + (size_t)h * DK +
                                                                        (size_t)row * kq_stride + piece * EPP);
                }
            }
        }
        if constexpr (DIAG) {
#pragma unroll
            for (int x = 0; x < (DK + NTH - 1) / NTH; ++x)
                pf.gc[x] = (tid + NTH * x < DK) ? a.gc_vec[ch * DK + tid + NTH * x] : 0.f;
        }
#pragma unroll
        for (int it = 0; it < C::UV; ++it) {
            const int u = tid + NTH * it;
            const int tq = u / VPP, pv = u % VPP;
#pragma unroll
            for (int rr = 0; rr < 4; ++rr) {
                const int row = 4 * tq + rr;
                pf.v[it][rr] = make_uint4(0, 0, 0, 0);
                if (((16 * VPP) % NTH == 0 || u < 16 * VPP) && row < clen)
                    pf.v[it][rr] = *reinterpret_cast<const uint4*>(vb + (size_t)row * v_stride + pv * EPP);
            }
        }
        const uint4* tsrc = reinterpret_cast<const uint4*>(reinterpret_cast<const char*>(a.wsT) + ch * ws_record_bytes<E>());
        const uint4* psrc = reinterpret_cast<const uint4*>(reinterpret_cast<const char*>(a.wsP) + ch * ws_record_bytes<E>());
#pragma unroll
        for (int it = 0; it < C::UT; ++it) {
            const int i = tid + NTH * it;
            pf.t[it] = make_uint4(0, 0, 0, 0); pf.p[it] = make_uint4(0, 0, 0, 0);
            if (C::TP16 % NTH == 0 || i < C::TP16) { pf.t[it] = tsrc[i]; pf.p[it] = psrc[i]; }
        }
        pf.gv = a.wsG[ch * 128 + (tid & 63)];
        pf.gl = a.wsG[ch * 128 + 63];
        pf.rq = a.wsG[ch * 128 + 64 + (tid & 63)];       // 1/||q_i||, or 1 (read-out not normalised)
    };

    // ---- registers -> LDS stage, in MFMA operand order ----------------------------------------
    auto stash = [&](const Prefetch<E, DK, NW, DIAG>& pf, char* st) {
        E* Krq = reinterpret_cast<E*>(st);
        E* Qrq = reinterpret_cast<E*>(st + C::OFF_Q);
        E* Ktq = reinterpret_cast<E*>(st + C::OFF_KT);
        E* Vtq = reinterpret_cast<E*>(st + C::OFF_V);
#pragma unroll
        for (int it = 0; it < C::UK; ++it) {
            const int u = tid + NTH * it;
            if ((16 * PPR) % NTH == 0 || u < 16 * PPR) {
                const int tq = u / PPR, piece = u % PPR;
#pragma unroll
                for (int rr = 0; rr < 4; ++rr) {
                    store_rq_piece(Krq, KP, 4 * tq + rr, piece, pf.k[it][rr]);
                    store_rq_piece(Qrq, KP, 4 * tq + rr, piece, pf.q[it][rr]);
                }
                if constexpr (DIAG) store_tq_rows(Ktq, 2, tq, piece, pf.kt[it], 0);
                else                store_tq_rows(Ktq, 2, tq, piece, pf.k[it], 0);
            }
        }
#pragma unroll
        for (int it = 0; it < C::UV; ++it) {
            const int u = tid + NTH * it;
            if ((16 * VPP) % NTH == 0 || u < 16 * VPP) store_tq_rows(Vtq, 2, u / VPP, u % VPP, pf.v[it], 0);
        }
#pragma unroll
        for (int it = 0; it < C::UT; ++it) {
            const int i = tid + NTH * it;
            if (C::TP16 % NTH == 0 || i < C::TP16) {
                reinterpret_cast<uint4*>(st + C::OFF_T)[i] = pf.t[it];
                reinterpret_cast<uint4*>(st + C::OFF_P)[i] = pf.p[it];
            }
        }
        if (tid < 64) {
            reinterpret_cast<float*>(st + C::OFF_EG)[tid] = expf(pf.gv);            // gamma_i
            reinterpret_cast<float*>(st + C::OFF_ED)[tid] = expf(pf.gl - pf.gv);    // gamma_C / gamma_i
            reinterpret_cast<float*>(st + C::OFF_EQ)[tid] = expf(pf.gv) * pf.rq;    // scale of the Q S term
        }
        if constexpr (DIAG) {
#pragma unroll
            for (int x = 0; x < (DK + NTH - 1) / NTH; ++x)
                if (tid + NTH * x < DK) reinterpret_cast<float*>(st + C::OFF_GC)[tid + NTH * x] = pf.gc[x];
        }
    };

    // ---- the chunk recurrence for this wave's 16 columns, operands from LDS stage `st` ----------
    auto compute = [&](const char* st, E* Ost) {
        const E* Krq = reinterpret_cast<const E*>(st);
        const E* Qrq = reinterpret_cast<const E*>(st + C::OFF_Q);
        const E* Ktq = reinterpret_cast<const E*>(st + C::OFF_KT);
        const E* Trq = reinterpret_cast<const E*>(st + C::OFF_T);
        const E* Prq = reinterpret_cast<const E*>(st + C::OFF_P);
        const E* Vtq = reinterpret_cast<const E*>(st + C::OFF_V);
        const float* eg = reinterpret_cast<const float*>(st + C::OFF_EG);
        const float* ed = reinterpret_cast<const float*>(st + C::OFF_ED);

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
                const Slot<E> sl = load_slot(Trq, tri_pair(it, jp), lane);
                mma32<E>(U[it], sl, Xq[2 * jp], Xq[2 * jp + 1]);
            }
            Uq[it] = acc_to_quad<E>(U[it]);
            Udq[it] = acc_to_quad<E>(U[it] * ld_acc4(ed + 16 * it + 4 * g));
        }
        // state first: it is the only thing the next chunk waits for
        const float gC = eg[63];
#pragma unroll
        for (int kt = 0; kt < KB; ++kt) {
            if constexpr (DIAG) S[kt] = S[kt] * ld_acc4(reinterpret_cast<const float*>(st + C::OFF_GC) + 16 * kt + 4 * g);
            else                S[kt] = S[kt] * gC;
#pragma unroll
            for (int jp = 0; jp < 2; ++jp) {
                const Slot<E> sk = load_slot(Ktq, kt * 2 + jp, lane);
                mma32<E>(S[kt], sk, Udq[2 * jp], Udq[2 * jp + 1]);
            }
        }
#pragma unroll
        for (int it = 0; it < 4; ++it) {
            floatx4 o = ld_acc4(reinterpret_cast<const float*>(st + C::OFF_EQ) + 16 * it + 4 * g) * qs[it];
#pragma unroll
            for (int jp = 0; jp <= (it >> 1); ++jp) {   // P is lower triangular
                const Slot<E> sp = load_slot(Prq, tri_pair(it, jp), lane);
                mma32<E>(o, sp, Uq[2 * jp], Uq[2 * jp + 1]);
            }
#pragma unroll
            for (int e = 0; e < 4; ++e) Ost[(16 * it + 4 * g + e) * OLD + 16 * wave + r] = from_float<E>(o[e]);
        }
    };

    // ---- staged output tile -> global, 16 bytes per lane ----------------------------------------
    auto write_out = [&](int c, const E* Ost) {
        const long tok0 = t0 + 64L * c;
        const int clen = min(64, len - 64 * c);
        E* ob = a.o + (size_t)tok0 * v_stride + (size_t)h * a.dv + slice * SLW;
#pragma unroll
        for (int it = 0; it < (64 * VPP + NTH - 1) / NTH; ++it) {
            const int i = tid + NTH * it;
            const int row = i / VPP, pv = i % VPP;
            if (row < clen)
                *reinterpret_cast<uint4*>(ob + (size_t)row * v_stride + pv * EPP) =
                    *reinterpret_cast<const uint4*>(Ost + row * OLD + pv * EPP);
        }
    };

    Prefetch<E, DK, NW, DIAG> pf;
    if constexpr (C::STAGES == 2) {
        char* stage0 = lds;
        char* stage1 = lds + C::STAGE;
        E* ost0 = reinterpret_cast<E*>(lds + 2 * C::STAGE);
        E* ost1 = reinterpret_cast<E*>(lds + 2 * C::STAGE + C::OSB);
        if (nch > 0) { fetch(0, pf); stash(pf, stage0); }
        __syncthreads();
        for (int c = 0; c < nch; ++c) {
            char* cur = (c & 1) ? stage1 : stage0;
            char* nxt = (c & 1) ? stage0 : stage1;
            E* ost = (c & 1) ? ost1 : ost0;
            const bool more = c + 1 < nch;
            if (more) fetch(c + 1, pf);                  // in flight while this chunk's products run
            compute(cur, ost);
            if (more) stash(pf, nxt);
            // One barrier per chunk.  It orders (i) this chunk's staged outputs before their write-out,
            // (ii) the next chunk's operands before their use, (iii) all reads of `cur` before it is
            // overwritten one iteration later, and (iv) the write-out of chunk c-1 (done by every wave
            // before it arrives here) before `ost` of that parity is staged again in chunk c+1.
            __syncthreads();
            write_out(c, ost);
        }
    } else {
        char* stage0 = lds;
        E* ost = reinterpret_cast<E*>(lds + C::STAGE);
        for (int c = 0; c < nch; ++c) {
            __syncthreads();                             // previous chunk's operands and staging tile are free
            fetch(c, pf);
            stash(pf, stage0);
            __syncthreads();
            compute(stage0, ost);
            __syncthreads();
            write_out(c, ost);
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

template <typename E, int DK, bool DIAG>
static hipError_t launch_scan_dk(const ScanArgs<E>& a, int waves, hipStream_t st)
{
    const int n_states = a.n_seq > 0 ? a.n_seq : a.N;
    const int n_chains = n_states * a.H;
    if (n_chains == 0) return hipSuccess;
    const int nsl = a.dv / (16 * waves);
    const dim3 grid((unsigned)(((n_chains + 7) / 8) * 8 * nsl));
    switch (waves) {
        case 1: hipLaunchKernelGGL((scan_kernel<E, DK, 1, DIAG>), grid, dim3(64), 0, st, a); break;
        case 2: hipLaunchKernelGGL((scan_kernel<E, DK, 2, DIAG>), grid, dim3(128), 0, st, a); break;
        default:
            if constexpr (sizeof(E) == 2 && !DIAG) { hipLaunchKernelGGL((scan_kernel<E, DK, 4, false>), grid, dim3(256), 0, st, a); break; }
            else return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

template <typename E> hipError_t launch_scan(const ScanArgs<E>& a, int dk, int waves, hipStream_t st)
{
    if (dk == 64) return launch_scan_dk<E, 64, false>(a, waves, st);
    return launch_scan_dk<E, 128, false>(a, waves, st);
}
template hipError_t launch_scan<float>(const ScanArgs<float>&, int, int, hipStream_t);
template hipError_t launch_scan<bf16_t>(const ScanArgs<bf16_t>&, int, int, hipStream_t);

// diagonal gating: waves = 1 or 2
template <typename E> hipError_t launch_scan_diag(const ScanArgs<E>& a, int dk, int waves, hipStream_t st)
{
    if (waves != 1 && waves != 2) return hipErrorInvalidValue;
    if (dk == 64) return launch_scan_dk<E, 64, true>(a, waves, st);
    return launch_scan_dk<E, 128, true>(a, waves, st);
}
template hipError_t launch_scan_diag<float>(const ScanArgs<float>&, int, int, hipStream_t);
template hipError_t launch_scan_diag<bf16_t>(const ScanArgs<bf16_t>&, int, int, hipStream_t);

}  // namespace kla
