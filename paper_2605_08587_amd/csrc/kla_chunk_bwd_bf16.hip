// bf16 state sweeps of the backward pass (see kla_chunk_bwd.hip for the algebra and for what each sweep leaves
// behind), built like the forward's bf16 scan kernel (kla_chunk_scan_bf16.hip): operands travel global -> LDS
// directly through a ring of stages filled by a copy wave, K and Q sit as swizzled token-major rows, the
// contraction-along-a-column operands (K^T, Q^T, the V / dO tile) come from the transposing LDS read, and the
// fp32 state (or state gradient) of 16 columns per wave stays in MFMA accumulators with the permuted feature
// index of that kernel: element e of lane (r, g) of tile kt = 2 kp + b is feature 32 kp + 8 g + 4 b + e.
//
//   REV = false   forward sweep:  X = V - D_gamma K S,  U = T' X,  S <- gamma_C S + K^T diag(gamma_C/gamma_i) U;
//                 leaves S_c (before the chunk), X and U.
//   REV = true    backward sweep: dU = P^T dO + diag(gamma_C/gamma_i) K dS',  Y = M^T dU,  dV = B Y,
//                 dS <- gamma_C dS' + Q^T D_gamma dO - K^T D_gamma dV;  leaves dS'_c, Y, dV and finally dh0.
//
// A short last chunk re-reads its last valid row for the rows beyond it (as in the forward).  Those rows have
// beta = 0, zero rows and columns in T' and P^T and unit rows in M, so they reach neither U, Y (valid rows), dV nor
// the state; the one place where they would, Q^T D_gamma dO, has their gamma masked to zero.
#include "kla_bf16_ops.hpp"
#include "kla_common.hpp"
#include "kla_kernels.hpp"
#include "kla_mma.hpp"

namespace kla {

namespace {

template <int DK, int NW, bool REV>
struct SweepCfg16 {
    static constexpr int NTH = 64 * NW;                  // compute threads (the workgroup has one more wave)
    static constexpr int KB = DK / 16, KP = DK / 32;
    static constexpr int SLW = 16 * NW;                  // state columns per workgroup
    static constexpr int RB = DK * 2;                    // bytes per K/Q row
    static constexpr int PPR = DK / 8;                   // 16-byte pieces per K/Q row
    static constexpr int RPB = 1024 / RB;                // K/Q rows per 1 KiB copy block
    static constexpr int NKB = 64 / RPB;                 // copy blocks of a K (or Q) tile
    static constexpr int VRW = SLW * 2;                  // bytes per row of the V / dO slice
    static constexpr int VPP = VRW / 16;
    static constexpr int RPV = 64 / VPP;
    static constexpr int NVB = 64 / RPV;
    static constexpr int TPB = kTriPairs * 64 * 16;      // bytes of one triangular operand area
    static constexpr int NTB = (REV ? 2 : 1) * TPB / 1024;   // forward: T'; backward: M^T | P^T
    // stage: K rows | (Q rows) | T'  or  M^T | P^T | V or dO slice | gamma_i | gamma_C/gamma_i | beta_i | (1/||q_i||)
    static constexpr int OFF_Q = 64 * RB;
    static constexpr int OFF_T = (REV ? 2 : 1) * 64 * RB, OFF_P = OFF_T + TPB, OFF_V = OFF_T + (REV ? 2 : 1) * TPB,
                         OFF_EG = OFF_V + 64 * VRW, STAGE = OFF_EG + (REV ? 1024 : 768);
    static constexpr int ORB = NW <= 2 ? 96 : 160;       // row stride of a staging tile (see the forward kernel)
    static constexpr int OSB = 64 * ORB;
    // Forward: two staged tiles and the workgroup's part of the checkpoint per chunk, in two parities, all written out by
    // the store wave.  Reverse: a stage also holds Q, M^T and P^T, and what decides its speed is a ring of three stages
    // (the copies of a chunk then have two visits to arrive): the staging tiles get one parity only (a counter in LDS
    // tells the compute waves that the store wave has read them) and the checkpoint is stored by the compute waves.
    static constexpr int NPAR = REV ? 1 : 2;
    static constexpr int CKB = REV ? 0 : SLW * DK * 2;
    static constexpr int NST = (3 * STAGE + 2 * NPAR * OSB + 2 * CKB <= 160 * 1024) ? 3 : 2;   // LDS ring depth
    static constexpr int OFF_CK = NST * STAGE + 2 * NPAR * OSB;
    static constexpr int LDS = OFF_CK + 2 * CKB;
    static constexpr int NDMA = (REV ? 2 : 1) * NKB + NTB + NVB + 1;
    static_assert(LDS <= 160 * 1024 && NDMA < 64, "LDS budget of a gfx950 CU; 6-bit vmcnt");
};

}  // namespace

template <int DK, int NW, bool REV>
__global__ __launch_bounds__(64 * NW + 128) void bwd_sweep_bf16_kernel(BwdArgs<bf16_t> a)
{
    typedef SweepCfg16<DK, NW, REV> C;
    constexpr int NTH = C::NTH, KB = C::KB, KP = C::KP, SLW = C::SLW, RB = C::RB, PPR = C::PPR, RPB = C::RPB,
                  VRW = C::VRW, VPP = C::VPP, RPV = C::RPV, ORB = C::ORB, NST = C::NST;

    __shared__ __attribute__((aligned(1024))) char lds[C::LDS];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int r = lane & 15, g = lane >> 4;

    const int nsl = a.dv_dim / SLW;
    const int n_states = a.n_seq > 0 ? a.n_seq : (a.seg_G > 0 ? a.N * a.seg_G : a.N);
    const int xcd = blockIdx.x & 7, pidx = blockIdx.x >> 3;
    const int chain = (pidx / nsl) * 8 + xcd, slice = pidx % nsl;
    if (chain >= n_states * a.H) return;
    const int s = chain / a.H, h = chain % a.H;
    long t0; int len, ch0;
    if (a.cu_seqlens) { t0 = a.cu_seqlens[s]; len = a.cu_seqlens[s + 1] - (int)t0; ch0 = a.chunk_off[s]; }
    else if (a.seg_G > 0) {                              // segment sg of sequence n: chunks [sg Lc, (sg + 1) Lc)
        const int n = s / a.seg_G, sg = s % a.seg_G;
        const int tok = min(sg * a.seg_Lc * 64, a.T);
        t0 = (long)n * a.T + tok;
        len = min(a.seg_Lc * 64, a.T - tok);
        ch0 = n * a.NT + sg * a.seg_Lc;
    }
    else              { t0 = (long)s * a.T;   len = a.T;                           ch0 = s * a.NT; }
    const bool store = (a.opts & kOptNoStore) == 0;      // off: only the state is carried (segment pre-pass)
    const int nch = (len + 63) / 64;
    const int col = slice * SLW + 16 * wave + r;

    // forward: the state; backward: its gradient
    const float* init = REV ? a.d_hT : a.h0;
    floatx4 S[KB];
#pragma unroll
    for (int kt = 0; kt < KB; ++kt)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int f = 32 * (kt >> 1) + 8 * g + 4 * (kt & 1) + e;
            S[kt][e] = (init && wave < NW) ? init[((size_t)chain * DK + f) * a.dv_dim + col] : 0.f;   // not the copy wave
        }

    const size_t kq_row = (size_t)a.H * DK * 2, v_row = (size_t)a.H * a.dv_dim * 2;     // bytes between tokens
    const char* kbase = reinterpret_cast<const char*>(a.k) + (size_t)t0 * kq_row + (size_t)h * DK * 2;
    const char* qbase = reinterpret_cast<const char*>(a.q) + (size_t)t0 * kq_row + (size_t)h * DK * 2;
    const char* vbase = reinterpret_cast<const char*>(REV ? a.d_o : a.v) + (size_t)t0 * v_row + ((size_t)h * a.dv_dim + slice * SLW) * 2;
    constexpr int REC = bwd_record_bytes<bf16_t>();
    const char* tpbase = a.rec + ((size_t)ch0 * a.H + h) * REC;

    // ---- loop-invariant per-lane offsets (as in the forward kernel) -----------------------------------
    const int lrow = lane / PPR, pcol = lane % PPR;
    constexpr int NGK = 8 / RPB;                        // the swizzle has period 8 rows
    int gk[NGK];
#pragma unroll
    for (int j = 0; j < NGK; ++j)
        gk[j] = lrow * (int)kq_row + ((pcol ^ swz_piece<DK>(RPB * j + lrow)) * 16);
    const int gv = (lane / VPP) * (int)v_row + (lane % VPP) * 16;
    int oK[KP];
#pragma unroll
    for (int kp = 0; kp < KP; ++kp) oK[kp] = r * RB + (((4 * kp + g) ^ swz_piece<DK>(r)) * 16);
    const int a4 = r >> 2, c4 = r & 3;
    int oKT[KP];
#pragma unroll
    for (int kp = 0; kp < KP; ++kp) oKT[kp] = (4 * g + a4) * RB + (((4 * kp + c4) ^ swz_piece<DK>(4 * g + a4)) * 16);
    const int oV = (4 * g + a4) * VRW + (16 * wave + 4 * c4) * 2;
    const int oO = (4 * g + (r & 3)) * ORB + (16 * wave + 4 * (r >> 2)) * 2;
    const bool q_lo = (r & 3) < 2;
    const uint32_t psel = (r & 1) ? 0x03020706u : 0x05040100u;

    // ---- global -> LDS copy of everything chunk c needs ---------------------------------------------------
    auto issue = [&](int c, char* st) {
        const int clen = min(64, len - 64 * c);
        const char* kc = kbase + (size_t)(64 * c) * kq_row;
        const char* qc = qbase + (size_t)(64 * c) * kq_row;
        const char* vc = vbase + (size_t)(64 * c) * v_row;
        const char* tc = tpbase + (size_t)c * a.H * REC;
        if (clen == 64) {
            static_for<C::NKB>([&](auto i) {
                const int b = i;
                const size_t o = (size_t)(b * RPB) * kq_row;
                const int lo = gk[b % NGK];
                dma16(kc + o, lo, st + b * 1024);
                if constexpr (REV) dma16(qc + o, lo, st + C::OFF_Q + b * 1024);
            });
            static_for<C::NVB>([&](auto i) {
                const int b = i;
                dma16(vc + (size_t)(b * RPV) * v_row, gv, st + C::OFF_V + b * 1024);
            });
        } else {                                         // ragged last chunk: clamp the row
            static_for<C::NKB>([&](auto i) {
                const int b = i;
                const int row = b * RPB + lrow;
                const int lo = min(row, clen - 1) * (int)kq_row + ((pcol ^ swz_piece<DK>(row)) * 16);
                dma16(kc, lo, st + b * 1024);
                if constexpr (REV) dma16(qc, lo, st + C::OFF_Q + b * 1024);
            });
            static_for<C::NVB>([&](auto i) {
                const int b = i;
                const int row = b * RPV + lane / VPP;
                dma16(vc, min(row, clen - 1) * (int)v_row + (lane % VPP) * 16, st + C::OFF_V + b * 1024);
            });
        }
        // forward: T' (first half of the record); backward: M^T | P^T (second and third)
        static_for<C::NTB>([&](auto i) {
            const int b = i;
            dma16(tc + (REV ? C::TPB : 0) + b * 1024, lane * 16, st + C::OFF_T + b * 1024);
        });
        // gamma_i | gamma_C/gamma_i | beta_i, and for the reverse sweep 1/||q_i|| (the fifth vector of the record)
        if constexpr (REV) dma16(tc + 3 * C::TPB, lane < 48 ? lane * 16 : 1024 + (lane - 48) * 16, st + C::OFF_EG);
        else if (lane < 48) dma16(tc + 3 * C::TPB, lane * 16, st + C::OFF_EG);
    };

    // 4x4 transposition inside each quad of lanes, then one 64-bit write: lane (r, g) ends up with row 4 g + (r & 3),
    // columns 4 (r >> 2) .. + 3 of the wave's 16
    auto stage_quad = [&](u32x2 ob, char* dst) { *reinterpret_cast<u32x2*>(dst) = quad_transpose4x4(ob, q_lo, psel); };

    // ---- one chunk for this wave's 16 columns -----------------------------------------------------------
    auto compute = [&](const char* st, char* ost, char* ckb, int c, int vis) {
        const char* pS = st + lane * 16;
        const char* pV = st + C::OFF_V + oV;
        const char* pG = st + C::OFF_EG + 16 * g;
        auto kslot = [&](int it, int kp) {
            return ld16(st + oK[kp] + 16 * it * RB);
        };
        auto ktslot = [&](int kt, int jp, int base, u32x2& q0, u32x2& q1) {      // base 0: K^T, OFF_Q: Q^T
            const int kp = kt >> 1, b = kt & 1;
            const char* p = st + oKT[kp] + base + 32 * jp * RB + 8 * b;
            q0 = lds_read_tr(p);
            q1 = lds_read_tr(p + 16 * RB);
        };

        const float gC = *reinterpret_cast<const float*>(st + C::OFF_EG + 63 * 4);
        u32x2 Sq[KB];
#pragma unroll
        for (int kt = 0; kt < KB; ++kt) { Sq[kt] = to_quad(S[kt]); S[kt] = S[kt] * gC; }
        if (store) {
            // checkpoint, transposed ([column][feature]): features 32 kp + 8 g .. + 7 of this lane's column are 16
            // contiguous bytes.
            if constexpr (C::CKB > 0) {
                // staged in LDS for the store wave; the 16-byte pieces of a column are XORed with the column so that the
                // eight lanes a 128-bit write serves per cycle fall into different banks
                const int cl = 16 * wave + r;
                char* ck = ckb + cl * (DK * 2);
#pragma unroll
                for (int kp = 0; kp < KP; ++kp) {
                    const u32x4 w = {Sq[2 * kp].x, Sq[2 * kp].y, Sq[2 * kp + 1].x, Sq[2 * kp + 1].y};
                    st16(ck + (((4 * kp + g) ^ (cl & 7)) * 16), w);
                }
            } else {
                bf16_t* ck = (REV ? a.ds_chk : a.s_chk) + (((size_t)(ch0 + c) * a.H + h) * a.dv_dim + col) * DK + 8 * g;
#pragma unroll
                for (int kp = 0; kp < KP; ++kp) {
                    const u32x4 w = {Sq[2 * kp].x, Sq[2 * kp].y, Sq[2 * kp + 1].x, Sq[2 * kp + 1].y};
                    __builtin_nontemporal_store(w, reinterpret_cast<u32x4*>(ck + 32 * kp));
                }
            }
        }

        // ---- K S or K dS'
        floatx4 ks[4];
#pragma unroll
        for (int it = 0; it < 4; ++it) ks[it] = floatx4{0.f, 0.f, 0.f, 0.f};
        u32x4 ka[2][4];
#pragma unroll
        for (int it = 0; it < 4; ++it) ka[0][it] = kslot(it, 0);
#pragma unroll
        for (int kp = 0; kp < KP; ++kp) {
            if (kp + 1 < KP) {
#pragma unroll
                for (int it = 0; it < 4; ++it) ka[(kp + 1) & 1][it] = kslot(it, kp + 1);
            }
#pragma unroll
            for (int it = 0; it < 4; ++it) mma_bf16(ks[it], ka[kp & 1][it], Sq[2 * kp], Sq[2 * kp + 1]);
        }
        u32x2 vq[4];
        floatx4 egv[4], edv[4];
#pragma unroll
        for (int it = 0; it < 4; ++it) {
            vq[it] = lds_read_tr(pV + 16 * it * VRW);
            egv[it] = ld_f4(pG + 64 * it);
            edv[it] = ld_f4(pG + 256 + 64 * it);
        }
        u32x4 tsl[kTriPairs];
#pragma unroll
        for (int i = 0; i < kTriPairs; ++i) tsl[i] = ld16(pS + C::OFF_T + i * 1024);
        u32x2 kt[2][KB][2];                              // [token pair jp][state tile][token block]

        if constexpr (!REV) {
            u32x2 Xq[4];
#pragma unroll
            for (int it = 0; it < 4; ++it) {
                Xq[it] = to_quad(quad_to_f(vq[it]) - egv[it] * ks[it]);       // eq. (6), right-hand side without B
                stage_quad(Xq[it], ost + oO + 16 * it * ORB);
            }
#pragma unroll
            for (int t = 0; t < KB; ++t) ktslot(t, 0, 0, kt[0][t][0], kt[0][t][1]);
            floatx4 U[4];
#pragma unroll
            for (int it = 0; it < 4; ++it) {
                U[it] = floatx4{0.f, 0.f, 0.f, 0.f};
                mma_bf16(U[it], tsl[tri_pair(it, 0)], Xq[0], Xq[1]);
            }
            mma_bf16(U[2], tsl[tri_pair(2, 1)], Xq[2], Xq[3]);
            mma_bf16(U[3], tsl[tri_pair(3, 1)], Xq[2], Xq[3]);
#pragma unroll
            for (int t = 0; t < KB; ++t) ktslot(t, 1, 0, kt[1][t][0], kt[1][t][1]);
            u32x2 Udq[4];
#pragma unroll
            for (int it = 0; it < 4; ++it) Udq[it] = to_quad(U[it] * edv[it]);   // U itself is not kept: the assembly forms it again from T' and X
#pragma unroll
            for (int t = 0; t < KB; ++t) mma_bf16(S[t], kt[0][t][0], kt[0][t][1], Udq[0], Udq[1]);
#pragma unroll
            for (int t = 0; t < KB; ++t) mma_bf16(S[t], kt[1][t][0], kt[1][t][1], Udq[2], Udq[3]);
        } else {
            const int clen = min(64, len - 64 * c);
            u32x4 psl[kTriPairs];
#pragma unroll
            for (int i = 0; i < kTriPairs; ++i) psl[i] = ld16(pS + C::OFF_P + i * 1024);
            // ---- dU = diag(gamma_C/gamma_i) K dS' + P^T dO   (P^T upper triangular)
            floatx4 dU[4];
#pragma unroll
            for (int it = 0; it < 4; ++it) dU[it] = edv[it] * ks[it];
            mma_bf16(dU[0], psl[triu_pair(0, 0)], vq[0], vq[1]);
            mma_bf16(dU[1], psl[triu_pair(1, 0)], vq[0], vq[1]);
#pragma unroll
            for (int it = 0; it < 4; ++it) mma_bf16(dU[it], psl[triu_pair(it, 1)], vq[2], vq[3]);
            u32x2 dUq[4];
#pragma unroll
            for (int it = 0; it < 4; ++it) dUq[it] = to_quad(dU[it]);
#pragma unroll
            for (int t = 0; t < KB; ++t) ktslot(t, 0, C::OFF_Q, kt[0][t][0], kt[0][t][1]);
            // ---- Y = M^T dU
            floatx4 Y[4];
#pragma unroll
            for (int it = 0; it < 4; ++it) Y[it] = floatx4{0.f, 0.f, 0.f, 0.f};
            mma_bf16(Y[0], tsl[triu_pair(0, 0)], dUq[0], dUq[1]);
            mma_bf16(Y[1], tsl[triu_pair(1, 0)], dUq[0], dUq[1]);
#pragma unroll
            for (int it = 0; it < 4; ++it) mma_bf16(Y[it], tsl[triu_pair(it, 1)], dUq[2], dUq[3]);
#pragma unroll
            for (int t = 0; t < KB; ++t) ktslot(t, 1, C::OFF_Q, kt[1][t][0], kt[1][t][1]);
            u32x2 gdOq[4], gdXq[4];
            if constexpr (C::NPAR == 1) {
                // one staging parity: the store wave must have read the tiles of the previous visit (it does so right
                // after the barrier, a whole visit ago; the wait is a formality, and bounded)
                for (int spin = 0; *reinterpret_cast<const volatile int*>(lds + NST * C::STAGE + 64) < vis - 1 && spin < (1 << 15); ++spin)
                    __builtin_amdgcn_s_sleep(1);
                asm volatile("" ::: "memory");
            }
#pragma unroll
            for (int it = 0; it < 4; ++it) {
                const floatx4 dx = Y[it] * ld_f4(pG + 512 + 64 * it);           // dV = B Y
                stage_quad(to_quad(Y[it]), ost + oO + 16 * it * ORB);
                stage_quad(to_quad(dx), ost + C::OSB + oO + 16 * it * ORB);
                floatx4 eg = egv[it];
#pragma unroll
                for (int e = 0; e < 4; ++e) eg[e] = (16 * it + 4 * g + e < clen) ? eg[e] : 0.f;   // rows past a ragged end
                gdOq[it] = to_quad(eg * ld_f4(pG + 768 + 64 * it) * quad_to_f(vq[it]));   // D_gamma dO / ||q||
                gdXq[it] = to_quad(-(eg * dx));
            }
            // ---- dS = gamma_C dS' + Q^T D_gamma dO - K^T D_gamma dV
#pragma unroll
            for (int t = 0; t < KB; ++t) mma_bf16(S[t], kt[0][t][0], kt[0][t][1], gdOq[0], gdOq[1]);
#pragma unroll
            for (int t = 0; t < KB; ++t) mma_bf16(S[t], kt[1][t][0], kt[1][t][1], gdOq[2], gdOq[3]);
#pragma unroll
            for (int t = 0; t < KB; ++t) ktslot(t, 0, 0, kt[0][t][0], kt[0][t][1]);
#pragma unroll
            for (int t = 0; t < KB; ++t) ktslot(t, 1, 0, kt[1][t][0], kt[1][t][1]);
#pragma unroll
            for (int t = 0; t < KB; ++t) mma_bf16(S[t], kt[0][t][0], kt[0][t][1], gdXq[0], gdXq[1]);
#pragma unroll
            for (int t = 0; t < KB; ++t) mma_bf16(S[t], kt[1][t][0], kt[1][t][1], gdXq[2], gdXq[3]);
        }
    };

    // Everything chunk c leaves in memory goes out through one wave that does nothing else, 16 bytes per lane: the two
    // staged tiles (forward: X, U; backward: Y, dV) and the workgroup's columns of the checkpoint.  The compute waves
    // never issue a global store, so they never stand in the store queue.
    auto write_out = [&](int c, const char* ost, const char* ckb) {
        const int clen = min(64, len - 64 * c);
        const size_t off = (size_t)(t0 + 64L * c) * v_row + ((size_t)h * a.dv_dim + slice * SLW) * 2;
        char* o0 = reinterpret_cast<char*>(REV ? a.Y : a.X) + off;
        char* o1 = reinterpret_cast<char*>(a.dv) + off;          // backward sweep only
#pragma unroll
        for (int it = 0; it < VPP; ++it) {
            const int i = lane + 64 * it;
            const int row = i / VPP, pv = i % VPP;
            if (row < clen) {
                __builtin_nontemporal_store(ld16(ost + row * ORB + pv * 16), reinterpret_cast<u32x4*>(o0 + (size_t)row * v_row + pv * 16));
                if constexpr (REV) __builtin_nontemporal_store(ld16(ost + C::OSB + row * ORB + pv * 16), reinterpret_cast<u32x4*>(o1 + (size_t)row * v_row + pv * 16));
            }
        }
        if constexpr (C::CKB > 0) {
            char* ck = reinterpret_cast<char*>(REV ? a.ds_chk : a.s_chk) +
                       (((size_t)(ch0 + c) * a.H + h) * a.dv_dim + slice * SLW) * (DK * 2);
#pragma unroll
            for (int it = 0; it < C::CKB / 1024; ++it) {
                const int i = lane + 64 * it;
                const int cl = i / PPR, pp = i % PPR;        // column of the workgroup, physical piece
                __builtin_nontemporal_store(ld16(ckb + i * 16), reinterpret_cast<u32x4*>(ck + cl * (DK * 2) + ((pp ^ (cl & 7)) * 16)));
            }
        }
    };

    char* ost0 = lds + NST * C::STAGE;
    char* ost1 = C::NPAR == 2 ? ost0 + 2 * C::OSB : ost0;
    char* ckb0 = lds + C::OFF_CK;
    // last visit whose staged tiles the store wave has read (one staging parity only); in the padding of the first
    // staging row (a row holds at most 64 of its ORB = 96 bytes)
    int* oflag = reinterpret_cast<int*>(ost0 + 64);
    if (C::NPAR == 1 && tid == 0) *oflag = -1;
    // chunks are visited in the order i = 0 .. nch-1; the backward sweep starts at the last chunk
    auto chunk_of = [&](int i) { return REV ? nch - 1 - i : i; };

    if (wave == NW + 1) {
        // ---- the store wave: after the barrier that ends visit i, chunk_of(i) is complete in the staging areas of
        //      parity i & 1, which the compute waves write again only in visit i + 2, behind the barrier this wave
        //      reaches next
        __syncthreads();
        for (int i = 0; i < nch; ++i) {
            __syncthreads();
            if (store) write_out(chunk_of(i), (i & 1) ? ost1 : ost0, ckb0 + (i & 1) * C::CKB);
            if constexpr (C::NPAR == 1) {
                asm volatile("" ::: "memory");
                if (lane == 0) *reinterpret_cast<volatile int*>(oflag) = i;      // behind the reads above, in order
            }
        }
        return;
    }

    if (wave == NW) {
        // ---- the copy wave: keeps the next NST-1 chunks on their way while one is computed -----------------
#pragma unroll
        for (int p = 0; p < NST - 1; ++p)
            if (p < nch) issue(chunk_of(p), lds + p * C::STAGE);
        if (NST == 3 && nch > 1) wait_vmcnt<C::NDMA>(); else wait_vmcnt<0>();
        __syncthreads();
        int spre = NST - 1;
        for (int i = 0; i < nch; ++i) {
            const bool ahead = i + NST - 1 < nch;
            if (ahead) issue(chunk_of(i + NST - 1), lds + spre * C::STAGE);
            if (NST == 3 && ahead) wait_vmcnt<C::NDMA>(); else wait_vmcnt<0>();
            __syncthreads();
            spre = (spre + 1 == NST) ? 0 : spre + 1;
        }
        return;
    }

    // ---- compute waves (same barrier discipline as the forward kernel) --------------------------------------
    __syncthreads();
    int scur = 0;
    for (int i = 0; i < nch; ++i) {
        const int c = chunk_of(i);
        char* ost = (i & 1) ? ost1 : ost0;
        compute(lds + scur * C::STAGE, ost, ckb0 + (i & 1) * C::CKB, c, i);
        __syncthreads();
        scur = (scur + 1 == NST) ? 0 : scur + 1;
    }

    if (REV && a.dh0) {
#pragma unroll
        for (int kt = 0; kt < KB; ++kt)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int f = 32 * (kt >> 1) + 8 * g + 4 * (kt & 1) + e;
                a.dh0[((size_t)chain * DK + f) * a.dv_dim + col] = S[kt][e];
            }
    }
}

// =================================================================================================
// per chunk-head contractions (bf16): the algebra of bwd_assemble_kernel in kla_chunk_bwd.hip on direct
// global -> LDS copies.  Every operand sits in LDS as plain swizzled rows: the slab of S^T and dS'^T (64 rows of
// d_k) and the K, Q tiles exactly like a K tile of the sweeps, the [64 tokens x 64 columns] slabs of dO, U, Y, X
// like a K tile of d_k = 64.  Operands contracted along a row are two 64-bit reads, operands contracted down a
// column (S^T, dS'^T, K, Q) come from the transposing read, which makes lane r of an output tile the feature
// 32 kp + 8 (r / 4) + 4 b + r % 4 of tile 2 kp + b; the K and Q values that meet those outputs are read the same
// way, and the 4x4 transposition before the staged write-out puts the features back in order.
// A short last chunk re-reads its last valid row for the rows beyond it; the rows of A o dP and D', of the
// <.,k> sums and of dg that belong to those rows are masked to zero.
// =================================================================================================
namespace {
// acc + x.lo * y.lo + x.hi * y.hi for two packed bf16 pairs (v_dot2c_f32_bf16)
__device__ __forceinline__ float dot2_bf16(uint32_t x, uint32_t y, float acc)
{
    typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
    return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, x), __builtin_bit_cast(bf16x2_t, y), acc, false);
}
}  // namespace

template <int DK>
__global__ __launch_bounds__(256, 2) void bwd_assemble_bf16_kernel(BwdArgs<bf16_t> a)
{
    constexpr int KB = DK / 16, KP = DK / 32;
    constexpr int RB = DK * 2, PPR = DK / 8, RPB = 1024 / RB, NKB = 64 / RPB;      // [64 x d_k] tiles
    constexpr int RBA = 64, NAB = 4;                 // [64 tokens x 32 columns] slabs: 4 blocks of 16 rows of 64 bytes
    constexpr int TK = 64 * RB, TS = 32 * RB, NSB = TS / 1024, TA = 64 * RBA;
    constexpr int kLd = 68, MB = 64 * kLd * 4;
    // first phase, two buffers of one 32-column slab each: S^T | dS'^T | dO | U | Y | X (U is formed here, from T' and X)
    constexpr int OFF_S = 0, OFF_DS = TS, OFF_DO = 2 * TS, OFF_U = OFF_DO + TA, OFF_Y = OFF_U + TA, OFF_X = OFF_Y + TA;
    constexpr int SLAB = 2 * TS + 4 * TA;
    constexpr int PH1 = 2 * SLAB;
    // second phase: K | Q | A o dP | D'.  K and Q are fetched into the first buffer while the last slab (always in the
    // second one: d_v / 32 is even) is being used.
    constexpr int OFF_K = 0, OFF_Q = TK, OFF_E1 = 2 * TK, OFF_DP = 2 * TK + MB;
    constexpr int PH2 = 2 * TK + 2 * MB;
    constexpr int BIG = PH1 > PH2 ? PH1 : PH2;
    static_assert(2 * TK <= SLAB, "the K and Q tiles fit one slab buffer");
    constexpr int ORQ = RB + 16;                     // row stride of the dq / dk staging tiles (over A o dP and D')
    static_assert(64 * ORQ <= MB, "staging tiles fit the fp32 matrices they replace");
    __shared__ __attribute__((aligned(1024))) char lds[BIG];
    __shared__ __attribute__((aligned(1024))) char tp_s[kTriPairs * 1024];       // T' of the chunk, as the record holds it
    __shared__ __attribute__((aligned(16))) float eg_s[64], ed_s[64], beta_s[64], invden_s[64], rq_s[64], g_s[64], yx_s[64],
        dg_s[64], dbeta_s[64];
    __shared__ float red_s[8];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int r = lane & 15, g = lane >> 4;

    const int h = blockIdx.x % a.H;
    const int cg = blockIdx.x / a.H;
    const ChunkPos cp = chunk_pos(a.cu_seqlens, a.chunk_off, a.n_seq, a.T, a.NT, cg);
    const long tok0 = cp.tok0;
    const int clen = cp.clen;
    const size_t kq_row = (size_t)a.H * DK * 2, v_row = (size_t)a.H * a.dv_dim * 2;
    const char* rec = a.rec + (size_t)blockIdx.x * bwd_record_bytes<bf16_t>();
    // With the normalised read-out (Sec. 3.3) the query that meets the state is q^ = q / ||q||.  Scaling the rows of dO
    // by 1/||q_i|| wherever they meet U or S gives dQ' = diag(1/||q||) dL/dq^ directly, (A o dP')^T Q is what dK
    // needs, q_i . dQ'_i is what dg needs, and dq_i = dQ'_i - (q_i . dQ'_i) q_i / ||q_i||^2 at the end.
    const bool norm_q = (a.opts & kOptNormalizeQ) != 0;
    {
        const float* vec = reinterpret_cast<const float*>(rec + 3 * ws_half_bytes<bf16_t>());
        float* dst = wave == 0 ? eg_s : (wave == 1 ? ed_s : (wave == 2 ? beta_s : invden_s));
        dst[lane] = vec[tid];
        if (wave == 1) rq_s[lane] = vec[256 + lane];
        if (wave == 0) g_s[lane] = lane < clen ? a.log_alpha[(size_t)(tok0 + lane) * a.H + h] : 0.f;
    }

    // ---- per-lane offsets ---------------------------------------------------------------------------
    // copies of [rows x d_k] tiles and of [64 x 32] slabs, swizzled on the global side (the 16-byte column index is
    // XORed with swz_piece(row) resp. (row / 2) % 4)
    const int lrow = lane / PPR, pcol = lane % PPR;
    const int lrowA = lane >> 2, pcolA = lane & 3;
    // The per-lane part of a checkpoint copy's address depends on the block only through b % NGK (the swizzle has
    // period 8 rows).  Rows past the end of a ragged chunk re-read its last one.
    const bool full = clen == 64;
    constexpr int NGK = 8 / RPB;
    int gst[NGK];
#pragma unroll
    for (int j = 0; j < NGK; ++j) gst[j] = lrow * RB + ((pcol ^ swz_piece<DK>(RPB * j + lrow)) * 16);
    const int gsl = lrowA * (int)v_row + ((pcolA ^ ((lrowA >> 1) & 3)) * 16);
    auto copy_tile = [&](const char* src, size_t stride, char* dst, int b0, int b1) {       // blocks [b0, b1) of a [64 x d_k] tile
        for (int b = b0; b < b1; ++b) {
            const int row = b * RPB + lrow;
            dma16(src, min(row, clen - 1) * (int)stride + ((pcol ^ swz_piece<DK>(row)) * 16), dst + b * 1024);
        }
    };
    auto copy_state = [&](const char* src, char* dst) {                                      // 32 rows of a checkpoint: never ragged
        static_for<NSB>([&](auto bb) {
            const int b = bb;
            dma16(src + b * RPB * RB, gst[b % NGK], dst + b * 1024);
        });
    };
    auto copy_slab = [&](const char* src, char* dst) {                                       // 4 blocks of 16 token rows x 64 bytes
        static_for<NAB>([&](auto bb) {
            const int b = bb;
            if (full) dma16(src + (size_t)(b * 16) * v_row, gsl, dst + b * 1024);
            else      dma16(src, min(b * 16 + lrowA, clen - 1) * (int)v_row + ((pcolA ^ ((lrowA >> 1) & 3)) * 16), dst + b * 1024);
        });
    };
    // row-contracted operand of a slab: token row 16 t + r, contraction indices {4 g .. +3 | 16 + 4 g .. +3}
    const int arow = r * RBA + (g & 1) * 8, asw = (r >> 1) & 3;
    const int acol0 = ((g >> 1) ^ asw) * 16, acol1 = ((2 + (g >> 1)) ^ asw) * 16;
    auto aslot = [&](const char* tile, int t, u32x2& q0, u32x2& q1) {
        const char* p = tile + 16 * t * RBA + arow;
        q0 = *reinterpret_cast<const u32x2*>(p + acol0);
        q1 = *reinterpret_cast<const u32x2*>(p + acol1);
    };
    // column-contracted operand of a [64 x d_k] tile through the transposing read (as K^T in the sweeps)
    const int a4 = r >> 2, c4 = r & 3;
    int oKT[KP];
#pragma unroll
    for (int kp = 0; kp < KP; ++kp) oKT[kp] = (4 * g + a4) * RB + (((4 * kp + c4) ^ swz_piece<DK>(4 * g + a4)) * 16);
    auto tslot = [&](const char* tile, int kt, int jp, u32x2& q0, u32x2& q1) {
        const int kp = kt >> 1, b = kt & 1;
        const char* p = tile + oKT[kp] + 32 * jp * RB + 8 * b;
        q0 = lds_read_tr(p);
        q1 = lds_read_tr(p + 16 * RB);
    };

    // U = T' X is not read back from the forward sweep but formed again, slab by slab: the T' tile pairs of this wave's 16
    // rows (A operands, copied from the record into LDS once), the X slab through the transposing read (B operands), the
    // result put into the slab's U area in the layout a copied slab has.  Per lane: where its 8 bytes of an X row sit.
    for (int i = wave; i < kTriPairs; i += 4) dma16(rec + i * 1024, lane * 16, tp_s + i * 1024);   // lands with the first slab
    // (column tile 0; tile 1 is two 16-byte pieces further, i.e. the same offsets with bit 5 flipped)
    const int xo = (4 * g + a4) * RBA + ((((c4 >> 1)) ^ ((2 * g + (a4 >> 1)) & 3)) * 16) + (c4 & 1) * 8;
    const int urow = 16 * wave + 4 * g + (r & 3);            // after the 4x4 transposition a lane holds 4 columns of one row
    const int uo = urow * RBA + ((((r >> 3)) ^ ((urow >> 1) & 3)) * 16) + ((r >> 2) & 1) * 8;
    floatx4 dQ[KB], dKr[KB], dKw[KB], dP[4], N1[4];
#pragma unroll
    for (int ct = 0; ct < KB; ++ct) { dQ[ct] = floatx4{0.f, 0.f, 0.f, 0.f}; dKr[ct] = dQ[ct]; dKw[ct] = dQ[ct]; }
#pragma unroll
    for (int jt = 0; jt < 4; ++jt) { dP[jt] = floatx4{0.f, 0.f, 0.f, 0.f}; N1[jt] = dP[jt]; }
    float yx = 0.f, sdot = 0.f;

    // ---- first phase: everything that contracts over d_v, 32 columns at a time; the next slab (after the last
    //      one: K and Q) is on its way while a slab is used ---------------------------------------------------
    const char* Sg = reinterpret_cast<const char*>(a.s_chk) + (size_t)blockIdx.x * DK * a.dv_dim * 2;
    const char* dSg = reinterpret_cast<const char*>(a.ds_chk) + (size_t)blockIdx.x * DK * a.dv_dim * 2;
    const size_t vrow0 = (size_t)tok0 * v_row + (size_t)h * a.dv_dim * 2;
    auto issue_slab = [&](int sl, char* buf) {
        if (wave == 0)      copy_state(Sg + (size_t)(32 * sl) * RB, buf + OFF_S);
        else if (wave == 1) copy_state(dSg + (size_t)(32 * sl) * RB, buf + OFF_DS);
        else if (wave == 2) copy_slab(reinterpret_cast<const char*>(a.d_o) + vrow0 + 64 * sl, buf + OFF_DO);
        else {
            copy_slab(reinterpret_cast<const char*>(a.Y) + vrow0 + 64 * sl, buf + OFF_Y);
            copy_slab(reinterpret_cast<const char*>(a.X) + vrow0 + 64 * sl, buf + OFF_X);
        }
    };
    const int ns = a.dv_dim / 32;
    issue_slab(0, lds);
    for (int sl = 0; sl < ns; ++sl) {
        const char* buf = lds + (sl & 1) * SLAB;
        wait_vmcnt<0>();
        __syncthreads();                             // slab sl has landed; slab sl-1 is no longer read
        if (sl + 1 < ns) issue_slab(sl + 1, lds + ((sl + 1) & 1) * SLAB);
        else {
            const char* kb = reinterpret_cast<const char*>(a.k) + (size_t)tok0 * kq_row + (size_t)h * DK * 2;
            const char* qb = reinterpret_cast<const char*>(a.q) + (size_t)tok0 * kq_row + (size_t)h * DK * 2;
            if (wave < 2) copy_tile(kb, kq_row, lds + OFF_K, wave * (NKB / 2), (wave + 1) * (NKB / 2));
            else          copy_tile(qb, kq_row, lds + OFF_Q, (wave - 2) * (NKB / 2), (wave - 1) * (NKB / 2));
        }
        // U = T' X: this wave's 16 rows of the slab.  (The lane index is passed through an empty asm so that the two
        // transposition constants are formed here and not kept in registers until the staging of dq and dk, where the
        // kernel has none to spare.)
        int r1 = r;
        asm volatile("" : "+v"(r1));
        const bool q_lo = (r1 & 3) < 2;
        const uint32_t psel = (r1 & 1) ? 0x03020706u : 0x05040100u;
#pragma unroll
        for (int ct = 0; ct < 2; ++ct) {
            floatx4 u = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int jp = 0; jp < 2; ++jp) {
                if (2 * jp <= wave) {                      // T' is lower triangular (wave-uniform)
                    const char* xp = buf + OFF_X + 32 * jp * RBA + (xo ^ (32 * ct));
                    mma_bf16(u, ld16(tp_s + tri_pair(wave, jp) * 1024 + lane * 16), lds_read_tr(xp), lds_read_tr(xp + 16 * RBA));
                }
            }
            *reinterpret_cast<u32x2*>(lds + (sl & 1) * SLAB + OFF_U + (uo ^ (32 * ct))) = quad_transpose4x4(to_quad(u), q_lo, psel);
        }
        // Y_i . X_i and <dS', S>: plain 16-byte pieces, the swizzle is the same for both tiles of a pair
        {
            const u32x4 y = ld16(buf + OFF_Y + tid * 16), x = ld16(buf + OFF_X + tid * 16);
#pragma unroll
            for (int m = 0; m < 4; ++m) yx = dot2_bf16(y[m], x[m], yx);
#pragma unroll
            for (int pc = 0; pc < TS / 16 / 256; ++pc) {
                const int o = (tid + 256 * pc) * 16;
                const u32x4 sv = ld16(buf + OFF_S + o), dv = ld16(buf + OFF_DS + o);
#pragma unroll
                for (int m = 0; m < 4; ++m) sdot = dot2_bf16(sv[m], dv[m], sdot);
            }
        }
        __syncthreads();                             // every wave's rows of U are in the slab
        u32x2 do0, do1, u0, u1, y0, y1;
        aslot(buf + OFF_DO, wave, do0, do1);
        aslot(buf + OFF_U, wave, u0, u1);
        aslot(buf + OFF_Y, wave, y0, y1);
#pragma unroll
        for (int ct = 0; ct < KB; ++ct) {
            u32x2 s0, s1, d0, d1;
            tslot(buf + OFF_S, ct, 0, s0, s1);
            tslot(buf + OFF_DS, ct, 0, d0, d1);
            mma_bf16(dQ[ct], do0, do1, s0, s1);            // dO S^T
            mma_bf16(dKr[ct], y0, y1, s0, s1);             // Y S^T
            mma_bf16(dKw[ct], u0, u1, d0, d1);             // U dS'^T
        }
        static_for<4>([&](auto jt) {
            if (jt <= wave) {                              // lower-triangular tiles only
                u32x2 b0, b1;
                aslot(buf + OFF_U, jt, b0, b1);
                mma_bf16(dP[jt], do0, do1, b0, b1);        // dO U^T
                mma_bf16(N1[jt], y0, y1, b0, b1);          // Y U^T
            }
        });
    }
    if (wave == 0) {                                 // g_i = log gamma_i
        float x = g_s[lane];
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) { const float y = __shfl_up(x, off, kWave); if (lane >= off) x += y; }
        g_s[lane] = x * 1.44269504088896341f;        // in units of log 2: the decay ratios below are exp2 of differences
    }
    {   // D_gamma dO S^T,  -D_gamma dX S^T (dX = B Y),  diag(gamma_C/gamma_i) U dS'^T
        const floatx4 egv = ld_f4(reinterpret_cast<const char*>(eg_s + 16 * wave + 4 * g));
        const floatx4 edv = ld_f4(reinterpret_cast<const char*>(ed_s + 16 * wave + 4 * g));
        const floatx4 ngb = -(egv * ld_f4(reinterpret_cast<const char*>(beta_s + 16 * wave + 4 * g)));
        const floatx4 egq = egv * ld_f4(reinterpret_cast<const char*>(rq_s + 16 * wave + 4 * g));
#pragma unroll
        for (int ct = 0; ct < KB; ++ct) { dQ[ct] = dQ[ct] * egq; dKr[ct] = dKr[ct] * ngb; dKw[ct] = dKw[ct] * edv; }
    }
    yx += __shfl_xor(yx, 1, kWave); yx += __shfl_xor(yx, 2, kWave);      // the 4 threads of a row are neighbours
    if ((tid & 3) == 0) yx_s[tid >> 2] = yx;
    sdot = wave_sum(sdot);
    if (lane == 0) red_s[wave] = sdot;
    wait_vmcnt<0>();                                 // this wave's part of K and Q
    __syncthreads();                                 // the slab areas are dead from here on

    // ---- second phase: A o dP and D' = -A^- o (Y U^T) as fp32 matrices ------------------------------------------
    float* E1 = reinterpret_cast<float*>(lds + OFF_E1);
    float* Dp = reinterpret_cast<float*>(lds + OFF_DP);
    static_for<4>([&](auto jt) {
        const int j = 16 * jt + r;
        const float gj = g_s[j];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int i = 16 * wave + 4 * g + e;
            const float dec = (jt <= wave && j <= i && i < clen) ? __builtin_amdgcn_exp2f(g_s[i] - gj) : 0.f;
            E1[i * kLd + j] = dec * rq_s[i] * dP[jt][e];
            Dp[i * kLd + j] = (j < i) ? -dec * N1[jt][e] : 0.f;
        }
    });
    __syncthreads();

    // K and Q of this wave's rows as accumulator tiles: token 16 wave + 4 g + e, feature of (tile ct, lane r)
    auto kacc = [&](int off, int ct) {
        u32x2 q0, q1;
        tslot(lds + off, ct, wave >> 1, q0, q1);
        return quad_to_f((wave & 1) ? q1 : q0);
    };
    floatx4 rowmask;                                 // 1 for the rows of the chunk, 0 past a ragged end
#pragma unroll
    for (int e = 0; e < 4; ++e) rowmask[e] = (16 * wave + 4 * g + e < clen) ? 1.f : 0.f;
    float zsum = 0.f;                                // sum_i (gamma_C/gamma_i) k_i . (dS' U_i)
#pragma unroll
    for (int ct = 0; ct < KB; ++ct) {
        const floatx4 kk = kacc(OFF_K, ct);
#pragma unroll
        for (int e = 0; e < 4; ++e) zsum += rowmask[e] * dKw[ct][e] * kk[e];
    }
    zsum = wave_sum(zsum);
    if (lane == 0) red_s[4 + wave] = zsum;

    floatx4 E2[KB];
#pragma unroll
    for (int ct = 0; ct < KB; ++ct) E2[ct] = floatx4{0.f, 0.f, 0.f, 0.f};
    const int row_a = 16 * wave + r;
    auto rows_slot = [&](const float* m, int jp, u32x2& q0, u32x2& q1) {
        q0 = to_quad(ld_f4(reinterpret_cast<const char*>(m + row_a * kLd + 32 * jp + 4 * g)));
        q1 = to_quad(ld_f4(reinterpret_cast<const char*>(m + row_a * kLd + 32 * jp + 16 + 4 * g)));
    };
    auto cols_slot = [&](const float* m, const float* scale, int jp, u32x2& q0, u32x2& q1) {
        floatx4 x0, x1;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int i0 = 32 * jp + 4 * g + e, i1 = i0 + 16;
            x0[e] = m[i0 * kLd + row_a]; x1[e] = m[i1 * kLd + row_a];
            if (scale) { x0[e] *= scale[i0]; x1[e] *= scale[i1]; }
        }
        q0 = to_quad(x0); q1 = to_quad(x1);
    };
    static_for<2>([&](auto jp) {
        if (jp <= (wave >> 1)) {
            u32x2 e0, e1, d0, d1;
            rows_slot(E1, jp, e0, e1);
            rows_slot(Dp, jp, d0, d1);
#pragma unroll
            for (int ct = 0; ct < KB; ++ct) {
                u32x2 k0, k1;
                tslot(lds + OFF_K, ct, jp, k0, k1);
                mma_bf16(dQ[ct], e0, e1, k0, k1);          // (A o dP) K
                mma_bf16(E2[ct], d0, d1, k0, k1);          // D' K
            }
        }
        if (jp >= (wave >> 1)) {
            u32x2 e0, e1, d0, d1;
            cols_slot(E1, nullptr, jp, e0, e1);
            cols_slot(Dp, beta_s, jp, d0, d1);
#pragma unroll
            for (int ct = 0; ct < KB; ++ct) {
                u32x2 k0, k1, q0, q1;
                tslot(lds + OFF_Q, ct, jp, q0, q1);
                tslot(lds + OFF_K, ct, jp, k0, k1);
                mma_bf16(dKw[ct], e0, e1, q0, q1);         // (A o dP)^T Q
                mma_bf16(dKw[ct], d0, d1, k0, k1);         // (B D')^T K
            }
        }
    });

    // ---- rows: dbeta, dg, the beta term of dK -----------------------------------------------------------
    float dbr[4] = {0.f, 0.f, 0.f, 0.f}, dgr[4] = {0.f, 0.f, 0.f, 0.f}, dqr[4] = {0.f, 0.f, 0.f, 0.f};
    floatx4 kk[KB];
    const floatx4 bev = ld_f4(reinterpret_cast<const char*>(beta_s + 16 * wave + 4 * g));
#pragma unroll
    for (int ct = 0; ct < KB; ++ct) {
        kk[ct] = kacc(OFF_K, ct);
        const floatx4 qq = kacc(OFF_Q, ct);
        dKr[ct] = dKr[ct] + bev * E2[ct];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            dbr[e] += E2[ct][e] * kk[ct][e];
            dqr[e] += dQ[ct][e] * qq[e];
            dgr[e] += (dKr[ct][e] - dKw[ct][e]) * kk[ct][e];
        }
    }
    floatx4 c5, cq;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const int i = 16 * wave + 4 * g + e;
        float db = dbr[e], dgv = dgr[e], dqv = dqr[e];
#pragma unroll
        for (int off = 1; off < 16; off <<= 1) {
            db += __shfl_xor(db, off, kWave); dgv += __shfl_xor(dgv, off, kWave); dqv += __shfl_xor(dqv, off, kWave);
        }
        db += yx_s[i];
        if (r == 0) { dbeta_s[i] = db; dg_s[i] = rowmask[e] * (dgv + dqv); }
        cq[e] = -dqv * rq_s[i] * rq_s[i];
        c5[e] = (a.opts & kOptGdnBeta) ? 0.f : -2.f * beta_s[i] * db * invden_s[i];   // beta = eta does not depend on k
    }
    __syncthreads();                                 // every wave is done with A o dP and D': they become staging tiles

    // ---- dq, dk: 4x4 transposition inside each quad of lanes, staged rows, 16-byte stores ----------------
    {
        char* sq = lds + OFF_E1;
        char* sk = lds + OFF_DP;
        const bool q_lo = (r & 3) < 2;
        const uint32_t psel = (r & 1) ? 0x03020706u : 0x05040100u;
        auto stage_quad = [&](u32x2 ob, char* dst) { *reinterpret_cast<u32x2*>(dst) = quad_transpose4x4(ob, q_lo, psel); };
        // after the transposition lane (r, g) holds token row 16 wave + 4 g + r % 4, features 32 kp + 8 (r / 4) + 4 b .. + 3
        const int orow = (16 * wave + 4 * g + (r & 3)) * ORQ + 16 * (r >> 2);
#pragma unroll
        for (int ct = 0; ct < KB; ++ct) {
            const int fo = orow + 64 * (ct >> 1) + 8 * (ct & 1);
            if (norm_q) dQ[ct] = dQ[ct] + cq * kacc(OFF_Q, ct);
            stage_quad(to_quad(dQ[ct]), sq + fo);
            stage_quad(to_quad(dKr[ct] + dKw[ct] + c5 * kk[ct]), sk + fo);
        }
        __syncthreads();
        char* qo = reinterpret_cast<char*>(a.dq) + (size_t)tok0 * kq_row + (size_t)h * DK * 2;
        char* ko = reinterpret_cast<char*>(a.dk) + (size_t)tok0 * kq_row + (size_t)h * DK * 2;
#pragma unroll
        for (int it = 0; it < 64 * PPR / 256; ++it) {
            const int i = tid + 256 * it, row = i / PPR, pc = i % PPR;
            if (row < clen) {
                __builtin_nontemporal_store(ld16(sq + row * ORQ + pc * 16), reinterpret_cast<u32x4*>(qo + (size_t)row * kq_row + pc * 16));
                __builtin_nontemporal_store(ld16(sk + row * ORQ + pc * 16), reinterpret_cast<u32x4*>(ko + (size_t)row * kq_row + pc * 16));
            }
        }
    }
    if (wave == 0) {
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

hipError_t launch_bwd_assemble_bf16(const BwdArgs<bf16_t>& a, int dk, long n_chunks, hipStream_t st)
{
    if (n_chunks == 0) return hipSuccess;
    const dim3 grid((unsigned)(n_chunks * a.H)), block(256);
    if (dk == 64) hipLaunchKernelGGL((bwd_assemble_bf16_kernel<64>), grid, block, 0, st, a);
    else          hipLaunchKernelGGL((bwd_assemble_bf16_kernel<128>), grid, block, 0, st, a);
    return hipGetLastError();
}

template <int DK, bool REV>
static hipError_t launch_sweep_dk(const BwdArgs<bf16_t>& a, int waves, hipStream_t st)
{
    const int n_chains = (a.n_seq > 0 ? a.n_seq : (a.seg_G > 0 ? a.N * a.seg_G : a.N)) * a.H;
    if (n_chains == 0) return hipSuccess;
    const dim3 grid((unsigned)(((n_chains + 7) / 8) * 8 * (a.dv_dim / (16 * waves))));
    if (waves == 1) hipLaunchKernelGGL((bwd_sweep_bf16_kernel<DK, 1, REV>), grid, dim3(192), 0, st, a);
    else            hipLaunchKernelGGL((bwd_sweep_bf16_kernel<DK, 2, REV>), grid, dim3(256), 0, st, a);
    return hipGetLastError();
}

hipError_t launch_bwd_states_bf16(const BwdArgs<bf16_t>& a, int dk, int waves, hipStream_t st)
{
    if (waves != 1 && waves != 2) return hipErrorInvalidValue;
    return dk == 64 ? launch_sweep_dk<64, false>(a, waves, st) : launch_sweep_dk<128, false>(a, waves, st);
}
hipError_t launch_bwd_scan_bf16(const BwdArgs<bf16_t>& a, int dk, int waves, hipStream_t st)
{
    if (waves != 1 && waves != 2) return hipErrorInvalidValue;
    return dk == 64 ? launch_sweep_dk<64, true>(a, waves, st) : launch_sweep_dk<128, true>(a, waves, st);
}

}  // namespace kla
