// bf16 inter-chunk stage: the recurrence of eqs. (6)-(8) per chunk, with the fp32 state of 16 columns
// per wave held in MFMA accumulators for the whole sequence (see kla_chunk_scan.hip for the algebra),
// built around the latency of the serial chunk loop on gfx950:
//
//   * Operands go global memory -> LDS directly (global_load_lds_dwordx4: lane l's 16 bytes land at
//     LDS base + 16 l, the global address is free per lane), two chunks ahead into a three-stage LDS
//     ring, so no registers and no LDS store instructions are spent on staging and a chunk's operands
//     have two chunk times to arrive.  One barrier per chunk.
//   * The copies are issued by one extra wave of the workgroup that does nothing else.  The vector
//     memory counter retires in order, so in a wave that also stores outputs every copy would queue
//     behind the (slow) acknowledgement of the stores before it; the copy wave has no stores, and
//     the compute waves never wait for memory at all.
//   * K, Q and the V slice sit in LDS as plain token-major rows; the 16-byte columns of K and Q are
//     XOR-swizzled by the row (applied on the global side of the copy) so that both kinds of read
//     below are spread over the banks.
//   * A operands whose contraction runs along a row (K S, Q S) are single 128-bit LDS reads of 8
//     consecutive features.  To make that match the accumulator-as-B-operand trick of kla_mma.hpp,
//     the state tiles carry a permuted feature index: element e of lane (r, g) of state tile
//     kt = 2*kp + b is feature 32*kp + 8*g + 4*b + e.
//   * A operands whose contraction runs down a column (K^T for the state update, and the V tile
//     that initialises an accumulator) are read with the transposing LDS load
//     (ds_read_b64_tr_b16): in each group of 16 lanes, lane j supplies the address of 4 consecutive
//     elements, lanes 4a..4a+3 together forming row a of a 4x16 block, and lane i receives column
//     i of that block.  No transposed copy of K exists anywhere.
//   * Every per-lane LDS offset is computed once before the loop; inside it an access is
//     stage base + lane offset + immediate.
//   * A short last chunk is handled without zero filling: rows beyond it re-read the last valid row;
//     their T' rows and columns are zero (beta = 0 there), so they contribute nothing to U, to the
//     state or to any stored output.
#include "kla_bf16_ops.hpp"
#include "kla_common.hpp"
#include "kla_kernels.hpp"
#include "kla_mma.hpp"

namespace kla {

namespace {

template <int DK, int NW, bool DG = false>
struct Cfg {
    static constexpr int NTH = 64 * NW;                  // compute threads (the workgroup has one more wave)
    static constexpr int KB = DK / 16, KP = DK / 32;
    static constexpr int SLW = 16 * NW;                  // state columns per workgroup
    static constexpr int RB = DK * 2;                    // bytes per K/Q row
    static constexpr int PPR = DK / 8;                   // 16-byte pieces per K/Q row
    static constexpr int RPB = 1024 / RB;                // K/Q rows per 1 KiB copy block
    static constexpr int NKB = 64 / RPB;                 // copy blocks of a K (or Q) tile
    static constexpr int VRW = SLW * 2;                  // bytes per V slice row (unpadded: filled by the copy engine)
    static constexpr int VPP = VRW / 16;                 // pieces per V row
    static constexpr int RPV = 64 / VPP;                 // V rows per copy block
    static constexpr int NVB = 64 / RPV;                 // copy blocks of the V slice (= 2 NW)
    static constexpr int TPB = kTriPairs * 64 * 16;      // bytes of one T' or P area; [T' | P] is one 12 KiB record
    static constexpr int NTB = 2 * TPB / 1024;           // = 12
    // DG (diagonal gating): a third [64 x d_k] tile, the K operand of the state update, and gamma_C per channel
    static constexpr int OFF_Q = 64 * RB, OFF_K2 = 2 * 64 * RB, OFF_T = (DG ? 3 : 2) * 64 * RB, OFF_P = OFF_T + TPB,
                         OFF_V = OFF_T + 2 * TPB, OFF_EG = OFF_V + 64 * VRW, OFF_ED = OFF_EG + 256, OFF_EQ = OFF_ED + 256,
                         OFF_GC = OFF_EQ + 256, STAGE = OFF_GC + (DG ? 512 : 0);
    // row stride of the output staging tile: 24 (NW <= 2) or 40 (NW = 4) dwords, so that the 8-dword spans which
    // one wave writes into 8 consecutive rows fall into disjoint banks
    static constexpr int ORB = NW <= 2 ? 96 : 160;
    static constexpr int OSB = 64 * ORB;
    static constexpr int NST = (3 * STAGE + 2 * OSB <= 160 * 1024) ? 3 : 2;   // LDS ring depth
    static constexpr int LDS = NST * STAGE + 2 * OSB;
    static constexpr int NDMA = (DG ? 3 : 2) * NKB + NTB + NVB + 1 + (DG ? 1 : 0);   // copy instructions per chunk (+1: decay factors)
    static_assert(LDS <= 160 * 1024 && (NST != 3 || NDMA < 64), "LDS budget of a gfx950 CU; 6-bit vmcnt (counted waits only with three stages)");
};

}  // namespace

// NQ: normalised read-out (Sec. 3.3): the output rows are scaled by 1/||q_i||, which stage 1 folded into P and
// into the third vector of the record, gamma_i/||q_i||, read here in place of gamma_i for the Q S term.
// DG: diagonal gating (App. B): a.k = K o Gamma and a.q = Q o Gamma feed K S and Q S, a.kt_src = K o (gamma_C/Gamma)
// the state update, the records carry unit decay vectors and the state rows decay by a.gc_vec (see intra_diag_kernel).
template <int DK, int NW, bool NQ, bool DG = false>
__global__ __launch_bounds__(64 * NW + 64) void scan_bf16_kernel(ScanArgs<bf16_t> a)
{
    typedef Cfg<DK, NW, DG> C;
    constexpr int NTH = C::NTH, KB = C::KB, KP = C::KP, SLW = C::SLW, RB = C::RB, PPR = C::PPR, RPB = C::RPB,
                  VRW = C::VRW, VPP = C::VPP, RPV = C::RPV, ORB = C::ORB, NST = C::NST;

    __shared__ __attribute__((aligned(1024))) char lds[C::LDS];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int r = lane & 15, g = lane >> 4;

    // ---- workgroup -> (sequence, head, column slice); slices of one head share an XCD (ids congruent mod 8)
    const int nsl = a.dv / SLW;
    const int n_states = a.n_seq > 0 ? a.n_seq : (a.seg_G > 0 ? a.N * a.seg_G : a.N);
    const int n_chains = n_states * a.H;
    const int xcd = blockIdx.x & 7, pidx = blockIdx.x >> 3;
    const int chain = (pidx / nsl) * 8 + xcd, slice = pidx % nsl;
    if (chain >= n_chains) return;
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
    const int nch = (len + 63) / 64;
    const int col = slice * SLW + 16 * wave + r;

    // state tile kt = 2*kp + b, element e  <->  feature 32*kp + 8*g + 4*b + e, column `col`
    floatx4 S[KB];
#pragma unroll
    for (int kt = 0; kt < KB; ++kt)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int f = 32 * (kt >> 1) + 8 * g + 4 * (kt & 1) + e;
            S[kt][e] = (a.h0 && wave < NW) ? a.h0[((size_t)chain * DK + f) * a.dv + col] : 0.f;   // not the copy wave
        }

    const size_t kq_row = (size_t)a.H * DK * 2, v_row = (size_t)a.H * a.dv * 2;     // bytes between tokens
    const char* kbase = reinterpret_cast<const char*>(a.k) + (size_t)t0 * kq_row + (size_t)h * DK * 2;
    const char* qbase = reinterpret_cast<const char*>(a.q) + (size_t)t0 * kq_row + (size_t)h * DK * 2;
    const char* vbase = reinterpret_cast<const char*>(a.v) + (size_t)t0 * v_row + ((size_t)h * a.dv + slice * SLW) * 2;
    const char* k2base = DG ? reinterpret_cast<const char*>(a.kt_src) + (size_t)t0 * kq_row + (size_t)h * DK * 2 : nullptr;
    const char* gcbase = DG ? reinterpret_cast<const char*>(a.gc_vec) + ((size_t)ch0 * a.H + h) * DK * 4 : nullptr;
    constexpr int REC = ws_record_bytes<bf16_t>();
    const char* tpbase = reinterpret_cast<const char*>(a.wsT) + ((size_t)ch0 * a.H + h) * REC;

    // ---- loop-invariant per-lane offsets ------------------------------------------------------------
    // copy engine, global side: lane l of copy block b fills LDS bytes [1024 b + 16 l, +16) of a tile, i.e.
    // row 1024 b / RB + l / PPR, physical column l % PPR, which holds logical column (l % PPR) ^ swz(row).
    // (row & 7) depends on the block only through its parity (RPB = 4) or not at all (RPB = 8).
    const int lrow = lane / PPR, pcol = lane % PPR;
    int gk[2];
#pragma unroll
    for (int par = 0; par < 2; ++par)
        gk[par] = lrow * (int)kq_row + ((pcol ^ swz_bits(RPB * par + lrow)) * 16);
    const int gv = (lane / VPP) * (int)v_row + (lane % VPP) * 16;
    // LDS reads.  K/Q row slots: token row 16 it + r, logical column 4 kp + g = 8 m + 4 par + g:
    int oK[2];
#pragma unroll
    for (int par = 0; par < 2; ++par) oK[par] = r * RB + (((4 * par + g) ^ swz_bits(r)) * 16);
    // K^T slots through the transposing read: source lane (a4, c4) points at token 4 g + a4 (+ 16 beta + 32 jp),
    // logical column 8 m + 4 par + c4, half b.
    const int a4 = r >> 2, c4 = r & 3;
    int oKT[2];
#pragma unroll
    for (int par = 0; par < 2; ++par) oKT[par] = (4 * g + a4) * RB + (((4 * par + c4) ^ swz_bits(4 * g + a4)) * 16);
    const int oV = (4 * g + a4) * VRW + (16 * wave + 4 * c4) * 2;      // V tile rows 4 g + a4 (+ 16 it)
    // staging tile: after the 4x4 transposition below lane (r, g) holds row 4 g + (r & 3) (+ 16 it), columns
    // 4 (r >> 2) .. + 3 of this wave's 16
    const int oO = (4 * g + (r & 3)) * ORB + (16 * wave + 4 * (r >> 2)) * 2;
    const bool q_lo = (r & 3) < 2;                       // lane sits in the upper half of its quad's 4x4 block
    const uint32_t psel = (r & 1) ? 0x03020706u : 0x05040100u;   // byte selectors of the 2x2 step (see below)

    // ---- global -> LDS copy of everything chunk c needs except the decay factors ---------------------
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
                const int lo = (RPB == 4 && (b & 1)) ? gk[1] : gk[0];
                dma16(kc + o, lo, st + b * 1024);
                dma16(qc + o, lo, st + C::OFF_Q + b * 1024);
                if constexpr (DG) dma16(k2base + (size_t)(64 * c) * kq_row + o, lo, st + C::OFF_K2 + b * 1024);
            });
            static_for<C::NVB>([&](auto i) {
                const int b = i;
                dma16(vc + (size_t)(b * RPV) * v_row, gv, st + C::OFF_V + b * 1024);
            });
        } else {                                         // ragged last chunk: clamp the row
            static_for<C::NKB>([&](auto i) {
                const int b = i;
                const int row = b * RPB + lrow;
                const int lo = min(row, clen - 1) * (int)kq_row + ((pcol ^ swz_bits(row)) * 16);
                dma16(kc, lo, st + b * 1024);
                dma16(qc, lo, st + C::OFF_Q + b * 1024);
                if constexpr (DG) dma16(k2base + (size_t)(64 * c) * kq_row, lo, st + C::OFF_K2 + b * 1024);
            });
            static_for<C::NVB>([&](auto i) {
                const int b = i;
                const int row = b * RPV + lane / VPP;
                dma16(vc, min(row, clen - 1) * (int)v_row + (lane % VPP) * 16, st + C::OFF_V + b * 1024);
            });
        }
        static_for<C::NTB>([&](auto i) {
            const int b = i;
            dma16(tc + b * 1024, lane * 16, st + C::OFF_T + b * 1024);
        });
        if (lane < 48) dma16(tc + 2 * C::TPB, lane * 16, st + C::OFF_EG);   // gamma_i | gamma_C/gamma_i | gamma_i/||q_i||: 768 bytes
        if constexpr (DG) {
            if (lane < DK / 4) dma16(gcbase + (size_t)c * a.H * DK * 4, lane * 16, st + C::OFF_GC);   // gamma_C per channel
        }
    };

    // ---- one chunk of the recurrence for this wave's 16 columns ------------------------------------
    auto compute = [&](const char* st, char* ost) {
        const char* pK0 = st + oK[0];
        const char* pK1 = st + oK[1];
        const char* pT0 = st + oKT[0];
        const char* pT1 = st + oKT[1];
        const char* pS = st + lane * 16;                 // T' / P slots
        const char* pV = st + C::OFF_V + oV;
        const char* pG = st + C::OFF_EG + 16 * g;        // 4 consecutive floats: rows 4 g .. 4 g + 3
        auto kslot = [&](int it, int kp, int base) {     // base 0: K, OFF_Q: Q
            return ld16(((kp & 1) ? pK1 : pK0) + base + 16 * it * RB + 128 * (kp >> 1));
        };
        auto ktslot = [&](int kt, int jp, u32x2& q0, u32x2& q1) {
            const int kp = kt >> 1, b = kt & 1;
            const char* p = ((kp & 1) ? pT1 : pT0) + (DG ? C::OFF_K2 : 0) + 32 * jp * RB + 128 * (kp >> 1) + 8 * b;
            q0 = lds_read_tr(p);
            q1 = lds_read_tr(p + 16 * RB);
        };

        // bf16 copy of the incoming state (B operand of K S and Q S); the fp32 state is decayed right away
        const float gC = *reinterpret_cast<const float*>(st + C::OFF_EG + 63 * 4);
        u32x2 Sq[KB];
#pragma unroll
        for (int kt = 0; kt < KB; ++kt) {
            Sq[kt] = to_quad(S[kt]);
            // diagonal gating: row (feature) f of the state decays by gamma_C[f]; tile kt, element e is feature
            // 32 (kt / 2) + 8 g + 4 (kt % 2) + e
            if constexpr (DG) S[kt] = S[kt] * ld_f4(st + C::OFF_GC + (32 * (kt >> 1) + 8 * g + 4 * (kt & 1)) * 4);
            else              S[kt] = S[kt] * gC;
        }

        // Products are issued "independent first": consecutive MFMAs write different accumulators, so that a
        // dependent one (same accumulator) follows only several instructions later.
        // ---- K S (on the serial chain): A slots are 8 consecutive features of a token row
        floatx4 ks[4], qs[4];
#pragma unroll
        for (int it = 0; it < 4; ++it) { ks[it] = floatx4{0.f, 0.f, 0.f, 0.f}; qs[it] = floatx4{0.f, 0.f, 0.f, 0.f}; }
        u32x4 ka[2][4];
#pragma unroll
        for (int it = 0; it < 4; ++it) ka[0][it] = kslot(it, 0, 0);
#pragma unroll
        for (int kp = 0; kp < KP; ++kp) {
            if (kp + 1 < KP) {
#pragma unroll
                for (int it = 0; it < 4; ++it) ka[(kp + 1) & 1][it] = kslot(it, kp + 1, 0);
            }
#pragma unroll
            for (int it = 0; it < 4; ++it) mma_bf16(ks[it], ka[kp & 1][it], Sq[2 * kp], Sq[2 * kp + 1]);
        }
        // operands of the solve and of Q S, in flight while K S drains
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
        u32x4 qa[2][4];
#pragma unroll
        for (int it = 0; it < 4; ++it) qa[0][it] = kslot(it, 0, C::OFF_Q);

        // ---- Q S (off the chain) fills the matrix pipe while X = V - D_gamma K S is formed on the VALU
#pragma unroll
        for (int kp = 0; kp < KP; ++kp) {
            if (kp + 1 < KP) {
#pragma unroll
                for (int it = 0; it < 4; ++it) qa[(kp + 1) & 1][it] = kslot(it, kp + 1, C::OFF_Q);
            }
#pragma unroll
            for (int it = 0; it < 4; ++it) mma_bf16(qs[it], qa[kp & 1][it], Sq[2 * kp], Sq[2 * kp + 1]);
        }
        u32x2 Xq[4];
#pragma unroll
        for (int it = 0; it < 4; ++it) Xq[it] = to_quad(quad_to_f(vq[it]) - egv[it] * ks[it]);

        // K^T slots of the first state tiles and the P slots: on their way during the solve
        u32x2 kt[2][KB][2];                              // [token pair jp][state tile][token block]
#pragma unroll
        for (int t = 0; t < KB; ++t) ktslot(t, 0, kt[0][t][0], kt[0][t][1]);

        // ---- U = T' X (T' lower triangular)
        floatx4 U[4];
#pragma unroll
        for (int it = 0; it < 4; ++it) {
            U[it] = floatx4{0.f, 0.f, 0.f, 0.f};
            mma_bf16(U[it], tsl[tri_pair(it, 0)], Xq[0], Xq[1]);
        }
        mma_bf16(U[2], tsl[tri_pair(2, 1)], Xq[2], Xq[3]);
        mma_bf16(U[3], tsl[tri_pair(3, 1)], Xq[2], Xq[3]);
#pragma unroll
        for (int t = 0; t < KB; ++t) ktslot(t, 1, kt[1][t][0], kt[1][t][1]);
        u32x4 psl[kTriPairs];
#pragma unroll
        for (int i = 0; i < kTriPairs; ++i) psl[i] = ld16(pS + C::OFF_P + i * 1024);

        u32x2 Uq[4], Udq[4];
#pragma unroll
        for (int it = 0; it < 4; ++it) {
            Udq[it] = to_quad(U[it] * edv[it]);
            Uq[it] = to_quad(U[it]);
        }

        // ---- S = gamma_C S + K^T (diag(gamma_C/gamma_i) U): the only thing the next chunk waits for
#pragma unroll
        for (int t = 0; t < KB; ++t) mma_bf16(S[t], kt[0][t][0], kt[0][t][1], Udq[0], Udq[1]);
#pragma unroll
        for (int t = 0; t < KB; ++t) mma_bf16(S[t], kt[1][t][0], kt[1][t][1], Udq[2], Udq[3]);

        // ---- O = D_gamma Q S + P U (P lower triangular), staged token-major for 16-byte global stores
        floatx4 o[4];
#pragma unroll
        for (int it = 0; it < 4; ++it) {
            if constexpr (NQ) o[it] = ld_f4(pG + 512 + 64 * it) * qs[it]; else o[it] = egv[it] * qs[it];
            mma_bf16(o[it], psl[tri_pair(it, 0)], Uq[0], Uq[1]);
        }
        mma_bf16(o[2], psl[tri_pair(2, 1)], Uq[2], Uq[3]);
        mma_bf16(o[3], psl[tri_pair(3, 1)], Uq[2], Uq[3]);
        // transposed 4x4 inside each quad of lanes (see quad_transpose4x4): one 64-bit LDS write per tile (a compute
        // wave is bound by its instruction count)
#pragma unroll
        for (int it = 0; it < 4; ++it)
            *reinterpret_cast<u32x2*>(ost + oO + 16 * it * ORB) = quad_transpose4x4(to_quad(o[it]), q_lo, psel);
    };

    auto write_out = [&](int c, const char* ost) {
        const int clen = min(64, len - 64 * c);
        char* ob = reinterpret_cast<char*>(a.o) + (size_t)(t0 + 64L * c) * v_row + ((size_t)h * a.dv + slice * SLW) * 2;
#pragma unroll
        for (int it = 0; it < 64 * VPP / NTH; ++it) {
            const int i = tid + NTH * it;
            const int row = i / VPP, pv = i % VPP;
            // outputs are written once and not read again by this kernel: streamed past the caches
            if (row < clen) __builtin_nontemporal_store(ld16(ost + row * ORB + pv * 16), reinterpret_cast<u32x4*>(ob + (size_t)row * v_row + pv * 16));
        }
    };

    char* ost0 = lds + NST * C::STAGE;
    char* ost1 = ost0 + C::OSB;

    if (wave == NW) {
        // ---- the copy wave: keeps chunks c+1 .. c+NST-1 on their way while chunk c is computed ---------
#pragma unroll
        for (int p = 0; p < NST - 1; ++p)
            if (p < nch) issue(p, lds + p * C::STAGE);
        if (NST == 3 && nch > 1) wait_vmcnt<(NST == 3 ? C::NDMA : 0)>(); else wait_vmcnt<0>();      // chunk 0 has landed
        __syncthreads();
        int spre = NST - 1;                              // ring position of chunk c + NST - 1
        for (int c = 0; c < nch; ++c) {
            const bool ahead = c + NST - 1 < nch;
            // the stage being refilled was read by chunk c-1, which every wave finished before the last barrier
            if (ahead) issue(c + NST - 1, lds + spre * C::STAGE);
            // Copies retire in order and this wave issues nothing else: all but the NDMA just issued (when
            // NST = 3) have landed once the counter is down to NDMA, i.e. chunk c+1 is complete.
            if (NST == 3 && ahead) wait_vmcnt<(NST == 3 ? C::NDMA : 0)>(); else wait_vmcnt<0>();
            __syncthreads();
            spre = (spre + 1 == NST) ? 0 : spre + 1;
        }
        return;
    }

    // ---- compute waves ---------------------------------------------------------------------------------
    __syncthreads();                                     // chunk 0 is in stage 0
    int scur = 0;                                        // ring position of chunk c
    for (int c = 0; c < nch; ++c) {
        char* ost = (c & 1) ? ost1 : ost0;
        compute(lds + scur * C::STAGE, ost);
        // One barrier per chunk: staged outputs before their write-out; chunk c+1's operands before their
        // use; all reads of this stage before it is refilled next iteration; and the write-out of chunk
        // c-1 (finished by every compute wave before it arrives here) before the staging tile of that
        // parity is written again in chunk c+1.
        __syncthreads();
        write_out(c, ost);
        scur = (scur + 1 == NST) ? 0 : scur + 1;
    }

    if (a.hT) {
#pragma unroll
        for (int kt = 0; kt < KB; ++kt)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int f = 32 * (kt >> 1) + 8 * g + 4 * (kt & 1) + e;
                a.hT[((size_t)chain * DK + f) * a.dv + col] = S[kt][e];
            }
    }
}

template <int DK>
static hipError_t launch_dk(const ScanArgs<bf16_t>& a, int waves, hipStream_t st)
{
    const int n_states = a.n_seq > 0 ? a.n_seq : (a.seg_G > 0 ? a.N * a.seg_G : a.N);
    const int n_chains = n_states * a.H;
    if (n_chains == 0) return hipSuccess;
    const int nsl = a.dv / (16 * waves);
    const dim3 grid((unsigned)(((n_chains + 7) / 8) * 8 * nsl));
    const bool nq = (a.opts & kOptNormalizeQ) != 0;
    switch (waves) {
        case 1:
            if (nq) hipLaunchKernelGGL((scan_bf16_kernel<DK, 1, true>), grid, dim3(128), 0, st, a);
            else    hipLaunchKernelGGL((scan_bf16_kernel<DK, 1, false>), grid, dim3(128), 0, st, a);
            break;
        case 2:
            if (nq) hipLaunchKernelGGL((scan_bf16_kernel<DK, 2, true>), grid, dim3(192), 0, st, a);
            else    hipLaunchKernelGGL((scan_bf16_kernel<DK, 2, false>), grid, dim3(192), 0, st, a);
            break;
        default:
            if (nq) hipLaunchKernelGGL((scan_bf16_kernel<DK, 4, true>), grid, dim3(320), 0, st, a);
            else    hipLaunchKernelGGL((scan_bf16_kernel<DK, 4, false>), grid, dim3(320), 0, st, a);
            break;
    }
    return hipGetLastError();
}

hipError_t launch_scan_bf16(const ScanArgs<bf16_t>& a, int dk, int waves, hipStream_t st)
{
    if (dk == 64) return launch_dk<64>(a, waves, st);
    return launch_dk<128>(a, waves, st);
}

// diagonal gating: waves = 1 or 2, fixed-length or packed batches, no options, no segments
template <int DK>
static hipError_t launch_diag_dk(const ScanArgs<bf16_t>& a, int waves, hipStream_t st)
{
    const int n_chains = (a.n_seq > 0 ? a.n_seq : a.N) * a.H;
    if (n_chains == 0) return hipSuccess;
    const dim3 grid((unsigned)(((n_chains + 7) / 8) * 8 * (a.dv / (16 * waves))));
    if (waves == 1) hipLaunchKernelGGL((scan_bf16_kernel<DK, 1, false, true>), grid, dim3(128), 0, st, a);
    else            hipLaunchKernelGGL((scan_bf16_kernel<DK, 2, false, true>), grid, dim3(192), 0, st, a);
    return hipGetLastError();
}
hipError_t launch_scan_bf16_diag(const ScanArgs<bf16_t>& a, int dk, int waves, hipStream_t st)
{
    if ((waves != 1 && waves != 2) || a.seg_G > 0 || !a.kt_src || !a.gc_vec) return hipErrorInvalidValue;
    return dk == 64 ? launch_diag_dk<64>(a, waves, st) : launch_diag_dk<128>(a, waves, st);
}

}  // namespace kla
