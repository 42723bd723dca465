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
//   * Fused mode (FU): no separate intra-chunk stage and no workspace.  Four more waves of the workgroup
//     ("helpers", on the SIMDs that have no compute wave) produce the solve operands, P and the decay vectors of
//     the chunks two and one steps ahead, straight into two LDS record buffers, so K and Q are read from memory
//     once and the per-chunk objects never leave the CU (see the helper section below).  A seventh wave, otherwise
//     idle, writes the staged outputs to memory.
//   * A short last chunk is handled without zero filling: rows beyond it re-read the last valid row;
//     their T' rows and columns are zero (beta = 0 there), so they contribute nothing to U, to the
//     state or to any stored output.
#include "kla_bf16_ops.hpp"
#include "kla_common.hpp"
#include "kla_kernels.hpp"
#include "kla_mma.hpp"

namespace kla {

namespace {

template <int DK, int NW, bool DG = false, bool FU = false>
struct Cfg {
    static_assert(!(DG && FU), "the fused mode has no diagonal-gating variant");
    static constexpr int NTH = 64 * NW;                  // compute threads (the workgroup has one or three more waves)
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
    // DG (diagonal gating): a third [64 x d_k] tile, the K operand of the state update, and gamma_C per channel.
    // FU: a ring stage holds K, Q and the V slice only; the record [T' | P | three vectors] of a chunk lives in one of
    // two record buffers behind the ring, written by a helper wave.
    static constexpr int OFF_Q = 64 * RB, OFF_K2 = 2 * 64 * RB, OFF_T = (DG ? 3 : 2) * 64 * RB, OFF_P = OFF_T + TPB,
                         OFF_V = FU ? OFF_T : OFF_T + 2 * TPB, OFF_EG = OFF_V + 64 * VRW, OFF_ED = OFF_EG + 256,
                         OFF_EQ = OFF_ED + 256, OFF_GC = OFF_EQ + 256, STAGE = FU ? OFF_EG : OFF_GC + (DG ? 512 : 0);
    // where a compute wave finds T', P and the vectors, relative to the ring stage (not fused) or the record buffer
    static constexpr int R_T = FU ? 0 : OFF_T, R_P = FU ? TPB : OFF_P, R_EG = FU ? 2 * TPB : OFF_EG;
    static constexpr int RECB = 2 * TPB + 1024;          // bytes of a record buffer: [T-area | P | four vectors of 64 fp32]
    static constexpr int HSCR_T = 4096 + 6 * 256, HSCR_P = 6 * 256;   // private LDS of a T-side / P-side helper wave
    // row stride of the output staging tile: 24 (NW <= 2) or 40 (NW = 4) dwords, so that the 8-dword spans which
    // one wave writes into 8 consecutive rows fall into disjoint banks
    static constexpr int ORB = NW <= 2 ? 96 : 160;
    static constexpr int OSB = 64 * ORB;
    static constexpr int EXTRA = FU ? 2 * RECB + 2 * HSCR_T + 2 * HSCR_P : 0;
    static constexpr int NST = (3 * STAGE + 2 * OSB + EXTRA <= 160 * 1024) ? 3 : 2;   // LDS ring depth
    static constexpr int LDS = NST * STAGE + 2 * OSB + EXTRA;
    static constexpr int OFF_REC = NST * STAGE + 2 * OSB, OFF_HST = OFF_REC + 2 * RECB, OFF_HSP = OFF_HST + 2 * HSCR_T;   // FU only
    // copy instructions per chunk (+1: decay factors)
    static constexpr int NDMA = FU ? NVB : (DG ? 3 : 2) * NKB + NTB + NVB + 1 + (DG ? 1 : 0);
    // Split schedule of a two-stage ring (diagonal gating at d_k = 128, whose stage holds three K-sized tiles): a chunk's
    // copies go out in two parts, each a full step before its first use, with a second barrier in the step between
    // them.  N_FIRST, N_REST: copy instructions of the two parts.
    static constexpr bool SPLIT = DG && NST == 2;
    static constexpr int N_FIRST = NKB + NVB + NTB / 2 + 2, N_REST = 2 * NKB + NTB / 2;
    static_assert(!SPLIT || (N_FIRST + N_REST == NDMA && N_FIRST < 64 && N_REST < 64), "parts of the split schedule; 6-bit vmcnt");
    // waves of a workgroup: compute waves, then the copy wave and the wave that writes the outputs; fused: compute
    // waves, two T-side helpers, the copy wave, the write-out wave - placed so that the two P-side helpers after it land
    // on the SIMDs of the T-side ones - and those two
    static constexpr int NWAVES = NW + (FU ? 6 : 2);
    static constexpr int W_COPY = FU ? NW + 2 : NW;
    static constexpr int W_P = NW + 4, W_IDLE = FU ? NW + 3 : NW + 1;
    static_assert(LDS <= 160 * 1024 && (NST != 3 || NDMA < 64), "LDS budget of a gfx950 CU; 6-bit vmcnt (counted waits only with three stages)");
    static_assert(!FU || NST == 3, "fused mode is laid out for the three-stage ring");
};


// ---- helper waves of the fused mode ------------------------------------------------------------------------
// Four waves, on the two SIMDs that have no compute wave, produce the record of every chunk two steps ahead of its use:
// a "T-side" and a "P-side" wave for the even chunks, another pair for the odd ones; a wave takes two chunk steps per
// record (phase A in step c - 2, phase B in step c - 1), and the two waves that share a SIMD fill each other's stalls.
//
// T-side.  The unit lower triangular system of eq. (6), (I + L) U = B X with L = B (A^- o K K^T), is handed to the
// compute waves as a block forward substitution over its four 16-row blocks,
//
//     U_0 = (D_0 B_0) X_0,     U_t = D_t (B_t X_t - sum_{j<t} L_tj U_j),     D_t = (I + L_tt)^{-1},
//
// so only the four 16x16 diagonal blocks are inverted and no product of blocks is formed: the 64x64 "T-area" of the
// record holds [D_0 B_0; L10 D_1; L20 L21 D_2; L30 L31 L32 D_3] in the tile-pair layout of T' (kla_mma.hpp), and a
// fourth vector carries beta.  The wave works on transposed tiles: the accumulator tile of (K_tj K_ti^T) - lane
// (r, g) holds rows 4g..4g+3 of column r - is exactly the A-operand quad order of tile (ti, tj) of L that the record
// stores.  Tiles live in registers; the only LDS the wave touches is its private scratch (per-token tables, the four
// diagonal blocks on their way between layouts) and, at the very end, the record buffer.
//   phase A  the K row slots (loaded from global memory during the step before) go on into the ring stage of the
//            chunk; g = prefix sum of log alpha (units of log 2), decay tables; K K^T on bf16 MFMA (the ten lower
//            tiles); beta of eq. (3) from its diagonal; decay, mask and beta applied to the diagonal tiles, which go
//            to the scratch.
//   phase B  decay and beta on the six strictly lower tiles; the four diagonal blocks inverted by forward
//            substitution, each block by one group of 16 lanes (lane = column, the rows of L read from the scratch by
//            the whole group at once); everything rounded to bf16 and written in operand order.
// P-side.  P = A o Q K^T of eq. (7) (with 1/||q_i|| on its rows for the normalised read-out), the ten lower tiles as
// (Q K^T)^T so that they too come out in A-operand order, and the three decay vectors gamma_i, gamma_C/gamma_i,
// gamma_i/||q_i||.  Phase A stores its Q row slots into the ring stage, takes the K row slots from there (the T-side wave
// of the same chunk stores them in the same step and says so through a word in LDS), forms the products and scales the
// upper rows of tiles; phase B finishes the diagonal tiles and the last row and writes the record.
//
// K and Q are therefore read from memory once per workgroup, into registers, one step before phase A uses them (a chunk
// step is shorter than a trip to memory); the ring's K and Q tiles are written from those registers, and only the V slice
// comes through the copy engine.  How the work is split between the two phases of each wave follows from per-wave
// timestamps: in every step each of the two helper SIMDs runs one phase A and one phase B, and the four phases are
// balanced to within a few percent of each other and of a compute wave's step.
//
// Decay ratios off the diagonal tiles are the product of two factors <= 1, gamma_I / gamma_ref and
// gamma_ref / gamma_J with ref the first token of I's tile (J < ref <= I there): 2^x is evaluated a few times per
// lane instead of once per element, and no factor can overflow.  On the diagonal tiles 2^(g_I - g_J) is taken
// directly (masked to J <= I before the exponential).
template <int DK>
struct HelperBase {
    static constexpr int KP = DK / 32;
    static constexpr int TPB = kTriPairs * 64 * 16;

    float la_pre;                           // log alpha of token `lane`

    __device__ __forceinline__ static void wave_lds_fence()
    {
        // One wave, and the LDS executes a wave's operations in order: all that is needed between a write by one lane
        // and a read by another is that the compiler keeps them in program order.  (A real fence would also wait for the
        // global loads in flight, which are the very thing these phases overlap with.)
        asm volatile("" ::: "memory");
    }
    // the instruction scheduler does not move anything across this point: keeps the loads where the register budget
    // of 256 per lane (two waves per SIMD) has room for them
    __device__ __forceinline__ static void pin() { __builtin_amdgcn_sched_barrier(0); }
    // Every phase starts from a lane index the compiler cannot see through: otherwise it computes the dozens of
    // lane-dependent addresses and masks of all phases once, before the chunk loop, and keeps them in registers for
    // its whole length - registers the phases themselves need.
    __device__ __forceinline__ static int opaque(int x) { asm volatile("" : "+v"(x)); return x; }

    // lane (r, g) takes, for each block of 16 rows, the eight features 32 kp + 8 g .. + 7 of row r of the block
    // (rows beyond a short chunk repeat its last row).  The byte offsets of the four rows inside a full chunk are kept
    // in registers for the whole sequence.
    int ro_full[4];
    __device__ __forceinline__ void init_rows(int lane, int kq_row)
    {
#pragma unroll
        for (int it = 0; it < 4; ++it) ro_full[it] = (16 * it + (lane & 15)) * kq_row + 16 * (lane >> 4);
    }
    // tile: chunk base of K or of Q for this head; dst: KP x 4 row slots
    __device__ __forceinline__ void load_slots(u32x4 (&dst)[KP][4], const char* tile, int lane, int clen, int kq_row) const
    {
        const int lim = (clen - 1) * kq_row + 16 * (lane >> 4);     // the offsets grow with the row: clamping them clamps the row
        static_for<4>([&](auto itc) {
            constexpr int it = itc;
            const int ro = min(ro_full[it], lim);
            static_for<KP>([&](auto kpc) {
                constexpr int kp = kpc;
                dst[kp][it] = ld16(tile + ro + 64 * kp);
            });
        });
    }
    // The helpers are also the ones that bring K and Q on chip: the row slots they loaded for their own products go
    // on into the ring stage of the chunk, in the swizzled token-major layout the compute waves read (row 16 it + r,
    // logical 16-byte column 4 kp + g).
    __device__ __forceinline__ static void store_slots(const u32x4 (&src)[KP][4], char* tile, int lane)
    {
        const int r = lane & 15, g = lane >> 4;
        static_for<4>([&](auto itc) {
            constexpr int it = itc;
            char* row = tile + (16 * it + r) * (DK * 2);
            static_for<KP>([&](auto kpc) {
                constexpr int kp = kpc;
                st16(row + (((4 * kp + g) ^ swz_piece<DK>(r)) * 16), src[kp][it]);     // the swizzle has period 8 rows
            });
        });
    }
    __device__ __forceinline__ static u32x4 ring_slot(const char* tile, int it, int kp, int lane)
    {
        const int r = lane & 15, g = lane >> 4;
        return ld16(tile + (16 * it + r) * (DK * 2) + (((4 * kp + g) ^ swz_piece<DK>(r)) * 16));
    }

    // Inclusive prefix sum of log alpha over the 64 lanes, in units of log 2 (every decay factor is then one
    // v_exp_f32): inside each row of 16 lanes by DPP shifts, the rows joined through the scalar unit.  Writes the
    // tables every consumer needs - g, and gamma_ref(ti) / gamma_J for ti = 1..3 - and returns g of this lane;
    // av = gamma_I / gamma_ref(I), gl2 = g of the last token.
    __device__ __forceinline__ float scan_gates(float* tab_g2, float* tab_b, int lane, float& av, float& gl2) const
    {
        const int g = lane >> 4;
        float x = la_pre;
        x += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0x111, 0xf, 0xf, true));   // row_shr:1
        x += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0x112, 0xf, 0xf, true));   // row_shr:2
        x += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0x114, 0xf, 0xf, true));   // row_shr:4
        x += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0x118, 0xf, 0xf, true));   // row_shr:8
        {
            const float r0 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(x), 15));
            const float r1 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(x), 31));
            const float r2 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(x), 47));
            x += g == 0 ? 0.f : (g == 1 ? r0 : (g == 2 ? r0 + r1 : (r0 + r1) + r2));
        }
        const float x2 = x * 1.44269504088896341f;
        gl2 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(x2), 63));
        // ref = first lane of I's row (DPP row_newbcast:0)
        av = __builtin_amdgcn_exp2f(x2 - __int_as_float(__builtin_amdgcn_mov_dpp(__float_as_int(x2), 0x150, 0xf, 0xf, true)));
        tab_g2[lane] = x2;
#pragma unroll
        for (int ti = 1; ti < 4; ++ti) {                 // unused for J >= 16 ti
            const float gref = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(x2), 16 * ti));
            tab_b[64 * (ti - 1) + lane] = __builtin_amdgcn_exp2f(fminf(gref - x2, 0.f));
        }
        return x2;
    }
    // The results of phase A are wanted in registers when the phase ends: without this the compiler moves the arithmetic
    // that produces them behind the barrier, next to their use in phase B, where the prefetched operands need the room.
    __device__ __forceinline__ static void keep(u32x2& q) { asm volatile("" : "+v"(q.x), "+v"(q.y)); }
    __device__ __forceinline__ static void keep(floatx4& x) { asm volatile("" : "+v"(x[0]), "+v"(x[1]), "+v"(x[2]), "+v"(x[3])); }
    __device__ __forceinline__ static void slot(char* rec, int base, int ctp, int lane, u32x2 q0, u32x2 q1)
    {
        const u32x4 v = {q0.x, q0.y, q1.x, q1.y};
        st16(rec + base + (ctp * 64 + lane) * 16, v);
    }
};

template <int DK>
struct THelper : HelperBase<DK> {
    typedef HelperBase<DK> B;
    using B::KP; using B::wave_lds_fence; using B::pin; using B::opaque;
    static constexpr int SCR = 4096 + 6 * 256;           // private scratch: four 16x16 fp32 blocks, six tables of 64
    // tables (floats): g, ||k||^2 then beta gamma_I/gamma_ref (same lane reads the one and writes the other), beta, b x 3
    static constexpr int T_G2 = 1024, T_BA = 1088, T_BETA = 1152, T_B = 1216;

    u32x4 ka[KP][4];                        // K row slots of the wave's next record
    float eta_pre;
    // The four 16x16 fp32 blocks in the scratch are row-major with the 16-byte pieces of a row permuted: piece c of row
    // `row` of block t sits at position c ^ (row / 2 % 4) ^ t.  With that, the stores of a tile (8 consecutive rows at one
    // piece per cycle), the broadcast row reads of the substitution (the four lane groups read the same row of four
    // different blocks) and the column reads that follow all spread over the LDS banks.
    __device__ __forceinline__ static int blk_piece(int t, int row, int c) { return (c ^ (row >> 1) ^ t) & 3; }
    // carried from phase A to phase B: the six strictly lower tiles of K K^T, transposed (tile (ti, tj) at index
    // ti (ti - 1) / 2 + tj, lane (r, g) holds k_I . k_J for I = 16 ti + r, J = 16 tj + 4 g + e); phase B scales them into
    // the tiles of L in A-operand order, in the shadow of its substitution chain
    floatx4 Gt[6];

    __device__ __forceinline__ void prefetch(const ScanArgs<bf16_t>& a, long tok0, int clen, int h, int lane_, const char* kc,
                                             int kq_row)
    {
        const int lane = opaque(lane_);
        eta_pre = lane < clen ? a.eta[(size_t)(tok0 + lane) * a.H + h] : 0.f;
        this->la_pre = lane < clen ? a.log_alpha[(size_t)(tok0 + lane) * a.H + h] : 0.f;
        this->load_slots(ka, kc, lane, clen, kq_row);
    }

    // ktile: the K tile of this chunk's ring stage
    __device__ __forceinline__ void phase_a(const ScanArgs<bf16_t>& a, float* hs, char* ktile, int* kflag, int c, int lane_)
    {
        const int lane = opaque(lane_);
        const int r = lane & 15, g = lane >> 4;
        const bool gdn = (a.opts & kOptGdnBeta) != 0;
        B::store_slots(ka, ktile, lane);
        wave_lds_fence();
        // a wave's LDS instructions are carried out in order: whoever sees the word sees the tile
        if (lane == 0) *reinterpret_cast<volatile int*>(kflag) = c;
        float av, gl2;
        this->scan_gates(hs + T_G2, hs + T_B, lane, av, gl2);

        // ---- K K^T: the diagonal tiles and the six strictly lower ones, all transposed (rows <- block tj, column <-
        //      block ti): scaled, they are handed on as they are, in A-operand order
        const floatx4 z4 = {0.f, 0.f, 0.f, 0.f};
        floatx4 Gd[4] = {z4, z4, z4, z4};
#pragma unroll
        for (int i = 0; i < 6; ++i) Gt[i] = z4;
        static_for<KP>([&](auto kc_) {
            constexpr int kp = kc_;
            const u32x4* kk = ka[kp];
            static_for<4>([&](auto tic) {
                constexpr int ti = tic;
                const u32x2 kb0 = {kk[ti][0], kk[ti][1]}, kb1 = {kk[ti][2], kk[ti][3]};
                mma_bf16(Gd[ti], kk[ti], kb0, kb1);
                static_for<ti>([&](auto tjc) {
                    constexpr int tj = tjc;
                    mma_bf16(Gt[ti * (ti - 1) / 2 + tj], kk[tj], kb0, kb1);
                });
            });
        });
        wave_lds_fence();
        // ---- beta of eq. (3): ||k_i||^2 is the diagonal of K K^T (exact bf16 products, fp32 sums); the lane holding
        //      (i, i) hands it to lane i, which has eta_i and gamma_i / gamma_ref in registers
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            const float gii = (r & 3) == 0 ? Gd[t][0] : ((r & 3) == 1 ? Gd[t][1] : ((r & 3) == 2 ? Gd[t][2] : Gd[t][3]));
            if ((r >> 2) == g) hs[T_BA + 16 * t + r] = gii;
        }
        wave_lds_fence();
        {
            const float b = gdn ? eta_pre : kaczmarz_beta_fast(eta_pre, hs[T_BA + lane], a.eps);
            hs[T_BETA + lane] = b;
            hs[T_BA + lane] = b * av;
        }
        wave_lds_fence();

        // ---- decay, mask, beta on the tiles of L.  Row token I, column token J:
        //   I = 16 ti + r, J = 16 tj + 4 g + e
        // Every table value is read before the first block is written: the compiler keeps LDS reads behind earlier LDS
        // writes it cannot tell apart, and one round trip per tile would put this wave's whole phase on the LDS latency.
        floatx4 gq[4];
        float g2_r[4], beta_r[4];
        static_for<4>([&](auto tc) {
            constexpr int t = tc;
            gq[t] = *reinterpret_cast<const floatx4*>(hs + T_G2 + 16 * t + 4 * g);
            g2_r[t] = hs[T_G2 + 16 * t + r];
            beta_r[t] = hs[T_BETA + 16 * t + r];
        });
        static_for<4>([&](auto tc) {                     // diagonal tiles: 2^(g_I - g_J), J < I
            constexpr int t = tc;
            floatx4 l;
#pragma unroll
            for (int e = 0; e < 4; ++e)                  // strictly lower
                l[e] = (4 * g + e < r) ? beta_r[t] * __builtin_amdgcn_exp2f(fminf(g2_r[t] - gq[t][e], 0.f)) * Gd[t][e] : 0.f;
            // block t of L, row-major, for the substitution: L_tt[r][4 g + e] (see blk_piece)
            *reinterpret_cast<floatx4*>(hs + 256 * t + 16 * r + 4 * blk_piece(t, r, g)) = l;
        });
#pragma unroll
        for (int i = 0; i < 6; ++i) B::keep(Gt[i]);
    }

    __device__ __forceinline__ void phase_b(float* hs, char* rec, int lane_)
    {
        const int lane = opaque(lane_);
        const int r = lane & 15, g = lane >> 4;
        wave_lds_fence();
        // ---- strictly lower tiles of L: beta_I gamma_I/gamma_ref(I) (per row, lane r) times gamma_ref(I)/gamma_J.
        //      The factors are requested here; the products are formed below, while the first rows of the substitution
        //      are on their way from LDS.
        u32x2 Lq[6];
        floatx4 bq[6];
        float ba_r[4];
        static_for<4>([&](auto tic) {
            constexpr int ti = tic;
            if constexpr (ti > 0) {
                ba_r[ti] = hs[T_BA + 16 * ti + r];
                static_for<ti>([&](auto tjc) {
                    constexpr int tj = tjc;
                    bq[ti * (ti - 1) / 2 + tj] = *reinterpret_cast<const floatx4*>(hs + T_B + 64 * (ti - 1) + 16 * tj + 4 * g);
                });
            }
        });
        // ---- diagonal blocks: D_t = (I + L_tt)^{-1} by forward substitution on the blocks phase A left in the scratch;
        //      lane group g takes block g, lane r its column r; row i of L_tt is read by all 16 lanes of the group at
        //      once (a broadcast read), four rows ahead of its use
        {
            float* Lb = hs + 256 * g;
            const float* Lp[4];                          // Lp[x]: where piece x ^ g of a row starts
#pragma unroll
            for (int x = 0; x < 4; ++x) Lp[x] = Lb + 4 * (x ^ g);
            float xs[16];
            xs[0] = (r == 0) ? 1.f : 0.f;
            floatx4 rows[5][4];
            auto read_row = [&](auto ic) {
                constexpr int i = ic;
                if constexpr (i < 16) {
#pragma unroll
                    for (int c4 = 0; c4 < (i + 3) / 4; ++c4)
                        rows[i % 5][c4] = *reinterpret_cast<const floatx4*>(Lp[c4 ^ ((i >> 1) & 3)] + 16 * i);
                }
            };
            read_row(IntC<1>()); read_row(IntC<2>()); read_row(IntC<3>()); read_row(IntC<4>());
            static_for<4>([&](auto tic) {
                constexpr int ti = tic;
                static_for<ti>([&](auto tjc) {
                    constexpr int i = ti * (ti - 1) / 2 + tjc;
                    Lq[i] = to_quad((bq[i] * ba_r[ti]) * Gt[i]);
                });
            });
            static_for<15>([&](auto ic) {
                constexpr int i = ic + 1;
                read_row(IntC<i + 4>());
                float s0 = (i == r) ? 1.f : 0.f, s1 = 0.f;
                static_for<i>([&](auto rc) {
                    constexpr int rr = rc;
                    if constexpr (rr & 1) s1 -= rows[i % 5][rr >> 2][rr & 3] * xs[rr]; else s0 -= rows[i % 5][rr >> 2][rr & 3] * xs[rr];
                });
                xs[i] = s0 + s1;
            });
            wave_lds_fence();                            // every lane has read its rows of L
            // R_tt = D_t^T, row-major: R_tt[r][i] = D_t[i][r]
#pragma unroll
            for (int c4 = 0; c4 < 4; ++c4) {
                const floatx4 v = {xs[4 * c4], xs[4 * c4 + 1], xs[4 * c4 + 2], xs[4 * c4 + 3]};
                *reinterpret_cast<floatx4*>(Lb + 16 * r + 4 * blk_piece(g, r, c4)) = v;
            }
        }
        wave_lds_fence();
        floatx4 DA[4];                                   // D_t in A-operand order: D_t[r][4 g + j] = R_tt[4 g + j][r]
        {
            // element (row 4 g + e, column r) of block t sits in piece (r >> 2) ^ (2 g & 3) ^ (e >> 1) ^ t of its row
            const int cr = (r >> 2) ^ ((2 * g) & 3);
            int da[4];
#pragma unroll
            for (int x = 0; x < 4; ++x) da[x] = 64 * g + 4 * (cr ^ x) + (r & 3);
#pragma unroll
            for (int t = 0; t < 4; ++t)
#pragma unroll
                for (int e = 0; e < 4; ++e) DA[t][e] = hs[256 * t + 16 * e + da[(e >> 1) ^ t]];
        }

        // T-area of the record: the 16x16 blocks of the block forward substitution, in the tile-pair layout of T'
        // (record order (ti, jp) = (0,0) (1,0) (2,0) (2,1) (3,0) (3,1)):
        //     [D0 B0 | 0] [L10 | D1] [L20 | L21] [D2 | 0] [L30 | L31] [L32 | D3]
        // Only D0 carries beta on its columns (J = 4 g + e); for the other rows the scan applies beta to the right-hand side.
        const floatx4 bq0 = *reinterpret_cast<const floatx4*>(hs + T_BETA + 4 * g);
        const u32x2 zq = {0u, 0u};
        B::slot(rec, 0, 0, lane, to_quad(DA[0] * bq0), zq);
        B::slot(rec, 0, 1, lane, Lq[0], to_quad(DA[1]));
        B::slot(rec, 0, 2, lane, Lq[1], Lq[2]);
        B::slot(rec, 0, 3, lane, to_quad(DA[2]), zq);
        B::slot(rec, 0, 4, lane, Lq[3], Lq[4]);
        B::slot(rec, 0, 5, lane, Lq[5], to_quad(DA[3]));
        reinterpret_cast<float*>(rec + 2 * B::TPB)[192 + lane] = hs[T_BETA + lane];
    }
};

template <int DK, bool NQ>
struct PHelper : HelperBase<DK> {
    typedef HelperBase<DK> B;
    using B::KP; using B::wave_lds_fence; using B::pin; using B::opaque;
    static constexpr int SCR = 6 * 256;                  // private scratch: six tables of 64 floats
    static constexpr int T_G2 = 0, T_A = 64, T_RQ = 128, T_B = 192;
    // P^T tile (tj, ti), tj <= ti
    __host__ __device__ static constexpr int pidx(int tj, int ti) { return ti * (ti + 1) / 2 + tj; }

    u32x4 qa[KP][4];                        // Q row slots of the wave's next record (K comes through the ring stage)
    // carried from phase A to phase B
    static constexpr int TI_B = 3;          // strictly lower tiles (tj, ti) with ti >= TI_B are finished in phase B
    floatx4 GPd[4];                         // diagonal tiles of (K Q^T), row factors applied, before decay and mask
    floatx4 GPl[3];                         // tiles (tj, 3), row factors applied, before decay
    u32x2 Pt[10];                           // P^T tile (tj, ti) as A-operand quads, bf16: lane (r, g) holds P[I][J], I = 16 ti + r, J = 16 tj + 4 g + e
    float vgam, vdec, vgq;                  // lane = token: gamma_i, gamma_C / gamma_i, gamma_i / ||q_i||

    __device__ __forceinline__ void prefetch(const ScanArgs<bf16_t>& a, long tok0, int clen, int h, int lane_, const char* qc,
                                             int kq_row)
    {
        const int lane = opaque(lane_);
        this->la_pre = lane < clen ? a.log_alpha[(size_t)(tok0 + lane) * a.H + h] : 0.f;
        this->load_slots(qa, qc, lane, clen, kq_row);
    }

    // Phase A (step c - 2): Q goes on into the ring (the T-side wave does the same with K); gates, tables, query
    // norms; (Q K^T)^T on the matrix pipe; decay and mask.  qtile: the Q tile of the chunk's ring stage.
    // ktile, kflag, c: the K tile of the same ring stage, and the word that says the T-side wave has filled it for chunk c
    __device__ __forceinline__ void phase_a(float* hs, char* qtile, const char* ktile, const int* kflag, int c, int clen, int lane_)
    {
        const int lane = opaque(lane_);
        const int r = lane & 15, g = lane >> 4;
        floatx4 GP[10];                     // (K_tj Q_ti^T): accumulator tile (tj, ti), lane (r, g) holds k_J . q_I
        B::store_slots(qa, qtile, lane);
        float av, gl2;
        const float x2 = this->scan_gates(hs + T_G2, hs + T_B, lane, av, gl2);
        vgam = __builtin_amdgcn_exp2f(x2);
        vdec = __builtin_amdgcn_exp2f(gl2 - x2);
        hs[T_A + lane] = av;
        // K row slots from the ring stage, once the T-side wave of this chunk has stored them (it does so first thing in
        // the same step and waits for nobody, so the wait is short and always ends; the bound is a safeguard only)
        for (int spin = 0; *reinterpret_cast<const volatile int*>(kflag) != c && spin < (1 << 20); ++spin)
            __builtin_amdgcn_s_sleep(1);
        wave_lds_fence();
        u32x4 ka[KP][4];
        static_for<KP>([&](auto kpc) {
            static_for<4>([&](auto itc) { ka[kpc][itc] = B::ring_slot(ktile, itc, kpc, lane); });
        });
        const floatx4 z4 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int i = 0; i < 10; ++i) GP[i] = z4;
        float qss[4] = {0.f, 0.f, 0.f, 0.f};
        static_for<KP>([&](auto kc_) {
            constexpr int kp = kc_;
            static_for<4>([&](auto tic) {
                constexpr int ti = tic;
                const u32x4 q = qa[kp][ti];
                const u32x2 qb0 = {q[0], q[1]}, qb1 = {q[2], q[3]};
                static_for<ti + 1>([&](auto tjc) {
                    constexpr int tj = tjc;
                    mma_bf16(GP[pidx(tj, ti)], ka[kp][tj], qb0, qb1);      // rows <- K block tj, column <- Q block ti
                });
                if constexpr (NQ) {
#pragma unroll
                    for (int m = 0; m < 4; ++m) {
                        const float x0 = __uint_as_float(q[m] << 16), x1 = __uint_as_float(q[m] & 0xffff0000u);
                        qss[ti] += x0 * x0; qss[ti] += x1 * x1;
                    }
                }
            });
        });
        if constexpr (NQ) {
#pragma unroll
            for (int it = 0; it < 4; ++it) {
                float ss = qss[it];
                ss += __shfl_xor(ss, 16, kWave);
                ss += __shfl_xor(ss, 32, kWave);
                if (g == 0) hs[T_RQ + 16 * it + r] = ss > 0.f ? 1.0f / sqrtf(ss) : 0.f;
            }
            wave_lds_fence();
            vgq = vgam * hs[T_RQ + lane];
        } else {
            vgq = vgam;
            wave_lds_fence();
        }
        // ---- decay and mask.  Row token I = 16 ti + r, column token J = 16 tj + 4 g + e.
        static_for<4>([&](auto tic) {
            constexpr int ti = tic;
            const float rq_r = NQ ? hs[T_RQ + 16 * ti + r] : 1.f;
            // rows beyond a short chunk are zero: folded into the row factors
            const float live = (clen == 64 || 16 * ti + r < clen) ? 1.f : 0.f;
            const float aq_r = hs[T_A + 16 * ti + r] * rq_r * live;
            static_for<ti>([&](auto tjc) {
                constexpr int tj = tjc;
                if constexpr (ti < TI_B) {
                    const floatx4 bq = *reinterpret_cast<const floatx4*>(hs + T_B + 64 * (ti - 1) + 16 * tj + 4 * g);
                    Pt[pidx(tj, ti)] = to_quad((bq * aq_r) * GP[pidx(tj, ti)]);
                } else {
                    GPl[tj] = GP[pidx(tj, ti)] * aq_r;   // the last row of tiles gets its decay in phase B
                }
            });
            GPd[ti] = GP[pidx(ti, ti)] * (rq_r * live);  // the diagonal tiles get their decay and mask in phase B
        });
        static_for<4>([&](auto tic) {
            constexpr int ti = tic;
            B::keep(GPd[ti]);
            static_for<ti>([&](auto tjc) { if constexpr (ti < TI_B) B::keep(Pt[pidx(tjc, ti)]); else B::keep(GPl[tjc]); });
        });
    }

    // Phase B (step c - 1): decay and mask of the diagonal tiles, the record.
    __device__ __forceinline__ void phase_b(const float* hs, char* rec, int lane_)
    {
        const int lane = opaque(lane_);
        const int r = lane & 15, g = lane >> 4;
        const u32x2 zq = {0u, 0u};
        static_for<3>([&](auto tjc) {                    // tiles (tj, 3): gamma_ref(I) / gamma_J
            constexpr int tj = tjc;
            const floatx4 bq = *reinterpret_cast<const floatx4*>(hs + T_B + 64 * 2 + 16 * tj + 4 * g);
            Pt[pidx(tj, 3)] = to_quad(bq * GPl[tj]);
        });
        static_for<4>([&](auto tic) {                    // diagonal tiles: 2^(g_I - g_J), J <= I
            constexpr int ti = tic;
            const floatx4 gq = *reinterpret_cast<const floatx4*>(hs + T_G2 + 16 * ti + 4 * g);
            const float g2r = hs[T_G2 + 16 * ti + r];
            floatx4 p;
#pragma unroll
            for (int e = 0; e < 4; ++e)
                p[e] = (4 * g + e <= r) ? __builtin_amdgcn_exp2f(fminf(g2r - gq[e], 0.f)) * GPd[ti][e] : 0.f;
            Pt[pidx(ti, ti)] = to_quad(p);
        });
        // tile-pairs in record order (ti, jp) = (0,0) (1,0) (2,0) (2,1) (3,0) (3,1); tile (ti, tj) of P in A-operand order
        // is (P^T)(tj, ti)
        B::slot(rec, B::TPB, 0, lane, Pt[pidx(0, 0)], zq);
        B::slot(rec, B::TPB, 1, lane, Pt[pidx(0, 1)], Pt[pidx(1, 1)]);
        B::slot(rec, B::TPB, 2, lane, Pt[pidx(0, 2)], Pt[pidx(1, 2)]);
        B::slot(rec, B::TPB, 3, lane, Pt[pidx(2, 2)], zq);
        B::slot(rec, B::TPB, 4, lane, Pt[pidx(0, 3)], Pt[pidx(1, 3)]);
        B::slot(rec, B::TPB, 5, lane, Pt[pidx(2, 3)], Pt[pidx(3, 3)]);
        float* dec = reinterpret_cast<float*>(rec + 2 * B::TPB);
        dec[lane] = vgam;
        dec[64 + lane] = vdec;
        dec[128 + lane] = vgq;
    }
};

}  // namespace

// NQ: normalised read-out (Sec. 3.3): the output rows are scaled by 1/||q_i||, which stage 1 folded into P and
// into the third vector of the record, gamma_i/||q_i||, read here in place of gamma_i for the Q S term.
// DG: diagonal gating (App. B): a.k = K o Gamma and a.q = Q o Gamma feed K S and Q S, a.kt_src = K o (gamma_C/Gamma)
// the state update, the records carry unit decay vectors and the state rows decay by a.gc_vec (see intra_diag_kernel).
// FU: fused mode, see the top of the file; a.wsT / a.wsP / a.wsG are not used, a.log_alpha / a.eta / a.eps are.
template <int DK, int NW, bool NQ, bool DG = false, bool FU = false>
__global__ __launch_bounds__((64 * Cfg<DK, NW, DG, FU>::NWAVES)) void scan_bf16_kernel(ScanArgs<bf16_t> a)
{
    typedef Cfg<DK, NW, DG, FU> C;
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
    if (a.cu_seqlens) { t0 = a.cu_seqlens[s]; len = a.cu_seqlens[s + 1] - (int)t0; ch0 = FU ? 0 : a.chunk_off[s]; }
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
    const char* tpbase = FU ? nullptr : reinterpret_cast<const char*>(a.wsT) + ((size_t)ch0 * a.H + h) * REC;

    // ---- loop-invariant per-lane offsets ------------------------------------------------------------
    // copy engine, global side: lane l of copy block b fills LDS bytes [1024 b + 16 l, +16) of a tile, i.e.
    // row 1024 b / RB + l / PPR, physical column l % PPR, which holds logical column (l % PPR) ^ swz(row).
    // The swizzle has period 8 rows: it depends on the block through b % NGK.
    constexpr int NGK = 8 / RPB;
    const int lrow = lane / PPR, pcol = lane % PPR;
    int gk[NGK];
#pragma unroll
    for (int j = 0; j < NGK; ++j)
        gk[j] = lrow * (int)kq_row + ((pcol ^ swz_piece<DK>(RPB * j + lrow)) * 16);
    const int gv = (lane / VPP) * (int)v_row + (lane % VPP) * 16;
    // LDS reads.  K/Q row slots: token row 16 it + r, logical column 4 kp + g:
    int oK[KP];
#pragma unroll
    for (int kp = 0; kp < KP; ++kp) oK[kp] = r * RB + (((4 * kp + g) ^ swz_piece<DK>(r)) * 16);
    // K^T slots through the transposing read: source lane (a4, c4) points at token 4 g + a4 (+ 16 beta + 32 jp),
    // logical column 4 kp + c4, half b.
    const int a4 = r >> 2, c4 = r & 3;
    int oKT[KP];
#pragma unroll
    for (int kp = 0; kp < KP; ++kp) oKT[kp] = (4 * g + a4) * RB + (((4 * kp + c4) ^ swz_piece<DK>(4 * g + a4)) * 16);
    const int oV = (4 * g + a4) * VRW + (16 * wave + 4 * c4) * 2;      // V tile rows 4 g + a4 (+ 16 it)
    // staging tile: after the 4x4 transposition below lane (r, g) holds row 4 g + (r & 3) (+ 16 it), columns
    // 4 (r >> 2) .. + 3 of this wave's 16
    const int oO = (4 * g + (r & 3)) * ORB + (16 * wave + 4 * (r >> 2)) * 2;
    const bool q_lo = (r & 3) < 2;                       // lane sits in the upper half of its quad's 4x4 block
    const uint32_t psel = (r & 1) ? 0x03020706u : 0x05040100u;   // byte selectors of the 2x2 step (see below)

    // ---- global -> LDS copy of what chunk c needs ---------------------------------------------------
    // part 0: everything; parts 1 and 2: the split schedule of a two-stage ring (see the copy wave): 1 = what a chunk
    // step reads first (the K tile, the V slice, T', the vectors), 2 = the rest (Q, the second K tile, P).  One tile
    // after the other: the K, Q and second-K rows of one token sit at the same offset of three arrays, and requests for
    // them issued back to back meet in the same memory channel.
    auto issue = [&](int c, char* st, auto part_c) {
        constexpr int part = decltype(part_c)::value;
        constexpr bool first = part != 2, rest = part != 1;
        const int clen = min(64, len - 64 * c);
        auto tile = [&](const char* src, char* dst) {    // src: the chunk's first row of a [tokens][H][d_k] array
            if (clen == 64) {
                static_for<C::NKB>([&](auto i) {
                    const int b = i;
                    dma16(src + (size_t)(b * RPB) * kq_row, gk[b % NGK], dst + b * 1024);
                });
            } else {                                     // ragged last chunk: clamp the row
                static_for<C::NKB>([&](auto i) {
                    const int b = i;
                    const int row = b * RPB + lrow;
                    dma16(src, min(row, clen - 1) * (int)kq_row + ((pcol ^ swz_piece<DK>(row)) * 16), dst + b * 1024);
                });
            }
        };
        const char* tc = FU ? nullptr : tpbase + (size_t)c * a.H * REC;
        if constexpr (!FU && first) tile(kbase + (size_t)(64 * c) * kq_row, st);   // fused mode: the helper waves bring K and Q
        if constexpr (first) {
            const char* vc = vbase + (size_t)(64 * c) * v_row;
            if (clen == 64) {
                static_for<C::NVB>([&](auto i) {
                    const int b = i;
                    dma16(vc + (size_t)(b * RPV) * v_row, gv, st + C::OFF_V + b * 1024);
                });
            } else {
                static_for<C::NVB>([&](auto i) {
                    const int b = i;
                    const int row = b * RPV + lane / VPP;
                    dma16(vc, min(row, clen - 1) * (int)v_row + (lane % VPP) * 16, st + C::OFF_V + b * 1024);
                });
            }
            if constexpr (!FU) {
                static_for<C::NTB / 2>([&](auto i) {     // T': the first half of the record's tile area
                    const int b = i;
                    dma16(tc + b * 1024, lane * 16, st + C::OFF_T + b * 1024);
                });
                if (lane < 48) dma16(tc + 2 * C::TPB, lane * 16, st + C::OFF_EG);   // gamma_i | gamma_C/gamma_i | gamma_i/||q_i||: 768 bytes
            }
            if constexpr (DG) {
                if (lane < DK / 4) dma16(gcbase + (size_t)c * a.H * DK * 4, lane * 16, st + C::OFF_GC);   // gamma_C per channel
            }
        }
        if constexpr (rest) {
            if constexpr (!FU) {
                tile(qbase + (size_t)(64 * c) * kq_row, st + C::OFF_Q);
                if constexpr (DG) tile(k2base + (size_t)(64 * c) * kq_row, st + C::OFF_K2);
                static_for<C::NTB / 2>([&](auto i) {     // P: the second half
                    const int b = C::NTB / 2 + i;
                    dma16(tc + b * 1024, lane * 16, st + C::OFF_T + b * 1024);
                });
            }
        }
    };

    // ---- one chunk of the recurrence for this wave's 16 columns ------------------------------------
    // rc: where T', P and the vectors of this chunk are (the ring stage itself, or a record buffer when fused)
    auto compute = [&](const char* st, const char* rc, char* ost) {
        const char* pS = rc + lane * 16;                 // T' / P slots
        const char* pV = st + C::OFF_V + oV;
        const char* pG = rc + C::R_EG + 16 * g;          // 4 consecutive floats: rows 4 g .. 4 g + 3
        auto kslot = [&](int it, int kp, int base) {     // base 0: K, OFF_Q: Q
            return ld16(st + oK[kp] + base + 16 * it * RB);
        };
        auto ktslot = [&](int kt, int jp, u32x2& q0, u32x2& q1) {
            const int kp = kt >> 1, b = kt & 1;
            const char* p = st + oKT[kp] + (DG ? C::OFF_K2 : 0) + 32 * jp * RB + 8 * b;
            q0 = lds_read_tr(p);
            q1 = lds_read_tr(p + 16 * RB);
        };

        // bf16 copy of the incoming state (B operand of K S and Q S); the fp32 state is decayed right away
        const float gC = *reinterpret_cast<const float*>(rc + C::R_EG + 63 * 4);
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
        for (int i = 0; i < kTriPairs; ++i) tsl[i] = ld16(pS + C::R_T + i * 1024);
        // split schedule: Q, the second K tile and P of this chunk are guaranteed only behind this barrier
        if constexpr (C::SPLIT) __syncthreads();
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
        floatx4 Xf[3];                                   // fused mode: rows 16.. of X stay in fp32 until beta and the L U terms are in
        Xq[0] = to_quad(quad_to_f(vq[0]) - egv[0] * ks[0]);
#pragma unroll
        for (int it = 1; it < 4; ++it) {
            Xf[it - 1] = quad_to_f(vq[it]) - egv[it] * ks[it];
            if constexpr (!FU) Xq[it] = to_quad(Xf[it - 1]);
        }

        // K^T slots of the first state tiles and the P slots: on their way during the solve
        u32x2 kt[2][KB][2];                              // [token pair jp][state tile][token block]
#pragma unroll
        for (int t = 0; t < KB; ++t) ktslot(t, 0, kt[0][t][0], kt[0][t][1]);

        // ---- U = T' X (T' lower triangular); fused mode: the solve split at row 32 (see the helper section),
        //      U_top = T'11 X_top, U_bot = T22 (B_bot X_bot - L21 U_top)
        floatx4 U[4];
        u32x2 Uq[4], Udq[4];
        u32x4 psl[kTriPairs];
        if constexpr (!FU) {
#pragma unroll
            for (int it = 0; it < 4; ++it) {
                U[it] = floatx4{0.f, 0.f, 0.f, 0.f};
                mma_bf16(U[it], tsl[tri_pair(it, 0)], Xq[0], Xq[1]);
            }
            mma_bf16(U[2], tsl[tri_pair(2, 1)], Xq[2], Xq[3]);
            mma_bf16(U[3], tsl[tri_pair(3, 1)], Xq[2], Xq[3]);
#pragma unroll
            for (int t = 0; t < KB; ++t) ktslot(t, 1, kt[1][t][0], kt[1][t][1]);
#pragma unroll
            for (int i = 0; i < kTriPairs; ++i) psl[i] = ld16(pS + C::R_P + i * 1024);
#pragma unroll
            for (int it = 0; it < 4; ++it) {
                Udq[it] = to_quad(U[it] * edv[it]);
                Uq[it] = to_quad(U[it]);
            }
        }
        floatx4 o[4];
        if constexpr (!FU) {
            // ---- S = gamma_C S + K^T (diag(gamma_C/gamma_i) U): the only thing the next chunk waits for
#pragma unroll
            for (int t = 0; t < KB; ++t) mma_bf16(S[t], kt[0][t][0], kt[0][t][1], Udq[0], Udq[1]);
#pragma unroll
            for (int t = 0; t < KB; ++t) mma_bf16(S[t], kt[1][t][0], kt[1][t][1], Udq[2], Udq[3]);

            // ---- O = D_gamma Q S + P U (P lower triangular), staged token-major for 16-byte global stores
#pragma unroll
            for (int it = 0; it < 4; ++it) {
                if constexpr (NQ) o[it] = ld_f4(pG + 512 + 64 * it) * qs[it]; else o[it] = egv[it] * qs[it];
                mma_bf16(o[it], psl[tri_pair(it, 0)], Uq[0], Uq[1]);
            }
            mma_bf16(o[2], psl[tri_pair(2, 1)], Uq[2], Uq[3]);
            mma_bf16(o[3], psl[tri_pair(3, 1)], Uq[2], Uq[3]);
        } else {
            // Fused mode: block forward substitution over the four 16-row blocks (see the helper section for the record's
            // tiles), U_0 = (D0 B0) X_0, U_t = D_t (B_t X_t - sum_{j<t} L_tj U_j).  Its chain of eight dependent
            // products is interleaved with the products that need only the rows already solved: the first half of the
            // state update and of P U.
            const u32x2 zq = {0u, 0u};
            const floatx4 z4 = {0.f, 0.f, 0.f, 0.f};
            const floatx4 bv1 = ld_f4(pG + 768 + 64), bv2 = ld_f4(pG + 768 + 128), bv3 = ld_f4(pG + 768 + 192);   // beta of rows 16 t + 4 g ..
            U[0] = z4; mma_bf16(U[0], tsl[tri_pair(0, 0)], Xq[0], zq);
#pragma unroll
            for (int t = 0; t < KB; ++t) ktslot(t, 1, kt[1][t][0], kt[1][t][1]);
#pragma unroll
            for (int i = 0; i < kTriPairs; ++i) psl[i] = ld16(pS + C::R_P + i * 1024);
#pragma unroll
            for (int it = 0; it < 4; ++it) {
                if constexpr (NQ) o[it] = ld_f4(pG + 512 + 64 * it) * qs[it]; else o[it] = egv[it] * qs[it];
            }
            Uq[0] = to_quad(U[0]); Udq[0] = to_quad(U[0] * edv[0]);
            floatx4 W = z4; mma_bf16(W, tsl[tri_pair(1, 0)], Uq[0], zq);                 // L10 U_0
            U[1] = z4; mma_bf16(U[1], tsl[tri_pair(1, 0)], zq, to_quad(bv1 * Xf[0] - W));   // D1 (..)
            Uq[1] = to_quad(U[1]); Udq[1] = to_quad(U[1] * edv[1]);
            W = z4; mma_bf16(W, tsl[tri_pair(2, 0)], Uq[0], Uq[1]);                       // L20 U_0 + L21 U_1
            floatx4 W3 = z4; mma_bf16(W3, tsl[tri_pair(3, 0)], Uq[0], Uq[1]);             // L30 U_0 + L31 U_1
#pragma unroll
            for (int t = 0; t < KB; ++t) mma_bf16(S[t], kt[0][t][0], kt[0][t][1], Udq[0], Udq[1]);
#pragma unroll
            for (int it = 0; it < 4; ++it) mma_bf16(o[it], psl[tri_pair(it, 0)], Uq[0], Uq[1]);
            U[2] = z4; mma_bf16(U[2], tsl[tri_pair(2, 1)], to_quad(bv2 * Xf[1] - W), zq);    // D2 (..)
            Uq[2] = to_quad(U[2]); Udq[2] = to_quad(U[2] * edv[2]);
            mma_bf16(W3, tsl[tri_pair(3, 1)], Uq[2], zq);                                  // + L32 U_2
            U[3] = z4; mma_bf16(U[3], tsl[tri_pair(3, 1)], zq, to_quad(bv3 * Xf[2] - W3));   // D3 (..)
            Uq[3] = to_quad(U[3]); Udq[3] = to_quad(U[3] * edv[3]);
#pragma unroll
            for (int t = 0; t < KB; ++t) mma_bf16(S[t], kt[1][t][0], kt[1][t][1], Udq[2], Udq[3]);
            mma_bf16(o[2], psl[tri_pair(2, 1)], Uq[2], Uq[3]);
            mma_bf16(o[3], psl[tri_pair(3, 1)], Uq[2], Uq[3]);
        }
        // transposed 4x4 inside each quad of lanes (see quad_transpose4x4): one 64-bit LDS write per tile (a compute
        // wave is bound by its instruction count)
#pragma unroll
        for (int it = 0; it < 4; ++it)
            *reinterpret_cast<u32x2*>(ost + oO + 16 * it * ORB) = quad_transpose4x4(to_quad(o[it]), q_lo, psel);
    };

    // The staged output tile of chunk c goes to memory 16 bytes per thread, by a wave that has nothing else to do, so
    // that the compute waves go straight on to the next chunk (the write-out cost them 250 of a step's 2 800 cycles).
    auto write_out = [&](int c, const char* ost, int t_idx, auto n_thr) {
        constexpr int NT = decltype(n_thr)::value;
        const int clen = min(64, len - 64 * c);
        char* ob = reinterpret_cast<char*>(a.o) + (size_t)(t0 + 64L * c) * v_row + ((size_t)h * a.dv + slice * SLW) * 2;
#pragma unroll
        for (int it = 0; it < 64 * VPP / NT; ++it) {
            const int i = t_idx + NT * it;
            const int row = i / VPP, pv = i % VPP;
            // outputs are written once and not read again by this kernel: streamed past the caches
            if (row < clen) __builtin_nontemporal_store(ld16(ost + row * ORB + pv * 16), reinterpret_cast<u32x4*>(ob + (size_t)row * v_row + pv * 16));
        }
    };

    char* ost0 = lds + NST * C::STAGE;
    char* ost1 = ost0 + C::OSB;

    // Fused mode: every wave passes nch + 2 barriers.  Step s = -2 .. nch - 1 ends with one; in step s the compute waves
    // work on chunk s, the helpers of parity (s & 1) are in phase A of chunk s + 2 and those of the other parity in
    // phase B of chunk s + 1, whose record goes into buffer (s + 1) & 1, which chunk s - 1 left free.
    if constexpr (FU) {
        // K reaches the P-side wave of a chunk through the ring stage, where the T-side wave of the same chunk puts it in
        // the same step: a word per chunk parity says which chunk's K is there.  The two words live in the padding of the
        // first two rows of the output staging tile (a row holds at most 64 of its ORB = 96 bytes).
        if (tid < 2) *reinterpret_cast<int*>(ost0 + 64 + C::ORB * tid) = -1;
        __syncthreads();
        if (wave == C::W_IDLE) {
            // Sits where it does so that the P-side helpers land on the SIMDs of the T-side ones (see Cfg::NWAVES); its
            // work is the write-out: after the barrier that ends step s, chunk s is complete in the staging tile of its
            // parity, which the compute waves write again only in step s + 2, behind the barrier this wave reaches next.
            for (int s = -2; s < nch; ++s) {
                __syncthreads();
                if (s >= 0) write_out(s, (s & 1) ? ost1 : ost0, lane, IntC<64>());
            }
            return;
        }
        // A helper of parity hh takes the chunks c = hh, hh + 2, ..: phase A in step c - 2, phase B in step c - 1, so it
        // simply alternates the two (the odd one idles through step -2), and tops up the barrier count at the end.
        if (wave == NW || wave == NW + 1) {              // T-side helpers
            const int hh = wave - NW;
            float* hs = reinterpret_cast<float*>(lds + C::OFF_HST + hh * C::HSCR_T);
            THelper<DK> hp;
            hp.init_rows(lane, (int)kq_row);
            auto fetch = [&](int c) {
                hp.prefetch(a, t0 + 64L * c, min(64, len - 64 * c), h, lane, kbase + (size_t)(64 * c) * kq_row, (int)kq_row);
            };
            int nb = 0;
            if (hh < nch) fetch(hh);                     // this wave's first record
            if (hh == 1) { __syncthreads(); ++nb; }
            for (int c = hh; c < nch; c += 2) {
                hp.phase_a(a, hs, lds + (c % NST) * C::STAGE, reinterpret_cast<int*>(ost0 + 64 + C::ORB * hh), c, lane);
                __syncthreads(); ++nb;
                if (c + 2 < nch) fetch(c + 2);           // on their way during this step, used in the next
                hp.phase_b(hs, lds + C::OFF_REC + (c & 1) * C::RECB, lane);
                __syncthreads(); ++nb;
            }
            for (; nb < nch + 2; ++nb) __syncthreads();
            return;
        }
        if (wave == C::W_P || wave == C::W_P + 1) {          // P-side helpers
            // the P-side wave of the even chunks shares its SIMD with the T-side wave of the odd ones and vice versa: in
            // every step each of the two SIMDs then has one wave in phase A and one in phase B
            const int hh = 1 - (wave - C::W_P);
            float* hs = reinterpret_cast<float*>(lds + C::OFF_HSP + hh * C::HSCR_P);
            PHelper<DK, NQ> hp;
            hp.init_rows(lane, (int)kq_row);
            auto fetch = [&](int c) {
                hp.prefetch(a, t0 + 64L * c, min(64, len - 64 * c), h, lane, qbase + (size_t)(64 * c) * kq_row, (int)kq_row);
            };
            int nb = 0;
            if (hh < nch) fetch(hh);
            if (hh == 1) { __syncthreads(); ++nb; }
            for (int c = hh; c < nch; c += 2) {
                hp.phase_a(hs, lds + (c % NST) * C::STAGE + C::OFF_Q, lds + (c % NST) * C::STAGE,
                           reinterpret_cast<const int*>(ost0 + 64 + C::ORB * hh), c, min(64, len - 64 * c), lane);
                __syncthreads(); ++nb;
                if (c + 2 < nch) fetch(c + 2);
                hp.phase_b(hs, lds + C::OFF_REC + (c & 1) * C::RECB, lane);
                __syncthreads(); ++nb;
            }
            for (; nb < nch + 2; ++nb) __syncthreads();
            return;
        }
    }

    if constexpr (C::SPLIT) {
        if (wave == C::W_COPY) {
            // ---- the copy wave, split schedule.  With two stages a chunk's copies cannot start before the step in
            // which the chunk before it is computed; issued and awaited in one piece they would have to be issued and
            // to land, one after the other, within that step (measured: 2.2 us for the 66 KB, against 1.2 us of
            // compute).  In two parts, each has a full step: the first part of chunk c + 1 goes out at the start of
            // step c and is awaited at its end; the second part goes out behind the barrier in step c and is awaited
            // before that barrier of step c + 1.  The stage they fill was left by chunk c - 1 at the end of its step.
            // Copies retire in order, so "all but the last n" is a wait on the counter.
            if (nch > 0) {
                issue(0, lds, IntC<1>());
                issue(0, lds, IntC<2>());
                wait_vmcnt<C::N_REST>();                 // first part of chunk 0
            }
            __syncthreads();
            for (int c = 0; c < nch; ++c) {
                const bool ahead = c + 1 < nch;
                char* nx = lds + ((c + 1) & 1) * C::STAGE;
                if (ahead) { issue(c + 1, nx, IntC<1>()); wait_vmcnt<C::N_FIRST>(); } else wait_vmcnt<0>();   // second part of chunk c
                __syncthreads();                         // in step c, before the first read of Q
                if (ahead) { issue(c + 1, nx, IntC<2>()); wait_vmcnt<C::N_REST>(); } else wait_vmcnt<0>();    // first part of chunk c + 1
                __syncthreads();                         // end of step c
            }
            return;
        }
    }
    if (wave == C::W_COPY) {
        // ---- the copy wave: keeps chunks c+1 .. c+NST-1 on their way while chunk c is computed ---------
#pragma unroll
        for (int p = 0; p < NST - 1; ++p)
            if (p < nch) issue(p, lds + p * C::STAGE, IntC<0>());
        if constexpr (FU) __syncthreads();               // step -2
        if (NST == 3 && nch > 1) wait_vmcnt<(NST == 3 ? C::NDMA : 0)>(); else wait_vmcnt<0>();      // chunk 0 has landed
        __syncthreads();
        int spre = NST - 1;                              // ring position of chunk c + NST - 1
        for (int c = 0; c < nch; ++c) {
            const bool ahead = c + NST - 1 < nch;
            // the stage being refilled was read by chunk c-1, which every wave finished before the last barrier
            if (ahead) issue(c + NST - 1, lds + spre * C::STAGE, IntC<0>());
            // Copies retire in order and this wave issues nothing else: all but the NDMA just issued (when
            // NST = 3) have landed once the counter is down to NDMA, i.e. chunk c+1 is complete.
            if (NST == 3 && ahead) wait_vmcnt<(NST == 3 ? C::NDMA : 0)>(); else wait_vmcnt<0>();
            __syncthreads();
            spre = (spre + 1 == NST) ? 0 : spre + 1;
        }
        return;
    }

    if constexpr (!FU) {
        if (wave == C::W_IDLE) {
            // ---- the write-out wave: behind the barrier that ends step c, chunk c is complete in the staging tile of
            // its parity, which the compute waves write again only in step c + 2, behind the barrier this wave reaches
            // after the write-out
            __syncthreads();
            for (int c = 0; c < nch; ++c) {
                if constexpr (C::SPLIT) __syncthreads();
                __syncthreads();
                write_out(c, (c & 1) ? ost1 : ost0, lane, IntC<64>());
            }
            return;
        }
    }

    // ---- compute waves ---------------------------------------------------------------------------------
    if constexpr (FU) __syncthreads();                   // step -2
    __syncthreads();                                     // chunk 0 is in stage 0 (and its record in buffer 0)
    int scur = 0;                                        // ring position of chunk c
    for (int c = 0; c < nch; ++c) {
        char* ost = (c & 1) ? ost1 : ost0;
        compute(lds + scur * C::STAGE, FU ? lds + C::OFF_REC + (c & 1) * C::RECB : lds + scur * C::STAGE, ost);
        // The barrier that ends a chunk step: staged outputs before their write-out; chunk c+1's operands before
        // their use; all reads of this stage before it is refilled; and the write-out of chunk c-1 (finished by
        // its wave before it arrives here) before the staging tile of that parity is written again in chunk c+1.
        __syncthreads();
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
            if (nq) hipLaunchKernelGGL((scan_bf16_kernel<DK, 1, true>), grid, dim3(64 * 3), 0, st, a);
            else    hipLaunchKernelGGL((scan_bf16_kernel<DK, 1, false>), grid, dim3(64 * 3), 0, st, a);
            break;
        case 2:
            if (nq) hipLaunchKernelGGL((scan_bf16_kernel<DK, 2, true>), grid, dim3(64 * 4), 0, st, a);
            else    hipLaunchKernelGGL((scan_bf16_kernel<DK, 2, false>), grid, dim3(64 * 4), 0, st, a);
            break;
        default:
            if (nq) hipLaunchKernelGGL((scan_bf16_kernel<DK, 4, true>), grid, dim3(64 * 6), 0, st, a);
            else    hipLaunchKernelGGL((scan_bf16_kernel<DK, 4, false>), grid, dim3(64 * 6), 0, st, a);
            break;
    }
    return hipGetLastError();
}

hipError_t launch_scan_bf16(const ScanArgs<bf16_t>& a, int dk, int waves, hipStream_t st)
{
    if (dk == 64) return launch_dk<64>(a, waves, st);
    return launch_dk<128>(a, waves, st);
}

template <int DK>
static hipError_t launch_fused_dk(const ScanArgs<bf16_t>& a, int waves, hipStream_t st)
{
    const int n_states = a.n_seq > 0 ? a.n_seq : (a.seg_G > 0 ? a.N * a.seg_G : a.N);
    const int n_chains = n_states * a.H;
    if (n_chains == 0) return hipSuccess;
    const dim3 grid((unsigned)(((n_chains + 7) / 8) * 8 * (a.dv / (16 * waves))));
    const bool nq = (a.opts & kOptNormalizeQ) != 0;
    if (waves == 1) {
        if (nq) hipLaunchKernelGGL((scan_bf16_kernel<DK, 1, true, false, true>), grid, dim3(64 * Cfg<DK, 1, false, true>::NWAVES), 0, st, a);
        else    hipLaunchKernelGGL((scan_bf16_kernel<DK, 1, false, false, true>), grid, dim3(64 * Cfg<DK, 1, false, true>::NWAVES), 0, st, a);
    } else {
        if (nq) hipLaunchKernelGGL((scan_bf16_kernel<DK, 2, true, false, true>), grid, dim3(64 * Cfg<DK, 2, false, true>::NWAVES), 0, st, a);
        else    hipLaunchKernelGGL((scan_bf16_kernel<DK, 2, false, false, true>), grid, dim3(64 * Cfg<DK, 2, false, true>::NWAVES), 0, st, a);
    }
    return hipGetLastError();
}
hipError_t launch_scan_fused_bf16(const ScanArgs<bf16_t>& a, int dk, int waves, hipStream_t st)
{
    if ((waves != 1 && waves != 2) || !a.log_alpha || !a.eta) return hipErrorInvalidValue;
    return dk == 64 ? launch_fused_dk<64>(a, waves, st) : launch_fused_dk<128>(a, waves, st);
}

// diagonal gating: waves = 1 or 2, fixed-length or packed batches, no options, no segments
template <int DK>
static hipError_t launch_diag_dk(const ScanArgs<bf16_t>& a, int waves, hipStream_t st)
{
    const int n_chains = (a.n_seq > 0 ? a.n_seq : a.N) * a.H;
    if (n_chains == 0) return hipSuccess;
    const dim3 grid((unsigned)(((n_chains + 7) / 8) * 8 * (a.dv / (16 * waves))));
    if (waves == 1) hipLaunchKernelGGL((scan_bf16_kernel<DK, 1, false, true>), grid, dim3(64 * 3), 0, st, a);
    else            hipLaunchKernelGGL((scan_bf16_kernel<DK, 2, false, true>), grid, dim3(64 * 4), 0, st, a);
    return hipGetLastError();
}
hipError_t launch_scan_bf16_diag(const ScanArgs<bf16_t>& a, int dk, int waves, hipStream_t st)
{
    if ((waves != 1 && waves != 2) || a.seg_G > 0 || !a.kt_src || !a.gc_vec) return hipErrorInvalidValue;
    return dk == 64 ? launch_diag_dk<64>(a, waves, st) : launch_diag_dk<128>(a, waves, st);
}

}  // namespace kla
