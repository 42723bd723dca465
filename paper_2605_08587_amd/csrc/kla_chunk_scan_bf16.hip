// bf16 inter-chunk stage: same recurrence as kla_chunk_scan.hip (eqs. (6)-(8) per chunk, the fp32
// state of 16 columns per wave held in MFMA accumulators for the whole sequence), tuned for the
// latency of the serial chunk loop on gfx950:
//
//   * K, Q and the V slice are staged in LDS as plain token-major rows (16-byte columns XOR-swizzled
//     by the row), written with full 128-bit stores in the order they arrive from global memory.
//   * A operands whose contraction runs along a row (K S, Q S) are single 128-bit LDS reads of 8
//     consecutive features.  To make that match the accumulator-as-B-operand trick of kla_mma.hpp,
//     the state tiles carry a permuted feature index: element e of lane (r, g) of state tile
//     kt = 2*kp + b is feature 32*kp + 8*g + 4*b + e.
//   * A operands whose contraction runs down a column (K^T for the state update, and the V tile
//     that initialises an accumulator) are read with the transposing LDS load
//     (ds_read_b64_tr_b16): in each group of 16 lanes, lane j supplies the address of 4 consecutive
//     elements, lanes 4a..4a+3 together forming row a of a 4x16 block, and lane i receives column
//     i of that block.  No transposed copy of K exists anywhere.
//   * LDS reads are issued in batches ahead of the MFMAs that consume them, the next chunk's
//     operands travel global -> registers -> other LDS stage behind the current chunk's products,
//     and there is one barrier per chunk.
//   * A short last chunk is handled without branches: rows beyond it re-read the last valid row;
//     their T' rows and columns are zero (beta = 0 there), so they contribute nothing to U, to the
//     state or to any stored output.
#include "kla_common.hpp"
#include "kla_kernels.hpp"
#include "kla_mma.hpp"

namespace kla {

namespace {

typedef short short4v __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));   // native 128-bit register value (never a stack object)
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ u32x4 ld16(const void* p) { return *reinterpret_cast<const u32x4*>(p); }
__device__ __forceinline__ void st16(void* p, u32x4 v) { *reinterpret_cast<u32x4*>(p) = v; }
typedef __attribute__((address_space(3))) short4v* lds_short4_ptr;

// 16-byte column swizzle of a token-major LDS tile: rows t..t+7 of one logical column land in 8
// different bank groups (conflict-free 128-bit row reads), and the 16 lanes of a transposing read
// (4 rows x 4 columns) land on 8 groups, two lanes each.
__device__ __forceinline__ int swz(int col16, int row)
{
    return col16 ^ (((row & 1) << 2) | ((row >> 1) & 3));
}

__device__ __forceinline__ u32x2 lds_read_tr(const char* p)
{
    const short4v v = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_short4_ptr)(p));
    return __builtin_bit_cast(u32x2, v);
}

__device__ __forceinline__ void mma_bf16(floatx4& acc, u32x4 a, u32x2 b0, u32x2 b1)
{
    const u32x4 b = {b0.x, b0.y, b1.x, b1.y};
    acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, a), __builtin_bit_cast(bf16x8_t, b),
                                                  acc, 0, 0, 0);
}
__device__ __forceinline__ void mma_bf16(floatx4& acc, u32x2 a0, u32x2 a1, u32x2 b0, u32x2 b1)
{
    const u32x4 a = {a0.x, a0.y, a1.x, a1.y};
    mma_bf16(acc, a, b0, b1);
}
__device__ __forceinline__ u32x2 to_quad(floatx4 x)
{
    const u32x2 q = {pack_bf16x2(x[0], x[1]), pack_bf16x2(x[2], x[3])};
    return q;
}
__device__ __forceinline__ floatx4 quad_to_f(u32x2 q)
{
    floatx4 r;
    r[0] = bf16_bits_to_float(q.x & 0xffffu); r[1] = bf16_bits_to_float(q.x >> 16);
    r[2] = bf16_bits_to_float(q.y & 0xffffu); r[3] = bf16_bits_to_float(q.y >> 16);
    return r;
}
__device__ __forceinline__ floatx4 ld_f4(const float* p) { return *reinterpret_cast<const floatx4*>(p); }

template <int DK, int NW>
struct Cfg {
    static constexpr int NTH = 64 * NW;
    static constexpr int KB = DK / 16, KP = DK / 32;
    static constexpr int SLW = 16 * NW;                  // state columns per workgroup
    static constexpr int RB = DK * 2;                    // bytes per K/Q row in LDS
    static constexpr int PPR = DK / 8;                   // 16-byte pieces per K/Q row
    static constexpr int VPP = SLW / 8;                  // pieces per V/O slice row
    static constexpr int VRB = SLW * 2 + 16;             // padded V / O row stride in LDS
    static constexpr int TPB = kTriPairs * 64 * 16;      // bytes of one T' or P area
    static constexpr int OFF_Q = 64 * RB, OFF_T = 2 * 64 * RB, OFF_P = OFF_T + TPB, OFF_V = OFF_P + TPB,
                         OFF_EG = OFF_V + 64 * VRB, OFF_ED = OFF_EG + 256, STAGE = OFF_ED + 256;
    static constexpr int OSB = 64 * VRB;                 // output staging tile
    static constexpr int LDS = 2 * (STAGE + OSB);
    static constexpr int UKQ = 64 * PPR / NTH;           // K (and Q) pieces per thread
    static constexpr int UV = 64 * VPP / NTH;            // V pieces per thread (= 2)
    static constexpr int TP16 = TPB / 16;
    static constexpr int UT = (TP16 + NTH - 1) / NTH;
    static_assert(64 * PPR % NTH == 0 && 64 * VPP % NTH == 0, "piece counts must divide");
    static_assert(LDS <= 160 * 1024, "LDS budget of a gfx950 CU");
};

template <int DK, int NW> struct Pref {
    typedef Cfg<DK, NW> C;
    u32x4 k[C::UKQ], q[C::UKQ], v[C::UV], t[C::UT], p[C::UT];
    float gv, gl;
};

}  // namespace

template <int DK, int NW>
__global__ __launch_bounds__(64 * NW) void scan_bf16_kernel(ScanArgs<bf16_t> a)
{
    typedef Cfg<DK, NW> C;
    constexpr int NTH = C::NTH, KB = C::KB, KP = C::KP, SLW = C::SLW, RB = C::RB, PPR = C::PPR, VPP = C::VPP,
                  VRB = C::VRB;

    __shared__ __attribute__((aligned(16))) char lds[C::LDS];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int r = lane & 15, g = lane >> 4;

    // ---- workgroup -> (sequence, head, column slice); slices of one head share an XCD (ids congruent mod 8)
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
    const int col = slice * SLW + 16 * wave + r;

    // state tile kt = 2*kp + b, element e  <->  feature 32*kp + 8*g + 4*b + e, column `col`
    floatx4 S[KB];
#pragma unroll
    for (int kt = 0; kt < KB; ++kt)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int f = 32 * (kt >> 1) + 8 * g + 4 * (kt & 1) + e;
            S[kt][e] = a.h0 ? a.h0[((size_t)chain * DK + f) * a.dv + col] : 0.f;
        }

    const size_t kq_stride = (size_t)a.H * DK, v_stride = (size_t)a.H * a.dv;
    const bf16_t* kbase = a.k + (size_t)t0 * kq_stride + (size_t)h * DK;
    const bf16_t* qbase = a.q + (size_t)t0 * kq_stride + (size_t)h * DK;
    const bf16_t* vbase = a.v + (size_t)t0 * v_stride + (size_t)h * a.dv + slice * SLW;

    // ---- global -> registers -----------------------------------------------------------------------
    auto fetch = [&](int c, Pref<DK, NW>& pf) {
        const int last = min(64, len - 64 * c) - 1;      // rows beyond the chunk re-read its last row
        const size_t ch = (size_t)(ch0 + c) * a.H + h;
        static_for<C::UKQ>([&](auto it) {
            const int i = tid + NTH * it;
            const size_t off = (size_t)(64 * c + min(i / PPR, last)) * kq_stride + (i % PPR) * 8;
            pf.k[it] = ld16(kbase + off);
            pf.q[it] = ld16(qbase + off);
        });
        static_for<C::UV>([&](auto it) {
            const int i = tid + NTH * it;
            pf.v[it] = ld16(vbase + (size_t)(64 * c + min(i / VPP, last)) * v_stride + (i % VPP) * 8);
        });
        const u32x4* tsrc = reinterpret_cast<const u32x4*>(reinterpret_cast<const char*>(a.wsT) + ch * C::TPB);
        const u32x4* psrc = reinterpret_cast<const u32x4*>(reinterpret_cast<const char*>(a.wsP) + ch * C::TPB);
        static_for<C::UT>([&](auto it) {
            const int i = min(tid + NTH * it, C::TP16 - 1);
            pf.t[it] = tsrc[i]; pf.p[it] = psrc[i];
        });
        pf.gv = a.wsG[ch * 64 + lane];
        pf.gl = a.wsG[ch * 64 + 63];
    };

    // ---- registers -> LDS stage ----------------------------------------------------------------------
    auto stash = [&](const Pref<DK, NW>& pf, char* st) {
        static_for<C::UKQ>([&](auto it) {
            const int i = tid + NTH * it;
            const int row = i / PPR, piece = i % PPR;
            const int o = row * RB + swz(piece, row) * 16;
            st16(st + o, pf.k[it]);
            st16(st + C::OFF_Q + o, pf.q[it]);
        });
        static_for<C::UV>([&](auto it) {
            const int i = tid + NTH * it;
            st16(st + C::OFF_V + (i / VPP) * VRB + (i % VPP) * 16, pf.v[it]);
        });
        static_for<C::UT>([&](auto it) {
            const int i = tid + NTH * it;
            if (C::TP16 % NTH == 0 || i < C::TP16) {
                st16(st + C::OFF_T + i * 16, pf.t[it]);
                st16(st + C::OFF_P + i * 16, pf.p[it]);
            }
        });
        if (tid < 64) {
            reinterpret_cast<float*>(st + C::OFF_EG)[tid] = expf(pf.gv);            // gamma_i
            reinterpret_cast<float*>(st + C::OFF_ED)[tid] = expf(pf.gl - pf.gv);    // gamma_C / gamma_i
        }
    };

    // ---- one chunk of the recurrence for this wave's 16 columns ------------------------------------
    auto compute = [&](const char* st, char* ost) {
        const char* Kr = st;
        const char* Qr = st + C::OFF_Q;
        const float* eg = reinterpret_cast<const float*>(st + C::OFF_EG);
        const float* ed = reinterpret_cast<const float*>(st + C::OFF_ED);

        u32x2 Sq[KB];
#pragma unroll
        for (int kt = 0; kt < KB; ++kt) Sq[kt] = to_quad(S[kt]);

        // operands that do not depend on the state: T' slots, V tile, decay factors
        u32x4 tsl[kTriPairs];
#pragma unroll
        for (int i = 0; i < kTriPairs; ++i) tsl[i] = ld16(st + C::OFF_T + (i * 64 + lane) * 16);
        u32x2 vq[4];
        floatx4 egv[4], edv[4];
#pragma unroll
        for (int it = 0; it < 4; ++it) {
            // lane j of a 16-lane group supplies row a = j/4 (token 16*it + 4*g + a), columns 4*(j%4)..+3
            vq[it] = lds_read_tr(st + C::OFF_V + (16 * it + 4 * g + (r >> 2)) * VRB + (16 * wave + 4 * (r & 3)) * 2);
            egv[it] = ld_f4(eg + 16 * it + 4 * g);
            edv[it] = ld_f4(ed + 16 * it + 4 * g);
        }

        // K S and Q S: A slots are 8 consecutive features of token row 16*it + r
        floatx4 ks[4], qs[4];
        u32x4 ka[KP], qa[KP];
#pragma unroll
        for (int kp = 0; kp < KP; ++kp) {
            const int o = r * RB + swz(4 * kp + g, r) * 16;
            ka[kp] = ld16(Kr + o);
            qa[kp] = ld16(Qr + o);
        }
#pragma unroll
        for (int it = 0; it < 4; ++it) {
            u32x4 kn[KP], qn[KP];
            if (it < 3) {
#pragma unroll
                for (int kp = 0; kp < KP; ++kp) {
                    const int row = 16 * (it + 1) + r;
                    const int o = row * RB + swz(4 * kp + g, row) * 16;
                    kn[kp] = ld16(Kr + o);
                    qn[kp] = ld16(Qr + o);
                }
            }
            ks[it] = floatx4{0.f, 0.f, 0.f, 0.f};
            qs[it] = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int kp = 0; kp < KP; ++kp) mma_bf16(ks[it], ka[kp], Sq[2 * kp], Sq[2 * kp + 1]);
#pragma unroll
            for (int kp = 0; kp < KP; ++kp) mma_bf16(qs[it], qa[kp], Sq[2 * kp], Sq[2 * kp + 1]);
            if (it < 3) {
#pragma unroll
                for (int kp = 0; kp < KP; ++kp) { ka[kp] = kn[kp]; qa[kp] = qn[kp]; }
            }
        }

        // X = V - D_gamma K S ;  U = T' X
        u32x2 Xq[4];
#pragma unroll
        for (int it = 0; it < 4; ++it) Xq[it] = to_quad(quad_to_f(vq[it]) - egv[it] * ks[it]);

        // first K^T slots for the state update: issue before the solve so they arrive during it
        auto kt_slot = [&](int kt, int jp, u32x2& q0, u32x2& q1) {
            const int kp = kt >> 1, b = kt & 1;
            const int a4 = r >> 2, c4 = r & 3;
            const int tok = 32 * jp + 4 * g + a4;
            q0 = lds_read_tr(Kr + tok * RB + swz(4 * kp + c4, tok) * 16 + 8 * b);
            q1 = lds_read_tr(Kr + (tok + 16) * RB + swz(4 * kp + c4, tok + 16) * 16 + 8 * b);
        };
        u32x2 kt0[2][2];
        kt_slot(0, 0, kt0[0][0], kt0[0][1]);
        kt_slot(0, 1, kt0[1][0], kt0[1][1]);

        floatx4 U[4];
        u32x2 Uq[4], Udq[4];
#pragma unroll
        for (int it = 0; it < 4; ++it) {
            U[it] = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int jp = 0; jp <= (it >> 1); ++jp) {
                const u32x4 sl = tsl[tri_pair(it, jp)];
                mma_bf16(U[it], sl, Xq[2 * jp], Xq[2 * jp + 1]);
            }
        }
#pragma unroll
        for (int it = 0; it < 4; ++it) {
            Uq[it] = to_quad(U[it]);
            Udq[it] = to_quad(U[it] * edv[it]);
        }
        // P slots for the outputs: in flight during the state update
        u32x4 psl[kTriPairs];
#pragma unroll
        for (int i = 0; i < kTriPairs; ++i) psl[i] = ld16(st + C::OFF_P + (i * 64 + lane) * 16);

        // S = gamma_C S + K^T (diag(gamma_C/gamma_i) U): the only thing the next chunk waits for
        const float gC = eg[63];
#pragma unroll
        for (int kt = 0; kt < KB; ++kt) {
            u32x2 nx[2][2];
            if (kt + 1 < KB) {
                kt_slot(kt + 1, 0, nx[0][0], nx[0][1]);
                kt_slot(kt + 1, 1, nx[1][0], nx[1][1]);
            }
            S[kt] = S[kt] * gC;
            mma_bf16(S[kt], kt0[0][0], kt0[0][1], Udq[0], Udq[1]);
            mma_bf16(S[kt], kt0[1][0], kt0[1][1], Udq[2], Udq[3]);
            if (kt + 1 < KB) {
                kt0[0][0] = nx[0][0]; kt0[0][1] = nx[0][1]; kt0[1][0] = nx[1][0]; kt0[1][1] = nx[1][1];
            }
        }

        // O = D_gamma Q S + P U, staged token-major for 16-byte global stores
#pragma unroll
        for (int it = 0; it < 4; ++it) {
            floatx4 o = egv[it] * qs[it];
#pragma unroll
            for (int jp = 0; jp <= (it >> 1); ++jp) mma_bf16(o, psl[tri_pair(it, jp)], Uq[2 * jp], Uq[2 * jp + 1]);
#pragma unroll
            for (int e = 0; e < 4; ++e)
                *reinterpret_cast<uint16_t*>(ost + (16 * it + 4 * g + e) * VRB + (16 * wave + r) * 2) =
                    (uint16_t)float_to_bf16_bits(o[e]);
        }
    };

    auto write_out = [&](int c, const char* ost) {
        const int clen = min(64, len - 64 * c);
        bf16_t* ob = a.o + (size_t)(t0 + 64L * c) * v_stride + (size_t)h * a.dv + slice * SLW;
#pragma unroll
        for (int it = 0; it < C::UV; ++it) {
            const int i = tid + NTH * it;
            const int row = i / VPP, pv = i % VPP;
            if (row < clen)
                st16(ob + (size_t)row * v_stride + pv * 8, ld16(ost + row * VRB + pv * 16));
        }
    };

    Pref<DK, NW> pf;
    char* stage0 = lds;
    char* stage1 = lds + C::STAGE;
    char* ost0 = lds + 2 * C::STAGE;
    char* ost1 = ost0 + C::OSB;
    if (nch > 0) { fetch(0, pf); stash(pf, stage0); }
    __syncthreads();
    for (int c = 0; c < nch; ++c) {
        char* cur = (c & 1) ? stage1 : stage0;
        char* nxt = (c & 1) ? stage0 : stage1;
        char* ost = (c & 1) ? ost1 : ost0;
        const bool more = c + 1 < nch;
        if (more && !(a.debug & 1)) fetch(c + 1, pf);                      // in flight while this chunk's products run
        if (!(a.debug & 2)) compute(cur, ost);
        if (more && !(a.debug & 4)) stash(pf, nxt);
        // One barrier per chunk: staged outputs before their write-out; the next chunk's operands
        // before their use; all reads of `cur` before it is overwritten one iteration later; and the
        // write-out of chunk c-1 (finished by every wave before it arrives here) before the staging
        // tile of that parity is written again in chunk c+1.
        __syncthreads();
        write_out(c, ost);
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
    const int n_states = a.n_seq > 0 ? a.n_seq : a.N;
    const int n_chains = n_states * a.H;
    if (n_chains == 0) return hipSuccess;
    const int nsl = a.dv / (16 * waves);
    const dim3 grid((unsigned)(((n_chains + 7) / 8) * 8 * nsl));
    switch (waves) {
        case 1: hipLaunchKernelGGL((scan_bf16_kernel<DK, 1>), grid, dim3(64), 0, st, a); break;
        case 2: hipLaunchKernelGGL((scan_bf16_kernel<DK, 2>), grid, dim3(128), 0, st, a); break;
        default: hipLaunchKernelGGL((scan_bf16_kernel<DK, 4>), grid, dim3(256), 0, st, a); break;
    }
    return hipGetLastError();
}

hipError_t launch_scan_bf16(const ScanArgs<bf16_t>& a, int dk, int waves, hipStream_t st)
{
    if (dk == 64) return launch_dk<64>(a, waves, st);
    return launch_dk<128>(a, waves, st);
}

}  // namespace kla
