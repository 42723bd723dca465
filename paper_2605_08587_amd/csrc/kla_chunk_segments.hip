// Segment-parallel inter-chunk stage for long sequences in small batches (bf16).
//
// The chunk recurrence of eq. (8) is affine in the state: over a run of chunks, S_out = M S_in + N with
// M = prod_c (gamma_C I - K^T D T' D_gamma K)_c (d_k x d_k) and N the state the run produces from S_in = 0
// (App. B writes the same thing token by token as S_i = P_i S_0 + H_i).  A batch of few (sequence, head)
// chains that are thousands of chunks long leaves most of the chip idle in the serial scan, so each sequence
// is cut into G segments of whole chunks and the scan becomes three launches:
//
//   1. scan_maps_bf16_kernel: for every segment but the last of a sequence, M and N at once, by running the
//      recurrence on d_v + d_k columns: the value columns from S = 0 with the real V, the "phi" columns from
//      S = I with V = 0.  No outputs, no Q, no P: only the chain part of a chunk (K S, X, U = T'X, state
//      update), 32 columns per workgroup.
//   2. segment_combine_kernel: S_in(0) = h0, S_in(g+1) = M_g S_in(g) + N_g, in fp32 (G - 1 small products).
//   3. the ordinary scan kernel over all N x G segments at once, each starting from its S_in (the kernel's
//      segmented mode), which also produces the outputs; segment_gather_kernel then copies the last segment's
//      final state to h_T.
//
// Layouts, swizzles, the copy wave and the operand tricks are those of kla_chunk_scan_bf16.hip.
#include "kla_bf16_ops.hpp"
#include "kla_common.hpp"
#include "kla_kernels.hpp"
#include "kla_mma.hpp"

namespace kla {

namespace {

template <int DK>
struct MapCfg {
    static constexpr int NW = 2;                         // compute waves, 16 columns each
    static constexpr int KB = DK / 16, KP = DK / 32;
    static constexpr int SLW = 16 * NW;
    static constexpr int RB = DK * 2, PPR = DK / 8, RPB = 1024 / RB, NKB = 64 / RPB;
    static constexpr int VRW = SLW * 2, VPP = VRW / 16, RPV = 64 / VPP, NVB = 64 / RPV;
    static constexpr int TPB = kTriPairs * 64 * 16, NTB = TPB / 1024;
    static constexpr int OFF_T = 64 * RB, OFF_V = OFF_T + TPB, OFF_EG = OFF_V + 64 * VRW, STAGE = OFF_EG + 512;
    static constexpr int NST = 3;
    static constexpr int LDS = NST * STAGE;
    static constexpr int NDMA_V = NKB + NTB + NVB + 1;   // copy instructions per chunk, value columns
    static constexpr int NDMA_P = NKB + NTB + 1;         // ... phi columns (no V)
    static_assert(LDS <= 160 * 1024 && NDMA_V < 32, "LDS budget; two chunks of copies within the 6-bit vmcnt");
};

}  // namespace

// grid: (map chains rounded up to 8) x (d_v + d_k) / 32 workgroups of 2 compute waves + 1 copy wave.
// Map chain = ((n (G-1) + sg) H + h): segment sg < G-1 of sequence n, head h.
// maps: per map chain [N: DK x dv | M: DK x DK] fp32.
// BREC: the records are those of the backward pass ([T' | M^T | P^T | vectors], see bwd_record_bytes).
template <int DK, bool BREC = false>
__global__ __launch_bounds__(192) void scan_maps_bf16_kernel(ScanArgs<bf16_t> a, float* __restrict__ maps)
{
    typedef MapCfg<DK> C;
    constexpr int NW = C::NW, KB = C::KB, KP = C::KP, SLW = C::SLW, RB = C::RB, PPR = C::PPR, RPB = C::RPB,
                  VRW = C::VRW, VPP = C::VPP, RPV = C::RPV, NST = C::NST;

    __shared__ __attribute__((aligned(1024))) char lds[C::LDS];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int r = lane & 15, g = lane >> 4;

    const int vsl = a.dv / SLW, nsl = (a.dv + DK) / SLW;
    const int n_chains = a.N * (a.seg_G - 1) * a.H;
    const int xcd = blockIdx.x & 7, pidx = blockIdx.x >> 3;
    const int chain = (pidx / nsl) * 8 + xcd, slice = pidx % nsl;
    if (chain >= n_chains) return;
    const int sidx = chain / a.H, h = chain % a.H;
    const int n = sidx / (a.seg_G - 1), sg = sidx % (a.seg_G - 1);
    // every segment but the last of a sequence consists of seg_Lc whole chunks
    const long t0 = (long)n * a.T + (long)sg * a.seg_Lc * 64;
    const int nch = a.seg_Lc;
    const int ch0 = n * a.NT + sg * a.seg_Lc;
    const bool phi = slice >= vsl;                       // workgroup-uniform
    const int col = (phi ? (slice - vsl) : slice) * SLW + 16 * wave + r;   // column of N, or of M

    // state tile kt = 2*kp + b, element e  <->  feature 32*kp + 8*g + 4*b + e
    floatx4 S[KB];
#pragma unroll
    for (int kt = 0; kt < KB; ++kt)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int f = 32 * (kt >> 1) + 8 * g + 4 * (kt & 1) + e;
            S[kt][e] = (phi && f == col) ? 1.f : 0.f;
        }

    const size_t kq_row = (size_t)a.H * DK * 2, v_row = (size_t)a.H * a.dv * 2;     // bytes between tokens
    const char* kbase = reinterpret_cast<const char*>(a.k) + (size_t)t0 * kq_row + (size_t)h * DK * 2;
    const char* vbase = reinterpret_cast<const char*>(a.v) + (size_t)t0 * v_row + ((size_t)h * a.dv + (phi ? 0 : slice) * SLW) * 2;
    constexpr int REC = BREC ? bwd_record_bytes<bf16_t>() : ws_record_bytes<bf16_t>();
    constexpr int VEC = (BREC ? 3 : 2) * C::TPB;         // offset of gamma_i | gamma_C/gamma_i in a record
    const char* tpbase = reinterpret_cast<const char*>(a.wsT) + ((size_t)ch0 * a.H + h) * REC;

    if (wave == NW) {
        // ---- the copy wave ---------------------------------------------------------------------------
        const int lrow = lane / PPR, pcol = lane % PPR;
        constexpr int NGK = 8 / RPB;                    // the swizzle has period 8 rows
        int gk[NGK];
#pragma unroll
        for (int j = 0; j < NGK; ++j)
            gk[j] = lrow * (int)kq_row + ((pcol ^ swz_piece<DK>(RPB * j + lrow)) * 16);
        const int gv = (lane / VPP) * (int)v_row + (lane % VPP) * 16;
        auto issue = [&](int c, char* st) {
            const char* kc = kbase + (size_t)(64 * c) * kq_row;
            const char* tc = tpbase + (size_t)c * a.H * REC;
            static_for<C::NKB>([&](auto i) {
                const int b = i;
                dma16(kc + (size_t)(b * RPB) * kq_row, gk[b % NGK], st + b * 1024);
            });
            static_for<C::NTB>([&](auto i) {
                const int b = i;
                dma16(tc + b * 1024, lane * 16, st + C::OFF_T + b * 1024);
            });
            if (!phi) {
                const char* vc = vbase + (size_t)(64 * c) * v_row;
                static_for<C::NVB>([&](auto i) {
                    const int b = i;
                    dma16(vc + (size_t)(b * RPV) * v_row, gv, st + C::OFF_V + b * 1024);
                });
            }
            if (lane < 32) dma16(tc + VEC, lane * 16, st + C::OFF_EG);              // gamma_i | gamma_C/gamma_i
        };
        auto wait_behind = [&](bool ahead) {             // all but the copies of the newest chunk have landed
            if (!ahead) wait_vmcnt<0>();
            else if (phi) wait_vmcnt<C::NDMA_P>();
            else wait_vmcnt<C::NDMA_V>();
        };
#pragma unroll
        for (int p = 0; p < NST - 1; ++p)
            if (p < nch) issue(p, lds + p * C::STAGE);
        wait_behind(nch > 1);                            // chunk 0 has landed
        __syncthreads();
        int spre = NST - 1;
        for (int c = 0; c < nch; ++c) {
            const bool ahead = c + NST - 1 < nch;
            if (ahead) issue(c + NST - 1, lds + spre * C::STAGE);   // refills the stage chunk c-1 was read from
            wait_behind(ahead);                          // chunk c+1 is complete
            __syncthreads();
            spre = (spre + 1 == NST) ? 0 : spre + 1;
        }
        return;
    }

    // ---- compute waves: the chain part of the chunk recurrence ---------------------------------------
    int oK[KP], oKT[KP];
    const int a4 = r >> 2, c4 = r & 3;
#pragma unroll
    for (int kp = 0; kp < KP; ++kp) {
        oK[kp] = r * RB + (((4 * kp + g) ^ swz_piece<DK>(r)) * 16);
        oKT[kp] = (4 * g + a4) * RB + (((4 * kp + c4) ^ swz_piece<DK>(4 * g + a4)) * 16);
    }
    const int oV = (4 * g + a4) * VRW + (16 * wave + 4 * c4) * 2;

    __syncthreads();                                     // chunk 0 is in stage 0
    int scur = 0;
    for (int c = 0; c < nch; ++c) {
        const char* st = lds + scur * C::STAGE;
        const char* pG = st + C::OFF_EG + 16 * g;
        const float gC = *reinterpret_cast<const float*>(st + C::OFF_EG + 63 * 4);
        u32x2 Sq[KB];
#pragma unroll
        for (int kt = 0; kt < KB; ++kt) { Sq[kt] = to_quad(S[kt]); S[kt] = S[kt] * gC; }

        // K S
        floatx4 ks[4];
#pragma unroll
        for (int it = 0; it < 4; ++it) ks[it] = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int kp = 0; kp < KP; ++kp)
#pragma unroll
            for (int it = 0; it < 4; ++it)
                mma_bf16(ks[it], ld16(st + oK[kp] + 16 * it * RB), Sq[2 * kp], Sq[2 * kp + 1]);

        // X = V - D_gamma K S (V = 0 in the phi columns);  U = T' X
        u32x2 Xq[4];
        floatx4 edv[4];
#pragma unroll
        for (int it = 0; it < 4; ++it) {
            floatx4 vv = {0.f, 0.f, 0.f, 0.f};
            if (!phi) vv = quad_to_f(lds_read_tr(st + C::OFF_V + oV + 16 * it * VRW));
            Xq[it] = to_quad(vv - ld_f4(pG + 64 * it) * ks[it]);
            edv[it] = ld_f4(pG + 256 + 64 * it);
        }
        u32x4 tsl[kTriPairs];
#pragma unroll
        for (int i = 0; i < kTriPairs; ++i) tsl[i] = ld16(st + C::OFF_T + i * 1024 + lane * 16);
        floatx4 U[4];
#pragma unroll
        for (int it = 0; it < 4; ++it) {
            U[it] = floatx4{0.f, 0.f, 0.f, 0.f};
            mma_bf16(U[it], tsl[tri_pair(it, 0)], Xq[0], Xq[1]);
        }
        mma_bf16(U[2], tsl[tri_pair(2, 1)], Xq[2], Xq[3]);
        mma_bf16(U[3], tsl[tri_pair(3, 1)], Xq[2], Xq[3]);
        u32x2 Udq[4];
#pragma unroll
        for (int it = 0; it < 4; ++it) Udq[it] = to_quad(U[it] * edv[it]);

        // S = gamma_C S + K^T (diag(gamma_C/gamma_i) U)
#pragma unroll
        for (int jp = 0; jp < 2; ++jp)
#pragma unroll
            for (int t = 0; t < KB; ++t) {
                const int kp = t >> 1, b = t & 1;
                const char* p = st + oKT[kp] + 32 * jp * RB + 8 * b;
                mma_bf16(S[t], lds_read_tr(p), lds_read_tr(p + 16 * RB), Udq[2 * jp], Udq[2 * jp + 1]);
            }
        __syncthreads();   // chunk c+1's operands before their use; all reads of this stage before its refill
        scur = (scur + 1 == NST) ? 0 : scur + 1;
    }

    float* out = maps + (size_t)chain * DK * (a.dv + DK) + (phi ? (size_t)DK * a.dv : 0);
    const int ld = phi ? DK : a.dv;
#pragma unroll
    for (int kt = 0; kt < KB; ++kt)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int f = 32 * (kt >> 1) + 8 * g + 4 * (kt & 1) + e;
            out[(size_t)f * ld + col] = S[kt][e];
        }
}

// S_in(0) = h0 (or 0), S_in(g+1) = M_g S_in(g) + N_g, in fp32.  The G - 1 steps are serial, so the work of a step
// is spread wide: one workgroup per (sequence, head, 8 state columns), thread t owns row t/2 and 4 of the
// columns, reads its row of M_g with all loads in flight at once, and takes S_in(g) from LDS.
template <int DK>
__global__ __launch_bounds__(2 * DK) void segment_combine_kernel(const float* __restrict__ h0, const float* __restrict__ maps,
                                                                float* __restrict__ seg_state, int H, int dv, int G)
{
    typedef float f4 __attribute__((ext_vector_type(4)));
    __shared__ __attribute__((aligned(16))) f4 Ss[DK][2];
    const int nh = blockIdx.x, c0 = blockIdx.y * 8;      // nh = n H + h
    const int n = nh / H, h = nh % H;
    const int row = threadIdx.x >> 1, half = threadIdx.x & 1;
    const int col = c0 + 4 * half;
    f4 acc = {0.f, 0.f, 0.f, 0.f};
    if (h0) acc = *reinterpret_cast<const f4*>(h0 + ((size_t)nh * DK + row) * dv + col);
    for (int sg = 0; sg < G; ++sg) {
        *reinterpret_cast<f4*>(seg_state + ((size_t)((n * G + sg) * H + h) * DK + row) * dv + col) = acc;
        if (sg + 1 == G) break;
        const float* mp = maps + (size_t)((n * (G - 1) + sg) * H + h) * DK * (dv + DK);
        const f4* Mrow = reinterpret_cast<const f4*>(mp + (size_t)DK * dv + (size_t)row * DK);
        f4 m[DK / 4];
#pragma unroll
        for (int i = 0; i < DK / 4; ++i) m[i] = Mrow[i];
        const f4 nn = *reinterpret_cast<const f4*>(mp + (size_t)row * dv + col);
        Ss[row][half] = acc;
        __syncthreads();
        acc = nn;
#pragma unroll
        for (int i = 0; i < DK / 4; ++i)
#pragma unroll
            for (int kk = 0; kk < 4; ++kk) acc += m[i][kk] * Ss[4 * i + kk][half];
        __syncthreads();                                 // every thread has read Ss before it is overwritten
    }
}

// The backward counterpart: g(s-1) = M_s^T g(s) + b(s) down the segments (see launch_segment_combine_rev).  Same
// decomposition; thread (row, half) reads column `row` of M_s, which consecutive rows read from consecutive addresses.
template <int DK>
__global__ __launch_bounds__(2 * DK) void segment_combine_rev_kernel(const float* __restrict__ maps, const float* __restrict__ bseg,
                                                                    float* __restrict__ gseg, int H, int dv, int G)
{
    typedef float f4 __attribute__((ext_vector_type(4)));
    __shared__ __attribute__((aligned(16))) f4 Gs[DK][2];
    const int nh = blockIdx.x, c0 = blockIdx.y * 8;      // nh = n H + h
    const int n = nh / H, h = nh % H;
    const int row = threadIdx.x >> 1, half = threadIdx.x & 1;
    const int col = c0 + 4 * half;
    auto at = [&](int sg) { return ((size_t)((n * G + sg) * H + h) * DK + row) * dv + col; };
    // g(G-2) = b(G-1): the last segment's sweep already ran with its true incoming gradient
    f4 acc = *reinterpret_cast<const f4*>(bseg + at(G - 1));
    *reinterpret_cast<f4*>(gseg + at(G - 2)) = acc;
    for (int sg = G - 2; sg >= 1; --sg) {                // g(sg-1) = M_sg^T g(sg) + b(sg)
        const float* mp = maps + (size_t)((n * (G - 1) + sg) * H + h) * DK * (dv + DK) + (size_t)DK * dv;   // M of segment sg
        Gs[row][half] = acc;
        __syncthreads();
        acc = *reinterpret_cast<const f4*>(bseg + at(sg));
#pragma unroll 8
        for (int i = 0; i < DK; ++i) acc += mp[(size_t)i * DK + row] * Gs[i][half];
        *reinterpret_cast<f4*>(gseg + at(sg - 1)) = acc;
        __syncthreads();                                 // every thread has read Gs before it is overwritten
    }
}

__global__ void segment_scatter_kernel(const float* __restrict__ d_hT, float* __restrict__ gseg, int H, long per_head,
                                       int G, long total)
{
    const long i = (long)blockIdx.x * 256 + threadIdx.x;       // index into gseg
    if (i >= total) return;
    const long sh = i / per_head, e = i % per_head;            // sh = (n G + sg) H + h
    const long s = sh / H, h = sh % H;
    const long n = s / G, sg = s % G;
    gseg[i] = (sg == G - 1 && d_hT) ? d_hT[(n * H + h) * per_head + e] : 0.f;
}

__global__ void segment_gather_kernel(const float* __restrict__ seg_state, float* __restrict__ hT, int H, long per_head,
                                      int G, int g_last, long total)
{
    const long i = (long)blockIdx.x * 256 + threadIdx.x;
    if (i >= total) return;
    const long nh = i / per_head, e = i % per_head;
    const long n = nh / H, h = nh % H;
    hT[i] = seg_state[((n * G + g_last) * H + h) * per_head + e];
}

hipError_t launch_segment_maps_bf16(const ScanArgs<bf16_t>& a, int dk, float* maps, hipStream_t st)
{
    const int n_chains = a.N * (a.seg_G - 1) * a.H;
    if (n_chains <= 0) return hipSuccess;
    const int nsl = (a.dv + dk) / 32;
    const dim3 grid((unsigned)(((n_chains + 7) / 8) * 8 * nsl));
    if (dk == 64) hipLaunchKernelGGL((scan_maps_bf16_kernel<64>), grid, dim3(192), 0, st, a, maps);
    else          hipLaunchKernelGGL((scan_maps_bf16_kernel<128>), grid, dim3(192), 0, st, a, maps);
    return hipGetLastError();
}

hipError_t launch_segment_maps_bwdrec_bf16(const ScanArgs<bf16_t>& a, int dk, float* maps, hipStream_t st)
{
    const int n_chains = a.N * (a.seg_G - 1) * a.H;
    if (n_chains <= 0) return hipSuccess;
    const int nsl = (a.dv + dk) / 32;
    const dim3 grid((unsigned)(((n_chains + 7) / 8) * 8 * nsl));
    if (dk == 64) hipLaunchKernelGGL((scan_maps_bf16_kernel<64, true>), grid, dim3(192), 0, st, a, maps);
    else          hipLaunchKernelGGL((scan_maps_bf16_kernel<128, true>), grid, dim3(192), 0, st, a, maps);
    return hipGetLastError();
}

hipError_t launch_segment_combine(const float* h0, const float* maps, float* seg_state, int N, int H, int dk, int dv,
                                  int G, hipStream_t st)
{
    const dim3 grid((unsigned)(N * H), (unsigned)(dv / 8));
    if (dk == 64) hipLaunchKernelGGL((segment_combine_kernel<64>), grid, dim3(128), 0, st, h0, maps, seg_state, H, dv, G);
    else          hipLaunchKernelGGL((segment_combine_kernel<128>), grid, dim3(256), 0, st, h0, maps, seg_state, H, dv, G);
    return hipGetLastError();
}

hipError_t launch_segment_combine_rev(const float* maps, const float* bseg, float* gseg, int N, int H, int dk, int dv,
                                      int G, hipStream_t st)
{
    if (G < 2) return hipSuccess;
    const dim3 grid((unsigned)(N * H), (unsigned)(dv / 8));
    if (dk == 64) hipLaunchKernelGGL((segment_combine_rev_kernel<64>), grid, dim3(128), 0, st, maps, bseg, gseg, H, dv, G);
    else          hipLaunchKernelGGL((segment_combine_rev_kernel<128>), grid, dim3(256), 0, st, maps, bseg, gseg, H, dv, G);
    return hipGetLastError();
}

hipError_t launch_segment_scatter(const float* d_hT, float* gseg, int N, int H, int dk, int dv, int G, hipStream_t st)
{
    const long per_head = (long)dk * dv, total = (long)N * G * H * per_head;
    if (total == 0) return hipSuccess;
    hipLaunchKernelGGL(segment_scatter_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, d_hT, gseg, H,
                       per_head, G, total);
    return hipGetLastError();
}

hipError_t launch_segment_gather(const float* seg_state, float* hT, int N, int H, int dk, int dv, int G, int g_last,
                                 hipStream_t st)
{
    const long per_head = (long)dk * dv, total = (long)N * H * per_head;
    hipLaunchKernelGGL(segment_gather_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, seg_state, hT, H,
                       per_head, G, g_last, total);
    return hipGetLastError();
}

}  // namespace kla
