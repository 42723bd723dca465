// C ABI of the library (declared in include/kla.h): argument validation, workspace carving and
// launch sequencing.  No allocation, no state but the per-device address of the static scratch array, nothing read
// from the environment; everything is enqueued on the caller's stream.
#include <math.h>

#include <mutex>

#include "../../include/kla.h"
#include "kla_kernels.hpp"

namespace {

using kla::bf16_t;

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline size_t round256(size_t x) { return (x + 255) & ~(size_t)255; }
inline bool dk_ok(int dk) { return dk == 64 || dk == 128; }
inline bool dv_ok(int dv) { return dv == 64 || dv == 128 || dv == 256; }
inline bool dt_ok(int dt) { return dt == KLA_F32 || dt == KLA_BF16; }
inline size_t elem_bytes(int dt) { return dt == KLA_BF16 ? 2 : 4; }

static_assert(KLA_OPT_NORMALIZE_Q == (int)kla::kOptNormalizeQ && KLA_OPT_GDN_BETA == (int)kla::kOptGdnBeta, "option bits");

// The tuning fields of the `opts` argument (KLA_TUNE_* in include/kla.h), decoded.  Zero everywhere = the library's choice.
struct Tune {
    int scan_waves = 0;      // 1, 2, 4 compute waves per scan workgroup
    int segments = 0;        // 1 = never cut sequences into segments, n = cut into n
    bool generic_scan = false, generic_intra = false, generic_bwd = false, unfused = false, fused = false;
    int decode_slice = 0;    // 32, 64, 128, 256 state columns per decode workgroup
    int decode_nt = -1;      // bit 0: non-temporal state loads, bit 1: non-temporal state stores
};
constexpr unsigned kOptMask = KLA_OPT_NORMALIZE_Q | KLA_OPT_GDN_BETA;
constexpr unsigned kTuneMask = 0x03ffff00u;

bool parse_tune(unsigned opts, Tune* t)
{
    if (opts & ~(kOptMask | kTuneMask)) return false;
    const unsigned w = (opts >> 8) & 3u, sg = (opts >> 10) & 31u, ds = (opts >> 18) & 7u, nt = (opts >> 21) & 7u;
    if (sg > 16 || ds > 4 || nt > 4) return false;
    t->scan_waves = w == 0 ? 0 : (w == 3 ? 4 : (int)w);
    t->segments = (int)sg;
    t->generic_scan = (opts & KLA_TUNE_GENERIC_SCAN) != 0;
    t->generic_intra = (opts & KLA_TUNE_GENERIC_INTRA) != 0;
    t->generic_bwd = (opts & KLA_TUNE_GENERIC_BWD) != 0;
    t->unfused = (opts & KLA_TUNE_UNFUSED) != 0;
    t->fused = (opts & KLA_TUNE_FUSED) != 0;
    if (t->fused && t->unfused) return false;
    t->decode_slice = ds == 0 ? 0 : 16 << ds;
    t->decode_nt = nt == 0 ? -1 : (int)nt - 1;
    return true;
}

struct Plan {
    long n_chunks;       // over all sequences
    int n_states;        // sequences
    size_t off_T, off_P, off_G, off_C, off_M, off_S, total;
    int seg_G, seg_Lc;   // segment-parallel scan: segments per sequence (1 = off) and chunks per segment
    int waves;           // compute waves per scan workgroup (of the unsegmented scan)
    bool fused;          // bf16 only: one kernel, no intra-chunk stage, nothing in the workspace
    Tune tune;
};

// Segments per sequence for the scan stage.  A small fixed-length bf16 batch of long sequences (at most 128
// sixteen-column chains, at least 64 chunks) is cut so that about 256 workgroups of two chains run (measured
// on one 65K-token sequence of 8 heads: 1.24 ms unsegmented, 0.70 ms with 4 segments, 0.57 ms with 8, 0.71 ms
// with 16); the tuning field KLA_TUNE_SCAN_SEGMENTS(n) forces n (1 = never).  Returns the number of non-empty segments and sets the chunks per segment.
int plan_segments(int N, int NT, int H, int dv, int dt, int n_seq, const Tune& tune, int* Lc)
{
    *Lc = NT;
    if (dt != KLA_BF16 || n_seq > 0 || N <= 0 || NT < 2) return 1;
    if (tune.generic_scan) return 1;                 // generic kernels: never
    const long groups = (long)N * H * (dv / 16);
    int want = 1;
    if (tune.segments >= 1) want = tune.segments;
    else if (groups <= 128 && NT >= 64) {
        // up to 512 sixteen-column chains (256 workgroups of two compute waves), segments of at least 16 chunks
        want = 1;
        while (want < 16 && (long)want * 2 * groups <= 512 && NT / (want * 2) >= 16) want *= 2;
    }
    if (want > NT) want = NT;
    if (want <= 1) return 1;
    const int lc = (NT + want - 1) / want;
    const int G = (NT + lc - 1) / lc;
    if (G <= 1) return 1;
    *Lc = lc;
    return G;
}

int scan_waves(int n_chains, int dv, int dt, const Tune& tune);

// Validates the size arguments shared by the chunk entry points and lays out the workspace.
int make_plan(int N, int T, int H, int dk, int dv, int chunk, int dt, const int32_t* cu_host, int n_seq, unsigned opts, Plan* p)
{
    if (!parse_tune(opts, &p->tune)) return KLA_ERR_SHAPE;
    if (!dt_ok(dt)) return KLA_ERR_DTYPE;
    if (N < 0 || T < 0 || H <= 0 || n_seq < 0 || !dk_ok(dk) || !dv_ok(dv) || chunk != 64) return KLA_ERR_SHAPE;
    long n_chunks = 0;
    if (n_seq > 0) {
        if (N != 1) return KLA_ERR_SHAPE;
        if (!cu_host) return KLA_ERR_NULL;
        if (cu_host[0] != 0) return KLA_ERR_SEQLENS;
        for (int s = 0; s < n_seq; ++s) {
            if (cu_host[s + 1] < cu_host[s]) return KLA_ERR_SEQLENS;
            n_chunks += (cu_host[s + 1] - cu_host[s] + 63) / 64;
        }
        if (cu_host[n_seq] != T) return KLA_ERR_SEQLENS;
        p->n_states = n_seq;
    } else {
        if (cu_host) return KLA_ERR_SHAPE;
        n_chunks = (long)N * ((T + 63) / 64);
        p->n_states = N;
    }
    if (n_chunks * H > 0x7fffffffL || (long)p->n_states * H * (dv / 16) > 0x7fffffffL) return KLA_ERR_SHAPE;
    p->n_chunks = n_chunks;
    // per chunk-head one record [T' | P], each 6 tile-pairs x 64 slots of 8 elements
    const size_t half = (size_t)384 * 8 * elem_bytes(dt);
    p->off_T = 0;
    p->off_P = half;
    p->off_G = round256((size_t)n_chunks * H * (2 * half + 768));   // + three vectors of 64 fp32 (see kla_mma.hpp)
    p->off_C = round256(p->off_G + (size_t)n_chunks * H * 128 * sizeof(float));      // g and 1/||q||
    p->off_M = round256(p->off_C + (size_t)(n_seq + 1) * sizeof(int32_t));
    p->seg_G = plan_segments(N, (T + 63) / 64, H, dv, dt, n_seq, p->tune, &p->seg_Lc);
    // per (sequence, head): G - 1 maps [N | M] and G incoming states, fp32
    const size_t maps = p->seg_G > 1 ? (size_t)N * (p->seg_G - 1) * H * dk * (dv + dk) * sizeof(float) : 0;
    const size_t states = p->seg_G > 1 ? (size_t)N * p->seg_G * H * dk * dv * sizeof(float) : 0;
    p->off_S = round256(p->off_M + maps);
    p->total = round256(p->off_S + states);
    p->waves = scan_waves(p->n_states * H, dv, dt, p->tune);
    // bf16, a plain scan of two compute waves per workgroup (512 .. 2047 sixteen-column chains, e.g. 8 x 8 heads of 128
    // columns): the fused kernel, which keeps the per-chunk objects on chip and needs nothing of the workspace (a token
    // size is still reported and asked for).  Measured: 0.116 against 0.124 ms on 8 x 8 heads x 4096 tokens; with one
    // compute wave per workgroup (few chains) its helper waves redo the per-chunk work once per 16 columns and the
    // two-kernel form wins (1.38 against 1.83 ms on one 65K sequence, unsegmented), as it does for wide value heads
    // run with two waves (0.55 against 0.64 ms on 16 packed sequences, 16 heads, d_v = 256).  KLA_TUNE_FUSED forces it
    // wherever it can run (one or two compute waves, no segments).
    p->fused = dt == KLA_BF16 && p->seg_G <= 1 && !p->tune.unfused && !p->tune.generic_scan && !p->tune.generic_intra &&
               (p->tune.fused ? p->waves <= 2 : (p->waves == 2 && dv <= 128));
    if (p->fused) p->total = 256;
    return KLA_OK;
}

int scan_waves(int n_chains, int dv, int dt, const Tune& tune)
{
    int w;
    if (tune.scan_waves) w = tune.scan_waves;        // tuning field: 1, 2 or 4 waves (16 state columns each) per workgroup
    else {
        // enough workgroups to cover the 256 CUs, else the widest slice that still gives >= 2 waves of loaders
        // workgroups for w waves: chains8 * dv / (16 w).  Wide slices halve the operand re-reads but need
        // enough workgroups to cover the 256 CUs; a lone long sequence is latency-bound and runs best narrow.
        const long chains8 = ((long)n_chains + 7) / 8 * 8;
        const long wg1 = chains8 * (dv / 16);
        w = (wg1 / 4 >= 512) ? 4 : ((wg1 / 2 >= 192) ? 2 : 1);
    }
    if (dt == KLA_F32 && w > 2) w = 2;            // fp32 operands take twice the LDS
    while (16 * w > dv) w >>= 1;
    return w;
}

template <typename E>
int chunk_fwd_impl(const void* q, const void* k, const void* v, const float* log_alpha, const float* eta, float eps,
                   const float* h0, void* o, float* hT, const int32_t* cu_dev, int n_seq, int N, int T, int H, int dk,
                   int dv, const Plan& pl, char* ws, int stages, float* Tb_out, float* P_out, float* g_out,
                   hipStream_t st, unsigned opts)
{
    E* wsT = reinterpret_cast<E*>(ws + pl.off_T);
    E* wsP = reinterpret_cast<E*>(ws + pl.off_P);
    float* wsG = reinterpret_cast<float*>(ws + pl.off_G);
    int* chunk_off = reinterpret_cast<int*>(ws + pl.off_C);
    const int NT = (T + 63) / 64;
    const bool intra = (stages & 1) != 0, scan = (stages & 2) != 0, unpack = (stages & 4) != 0;

    kla::IntraArgs<E> ia;
    ia.q = static_cast<const E*>(q); ia.k = static_cast<const E*>(k);
    ia.log_alpha = log_alpha; ia.eta = eta; ia.eps = eps;
    ia.cu_seqlens = n_seq > 0 ? cu_dev : nullptr; ia.chunk_off = chunk_off; ia.n_seq = n_seq;
    ia.T = T; ia.NT = NT; ia.H = H;
    ia.wsT = wsT; ia.wsP = wsP; ia.wsG = wsG; ia.opts = opts;   // option bits only (the callers strip the tuning fields)
    if constexpr (sizeof(E) == 2) {
        if (stages == 3 && pl.fused) {
            kla::ScanArgs<E> fa;
            fa.q = static_cast<const E*>(q); fa.k = static_cast<const E*>(k); fa.v = static_cast<const E*>(v);
            fa.h0 = h0; fa.o = static_cast<E*>(o); fa.hT = hT;
            fa.cu_seqlens = n_seq > 0 ? cu_dev : nullptr; fa.chunk_off = nullptr; fa.n_seq = n_seq;
            fa.N = N; fa.T = T; fa.NT = NT; fa.H = H; fa.dv = dv;
            fa.wsT = nullptr; fa.wsP = nullptr; fa.wsG = nullptr; fa.opts = opts;
            fa.seg_G = 0; fa.seg_Lc = 0; fa.kt_src = nullptr; fa.gc_vec = nullptr;
            fa.log_alpha = log_alpha; fa.eta = eta; fa.eps = eps;
            return kla::launch_scan_fused_bf16(fa, dk, pl.waves, st) == hipSuccess ? KLA_OK : KLA_ERR_HIP;
        }
    }
    if (intra && n_seq > 0 && kla::launch_chunk_offsets(cu_dev, n_seq, chunk_off, st) != hipSuccess) return KLA_ERR_HIP;
    if (intra) {
        bool done = false;
        if constexpr (sizeof(E) == 2) {
            if (!pl.tune.generic_intra) {                // else the element-type-generic kernel (A/B testing)
                if (kla::launch_intra_bf16(ia, dk, (int)pl.n_chunks, st) != hipSuccess) return KLA_ERR_HIP;
                done = true;
            }
        }
        if (!done && kla::launch_intra<E>(ia, dk, (int)pl.n_chunks, st) != hipSuccess) return KLA_ERR_HIP;
    }
    if (unpack && kla::launch_unpack<E>(wsT, wsP, wsG, Tb_out, P_out, g_out, pl.n_chunks * H, st) != hipSuccess)
        return KLA_ERR_HIP;
    if (!scan) return KLA_OK;
    kla::ScanArgs<E> sa;
    sa.q = static_cast<const E*>(q); sa.k = static_cast<const E*>(k); sa.v = static_cast<const E*>(v);
    sa.h0 = h0; sa.o = static_cast<E*>(o); sa.hT = hT;
    sa.cu_seqlens = ia.cu_seqlens; sa.chunk_off = chunk_off; sa.n_seq = n_seq;
    sa.N = N; sa.T = T; sa.NT = NT; sa.H = H; sa.dv = dv;
    sa.wsT = wsT; sa.wsP = wsP; sa.wsG = wsG; sa.opts = opts;
    sa.seg_G = 0; sa.seg_Lc = 0; sa.kt_src = nullptr; sa.gc_vec = nullptr;
    sa.log_alpha = log_alpha; sa.eta = eta; sa.eps = eps;
    if constexpr (sizeof(E) == 2) {
        if (pl.seg_G > 1) {
            // segment-parallel scan: maps of all segments but the last, their prefix composition, then every
            // segment at once from its incoming state (see kla_chunk_segments.hip)
            float* maps = reinterpret_cast<float*>(ws + pl.off_M);
            float* seg_state = reinterpret_cast<float*>(ws + pl.off_S);
            sa.seg_G = pl.seg_G; sa.seg_Lc = pl.seg_Lc;
            if (kla::launch_segment_maps_bf16(sa, dk, maps, st) != hipSuccess) return KLA_ERR_HIP;
            if (kla::launch_segment_combine(h0, maps, seg_state, N, H, dk, dv, pl.seg_G, st) != hipSuccess) return KLA_ERR_HIP;
            sa.h0 = seg_state; sa.hT = seg_state;
            const int wseg = scan_waves(pl.n_states * pl.seg_G * H, dv, KLA_BF16, pl.tune);
            if (kla::launch_scan_bf16(sa, dk, wseg, st) != hipSuccess) return KLA_ERR_HIP;
            if (hT && kla::launch_segment_gather(seg_state, hT, N, H, dk, dv, pl.seg_G, pl.seg_G - 1, st) != hipSuccess)
                return KLA_ERR_HIP;
            return KLA_OK;
        }
    }
    const int waves = pl.waves;
    if constexpr (sizeof(E) == 2) {
        if (!pl.tune.generic_scan)                       // else the element-type-generic kernel (A/B testing)
            return kla::launch_scan_bf16(sa, dk, waves, st) == hipSuccess ? KLA_OK : KLA_ERR_HIP;
    }
    if (kla::launch_scan<E>(sa, dk, waves, st) != hipSuccess) return KLA_ERR_HIP;
    return KLA_OK;
}

// ---- backward pass ---------------------------------------------------------------------------------
struct BwdPlan {
    Plan base;
    size_t off_rec, off_C, off_S, off_dS, off_X, off_U, off_Y, total;
    // segment-parallel sweeps (base.seg_G > 1): maps of the segments, states entering them, and for the reverse
    // direction the state gradients leaving them and what each segment's pre-pass returns; all fp32
    size_t off_maps, off_segS, off_segG, off_segB;
};

int make_bwd_plan(int N, int T, int H, int dk, int dv, int chunk, int dt, const int32_t* cu_host, int n_seq, unsigned opts,
                  BwdPlan* p)
{
    const int rc = make_plan(N, T, H, dk, dv, chunk, dt, cu_host, n_seq, opts, &p->base);
    if (rc != KLA_OK) return rc;
    const size_t half = (size_t)384 * 8 * elem_bytes(dt);
    const size_t ch = (size_t)p->base.n_chunks * H;
    const size_t states = ch * dk * dv * elem_bytes(dt);          // checkpoints are kept in the element type
    const size_t rows = (size_t)N * T * H * dv * elem_bytes(dt);
    p->off_rec = 0;                                              // [T' | M^T | P^T | five vectors] per chunk-head
    p->off_C = round256(ch * (3 * half + 1280));
    p->off_S = round256(p->off_C + (size_t)(n_seq + 1) * sizeof(int32_t));
    p->off_dS = round256(p->off_S + states);
    // the bf16 kernels do not keep U (their assembly forms it again from T' and X); the generic ones do
    const size_t rows_u = (dt == KLA_BF16 && !p->base.tune.generic_bwd) ? 0 : rows;
    p->off_X = round256(p->off_dS + states);
    p->off_U = round256(p->off_X + rows);
    p->off_Y = round256(p->off_U + rows_u);
    const int G = p->base.seg_G;
    const size_t maps = G > 1 ? (size_t)N * (G - 1) * H * dk * (dv + dk) * sizeof(float) : 0;
    const size_t segst = G > 1 ? (size_t)N * G * H * dk * dv * sizeof(float) : 0;
    p->off_maps = round256(p->off_Y + rows);
    p->off_segS = round256(p->off_maps + maps);
    p->off_segG = round256(p->off_segS + segst);
    p->off_segB = round256(p->off_segG + segst);
    p->total = round256(p->off_segB + segst);
    return KLA_OK;
}

template <typename E>
int chunk_bwd_impl(const void* q, const void* k, const void* v, const float* log_alpha, const float* eta, float eps,
                   const float* h0, const void* d_o, const float* d_hT, void* dq, void* dk_, void* dv_,
                   float* dlog_alpha, float* deta, float* dh0, const int32_t* cu_dev, int n_seq, int N, int T, int H,
                   int dk, int dv, const BwdPlan& pl, char* ws, hipStream_t st, unsigned opts)
{
    int* chunk_off = reinterpret_cast<int*>(ws + pl.off_C);
    const int NT = (T + 63) / 64;
    if (n_seq > 0 && kla::launch_chunk_offsets(cu_dev, n_seq, chunk_off, st) != hipSuccess) return KLA_ERR_HIP;

    kla::IntraArgs<E> ia;
    ia.q = static_cast<const E*>(q); ia.k = static_cast<const E*>(k);
    ia.log_alpha = log_alpha; ia.eta = eta; ia.eps = eps;
    ia.cu_seqlens = n_seq > 0 ? cu_dev : nullptr; ia.chunk_off = chunk_off; ia.n_seq = n_seq;
    ia.T = T; ia.NT = NT; ia.H = H;
    ia.wsT = reinterpret_cast<E*>(ws + pl.off_rec); ia.wsP = nullptr; ia.wsG = nullptr; ia.opts = opts;
    bool fast = false;                                // bf16: the specialised kernels, unless the generic ones are asked for (A/B testing)
    if constexpr (sizeof(E) == 2) fast = !pl.base.tune.generic_bwd;
    if constexpr (sizeof(E) == 2) {
        if (fast && kla::launch_intra_bwd_bf16(ia, dk, (int)pl.base.n_chunks, st) != hipSuccess) return KLA_ERR_HIP;
    }
    if (!fast && kla::launch_intra_bwd<E>(ia, dk, (int)pl.base.n_chunks, st) != hipSuccess) return KLA_ERR_HIP;

    kla::BwdArgs<E> ba;
    ba.q = ia.q; ba.k = ia.k; ba.v = static_cast<const E*>(v);
    ba.log_alpha = log_alpha; ba.eta = eta; ba.eps = eps;
    ba.h0 = h0; ba.d_o = static_cast<const E*>(d_o); ba.d_hT = d_hT;
    ba.dq = static_cast<E*>(dq); ba.dk = static_cast<E*>(dk_); ba.dv = static_cast<E*>(dv_);
    ba.dlog_alpha = dlog_alpha; ba.deta = deta; ba.dh0 = dh0;
    ba.cu_seqlens = ia.cu_seqlens; ba.chunk_off = chunk_off; ba.n_seq = n_seq;
    ba.N = N; ba.T = T; ba.NT = NT; ba.H = H; ba.dv_dim = dv;
    ba.rec = ws + pl.off_rec;
    ba.s_chk = reinterpret_cast<E*>(ws + pl.off_S); ba.ds_chk = reinterpret_cast<E*>(ws + pl.off_dS);
    ba.X = reinterpret_cast<E*>(ws + pl.off_X); ba.U = reinterpret_cast<E*>(ws + pl.off_U);
    ba.Y = reinterpret_cast<E*>(ws + pl.off_Y);
    ba.opts = opts;
    ba.seg_G = 0; ba.seg_Lc = 0;
    if constexpr (sizeof(E) == 2) {
        if (fast && pl.base.seg_G > 1) {
            // Segment-parallel sweeps for a few long sequences (see kla_chunk_segments.hip).  Forward: maps of all
            // segments but the last, their composition, then every segment at once from its incoming state.  Reverse:
            // the recursion dS = A dS' + b of a segment is affine with A the transpose of the forward map, so a
            // pre-pass that stores nothing gives every b (the last segment runs with its true d_hT), the composition
            // runs down the segments, and the real sweep starts every segment from its incoming gradient.
            const int G = pl.base.seg_G;
            float* maps = reinterpret_cast<float*>(ws + pl.off_maps);
            float* segS = reinterpret_cast<float*>(ws + pl.off_segS);
            float* segG = reinterpret_cast<float*>(ws + pl.off_segG);
            float* segB = reinterpret_cast<float*>(ws + pl.off_segB);
            kla::ScanArgs<E> sa;
            sa.q = ba.q; sa.k = ba.k; sa.v = ba.v; sa.h0 = nullptr; sa.o = nullptr; sa.hT = nullptr;
            sa.cu_seqlens = nullptr; sa.chunk_off = chunk_off; sa.n_seq = 0;
            sa.N = N; sa.T = T; sa.NT = NT; sa.H = H; sa.dv = dv;
            sa.wsT = reinterpret_cast<const E*>(ws + pl.off_rec); sa.wsP = nullptr; sa.wsG = nullptr; sa.opts = 0u;
            sa.seg_G = G; sa.seg_Lc = pl.base.seg_Lc; sa.kt_src = nullptr; sa.gc_vec = nullptr;
            if (kla::launch_segment_maps_bwdrec_bf16(sa, dk, maps, st) != hipSuccess) return KLA_ERR_HIP;
            if (kla::launch_segment_combine(h0, maps, segS, N, H, dk, dv, G, st) != hipSuccess) return KLA_ERR_HIP;
            if (kla::launch_segment_scatter(d_hT, segG, N, H, dk, dv, G, st) != hipSuccess) return KLA_ERR_HIP;
            ba.seg_G = G; ba.seg_Lc = pl.base.seg_Lc;
            const long sc8 = ((long)N * G * H + 7) / 8 * 8;
            const int wseg = (sc8 * (dv / 32) >= 192) ? 2 : 1;
            ba.h0 = segS;
            if (kla::launch_bwd_states_bf16(ba, dk, wseg, st) != hipSuccess) return KLA_ERR_HIP;
            ba.d_hT = segG; ba.dh0 = segB; ba.opts = opts | kla::kOptNoStore;
            if (kla::launch_bwd_scan_bf16(ba, dk, wseg, st) != hipSuccess) return KLA_ERR_HIP;          // pre-pass: b per segment
            if (kla::launch_segment_combine_rev(maps, segB, segG, N, H, dk, dv, G, st) != hipSuccess) return KLA_ERR_HIP;
            ba.opts = opts;
            if (kla::launch_bwd_scan_bf16(ba, dk, wseg, st) != hipSuccess) return KLA_ERR_HIP;          // the real sweep
            if (dh0 && kla::launch_segment_gather(segB, dh0, N, H, dk, dv, G, 0, st) != hipSuccess) return KLA_ERR_HIP;
            ba.seg_G = 0; ba.seg_Lc = 0; ba.h0 = h0; ba.d_hT = d_hT; ba.dh0 = dh0;
            return kla::launch_bwd_assemble_bf16(ba, dk, pl.base.n_chunks, st) == hipSuccess ? KLA_OK : KLA_ERR_HIP;
        }
    }
    // two waves (32 state columns) per workgroup once that still gives a workgroup per CU
    const long chains8 = ((long)pl.base.n_states * H + 7) / 8 * 8;
    const int waves = (chains8 * (dv / 32) >= 192) ? 2 : 1;
    if constexpr (sizeof(E) == 2) {
        if (fast) {
            if (kla::launch_bwd_states_bf16(ba, dk, waves, st) != hipSuccess) return KLA_ERR_HIP;
            if (kla::launch_bwd_scan_bf16(ba, dk, waves, st) != hipSuccess) return KLA_ERR_HIP;
            return kla::launch_bwd_assemble_bf16(ba, dk, pl.base.n_chunks, st) == hipSuccess ? KLA_OK : KLA_ERR_HIP;
        }
    }
    if (kla::launch_bwd_states<E>(ba, dk, waves, st) != hipSuccess) return KLA_ERR_HIP;
    if (kla::launch_bwd_scan<E>(ba, dk, waves, st) != hipSuccess) return KLA_ERR_HIP;
    if (kla::launch_bwd_assemble<E>(ba, dk, pl.base.n_chunks, st) != hipSuccess) return KLA_ERR_HIP;
    return KLA_OK;
}

// ---- diagonal gating ----------------------------------------------------------------------------------
struct DiagPlan {
    Plan base;
    size_t off_kp, off_qp, off_kt, off_gc, total;
};

int make_diag_plan(int N, int T, int H, int dk, int dv, int chunk, int dt, const int32_t* cu_host, int n_seq, unsigned opts,
                   DiagPlan* p)
{
    // the layout of the two-kernel forward (the fused kernel has no diagonal-gating variant), no segments
    const int rc = make_plan(N, T, H, dk, dv, chunk, dt, cu_host, n_seq, (opts & ~(31u << 10) & ~KLA_TUNE_FUSED) | KLA_TUNE_UNFUSED | KLA_TUNE_SCAN_SEGMENTS(1), &p->base);
    if (rc != KLA_OK) return rc;
    const size_t rows = (size_t)N * T * H * dk * elem_bytes(dt);
    // The three operand arrays are read row by row at the same time.  Their sizes are large powers of two for the usual
    // shapes, so without the 256-byte steps below the rows of one token would sit in the same memory channel in all
    // three (measured: the scan of the config-2 shape takes 13 us longer).
    p->off_kp = round256(p->base.off_M);             // the forward plan up to its chunk offsets; no segment maps here
    p->off_qp = round256(p->off_kp + rows) + 256;
    p->off_kt = round256(p->off_qp + rows) + 256;
    p->off_gc = round256(p->off_kt + rows) + 256;
    p->total = round256(p->off_gc + (size_t)p->base.n_chunks * H * dk * sizeof(float));
    return KLA_OK;
}

template <typename E>
int chunk_fwd_diag_impl(const void* q, const void* k, const void* v, const float* log_alpha, const float* eta, float eps,
                        const float* h0, void* o, float* hT, const int32_t* cu_dev, int n_seq, int N, int T, int H,
                        int dk, int dv, const DiagPlan& pl, char* ws, hipStream_t st, unsigned opts)
{
    int* chunk_off = reinterpret_cast<int*>(ws + pl.base.off_C);
    const int NT = (T + 63) / 64;
    if (n_seq > 0 && kla::launch_chunk_offsets(cu_dev, n_seq, chunk_off, st) != hipSuccess) return KLA_ERR_HIP;
    kla::IntraDiagArgs<E> ia;
    ia.q = static_cast<const E*>(q); ia.k = static_cast<const E*>(k);
    ia.log_alpha = log_alpha; ia.eta = eta; ia.eps = eps;
    ia.cu_seqlens = n_seq > 0 ? cu_dev : nullptr; ia.chunk_off = chunk_off; ia.n_seq = n_seq;
    ia.T = T; ia.NT = NT; ia.H = H;
    ia.wsT = reinterpret_cast<E*>(ws + pl.base.off_T); ia.wsG = reinterpret_cast<float*>(ws + pl.base.off_G);
    ia.kplus = reinterpret_cast<E*>(ws + pl.off_kp); ia.qplus = reinterpret_cast<E*>(ws + pl.off_qp);
    ia.ktilde = reinterpret_cast<E*>(ws + pl.off_kt); ia.gc = reinterpret_cast<float*>(ws + pl.off_gc);
    ia.opts = opts;
    if (kla::launch_intra_diag<E>(ia, dk, (int)pl.base.n_chunks, st) != hipSuccess) return KLA_ERR_HIP;

    kla::ScanArgs<E> sa;
    sa.q = ia.qplus; sa.k = ia.kplus; sa.v = static_cast<const E*>(v);
    sa.h0 = h0; sa.o = static_cast<E*>(o); sa.hT = hT;
    sa.cu_seqlens = ia.cu_seqlens; sa.chunk_off = chunk_off; sa.n_seq = n_seq;
    sa.N = N; sa.T = T; sa.NT = NT; sa.H = H; sa.dv = dv;
    sa.wsT = ia.wsT; sa.wsP = reinterpret_cast<E*>(ws + pl.base.off_P); sa.wsG = ia.wsG; sa.opts = 0u;
    sa.seg_G = 0; sa.seg_Lc = 0; sa.kt_src = ia.ktilde; sa.gc_vec = ia.gc;
    const long chains8 = ((long)pl.base.n_states * H + 7) / 8 * 8;
    const int waves = (chains8 * (dv / 32) >= 192) ? 2 : 1;
    if constexpr (sizeof(E) == 2) {
        if (!pl.base.tune.generic_scan)                  // else the element-type-generic kernel (A/B testing)
            return kla::launch_scan_bf16_diag(sa, dk, waves, st) == hipSuccess ? KLA_OK : KLA_ERR_HIP;
    }
    return kla::launch_scan_diag<E>(sa, dk, waves, st) == hipSuccess ? KLA_OK : KLA_ERR_HIP;
}

// ---- scratch of the entry point that allocates nothing (kla_chunk_fwd_static) --------------------------
// A file-scope device array: every GPU the library runs on holds its own copy at its own address until the
// process ends.  In host code the array's name is only a handle for hipGetSymbolAddress; the address that
// kernels receive is looked up once per device, with that device current, and kept.
constexpr size_t kStaticScratchBytes = (size_t)KLA_STATIC_SCRATCH_BYTES;
constexpr int kMaxDevices = 64;
__device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
std::mutex scratch_mutex;
void* scratch_ptr[kMaxDevices];        // device address of `scratch` per device ordinal, NULL until looked up

// Device address of this device's copy of `scratch` (first call on a device: one symbol lookup), or NULL.
void* static_scratch()
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
    std::lock_guard<std::mutex> lock(scratch_mutex);
    if (!scratch_ptr[dev]) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess) { (void)hipGetLastError(); return nullptr; }
        scratch_ptr[dev] = p;
    }
    return scratch_ptr[dev];
}

}  // namespace

extern "C" {

const char* kla_status_string(int code)
{
    switch (code) {
        case KLA_OK: return "KLA_OK";
        case KLA_ERR_NULL: return "KLA_ERR_NULL: a required pointer is NULL";
        case KLA_ERR_SHAPE: return "KLA_ERR_SHAPE: unsupported or inconsistent sizes";
        case KLA_ERR_DTYPE: return "KLA_ERR_DTYPE: unknown element type";
        case KLA_ERR_ALIGN: return "KLA_ERR_ALIGN: pointer not 16-byte aligned";
        case KLA_ERR_WORKSPACE: return "KLA_ERR_WORKSPACE: workspace missing, misaligned or too small";
        case KLA_ERR_SEQLENS: return "KLA_ERR_SEQLENS: bad cu_seqlens";
        case KLA_ERR_HIP: return "KLA_ERR_HIP: kernel launch failed";
        default: return "unknown kla status";
    }
}

size_t kla_chunk_fwd_workspace_bytes(int N, int T, int H, int dk, int dv, int chunk, kla_dtype dt,
                                     const int32_t* cu_seqlens_host, int n_seq)
{
    return kla_chunk_fwd_workspace_bytes_opts(N, T, H, dk, dv, chunk, dt, cu_seqlens_host, n_seq, 0u);
}

size_t kla_chunk_fwd_workspace_bytes_opts(int N, int T, int H, int dk, int dv, int chunk, kla_dtype dt,
                                          const int32_t* cu_seqlens_host, int n_seq, unsigned opts)
{
    Plan pl;
    if (make_plan(N, T, H, dk, dv, chunk, (int)dt, cu_seqlens_host, n_seq, opts, &pl) != KLA_OK) return 0;
    return pl.total;
}

// Everything kla_chunk_fwd checks except its workspace; fills the plan.
static int chunk_fwd_validate(const void* q, const void* k, const void* v, const float* log_alpha, const float* eta,
                              float eps, const float* h0, void* o, float* hT, const int32_t* cu_seqlens_dev,
                              const int32_t* cu_seqlens_host, int n_seq, int N, int T, int H, int dk, int dv, int chunk,
                              kla_dtype dt, unsigned opts, Plan* pl)
{
    const int rc = make_plan(N, T, H, dk, dv, chunk, (int)dt, cu_seqlens_host, n_seq, opts, pl);
    if (rc != KLA_OK) return rc;
    if (!(eps >= 0.0f) || isinf(eps)) return KLA_ERR_SHAPE;
    if (n_seq > 0 && !cu_seqlens_dev) return KLA_ERR_NULL;
    if (n_seq == 0 && cu_seqlens_dev) return KLA_ERR_SHAPE;
    const bool any_tokens = (long)N * T > 0;
    if (any_tokens && (!q || !k || !v || !log_alpha || !eta || !o)) return KLA_ERR_NULL;
    if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(o) || !aligned16(h0) || !aligned16(hT) ||
        (reinterpret_cast<uintptr_t>(log_alpha) & 3u) || (reinterpret_cast<uintptr_t>(eta) & 3u))
        return KLA_ERR_ALIGN;
    return KLA_OK;
}

static int chunk_fwd_launch(const void* q, const void* k, const void* v, const float* log_alpha, const float* eta,
                            float eps, const float* h0, void* o, float* hT, const int32_t* cu_seqlens_dev, int n_seq,
                            int N, int T, int H, int dk, int dv, kla_dtype dt, const Plan& pl, void* workspace,
                            void* hip_stream, int stages, unsigned opts)
{
    if (pl.n_states == 0) return KLA_OK;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    char* ws = static_cast<char*>(workspace);
    opts &= kOptMask;                                    // the tuning fields live on in pl.tune
    if (dt == KLA_BF16)
        return chunk_fwd_impl<bf16_t>(q, k, v, log_alpha, eta, eps, h0, o, hT, cu_seqlens_dev, n_seq, N, T, H, dk, dv,
                                      pl, ws, stages, nullptr, nullptr, nullptr, st, opts);
    return chunk_fwd_impl<float>(q, k, v, log_alpha, eta, eps, h0, o, hT, cu_seqlens_dev, n_seq, N, T, H, dk, dv, pl, ws,
                                 stages, nullptr, nullptr, nullptr, st, opts);
}

static int chunk_fwd_checked(const void* q, const void* k, const void* v, const float* log_alpha, const float* eta,
                             float eps, const float* h0, void* o, float* hT, const int32_t* cu_seqlens_dev,
                             const int32_t* cu_seqlens_host, int n_seq, int N, int T, int H, int dk, int dv, int chunk,
                             kla_dtype dt, void* workspace, size_t workspace_bytes, void* hip_stream, int stages,
                             unsigned opts)
{
    Plan pl;
    const int rc = chunk_fwd_validate(q, k, v, log_alpha, eta, eps, h0, o, hT, cu_seqlens_dev, cu_seqlens_host, n_seq, N,
                                      T, H, dk, dv, chunk, dt, opts, &pl);
    if (rc != KLA_OK) return rc;
    if (!workspace) return KLA_ERR_WORKSPACE;
    if ((reinterpret_cast<uintptr_t>(workspace) & 255u) != 0 || workspace_bytes < pl.total) return KLA_ERR_WORKSPACE;
    return chunk_fwd_launch(q, k, v, log_alpha, eta, eps, h0, o, hT, cu_seqlens_dev, n_seq, N, T, H, dk, dv, dt, pl,
                            workspace, hip_stream, stages, opts);
}

int kla_chunk_fwd(const void* q, const void* k, const void* v, const float* log_alpha, const float* eta, float eps,
                  const float* h0, void* o, float* hT, const int32_t* cu_seqlens_dev, const int32_t* cu_seqlens_host,
                  int n_seq, int N, int T, int H, int dk, int dv, int chunk, kla_dtype dt, void* workspace,
                  size_t workspace_bytes, void* hip_stream)
{
    return chunk_fwd_checked(q, k, v, log_alpha, eta, eps, h0, o, hT, cu_seqlens_dev, cu_seqlens_host, n_seq, N, T, H,
                             dk, dv, chunk, dt, workspace, workspace_bytes, hip_stream, 3, 0u);
}

int kla_chunk_fwd_opts(const void* q, const void* k, const void* v, const float* log_alpha, const float* eta, float eps,
                       const float* h0, void* o, float* hT, const int32_t* cu_seqlens_dev,
                       const int32_t* cu_seqlens_host, int n_seq, int N, int T, int H, int dk, int dv, int chunk,
                       kla_dtype dt, void* workspace, size_t workspace_bytes, void* hip_stream, unsigned opts)
{
    return chunk_fwd_checked(q, k, v, log_alpha, eta, eps, h0, o, hT, cu_seqlens_dev, cu_seqlens_host, n_seq, N, T, H,
                             dk, dv, chunk, dt, workspace, workspace_bytes, hip_stream, 3, opts);
}

int kla_chunk_fwd_static(const void* q, const void* k, const void* v, const float* log_alpha, const float* eta,
                         float eps, const float* h0, void* o, float* hT, const int32_t* cu_seqlens_dev,
                         const int32_t* cu_seqlens_host, int n_seq, int N, int T, int H, int dk, int dv, int chunk,
                         kla_dtype dt, void* hip_stream)
{
    Plan pl;
    const int rc = chunk_fwd_validate(q, k, v, log_alpha, eta, eps, h0, o, hT, cu_seqlens_dev, cu_seqlens_host, n_seq, N,
                                      T, H, dk, dv, chunk, dt, 0u, &pl);
    if (rc != KLA_OK) return rc;
    if (pl.total > kStaticScratchBytes) return KLA_ERR_WORKSPACE;      // refused before any HIP call
    if (pl.n_states == 0) return KLA_OK;
    void* ws = static_scratch();
    if (!ws) return KLA_ERR_HIP;
    return chunk_fwd_launch(q, k, v, log_alpha, eta, eps, h0, o, hT, cu_seqlens_dev, n_seq, N, T, H, dk, dv, dt, pl, ws,
                            hip_stream, 3, 0u);
}

size_t kla_chunk_bwd_workspace_bytes(int N, int T, int H, int dk, int dv, int chunk, kla_dtype dt,
                                     const int32_t* cu_seqlens_host, int n_seq)
{
    return kla_chunk_bwd_workspace_bytes_opts(N, T, H, dk, dv, chunk, dt, cu_seqlens_host, n_seq, 0u);
}

size_t kla_chunk_bwd_workspace_bytes_opts(int N, int T, int H, int dk, int dv, int chunk, kla_dtype dt,
                                          const int32_t* cu_seqlens_host, int n_seq, unsigned opts)
{
    BwdPlan pl;
    if (make_bwd_plan(N, T, H, dk, dv, chunk, (int)dt, cu_seqlens_host, n_seq, opts, &pl) != KLA_OK) return 0;
    return pl.total;
}

int kla_chunk_bwd(const void* q, const void* k, const void* v, const float* log_alpha, const float* eta, float eps,
                  const float* h0, const void* d_o, const float* d_hT, void* dq, void* dk_, void* dv_,
                  float* dlog_alpha, float* deta, float* dh0, const int32_t* cu_seqlens_dev,
                  const int32_t* cu_seqlens_host, int n_seq, int N, int T, int H, int dk, int dv, int chunk,
                  kla_dtype dt, void* workspace, size_t workspace_bytes, void* hip_stream)
{
    return kla_chunk_bwd_opts(q, k, v, log_alpha, eta, eps, h0, d_o, d_hT, dq, dk_, dv_, dlog_alpha, deta, dh0,
                              cu_seqlens_dev, cu_seqlens_host, n_seq, N, T, H, dk, dv, chunk, dt, workspace,
                              workspace_bytes, hip_stream, 0u);
}

int kla_chunk_bwd_opts(const void* q, const void* k, const void* v, const float* log_alpha, const float* eta, float eps,
                       const float* h0, const void* d_o, const float* d_hT, void* dq, void* dk_, void* dv_,
                       float* dlog_alpha, float* deta, float* dh0, const int32_t* cu_seqlens_dev,
                       const int32_t* cu_seqlens_host, int n_seq, int N, int T, int H, int dk, int dv, int chunk,
                       kla_dtype dt, void* workspace, size_t workspace_bytes, void* hip_stream, unsigned opts)
{
    BwdPlan pl;
    const int rc = make_bwd_plan(N, T, H, dk, dv, chunk, (int)dt, cu_seqlens_host, n_seq, opts, &pl);
    if (rc != KLA_OK) return rc;
    opts &= kOptMask;
    if (!(eps >= 0.0f) || isinf(eps)) return KLA_ERR_SHAPE;
    if (n_seq > 0 && !cu_seqlens_dev) return KLA_ERR_NULL;
    if (n_seq == 0 && cu_seqlens_dev) return KLA_ERR_SHAPE;
    const bool any_tokens = (long)N * T > 0;
    if (any_tokens && (!q || !k || !v || !log_alpha || !eta || !d_o || !dq || !dk_ || !dv_ || !dlog_alpha || !deta))
        return KLA_ERR_NULL;
    if (!workspace) return KLA_ERR_WORKSPACE;
    if ((reinterpret_cast<uintptr_t>(workspace) & 255u) != 0 || workspace_bytes < pl.total) return KLA_ERR_WORKSPACE;
    if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(d_o) || !aligned16(dq) || !aligned16(dk_) ||
        !aligned16(dv_) || !aligned16(h0) || !aligned16(d_hT) || !aligned16(dh0) ||
        (reinterpret_cast<uintptr_t>(log_alpha) & 3u) || (reinterpret_cast<uintptr_t>(eta) & 3u) ||
        (reinterpret_cast<uintptr_t>(dlog_alpha) & 3u) || (reinterpret_cast<uintptr_t>(deta) & 3u))
        return KLA_ERR_ALIGN;
    if (pl.base.n_states == 0) return KLA_OK;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    char* ws = static_cast<char*>(workspace);
    if (dt == KLA_BF16)
        return chunk_bwd_impl<bf16_t>(q, k, v, log_alpha, eta, eps, h0, d_o, d_hT, dq, dk_, dv_, dlog_alpha, deta, dh0,
                                      cu_seqlens_dev, n_seq, N, T, H, dk, dv, pl, ws, st, opts);
    return chunk_bwd_impl<float>(q, k, v, log_alpha, eta, eps, h0, d_o, d_hT, dq, dk_, dv_, dlog_alpha, deta, dh0,
                                 cu_seqlens_dev, n_seq, N, T, H, dk, dv, pl, ws, st, opts);
}

size_t kla_chunk_fwd_diag_workspace_bytes(int N, int T, int H, int dk, int dv, int chunk, kla_dtype dt,
                                          const int32_t* cu_seqlens_host, int n_seq)
{
    DiagPlan pl;
    if (make_diag_plan(N, T, H, dk, dv, chunk, (int)dt, cu_seqlens_host, n_seq, 0u, &pl) != KLA_OK) return 0;
    return pl.total;
}

int kla_chunk_fwd_diag(const void* q, const void* k, const void* v, const float* log_alpha, const float* eta, float eps,
                       const float* h0, void* o, float* hT, const int32_t* cu_seqlens_dev,
                       const int32_t* cu_seqlens_host, int n_seq, int N, int T, int H, int dk, int dv, int chunk,
                       kla_dtype dt, void* workspace, size_t workspace_bytes, void* hip_stream)
{
    return kla_chunk_fwd_diag_opts(q, k, v, log_alpha, eta, eps, h0, o, hT, cu_seqlens_dev, cu_seqlens_host, n_seq, N, T, H,
                                   dk, dv, chunk, dt, workspace, workspace_bytes, hip_stream, 0u);
}

int kla_chunk_fwd_diag_opts(const void* q, const void* k, const void* v, const float* log_alpha, const float* eta, float eps,
                            const float* h0, void* o, float* hT, const int32_t* cu_seqlens_dev,
                            const int32_t* cu_seqlens_host, int n_seq, int N, int T, int H, int dk, int dv, int chunk,
                            kla_dtype dt, void* workspace, size_t workspace_bytes, void* hip_stream, unsigned opts)
{
    DiagPlan pl;
    const int rc = make_diag_plan(N, T, H, dk, dv, chunk, (int)dt, cu_seqlens_host, n_seq, opts, &pl);
    if (rc != KLA_OK) return rc;
    opts &= kOptMask;
    if (!(eps >= 0.0f) || isinf(eps)) return KLA_ERR_SHAPE;
    if (n_seq > 0 && !cu_seqlens_dev) return KLA_ERR_NULL;
    if (n_seq == 0 && cu_seqlens_dev) return KLA_ERR_SHAPE;
    const bool any_tokens = (long)N * T > 0;
    if (any_tokens && (!q || !k || !v || !log_alpha || !eta || !o)) return KLA_ERR_NULL;
    if (!workspace) return KLA_ERR_WORKSPACE;
    if ((reinterpret_cast<uintptr_t>(workspace) & 255u) != 0 || workspace_bytes < pl.total) return KLA_ERR_WORKSPACE;
    if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(o) || !aligned16(h0) || !aligned16(hT) ||
        (reinterpret_cast<uintptr_t>(log_alpha) & 3u) || (reinterpret_cast<uintptr_t>(eta) & 3u))
        return KLA_ERR_ALIGN;
    if (pl.base.n_states == 0) return KLA_OK;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    char* ws = static_cast<char*>(workspace);
    if (dt == KLA_BF16)
        return chunk_fwd_diag_impl<bf16_t>(q, k, v, log_alpha, eta, eps, h0, o, hT, cu_seqlens_dev, n_seq, N, T, H, dk, dv,
                                           pl, ws, st, opts);
    return chunk_fwd_diag_impl<float>(q, k, v, log_alpha, eta, eps, h0, o, hT, cu_seqlens_dev, n_seq, N, T, H, dk, dv, pl,
                                      ws, st, opts);
}

int kla_decode_step_diag(const void* q, const void* k, const void* v, const float* log_alpha, const float* eta,
                         float eps, float* S, void* o, int B, int H, int dk, int dv, kla_dtype dt, void* hip_stream)
{
    return kla_decode_step_diag_opts(q, k, v, log_alpha, eta, eps, S, o, B, H, dk, dv, dt, hip_stream, 0u);
}

int kla_decode_step_diag_opts(const void* q, const void* k, const void* v, const float* log_alpha, const float* eta,
                              float eps, float* S, void* o, int B, int H, int dk, int dv, kla_dtype dt, void* hip_stream,
                              unsigned opts)
{
    if (!dt_ok((int)dt)) return KLA_ERR_DTYPE;
    Tune tune;
    if (!parse_tune(opts, &tune)) return KLA_ERR_SHAPE;
    opts &= kOptMask;
    if (B < 0 || H <= 0 || !dk_ok(dk) || !dv_ok(dv) || (long)B * H > 0x7fffffffL) return KLA_ERR_SHAPE;
    if (!(eps >= 0.0f) || isinf(eps)) return KLA_ERR_SHAPE;
    if (B == 0) return KLA_OK;
    if (!q || !k || !v || !log_alpha || !eta || !S || !o) return KLA_ERR_NULL;
    if (!aligned16(S) || (reinterpret_cast<uintptr_t>(q) & 3u) || (reinterpret_cast<uintptr_t>(k) & 3u) ||
        (reinterpret_cast<uintptr_t>(v) & 3u) || (reinterpret_cast<uintptr_t>(o) & 3u) ||
        (reinterpret_cast<uintptr_t>(log_alpha) & 3u) || (reinterpret_cast<uintptr_t>(eta) & 3u))
        return KLA_ERR_ALIGN;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    hipError_t e;
    if (dt == KLA_BF16)
        e = kla::launch_decode<bf16_t>(static_cast<const bf16_t*>(q), static_cast<const bf16_t*>(k),
                                       static_cast<const bf16_t*>(v), log_alpha, eta, eps, S, static_cast<bf16_t*>(o),
                                       B * H, dk, dv, 64, tune.decode_nt, kla::kOptDiagDecay | opts, st);
    else
        e = kla::launch_decode<float>(static_cast<const float*>(q), static_cast<const float*>(k),
                                      static_cast<const float*>(v), log_alpha, eta, eps, S, static_cast<float*>(o),
                                      B * H, dk, dv, 64, tune.decode_nt, kla::kOptDiagDecay | opts, st);
    return e == hipSuccess ? KLA_OK : KLA_ERR_HIP;
}

int kla_debug_chunk_stage(const void* q, const void* k, const void* v, const float* log_alpha, const float* eta,
                          float eps, const float* h0, void* o, float* hT, const int32_t* cu_seqlens_dev,
                          const int32_t* cu_seqlens_host, int n_seq, int N, int T, int H, int dk, int dv, int chunk,
                          kla_dtype dt, void* workspace, size_t workspace_bytes, void* hip_stream, int stage)
{
    if (stage != 1 && stage != 2) return KLA_ERR_SHAPE;
    return chunk_fwd_checked(q, k, v, log_alpha, eta, eps, h0, o, hT, cu_seqlens_dev, cu_seqlens_host, n_seq, N, T, H,
                             dk, dv, chunk, dt, workspace, workspace_bytes, hip_stream, stage, KLA_TUNE_UNFUSED);
}

int kla_debug_intra_chunk(const void* q, const void* k, const float* log_alpha, const float* eta, float eps,
                          float* Tb_out, float* P_out, float* g_out, const int32_t* cu_seqlens_dev,
                          const int32_t* cu_seqlens_host, int n_seq, int N, int T, int H, int dk, int chunk,
                          kla_dtype dt, void* workspace, size_t workspace_bytes, void* hip_stream)
{
    Plan pl;
    const int rc = make_plan(N, T, H, dk, 64, chunk, (int)dt, cu_seqlens_host, n_seq, KLA_TUNE_UNFUSED, &pl);
    if (rc != KLA_OK) return rc;
    if (!(eps >= 0.0f) || isinf(eps)) return KLA_ERR_SHAPE;
    if (n_seq > 0 && !cu_seqlens_dev) return KLA_ERR_NULL;
    if (n_seq == 0 && cu_seqlens_dev) return KLA_ERR_SHAPE;
    if (!q || !k || !log_alpha || !eta || !Tb_out || !P_out || !g_out) return KLA_ERR_NULL;
    if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255u) != 0 || workspace_bytes < pl.total)
        return KLA_ERR_WORKSPACE;
    if (!aligned16(q) || !aligned16(k)) return KLA_ERR_ALIGN;
    if (pl.n_chunks == 0) return KLA_OK;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    char* ws = static_cast<char*>(workspace);
    if (dt == KLA_BF16)
        return chunk_fwd_impl<bf16_t>(q, k, nullptr, log_alpha, eta, eps, nullptr, nullptr, nullptr, cu_seqlens_dev,
                                      n_seq, N, T, H, dk, 64, pl, ws, 5, Tb_out, P_out, g_out, st, 0u);
    return chunk_fwd_impl<float>(q, k, nullptr, log_alpha, eta, eps, nullptr, nullptr, nullptr, cu_seqlens_dev, n_seq, N,
                                 T, H, dk, 64, pl, ws, 5, Tb_out, P_out, g_out, st, 0u);
}

int kla_debug_peak_probe(int kind, void* buf, void* aux, size_t bytes, int iters, void* hip_stream)
{
    if (kind < 0 || kind > 3 || iters < 0) return KLA_ERR_SHAPE;
    if (kind == 3) {
        const int ni = iters & 255, depth = 1 + (iters >> 8);
        if ((ni != 16 && ni != 32 && ni != 48 && ni != 60) || depth > 2) return KLA_ERR_SHAPE;
        if (!buf) return KLA_ERR_NULL;
        if (!aligned16(buf)) return KLA_ERR_ALIGN;
        if (bytes < (size_t)8 * 64 * ni * 4 * 2048) return KLA_ERR_WORKSPACE;
    } else if (kind == 2) {
        if (bytes == 0 || bytes > 0x7fffffffu || iters == 0) return KLA_ERR_SHAPE;
        if (!aux) return KLA_ERR_NULL;
    } else {
        if (bytes == 0 || bytes % 65536 != 0 || bytes / 65536 > 0x7fffffffu) return KLA_ERR_SHAPE;
        if (!buf || (kind == 1 && !aux)) return KLA_ERR_NULL;
        if (!aligned16(buf)) return KLA_ERR_ALIGN;
    }
    return kla::launch_probe(kind, buf, aux, bytes, iters, static_cast<hipStream_t>(hip_stream)) == hipSuccess ? KLA_OK : KLA_ERR_HIP;
}

int kla_decode_step(const void* q, const void* k, const void* v, const float* log_alpha, const float* eta, float eps,
                    float* S, void* o, int B, int H, int dk, int dv, kla_dtype dt, void* hip_stream)
{
    return kla_decode_step_opts(q, k, v, log_alpha, eta, eps, S, o, B, H, dk, dv, dt, hip_stream, 0u);
}

int kla_decode_step_opts(const void* q, const void* k, const void* v, const float* log_alpha, const float* eta,
                         float eps, float* S, void* o, int B, int H, int dk, int dv, kla_dtype dt, void* hip_stream,
                         unsigned opts)
{
    if (!dt_ok((int)dt)) return KLA_ERR_DTYPE;
    Tune tune;
    if (!parse_tune(opts, &tune)) return KLA_ERR_SHAPE;
    opts &= kOptMask;
    if (B < 0 || H <= 0 || !dk_ok(dk) || !dv_ok(dv) || (long)B * H > 0x7fffffffL) return KLA_ERR_SHAPE;
    if (!(eps >= 0.0f) || isinf(eps)) return KLA_ERR_SHAPE;
    if (B == 0) return KLA_OK;
    if (!q || !k || !v || !log_alpha || !eta || !S || !o) return KLA_ERR_NULL;
    if (!aligned16(S) || (reinterpret_cast<uintptr_t>(q) & 3u) || (reinterpret_cast<uintptr_t>(k) & 3u) ||
        (reinterpret_cast<uintptr_t>(v) & 3u) || (reinterpret_cast<uintptr_t>(o) & 3u) ||
        (reinterpret_cast<uintptr_t>(log_alpha) & 3u) || (reinterpret_cast<uintptr_t>(eta) & 3u))
        return KLA_ERR_ALIGN;
    // State columns per workgroup: 128 (measured best at 512 workgroups, e.g. 64 x 8 states of 128 columns), narrower for
    // small batches so that about 512 workgroups still share the chip (B = 1, H = 8: 3.2 us per step with 32 columns,
    // 4.2 us with 128).  The tuning field KLA_TUNE_DECODE_SLICE(32 | 64 | 128 | 256) overrides.
    int slice = dv < 128 ? dv : 128;
    while (slice > 32 && (long)B * H * (dv / slice) < 512) slice >>= 1;
    if (tune.decode_slice) slice = tune.decode_slice;
    if (slice > dv) slice = dv;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    hipError_t e;
    if (dt == KLA_BF16)
        e = kla::launch_decode<bf16_t>(static_cast<const bf16_t*>(q), static_cast<const bf16_t*>(k),
                                       static_cast<const bf16_t*>(v), log_alpha, eta, eps, S, static_cast<bf16_t*>(o),
                                       B * H, dk, dv, slice, tune.decode_nt, opts, st);
    else
        e = kla::launch_decode<float>(static_cast<const float*>(q), static_cast<const float*>(k),
                                      static_cast<const float*>(v), log_alpha, eta, eps, S, static_cast<float*>(o),
                                      B * H, dk, dv, slice, tune.decode_nt, opts, st);
    return e == hipSuccess ? KLA_OK : KLA_ERR_HIP;
}

int kla_beta(const void* k, const float* eta, float eps, float* beta, long n_token_heads, int dk, kla_dtype dt,
             void* hip_stream)
{
    if (!dt_ok((int)dt)) return KLA_ERR_DTYPE;
    if (n_token_heads < 0 || !dk_ok(dk) || (n_token_heads * (dk / 8) + 255) / 256 > 0x7fffffffL) return KLA_ERR_SHAPE;
    if (!(eps >= 0.0f) || isinf(eps)) return KLA_ERR_SHAPE;
    if (n_token_heads == 0) return KLA_OK;
    if (!k || !eta || !beta) return KLA_ERR_NULL;
    if (!aligned16(k)) return KLA_ERR_ALIGN;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    const hipError_t e = dt == KLA_BF16
        ? kla::launch_beta<bf16_t>(static_cast<const bf16_t*>(k), eta, eps, beta, n_token_heads, dk, st)
        : kla::launch_beta<float>(static_cast<const float*>(k), eta, eps, beta, n_token_heads, dk, st);
    return e == hipSuccess ? KLA_OK : KLA_ERR_HIP;
}

}  // extern "C"
