// Host-side declarations of the kernel launchers (one translation unit per stage).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "kla_common.hpp"

namespace kla {

// option bits (the values of KLA_OPT_* in include/kla.h)
constexpr unsigned kOptNormalizeQ = 1u, kOptGdnBeta = 2u;
// internal: diagonal gating (log_alpha holds d_k values per token and head); set by the *_diag entry points only
constexpr unsigned kOptDiagDecay = 0x100u;
// internal: a backward sweep that only carries its state through the chunks (no checkpoints, no rows written)
constexpr unsigned kOptNoStore = 0x200u;

// ---- decode step and stand-alone coefficient -----------------------------------------------
template <typename T>
hipError_t launch_decode(const T* q, const T* k, const T* v, const float* log_alpha, const float* eta, float eps,
                         float* S, T* o, int BH, int dk, int dv, int slice, int nt_force, unsigned opts, hipStream_t st);
template <typename T>
hipError_t launch_beta(const T* k, const float* eta, float eps, float* beta, long n_rows, int dk, hipStream_t st);

// ---- chunkwise forward ------------------------------------------------------------------------
// Workspace areas, all indexed by chunk-head ch = global_chunk * H + h:
//   wsT, wsP : per chunk-head one record [T' | P | gamma_i | gamma_C/gamma_i | gamma_i/||q_i||]; T' and P are 6
//              tile-pairs x 64 operand slots of 8 elements (see kla_mma.hpp), the three vectors 64 fp32 each;
//              wsP = wsT + one half, both advance by a whole record
//   wsG      : 128 fp32 per chunk-head: g_i = log gamma_i, then 1/||q_i|| (1 unless the read-out is normalised)
//   chunk_off: int32 [n_seq + 1], packed batches only
template <typename E> struct IntraArgs {
    const E* q; const E* k;
    const float* log_alpha; const float* eta; float eps;
    const int* cu_seqlens; const int* chunk_off; int n_seq;
    int T, NT, H;
    E* wsT; E* wsP; float* wsG;
    unsigned opts;                               // kOptNormalizeQ | kOptGdnBeta
};
template <typename E> hipError_t launch_intra(const IntraArgs<E>& a, int dk, int n_chunks, hipStream_t st);
// the records of the backward pass (see bwd_record_bytes in kla_mma.hpp) at a.wsT; a.wsP, a.wsG unused; a.opts: kOptNormalizeQ | kOptGdnBeta
template <typename E> hipError_t launch_intra_bwd(const IntraArgs<E>& a, int dk, int n_chunks, hipStream_t st);

// Diagonal gating (App. B): log_alpha is [tokens, H, dk].  Besides the records (with unit decay vectors) the stage
// writes the operands the scan is then given in place of k and q - kplus = K o Gamma, qplus = Q o Gamma (rows of the
// K S and Q S products), ktilde = K o (gamma_C / Gamma) (the state update) - and gc = gamma_C per channel,
// [chunk-head][dk] fp32.
template <typename E> struct IntraDiagArgs {
    const E* q; const E* k;
    const float* log_alpha; const float* eta; float eps;
    const int* cu_seqlens; const int* chunk_off; int n_seq;
    int T, NT, H;
    E* wsT; float* wsG;
    E* kplus; E* qplus; E* ktilde; float* gc;
    unsigned opts;                               // kOptNormalizeQ (folded into qplus and P) | kOptGdnBeta
};
template <typename E> hipError_t launch_intra_diag(const IntraDiagArgs<E>& a, int dk, int n_chunks, hipStream_t st);

template <typename E> struct ScanArgs {
    const E* q; const E* k; const E* v;
    const float* h0; E* o; float* hT;
    const int* cu_seqlens; const int* chunk_off; int n_seq;
    int N, T, NT, H, dv;
    const E* wsT; const E* wsP; const float* wsG;
    unsigned opts;
    // Segmented mode (seg_G > 0, fixed-length batches only): "sequence" s of the kernel is segment s % seg_G of
    // sequence s / seg_G, seg_Lc chunks long (the last one of a sequence takes what is left), and h0 / hT are
    // indexed by segment.
    int seg_G, seg_Lc;
    // Diagonal gating (generic kernel only): the transposed K operand of the state update comes from kt_src instead of
    // k, and the state decays per row by gc_vec[chunk-head][dk] instead of by gamma_C.  Both NULL otherwise.
    const E* kt_src; const float* gc_vec;
    // Fused bf16 scan only (the stage forms T', P and the decay vectors itself; wsT, wsP, wsG unused): the gates.
    const float* log_alpha = nullptr; const float* eta = nullptr; float eps = 0.f;
};
// waves = 1, 2 or 4: each wave of a workgroup carries 16 state columns through the whole sequence
template <typename E> hipError_t launch_scan(const ScanArgs<E>& a, int dk, int waves, hipStream_t st);
template <typename E> hipError_t launch_scan_diag(const ScanArgs<E>& a, int dk, int waves, hipStream_t st);

// bf16 specialisations (direct global->LDS copies, swizzled token-major staging, transposing LDS reads)
hipError_t launch_intra_bf16(const IntraArgs<bf16_t>& a, int dk, int n_chunks, hipStream_t st);
hipError_t launch_scan_bf16(const ScanArgs<bf16_t>& a, int dk, int waves, hipStream_t st);
hipError_t launch_scan_bf16_diag(const ScanArgs<bf16_t>& a, int dk, int waves, hipStream_t st);   // diagonal gating
// Fused forward (no intra-chunk stage, no workspace): waves = 1 or 2; fixed-length, packed or segmented batches.
hipError_t launch_scan_fused_bf16(const ScanArgs<bf16_t>& a, int dk, int waves, hipStream_t st);

// Segment-parallel scan of long sequences in small batches (bf16): per-segment affine maps of the state, their
// prefix composition, then the ordinary scan over all segments at once.  `maps` holds (G-1) x [N | M] per
// sequence and head, `seg_state` the G incoming states; both fp32, in the workspace.
hipError_t launch_segment_maps_bf16(const ScanArgs<bf16_t>& a, int dk, float* maps, hipStream_t st);
// the same maps from the records of the backward pass (a.wsT = record base; see bwd_record_bytes)
hipError_t launch_segment_maps_bwdrec_bf16(const ScanArgs<bf16_t>& a, int dk, float* maps, hipStream_t st);
// Reverse composition for the backward pass: g(G-1) = d_hT (or 0), g(G-2) = b(G-1), g(s-1) = M_s^T g(s) + b(s) for
// s = G-2 .. 1, where g(s) is the gradient of the state leaving segment s and b(s) what the reverse sweep of segment s
// returns for a zero g(s) (for the last segment: for its true g).  gseg, bseg: [N * G][H][dk][dv] fp32.
hipError_t launch_segment_combine_rev(const float* maps, const float* bseg, float* gseg, int N, int H, int dk, int dv,
                                      int G, hipStream_t st);
// gseg = 0 except the last segment of every sequence, which gets d_hT (or 0 when d_hT is NULL)
hipError_t launch_segment_scatter(const float* d_hT, float* gseg, int N, int H, int dk, int dv, int G, hipStream_t st);
hipError_t launch_segment_combine(const float* h0, const float* maps, float* seg_state, int N, int H, int dk, int dv,
                                  int G, hipStream_t st);
hipError_t launch_segment_gather(const float* seg_state, float* hT, int N, int H, int dk, int dv, int G, int g_last,
                                 hipStream_t st);

// ---- chunkwise backward (gradient of sum <d_o, o> + sum <d_hT, hT>) ----------------------------------
// Stage 1 (launch_intra_bwd) leaves one record per chunk-head at `rec`.  Stage 2 walks every (sequence, head)
// forward and leaves, per chunk, the incoming state S_c and the rows X = V - D_gamma K S_c and U = T' X of eq. (6).
// Stage 3 walks backward and leaves the gradient dS'_c of the state each chunk hands on and Y = M^T dU, and writes
// dv = B Y and dh0.  Stage 4 contracts those over d_v per chunk-head and writes dq, dk, dlog_alpha, deta.
// X, U, Y are laid out like v.  The state checkpoints are stored transposed and in the element type:
// [chunk-head][d_v][d_k], because stage 4 uses them only as MFMA operands contracted over d_v.
template <typename E> struct BwdArgs {
    const E* q; const E* k; const E* v;
    const float* log_alpha; const float* eta; float eps;
    const float* h0; const E* d_o; const float* d_hT;
    E* dq; E* dk; E* dv; float* dlog_alpha; float* deta; float* dh0;
    const int* cu_seqlens; const int* chunk_off; int n_seq;
    int N, T, NT, H, dv_dim;
    const char* rec;                 // stage-1 records
    E* s_chk; E* ds_chk;             // [n_chunks * H][dv][dk]
    E* X; E* U; E* Y;                // [tokens][H][dv]
    unsigned opts;                   // kOptGdnBeta: beta = eta, so dk has no term through the coefficient; kOptNormalizeQ:
                                     // read-out divided by ||q||; kOptNoStore (sweeps only, internal)
    // Segmented sweeps (seg_G > 0, fixed-length bf16 batches only; see ScanArgs): h0, d_hT and dh0 are then indexed by
    // segment, [N * seg_G][H][dk][dv].
    int seg_G, seg_Lc;
};
template <typename E> hipError_t launch_bwd_states(const BwdArgs<E>& a, int dk, int waves, hipStream_t st);
template <typename E> hipError_t launch_bwd_scan(const BwdArgs<E>& a, int dk, int waves, hipStream_t st);
// bf16 specialisations of the two sweeps (copy wave, LDS ring, transposing reads: see kla_chunk_bwd_bf16.hip)
hipError_t launch_intra_bwd_bf16(const IntraArgs<bf16_t>& a, int dk, int n_chunks, hipStream_t st);
hipError_t launch_bwd_states_bf16(const BwdArgs<bf16_t>& a, int dk, int waves, hipStream_t st);
hipError_t launch_bwd_scan_bf16(const BwdArgs<bf16_t>& a, int dk, int waves, hipStream_t st);
hipError_t launch_bwd_assemble_bf16(const BwdArgs<bf16_t>& a, int dk, long n_chunks, hipStream_t st);
template <typename E> hipError_t launch_bwd_assemble(const BwdArgs<E>& a, int dk, long n_chunks, hipStream_t st);

// measurement probes (kla_probe.hip)
hipError_t launch_probe(int kind, void* buf, void* aux, size_t bytes, int iters, hipStream_t st);

hipError_t launch_chunk_offsets(const int* cu_seqlens, int n_seq, int* chunk_off, hipStream_t st);
template <typename E>
hipError_t launch_unpack(const E* wsT, const E* wsP, const float* wsG, float* Tb, float* P, float* gout, long n_ch,
                         hipStream_t st);

}  // namespace kla
