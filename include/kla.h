/*
 * kla.h - C ABI of the MI355X (gfx950) Kaczmarz Linear Attention hot path.
 *
 * The library computes, per sequence and per head, the gated delta-rule
 * recurrence of the paper (Sec. 3.1 eq. (3), Sec. 3.3 Algorithm 1):
 *
 *     S~   = alpha_t S_{t-1}                      alpha_t = exp(log_alpha_t)
 *     e_t  = v_t - S~^T k_t
 *     beta = eta_t / (||k_t||^2 + eps)            (beta := 0 when the denominator is 0)
 *     S_t  = S~ + beta k_t e_t^T
 *     o_t  = S_t^T q_t                            (no query normalisation in the plain entry points;
 *                                                  the *_opts ones offer Sec. 3.3's o_t / ||q_t||)
 *
 * with the state S a d_k x d_v matrix (Sec. 2), stored row-major with d_v
 * contiguous, always fp32.  The same map written for R = S^T is eq. (5).
 *
 * Conventions for every entry point
 *   - All data pointers are DEVICE pointers unless a parameter says "host".
 *   - The caller owns every buffer and keeps it alive until the stream has
 *     passed the call.  The library allocates and frees nothing and is thread-safe; the
 *     only state it keeps is, per device, the address of the scratch array of
 *     kla_chunk_fwd_static; it reads nothing from the environment.  Work is enqueued on `hip_stream`
 *     (a hipStream_t, NULL = the default stream); the call returns without
 *     waiting for it.
 *   - Return value: KLA_OK or a negative kla_status.  A validation failure is
 *     reported before anything is launched and leaves all outputs untouched.  A
 *     failed launch is reported as KLA_ERR_HIP.
 *   - q, k, v, o share one element type (kla_dtype).  Gates, eps, states are fp32.
 *   - Token-major layout: a tensor "[N, T, H, D]" is contiguous with D fastest.
 *     Data pointers must be 16-byte aligned.
 *   - Supported shapes: dk in {64, 128}; dv in {64, 128, 256}; chunk == 64.
 */
#ifndef KLA_H
#define KLA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Element type of q, k, v, o.  Passed as a plain int, so that a value that is neither of the two comes back as
 * KLA_ERR_DTYPE (an enum parameter holding any other value is undefined behaviour in C++). */
enum { KLA_F32 = 0, KLA_BF16 = 1 };
typedef int kla_dtype;

typedef enum {
    KLA_OK = 0,
    KLA_ERR_NULL = -1,       /* a required pointer is NULL                               */
    KLA_ERR_SHAPE = -2,      /* unsupported or inconsistent sizes, or eps < 0            */
    KLA_ERR_DTYPE = -3,      /* unknown kla_dtype                                        */
    KLA_ERR_ALIGN = -4,      /* a data pointer is not 16-byte aligned                    */
    KLA_ERR_WORKSPACE = -5,  /* workspace missing or smaller than the query reports      */
    KLA_ERR_SEQLENS = -6,    /* host cu_seqlens not starting at 0, decreasing, or != T   */
    KLA_ERR_HIP = -7         /* the HIP runtime refused a launch                         */
} kla_status;

/* Human-readable name of a status code (static storage, never NULL). */
const char *kla_status_string(int code);

/*
 * Bytes of device scratch kla_chunk_fwd needs for these sizes (0 on invalid sizes).  It covers the per-chunk
 * objects of eqs. (6)-(7) and, for a small bf16 batch of long sequences, the per-segment state maps of the
 * segment-parallel scan (where the fused bf16 kernel runs, which keeps those objects on chip, only a token 256
 * bytes); ask again whenever a size or the element type changes.
 * For a packed batch pass the host copy of cu_seqlens and n_seq > 0 (then N must be 1
 * and T the total token count); otherwise cu_seqlens_host = NULL, n_seq = 0.
 */
size_t kla_chunk_fwd_workspace_bytes(int N, int T, int H, int dk, int dv, int chunk, kla_dtype dt,
                                     const int32_t *cu_seqlens_host, int n_seq);

/*
 * Chunkwise-parallel forward (Sec. 4, Algorithm 1 right panel, eqs. (6)-(8)): for every
 * sequence and head, the outputs o_t of all tokens and the state after the last token.
 * The result equals the token loop above; chunks of 64 tokens are counted from each
 * sequence's own first token and never straddle sequences; a sequence of any length >= 0 is
 * accepted (a short last chunk is handled inside the kernels).
 *
 *   q, k        [N, T, H, dk]  dt         in
 *   v           [N, T, H, dv]  dt         in
 *   log_alpha   [N, T, H]      fp32       in   natural log of the decay gate (<= 0 expected)
 *   eta         [N, T, H]      fp32       in   write gate (0..1 expected)
 *   eps                                   in   stabiliser of eq. (3), >= 0
 *   h0          [n_states, H, dk, dv] fp32 in  initial states, or NULL for zeros
 *   o           [N, T, H, dv]  dt         out  must not alias an input
 *   hT          [n_states, H, dk, dv] fp32 out final states, or NULL if unwanted; may alias h0
 *   cu_seqlens_dev  [n_seq+1] int32 device, or NULL for a fixed-length batch
 *   cu_seqlens_host same values on the host (used for grid sizing and validation), or NULL
 *   n_seq       number of packed sequences; 0 for fixed length.  If n_seq > 0 then N == 1,
 *               T is the total token count and n_states = n_seq; otherwise n_states = N.
 *   workspace   device scratch of at least kla_chunk_fwd_workspace_bytes(...) bytes,
 *               256-byte aligned; contents undefined on return.
 */
int kla_chunk_fwd(const void *q, const void *k, const void *v,
                  const float *log_alpha, const float *eta, float eps,
                  const float *h0, void *o, float *hT,
                  const int32_t *cu_seqlens_dev, const int32_t *cu_seqlens_host, int n_seq,
                  int N, int T, int H, int dk, int dv, int chunk, kla_dtype dt,
                  void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * kla_chunk_fwd for callers that cannot allocate device memory and have no workspace to hand over: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, results and error
 * codes as kla_chunk_fwd (same kernels) without `workspace` / `workspace_bytes`: whatever kla_chunk_fwd would
 * keep in its workspace - the per-chunk objects of the two-kernel form (fp32 inputs, wide value heads), the maps
 * and states of the segment-parallel scan - goes to a fixed scratch array of KLA_STATIC_SCRATCH_BYTES that is part
 * of the library's device image (every GPU the library is used on holds its own copy from the first use there
 * until the process ends).  The call allocates and frees nothing, neither directly nor through another library.
 *   - A problem whose kla_chunk_fwd_workspace_bytes(...) exceeds KLA_STATIC_SCRATCH_BYTES is refused with
 *     KLA_ERR_WORKSPACE before anything is launched (32 MiB holds about 2 400 chunk-heads of the two-kernel form
 *     in bf16, 1 200 in fp32; bf16 problems that run the fused kernel need none of it and are never refused).
 *   - The first call on a device looks up the device address of the array (one hipGetSymbolAddress, which may load
 *     the library's code onto that device): make it outside any stream capture.  KLA_ERR_HIP if the lookup fails.
 *   - All calls on one GPU share the one array: two calls that may overlap in time on the same GPU (different
 *     streams, or different threads) race; calls on one stream, or on different GPUs, do not.  Nothing in the
 *     array has to start at zero, every call writes what it reads.
 */
#define KLA_STATIC_SCRATCH_BYTES (32u << 20)
int kla_chunk_fwd_static(const void *q, const void *k, const void *v,
                         const float *log_alpha, const float *eta, float eps,
                         const float *h0, void *o, float *hT,
                         const int32_t *cu_seqlens_dev, const int32_t *cu_seqlens_host, int n_seq,
                         int N, int T, int H, int dk, int dv, int chunk, kla_dtype dt,
                         void *hip_stream);

/*
 * One recurrent decode step (Algorithm 1 left panel) for B*H independent states.
 *
 *   q, k        [B, H, dk] dt     in
 *   v           [B, H, dv] dt     in
 *   log_alpha, eta [B, H]  fp32   in
 *   S           [B, H, dk, dv] fp32   in/out, updated IN PLACE to S_t
 *   o           [B, H, dv] dt     out
 */
int kla_decode_step(const void *q, const void *k, const void *v,
                    const float *log_alpha, const float *eta, float eps,
                    float *S, void *o,
                    int B, int H, int dk, int dv, kla_dtype dt, void *hip_stream);

/*
 * Options of the *_opts entry points (bit flags; any other bit is KLA_ERR_SHAPE).
 *   KLA_OPT_NORMALIZE_Q  the read-out of Sec. 3.3 / Algorithm 1 (left) as printed,
 *                        o_t = S_t^T q_t / ||q_t||, with o_t = 0 for a zero query; the norm is
 *                        taken over the stored q in fp32.  States are not affected.
 *   KLA_OPT_GDN_BETA     beta_t = eta_t: the gated delta rule the paper starts from (Table 2; the
 *                        "w/o normalization" row of its ablation) instead of eq. (3); eps is
 *                        then unused.
 */
enum { KLA_OPT_NORMALIZE_Q = 1, KLA_OPT_GDN_BETA = 2 };

/*
 * Tuning fields of the same `opts` argument (bits 8..25), for tests and A/B measurements: every setting computes
 * the same results up to rounding, 0 in a field is the library's own choice (the measured best), and a value
 * outside a field's range is KLA_ERR_SHAPE.  They replace any reading of the environment: a call's behaviour
 * depends on its arguments alone.  The workspace needed depends on some of them (segments, the generic and
 * unfused forms), so pass the same `opts` to the *_workspace_bytes_opts query and to the call.
 *   KLA_TUNE_SCAN_WAVES(n)     n = 1, 2, 4: compute waves (16 state columns each) per workgroup of the scan stage
 *   KLA_TUNE_SCAN_SEGMENTS(n)  n = 1: never cut sequences for the segment-parallel scan; n = 2..16: cut into n
 *   KLA_TUNE_GENERIC_SCAN / _INTRA / _BWD   bf16 inputs through the element-type-generic kernels of the fp32 path
 *   KLA_TUNE_UNFUSED           bf16 forward as two kernels (intra-chunk stage, then scan) where one fused kernel would run
 *   KLA_TUNE_FUSED             bf16 forward as the one fused kernel wherever it can run (one or two compute waves per
 *                              workgroup, no segments), also where the two-kernel form is the library's choice
 *   KLA_TUNE_DECODE_SLICE(n)   n = 32, 64, 128, 256: state columns per workgroup of the decode step
 *   KLA_TUNE_DECODE_NT(n)      n = 0..3: bit 0 non-temporal state loads, bit 1 non-temporal state stores
 */
#define KLA_TUNE_SCAN_WAVES(n)    ((unsigned)((n) == 4 ? 3 : (n)) << 8)
#define KLA_TUNE_SCAN_SEGMENTS(n) ((unsigned)(n) << 10)
#define KLA_TUNE_GENERIC_SCAN     (1u << 15)
#define KLA_TUNE_GENERIC_INTRA    (1u << 16)
#define KLA_TUNE_GENERIC_BWD      (1u << 17)
#define KLA_TUNE_DECODE_SLICE(n)  ((unsigned)((n) == 32 ? 1 : (n) == 64 ? 2 : (n) == 128 ? 3 : (n) == 256 ? 4 : 7) << 18)
#define KLA_TUNE_DECODE_NT(n)     ((unsigned)((n) + 1) << 21)
#define KLA_TUNE_UNFUSED          (1u << 24)
#define KLA_TUNE_FUSED            (1u << 25)

/* Workspace of kla_chunk_fwd_opts(..., opts) / kla_chunk_bwd_opts(..., opts) (0 on invalid sizes or fields);
 * the plain queries are these with opts = 0. */
size_t kla_chunk_fwd_workspace_bytes_opts(int N, int T, int H, int dk, int dv, int chunk, kla_dtype dt,
                                          const int32_t *cu_seqlens_host, int n_seq, unsigned opts);
size_t kla_chunk_bwd_workspace_bytes_opts(int N, int T, int H, int dk, int dv, int chunk, kla_dtype dt,
                                          const int32_t *cu_seqlens_host, int n_seq, unsigned opts);

/* kla_chunk_fwd with options; kla_chunk_fwd(...) is kla_chunk_fwd_opts(..., 0).  Same workspace. */
int kla_chunk_fwd_opts(const void *q, const void *k, const void *v,
                       const float *log_alpha, const float *eta, float eps,
                       const float *h0, void *o, float *hT,
                       const int32_t *cu_seqlens_dev, const int32_t *cu_seqlens_host, int n_seq,
                       int N, int T, int H, int dk, int dv, int chunk, kla_dtype dt,
                       void *workspace, size_t workspace_bytes, void *hip_stream, unsigned opts);

/* kla_decode_step with options; kla_decode_step(...) is kla_decode_step_opts(..., 0). */
int kla_decode_step_opts(const void *q, const void *k, const void *v,
                         const float *log_alpha, const float *eta, float eps,
                         float *S, void *o,
                         int B, int H, int dk, int dv, kla_dtype dt, void *hip_stream, unsigned opts);

/*
 * Backward pass of kla_chunk_fwd (no options): gradients of
 *     L = sum_t <d_o_t, o_t> + sum <d_hT, hT>
 * with respect to q, k, v, log_alpha, eta and h0.  The paper trains with this operator but states
 * only its forward map (Algorithm 1; eqs. (3), (6)-(8)); the gradients are those equations
 * differentiated chunk by chunk, including the dependence of beta_t on k_t through eq. (3)
 * (d beta / d k = -2 eta k / (||k||^2 + eps)^2), which the delta rule with beta = eta does not have.
 * The forward quantities are recomputed, not saved: only the inputs of the forward call are needed.
 *
 *   q, k, v, log_alpha, eta, eps, h0, cu_seqlens_*, n_seq, N, T, H, dk, dv, chunk, dt: as in kla_chunk_fwd
 *   d_o         [N, T, H, dv]  dt                in   gradient of the outputs
 *   d_hT        [n_states, H, dk, dv] fp32       in   gradient of the final states, or NULL for zeros
 *   dq, dk_     [N, T, H, dk]  dt                out
 *   dv_         [N, T, H, dv]  dt                out
 *   dlog_alpha, deta  [N, T, H] fp32             out
 *   dh0         [n_states, H, dk, dv] fp32       out  or NULL if unwanted
 *   workspace   device scratch of at least kla_chunk_bwd_workspace_bytes(...) bytes, 256-byte aligned.
 *               It holds, per chunk and head, the incoming state and the gradient of the outgoing state
 *               (dk x dv each, in dt) and three [N, T, H, dv] arrays in dt (two for bf16), so it is much larger
 *               than the forward's: about (2 * dk * dv / 64 + 3 * dv) * sizeof(dt) bytes per token and head.
 *               For a small bf16 batch of long sequences it also holds the per-segment maps and states of the
 *               segment-parallel sweeps (as in kla_chunk_fwd).
 * Outputs must not alias inputs or each other.  Same error codes and conventions as kla_chunk_fwd;
 * rows of the outputs are written for every token of every sequence, nothing else is touched.
 * The result is deterministic (no atomics).
 */
size_t kla_chunk_bwd_workspace_bytes(int N, int T, int H, int dk, int dv, int chunk, kla_dtype dt,
                                     const int32_t *cu_seqlens_host, int n_seq);
int kla_chunk_bwd(const void *q, const void *k, const void *v,
                  const float *log_alpha, const float *eta, float eps,
                  const float *h0, const void *d_o, const float *d_hT,
                  void *dq, void *dk_, void *dv_, float *dlog_alpha, float *deta, float *dh0,
                  const int32_t *cu_seqlens_dev, const int32_t *cu_seqlens_host, int n_seq,
                  int N, int T, int H, int dk, int dv, int chunk, kla_dtype dt,
                  void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * kla_chunk_bwd with options: the backward of kla_chunk_fwd_opts(..., opts), same option bits.
 *   KLA_OPT_GDN_BETA     beta_t = eta_t: d eta = d beta and dk loses its term through the coefficient.
 *   KLA_OPT_NORMALIZE_Q  d_o is the gradient of o_t = S_t^T q_t / ||q_t|| (Sec. 3.3); dq is the gradient with respect to
 *                        the stored q (orthogonal to q_t, since o_t does not depend on the length of q_t), 0 for a zero
 *                        query.
 * kla_chunk_bwd(...) is kla_chunk_bwd_opts(..., 0).  Same workspace.
 */
int kla_chunk_bwd_opts(const void *q, const void *k, const void *v,
                       const float *log_alpha, const float *eta, float eps,
                       const float *h0, const void *d_o, const float *d_hT,
                       void *dq, void *dk_, void *dv_, float *dlog_alpha, float *deta, float *dh0,
                       const int32_t *cu_seqlens_dev, const int32_t *cu_seqlens_host, int n_seq,
                       int N, int T, int H, int dk, int dv, int chunk, kla_dtype dt,
                       void *workspace, size_t workspace_bytes, void *hip_stream, unsigned opts);

/*
 * Diagonal gating (App. B, "Extension to diagonal gating"; App. A, decay-agnostic remark): the decay operator is
 * D_t = diag(alpha_t) with one decay per key channel, S~ = diag(alpha_t) S_{t-1} (row i of the d_k x d_v state is
 * scaled by alpha_t[i]); the residual, the Kaczmarz coefficient of eq. (3), the write and the read-out are unchanged.
 * Inside a chunk gamma_i becomes a vector and every decay ratio acts elementwise inside the inner products
 * (L_ij = beta_i sum_c k_ic k_jc gamma_ic/gamma_jc, and likewise for A o Q K^T, the right-hand side and eq. (8)).
 *
 *   log_alpha   [N, T, H, dk] fp32 (chunk forward) or [B, H, dk] fp32 (decode step): natural log of alpha_t per channel
 * Every other argument, the conventions and the error codes are those of kla_chunk_fwd / kla_decode_step.  The
 * workspace (kla_chunk_fwd_diag_workspace_bytes) also holds three [N, T, H, dk] arrays in dt: the keys and queries
 * with the chunk-local decay folded in, which the scan stage consumes.
 */
size_t kla_chunk_fwd_diag_workspace_bytes(int N, int T, int H, int dk, int dv, int chunk, kla_dtype dt,
                                          const int32_t *cu_seqlens_host, int n_seq);
int kla_chunk_fwd_diag(const void *q, const void *k, const void *v,
                       const float *log_alpha, const float *eta, float eps,
                       const float *h0, void *o, float *hT,
                       const int32_t *cu_seqlens_dev, const int32_t *cu_seqlens_host, int n_seq,
                       int N, int T, int H, int dk, int dv, int chunk, kla_dtype dt,
                       void *workspace, size_t workspace_bytes, void *hip_stream);
int kla_decode_step_diag(const void *q, const void *k, const void *v,
                         const float *log_alpha, const float *eta, float eps,
                         float *S, void *o,
                         int B, int H, int dk, int dv, kla_dtype dt, void *hip_stream);

/* The two diagonal-gating calls with the option bits of kla_chunk_fwd_opts (same meaning: Sec. 3.3 read-out, Table 2's
 * beta_t = eta_t); kla_chunk_fwd_diag(...) and kla_decode_step_diag(...) are these with opts = 0.  Same workspace. */
int kla_chunk_fwd_diag_opts(const void *q, const void *k, const void *v,
                            const float *log_alpha, const float *eta, float eps,
                            const float *h0, void *o, float *hT,
                            const int32_t *cu_seqlens_dev, const int32_t *cu_seqlens_host, int n_seq,
                            int N, int T, int H, int dk, int dv, int chunk, kla_dtype dt,
                            void *workspace, size_t workspace_bytes, void *hip_stream, unsigned opts);
int kla_decode_step_diag_opts(const void *q, const void *k, const void *v,
                              const float *log_alpha, const float *eta, float eps,
                              float *S, void *o,
                              int B, int H, int dk, int dv, kla_dtype dt, void *hip_stream, unsigned opts);

/*
 * The Kaczmarz coefficient alone (eq. (3)): beta[i] = eta[i] / (||k_i||^2 + eps), 0 when the
 * denominator is 0, for n_token_heads rows of dk elements.
 *   k [n_token_heads, dk] dt in;  eta [n_token_heads] fp32 in;  beta [n_token_heads] fp32 out.
 */
int kla_beta(const void *k, const float *eta, float eps, float *beta,
             long n_token_heads, int dk, kla_dtype dt, void *hip_stream);

/*
 * Test hook: the per-chunk objects the first stage of kla_chunk_fwd leaves in its workspace,
 * unpacked to plain row-major fp32 so that they can be compared one by one with eqs. (6)-(7).
 * Arguments as in kla_chunk_fwd.  For every chunk c (global chunk index, sequences in order)
 * and head h:
 *   Tb_out  [n_chunks, H, 64, 64]  (I + B(A^- o K K^T))^{-1} B, i.e. the solve of eq. (6) as a matrix
 *   P_out   [n_chunks, H, 64, 64]  A o Q K^T (lower triangle incl. diagonal) of eq. (7)
 *   g_out   [n_chunks, H, 64]      chunk-local running sum of log_alpha (log gamma_i)
 * Rows and columns beyond a short last chunk are zero (g repeats its last value).
 * The values are those the second stage of the two-kernel form consumes (rounded to dt for dt = bf16); workspace
 * from kla_chunk_fwd_workspace_bytes_opts(..., KLA_TUNE_UNFUSED) with dv = 64.
 */
int kla_debug_intra_chunk(const void *q, const void *k,
                          const float *log_alpha, const float *eta, float eps,
                          float *Tb_out, float *P_out, float *g_out,
                          const int32_t *cu_seqlens_dev, const int32_t *cu_seqlens_host, int n_seq,
                          int N, int T, int H, int dk, int chunk, kla_dtype dt,
                          void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * Profiling hook: one stage of the two-kernel form of kla_chunk_fwd alone (KLA_TUNE_UNFUSED; workspace from
 * kla_chunk_fwd_workspace_bytes_opts(..., KLA_TUNE_UNFUSED)), so that each kernel can be timed between two
 * events.  Arguments as in kla_chunk_fwd.  stage = 1: the intra-chunk stage (fills the workspace);
 * stage = 2: the scan stage (consumes a workspace that stage 1 filled for the same inputs, writes
 * o and hT).  Any other stage is KLA_ERR_SHAPE.
 */
int kla_debug_chunk_stage(const void *q, const void *k, const void *v,
                          const float *log_alpha, const float *eta, float eps,
                          const float *h0, void *o, float *hT,
                          const int32_t *cu_seqlens_dev, const int32_t *cu_seqlens_host, int n_seq,
                          int N, int T, int H, int dk, int dv, int chunk, kla_dtype dt,
                          void *workspace, size_t workspace_bytes, void *hip_stream, int stage);

/*
 * Measurement hook: what this GPU delivers for the access patterns the rooflines of the hot path are quoted
 * against (none of the method's arithmetic runs).  bench.py reports the results as second denominators beside the
 * published peaks.
 *   kind 0  in-place streaming, x <- 2 x over `bytes` of fp32 at buf (a multiple of 65536): every byte read once and
 *           written once, one workgroup per 64 KiB with all loads first, as in the decode step; iters != 0 selects
 *           non-temporal loads and stores.  aux unused.
 *   kind 1  read-only streaming of `bytes` at buf; aux receives bytes / 16384 floats.
 *   kind 2  dense bf16 matrix pipe: `bytes` workgroups of four waves, each wave `iters` rounds of eight
 *           independent 16x16x32 products (16384 flop each per wave); aux receives 256 floats per workgroup.
 *   kind 3  the copy wave of the chunk kernels alone: 256 workgroups, 64 steps; per step one wave brings n copies of
 *           1 KiB (256-byte rows 2 KiB apart; four workgroups of an XCD share the rows) from buf into LDS through a
 *           ring one or two steps deep, one barrier per step.  iters = n + 256 (depth - 1), n one of 16, 32, 48, 60;
 *           `bytes` = size of buf, at least n x 4 MiB (else KLA_ERR_WORKSPACE).  aux unused.
 */
int kla_debug_peak_probe(int kind, void *buf, void *aux, size_t bytes, int iters, void *hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* KLA_H */
