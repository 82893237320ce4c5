/* cottn.h — C ABI of the cosine-attention (Cottention) library for MI355X (gfx950).
 *
 * Operation (paper notation: N(X) = row-wise L2 normalisation, Sec. 3.2; M = lower-triangular
 * ones including the diagonal, Sec. 4).  With Qh = N(Q), Kh = N(K) and a given positive
 * per-head scale s[h] (the stabiliser of Sec. 3.3 taken as a number):
 *
 *   causal         O = s_h * (Qh Kh^T (.) M) V                          (Sec. 4, eq. attn_1)
 *                  computed in linear memory as the cumulative sum of Kh^T V states
 *                  (Sec. 4, eq. attn_2), regrouped into chunks of `chunk` rows;
 *   bidirectional  O = s_h * Qh (Kh^T V)                                (Sec. 4, eq. subQuadCos)
 *   decode step    S <- S + kh^T v ;  o = s_h * qh S                    (Sec. 5, eq. hidden_state_obs)
 *   backward       the three gradient formulas of Sec. 4 followed by the chain rule through
 *                  the normalisation and the scale: gradients are with respect to the RAW
 *                  Q, K, V and to s.
 *
 * Conventions common to every entry point
 *   - All tensor arguments are DEVICE pointers, contiguous, row-major, innermost dimension d:
 *     Q, K, V, O, dO, dQ, dK, dV are [B][H][N][d]; q, k, v, o are [B][H][d]; s and ds are
 *     float[H]; states are float[B][H][d][d] laid out [d_key][d_value] = sum_j kh_j^T v_j
 *     and do NOT contain s (it is applied at read-out, so a state written by
 *     cottn_fwd_causal can be continued by cottn_step).
 *   - `dtype` is the storage type of Q, K, V, O, dO, dQ, dK, dV, q, k, v, o:
 *     COTTN_F32 (fp32 arithmetic), COTTN_BF16 or COTTN_F16 (16-bit MFMA operands, fp32
 *     accumulation, outputs rounded to nearest-even; with COTTN_F16 the operands the kernels
 *     keep in 16 bits, among them the running d x d state, must stay below 65504 in magnitude).
 *     s, ds, states and the workspace are always fp32.
 *   - Normalisation is x / max(||x||_2, eps); rows with ||x|| <= eps are x / eps.
 *   - The caller owns every buffer.  The library allocates nothing, frees nothing, never
 *     synchronises, and enqueues all work on `hip_stream` (a hipStream_t; NULL = the default
 *     stream).  Inputs are read-only; outputs are fully overwritten (ds is overwritten, not
 *     accumulated into).  Outputs must not alias inputs.
 *   - Base pointers of tensors must be 16-byte aligned; the workspace 256-byte aligned.
 *   - Supported shapes: d in {32, 64, 128}; B, H, N >= 1 (N == 0 is accepted and does
 *     nothing but define the outputs that do not depend on rows); chunk in {0, 64, 128, 256}
 *     for the 16-bit types (0 = library default, 64; d = 128 supports 64 only), and chunk in
 *     {0, 32} for fp32.
 *     N need not be a multiple of chunk.  64 is the tuned chunk size: 128 and 256 are exact
 *     and tested but slower in this design (more registers than two workgroups per compute
 *     unit leave a wave), and are kept for experiments with the state traffic.
 *   - The paper keeps two head dimensions apart (Sec. 2.1: d_H_key for queries and keys,
 *     d_H_value for values and outputs; its experiments use equal ones).  The entry points
 *     with one `d` take d_key = d_value = d; the *_dkdv entry points at the end of this header
 *     take both.
 *   - Return value: COTTN_OK or a cottn_status error code.  Argument errors are detected
 *     before anything is enqueued (so they can be exercised without a GPU); HIP launch
 *     failures return COTTN_E_HIP.  No entry point throws, aborts or prints.
 *   - Code shared between the passes: the backward has scan kernels of its own; what it
 *     shares with the forward is the kernel that reduces Kh^T V (or Qh^T dO) over a segment
 *     (the backward launches it only when it is not handed the forward's saved states), the
 *     tile staging / normalisation helpers and the small state-carry kernels.
 *   - `workspace` must hold at least cottn_workspace_bytes(op, ...) bytes for the same
 *     arguments; it may be NULL when that size is 0.  Its contents on entry are ignored
 *     and on exit unspecified.  Calls that share a workspace must be ordered on one stream.
 */
#ifndef COTTN_H
#define COTTN_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum { COTTN_F32 = 0, COTTN_BF16 = 1, COTTN_F16 = 2 } cottn_dtype;

typedef enum {
  COTTN_OK = 0,
  COTTN_E_NULL = 1,      /* a required pointer is NULL */
  COTTN_E_SHAPE = 2,     /* B, H, N, d or chunk outside the supported set */
  COTTN_E_DTYPE = 3,     /* dtype is none of COTTN_F32, COTTN_BF16, COTTN_F16 */
  COTTN_E_ALIGN = 4,     /* a pointer is not aligned as required */
  COTTN_E_WORKSPACE = 5, /* workspace NULL or smaller than cottn_workspace_bytes() */
  COTTN_E_HIP = 6,       /* a HIP call failed (launch error) */
  COTTN_E_ARG = 7        /* any other invalid argument (eps <= 0, unknown op, ...) */
} cottn_status;

typedef enum {
  COTTN_OP_FWD_CAUSAL = 0,
  COTTN_OP_BWD_CAUSAL = 1,
  COTTN_OP_FWD_BIDIR = 2,
  COTTN_OP_BWD_BIDIR = 3,
  COTTN_OP_STEP = 4
} cottn_op;

/* Bytes of workspace the given operation needs for these arguments (0 for COTTN_OP_STEP).
 * Returns (size_t)-1 if the arguments are not supported.  Host only; touches no GPU. */
size_t cottn_workspace_bytes(int op, int B, int H, int N, int d, int chunk, int dtype);

/* Number of sequence segments per (batch, head) the library will scan in parallel for
 * these arguments (1 = one serial chunk scan per (b, h)); 0 if unsupported.  Informational:
 * the chunked regrouping of the cumulative sum of eq. attn_2 is exact for any value.
 * cottn_tune_segments(g) forces the value for later calls made by the CALLING THREAD (g <= 0
 * restores the built-in heuristic); it is a knob for tests and tuning runs and the only state
 * the library keeps between calls besides the profiling totals below.  A backward call that is
 * handed a forward's workspace assumes the split it computes itself: do not change the tuning
 * between a forward call and the backward call that takes its workspace (the states would be
 * read in another layout: wrong gradients, no error). */
int cottn_segments(int op, int B, int H, int N, int d, int chunk, int dtype);
void cottn_tune_segments(int segments);

/* Static, NUL-terminated description of a status code. */
const char* cottn_status_string(int status);

/* Causal forward (Sec. 4, eq. attn_1 / attn_2).
 *   Q, K, V [B][H][N][d] in, s [H] in, O [B][H][N][d] out.
 *   state: NULL, or float[B][H][d][d] out = sum over all N rows of kh^T v (Sec. 5's hidden
 *   state after the last token, transposed to [d_key][d_value], without s). */
int cottn_fwd_causal(const void* Q, const void* K, const void* V, const float* s, void* O,
                     float* state, void* workspace, size_t workspace_bytes, int B, int H, int N,
                     int d, int chunk, int dtype, float eps, void* hip_stream);

/* cottn_fwd_causal for callers that cannot allocate device memory and have no workspace to
 * hand over: code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  Same arguments, results and errors as cottn_fwd_causal without the two workspace
 * arguments: the segment states live in a COTTN_STATIC_WORKSPACE_BYTES array inside the
 * library's own device code (each GPU the library runs on holds it until the process ends).
 * Shapes whose cottn_workspace_bytes(COTTN_OP_FWD_CAUSAL, ...) exceeds that size are rejected
 * with COTTN_E_WORKSPACE before anything is enqueued.  The call allocates and frees nothing
 * (the array's address is looked up once per device, on the first call with that device
 * current; hip_stream must belong to the current device).  Every call on a GPU uses that
 * GPU's one array: calls that may overlap on one GPU (different streams, different threads)
 * race on it and must be ordered by the caller.  Nothing in the array has to be cleared
 * between calls. */
#define COTTN_STATIC_WORKSPACE_BYTES (16u << 20)
int cottn_fwd_causal_static(const void* Q, const void* K, const void* V, const float* s, void* O,
                            float* state, int B, int H, int N, int d, int chunk, int dtype,
                            float eps, void* hip_stream);

/* The same for a sequence that continues an earlier one (a long prompt fed in pieces, Sec. 5:
 * the hidden state carries everything the later tokens need from the earlier ones).
 *   state_in: float[B][H][d][d] in, the state after the tokens before this piece (what an
 *   earlier call left in `state`, or cottn_step's state); O_i = s qh_i (state_in + sum_{j<=i}
 *   kh_j^T v_j) and `state` (may be NULL) receives state_in + the sum over this piece.
 *   state_in and state must not be the same buffer (COTTN_E_ARG): workgroups read the one
 *   while others write the other.  N = 0 copies state_in to state.  With a small N this is
 *   also a several-token decode step: it gives what N calls of cottn_step give. */
int cottn_fwd_causal_from_state(const void* Q, const void* K, const void* V, const float* s,
                                const float* state_in, void* O, float* state, void* workspace,
                                size_t workspace_bytes, int B, int H, int N, int d, int chunk,
                                int dtype, float eps, void* hip_stream);

/* Causal backward (Sec. 4, gradient formulas; dK and dV use the cumulative sum that runs
 * backward in time).  Takes the raw Q, K, V of the forward call and dO = dL/dO; writes
 * dQ, dK, dV (same shape and dtype) and ds[H] = dL/ds (overwritten).
 *   fwd_workspace: NULL, or the workspace that a completed cottn_fwd_causal call with the same
 *   K, V, B, H, N, d, chunk, dtype and eps used, untouched since (device pointer, read only,
 *   fwd_workspace_bytes as passed there).  It holds the forward-time segment states of
 *   Kh^T V, which the backward needs again: given them it does not rebuild them from K and V.
 *   They are taken over only for the 16-bit types and when forward and backward split the sequence
 *   the same way (cottn_segments agrees for both ops); otherwise the argument is ignored.
 *   Contents that do not come from such a call give wrong gradients, not an error. */
int cottn_bwd_causal(const void* Q, const void* K, const void* V, const float* s, const void* dO,
                     void* dQ, void* dK, void* dV, float* ds, const void* fwd_workspace,
                     size_t fwd_workspace_bytes, void* workspace, size_t workspace_bytes, int B,
                     int H, int N, int d, int chunk, int dtype, float eps, void* hip_stream);

/* The causal backward for one piece of a sequence that is processed in pieces (a sequence too
 * long for one call, or cut across devices).  The two cumulative sums of Sec. 4 cross the
 * piece boundaries as d x d states: the pieces' forward calls run first to last handing on
 * `state` (cottn_fwd_causal_from_state); their backward calls run last to first handing on
 * the reverse-time state.  All states are float[B][H][d][d], [d_key][d_value], without s.
 *   state_in:      NULL (nothing precedes) or sum of kh_j^T v_j over the rows BEFORE this
 *                  piece: the state_in its forward call was given.
 *   rev_state_in:  NULL (nothing follows) or sum of qh_i^T dO_i over the rows AFTER this
 *                  piece: the rev_state_out of the following piece's backward call.
 *   rev_state_out: NULL or out, rev_state_in + the sum over this piece; must not be the same
 *                  buffer as rev_state_in (COTTN_E_ARG).
 * dQ, dK, dV are the gradients of this piece's rows given all pieces; ds[H] is this piece's
 * share of dL/ds (the caller adds the shares up).  fwd_workspace as in cottn_bwd_causal: that
 * of the piece's own forward call.  N = 0 sets ds to zero and copies rev_state_in to
 * rev_state_out (zeros without rev_state_in).  Chained over the pieces this gives exactly what
 * one call over the whole sequence gives. */
int cottn_bwd_causal_from_state(const void* Q, const void* K, const void* V, const float* s,
                                const void* dO, const float* state_in, const float* rev_state_in,
                                void* dQ, void* dK, void* dV, float* ds, float* rev_state_out,
                                const void* fwd_workspace, size_t fwd_workspace_bytes,
                                void* workspace, size_t workspace_bytes, int B, int H, int N, int d,
                                int chunk, int dtype, float eps, void* hip_stream);

/* Bidirectional forward (Sec. 4, eq. subQuadCos, right-hand side).
 *   state: NULL, or float[B][H][d][d] out = Kh^T V. */
int cottn_fwd_bidir(const void* Q, const void* K, const void* V, const float* s, void* O,
                    float* state, void* workspace, size_t workspace_bytes, int B, int H, int N,
                    int d, int dtype, float eps, void* hip_stream);

/* Bidirectional backward: gradients of cottn_fwd_bidir with respect to raw Q, K, V and s
 * (the gradient formulas of Sec. 4 with the mask M removed).
 *   fwd_workspace: NULL, or the workspace of the matching completed cottn_fwd_bidir call,
 *   untouched since (same rules as for cottn_bwd_causal): it holds the segment totals of
 *   Kh^T V, which the backward then does not reduce again.  Taken over for bfloat16 and a
 *   split into few segments; otherwise ignored. */
int cottn_bwd_bidir(const void* Q, const void* K, const void* V, const float* s, const void* dO,
                    void* dQ, void* dK, void* dV, float* ds, const void* fwd_workspace,
                    size_t fwd_workspace_bytes, void* workspace, size_t workspace_bytes, int B,
                    int H, int N, int d, int dtype, float eps, void* hip_stream);

/* Padded batches: sequences of different lengths in one [B][H][N][d] tensor (Sec. 4 notes that
 * padding is masked by zeroing rows).  seq_len: int[B] device pointer, 0 <= seq_len[b] <= N
 * (values outside are clamped).  Rows at or beyond seq_len[b] do not exist: they are not read,
 * take part in no sum, and those rows of O, dQ, dK, dV are written as zeros.  Because the
 * stabiliser of Sec. 3.3 depends on each sequence's own length, the scale is one value per
 * (batch, head) here: s is float[B][H] and ds is float[B][H].  Everything else (state,
 * workspaces, fwd_workspace, errors) is as for the functions without the suffix;
 * cottn_workspace_bytes is the same. */
int cottn_fwd_causal_varlen(const void* Q, const void* K, const void* V, const float* s,
                            const int* seq_len, void* O, float* state, void* workspace,
                            size_t workspace_bytes, int B, int H, int N, int d, int chunk,
                            int dtype, float eps, void* hip_stream);
int cottn_bwd_causal_varlen(const void* Q, const void* K, const void* V, const float* s,
                            const int* seq_len, const void* dO, void* dQ, void* dK, void* dV,
                            float* ds, const void* fwd_workspace, size_t fwd_workspace_bytes,
                            void* workspace, size_t workspace_bytes, int B, int H, int N, int d,
                            int chunk, int dtype, float eps, void* hip_stream);
int cottn_fwd_bidir_varlen(const void* Q, const void* K, const void* V, const float* s,
                           const int* seq_len, void* O, float* state, void* workspace,
                           size_t workspace_bytes, int B, int H, int N, int d, int dtype, float eps,
                           void* hip_stream);
int cottn_bwd_bidir_varlen(const void* Q, const void* K, const void* V, const float* s,
                           const int* seq_len, const void* dO, void* dQ, void* dK, void* dV,
                           float* ds, const void* fwd_workspace, size_t fwd_workspace_bytes,
                           void* workspace, size_t workspace_bytes, int B, int H, int N, int d,
                           int dtype, float eps, void* hip_stream);

/* One recurrent decode step for B*H independent states (Sec. 5, eq. hidden_state_obs):
 *   state[b][h] += kh^T v  (in place), then  o[b][h] = s_h * qh state[b][h]
 * (the state is read AFTER the update).  q, k, v, o are [B][H][d] in `dtype`. */
int cottn_step(const void* q, const void* k, const void* v, const float* s, float* state,
               void* o, int B, int H, int d, int dtype, float eps, void* hip_stream);

/* ---- d_key != d_value (Sec. 2.1: d_H_key, d_H_value) ----------------------------------------
 * The same operations with queries and keys of dk features and values of dv features:
 *   Q, K, dQ, dK are [B][H][N][dk];  V, O, dO, dV are [B][H][N][dv];  q, k are [B][H][dk] and
 *   v, o [B][H][dv];  every state is float[B][H][dk][dv] = sum_j kh_j^T v_j.
 * dk and dv are each one of 32, 64, 128.  With dk == dv these calls are the ones above.  With
 * dk != dv: every dtype; chunk 0 or 64 for the 16-bit types (0 or 32 for fp32, as always).
 * Everything else (workspaces, fwd_workspace, errors, conventions) is as for the functions
 * without the suffix; sizes and splits come from the *_dkdv variants of the two queries. */
size_t cottn_workspace_bytes_dkdv(int op, int B, int H, int N, int dk, int dv, int chunk,
                                  int dtype);
int cottn_segments_dkdv(int op, int B, int H, int N, int dk, int dv, int chunk, int dtype);
int cottn_fwd_causal_dkdv(const void* Q, const void* K, const void* V, const float* s, void* O,
                          float* state, void* workspace, size_t workspace_bytes, int B, int H,
                          int N, int dk, int dv, int chunk, int dtype, float eps, void* hip_stream);
int cottn_bwd_causal_dkdv(const void* Q, const void* K, const void* V, const float* s,
                          const void* dO, void* dQ, void* dK, void* dV, float* ds,
                          const void* fwd_workspace, size_t fwd_workspace_bytes, void* workspace,
                          size_t workspace_bytes, int B, int H, int N, int dk, int dv, int chunk,
                          int dtype, float eps, void* hip_stream);
int cottn_fwd_bidir_dkdv(const void* Q, const void* K, const void* V, const float* s, void* O,
                         float* state, void* workspace, size_t workspace_bytes, int B, int H, int N,
                         int dk, int dv, int dtype, float eps, void* hip_stream);
int cottn_bwd_bidir_dkdv(const void* Q, const void* K, const void* V, const float* s,
                         const void* dO, void* dQ, void* dK, void* dV, float* ds,
                         const void* fwd_workspace, size_t fwd_workspace_bytes, void* workspace,
                         size_t workspace_bytes, int B, int H, int N, int dk, int dv, int dtype,
                         float eps, void* hip_stream);
int cottn_step_dkdv(const void* q, const void* k, const void* v, const float* s, float* state,
                    void* o, int B, int H, int dk, int dv, int dtype, float eps, void* hip_stream);

/* The learned stabiliser of Sec. 3.3 (eq. cosine2): scores are divided by n^sigma(m_h), n the
 * sequence length, m_h a learned scalar per head (the paper starts it at 0.5).  The entry
 * points above take the factor itself; these map between the two.  m, s, ds, dm: float[H]
 * device pointers; n >= 1.
 *   cottn_scale_from_m:   s[h]  = n^(-sigma(m[h]))
 *   cottn_scale_backward: dm[h] = ds[h] * ds_h/dm_h
 *                               = ds[h] * (-ln n) sigma(m[h]) (1 - sigma(m[h])) n^(-sigma(m[h]))
 * Outputs are overwritten.  Errors: COTTN_E_NULL, COTTN_E_SHAPE (H < 1), COTTN_E_ARG (n < 1 or
 * not finite), COTTN_E_ALIGN (pointers not 4-byte aligned), COTTN_E_HIP. */
int cottn_scale_from_m(const float* m, float* s, int H, float n, void* hip_stream);
int cottn_scale_backward(const float* m, const float* ds, float* dm, int H, float n,
                         void* hip_stream);
/* The same for a padded batch: n is each sequence's own length (a length below 1 counts as 1).
 *   s[b][h] = seq_len[b]^(-sigma(m[h]));   dm[h] = sum over b of ds[b][h] * ds_bh/dm_h. */
int cottn_scale_from_m_varlen(const float* m, const int* seq_len, float* s, int B, int H,
                              void* hip_stream);
int cottn_scale_backward_varlen(const float* m, const int* seq_len, const float* ds, float* dm,
                                int B, int H, void* hip_stream);

/* Per-kernel timing for benchmarks.  After cottn_profile_start(), every kernel the library
 * launches carries two HIP events of its own (attached to the dispatch, so they mark the
 * kernel's begin and end, not the gaps between launches); cottn_profile_stop() waits for
 * those events, adds each kernel's elapsed time to a per-kernel-name total and stops
 * recording.  The three getters read the totals gathered by the last start/stop pair:
 * cottn_profile_count() distinct kernel names, and for 0 <= i < count its name (static
 * storage), number of launches and summed duration in milliseconds.  Profiling adds the
 * cost of the event records (and their creation) to every launch; it is off by default.
 * Process-wide and not thread-safe: use it from one thread, with no other thread inside the
 * library. */
int cottn_profile_start(void);
int cottn_profile_stop(void);
int cottn_profile_count(void);
const char* cottn_profile_name(int i);
long cottn_profile_launches(int i);
double cottn_profile_ms(int i);

#ifdef __cplusplus
}
#endif
#endif /* COTTN_H */
