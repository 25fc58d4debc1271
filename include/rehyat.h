/*
 * rehyat.h -- C ABI of the MI355X (gfx950) Recurrent Hybrid Attention library.
 *
 * The operator is the hybrid attention of the ReHyAt paper, section 3.2
 * (Eq. 5-9: softmax attention inside a temporal chunk and kernelised linear
 * attention through learned feature maps phi_q, phi_k outside it, under one
 * joint normaliser), in its causal chunk-recurrent form of section 3.3
 * (Eq. 13-18: the linear part is read from a running state S = sum phi_k(k) v^T,
 * z = sum phi_k(k) over the tokens that have left the softmax window).
 *
 * Conventions shared by every entry point
 *  - Return value: REHYAT_OK (0) or a negative REHYAT_E_* code.  On a
 *    validation error nothing is launched and `out` is not written.  No
 *    exception or abort crosses this boundary.
 *  - q, k, v, out, the phi tensors and the workspace are DEVICE pointers owned
 *    by the caller; the library never frees or retains them beyond the call
 *    (the workspace pointer given to rehyat_set_workspace is retained until it
 *    is replaced or rehyat_shutdown is called).
 *  - Work is enqueued on `stream` (a hipStream_t passed as void*; NULL is the
 *    default stream) and the call returns without synchronising.
 *  - Tensors are contiguous, row-major, bf16 (IEEE bfloat16 bit patterns)
 *    unless stated otherwise.  Token index inside a head is
 *    frame * HW + position, frame-major, as in section 3.2's flattening of the
 *    (T, H, W) latent.
 *  - Alignment: q, k, v, out and the phi weight matrices must be 16-byte
 *    aligned (rows are moved 16 bytes at a time), fp32 tensors 4-byte aligned,
 *    a workspace 256-byte aligned; otherwise REHYAT_E_SHAPE (REHYAT_E_WORKSPACE
 *    for a workspace).
 *  - Results are deterministic: repeated calls give bit-identical outputs.
 *  - Calls that share a workspace must be ordered on one stream.  Entry points
 *    without a workspace argument share the one the library holds and are
 *    serialised by an internal lock; rehyat_forward_ws takes its workspace per
 *    call and may run concurrently with any other call on any stream as long as
 *    the workspaces differ.
 */
#ifndef REHYAT_H_
#define REHYAT_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define REHYAT_OK 0
#define REHYAT_E_NULL (-1)        /* a required pointer is NULL */
#define REHYAT_E_SHAPE (-2)       /* a size is non-positive or inconsistent, or a pointer misaligned */
#define REHYAT_E_UNSUPPORTED (-3) /* valid in the paper, not built here */
#define REHYAT_E_WORKSPACE (-4)   /* workspace missing, too small or misaligned */
#define REHYAT_E_HIP (-5)         /* a HIP runtime call failed */

/* Stabiliser c of Eq. 6 and Eq. 8.  The linear terms of Eq. 7 and 9 are not
 * rescaled by exp(-c), so the choice is part of the operator's definition. */
#define REHYAT_STAB_ROWMAX 0 /* c = largest exponent of the query row */
#define REHYAT_STAB_NONE 1   /* c = 0 (evaluated without overflow) */

/*
 * Feature maps phi_q and phi_k (section 3.2, "Characterization of phi";
 * appendix "Training Details": a two-layer per-head MLP followed by a split
 * into `degree` equal parts, part p raised element-wise to the power p):
 *   u = relu(W1 x + b1),  psi = relu(W2 u + b2),
 *   phi(x) = [psi[0 : D'/2], psi[D'/2 : D']^2]          (degree 2)
 * The struct lives in HOST memory; its pointer fields are DEVICE pointers:
 *   w1_* [H, hidden, d] bf16     b1_* [H, hidden] fp32
 *   w2_* [H, dprime, hidden] bf16  b2_* [H, dprime] fp32
 * Supported here: hidden == dprime == 2*d, degree == 2, act == 0 (ReLU).
 */
typedef struct {
  const void *w1_q, *b1_q, *w2_q, *b2_q;
  const void *w1_k, *b1_k, *w2_k, *b2_k;
  int32_t hidden;
  int32_t dprime;
  int32_t degree;
  int32_t act;
} rehyat_phi_params;

/*
 * Optional per-row components of Eq. 5-9 (test hook).  HOST struct of DEVICE
 * pointers, each nullable, all fp32:
 *   m  [B,H,N]    largest softmax exponent q_i.k_j/sqrt(d) of the row
 *   nS [B,H,N]    Eq. 8      aS [B,H,N,d]  Eq. 6   (both relative to exp(-m))
 *   nL [B,H,N]    Eq. 9      aL [B,H,N,d]  Eq. 7
 * With REHYAT_STAB_NONE, nL and aL are reported multiplied by exp(-m), the
 * scale on which they are merged with nS and aS.
 */
typedef struct {
  float *m, *nS, *aS, *nL, *aL;
} rehyat_debug_out;

/*
 * Chunk bookkeeping on the host (section 3.2 token layout; Eq. 12; Eq. 13).
 * Writes n_chunks = ceil(T / chunk) rows of five int64 to `table` (HOST
 * memory, may be NULL to query the count only):
 *   q_lo, q_hi : query token range of the chunk
 *   s_lo, s_hi : softmax window [max(q_lo - overlap*HW, 0), q_hi)
 *   l_hi       : the causal linear set is [0, l_hi), l_hi == s_lo
 * The kernels derive their ranges from the same formulas.
 * Errors: REHYAT_E_NULL (n_chunks NULL), REHYAT_E_SHAPE.
 */
int rehyat_chunk_plan(int T, int HW, int chunk, int overlap, int64_t *table,
                      int *n_chunks);

/*
 * Bytes of device workspace a forward call needs: chunk-state partial sums,
 * their prefix (the states S_t, z_t of Eq. 16) and the carry between windows
 * of chunks.  Depends on B, H, d and dprime only -- not on T, HW or chunk --
 * which is the constant-memory property of section 3.3, point (3).
 * Returns 0 for unsupported sizes.
 */
size_t rehyat_workspace_bytes(int B, int H, int d, int dprime);

/*
 * Give the library a caller-owned DEVICE workspace (256-byte aligned) for the
 * entry points that take none.  It is never replaced behind the caller's back:
 * a call that needs more than `bytes` returns REHYAT_E_WORKSPACE and launches
 * nothing.  Pass (NULL, 0) to return to library-owned memory: the library then
 * allocates with hipMalloc on first need, grows (free + allocate) when a later
 * call needs more, and keeps the buffer until rehyat_shutdown().  Growth
 * invalidates HIP graphs captured from earlier calls; while `stream` is being
 * captured the library neither allocates nor frees and returns
 * REHYAT_E_WORKSPACE instead -- size the workspace (one eager call, or
 * rehyat_set_workspace) before capturing.
 */
int rehyat_set_workspace(void *dev_ptr, size_t bytes);

/*
 * Hybrid attention forward (Eq. 5-9 with the causal sets of Eq. 13, evaluated
 * chunk-wise as Eq. 14-18), T_o = 0, row-max stabiliser.
 *   q, k, v : [B, H, N, d] bf16, N = T*HW        out : [B, H, N, d] bf16
 *   phi_params : HOST pointer (see above)
 *   T   latent frames, HW tokens per frame, chunk = T_c frames per chunk
 *       (a short last chunk when T % chunk != 0; chunk >= T is one chunk,
 *       i.e. plain softmax attention, Eq. 2)
 * Supported: d in {64, 128}; B*H <= 65535; N < 2^31; one softmax window
 * ((chunk + overlap) * HW tokens) below 2^31 bytes per head; anything beyond
 * returns REHYAT_E_SHAPE.
 */
int rehyat_forward(const void *q, const void *k, const void *v,
                   const rehyat_phi_params *phi_params, void *out, int B, int H,
                   int T, int HW, int d, int chunk, void *stream);

/*
 * Same operator with the remaining knobs of the paper:
 *   overlap   : T_o latent frames by which the softmax window reaches back
 *               (Eq. 12); the state then lags by the same amount (Eq. 13)
 *   causal    : 1 = Eq. 13.  0 = the bidirectional sets of Eq. 11-12: the
 *               linear part of chunk t covers every token outside its softmax
 *               window, before and after (the whole K, V are read before the
 *               first output; REHYAT_E_UNSUPPORTED if min(chunk + overlap, T)
 *               exceeds 64 frames)
 *   stab_mode : REHYAT_STAB_ROWMAX or REHYAT_STAB_NONE
 *   debug     : NULL, or HOST pointer to the component outputs
 */
int rehyat_forward_ex(const void *q, const void *k, const void *v,
                      const rehyat_phi_params *phi_params, void *out, int B,
                      int H, int T, int HW, int d, int chunk, int overlap,
                      int causal, int stab_mode, const rehyat_debug_out *debug,
                      void *stream);

/*
 * rehyat_forward_ex with the workspace passed per call (no debug outputs):
 * `workspace` is a DEVICE pointer, 256-byte aligned, of at least
 * rehyat_workspace_bytes(B, H, d, dprime) bytes, used only for the duration of
 * the enqueued work and not retained.  No library state is read or written, so
 * two streams, two layers or the two halves of a guidance pair can be in flight
 * at once, each with its own workspace (section 3.3 gives every sequence its
 * own running state).  Errors as rehyat_forward_ex, plus REHYAT_E_NULL
 * (workspace NULL) and REHYAT_E_WORKSPACE (misaligned or too small).
 */
int rehyat_forward_ws(const void *q, const void *k, const void *v,
                      const rehyat_phi_params *phi_params, void *out, int B,
                      int H, int T, int HW, int d, int chunk, int overlap,
                      int causal, int stab_mode, void *workspace,
                      size_t workspace_bytes, void *stream);

/*
 * rehyat_forward for callers that cannot allocate device memory (code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc):
 * same arguments, same kernels, same result as rehyat_forward, but chunk-state
 * partial sums, chunk states and the carry live in a fixed array of
 * REHYAT_NOALLOC_SCRATCH_BYTES (64 MiB) that is part of the library's device
 * image -- each GPU the library runs on holds it until the process ends --
 * and the call performs no hipMalloc / hipFree and no allocating library
 * routine.  The first call on each device looks the array's address up (the
 * HIP runtime loads that part of the device image then): make that one call
 * eagerly, outside any capture.  The chunks are processed in windows of as many chunk states
 * as fit the array (27 per window at B*H = 12, d = 128; at least one), so larger
 * B*H costs more, shorter launches; when not even one state per (b, h) fits
 * (B*H above 202 at d = 128) the call returns REHYAT_E_WORKSPACE and launches
 * nothing.  Nothing has to be cleared between calls: every element a kernel
 * reads is written earlier in the same call.  All calls on one GPU share that
 * GPU's array: calls that overlap in time on one GPU race (order them on one
 * stream); the internal lock only serialises the host side.
 */
#define REHYAT_NOALLOC_SCRATCH_BYTES ((size_t)64 << 20)
int rehyat_forward_noalloc(const void *q, const void *k, const void *v,
                           const rehyat_phi_params *phi_params, void *out,
                           int B, int H, int T, int HW, int d, int chunk,
                           void *stream);

/*
 * Gradient of a loss with respect to the parameters of the two feature maps,
 * for one step of the attention distillation of section 3.4 (Eq. 19), which
 * trains phi_q and phi_k of a block and nothing else:
 *     phi <- phi - eta * grad_phi E | y - y_hat |.
 * The caller supplies G = dL/dy_hat (for the L1 loss of Eq. 19,
 * sign(y_hat - y) / count); the call recomputes the forward pass (Eq. 5-9,
 * causal sets of Eq. 13, stabiliser REHYAT_STAB_ROWMAX, under which the softmax
 * terms do not depend on phi) and applies the chain rule through the linear
 * terms (Eq. 7, 9, 14-18) and the two-layer map with its degree-2 polynomial
 * features ("Characterization of phi").
 *
 *   q, k, v, phi_params, B, H, T, HW, d, chunk, overlap : as rehyat_forward_ex
 *   grad_out  [B, H, N, d] bf16 DEVICE  G
 *   out       [B, H, N, d] bf16 DEVICE.  With saved == NULL: nullable, receives
 *             y_hat of the recomputed forward pass.  With saved != NULL: input,
 *             y_hat as rehyat_forward_ex wrote it for the same arguments.
 *   saved     HOST struct, nullable.  A distillation step has already run the
 *             forward pass to form the loss; passing what it produced -- `out`
 *             and the components nS, nL [B, H, N] fp32 (DEVICE) of
 *             rehyat_debug_out, stabiliser REHYAT_STAB_ROWMAX -- skips the
 *             fused attention kernel here (the chunk states are still rebuilt:
 *             the forward workspace does not keep them).  NULL recomputes
 *             everything.
 *   grads     HOST struct of DEVICE pointers, fp32, same shapes as the
 *             parameters ([H, hidden, d], [H, hidden], [H, dprime, hidden],
 *             [H, dprime] for each map), summed over the batch; overwritten
 *   workspace DEVICE, 256-byte aligned, at least
 *             rehyat_phi_backward_workspace_bytes(...) bytes.  Unlike the
 *             forward workspace it grows with N: y_hat, dL/dy_hat / den and
 *             the gradient of the second layer's pre-activations are kept
 *             token by token (about 1 KB per token and head at d = 128), beside
 *             the per-workgroup partial sums of the weight gradients (about
 *             0.2 GB at d = 128 whenever B*H does not exceed 256).  Used only
 *             for the duration of the enqueued work; no library state is
 *             touched.
 *
 * Sums over tokens run in a fixed order: results are bit-reproducible.
 * Supported: d in {64, 128}, hidden = dprime = 2 d, degree 2, at most
 * REHYAT_BACKWARD_MAX_CHUNKS chunks (else REHYAT_E_UNSUPPORTED), N below
 * 2^31 / (4 d).  One chunk (chunk >= T) gives all-zero gradients.
 * rehyat_phi_backward_workspace_bytes returns 0 for sizes the call rejects.
 * Errors: as rehyat_forward_ex, plus REHYAT_E_NULL (grad_out, grads, one of its
 * pointers, workspace, or -- with saved -- out, nS or nL NULL) and
 * REHYAT_E_WORKSPACE.
 */
#define REHYAT_BACKWARD_MAX_CHUNKS 1024
typedef struct {
  void *w1_q, *b1_q, *w2_q, *b2_q;
  void *w1_k, *b1_k, *w2_k, *b2_k;
} rehyat_phi_grads;
typedef struct {
  const float *nS, *nL;
} rehyat_forward_saved;
size_t rehyat_phi_backward_workspace_bytes(int B, int H, int T, int HW, int d,
                                           int chunk);
int rehyat_phi_backward(const void *q, const void *k, const void *v,
                        const rehyat_phi_params *phi_params,
                        const void *grad_out, void *out,
                        const rehyat_forward_saved *saved,
                        const rehyat_phi_grads *grads, int B, int H, int T,
                        int HW, int d, int chunk, int overlap, void *workspace,
                        size_t workspace_bytes, void *stream);

/*
 * One step of the chunk-wise RNN (section 3.3, Eq. 14-18) for generation chunk by
 * chunk: the caller owns the state and the K/V window, the library holds nothing
 * between calls, and peak memory does not depend on how many chunks came before.
 *
 *   q_t           [B, H, n_q, d]    bf16 DEVICE  queries of the current chunk
 *   k_win, v_win  [B, H, n_win, d]  bf16 DEVICE  the softmax window T^S_t of
 *                 Eq. 12, oldest token first: the T_o overlap frames kept from
 *                 earlier chunks, then the current chunk's own tokens
 *   S [B, H, dprime, d] fp32, z [B, H, dprime] fp32  DEVICE, read and written:
 *                 on entry the sums of Eq. 14-15 over every token older than the
 *                 window (all zero before the first chunk); the read-out of
 *                 Eq. 16 uses these values.  On return the first n_absorb
 *                 tokens of the window have been added (Eq. 17-18): the tokens
 *                 that are no longer inside the next chunk's window.
 *   out_t         [B, H, n_q, d]    bf16 DEVICE  y of Eq. 5-9 for the chunk
 *   n_absorb      0 <= n_absorb <= n_win
 *   stab_mode     REHYAT_STAB_ROWMAX or REHYAT_STAB_NONE
 *
 * Feeding the chunks of a sequence in order, with the windows and n_absorb =
 * s_lo(t+1) - s_lo(t) of rehyat_chunk_plan, gives the outputs of
 * rehyat_forward_ex (same overlap) up to the rounding of a different summation
 * split.  Asynchronous on `stream`; uses the workspace like a forward call.
 * The state update (the pieces of Eq. 17-18 and their addition to S and z) does
 * not feed this chunk's output, so it runs beside the attention kernel on a
 * second stream that the library creates per device on first use (default
 * priority, kept until the process ends), forked from `stream` after the state
 * has been copied for the read-out and joined to it before the call's work on
 * `stream` is complete: to the caller the call is ordered on `stream` like any
 * other, also under stream capture (fork and join become graph edges).  When
 * the first call on a device happens while `stream` is being captured, nothing
 * is created and the update runs on `stream` itself.
 * Supported: d in {64, 128}.
 */
int rehyat_step(const void *q_t, const void *k_win, const void *v_win,
                const rehyat_phi_params *phi_params, float *S, float *z,
                void *out_t, int B, int H, int d, int n_q, int n_win,
                int n_absorb, int stab_mode, void *stream);

/*
 * Running state of the chunk-wise RNN (Eq. 14-15, 17-18) after absorbing
 * tokens [0, upto) of every head, as the state kernels compute it:
 *   S_out [B, H, dprime, d] fp32,  z_out [B, H, dprime] fp32  (DEVICE)
 * `upto` must be a multiple of HW.  Test hook for the state and prefix
 * kernels; uses the workspace like a forward call.
 */
int rehyat_state(const void *k, const void *v,
                 const rehyat_phi_params *phi_params, float *S_out, float *z_out,
                 int B, int H, int T, int HW, int d, int upto_frames,
                 void *stream);

/*
 * Per-kernel timing for benchmarks.  While enabled, every kernel launch of a
 * forward call is bracketed by HIP events recorded on the call's stream (the
 * only stream on which the launch's duration can be observed).  Up to 4096
 * launches are kept between reads; later ones are not timed.
 * rehyat_profile_read waits for the recorded events, then returns for each
 * kernel kind (0 = chunk state, 1 = prefix, 2 = fused attention) the summed
 * duration in milliseconds and the number of launches since the last read or
 * enable, in HOST arrays of three elements each, and clears the record.
 */
int rehyat_profile_enable(int on);
int rehyat_profile_read(double *total_ms, int *launches);

/*
 * Measurement hook, timing only.  The hardware deals the workgroups of a launch
 * round-robin to the chip's eight XCDs (workgroup index modulo 8).  With bit x of
 * `mask` clear, the attention kernel's workgroups on XCD x exit at once and
 * their rows of `out` are NOT written; the other XCDs do exactly their usual
 * share.  Timing such launches against full ones shows how much the work of one
 * XCD is slowed by activity on the others.  The mask is process-wide and stays
 * until changed; 0xFF (the default) is normal operation.  Bits above the low
 * eight are ignored; a mask with no low bit set is REHYAT_E_SHAPE.
 */
int rehyat_debug_set_xcd_mask(unsigned mask);

/* Free library-owned device memory.  Safe to call more than once. */
int rehyat_shutdown(void);

/* Static string for a status code. */
const char *rehyat_status_string(int code);

/* Library version: major * 10000 + minor * 100 + patch. */
int rehyat_version(void);

/* Name of the fused attention kernel instance launched for head width d, as a
 * profiler's kernel trace shows it ("" for an unsupported d). */
const char *rehyat_attn_kernel_name(int d);

/* Text of the last HIP error seen by this library ("" if none). */
const char *rehyat_last_hip_error(void);

#ifdef __cplusplus
}
#endif
#endif /* REHYAT_H_ */
