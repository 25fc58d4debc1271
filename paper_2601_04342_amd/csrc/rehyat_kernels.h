// Internal launch interfaces between the C-ABI host layer and the kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "rehyat_device.h"

namespace rehyat {

// ---- chunk-state kernel: partial sums of phi_k(K)^T V and phi_k(K) ----------
// Segment s of a window is the token range that enters the linear set between
// chunk (chunk0 + s) and the next one, [s_lo(chunk0+s), s_lo(chunk0+s+1))
// (Eq. 13, Eq. 17-18); each segment is cut into `nsplit` pieces, one workgroup
// per (batch*head, segment, piece).
struct StateArgs {
  const bf16_t* k;      // [BH, N, d]
  const bf16_t* v;      // [BH, N, d]
  const bf16_t* w1_k;   // [H, hidden, d]
  const float* b1_k;    // [H, hidden]
  const bf16_t* w2_k;   // [H, dprime, hidden]
  const float* b2_k;    // [H, dprime]
  float* partial;       // [BH, partial_slots, d*dprime + dprime] (S^T [d][dprime], then z)
  int H, T, HW, chunk, overlap;
  int chunk0;           // first chunk of the window
  int n_seg;            // segments computed in this launch
  int nsplit;           // pieces per segment
  int partial_slots;    // slot stride per (b, h)
  int n_items;          // BH * n_seg * nsplit
  int items_per_xcd;
  int64_t kv_bh_stride; // elements between the k (and v) rows of consecutive (b, h)
  int step_n;           // > 0: one segment, rows [0, step_n) of k / v (streaming step); the
                        // frame geometry above is then unused
  int query_segments;   // 1: segment s is the query range [q_lo, q_hi) of chunk chunk0 + s
                        // (the sums of phi_q(q) u^T behind the gradient of the chunk state)
};

// ---- prefix kernel: states S_t, z_t of the window's chunks ---------------------
struct PrefixArgs {
  const float* partial;  // as written by the state kernel
  float* carry;          // [BH, d*dprime + dprime] fp32, state at the window's first chunk
  bf16_t* state_s;       // [BH, state_slots, d, dprime] bf16 (S_t transposed)
  float* state_z;        // [BH, state_slots, dprime]
  int BH;
  int n_chunks;          // chunks in the window (states written)
  int n_seg;             // segments available (n_chunks or n_chunks - 1)
  int nsplit;
  int partial_slots, state_slots;
  int first_window;      // 1: state at the window's first chunk is zero (Eq. 14-15)
  int elems;             // d*dprime + dprime
  int s_elems;           // d*dprime
};

// ---- fused softmax + read-out + merge kernel -----------------------------------
struct AttnArgs {
  const bf16_t *q, *k, *v;
  bf16_t* out;
  const bf16_t* w1_q;
  const float* b1_q;
  const bf16_t* w2_q;
  const float* b2_q;
  const bf16_t* state_s;  // [BH, state_slots, d, dprime]
  const float* state_z;   // [BH, state_slots, dprime]
  float *dbg_m, *dbg_nS, *dbg_aS, *dbg_nL, *dbg_aL;
  float scale_log2e;      // log2(e) / sqrt(d)
  int H, T, HW, chunk, overlap;
  int chunk0, n_win_chunks;  // chunks [chunk0, chunk0 + n_win_chunks)
  int qtiles;                // query tiles per (full) chunk
  int state_slots;
  int stab_mode;
  int n_items, items_per_xcd;
  int n_short;           // > 0: the window's first chunk is chunk 0 (no linear part); its n_short
                         // = BH * qtiles items run last on every XCD (items_per_xcd then counts
                         // ceil(long / 8) + ceil(short / 8))
  int64_t q_bh_stride;   // elements between the q (and out) rows of consecutive (b, h)
  int64_t kv_bh_stride;  // same for k and v
  int step_nq, step_nwin;  // step_nq > 0 (streaming step): queries are rows [0, step_nq) of q,
                           // the softmax window is rows [0, step_nwin) of k / v, the linear
                           // state is slot 0; the frame geometry above is then unused
  int all_linear;          // 1: every chunk reads a state (bidirectional sets of Eq. 11-12)
  unsigned xcd_mask;       // measurement hook: workgroups on XCD x (index % 8) run only if bit x is set
};

// ---- transposes the carry into the [dprime][d] layout of the public state hook ----
struct StateOutArgs {
  const float* carry;  // [BH, d*dprime + dprime], S^T [d][dprime] then z
  float* S_out;        // [BH, dprime, d]
  float* z_out;        // [BH, dprime]
  int BH, d, dprime;
};

// ---- bidirectional states: everything outside each chunk's softmax window -----------
// state(c) = total - sum of the per-frame sums of the frames inside window c (Eq. 11-12);
// the per-frame sums of frames [frame0, frame0 + n_frames) are in `partial`
// (frame-major, nsplit pieces each), the total over all frames is in `total`.
struct BidirArgs {
  const float* partial;
  const float* total;    // [BH, d*dprime + dprime]
  bf16_t* state_s;       // [BH, state_slots, d, dprime]
  float* state_z;        // [BH, state_slots, dprime]
  int BH, T, chunk, overlap;
  int chunk0, n_chunks;  // chunks of this window -> state slots 0 .. n_chunks-1
  int frame0;            // first frame held in `partial`
  int nsplit, partial_slots, state_slots;
  int elems, s_elems;
};

// ---- streaming step: the caller's state feeds the read-out and absorbs the step's pieces ----
// state slot 0 <- the caller's S, z as they are on entry (bf16 S^T [d][dprime] and fp32 z: what
// Eq. 16 reads for this chunk); then S, z += the pieces the chunk-state kernel wrote (Eq. 17-18),
// in place, in the caller's layout.
struct StepStateArgs {
  float* S;              // [BH, dprime, d]   read and written
  float* z;              // [BH, dprime]      read and written
  const float* partial;  // [BH, partial_slots, d*dprime + dprime]: S^T [d][dprime], then z
  bf16_t* state_s;       // [BH, state_slots, d, dprime]
  float* state_z;        // [BH, state_slots, dprime]
  int BH, d, dprime;
  int nsplit;            // pieces to add (0: the state is only copied into slot 0)
  int partial_slots, state_slots;
  int write_slot;        // 1: slot 0 <- the state as it is before the pieces are added
};

// =================================================================================
// Gradient of the output with respect to the feature-map parameters: one step of the
// attention distillation of section 3.4 (Eq. 19) trains only phi_q and phi_k.
// With G = dL/dy_hat, den_i = n^S_i + n^L_i, u_i = G_i / den_i, w_i = -(G_i . y_i) / den_i:
//   dL/dPhi_q,i = S_t u_i + w_i z_t                 (queries of chunk t)
//   dL/dS_t = sum_i Phi_q,i u_i^T ,  dL/dz_t = sum_i w_i Phi_q,i
//   dL/dPhi_k,j = R_tau v_j + r_tau ,  R_tau = sum_{t > tau} dL/dS_t ,  r_tau likewise,
// for keys j of segment tau = [s_lo(tau), s_lo(tau+1)) (Eq. 13: they belong to the linear
// set of every later chunk), followed by the backward pass of the two-layer map.
// =================================================================================

// u = bf16(G / den), w = -(G . y) / den per token
struct PrepArgs {
  const bf16_t* g;    // [tokens, d] upstream gradient
  const bf16_t* y;    // [tokens, d] forward output
  const float* nS;    // [tokens]
  const float* nL;    // [tokens]
  bf16_t* u;          // [tokens, d]
  float* tokw;        // [tokens]
  int64_t tokens;
  int d;
};

// R_tau, r_tau: sums over the later chunks of the chunk-state gradients
struct SuffixArgs {
  const float* s_part;  // [BH, s_slots, elems]: segment s, piece p at slot s*s_nsplit + p; S^T part used
  const float* z_part;  // [(bh*n_seg + s)*z_nsplit + p][dp]
  bf16_t* Rt;           // [BH, slots, d, dp]  (transposed, as the forward chunk states)
  float* r;             // [BH, slots, dp]
  int BH, n_seg, s_nsplit, s_slots, z_nsplit, slots;
  int elems, s_elems, dp;
};

// bf16 matrices [n][R][C] -> [n][C][R]; in2/out2 (nullable): a second batch of n such matrices
struct TransposeArgs {
  const bf16_t* in;
  bf16_t* out;
  const bf16_t* in2;
  bf16_t* out2;
  int n, R, C;
};

// Activation gradients of one side (queries or keys): recomputes U = relu(W1 x + b1) and
// psi = relu(W2 U + b2), forms dPhi = M vec + tokw * zv for the token's segment, and writes
// dpsi = dPhi * dphi/dpsi token-major for the weight-gradient kernels.
struct ActGradArgs {
  const bf16_t* x;      // [BH, N, d]  q or k
  const bf16_t* vec;    // [BH, N, d]  u (query side) or v (key side)
  const float* tokw;    // [BH, N] per-token weight of zv (query side); unused on the key side (1)
  const bf16_t* w1;
  const float* b1;
  const bf16_t* w2;
  const float* b2;
  const bf16_t* M;      // [BH, slots, d, dp]  S_t (query side) or R_tau (key side), transposed
  const float* zv;      // [BH, slots, dp]     z_t or r_tau
  bf16_t* dpsi;         // [BH, N, dp]
  float* db2_part;      // [n_items, dp]  sum over the item's tokens of dpsi
  float* dz_part;       // [n_items, dp]  sum of tokw * phi (query side), or null
  int H, T, HW, chunk, overlap;
  int query_side;       // 1: segment s = queries of chunk s+1, slot s+1; 0: key segment s, slot s
  int n_seg, nsplit, slots, n_items, items_per_xcd;
};

// dW2 partial sums: part[f][hid] = sum over a token range of dpsi[tok][f] * U[tok][hid], with
// U = relu(W1 x + b1) recomputed from x (cheaper than moving it through HBM)
struct TnGemmArgs {
  const bf16_t* dpsi;   // [BH, N, 2d]
  const bf16_t* x;      // [BH, N, d]
  const bf16_t* w1;     // [H, 2d, d]
  const float* b1;      // [H, 2d]
  float* part;          // [BH * nsplit, 2d, 2d]
  int H;
  int64_t N, lo, hi;    // token range [lo, hi) of every (b, h)
  int nsplit, n_items, items_per_xcd;
};

// First-layer gradients: dU = (dpsi W2) * [U > 0] with U recomputed from x;
// part = x^T dU ([d][hidden]), then the column sums of dU ([hidden])
struct HidGradArgs {
  const bf16_t* dpsi;   // [BH, N, dp]
  const bf16_t* x;      // [BH, N, d]
  const bf16_t* w1;     // [H, hidden, d]
  const float* b1;      // [H, hidden]
  const bf16_t* w2t;    // [H, hidden, dp]  W2 transposed
  float* part;          // [BH * nsplit, d*hidden + hidden]
  int H;
  int64_t N, lo, hi;
  int nsplit, n_items, items_per_xcd;
};

// out[h][..] = sum over b and the per_bh partials of (b, h) of an [R][C] block found at
// part_off inside each partial; transposed on the way out if `transpose`
struct ReduceArgs {
  const float* part;
  float* out;           // [H, R*C]
  int B, H, per_bh;
  int64_t part_stride, part_off;
  int R, C, transpose;
};
// up to four such sums in one launch (one per gradient tensor of a side)
struct ReduceJobs {
  ReduceArgs job[4];
  int n;
};

hipError_t launch_prep(const PrepArgs& a, hipStream_t stream);
hipError_t launch_suffix(const SuffixArgs& a, hipStream_t stream);
hipError_t launch_transpose(const TransposeArgs& a, hipStream_t stream);
hipError_t launch_act_grad(const ActGradArgs& a, int d, int grid, hipStream_t stream);
hipError_t launch_tn_gemm(const TnGemmArgs& a, int d, int grid, hipStream_t stream);
hipError_t launch_hid_grad(const HidGradArgs& a, int d, int grid, hipStream_t stream);
hipError_t launch_reduce(const ReduceJobs& jobs, hipStream_t stream);
hipError_t launch_fill_zero(float* p, int64_t n, hipStream_t stream);

hipError_t launch_state(const StateArgs& a, int d, int grid, hipStream_t stream);
hipError_t launch_prefix(const PrefixArgs& a, hipStream_t stream);
hipError_t launch_attn(const AttnArgs& a, int d, int grid, hipStream_t stream);
int attn_query_tile(int d);  // query tokens per workgroup of the attention kernel
const char* attn_kernel_name(int d);  // the instance launched for head width d, as profilers show it
hipError_t launch_state_out(const StateOutArgs& a, hipStream_t stream);
hipError_t launch_step_state(const StepStateArgs& a, hipStream_t stream);
hipError_t launch_bidir_state(const BidirArgs& a, hipStream_t stream);
// S [BH, dprime, d] and z [BH, dprime] <- 0
hipError_t launch_zero_state(float* S, float* z, int BH, int d, int dprime, hipStream_t stream);

}  // namespace rehyat
