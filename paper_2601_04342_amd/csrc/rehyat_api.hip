// Host side of the C ABI declared in include/rehyat.h: argument validation, the
// window plan over chunks, workspace carving and kernel launches.  No numerics
// happen here.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdio>
#include <cstring>
#include <atomic>
#include <mutex>

#include "../../include/rehyat.h"
#include "rehyat_kernels.h"

namespace {

using namespace rehyat;

// Slot counts of a workspace: how many (segment, piece) partial sums and how many chunk
// states per (b, h) can be in flight; the window of chunks processed between two carries
// is min(partial / nsplit, state).  Every kernel takes both as arguments.
struct Slots {
  int partial, state;
};
constexpr Slots kSlots{64, 32};  // workspaces sized by rehyat_workspace_bytes
constexpr int kMaxSplit = 8;
constexpr int kCUs = 256;

// Device memory of the allocation-free entry point: one array per GPU, alive until the
// process ends.  In host code the name is only a handle for hipGetSymbolAddress; the
// address it returns (per device) is what kernels and the host layer use.
constexpr size_t kScratchBytes = REHYAT_NOALLOC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];
constexpr int kMaxDevices = 64;
void* g_scratch_ptr[kMaxDevices] = {};

struct Workspace {
  void* ptr = nullptr;
  size_t bytes = 0;
  bool owned = false;
};
Workspace g_ws;
std::mutex g_mu;
char g_hip_err[256] = "";
std::atomic<unsigned> g_xcd_mask{0xFFu};   // rehyat_debug_set_xcd_mask

// rehyat_step runs the state update of a chunk beside its attention kernel: a second stream
// per device, forked from and joined to the caller's stream with two events (all at the
// default priority; created on first use, kept until the process ends).
struct SideStream {
  hipStream_t s = nullptr;
  hipEvent_t fork = nullptr, join = nullptr;
};
SideStream g_side[kMaxDevices];

int hip_fail(hipError_t e, const char* what) {
  snprintf(g_hip_err, sizeof(g_hip_err), "%s: %s", what, hipGetErrorString(e));
  return REHYAT_E_HIP;
}

// optional per-kernel timing with HIP events on the caller's stream (calls that use the
// library-held workspace only: those are serialised by g_mu)
constexpr int kProfKinds = 3;  // state, prefix, attention
constexpr int kProfMaxPairs = 4096;
struct Profiler {
  bool on = false;
  hipEvent_t beg[kProfMaxPairs], end[kProfMaxPairs];
  int kind[kProfMaxPairs];
  int created = 0;  // events created so far
  int used = 0;     // pairs recorded since the last read
};
Profiler g_prof;

struct ProfScope {
  int slot = -1;
  hipStream_t st;
  ProfScope(bool enabled, int kind, hipStream_t s) : st(s) {
    if (!enabled || !g_prof.on || g_prof.used >= kProfMaxPairs) return;
    if (g_prof.used >= g_prof.created) {
      if (hipEventCreate(&g_prof.beg[g_prof.created]) != hipSuccess) return;
      if (hipEventCreate(&g_prof.end[g_prof.created]) != hipSuccess) return;
      ++g_prof.created;
    }
    slot = g_prof.used++;
    g_prof.kind[slot] = kind;
    (void)hipEventRecord(g_prof.beg[slot], st);
  }
  ~ProfScope() {
    if (slot >= 0) (void)hipEventRecord(g_prof.end[slot], st);
  }
};

size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

struct WsLayout {
  size_t partial, state_s, state_z, carry, total;
};

WsLayout ws_layout(int B, int H, int d, int dp, Slots sl) {
  const size_t BH = (size_t)B * H;
  const size_t elems = (size_t)d * dp + dp;
  WsLayout L;
  size_t off = 0;
  L.partial = off;
  off += align256(BH * sl.partial * elems * sizeof(float));
  L.state_s = off;
  off += align256(BH * sl.state * (size_t)d * dp * sizeof(bf16_t));
  L.state_z = off;
  off += align256(BH * sl.state * (size_t)dp * sizeof(float));
  L.carry = off;
  off += align256(BH * elems * sizeof(float));
  L.total = off;
  return L;
}

// Where one call's kernels find their device memory and stream.
struct Ctx {
  char* ws;
  WsLayout L;
  Slots sl;
  hipStream_t st;
  bool prof;  // record per-kernel events (library-held workspace only)
};

// The side stream of the current device, or nullptr when there is none and none can be made
// now (the caller's stream is being captured: nothing is created inside a capture).
SideStream* side_stream(hipStream_t main) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
  SideStream& ss = g_side[dev];
  if (ss.s) return &ss;
  hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
  if (hipStreamIsCapturing(main, &cap) != hipSuccess || cap != hipStreamCaptureStatusNone) return nullptr;
  hipStream_t st = nullptr;
  hipEvent_t a = nullptr, b = nullptr;
  if (hipStreamCreateWithFlags(&st, hipStreamNonBlocking) != hipSuccess) return nullptr;
  if (hipEventCreateWithFlags(&a, hipEventDisableTiming) != hipSuccess ||
      hipEventCreateWithFlags(&b, hipEventDisableTiming) != hipSuccess) {
    if (a) (void)hipEventDestroy(a);
    (void)hipStreamDestroy(st);
    return nullptr;
  }
  ss.s = st;
  ss.fork = a;
  ss.join = b;
  return &ss;
}

bool supported_dims(int d, int dp) { return (d == 64 || d == 128) && dp == 2 * d; }

// The library-held workspace (caller-set or library-owned), at least `need` bytes.  A
// caller-set buffer is never replaced; a library-owned one is allocated or grown here
// unless `st` is capturing (an allocation would break the capture, and a free would leave
// earlier graphs pointing at released memory).
int ensure_workspace(size_t need, hipStream_t st, char** base) {
  if (g_ws.ptr && g_ws.bytes >= need) {
    *base = (char*)g_ws.ptr;
    return REHYAT_OK;
  }
  if (g_ws.ptr && !g_ws.owned) return REHYAT_E_WORKSPACE;  // caller's buffer is too small
  hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
  hipError_t e = hipStreamIsCapturing(st, &cap);
  if (e != hipSuccess) return hip_fail(e, "hipStreamIsCapturing");
  if (cap != hipStreamCaptureStatusNone) return REHYAT_E_WORKSPACE;
  if (g_ws.ptr) {
    e = hipFree(g_ws.ptr);
    g_ws = Workspace();
    if (e != hipSuccess) return hip_fail(e, "hipFree(workspace)");
  }
  void* p = nullptr;
  e = hipMalloc(&p, need);
  if (e != hipSuccess) return hip_fail(e, "hipMalloc(workspace)");
  g_ws.ptr = p;
  g_ws.bytes = need;
  g_ws.owned = true;
  *base = (char*)p;
  return REHYAT_OK;
}

bool aligned16(const void* p) { return (((uintptr_t)p) & 15) == 0; }
bool aligned4(const void* p) { return (((uintptr_t)p) & 3) == 0; }

int check_phi(const rehyat_phi_params* p, int d) {
  if (!p) return REHYAT_E_NULL;
  if (!p->w1_q || !p->b1_q || !p->w2_q || !p->b2_q || !p->w1_k || !p->b1_k || !p->w2_k || !p->b2_k)
    return REHYAT_E_NULL;
  if (p->hidden < 1 || p->dprime < 1 || p->degree < 1) return REHYAT_E_SHAPE;
  if (p->dprime % p->degree) return REHYAT_E_SHAPE;
  if (p->hidden != 2 * d || p->dprime != 2 * d || p->degree != 2 || p->act != 0)
    return REHYAT_E_UNSUPPORTED;
  // weight rows are fetched 16 bytes at a time, biases as single floats
  if (!aligned16(p->w1_q) || !aligned16(p->w2_q) || !aligned16(p->w1_k) || !aligned16(p->w2_k))
    return REHYAT_E_SHAPE;
  if (!aligned4(p->b1_q) || !aligned4(p->b2_q) || !aligned4(p->b1_k) || !aligned4(p->b2_k))
    return REHYAT_E_SHAPE;
  return REHYAT_OK;
}

// pieces per segment: more workgroups when (b, h, segment) alone cannot fill the chip
int choose_nsplit(int BH, int n_seg_total, Slots sl) {
  if (n_seg_total < 1) return 1;
  int best = 1;
  double best_cost = 1e30;
  for (int ns = 1; ns <= kMaxSplit && ns <= sl.partial; ++ns) {
    int win = sl.partial / ns;
    if (win > sl.state) win = sl.state;
    const int segs = n_seg_total < win ? n_seg_total : win;
    const int windows = (n_seg_total + win - 1) / win;
    const long wgs = (long)BH * segs * ns;
    const double rounds = std::ceil((double)wgs / kCUs);
    // time in units of "one whole segment on one CU"
    const double cost = windows * rounds / ns;
    if (cost < best_cost * 0.9) {
      best_cost = cost;
      best = ns;
    }
  }
  return best;
}

int launch_state_window(const Ctx& c, const void* k, const void* v, const rehyat_phi_params* phi,
                        int B, int H, int T, int HW, int d, int chunk, int overlap, int chunk0,
                        int n_seg, int nsplit) {
  StateArgs s;
  s.k = (const bf16_t*)k;
  s.v = (const bf16_t*)v;
  s.w1_k = (const bf16_t*)phi->w1_k;
  s.b1_k = (const float*)phi->b1_k;
  s.w2_k = (const bf16_t*)phi->w2_k;
  s.b2_k = (const float*)phi->b2_k;
  s.partial = (float*)(c.ws + c.L.partial);
  s.H = H;
  s.T = T;
  s.HW = HW;
  s.chunk = chunk;
  s.overlap = overlap;
  s.chunk0 = chunk0;
  s.n_seg = n_seg;
  s.nsplit = nsplit;
  s.partial_slots = c.sl.partial;
  s.n_items = B * H * n_seg * nsplit;
  s.items_per_xcd = (s.n_items + 7) / 8;
  s.kv_bh_stride = (int64_t)T * HW * d;
  s.step_n = 0;
  s.query_segments = 0;
  ProfScope prof(c.prof, 0, c.st);
  hipError_t e = launch_state(s, d, s.items_per_xcd * 8, c.st);
  if (e != hipSuccess) return hip_fail(e, "state kernel launch");
  return REHYAT_OK;
}

int launch_prefix_window(const Ctx& c, int B, int H, int d, int dp, int n_chunks, int n_seg,
                         int nsplit, bool first) {
  PrefixArgs p;
  p.partial = (const float*)(c.ws + c.L.partial);
  p.carry = (float*)(c.ws + c.L.carry);
  p.state_s = (bf16_t*)(c.ws + c.L.state_s);
  p.state_z = (float*)(c.ws + c.L.state_z);
  p.BH = B * H;
  p.n_chunks = n_chunks;
  p.n_seg = n_seg;
  p.nsplit = nsplit;
  p.partial_slots = c.sl.partial;
  p.state_slots = c.sl.state;
  p.first_window = first ? 1 : 0;
  p.elems = d * dp + dp;
  p.s_elems = d * dp;
  ProfScope prof(c.prof, 1, c.st);
  hipError_t e = launch_prefix(p, c.st);
  if (e != hipSuccess) return hip_fail(e, "prefix kernel launch");
  return REHYAT_OK;
}

int launch_attn_window(const Ctx& c, const void* q, const void* k, const void* v,
                       const rehyat_phi_params* phi, void* out, const rehyat_debug_out* debug,
                       int B, int H, int T, int HW, int d, int chunk, int overlap, int c0,
                       int n_chunks, int qtiles, int stab_mode, bool bidir) {
  AttnArgs a;
  a.q = (const bf16_t*)q;
  a.k = (const bf16_t*)k;
  a.v = (const bf16_t*)v;
  a.out = (bf16_t*)out;
  a.w1_q = (const bf16_t*)phi->w1_q;
  a.b1_q = (const float*)phi->b1_q;
  a.w2_q = (const bf16_t*)phi->w2_q;
  a.b2_q = (const float*)phi->b2_q;
  a.state_s = (const bf16_t*)(c.ws + c.L.state_s);
  a.state_z = (const float*)(c.ws + c.L.state_z);
  a.dbg_m = debug ? debug->m : nullptr;
  a.dbg_nS = debug ? debug->nS : nullptr;
  a.dbg_aS = debug ? debug->aS : nullptr;
  a.dbg_nL = debug ? debug->nL : nullptr;
  a.dbg_aL = debug ? debug->aL : nullptr;
  a.scale_log2e = (float)(1.4426950408889634 / std::sqrt((double)d));
  a.H = H;
  a.T = T;
  a.HW = HW;
  a.chunk = chunk;
  a.overlap = overlap;
  a.chunk0 = c0;
  a.n_win_chunks = n_chunks;
  a.qtiles = qtiles;
  a.state_slots = c.sl.state;
  a.stab_mode = stab_mode;
  a.n_items = B * H * n_chunks * qtiles;
  a.items_per_xcd = (a.n_items + 7) / 8;
  a.n_short = 0;
  if (c0 == 0 && !bidir && n_chunks > 1) {   // chunk 0 has no read-out phase: its items go last
    a.n_short = B * H * qtiles;
    a.items_per_xcd = (a.n_items - a.n_short + 7) / 8 + (a.n_short + 7) / 8;
  }
  a.q_bh_stride = a.kv_bh_stride = (int64_t)T * HW * d;
  a.step_nq = a.step_nwin = 0;
  a.all_linear = bidir ? 1 : 0;
  a.xcd_mask = g_xcd_mask.load();
  hipError_t e;
  {
    ProfScope prof(c.prof, 2, c.st);
    e = launch_attn(a, d, a.items_per_xcd * 8, c.st);
  }
  if (e != hipSuccess) return hip_fail(e, "attention kernel launch");
  return REHYAT_OK;
}

// Bidirectional sets (Eq. 11-12): the linear part of chunk t covers every token outside
// its softmax window.  Per-frame sums F(f) of phi_k(k) v^T come from the chunk-state kernel
// run with one-frame segments; state(t) = sum_f F(f) - sum_{f in window t} F(f).
int forward_bidirectional(const Ctx& c, const void* q, const void* k, const void* v,
                          const rehyat_phi_params* phi, void* out, const rehyat_debug_out* debug,
                          int B, int H, int T, int HW, int d, int dp, int chunk, int overlap,
                          int stab_mode) {
  const int nc = num_chunks(T, chunk);
  const int qtile = attn_query_tile(d);
  const int qtiles = (int)(((int64_t)chunk * HW + qtile - 1) / qtile);
  if (nc == 1)  // the window is the whole sequence: plain softmax attention
    return launch_attn_window(c, q, k, v, phi, out, debug, B, H, T, HW, d, chunk, overlap, 0, 1,
                              qtiles, stab_mode, false);
  int win_frames = chunk + overlap;  // frames one window can span (both are <= T here)
  if (win_frames > T) win_frames = T;
  if (win_frames > c.sl.partial) return REHYAT_E_UNSUPPORTED;
  int nsplit = choose_nsplit(B * H, T, c.sl);
  while (nsplit > 1 && c.sl.partial / nsplit < win_frames) --nsplit;
  const int fwin = c.sl.partial / nsplit;  // frames whose sums fit the partial slots

  // pass 1: total over all frames, left in the carry
  for (int f0 = 0; f0 < T; f0 += fwin) {
    const int n = (T - f0 < fwin) ? T - f0 : fwin;
    int rc = launch_state_window(c, k, v, phi, B, H, T, HW, d, 1, 0, f0, n, nsplit);
    if (rc != REHYAT_OK) return rc;
    rc = launch_prefix_window(c, B, H, d, dp, /*n_chunks=*/0, /*n_seg=*/n, nsplit, f0 == 0);
    if (rc != REHYAT_OK) return rc;
  }
  const bool resident = T <= fwin;  // every F(f) is still in the partial slots

  // pass 2: windows of chunks whose frames fit the partial slots together
  int cw = (fwin - overlap) / chunk;
  if (cw < 1) cw = 1;
  if (cw > c.sl.state) cw = c.sl.state;
  for (int c0 = 0; c0 < nc; c0 += cw) {
    const int c1 = (c0 + cw < nc) ? c0 + cw : nc;
    int F0 = c0 * chunk - overlap;
    if (F0 < 0) F0 = 0;
    int F1 = c1 * chunk;
    if (F1 > T) F1 = T;
    if (!resident) {
      int rc = launch_state_window(c, k, v, phi, B, H, T, HW, d, 1, 0, F0, F1 - F0, nsplit);
      if (rc != REHYAT_OK) return rc;
    }
    BidirArgs b;
    b.partial = (const float*)(c.ws + c.L.partial);
    b.total = (const float*)(c.ws + c.L.carry);
    b.state_s = (bf16_t*)(c.ws + c.L.state_s);
    b.state_z = (float*)(c.ws + c.L.state_z);
    b.BH = B * H;
    b.T = T;
    b.chunk = chunk;
    b.overlap = overlap;
    b.chunk0 = c0;
    b.n_chunks = c1 - c0;
    b.frame0 = resident ? 0 : F0;
    b.nsplit = nsplit;
    b.partial_slots = c.sl.partial;
    b.state_slots = c.sl.state;
    b.elems = d * dp + dp;
    b.s_elems = d * dp;
    hipError_t e;
    {
      ProfScope prof(c.prof, 1, c.st);
      e = launch_bidir_state(b, c.st);
    }
    if (e != hipSuccess) return hip_fail(e, "bidirectional state kernel launch");
    int rc = launch_attn_window(c, q, k, v, phi, out, debug, B, H, T, HW, d, chunk, overlap, c0,
                                c1 - c0, qtiles, stab_mode, true);
    if (rc != REHYAT_OK) return rc;
  }
  return REHYAT_OK;
}

// Argument checks shared by every forward entry point.  On success chunk and overlap are
// clamped to T (a chunk or an overlap longer than the video acts like T), so that no later
// sum of them can leave the range of int.
int validate_forward(const void* q, const void* k, const void* v, const rehyat_phi_params* phi,
                     const void* out, int B, int H, int T, int HW, int d, int* chunk, int* overlap,
                     int causal, int stab_mode) {
  if (!q || !k || !v || !out) return REHYAT_E_NULL;
  if (B < 1 || H < 1 || T < 1 || HW < 1 || d < 1 || *chunk < 1 || *overlap < 0) return REHYAT_E_SHAPE;
  if ((int64_t)T * HW >= ((int64_t)1 << 31)) return REHYAT_E_SHAPE;
  if ((int64_t)B * H > 65535) return REHYAT_E_SHAPE;
  if (*chunk > T) *chunk = T;
  if (*overlap > T) *overlap = T;
  {
    // one launch covers up to 32 chunks: its workgroup count must fit an int
    const int64_t tiles = ((int64_t)*chunk * HW + 63) / 64;
    if ((int64_t)B * H * kSlots.state * tiles >= ((int64_t)1 << 31)) return REHYAT_E_SHAPE;
    // tile offsets inside one softmax window or state segment are 32-bit
    int64_t wf = (int64_t)*chunk + *overlap;
    if (wf > T) wf = T;
    if (wf * HW * d * 2 >= ((int64_t)1 << 31)) return REHYAT_E_SHAPE;
  }
  if (d != 64 && d != 128) return REHYAT_E_UNSUPPORTED;
  int rc = check_phi(phi, d);
  if (rc != REHYAT_OK) return rc;
  if (stab_mode != REHYAT_STAB_ROWMAX && stab_mode != REHYAT_STAB_NONE) return REHYAT_E_SHAPE;
  if (causal != 0 && causal != 1) return REHYAT_E_SHAPE;
  // rows are fetched and stored 16 bytes at a time
  if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(out)) return REHYAT_E_SHAPE;
  return REHYAT_OK;
}

// The kernels of one forward call on validated arguments.
int forward_core(const Ctx& c, const void* q, const void* k, const void* v,
                 const rehyat_phi_params* phi, void* out, const rehyat_debug_out* debug, int B,
                 int H, int T, int HW, int d, int chunk, int overlap, int causal, int stab_mode) {
  const int dp = phi->dprime;
  if (causal == 0)
    return forward_bidirectional(c, q, k, v, phi, out, debug, B, H, T, HW, d, dp, chunk, overlap,
                                 stab_mode);
  const int nc = num_chunks(T, chunk);
  const int nsplit = choose_nsplit(B * H, nc - 1, c.sl);
  int win = c.sl.partial / nsplit;
  if (win > c.sl.state) win = c.sl.state;
  const int qtile = attn_query_tile(d);
  const int qtiles = (int)(((int64_t)chunk * HW + qtile - 1) / qtile);

  for (int c0 = 0; c0 < nc; c0 += win) {
    const int c1 = (c0 + win < nc) ? c0 + win : nc;
    const int n_chunks = c1 - c0;
    const int n_seg = (c1 < nc) ? n_chunks : n_chunks - 1;
    int rc;
    if (n_seg > 0) {
      rc = launch_state_window(c, k, v, phi, B, H, T, HW, d, chunk, overlap, c0, n_seg, nsplit);
      if (rc != REHYAT_OK) return rc;
    }
    if (nc > 1) {
      rc = launch_prefix_window(c, B, H, d, dp, n_chunks, n_seg, nsplit, c0 == 0);
      if (rc != REHYAT_OK) return rc;
    }
    rc = launch_attn_window(c, q, k, v, phi, out, debug, B, H, T, HW, d, chunk, overlap, c0,
                            n_chunks, qtiles, stab_mode, /*bidir=*/false);
    if (rc != REHYAT_OK) return rc;
  }
  return REHYAT_OK;
}

// ---- feature-map gradient (Eq. 19): workspace plan and launches ----------------------
struct BwdPlan {
  Slots sl;          // forward areas: one window holds every chunk
  WsLayout F;
  int nc, n_seg;     // chunks; segments (= chunks that read a state)
  int nsplit;        // pieces per segment (state and activation-gradient kernels)
  int nsplit_g;      // pieces per (b, h) of the weight-gradient kernels
  size_t yhat, nS, nL, u, tokw, Rt, rz, w2t_q, w2t_k, dpsi, p_w2, p_w1, p_b2, p_dz, total;
};

BwdPlan bwd_plan(int B, int H, int T, int HW, int d, int chunk) {
  BwdPlan P;
  const int dp = 2 * d, hid = 2 * d;
  const size_t BH = (size_t)B * H, N = (size_t)T * HW;
  P.nc = num_chunks(T, chunk);
  P.n_seg = P.nc > 1 ? P.nc - 1 : 1;
  P.nsplit = choose_nsplit((int)BH, P.n_seg, Slots{kMaxSplit * P.nc, P.nc});
  P.sl = Slots{P.n_seg * P.nsplit, P.nc};
  P.F = ws_layout(B, H, d, dp, P.sl);
  // weight-gradient kernels: one (b, h) token range cut so that the pieces about fill the chip
  int ns = (int)(kCUs / BH);
  if (ns < 1) ns = 1;
  const size_t tiles = (N + 63) / 64;
  if ((size_t)ns > tiles) ns = (int)tiles;
  P.nsplit_g = ns;
  size_t off = P.F.total;
  auto take = [&](size_t bytes) {
    const size_t o = off;
    off += align256(bytes);
    return o;
  };
  P.yhat = take(BH * N * d * sizeof(bf16_t));
  P.nS = take(BH * N * sizeof(float));
  P.nL = take(BH * N * sizeof(float));
  P.u = take(BH * N * d * sizeof(bf16_t));
  P.tokw = take(BH * N * sizeof(float));
  P.Rt = take(BH * P.nc * (size_t)dp * d * sizeof(bf16_t));
  P.rz = take(BH * P.nc * (size_t)dp * sizeof(float));
  P.w2t_q = take((size_t)H * hid * dp * sizeof(bf16_t));
  P.w2t_k = take((size_t)H * hid * dp * sizeof(bf16_t));
  P.dpsi = take(BH * N * dp * sizeof(bf16_t));
  P.p_w2 = take(BH * ns * (size_t)dp * hid * sizeof(float));
  P.p_w1 = take(BH * ns * ((size_t)d * hid + hid) * sizeof(float));
  P.p_b2 = take(BH * P.n_seg * P.nsplit * (size_t)dp * sizeof(float));
  P.p_dz = take(BH * P.n_seg * P.nsplit * (size_t)dp * sizeof(float));
  P.total = off;
  return P;
}

struct SideParams {   // one feature map and where its gradients go
  const void *w1, *b1, *w2, *b2;
  float *g_w1, *g_b1, *g_w2, *g_b2;
};

// Activation gradients, then the weight gradients, of one side.  `x` is q or k, `vec` is u or
// v, `M`/`zv` the per-segment matrices of dPhi = M vec + tokw zv; [lo, hi) is the token range
// of every (b, h) that the segments cover.
int backward_side(char* ws, const BwdPlan& P, hipStream_t st, const void* x, const void* vec,
                  const float* tokw, const SideParams& sp, const bf16_t* w2t, const bf16_t* M,
                  const float* zv, bool query_side, float* dz_part, int B, int H, int T, int HW,
                  int d, int chunk, int overlap, int64_t lo, int64_t hi) {
  const int dp = 2 * d, hid = 2 * d;
  const int BH = B * H;
  ActGradArgs g;
  g.x = (const bf16_t*)x;
  g.vec = (const bf16_t*)vec;
  g.tokw = tokw;
  g.w1 = (const bf16_t*)sp.w1;
  g.b1 = (const float*)sp.b1;
  g.w2 = (const bf16_t*)sp.w2;
  g.b2 = (const float*)sp.b2;
  g.M = M;
  g.zv = zv;
  g.dpsi = (bf16_t*)(ws + P.dpsi);
  g.db2_part = (float*)(ws + P.p_b2);
  g.dz_part = dz_part;
  g.H = H;
  g.T = T;
  g.HW = HW;
  g.chunk = chunk;
  g.overlap = overlap;
  g.query_side = query_side ? 1 : 0;
  g.n_seg = P.n_seg;
  g.nsplit = P.nsplit;
  g.slots = P.nc;
  g.n_items = BH * P.n_seg * P.nsplit;
  g.items_per_xcd = (g.n_items + 7) / 8;
  hipError_t e = launch_act_grad(g, d, g.items_per_xcd * 8, st);
  if (e != hipSuccess) return hip_fail(e, "activation-gradient kernel launch");

  const int n_items = BH * P.nsplit_g;
  TnGemmArgs t;
  t.dpsi = (const bf16_t*)(ws + P.dpsi);
  t.x = (const bf16_t*)x;
  t.w1 = (const bf16_t*)sp.w1;
  t.b1 = (const float*)sp.b1;
  t.part = (float*)(ws + P.p_w2);
  t.H = H;
  t.N = (int64_t)T * HW;
  t.lo = lo;
  t.hi = hi;
  t.nsplit = P.nsplit_g;
  t.n_items = n_items;
  t.items_per_xcd = (n_items + 7) / 8;
  e = launch_tn_gemm(t, d, t.items_per_xcd * 8, st);
  if (e != hipSuccess) return hip_fail(e, "second-layer gradient kernel launch");

  HidGradArgs hg;
  hg.dpsi = (const bf16_t*)(ws + P.dpsi);
  hg.x = (const bf16_t*)x;
  hg.w1 = (const bf16_t*)sp.w1;
  hg.b1 = (const float*)sp.b1;
  hg.w2t = w2t;
  hg.part = (float*)(ws + P.p_w1);
  hg.H = H;
  hg.N = (int64_t)T * HW;
  hg.lo = lo;
  hg.hi = hi;
  hg.nsplit = P.nsplit_g;
  hg.n_items = n_items;
  hg.items_per_xcd = (n_items + 7) / 8;
  e = launch_hid_grad(hg, d, hg.items_per_xcd * 8, st);
  if (e != hipSuccess) return hip_fail(e, "first-layer gradient kernel launch");

  // the four gradient tensors of this side from their partial sums, one launch
  ReduceJobs jobs;
  jobs.n = 4;
  for (int j = 0; j < 4; ++j) {
    jobs.job[j].B = B;
    jobs.job[j].H = H;
    jobs.job[j].part_off = 0;
    jobs.job[j].transpose = 0;
  }
  ReduceArgs& rw2 = jobs.job[0];
  rw2.part = (const float*)(ws + P.p_w2);
  rw2.out = sp.g_w2;
  rw2.per_bh = P.nsplit_g;
  rw2.part_stride = (int64_t)dp * hid;
  rw2.R = dp;
  rw2.C = hid;
  ReduceArgs& rw1 = jobs.job[1];   // partial is dW1^T [d][hidden]
  rw1.part = (const float*)(ws + P.p_w1);
  rw1.out = sp.g_w1;
  rw1.per_bh = P.nsplit_g;
  rw1.part_stride = (int64_t)d * hid + hid;
  rw1.R = d;
  rw1.C = hid;
  rw1.transpose = 1;
  ReduceArgs& rb1 = jobs.job[2];
  rb1 = rw1;
  rb1.out = sp.g_b1;
  rb1.part_off = (int64_t)d * hid;
  rb1.R = 1;
  rb1.C = hid;
  rb1.transpose = 0;
  ReduceArgs& rb2 = jobs.job[3];
  rb2.part = (const float*)(ws + P.p_b2);
  rb2.out = sp.g_b2;
  rb2.per_bh = P.n_seg * P.nsplit;
  rb2.part_stride = dp;
  rb2.R = 1;
  rb2.C = dp;
  e = launch_reduce(jobs, st);
  if (e != hipSuccess) return hip_fail(e, "reduce kernel launch");
  return REHYAT_OK;
}

// Largest slot counts whose layout fits `bytes` (equal partial and state slots, at most the
// default window); 0 slots when not even one fits.
Slots slots_that_fit(int B, int H, int d, int dp, size_t bytes) {
  Slots best{0, 0};
  for (int n = 1; n <= kSlots.state; ++n) {
    const Slots s{n, n};
    if (ws_layout(B, H, d, dp, s).total > bytes) break;
    best = s;
  }
  return best;
}

}  // namespace

extern "C" {

int rehyat_version(void) { return 304; }

const char* rehyat_status_string(int code) {
  switch (code) {
    case REHYAT_OK: return "ok";
    case REHYAT_E_NULL: return "a required pointer is NULL";
    case REHYAT_E_SHAPE: return "a size is non-positive or inconsistent, or a pointer is misaligned";
    case REHYAT_E_UNSUPPORTED: return "configuration not supported by this build";
    case REHYAT_E_WORKSPACE: return "workspace missing, too small or misaligned";
    case REHYAT_E_HIP: return "a HIP runtime call failed";
    default: return "unknown status code";
  }
}

const char* rehyat_last_hip_error(void) { return g_hip_err; }

const char* rehyat_attn_kernel_name(int d) { return (d == 64 || d == 128) ? attn_kernel_name(d) : ""; }

int rehyat_chunk_plan(int T, int HW, int chunk, int overlap, int64_t* table, int* n_chunks) {
  if (!n_chunks) return REHYAT_E_NULL;
  if (T < 1 || HW < 1 || chunk < 1 || overlap < 0) return REHYAT_E_SHAPE;
  if (chunk > T) chunk = T;      // same plan, and no sum below can overflow
  if (overlap > T) overlap = T;
  const int nc = num_chunks(T, chunk);
  if (table) {
    for (int t = 0; t < nc; ++t) {
      ChunkRange r = chunk_range(T, HW, chunk, overlap, t);
      int64_t* row = table + 5 * (int64_t)t;
      row[0] = r.q_lo;
      row[1] = r.q_hi;
      row[2] = r.s_lo;
      row[3] = r.s_hi;
      row[4] = r.l_hi;
    }
  }
  *n_chunks = nc;
  return REHYAT_OK;
}

size_t rehyat_workspace_bytes(int B, int H, int d, int dprime) {
  if (B < 1 || H < 1 || !supported_dims(d, dprime)) return 0;
  return ws_layout(B, H, d, dprime, kSlots).total;
}

int rehyat_set_workspace(void* dev_ptr, size_t bytes) {
  std::lock_guard<std::mutex> lock(g_mu);
  if (dev_ptr && (((uintptr_t)dev_ptr) & 255)) return REHYAT_E_WORKSPACE;
  if (dev_ptr && bytes == 0) return REHYAT_E_WORKSPACE;
  if (g_ws.ptr && g_ws.owned) {
    hipError_t e = hipFree(g_ws.ptr);
    g_ws = Workspace();
    if (e != hipSuccess) return hip_fail(e, "hipFree(workspace)");
  }
  g_ws = Workspace();
  if (dev_ptr) {
    g_ws.ptr = dev_ptr;
    g_ws.bytes = bytes;
    g_ws.owned = false;
  }
  return REHYAT_OK;
}

int rehyat_shutdown(void) {
  std::lock_guard<std::mutex> lock(g_mu);
  if (g_ws.ptr && g_ws.owned) {
    hipError_t e = hipFree(g_ws.ptr);
    g_ws = Workspace();
    if (e != hipSuccess) return hip_fail(e, "hipFree(workspace)");
  }
  g_ws = Workspace();
  return REHYAT_OK;
}

int rehyat_forward_ex(const void* q, const void* k, const void* v, const rehyat_phi_params* phi,
                      void* out, int B, int H, int T, int HW, int d, int chunk, int overlap,
                      int causal, int stab_mode, const rehyat_debug_out* debug, void* stream) {
  int rc = validate_forward(q, k, v, phi, out, B, H, T, HW, d, &chunk, &overlap, causal, stab_mode);
  if (rc != REHYAT_OK) return rc;
  std::lock_guard<std::mutex> lock(g_mu);
  Ctx c;
  c.sl = kSlots;
  c.L = ws_layout(B, H, d, phi->dprime, c.sl);
  c.st = (hipStream_t)stream;
  c.prof = true;
  rc = ensure_workspace(c.L.total, c.st, &c.ws);
  if (rc != REHYAT_OK) return rc;
  return forward_core(c, q, k, v, phi, out, debug, B, H, T, HW, d, chunk, overlap, causal, stab_mode);
}

int rehyat_forward_ws(const void* q, const void* k, const void* v, const rehyat_phi_params* phi,
                      void* out, int B, int H, int T, int HW, int d, int chunk, int overlap,
                      int causal, int stab_mode, void* workspace, size_t workspace_bytes,
                      void* stream) {
  int rc = validate_forward(q, k, v, phi, out, B, H, T, HW, d, &chunk, &overlap, causal, stab_mode);
  if (rc != REHYAT_OK) return rc;
  if (!workspace) return REHYAT_E_NULL;
  Ctx c;
  c.sl = kSlots;
  c.L = ws_layout(B, H, d, phi->dprime, c.sl);
  c.st = (hipStream_t)stream;
  c.prof = false;
  if ((((uintptr_t)workspace) & 255) || workspace_bytes < c.L.total) return REHYAT_E_WORKSPACE;
  c.ws = (char*)workspace;
  // no library state is touched: calls with distinct workspaces may run concurrently
  return forward_core(c, q, k, v, phi, out, nullptr, B, H, T, HW, d, chunk, overlap, causal, stab_mode);
}

int rehyat_forward_noalloc(const void* q, const void* k, const void* v, const rehyat_phi_params* phi,
                           void* out, int B, int H, int T, int HW, int d, int chunk, void* stream) {
  int overlap = 0;
  int rc = validate_forward(q, k, v, phi, out, B, H, T, HW, d, &chunk, &overlap, 1, REHYAT_STAB_ROWMAX);
  if (rc != REHYAT_OK) return rc;
  Ctx c;
  c.sl = slots_that_fit(B, H, d, phi->dprime, kScratchBytes);
  if (c.sl.state < 1) return REHYAT_E_WORKSPACE;  // B*H beyond what the fixed scratch array holds
  c.L = ws_layout(B, H, d, phi->dprime, c.sl);
  c.st = (hipStream_t)stream;
  c.prof = false;
  std::lock_guard<std::mutex> lock(g_mu);
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return hip_fail(e, "hipGetDevice");
  if (dev < 0 || dev >= kMaxDevices) return REHYAT_E_UNSUPPORTED;
  if (!g_scratch_ptr[dev]) {
    // each GPU holds its own copy of the array at its own address
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return hip_fail(e, "hipGetSymbolAddress(scratch)");
    if (!p || (((uintptr_t)p) & 255)) return REHYAT_E_WORKSPACE;
    g_scratch_ptr[dev] = p;
  }
  c.ws = (char*)g_scratch_ptr[dev];
  // every element of the scratch that a kernel reads is written earlier in the same call
  // (partials by the state kernel, states and carry by the prefix pass), so the previous
  // call's contents need no clearing
  return forward_core(c, q, k, v, phi, out, nullptr, B, H, T, HW, d, chunk, overlap, 1,
                      REHYAT_STAB_ROWMAX);
}

size_t rehyat_phi_backward_workspace_bytes(int B, int H, int T, int HW, int d, int chunk) {
  if (B < 1 || H < 1 || T < 1 || HW < 1 || chunk < 1 || (d != 64 && d != 128)) return 0;
  if ((int64_t)T * HW >= ((int64_t)1 << 31) / (4 * d) || (int64_t)B * H > 65535) return 0;
  if (chunk > T) chunk = T;
  if (num_chunks(T, chunk) > REHYAT_BACKWARD_MAX_CHUNKS) return 0;
  return bwd_plan(B, H, T, HW, d, chunk).total;
}

int rehyat_phi_backward(const void* q, const void* k, const void* v, const rehyat_phi_params* phi,
                        const void* grad_out, void* out, const rehyat_forward_saved* saved,
                        const rehyat_phi_grads* grads, int B, int H, int T, int HW, int d, int chunk,
                        int overlap, void* workspace, size_t workspace_bytes, void* stream) {
  if (!grad_out || !grads) return REHYAT_E_NULL;
  if (saved && (!out || !saved->nS || !saved->nL)) return REHYAT_E_NULL;
  if (saved && (!aligned4(saved->nS) || !aligned4(saved->nL))) return REHYAT_E_SHAPE;
  int rc = validate_forward(q, k, v, phi, out ? out : grad_out, B, H, T, HW, d, &chunk, &overlap, 1,
                            REHYAT_STAB_ROWMAX);
  if (rc != REHYAT_OK) return rc;
  if (!grads->w1_q || !grads->b1_q || !grads->w2_q || !grads->b2_q || !grads->w1_k ||
      !grads->b1_k || !grads->w2_k || !grads->b2_k)
    return REHYAT_E_NULL;
  if (!aligned16(grad_out)) return REHYAT_E_SHAPE;
  if (!aligned4(grads->w1_q) || !aligned4(grads->b1_q) || !aligned4(grads->w2_q) ||
      !aligned4(grads->b2_q) || !aligned4(grads->w1_k) || !aligned4(grads->b1_k) ||
      !aligned4(grads->w2_k) || !aligned4(grads->b2_k))
    return REHYAT_E_SHAPE;
  // tile offsets of the token-major activation buffers (rows of 4 d bytes) are 32-bit
  if ((int64_t)T * HW >= ((int64_t)1 << 31) / (4 * d)) return REHYAT_E_SHAPE;
  const int nc = num_chunks(T, chunk);
  if (nc > REHYAT_BACKWARD_MAX_CHUNKS) return REHYAT_E_UNSUPPORTED;
  // every chunk goes into one launch: its workgroup count must fit an int
  if ((int64_t)B * H * nc * (((int64_t)chunk * HW + 63) / 64) >= ((int64_t)1 << 31)) return REHYAT_E_SHAPE;
  if (!workspace) return REHYAT_E_NULL;
  const BwdPlan P = bwd_plan(B, H, T, HW, d, chunk);
  if ((((uintptr_t)workspace) & 255) || workspace_bytes < P.total) return REHYAT_E_WORKSPACE;
  char* ws = (char*)workspace;
  hipStream_t st = (hipStream_t)stream;
  const int dp = 2 * d, hid = 2 * d;
  const int BH = B * H;
  const int64_t N = (int64_t)T * HW;
  void* y = out ? out : (void*)(ws + P.yhat);

  Ctx c;
  c.ws = ws;
  c.L = P.F;
  c.sl = P.sl;
  c.st = st;
  c.prof = false;
  const int qtile = attn_query_tile(d);
  const int qtiles = (int)(((int64_t)chunk * HW + qtile - 1) / qtile);

  if (nc == 1) {
    // one chunk: plain softmax attention (Eq. 2), independent of phi -- all gradients are zero
    if (!saved) {
      rc = launch_attn_window(c, q, k, v, phi, y, nullptr, B, H, T, HW, d, chunk, overlap, 0, 1, qtiles,
                              REHYAT_STAB_ROWMAX, false);
      if (rc != REHYAT_OK) return rc;
    }
    float* gp[8] = {(float*)grads->w1_q, (float*)grads->b1_q, (float*)grads->w2_q, (float*)grads->b2_q,
                    (float*)grads->w1_k, (float*)grads->b1_k, (float*)grads->w2_k, (float*)grads->b2_k};
    const int64_t gn[4] = {(int64_t)H * hid * d, (int64_t)H * hid, (int64_t)H * dp * hid, (int64_t)H * dp};
    for (int i = 0; i < 8; ++i) {
      hipError_t e = launch_fill_zero(gp[i], gn[i % 4], st);
      if (e != hipSuccess) return hip_fail(e, "fill kernel launch");
    }
    return REHYAT_OK;
  }

  // ---- forward pass, every chunk state kept (one window) ----------------------------
  rc = launch_state_window(c, k, v, phi, B, H, T, HW, d, chunk, overlap, 0, P.n_seg, P.nsplit);
  if (rc != REHYAT_OK) return rc;
  rc = launch_prefix_window(c, B, H, d, dp, nc, P.n_seg, P.nsplit, true);
  if (rc != REHYAT_OK) return rc;
  const float* nS = saved ? saved->nS : (const float*)(ws + P.nS);
  const float* nL = saved ? saved->nL : (const float*)(ws + P.nL);
  if (!saved) {
    rehyat_debug_out dbg;
    dbg.m = dbg.aS = dbg.aL = nullptr;
    dbg.nS = (float*)(ws + P.nS);
    dbg.nL = (float*)(ws + P.nL);
    rc = launch_attn_window(c, q, k, v, phi, y, &dbg, B, H, T, HW, d, chunk, overlap, 0, nc, qtiles,
                            REHYAT_STAB_ROWMAX, false);
    if (rc != REHYAT_OK) return rc;
  }

  hipError_t e;
  TransposeArgs tr;   // W2 [dp][hidden] -> [hidden][dp] of both maps
  tr.n = H;
  tr.R = dp;
  tr.C = hid;
  tr.in = (const bf16_t*)phi->w2_q;
  tr.out = (bf16_t*)(ws + P.w2t_q);
  tr.in2 = (const bf16_t*)phi->w2_k;
  tr.out2 = (bf16_t*)(ws + P.w2t_k);
  e = launch_transpose(tr, st);
  if (e != hipSuccess) return hip_fail(e, "transpose kernel launch");

  // ---- u, w per token ---------------------------------------------------------------
  PrepArgs pa;
  pa.g = (const bf16_t*)grad_out;
  pa.y = (const bf16_t*)y;
  pa.nS = nS;
  pa.nL = nL;
  pa.u = (bf16_t*)(ws + P.u);
  pa.tokw = (float*)(ws + P.tokw);
  pa.tokens = (int64_t)BH * N;
  pa.d = d;
  e = launch_prep(pa, st);
  if (e != hipSuccess) return hip_fail(e, "gradient preparation kernel launch");

  // ---- dL/dS_t partial sums: the chunk-state kernel on (q, u) with phi_q, query segments ---
  {
    StateArgs s;
    s.k = (const bf16_t*)q;
    s.v = (const bf16_t*)(ws + P.u);
    s.w1_k = (const bf16_t*)phi->w1_q;
    s.b1_k = (const float*)phi->b1_q;
    s.w2_k = (const bf16_t*)phi->w2_q;
    s.b2_k = (const float*)phi->b2_q;
    s.partial = (float*)(ws + P.F.partial);
    s.H = H;
    s.T = T;
    s.HW = HW;
    s.chunk = chunk;
    s.overlap = overlap;
    s.chunk0 = 1;
    s.n_seg = P.n_seg;
    s.nsplit = P.nsplit;
    s.partial_slots = P.sl.partial;
    s.n_items = BH * P.n_seg * P.nsplit;
    s.items_per_xcd = (s.n_items + 7) / 8;
    s.kv_bh_stride = N * d;
    s.step_n = 0;
    s.query_segments = 1;
    e = launch_state(s, d, s.items_per_xcd * 8, st);
    if (e != hipSuccess) return hip_fail(e, "state-gradient kernel launch");
  }

  // ---- query side ----------------------------------------------------------------------
  SideParams sq{phi->w1_q, phi->b1_q, phi->w2_q, phi->b2_q,
                (float*)grads->w1_q, (float*)grads->b1_q, (float*)grads->w2_q, (float*)grads->b2_q};
  const ChunkRange c1 = chunk_range(T, HW, chunk, overlap, 1);
  rc = backward_side(ws, P, st, q, ws + P.u, (const float*)(ws + P.tokw), sq,
                     (const bf16_t*)(ws + P.w2t_q), (const bf16_t*)(ws + P.F.state_s),
                     (const float*)(ws + P.F.state_z), true, (float*)(ws + P.p_dz), B, H, T, HW, d,
                     chunk, overlap, c1.q_lo, N);
  if (rc != REHYAT_OK) return rc;

  // ---- R_tau, r_tau ------------------------------------------------------------------
  SuffixArgs sa;
  sa.s_part = (const float*)(ws + P.F.partial);
  sa.z_part = (const float*)(ws + P.p_dz);
  sa.Rt = (bf16_t*)(ws + P.Rt);
  sa.r = (float*)(ws + P.rz);
  sa.BH = BH;
  sa.n_seg = P.n_seg;
  sa.s_nsplit = P.nsplit;
  sa.s_slots = P.sl.partial;
  sa.z_nsplit = P.nsplit;
  sa.slots = nc;
  sa.elems = d * dp + dp;
  sa.s_elems = d * dp;
  sa.dp = dp;
  e = launch_suffix(sa, st);
  if (e != hipSuccess) return hip_fail(e, "suffix kernel launch");

  // ---- key side ------------------------------------------------------------------------
  SideParams sk{phi->w1_k, phi->b1_k, phi->w2_k, phi->b2_k,
                (float*)grads->w1_k, (float*)grads->b1_k, (float*)grads->w2_k, (float*)grads->b2_k};
  const ChunkRange cl = chunk_range(T, HW, chunk, overlap, nc - 1);
  return backward_side(ws, P, st, k, v, nullptr, sk, (const bf16_t*)(ws + P.w2t_k),
                       (const bf16_t*)(ws + P.Rt), (const float*)(ws + P.rz), false, nullptr, B, H, T,
                       HW, d, chunk, overlap, 0, cl.s_lo);
}

int rehyat_debug_set_xcd_mask(unsigned mask) {
  if ((mask & 0xFFu) == 0) return REHYAT_E_SHAPE;
  g_xcd_mask.store(mask & 0xFFu);
  return REHYAT_OK;
}

int rehyat_profile_enable(int on) {
  std::lock_guard<std::mutex> lock(g_mu);
  g_prof.on = on != 0;
  g_prof.used = 0;
  return REHYAT_OK;
}

int rehyat_profile_read(double* total_ms, int* launches) {
  if (!total_ms || !launches) return REHYAT_E_NULL;
  std::lock_guard<std::mutex> lock(g_mu);
  for (int i = 0; i < kProfKinds; ++i) {
    total_ms[i] = 0.0;
    launches[i] = 0;
  }
  for (int i = 0; i < g_prof.used; ++i) {
    hipError_t e = hipEventSynchronize(g_prof.end[i]);
    float ms = 0.f;
    if (e == hipSuccess) e = hipEventElapsedTime(&ms, g_prof.beg[i], g_prof.end[i]);
    if (e != hipSuccess) {
      g_prof.used = 0;
      return hip_fail(e, "profile event read");
    }
    total_ms[g_prof.kind[i]] += ms;
    launches[g_prof.kind[i]] += 1;
  }
  g_prof.used = 0;
  return REHYAT_OK;
}

int rehyat_forward(const void* q, const void* k, const void* v, const rehyat_phi_params* phi,
                   void* out, int B, int H, int T, int HW, int d, int chunk, void* stream) {
  return rehyat_forward_ex(q, k, v, phi, out, B, H, T, HW, d, chunk, /*overlap=*/0, /*causal=*/1,
                           REHYAT_STAB_ROWMAX, nullptr, stream);
}

int rehyat_step(const void* q_t, const void* k_win, const void* v_win, const rehyat_phi_params* phi,
                float* S, float* z, void* out_t, int B, int H, int d, int n_q, int n_win,
                int n_absorb, int stab_mode, void* stream) {
  if (!q_t || !k_win || !v_win || !S || !z || !out_t) return REHYAT_E_NULL;
  if (B < 1 || H < 1 || d < 1 || n_q < 1 || n_win < 1 || n_absorb < 0) return REHYAT_E_SHAPE;
  if (n_absorb > n_win) return REHYAT_E_SHAPE;
  if ((int64_t)B * H > 65535) return REHYAT_E_SHAPE;
  if ((int64_t)B * H * ((n_q + 63) / 64) >= ((int64_t)1 << 31)) return REHYAT_E_SHAPE;
  if ((int64_t)n_win * d * 2 >= ((int64_t)1 << 31)) return REHYAT_E_SHAPE;   // 32-bit tile offsets
  if (d != 64 && d != 128) return REHYAT_E_UNSUPPORTED;
  int rc = check_phi(phi, d);
  if (rc != REHYAT_OK) return rc;
  if (stab_mode != REHYAT_STAB_ROWMAX && stab_mode != REHYAT_STAB_NONE) return REHYAT_E_SHAPE;
  if (!aligned16(q_t) || !aligned16(k_win) || !aligned16(v_win) || !aligned16(out_t) ||
      !aligned4(S) || !aligned4(z))
    return REHYAT_E_SHAPE;
  const int dp = phi->dprime;
  hipStream_t st = (hipStream_t)stream;

  std::lock_guard<std::mutex> lock(g_mu);
  Ctx c;
  c.sl = kSlots;
  c.L = ws_layout(B, H, d, dp, c.sl);
  c.st = st;
  c.prof = true;
  rc = ensure_workspace(c.L.total, st, &c.ws);
  if (rc != REHYAT_OK) return rc;
  char* ws = c.ws;
  const WsLayout& L = c.L;

  hipError_t e;
  StepStateArgs ss;
  ss.S = S;
  ss.z = z;
  ss.partial = (const float*)(ws + L.partial);
  ss.state_s = (bf16_t*)(ws + L.state_s);
  ss.state_z = (float*)(ws + L.state_z);
  ss.BH = B * H;
  ss.d = d;
  ss.dprime = dp;
  ss.partial_slots = c.sl.partial;
  ss.state_slots = c.sl.state;
  // The read-out of this chunk uses the caller's state as it is (Eq. 16): slot 0 <- S, z.  The
  // tokens that leave the window are absorbed afterwards (Eq. 17-18: state kernel in pieces,
  // then S, z += the pieces, in place and in the caller's layout); the attention kernel does
  // not depend on that and runs beside it when a second stream is at hand.
  SideStream* side = n_absorb > 0 ? side_stream(st) : nullptr;
  hipStream_t upd = side ? side->s : st;   // stream of the state update
  int nsplit = 1;
  if (n_absorb > 0) {
    // One segment only, cut into pieces: one workgroup of the state kernel fills a CU, and a
    // piece pays the workgroup's set-up (its weight slices into registers) once.  Beside the
    // attention kernel, which spreads its workgroups over as many CUs, the pieces should fit
    // the CUs it leaves free; alone, three quarters of the chip measured best (480p shape,
    // 12 heads: 8 pieces forked, 16 serial; 25 pieces of one tile each were 30 % slower).
    const int attn_wgs = B * H * ((n_q + attn_query_tile(d) - 1) / attn_query_tile(d));
    int free_cus = side ? kCUs - attn_wgs : 3 * kCUs / 4;
    if (free_cus < kCUs / 4) free_cus = kCUs / 4;
    nsplit = free_cus / (B * H);
    if (nsplit < 1) nsplit = 1;
    if (nsplit > c.sl.partial) nsplit = c.sl.partial;
    const int max_pieces = (n_absorb + 63) / 64;
    if (nsplit > max_pieces) nsplit = max_pieces;
  }
  auto launch_absorb_pieces = [&]() -> int {
    StateArgs s;
    s.k = (const bf16_t*)k_win;
    s.v = (const bf16_t*)v_win;
    s.w1_k = (const bf16_t*)phi->w1_k;
    s.b1_k = (const float*)phi->b1_k;
    s.w2_k = (const bf16_t*)phi->w2_k;
    s.b2_k = (const float*)phi->b2_k;
    s.partial = (float*)(ws + L.partial);
    s.H = H;
    s.T = s.HW = s.chunk = 1;
    s.overlap = 0;
    s.chunk0 = 0;
    s.n_seg = 1;
    s.nsplit = nsplit;
    s.partial_slots = c.sl.partial;
    s.n_items = B * H * nsplit;
    s.items_per_xcd = (s.n_items + 7) / 8;
    s.kv_bh_stride = (int64_t)n_win * d;
    s.step_n = n_absorb;
    s.query_segments = 0;
    ProfScope prof(true, 0, upd);
    hipError_t es = launch_state(s, d, s.items_per_xcd * 8, upd);
    if (es != hipSuccess) return hip_fail(es, "state kernel launch");
    return REHYAT_OK;
  };
  if (side) {
    // caller's stream: slot 0 <- state; fork; second stream: pieces, then state += pieces
    ss.nsplit = 0;
    ss.write_slot = 1;
    {
      ProfScope prof(true, 1, st);
      e = launch_step_state(ss, st);
    }
    if (e != hipSuccess) return hip_fail(e, "step state kernel launch");
    e = hipEventRecord(side->fork, st);
    if (e == hipSuccess) e = hipStreamWaitEvent(side->s, side->fork, 0);
    if (e != hipSuccess) return hip_fail(e, "fork to the second stream");
    rc = launch_absorb_pieces();
    if (rc != REHYAT_OK) return rc;
    ss.nsplit = nsplit;
    ss.write_slot = 0;
    {
      ProfScope prof(true, 1, upd);
      e = launch_step_state(ss, upd);
    }
    if (e != hipSuccess) return hip_fail(e, "step state kernel launch");
    e = hipEventRecord(side->join, side->s);
    if (e != hipSuccess) return hip_fail(e, "hipEventRecord(join)");
  } else {
    // one stream: pieces, then slot 0 <- state and state += pieces in one kernel
    if (n_absorb > 0) {
      rc = launch_absorb_pieces();
      if (rc != REHYAT_OK) return rc;
    }
    ss.nsplit = n_absorb > 0 ? nsplit : 0;
    ss.write_slot = 1;
    ProfScope prof(true, 1, st);
    e = launch_step_state(ss, st);
    if (e != hipSuccess) return hip_fail(e, "step state kernel launch");
  }

  AttnArgs a;
  a.q = (const bf16_t*)q_t;
  a.k = (const bf16_t*)k_win;
  a.v = (const bf16_t*)v_win;
  a.out = (bf16_t*)out_t;
  a.w1_q = (const bf16_t*)phi->w1_q;
  a.b1_q = (const float*)phi->b1_q;
  a.w2_q = (const bf16_t*)phi->w2_q;
  a.b2_q = (const float*)phi->b2_q;
  a.state_s = (const bf16_t*)(ws + L.state_s);
  a.state_z = (const float*)(ws + L.state_z);
  a.dbg_m = a.dbg_nS = a.dbg_aS = a.dbg_nL = a.dbg_aL = nullptr;
  a.scale_log2e = (float)(1.4426950408889634 / std::sqrt((double)d));
  a.H = H;
  a.T = a.HW = a.chunk = 1;
  a.overlap = 0;
  a.chunk0 = 0;
  a.n_win_chunks = 1;
  const int qtile = attn_query_tile(d);
  a.qtiles = (n_q + qtile - 1) / qtile;
  a.state_slots = c.sl.state;
  a.stab_mode = stab_mode;
  a.n_items = B * H * a.qtiles;
  a.items_per_xcd = (a.n_items + 7) / 8;
  a.q_bh_stride = (int64_t)n_q * d;
  a.kv_bh_stride = (int64_t)n_win * d;
  a.step_nq = n_q;
  a.step_nwin = n_win;
  a.all_linear = 0;
  a.xcd_mask = 0xFFu;   // the measurement hook covers whole-sequence calls only
  a.n_short = 0;
  {
    ProfScope prof(true, 2, st);
    e = launch_attn(a, d, a.items_per_xcd * 8, st);
  }
  if (e != hipSuccess) return hip_fail(e, "attention kernel launch");
  if (side) {   // the call's work is complete, for the caller's stream, when both branches are
    e = hipStreamWaitEvent(st, side->join, 0);
    if (e != hipSuccess) return hip_fail(e, "join of the second stream");
  }
  return REHYAT_OK;
}

int rehyat_state(const void* k, const void* v, const rehyat_phi_params* phi, float* S_out,
                 float* z_out, int B, int H, int T, int HW, int d, int upto_frames, void* stream) {
  if (!k || !v || !S_out || !z_out) return REHYAT_E_NULL;
  if (B < 1 || H < 1 || T < 1 || HW < 1 || d < 1) return REHYAT_E_SHAPE;
  if (upto_frames < 0 || upto_frames > T) return REHYAT_E_SHAPE;
  if ((int64_t)T * HW >= ((int64_t)1 << 31)) return REHYAT_E_SHAPE;
  if ((int64_t)B * H > 65535) return REHYAT_E_SHAPE;
  if (d != 64 && d != 128) return REHYAT_E_UNSUPPORTED;
  int rc = check_phi(phi, d);
  if (rc != REHYAT_OK) return rc;
  if (!aligned16(k) || !aligned16(v) || !aligned4(S_out) || !aligned4(z_out)) return REHYAT_E_SHAPE;
  const int dp = phi->dprime;
  hipStream_t st = (hipStream_t)stream;
  if (upto_frames == 0) {  // s_0 = 0, z_0 = 0 (Eq. 14-15): a fill kernel, no workspace
    hipError_t e = launch_zero_state(S_out, z_out, B * H, d, dp, st);
    if (e != hipSuccess) return hip_fail(e, "state fill kernel launch");
    return REHYAT_OK;
  }
  std::lock_guard<std::mutex> lock(g_mu);
  Ctx c;
  c.sl = kSlots;
  c.L = ws_layout(B, H, d, dp, c.sl);
  c.st = st;
  c.prof = true;
  rc = ensure_workspace(c.L.total, st, &c.ws);
  if (rc != REHYAT_OK) return rc;
  // one frame per chunk, no overlap: segment f is frame f
  const int nsplit = choose_nsplit(B * H, upto_frames, c.sl);
  int win = c.sl.partial / nsplit;
  if (win > c.sl.state) win = c.sl.state;
  for (int c0 = 0; c0 < upto_frames; c0 += win) {
    const int n_seg = (upto_frames - c0 < win) ? upto_frames - c0 : win;
    rc = launch_state_window(c, k, v, phi, B, H, T, HW, d, 1, 0, c0, n_seg, nsplit);
    if (rc != REHYAT_OK) return rc;
    rc = launch_prefix_window(c, B, H, d, dp, n_seg, n_seg, nsplit, c0 == 0);
    if (rc != REHYAT_OK) return rc;
  }
  StateOutArgs o;
  o.carry = (const float*)(c.ws + c.L.carry);
  o.S_out = S_out;
  o.z_out = z_out;
  o.BH = B * H;
  o.d = d;
  o.dprime = dp;
  hipError_t e = launch_state_out(o, st);
  if (e != hipSuccess) return hip_fail(e, "state output kernel launch");
  return REHYAT_OK;
}

}  // extern "C"
