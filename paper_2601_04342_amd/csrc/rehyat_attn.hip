// Fused hybrid-attention output kernel for gfx950.
//
// One workgroup (4 waves) owns 32*QB*4 consecutive query tokens of one chunk of
// one (batch, head); each wave owns 32*QB of them and keeps, per query, the
// running softmax maximum and sum and the d-wide numerator in MFMA accumulators.
//
//   phase S (Eq. 6, 8): exponents K Q^T over the chunk's softmax window
//            (Eq. 12), online maximum/sum, numerator V^T P.
//   phase L (Eq. 7, 9, 16): phi_q of the wave's queries (two-layer MLP, second
//            half squared), then the read-out S_t^T phi_q and z_t . phi_q of
//            the chunk state, accumulated INTO the softmax numerator and
//            normaliser -- to the MFMA pipeline the D' state rows are just D'
//            more "keys" whose weights are the phi_q features.
//   merge  (Eq. 5): divide, round to bf16, store.
//
// Everything is computed transposed (keys / features in accumulator rows,
// queries in lanes) so that per-query statistics live in one lane and each
// product's accumulator is directly the B operand of the next product.
//
// All operands that are shared by the four waves (K and V tiles, then W1, W2
// and the chunk state) travel global -> LDS with direct loads into four LDS
// tile buffers, issued one or more steps ahead of their use.
#include <cstdio>
#include <type_traits>
#include <utility>

#include "rehyat_device.h"
#include "rehyat_kernels.h"

namespace rehyat {

// The exponentials of a row are taken relative to a reference that follows the row's
// running maximum lazily: it moves only when a tile's maximum exceeds it by more than
// this many powers of two, so the rescale of the running sums is rare after the first
// tile, and weights stay below 2^kLazyMax (harmless for bf16 weights and fp32 sums; the
// final division cancels the reference).  The true maximum is tracked beside it.
constexpr float kLazyMax = 8.0f;
// Query blocks of 32 per wave.  1 -> 128-query workgroups, two resident per CU, whose
// waves share each SIMD and fill each other's stalls; 2 (one wave per SIMD with twice the
// registers, half the LDS operand traffic per MFMA) measured 30 % slower at the 480p shape.
constexpr int kAttnQB = 1;
constexpr int kAttnNW = 4;   // waves per workgroup; queries per workgroup = 32 * kAttnQB * kAttnNW

template <int D, int QB, int NWV = 4>
struct AttnShape {
  static constexpr int HID = 2 * D;
  static constexpr int DP = 2 * D;
  static constexpr int KS = D / 16;    // k-steps across the head dimension
  static constexpr int DB = D / 32;    // 32-row blocks across the head dimension
  static constexpr int NW = NWV;       // waves per workgroup
  static constexpr int NT = 64 * NWV;  // threads
  static constexpr int QW = 32 * QB;   // queries per wave
  static constexpr int QT = NWV * QW;  // queries per workgroup
  static constexpr int KT = 64;        // keys per tile
  static constexpr int TILE_BYTES = 64 * D * 2;  // one LDS tile: 64 rows of 2D bytes
  static constexpr int LPT = TILE_BYTES / (1024 * NWV);  // direct-load instructions per wave per tile
};

// per-lane byte offsets of the fragment reads inside a K / V tile
template <int D>
struct FragOffsets {
  int k[D / 16];        // A fragment of K rows r (+32 per key block), k-step ks
  int v_lo[D / 32];     // transposing read, tokens 4g..4g+3 of a 16-token step, features 32db..
  int v_hi[D / 32];     // same, tokens 8+4g..
};

template <int D>
__device__ __forceinline__ FragOffsets<D> make_frag_offsets(int lane) {
  FragOffsets<D> f;
  const int g = lane >> 5, r = lane & 31, i = lane & 15;
#pragma unroll
  for (int ks = 0; ks < D / 16; ++ks) f.k[ks] = tile_off<2 * D>(r, 16 * ks + 8 * g);
#pragma unroll
  for (int db = 0; db < D / 32; ++db) {
    const int col = 32 * db + 16 * (r >> 4) + 4 * (i & 3);
    f.v_lo[db] = tile_off<2 * D>(4 * g + (i >> 2), col);
    f.v_hi[db] = tile_off<2 * D>(8 + 4 * g + (i >> 2), col);
  }
  return f;
}

// One 64-key tile of the softmax part for the wave's 32*QB queries (Eq. 6, 8):
// exponents K Q^T, online row maximum and sum, numerator += V^T P.
// E[kb][qb] register 4i+j = (key 32kb + 8i + 4g + j, query 32qb + r).
// LDS reads are issued one batch ahead of the MFMAs that consume them; the
// scheduling barriers keep the compiler from collapsing that order.
template <int D, int QB, bool TAIL>
__device__ __forceinline__ void softmax_tile(const char* Ks, const char* Vs, const FragOffsets<D>& fo,
                                             const bf16x8 (&Qr)[QB][D / 16], f32x16 (&O)[D / 32][QB],
                                             float (&mrun)[QB], float (&mtru)[QB], float (&lrun)[QB],
                                             float sc, int valid_keys, int lane) {
  using C = AttnShape<D, QB>;
  constexpr int KS = C::KS, DB = C::DB;
  constexpr int KB_BYTES = 32 * D * 2;   // 32 rows further down the tile
  constexpr int STEP_BYTES = 16 * D * 2; // 16 rows
  const int g = lane >> 5;
  const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  f32x16 E[2][QB];

  // ---- exponents: batches of two k-steps (4 fragments) ------------------------
  bf16x8 kf[2][2][2];  // [batch parity][k-step in batch][key block]
  auto read_k = [&](int b, int par) {
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
        kf[par][t][kb] = *reinterpret_cast<const bf16x8*>(Ks + fo.k[2 * b + t] + kb * KB_BYTES);
  };
  bf16x8 vf[2][DB];    // [batch parity][feature block]
  auto read_v = [&](int step, int par) {
#pragma unroll
    for (int db = 0; db < DB; ++db) {
      i16x4 lo = lds_read_tr(reinterpret_cast<const bf16_t*>(Vs + fo.v_lo[db] + step * STEP_BYTES));
      i16x4 hi = lds_read_tr(reinterpret_cast<const bf16_t*>(Vs + fo.v_hi[db] + step * STEP_BYTES));
      vf[par][db] = join_tr(lo, hi);
    }
  };
  read_k(0, 0);
#pragma unroll
  for (int b = 0; b < KS / 2; ++b) {
    if (b + 1 < KS / 2) read_k(b + 1, (b + 1) & 1);
    else read_v(0, 0);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int qb = 0; qb < QB; ++qb)
          E[kb][qb] = mfma(kf[b & 1][t][kb], Qr[qb][2 * b + t], (b == 0 && t == 0) ? zero : E[kb][qb]);
    __builtin_amdgcn_sched_barrier(0);
  }

  // ---- online softmax: new maximum, rescale of the running sums --------------------
  float mnew[QB], alpha[QB];
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    if (TAIL) {
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int e = 0; e < 16; ++e)
          if (32 * kb + 8 * (e >> 2) + 4 * g + (e & 3) >= valid_keys) E[kb][qb][e] = -INFINITY;
    }
    float mx = fmaxf(E[0][qb][0], E[1][qb][0]);
#pragma unroll
    for (int e = 1; e < 16; ++e) mx = fmaxf(mx, fmaxf(E[0][qb][e], E[1][qb][e]));
    mx = half_swap_max(mx);
    // exponents are kept unscaled; sc = log2(e)/sqrt(d) > 0 is folded into the exp2 argument
    const float mt = mx * sc;
    mtru[qb] = fmaxf(mtru[qb], mt);
    alpha[qb] = 1.0f;
    const bool grow = mt > mrun[qb] + kLazyMax;
    if (__any(grow)) {
      const float mref = grow ? mt : mrun[qb];
      alpha[qb] = __builtin_amdgcn_exp2f(mrun[qb] - mref);
      mrun[qb] = mref;
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int e = 0; e < 16; ++e) O[db][qb][e] *= alpha[qb];
    }
    mnew[qb] = mrun[qb];
  }
  __builtin_amdgcn_sched_barrier(0);

  // ---- numerator += V^T P, one 16-key step at a time.  The weights of a step (8 per
  // lane: registers 8(step&1).. of key block step>>1) are exponentiated just before its
  // products, so that the products of one step can run under the exponentials of the next
  // (one scheduling region; the group barriers below ask for that interleave).
  float sum[QB];
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) sum[qb] = 0.f;
#pragma unroll
  for (int step = 0; step < 4; ++step) {
    if (step + 1 < 4) read_v(step + 1, (step + 1) & 1);
    bf16x8 pf[QB];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
#pragma unroll
      for (int e = 8 * (step & 1); e < 8 * (step & 1) + 8; ++e) {
        float p = __builtin_amdgcn_exp2f(__builtin_fmaf(E[step >> 1][qb][e], sc, -mnew[qb]));
        E[step >> 1][qb][e] = p;
        sum[qb] += p;
      }
      pf[qb] = acc_to_operand(E[step >> 1][qb], step & 1);
    }
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int qb = 0; qb < QB; ++qb) O[db][qb] = mfma(vf[step & 1][db], pf[qb], O[db][qb]);
  }
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) lrun[qb] = lrun[qb] * alpha[qb] + sum[qb];
  if (QB == 1 && DB == 4) {
    // step 0's weights first, then each product followed by a share of the next step's work
    __builtin_amdgcn_sched_group_barrier(0x100, 8, 0);   // V fragments of step 1
    __builtin_amdgcn_sched_group_barrier(0x002, 8, 0);
    __builtin_amdgcn_sched_group_barrier(0x400, 8, 0);
    __builtin_amdgcn_sched_group_barrier(0x002, 12, 0);
#pragma unroll
    for (int s2 = 0; s2 < 3; ++s2)
#pragma unroll
      for (int m = 0; m < 4; ++m) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        if (s2 < 2) __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
        __builtin_amdgcn_sched_group_barrier(0x002, 2, 0);
        __builtin_amdgcn_sched_group_barrier(0x400, 2, 0);
        __builtin_amdgcn_sched_group_barrier(0x002, 3, 0);
      }
    __builtin_amdgcn_sched_group_barrier(0x008, 4, 0);
  }
  __builtin_amdgcn_sched_barrier(0);
}

// ---------------------------------------------------------------------------
// Phase L operand tiles and the order in which they stream through the four
// LDS tile buffers.  Tile kinds:
//   W1 tile j : W1 rows [64j, 64j+64), rows of 2D bytes (contiguous in memory)
//   W2 tile pb: W2 rows [32pb, 32pb+32); tile rows 0..31 hold their first k-half
//               (2D bytes), tile rows 32..63 the second
//   S tile pp : S_t^T columns [64pp, 64pp+64) of all D rows, rows of 128 bytes
// A step needs its tiles landed (at most `younger` tiles issued after them may
// still be in flight) and, after its barrier, issues up to two further tiles
// into buffers whose last readers have passed that barrier.
// ---------------------------------------------------------------------------
struct LinStep {
  int younger;        // tiles that may still be in flight when the step starts
  int n_issue;        // tiles issued after the step's barrier
  int kind[2], idx[2], buf[2];
  int buf_w, buf_s;   // buffers read by the step (W1 or W2 tile; S tile)
};
enum { kW1 = 0, kW2 = 1, kS = 2 };

template <int D>
struct LinSched;
template <>
struct LinSched<128> {   // 4 W1 steps, then 8 feature-block steps
  static constexpr int NPRO = 4;
  static constexpr LinStep pro(int i) { return LinStep{0, 1, {kW1, 0}, {i, 0}, {i, 0}, 0, 0}; }
  static constexpr LinStep step(int st) {
    switch (st) {
      case 0: return LinStep{3, 0, {0, 0}, {0, 0}, {0, 0}, 0, 0};
      case 1: return LinStep{2, 1, {kS, 0}, {0, 0}, {0, 0}, 1, 0};
      case 2: return LinStep{2, 1, {kW2, 0}, {0, 0}, {1, 0}, 2, 0};
      case 3: return LinStep{2, 1, {kW2, 0}, {1, 0}, {2, 0}, 3, 0};
      case 4: return LinStep{1, 1, {kS, 0}, {1, 0}, {3, 0}, 1, 0};
      case 5: return LinStep{1, 1, {kW2, 0}, {2, 0}, {1, 0}, 2, 0};
      case 6: return LinStep{0, 2, {kW2, kS}, {3, 2}, {2, 0}, 1, 3};
      case 7: return LinStep{1, 1, {kW2, 0}, {4, 0}, {1, 0}, 2, 3};
      case 8: return LinStep{0, 2, {kW2, kS}, {5, 3}, {2, 3}, 1, 0};
      case 9: return LinStep{1, 1, {kW2, 0}, {6, 0}, {1, 0}, 2, 0};
      case 10: return LinStep{0, 1, {kW2, 0}, {7, 0}, {2, 0}, 1, 3};
      default: return LinStep{0, 0, {0, 0}, {0, 0}, {0, 0}, 2, 3};
    }
  }
};
template <>
struct LinSched<64> {    // 2 W1 steps, then 4 feature-block steps
  static constexpr int NPRO = 4;
  static constexpr LinStep pro(int i) {
    switch (i) {
      case 0: return LinStep{0, 1, {kW1, 0}, {0, 0}, {0, 0}, 0, 0};
      case 1: return LinStep{0, 1, {kW1, 0}, {1, 0}, {1, 0}, 0, 0};
      case 2: return LinStep{0, 1, {kS, 0}, {0, 0}, {2, 0}, 0, 0};
      default: return LinStep{0, 1, {kW2, 0}, {0, 0}, {3, 0}, 0, 0};
    }
  }
  static constexpr LinStep step(int st) {
    switch (st) {
      case 0: return LinStep{3, 0, {0, 0}, {0, 0}, {0, 0}, 0, 0};
      case 1: return LinStep{2, 1, {kW2, 0}, {1, 0}, {0, 0}, 1, 0};
      case 2: return LinStep{1, 1, {kS, 0}, {1, 0}, {1, 0}, 3, 2};
      case 3: return LinStep{1, 1, {kW2, 0}, {2, 0}, {3, 0}, 0, 2};
      case 4: return LinStep{0, 1, {kW2, 0}, {3, 0}, {0, 0}, 3, 1};
      default: return LinStep{0, 0, {0, 0}, {0, 0}, {0, 0}, 0, 1};
    }
  }
};

template <int D, int ST>
struct LinStepC { static constexpr LinStep value = LinSched<D>::step(ST); };
template <int D, int I>
struct LinProC { static constexpr LinStep value = LinSched<D>::pro(I); };

// compile-time loop: f(integral_constant<int, 0>) ... f(integral_constant<int, N-1>)
template <typename F, int... I>
__device__ __forceinline__ void static_for_impl(F&& f, std::integer_sequence<int, I...>) {
  (f(std::integral_constant<int, I>{}), ...);
}
template <int N, typename F>
__device__ __forceinline__ void static_for(F&& f) {
  static_for_impl(f, std::make_integer_sequence<int, N>{});
}

// second bound: waves per SIMD the register budget is sized for
template <int D, int QB, int NWV>
__global__ void __launch_bounds__(64 * NWV, (QB == 1 ? 2 : 1))
attn_kernel(AttnArgs a) {
  using C = AttnShape<D, QB, NWV>;
  constexpr int HID = C::HID, DP = C::DP, KS = C::KS, DB = C::DB, NT = C::NT;
  constexpr int TB = C::TILE_BYTES, LPT = C::LPT;
  // Four tile buffers, declared as separate objects so that a pending direct
  // load into one of them does not make the compiler wait before reads of
  // another.  Phase S: K tiles in A0/A1, V tiles in A2/A3 (even/odd tile).
  __shared__ __attribute__((aligned(1024))) char A0[TB];
  __shared__ __attribute__((aligned(1024))) char A1[TB];
  __shared__ __attribute__((aligned(1024))) char A2[TB];
  __shared__ __attribute__((aligned(1024))) char A3[TB];
  __shared__ __attribute__((aligned(16))) float sb1[HID];
  __shared__ __attribute__((aligned(16))) float sb2[DP];
  __shared__ __attribute__((aligned(16))) float sz[DP];

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave-uniform for the compiler too
  const int g = lane >> 5;
  const int r = lane & 31;

  // ---- which work item -------------------------------------------------
  if (!((a.xcd_mask >> (blockIdx.x & 7)) & 1u)) return;   // measurement hook; all bits set normally
  int qt, tc, bh;
  if (a.n_short == 0) {
    const int item = xcd_swizzle(blockIdx.x, a.items_per_xcd);
    if (item >= a.n_items) return;
    // item = (bh * n_win_chunks + tc) * qtiles + qt, qt fastest
    qt = item % a.qtiles;
    const int rest = item / a.qtiles;
    tc = rest % a.n_win_chunks;
    bh = rest / a.n_win_chunks;
  } else {
    // The window starts at chunk 0, whose items have no read-out phase and are the shortest:
    // every XCD runs its share of them last, so that the launch does not end on long items.
    const int xcd = blockIdx.x & 7, i = blockIdx.x >> 3;
    const int n_long = a.n_items - a.n_short;
    const int per_long = (n_long + 7) / 8, per_short = (a.n_short + 7) / 8;
    if (i < per_long) {
      const int li = xcd * per_long + i;
      if (li >= n_long) return;
      const int per_bh = (a.n_win_chunks - 1) * a.qtiles;
      bh = li / per_bh;
      const int rest = li % per_bh;
      tc = 1 + rest / a.qtiles;
      qt = rest % a.qtiles;
    } else {
      const int si = xcd * per_short + (i - per_long);
      if (si >= a.n_short) return;
      bh = si / a.qtiles;
      tc = 0;
      qt = si % a.qtiles;
    }
  }
  const int t = a.chunk0 + tc;
  const int h = bh % a.H;
  ChunkRange cr;
  if (a.step_nq > 0) {  // streaming step: explicit ranges, state always read
    cr.q_lo = 0;
    cr.q_hi = a.step_nq;
    cr.s_lo = 0;
    cr.s_hi = a.step_nwin;
    cr.l_hi = 1;
  } else {
    cr = chunk_range(a.T, a.HW, a.chunk, a.overlap, t);
    if (a.all_linear) cr.l_hi = 1;
  }
  const int64_t q0 = cr.q_lo + (int64_t)qt * C::QT;
  if (q0 >= cr.q_hi) return;  // short last chunk: fewer query tiles
  const int64_t N = (int64_t)a.T * a.HW;  // rows per (b, h) of the debug outputs
  const bf16_t* Qg = a.q + (int64_t)bh * a.q_bh_stride;
  const bf16_t* Kg = a.k + (int64_t)bh * a.kv_bh_stride;
  const bf16_t* Vg = a.v + (int64_t)bh * a.kv_bh_stride;
  bf16_t* Og = a.out + (int64_t)bh * a.q_bh_stride;
  const bool has_linear = cr.l_hi > 0;

  // ---- queries of this wave, held as B operands ---------------------------
  const int64_t qw0 = q0 + wave * C::QW;
  // a wave whose 32 queries all lie beyond the chunk (last query tile) still moves its
  // share of every tile and meets every barrier, but computes nothing
  const bool wave_live = qw0 < cr.q_hi;
  bf16x8 Qr[QB][KS];
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    int64_t row = qw0 + 32 * qb + r;
    if (row > cr.q_hi - 1) row = cr.q_hi - 1;
    const bf16_t* p = Qg + row * D + 8 * g;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks)
      Qr[qb][ks] = *reinterpret_cast<const bf16x8*>(p + 16 * ks);
  }

  // numerator: O[db][qb] register 4i+j = (row d = 32db + 8i + 4g + j, query 32qb + r)
  f32x16 O[DB][QB];
#pragma unroll
  for (int db = 0; db < DB; ++db)
#pragma unroll
    for (int qb = 0; qb < QB; ++qb)
#pragma unroll
      for (int e = 0; e < 16; ++e) O[db][qb][e] = 0.f;
  float mrun[QB];  // reference of the exponentials (log2 units), lags the running maximum
  float mtru[QB];  // running maximum of exponent * log2(e)/sqrt(d)
  float lrun[QB];  // this lane half's share of the sum
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    mrun[qb] = -INFINITY;
    mtru[qb] = -INFINITY;
    lrun[qb] = 0.f;
  }
  const float sc = a.scale_log2e;

  // =========================== phase S =====================================
  {
    const FragOffsets<D> fo = make_frag_offsets<D>(lane);
    const int64_t s_lo = cr.s_lo, s_hi = cr.s_hi;
    const int n_full = (int)((s_hi - s_lo) / 64);
    const int rem = (int)((s_hi - s_lo) - 64 * (int64_t)((s_hi - s_lo) / 64));  // keys in the ragged last tile
    const char* const Kb = reinterpret_cast<const char*>(Kg + s_lo * D);
    const char* const Vb = reinterpret_cast<const char*>(Vg + s_lo * D);
    auto contiguous = [](int R) { return R * (2 * D); };
    // K and V of tile `it` into the given buffers
    auto run_tile = [&](auto TAILC, const char* Kt, const char* Vt, int valid) {
      constexpr bool TAIL = decltype(TAILC)::value;
      softmax_tile<D, QB, TAIL>(Kt, Vt, fo, Qr, O, mrun, mtru, lrun, sc, valid, lane);
    };
    const __amdgpu_buffer_rsrc_t Kr = make_rsrc(Kb), Vr = make_rsrc(Vb);
    auto issue_kv = [&](int it, char* kd, char* vd) {
      tile_load_buffer<2 * D, TB, NWV>(Kr, it * TB, kd, wave, lane, contiguous);
      tile_load_buffer<2 * D, TB, NWV>(Vr, it * TB, vd, wave, lane, contiguous);
    };
    if (n_full > 0) issue_kv(0, A0, A2);
      // per-head vectors of phase L (their loads complete long before phase L, whose
      // counted waits must see tile loads only)
    if (has_linear) {
      const float* zt = a.state_z + ((int64_t)bh * a.state_slots + tc) * DP;
      for (int i = tid; i < HID; i += NT) sb1[i] = a.b1_q[(int64_t)h * HID + i];
      for (int i = tid; i < DP; i += NT) {
        sb2[i] = a.b2_q[(int64_t)h * DP + i];
        sz[i] = zt[i];
      }
    }
    wait_loads_and_barrier<0>();   // also publishes the bias vectors
    // Two tiles per trip so that buffer choice is static.  The loads of tile
    // it+1 go into the other buffer pair, whose last readers (tile it-1) all
    // passed the barrier that ended the previous tile; they must have landed,
    // for every wave, by the barrier that ends tile it.
    for (int it = 0; it < n_full; it += 2) {
      if (it + 1 < n_full) issue_kv(it + 1, A1, A3);
      if (wave_live) run_tile(std::false_type{}, A0, A2, 64);
      wait_loads_and_barrier<0>();
      if (it + 1 < n_full) {
        if (it + 2 < n_full) issue_kv(it + 2, A0, A2);
        if (wave_live) run_tile(std::false_type{}, A1, A3, 64);
        wait_loads_and_barrier<0>();
      }
    }
    if (rem > 0) {
      // ragged last tile, outside the loop so that its index math is not kept
      // live in it; rows beyond the window re-read the last valid row (finite
      // values) and their keys are masked
      const int64_t goff = (int64_t)((s_hi - s_lo) / 64) * TB;
      auto clamped = [rem](int R) { return (R < rem ? R : rem - 1) * (2 * D); };
      tile_load_direct<2 * D, TB, NWV>(Kb + goff, A0, wave, lane, clamped);
      tile_load_direct<2 * D, TB, NWV>(Vb + goff, A2, wave, lane, clamped);
      wait_loads_and_barrier<0>();
      if (wave_live) run_tile(std::true_type{}, A0, A2, rem);
      wait_loads_and_barrier<0>();
    }
  }

  // complete the softmax normaliser across the two lane halves
  // All sums are relative to 2^-mrun; the components are reported relative to the
  // true maximum: dscale = 2^(mrun - mtru) <= 1.
  float nS[QB], dscale[QB];
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    nS[qb] = half_swap_sum(lrun[qb]);
    dscale[qb] = __builtin_amdgcn_exp2f(mrun[qb] - mtru[qb]);
  }

  // debug: softmax components
  if (a.dbg_m || a.dbg_nS || a.dbg_aS) {
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
      const int64_t row = qw0 + 32 * qb + r;
      if (row < cr.q_hi) {
        const int64_t o = (int64_t)bh * N + row;
        if (g == 0) {
          if (a.dbg_m) a.dbg_m[o] = mtru[qb] * 0.6931471805599453f;  // back from base 2
          if (a.dbg_nS) a.dbg_nS[o] = nS[qb] * dscale[qb];
        }
        if (a.dbg_aS) {
#pragma unroll
          for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
              f32x4 x = {O[db][qb][4 * i], O[db][qb][4 * i + 1], O[db][qb][4 * i + 2], O[db][qb][4 * i + 3]};
              *reinterpret_cast<f32x4*>(a.dbg_aS + o * D + 32 * db + 8 * i + 4 * g) = x * dscale[qb];
            }
        }
      }
    }
    // the counted waits of phase L must see tile loads only
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  }

  // =========================== phase L =====================================
  // The 32 rows of a W1 / W2 block are read in "quad-swapped" order (lane r takes
  // block row sigma(r), sigma exchanging bits 2 and 3 of r), so that the
  // accumulator of one product is, register for register, the B operand of the
  // next one in natural k order and no operand needs a permuted copy in memory.
  float nL[QB];
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) nL[qb] = 0.f;
  if (has_linear) {
    using SCH = LinSched<D>;
    constexpr int NW1 = HID / 64, NPB = DP / 32;
    const char* W1 = reinterpret_cast<const char*>(a.w1_q + (int64_t)h * HID * D);
    const char* W2 = reinterpret_cast<const char*>(a.w2_q + (int64_t)h * DP * HID);
    const char* St = reinterpret_cast<const char*>(a.state_s + ((int64_t)bh * a.state_slots + tc) * (int64_t)D * DP);

    const __amdgpu_buffer_rsrc_t W1r = make_rsrc(W1), W2r = make_rsrc(W2), Str = make_rsrc(St);
    auto issue_tile = [&](auto KIND, int idx, char* dst) {
      constexpr int kind = decltype(KIND)::value;
      if constexpr (kind == kW1) {
        tile_load_buffer<2 * D, TB, NWV>(W1r, idx * TB, dst, wave, lane, [](int R) { return R * (2 * D); });
      } else if constexpr (kind == kW2) {
        tile_load_buffer<2 * D, TB, NWV>(W2r, idx * 32 * (4 * D), dst, wave, lane,
                                       [](int R) { return (R & 31) * (4 * D) + (R >> 5) * (2 * D); });
      } else {
        tile_load_buffer<128, TB, NWV>(Str, idx * 128, dst, wave, lane, [](int R) { return R * (4 * D); });
      }
    };
    auto buf = [&](auto I) -> char* {
      constexpr int i = decltype(I)::value;
      if constexpr (i == 0) return A0;
      else if constexpr (i == 1) return A1;
      else if constexpr (i == 2) return A2;
      else return A3;
    };
    auto issue_all = [&](auto SD) {   // the tiles a step (or the prologue) issues
      constexpr LinStep sd = decltype(SD)::value;
      if constexpr (sd.n_issue > 0)
        issue_tile(std::integral_constant<int, sd.kind[0]>{}, sd.idx[0], buf(std::integral_constant<int, sd.buf[0]>{}));
      if constexpr (sd.n_issue > 1)
        issue_tile(std::integral_constant<int, sd.kind[1]>{}, sd.idx[1], buf(std::integral_constant<int, sd.buf[1]>{}));
    };
    // all K/V tiles are dead: the softmax loop ended with a barrier
    static_for<SCH::NPRO>([&](auto I) {
      issue_all(LinProC<D, decltype(I)::value>{});
    });

    // The softmax sums are relative to 2^-mrun: with c_i = row maximum (Eq. 6, 8) the
    // linear terms weigh 2^(mtru - mrun) beside them, with c = 0 they weigh 2^-mrun.
    float lin_scale[QB];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb)
      lin_scale[qb] = __builtin_amdgcn_exp2f((a.stab_mode == 1 ? 0.f : mtru[qb]) - mrun[qb]);

    // per-lane byte offsets inside a W tile: block row sigma(r), k-step ks
    const int sr = (r & 0x13) | ((r & 4) << 1) | ((r & 8) >> 1);
    int woff[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) woff[ks] = tile_off<2 * D>(sr, 16 * ks + 8 * g);
    // accumulator register 4i+j of lane half g is block row 8i+4g+j, which after
    // the row permutation is unit 16(i>>1) + 8g + 4(i&1) + j of the block
    auto unit_of = [&](int i) { return 16 * (i >> 1) + 8 * g + 4 * (i & 1); };

    bf16x8 Ub[QB][HID / 16];  // U^T = relu(W1 Q^T + b1) as B operands, natural k order
    static_for<NW1 + NPB>([&](auto ST) {
      constexpr int st = decltype(ST)::value;
      constexpr LinStep sd = LinStepC<D, st>::value;
      wait_loads_and_barrier<sd.younger * LPT>();
      issue_all(LinStepC<D, st>{});
      if (!wave_live) return;  // this step of this wave only (the lambda is one step)
      if constexpr (st < NW1) {
        // ---- two 32-row blocks of hidden units ------------------------------------
        const char* Ws = buf(std::integral_constant<int, sd.buf_w>{});
#pragma unroll
        for (int hb2 = 0; hb2 < 2; ++hb2) {
          const int hb = 2 * st + hb2;
          f32x16 acc[QB];
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            f32x4 bias = *reinterpret_cast<const f32x4*>(sb1 + 32 * hb + unit_of(i));
#pragma unroll
            for (int j = 0; j < 4; ++j)
#pragma unroll
              for (int qb = 0; qb < QB; ++qb) acc[qb][4 * i + j] = bias[j];
          }
#pragma unroll
          for (int ks = 0; ks < KS; ++ks) {
            bf16x8 wf = *reinterpret_cast<const bf16x8*>(Ws + hb2 * (32 * 2 * D) + woff[ks]);
#pragma unroll
            for (int qb = 0; qb < QB; ++qb) acc[qb] = mfma(wf, Qr[qb][ks], acc[qb]);
          }
#pragma unroll
          for (int qb = 0; qb < QB; ++qb) {
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[qb][e] = fmaxf(acc[qb][e], 0.f);
            Ub[qb][2 * hb + 0] = acc_to_operand(acc[qb], 0);
            Ub[qb][2 * hb + 1] = acc_to_operand(acc[qb], 1);
          }
        }
      } else {
        // ---- 32 features: psi^T = relu(W2 U^T + b2), phi, read-out ------------------
        const int pb = st - NW1;
        const char* Ws = buf(std::integral_constant<int, sd.buf_w>{});
        const char* Ss = buf(std::integral_constant<int, sd.buf_s>{});
        f32x16 acc[QB];
        float zv[16];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          f32x4 bias = *reinterpret_cast<const f32x4*>(sb2 + 32 * pb + unit_of(i));
          f32x4 zz = *reinterpret_cast<const f32x4*>(sz + 32 * pb + unit_of(i));
#pragma unroll
          for (int j = 0; j < 4; ++j) {
#pragma unroll
            for (int qb = 0; qb < QB; ++qb) acc[qb][4 * i + j] = bias[j];
            zv[4 * i + j] = zz[j];
          }
        }
#pragma unroll
        for (int half = 0; half < 2; ++half) {
#pragma unroll
          for (int ks = 0; ks < KS; ++ks) {
            bf16x8 wf = *reinterpret_cast<const bf16x8*>(Ws + half * (32 * 2 * D) + woff[ks]);
#pragma unroll
            for (int qb = 0; qb < QB; ++qb) acc[qb] = mfma(wf, Ub[qb][half * KS + ks], acc[qb]);
          }
        }
        const bool squared = (32 * pb >= DP / 2);
        bf16x8 Fb[QB][2];
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) {
          float part = 0.f;
#pragma unroll
          for (int e = 0; e < 16; ++e) {
            float x = fmaxf(acc[qb][e], 0.f);
            if (squared) x = x * x;
            // the read-out below rounds x to bf16 (MFMA operand); the normaliser takes it
            // unrounded: the 256 rounding errors of a row have random signs and relative size
            // 2^-9, far below the bar on n^L, and the rounding costs two instructions per feature
            x = x * lin_scale[qb];
            acc[qb][e] = x;
            part += x * zv[e];
          }
          nL[qb] += part;
          Fb[qb][0] = acc_to_operand(acc[qb], 0);
          Fb[qb][1] = acc_to_operand(acc[qb], 1);
        }
        // S tile: rows d, 64 columns = two feature blocks; this block's 32 columns
        // start at 32(pb&1), k-step sidx of it is chunk 4(pb&1) + 2 sidx + g
#pragma unroll
        for (int sidx = 0; sidx < 2; ++sidx) {
#pragma unroll
          for (int db = 0; db < DB; ++db) {
            const int row = 32 * db + r;
            const int c = (4 * (pb & 1) + 2 * sidx) | g;
            bf16x8 sf = *reinterpret_cast<const bf16x8*>(Ss + row * 128 + ((c ^ swz<128>(row)) << 4));
#pragma unroll
            for (int qb = 0; qb < QB; ++qb) O[db][qb] = mfma(sf, Fb[qb][sidx], O[db][qb]);
          }
        }
      }
    });
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) nL[qb] = half_swap_sum(nL[qb]);
  }

  // =========================== merge (Eq. 5) ================================
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    const int64_t row = qw0 + 32 * qb + r;
    if (row >= cr.q_hi) continue;
    const int64_t o = (int64_t)bh * N + row;
    if (g == 0 && a.dbg_nL) a.dbg_nL[o] = nL[qb] * dscale[qb];
    const float inv = 1.0f / (nS[qb] + nL[qb]);
#pragma unroll
    for (int db = 0; db < DB; ++db) {
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int col = 32 * db + 8 * i + 4 * g;
        if (a.dbg_aL) {
          f32x4 as = {0.f, 0.f, 0.f, 0.f};
          if (a.dbg_aS) as = *reinterpret_cast<const f32x4*>(a.dbg_aS + o * D + col);
          const float ds = dscale[qb];
          f32x4 x;
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            // the product is rounded as it was when a^S was stored (no fused multiply-subtract),
            // so an empty linear set reports exactly zero
            float t = O[db][qb][4 * i + j] * ds;
            asm volatile("" : "+v"(t));
            x[j] = t - as[j];
          }
          *reinterpret_cast<f32x4*>(a.dbg_aL + o * D + col) = x;
        }
        u32x2 pk;
        pk[0] = pack_bf16(O[db][qb][4 * i] * inv, O[db][qb][4 * i + 1] * inv);
        pk[1] = pack_bf16(O[db][qb][4 * i + 2] * inv, O[db][qb][4 * i + 3] * inv);
        *reinterpret_cast<u32x2*>(Og + row * D + col) = pk;
      }
    }
  }
}

int attn_query_tile(int d) { return AttnShape<128, kAttnQB, kAttnNW>::QT; }

const char* attn_kernel_name(int d) {
  static char name[2][48];
  char* n = name[d == 128 ? 0 : 1];
  snprintf(n, sizeof(name[0]), "attn_kernel<%d, %d, %d>", d == 128 ? 128 : 64, kAttnQB, kAttnNW);
  return n;
}

hipError_t launch_attn(const AttnArgs& a, int d, int grid, hipStream_t stream) {
  if (d == 128) {
    hipLaunchKernelGGL((attn_kernel<128, kAttnQB, kAttnNW>), dim3(grid), dim3(64 * kAttnNW), 0, stream, a);
  } else {
    hipLaunchKernelGGL((attn_kernel<64, kAttnQB, kAttnNW>), dim3(grid), dim3(64 * kAttnNW), 0, stream, a);
  }
  return hipGetLastError();
}

}  // namespace rehyat
