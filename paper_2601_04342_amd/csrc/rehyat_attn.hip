// Fused hybrid-attention output kernel for gfx950.
//
// One workgroup (4 waves) owns 256 consecutive query tokens of one chunk of one
// (batch, head); each wave owns 64 of them and keeps, per query, the running
// softmax maximum and sum and the d-wide numerator in MFMA accumulators.
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
#include <cstdlib>

#include "rehyat_device.h"
#include "rehyat_kernels.h"

namespace rehyat {

// query blocks of 32 per wave: 1 -> 128-query workgroups, two resident per CU;
// 2 -> 256-query workgroups, one per CU
#ifndef REHYAT_ATTN_QB
#define REHYAT_ATTN_QB 1
#endif
constexpr int kAttnQB = REHYAT_ATTN_QB;

template <int D, int QB>
struct AttnShape {
  static constexpr int HID = 2 * D;
  static constexpr int DP = 2 * D;
  static constexpr int KS = D / 16;    // k-steps across the head dimension
  static constexpr int DB = D / 32;    // 32-row blocks across the head dimension
  static constexpr int NT = 256;       // threads
  static constexpr int QW = 32 * QB;   // queries per wave
  static constexpr int QT = 4 * QW;    // queries per workgroup
  static constexpr int KT = 64;        // keys per tile
  static constexpr int TILE_BYTES = 64 * D * 2;  // one K or V tile in LDS (unpadded, chunk-swizzled)
  // phase L tiles (padded rows, staged through registers)
  static constexpr int LDK = D + 8;    // W1 slab row stride
  static constexpr int LDW2 = HID + 8; // W2 slab row stride
  static constexpr int LDS_S = 32 + 8; // state slab row stride
  static constexpr int BUFA = (64 * LDK > 32 * LDW2) ? 64 * LDK : 32 * LDW2;  // elements
  static constexpr int BUFB = D * LDS_S;
  static_assert(BUFA * 2 <= 2 * TILE_BYTES && BUFB * 2 <= 2 * TILE_BYTES, "phase L tiles alias the K/V tiles");
};

// ---------------------------------------------------------------------------
// K/V tiles in LDS: [64 rows][D] bf16 with unpadded rows, filled by direct
// global->LDS loads (each wave instruction moves 1 KB to consecutive LDS
// bytes, so rows cannot be padded).  Bank conflicts are avoided by permuting
// the 16-byte chunks of a row: chunk c of row `row` is stored at chunk position
// c ^ swz(row).  swz is a bijection of the rows that a 32x32x16 A-fragment read
// touches together (16 consecutive rows, same chunk) onto chunk positions, and
// it also separates the 4 consecutive rows that one transposing read touches.
// ---------------------------------------------------------------------------
template <int D>
__device__ __forceinline__ int swz(int row) {
  if (D == 128) return ((row & 3) << 2) | ((row >> 2) & 3);   // 16 chunks per 256-byte row
  return (((row >> 1) & 1) << 2) | ((row >> 2) & 3);           // 8 chunks per 128-byte row
}

// byte offset of element (row, col) inside a tile
template <int D>
__device__ __forceinline__ int tile_off(int row, int col) {
  return row * (2 * D) + ((((col >> 3) ^ swz<D>(row)) << 4) | ((col & 7) << 1));
}

// Direct loads of one 64-row tile: wave w moves the 1 KB blocks w, w+4, ...
// Lane i of a block fills LDS chunk slot i, so it fetches the global chunk that
// the swizzle assigns to that slot; swz depends on the row modulo 16 only, so a
// lane's byte offset inside the tile is `lane_off` for its first block and
// grows by 4096 per further block.
template <int D>
__device__ __forceinline__ int tile_lane_offset(int wave, int lane) {
  constexpr int CPR = D / 8;     // 16-byte chunks per row
  constexpr int RPB = 64 / CPR;  // rows per 1 KB block
  const int row = wave * RPB + lane / CPR;
  const int c = (lane % CPR) ^ swz<D>(row);
  return row * (2 * D) + c * 16;
}

template <int D>
__device__ __forceinline__ void tile_load_direct(const char* gtile, char* lds_tile, int lane_off, int wave) {
  constexpr int NBLK = (64 * 2 * D) / 1024;  // 1 KB blocks per tile
#pragma unroll
  for (int n = 0; n < NBLK / 4; ++n) {
    const char* src = gtile + (uint32_t)(lane_off + n * 4096);
    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)src,
                                     (__attribute__((address_space(3))) void*)(lds_tile + (wave + 4 * n) * 1024),
                                     16, 0, 0);
  }
}

// Same for a tile with only `valid_rows` rows in bounds: rows beyond re-read the
// last valid row (finite values; their keys are masked in the softmax).
template <int D>
__device__ __forceinline__ void tile_load_direct_tail(const char* gtile, char* lds_tile, int valid_rows,
                                                      int wave, int lane) {
  constexpr int CPR = D / 8;
  constexpr int RPB = 64 / CPR;
  constexpr int NBLK = (64 * 2 * D) / 1024;
#pragma unroll
  for (int n = 0; n < NBLK / 4; ++n) {
    const int j = wave + 4 * n;
    const int row = j * RPB + lane / CPR;
    const int c = (lane % CPR) ^ swz<D>(row);
    const int grow = row < valid_rows ? row : valid_rows - 1;
    const char* src = gtile + (uint32_t)(grow * (2 * D) + c * 16);
    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)src,
                                     (__attribute__((address_space(3))) void*)(lds_tile + j * 1024), 16, 0, 0);
  }
}

// per-lane byte offsets of the fragment reads inside a tile
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
  for (int ks = 0; ks < D / 16; ++ks) f.k[ks] = tile_off<D>(r, 16 * ks + 8 * g);
#pragma unroll
  for (int db = 0; db < D / 32; ++db) {
    const int col = 32 * db + 16 * (r >> 4) + 4 * (i & 3);
    f.v_lo[db] = tile_off<D>(4 * g + (i >> 2), col);
    f.v_hi[db] = tile_off<D>(8 + 4 * g + (i >> 2), col);
  }
  return f;
}

__device__ __forceinline__ bf16x8 join_tr(i16x4 lo, i16x4 hi) {
  typedef __attribute__((__vector_size__(8 * sizeof(short)))) short i16x8;
  i16x8 v = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
  return __builtin_bit_cast(bf16x8, v);
}

// One 64-key tile of the softmax part for the wave's 32*QB queries (Eq. 6, 8):
// exponents K Q^T, online row maximum and sum, numerator += V^T P.
// E[kb][qb] register 4i+j = (key 32kb + 8i + 4g + j, query 32qb + r).
// LDS reads are issued one batch ahead of the MFMAs that consume them; the
// scheduling barriers keep the compiler from collapsing that order.
template <int D, int QB, bool TAIL>
__device__ __forceinline__ void softmax_tile(const char* Ks, const char* Vs, const FragOffsets<D>& fo,
                                             const bf16x8 (&Qr)[QB][D / 16], f32x16 (&O)[D / 32][QB],
                                             float (&mrun)[QB], float (&lrun)[QB], float sc,
                                             int valid_keys, int lane) {
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

  // ---- online softmax -----------------------------------------------------------
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
    const float mnew = fmaxf(mrun[qb], mx * sc);
    const float alpha = __builtin_amdgcn_exp2f(mrun[qb] - mnew);
    mrun[qb] = mnew;
    float sum = 0.f;
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        float p = __builtin_amdgcn_exp2f(__builtin_fmaf(E[kb][qb][e], sc, -mnew));
        E[kb][qb][e] = p;
        sum += p;
      }
    lrun[qb] = lrun[qb] * alpha + sum;
    if (__any(alpha != 1.0f)) {
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int e = 0; e < 16; ++e) O[db][qb][e] *= alpha;
    }
  }
  __builtin_amdgcn_sched_barrier(0);

  // ---- numerator += V^T P, one 16-key step at a time --------------------------------
#pragma unroll
  for (int step = 0; step < 4; ++step) {
    if (step + 1 < 4) read_v(step + 1, (step + 1) & 1);
    __builtin_amdgcn_sched_barrier(0);
    bf16x8 pf[QB];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) pf[qb] = acc_to_operand(E[step >> 1][qb], step & 1);
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int qb = 0; qb < QB; ++qb) O[db][qb] = mfma(vf[step & 1][db], pf[qb], O[db][qb]);
    __builtin_amdgcn_sched_barrier(0);
  }
}

template <int D, int QB>
__global__ void __launch_bounds__(256, (QB == 1 ? 2 : 1))
attn_kernel(AttnArgs a) {
  using C = AttnShape<D, QB>;
  constexpr int HID = C::HID, DP = C::DP, KS = C::KS, DB = C::DB, NT = C::NT;
  // K tiles (two buffers) then V tiles (two buffers); phase L reuses the memory
  __shared__ __attribute__((aligned(1024))) char smem[4 * C::TILE_BYTES];
  bf16_t* const bufA = reinterpret_cast<bf16_t*>(smem);                       // phase L: W1 / W2 slabs
  bf16_t* const bufB = reinterpret_cast<bf16_t*>(smem + 2 * C::TILE_BYTES);   // phase L: state slabs
  __shared__ __attribute__((aligned(16))) float sb1[HID];
  __shared__ __attribute__((aligned(16))) float sb2[DP];
  __shared__ __attribute__((aligned(16))) float sz[DP];

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int g = lane >> 5;
  const int r = lane & 31;

  // ---- which work item -------------------------------------------------
  const int item = xcd_swizzle(blockIdx.x, a.items_per_xcd);
  if (item >= a.n_items) return;
  // item = (bh * n_win_chunks + tc) * qtiles + qt, qt fastest
  const int qt = item % a.qtiles;
  const int rest = item / a.qtiles;
  const int tc = rest % a.n_win_chunks;
  const int bh = rest / a.n_win_chunks;
  const int t = a.chunk0 + tc;
  const int h = bh % a.H;
  const ChunkRange cr = chunk_range(a.T, a.HW, a.chunk, a.overlap, t);
  const int64_t q0 = cr.q_lo + (int64_t)qt * C::QT;
  if (q0 >= cr.q_hi) return;  // short last chunk: fewer query tiles
  const int64_t N = (int64_t)a.T * a.HW;
  const bf16_t* Qg = a.q + (int64_t)bh * N * D;
  const bf16_t* Kg = a.k + (int64_t)bh * N * D;
  const bf16_t* Vg = a.v + (int64_t)bh * N * D;
  bf16_t* Og = a.out + (int64_t)bh * N * D;

  // ---- queries of this wave, held as B operands ---------------------------
  const int64_t qw0 = q0 + wave * C::QW;
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
  float mrun[QB];  // running max of exponent * log2(e)
  float lrun[QB];  // this lane half's share of the sum
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    mrun[qb] = -INFINITY;
    lrun[qb] = 0.f;
  }

  const float sc = a.scale_log2e;  // log2(e)/sqrt(d): mrun holds exponent * sc

  // =========================== phase S =====================================
  {
    const FragOffsets<D> fo = make_frag_offsets<D>(lane);
    const int lane_off = tile_lane_offset<D>(wave, lane);
    const int64_t s_lo = cr.s_lo, s_hi = cr.s_hi;
    const int n_full = (int)((s_hi - s_lo) / 64);
    const int rem = (int)((s_hi - s_lo) - 64 * (int64_t)n_full);  // keys in the ragged last tile
    char* const Kt = smem;
    char* const Vt = smem + 2 * C::TILE_BYTES;
    const char* const Kb = reinterpret_cast<const char*>(Kg + s_lo * D);
    const char* const Vb = reinterpret_cast<const char*>(Vg + s_lo * D);
    if (n_full > 0) {
      tile_load_direct<D>(Kb, Kt, lane_off, wave);
      tile_load_direct<D>(Vb, Vt, lane_off, wave);
    }
    __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): the tile has landed in LDS
    __syncthreads();
    for (int it = 0; it < n_full; ++it) {
      // Tile it+1 goes into the other buffer, whose last readers (tile it-1) all
      // passed the barrier that ended the previous iteration.
      if (it + 1 < n_full) {
        const int64_t goff = (int64_t)(it + 1) * C::TILE_BYTES;
        tile_load_direct<D>(Kb + goff, Kt + ((it + 1) & 1) * C::TILE_BYTES, lane_off, wave);
        tile_load_direct<D>(Vb + goff, Vt + ((it + 1) & 1) * C::TILE_BYTES, lane_off, wave);
      }
      softmax_tile<D, QB, false>(Kt + (it & 1) * C::TILE_BYTES, Vt + (it & 1) * C::TILE_BYTES, fo, Qr, O,
                                 mrun, lrun, sc, 64, lane);
      __builtin_amdgcn_s_waitcnt(0x0F70);
      __syncthreads();
    }
    if (rem > 0) {  // ragged last tile, outside the loop so that its index math is not kept live in it
      const int64_t goff = (int64_t)n_full * C::TILE_BYTES;
      tile_load_direct_tail<D>(Kb + goff, Kt, rem, wave, lane);
      tile_load_direct_tail<D>(Vb + goff, Vt, rem, wave, lane);
      __builtin_amdgcn_s_waitcnt(0x0F70);
      __syncthreads();
      softmax_tile<D, QB, true>(Kt, Vt, fo, Qr, O, mrun, lrun, sc, rem, lane);
    }
  }

  // complete the softmax normaliser across the two lane halves
  float nS[QB], mtrue[QB];
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    nS[qb] = half_swap_sum(lrun[qb]);
    mtrue[qb] = mrun[qb] * 0.6931471805599453f;  // back from base 2
  }

  // debug: softmax components
  if (a.dbg_m || a.dbg_nS || a.dbg_aS) {
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
      const int64_t row = qw0 + 32 * qb + r;
      if (row < cr.q_hi) {
        const int64_t o = (int64_t)bh * N + row;
        if (g == 0) {
          if (a.dbg_m) a.dbg_m[o] = mtrue[qb];
          if (a.dbg_nS) a.dbg_nS[o] = nS[qb];
        }
        if (a.dbg_aS) {
#pragma unroll
          for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
              f32x4 x = {O[db][qb][4 * i], O[db][qb][4 * i + 1], O[db][qb][4 * i + 2], O[db][qb][4 * i + 3]};
              *reinterpret_cast<f32x4*>(a.dbg_aS + o * D + 32 * db + 8 * i + 4 * g) = x;
            }
        }
      }
    }
  }

  // =========================== phase L =====================================
  float nL[QB];
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) nL[qb] = 0.f;
  if (cr.l_hi > 0) {
    const bf16_t* W1 = a.w1_q + (int64_t)h * HID * D;
    const bf16_t* W2 = a.w2_q + (int64_t)h * DP * HID;
    const bf16_t* St = a.state_s + ((int64_t)bh * a.state_slots + tc) * (int64_t)D * DP;  // [D][DP]
    const float* zt = a.state_z + ((int64_t)bh * a.state_slots + tc) * DP;
    __syncthreads();  // all waves are done with the K/V tiles
    for (int i = tid; i < HID; i += NT) sb1[i] = a.b1_q[(int64_t)h * HID + i];
    for (int i = tid; i < DP; i += NT) {
      sb2[i] = a.b2_q[(int64_t)h * DP + i];
      sz[i] = zt[i];
    }
    // with c = 0 the linear terms carry exp(-m) relative to the softmax terms
    float lin_scale[QB];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb)
      lin_scale[qb] = (a.stab_mode == 1) ? __builtin_amdgcn_exp2f(-mrun[qb]) : 1.f;

    // ---- U^T = relu(W1 Q^T + b1), kept as bf16 B operands -------------------
    bf16x8 Ub[QB][HID / 16];
    {
      TileRegs<64, D, NT> wreg;
      tile_load<64, D, NT, false>(wreg, W1, D, 64, tid);
      constexpr int NSLAB = HID / 64;
#pragma unroll
      for (int sl = 0; sl < NSLAB; ++sl) {
        __syncthreads();
        tile_store<64, D, NT, false>(wreg, bufA, C::LDK, tid);
        __syncthreads();
        if (sl + 1 < NSLAB) tile_load<64, D, NT, false>(wreg, W1 + (int64_t)(sl + 1) * 64 * D, D, 64, tid);
#pragma unroll
        for (int hb2 = 0; hb2 < 2; ++hb2) {
          const int hb = 2 * sl + hb2;  // 32-row block of hidden units
          f32x16 acc[QB];
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            f32x4 bias = *reinterpret_cast<const f32x4*>(sb1 + 32 * hb + 8 * i + 4 * g);
#pragma unroll
            for (int j = 0; j < 4; ++j)
#pragma unroll
              for (int qb = 0; qb < QB; ++qb) acc[qb][4 * i + j] = bias[j];
          }
#pragma unroll
          for (int ks = 0; ks < KS; ++ks) {
            bf16x8 wf = lds_read_frag(bufA + (32 * hb2 + r) * C::LDK + 16 * ks + 8 * g);
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
      }
    }

    // ---- per 32 features: psi^T = relu(W2 U^T + b2), phi, read-out ----------
    {
      TileRegs<32, HID, NT> wreg;
      TileRegs<D, 32, NT> sreg;
      tile_load<32, HID, NT, false>(wreg, W2, HID, 32, tid);
      tile_load<D, 32, NT, false>(sreg, St, DP, D, tid);
      constexpr int NPB = DP / 32;
#pragma unroll 1
      for (int pb = 0; pb < NPB; ++pb) {
        __syncthreads();
        tile_store<32, HID, NT, true>(wreg, bufA, C::LDW2, tid);
        tile_store<D, 32, NT, true>(sreg, bufB, C::LDS_S, tid);
        __syncthreads();
        if (pb + 1 < NPB) {
          tile_load<32, HID, NT, false>(wreg, W2 + (int64_t)(pb + 1) * 32 * HID, HID, 32, tid);
          tile_load<D, 32, NT, false>(sreg, St + (pb + 1) * 32, DP, D, tid);
        }
        f32x16 acc[QB];
        float zv[16];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          f32x4 bias = *reinterpret_cast<const f32x4*>(sb2 + 32 * pb + 8 * i + 4 * g);
          f32x4 zz = *reinterpret_cast<const f32x4*>(sz + 32 * pb + 8 * i + 4 * g);
#pragma unroll
          for (int j = 0; j < 4; ++j) {
#pragma unroll
            for (int qb = 0; qb < QB; ++qb) acc[qb][4 * i + j] = bias[j];
            zv[4 * i + j] = zz[j];
          }
        }
#pragma unroll
        for (int ks = 0; ks < HID / 16; ++ks) {
          bf16x8 wf = lds_read_frag(bufA + r * C::LDW2 + 16 * ks + 8 * g);
#pragma unroll
          for (int qb = 0; qb < QB; ++qb) acc[qb] = mfma(wf, Ub[qb][ks], acc[qb]);
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
            x = bf16_round(x * lin_scale[qb]);
            acc[qb][e] = x;
            part += x * zv[e];
          }
          nL[qb] += part;
          Fb[qb][0] = acc_to_operand(acc[qb], 0);
          Fb[qb][1] = acc_to_operand(acc[qb], 1);
        }
#pragma unroll
        for (int s = 0; s < 2; ++s) {
#pragma unroll
          for (int db = 0; db < DB; ++db) {
            bf16x8 sf = lds_read_frag(bufB + (32 * db + r) * C::LDS_S + 16 * s + 8 * g);
#pragma unroll
            for (int qb = 0; qb < QB; ++qb) O[db][qb] = mfma(sf, Fb[qb][s], O[db][qb]);
          }
        }
      }
    }
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) nL[qb] = half_swap_sum(nL[qb]);
  }

  // =========================== merge (Eq. 5) ================================
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    const int64_t row = qw0 + 32 * qb + r;
    if (row >= cr.q_hi) continue;
    const int64_t o = (int64_t)bh * N + row;
    if (g == 0 && a.dbg_nL) a.dbg_nL[o] = nL[qb];
    const float inv = 1.0f / (nS[qb] + nL[qb]);
#pragma unroll
    for (int db = 0; db < DB; ++db) {
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int col = 32 * db + 8 * i + 4 * g;
        if (a.dbg_aL) {
          f32x4 as = {0.f, 0.f, 0.f, 0.f};
          if (a.dbg_aS) as = *reinterpret_cast<const f32x4*>(a.dbg_aS + o * D + col);
          f32x4 x = {O[db][qb][4 * i] - as[0], O[db][qb][4 * i + 1] - as[1],
                     O[db][qb][4 * i + 2] - as[2], O[db][qb][4 * i + 3] - as[3]};
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

// Queries per workgroup: 128 (one 32-query block per wave, two workgroups per
// CU) or 256 (two blocks per wave, one workgroup per CU).  REHYAT_ATTN_QB=1|2
// in the environment overrides the default; read once.
static int attn_qb() {
  static int qb = [] {
    const char* e = getenv("REHYAT_ATTN_QB");
    int v = e ? atoi(e) : kAttnQB;
    return (v == 2) ? 2 : 1;
  }();
  return qb;
}

int attn_query_tile(int d) { return attn_qb() == 2 ? 256 : 128; }

hipError_t launch_attn(const AttnArgs& a, int d, int grid, hipStream_t stream) {
  const int qb = attn_qb();
  if (d == 128 && qb == 1) {
    hipLaunchKernelGGL((attn_kernel<128, 1>), dim3(grid), dim3(256), 0, stream, a);
  } else if (d == 128) {
    hipLaunchKernelGGL((attn_kernel<128, 2>), dim3(grid), dim3(256), 0, stream, a);
  } else if (qb == 1) {
    hipLaunchKernelGGL((attn_kernel<64, 1>), dim3(grid), dim3(256), 0, stream, a);
  } else {
    hipLaunchKernelGGL((attn_kernel<64, 2>), dim3(grid), dim3(256), 0, stream, a);
  }
  return hipGetLastError();
}

}  // namespace rehyat
