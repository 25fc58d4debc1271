// Chunk-state kernel for gfx950: for a range of key/value tokens of one
// (batch, head) computes the partial sums of the linear-attention state,
//   dS^T = V^T phi_k(K)   (d x D', fp32)      dz = sum_rows phi_k(K)   (D')
// i.e. the increments of Eq. 17-18, with the feature map phi_k (two-layer MLP,
// second half of the output squared) evaluated on the fly from K -- phi_k(K)
// never goes to HBM.
//
// One workgroup = 4 waves walks its token range in tiles of 64 tokens.  Wave w
// owns hidden units and output features [w*D/2, (w+1)*D/2): it produces that
// slice of U = relu(K W1^T + b1) for the tile (W1 resident in LDS), the four
// waves exchange U through LDS, then each wave forms its feature slice
// psi = relu(U W2^T + b2) with its W2 rows resident in registers, squares the
// upper half, and accumulates V^T phi into its d x D/2 slice of the state held
// in MFMA accumulators for the whole token range.
#include "rehyat_device.h"
#include "rehyat_kernels.h"

namespace rehyat {

template <int D>
__global__ void __launch_bounds__(256)
state_kernel(StateArgs a) {
  constexpr int HID = 2 * D, DP = 2 * D;
  constexpr int KS = D / 16;      // k-steps across the head dimension
  constexpr int KS2 = HID / 16;   // k-steps across the hidden layer
  constexpr int DB = D / 32;      // 32-row blocks of the head dimension
  constexpr int SL = DP / 4;      // features (and hidden units) per wave
  constexpr int CB = SL / 32;     // 32-wide blocks in a wave's slice
  constexpr int NT = 256;
  constexpr int LDX = D + 8;      // row stride of the K, V and W1 tiles
  constexpr int LDU = HID + 8;    // row stride of the U tile

  __shared__ __attribute__((aligned(16))) bf16_t W1s[HID * LDX];
  __shared__ __attribute__((aligned(16))) bf16_t Xs[64 * LDX];
  __shared__ __attribute__((aligned(16))) bf16_t Vs[64 * LDX];
  __shared__ __attribute__((aligned(16))) bf16_t Us[64 * LDU];
  __shared__ __attribute__((aligned(16))) float sb1[HID];

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int g = lane >> 5;
  const int r = lane & 31;

  const int item = xcd_swizzle(blockIdx.x, a.items_per_xcd);
  if (item >= a.n_items) return;
  const int sp = item % a.nsplit;
  const int rest = item / a.nsplit;
  const int seg = rest % a.n_seg;
  const int bh = rest / a.n_seg;
  const int h = bh % a.H;
  const int64_t N = (int64_t)a.T * a.HW;

  // token range of this piece
  const int tt = a.chunk0 + seg;
  const int nchunks = num_chunks(a.T, a.chunk);
  const int64_t seg_lo = chunk_range(a.T, a.HW, a.chunk, a.overlap, tt).s_lo;
  const int64_t seg_hi = (tt + 1 < nchunks) ? chunk_range(a.T, a.HW, a.chunk, a.overlap, tt + 1).s_lo : N;
  const int64_t len = seg_hi - seg_lo;
  const int64_t lo = seg_lo + (len * sp) / a.nsplit;
  const int64_t hi = seg_lo + (len * (sp + 1)) / a.nsplit;

  const bf16_t* Kg = a.k + (int64_t)bh * N * D;
  const bf16_t* Vg = a.v + (int64_t)bh * N * D;
  const bf16_t* W1 = a.w1_k + (int64_t)h * HID * D;
  const bf16_t* W2 = a.w2_k + (int64_t)h * DP * HID;

  // ---- resident operands ----------------------------------------------------
  {
    // W1 [HID][D] -> LDS, 64 rows at a time
#pragma unroll
    for (int sl = 0; sl < HID / 64; ++sl) {
      TileRegs<64, D, NT> w;
      tile_load<64, D, NT, false>(w, W1 + (int64_t)sl * 64 * D, D, 64, tid);
      tile_store<64, D, NT, false>(w, W1s + sl * 64 * LDX, LDX, tid);
    }
    for (int i = tid; i < HID; i += NT) sb1[i] = a.b1_k[(int64_t)h * HID + i];
  }
  // W2 rows of this wave's features as B operands: column = feature, k = hidden
  bf16x8 w2f[CB][KS2];
  float b2v[CB];
#pragma unroll
  for (int cb = 0; cb < CB; ++cb) {
    const int unit = wave * SL + 32 * cb + r;
    const bf16_t* p = W2 + (int64_t)unit * HID + 8 * g;
#pragma unroll
    for (int ks = 0; ks < KS2; ++ks) w2f[cb][ks] = *reinterpret_cast<const bf16x8*>(p + 16 * ks);
    b2v[cb] = a.b2_k[(int64_t)h * DP + unit];
  }

  // state slice: acc[db][cb] register 4i+j = (row d = 32db+8i+4g+j, feature wave*SL+32cb+r)
  f32x16 acc[DB][CB];
#pragma unroll
  for (int db = 0; db < DB; ++db)
#pragma unroll
    for (int cb = 0; cb < CB; ++cb)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[db][cb][e] = 0.f;
  float zacc[CB];
#pragma unroll
  for (int cb = 0; cb < CB; ++cb) zacc[cb] = 0.f;

  TileRegs<64, D, NT> kreg, vreg;
  if (lo < hi) {
    int valid = (int)((hi - lo) < 64 ? (hi - lo) : 64);
    tile_load<64, D, NT, true>(kreg, Kg + lo * D, D, valid, tid);
    tile_load<64, D, NT, true>(vreg, Vg + lo * D, D, valid, tid);
  }
  for (int64_t t0 = lo; t0 < hi; t0 += 64) {
    __syncthreads();  // previous tile consumed (also orders the W1 / bias staging)
    tile_store<64, D, NT, false>(kreg, Xs, LDX, tid);
    tile_store<64, D, NT, false>(vreg, Vs, LDX, tid);
    __syncthreads();
    if (t0 + 64 < hi) {
      int64_t rem = hi - (t0 + 64);
      int valid = (int)(rem < 64 ? rem : 64);
      tile_load<64, D, NT, true>(kreg, Kg + (t0 + 64) * D, D, valid, tid);
      tile_load<64, D, NT, true>(vreg, Vg + (t0 + 64) * D, D, valid, tid);
    }
    // ---- U^T slice = relu(W1[slice] X^T + b1[slice]) -> LDS as U[token][hidden]
#pragma unroll
    for (int tb = 0; tb < 2; ++tb) {
#pragma unroll
      for (int rb = 0; rb < CB; ++rb) {
        const int hrow = wave * SL + 32 * rb;  // first hidden unit of the block
        f32x16 u;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          f32x4 bias = *reinterpret_cast<const f32x4*>(sb1 + hrow + 8 * i + 4 * g);
#pragma unroll
          for (int j = 0; j < 4; ++j) u[4 * i + j] = bias[j];
        }
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
          bf16x8 wf = lds_read_frag(W1s + (hrow + r) * LDX + 16 * ks + 8 * g);
          bf16x8 xf = lds_read_frag(Xs + (32 * tb + r) * LDX + 16 * ks + 8 * g);
          u = mfma(wf, xf, u);
        }
        // register 4i+j = (hidden hrow+8i+4g+j, token 32tb+r)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          u32x2 pk;
          pk[0] = pack_bf16(fmaxf(u[4 * i], 0.f), fmaxf(u[4 * i + 1], 0.f));
          pk[1] = pack_bf16(fmaxf(u[4 * i + 2], 0.f), fmaxf(u[4 * i + 3], 0.f));
          *reinterpret_cast<u32x2*>(Us + (32 * tb + r) * LDU + hrow + 8 * i + 4 * g) = pk;
        }
      }
    }
    __syncthreads();  // U complete
    const bool tail = (t0 + 64 > hi);
#pragma unroll
    for (int tb = 0; tb < 2; ++tb) {
      // ---- psi slice = relu(U W2[slice]^T + b2): rows = tokens, columns = features
      f32x16 ps[CB];
#pragma unroll
      for (int cb = 0; cb < CB; ++cb)
#pragma unroll
        for (int e = 0; e < 16; ++e) ps[cb][e] = 0.f;
#pragma unroll
      for (int ks = 0; ks < KS2; ++ks) {
        bf16x8 uf = lds_read_frag(Us + (32 * tb + r) * LDU + 16 * ks + 8 * g);
#pragma unroll
        for (int cb = 0; cb < CB; ++cb) ps[cb] = mfma(uf, w2f[cb][ks], ps[cb]);
      }
      bf16x8 fb[CB][2];
#pragma unroll
      for (int cb = 0; cb < CB; ++cb) {
        const bool squared = (wave * SL + 32 * cb >= DP / 2);
        float part = 0.f;
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          float x = fmaxf(ps[cb][e] + b2v[cb], 0.f);
          if (squared) x = x * x;
          if (tail) {
            int64_t tok = t0 + 32 * tb + 8 * (e >> 2) + 4 * g + (e & 3);
            if (tok >= hi) x = 0.f;
          }
          x = bf16_round(x);
          ps[cb][e] = x;
          part += x;
        }
        zacc[cb] += part;
        fb[cb][0] = acc_to_operand(ps[cb], 0);
        fb[cb][1] = acc_to_operand(ps[cb], 1);
      }
      // ---- state slice += V^T phi
#pragma unroll
      for (int s = 0; s < 2; ++s) {
#pragma unroll
        for (int db = 0; db < DB; ++db) {
          bf16x8 vf = lds_read_frag_transposed(Vs, LDX, 32 * tb + 16 * s, 32 * db, lane);
#pragma unroll
          for (int cb = 0; cb < CB; ++cb) acc[db][cb] = mfma(vf, fb[cb][s], acc[db][cb]);
        }
      }
    }
  }

  // ---- write the partial: S^T [d][DP] fp32, then z [DP] ---------------------------
  float* P = a.partial + ((int64_t)bh * a.partial_slots + (int64_t)seg * a.nsplit + sp) * (int64_t)(D * DP + DP);
#pragma unroll
  for (int db = 0; db < DB; ++db)
#pragma unroll
    for (int cb = 0; cb < CB; ++cb)
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int row = 32 * db + 8 * (e >> 2) + 4 * g + (e & 3);
        P[row * DP + wave * SL + 32 * cb + r] = acc[db][cb][e];
      }
#pragma unroll
  for (int cb = 0; cb < CB; ++cb) {
    float ztot = zacc[cb] + __shfl_xor(zacc[cb], 32);
    if (g == 0) P[D * DP + wave * SL + 32 * cb + r] = ztot;
  }
}

template __global__ void state_kernel<64>(StateArgs);
template __global__ void state_kernel<128>(StateArgs);

hipError_t launch_state(const StateArgs& a, int d, int grid, hipStream_t stream) {
  if (d == 128) {
    hipLaunchKernelGGL(state_kernel<128>, dim3(grid), dim3(256), 0, stream, a);
  } else {
    hipLaunchKernelGGL(state_kernel<64>, dim3(grid), dim3(256), 0, stream, a);
  }
  return hipGetLastError();
}

}  // namespace rehyat
