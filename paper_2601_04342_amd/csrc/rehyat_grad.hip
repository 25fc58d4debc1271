// Kernels of the feature-map gradient for gfx950: dL/d(phi_q, phi_k parameters) for a given
// dL/dy_hat -- what one step of the attention distillation of section 3.4 (Eq. 19) needs,
// which trains nothing but the two feature maps of a block.
//
// With the per-row stabiliser the softmax terms of Eq. 5 do not depend on phi, so the
// chain rule runs through the linear terms only (Eq. 7, 9, 16):
//   u_i = G_i / den_i,  w_i = -(G_i . y_i) / den_i,  den_i = n^S_i + n^L_i
//   dL/dPhi_q,i = S_t u_i + w_i z_t
//   dL/dS_t = sum_i Phi_q,i u_i^T,  dL/dz_t = sum_i w_i Phi_q,i           (queries i of chunk t)
//   dL/dPhi_k,j = R_tau v_j + r_tau,  R_tau = sum_{t > tau} dL/dS_t        (keys j of segment tau)
// and then through phi = [psi_1, psi_2^2], psi = relu(W2 U + b2), U = relu(W1 x + b1).
//
// Kernels, in launch order for one side (queries, then keys):
//   prep_kernel       u, w per token (HBM-bound)
//   state_kernel      (rehyat_state.hip, query segments) dL/dS_t partial sums
//   act_grad_kernel   recomputes U and psi, forms dPhi and dpsi per token; writes dpsi
//                     token-major, and the partial sums of db2 and dL/dz_t
//   suffix_kernel     R_tau, r_tau from the partial sums
//   tn_gemm_kernel    dW2 = dpsi^T U over tokens (U recomputed from x)
//   hid_grad_kernel   dU = (dpsi W2) [U > 0]; dW1 = dU^T x, db1 = sum dU (sign of U recomputed)
//   reduce_kernel     sums the per-workgroup partials over batch and pieces
// The contraction kernels follow the chunk-state kernel's scheme: wave w owns 32 hidden
// units or features, weights of its slice live in registers as MFMA B operands, tiles of 64
// tokens arrive by direct global->LDS loads, products are computed with tokens in the
// accumulator rows so that an accumulator is directly the B operand of the token
// contraction that follows.
#include <type_traits>

#include "rehyat_device.h"
#include "rehyat_kernels.h"

namespace rehyat {

// ------------------------------------------------------------------------------------
// u_i = G_i / den_i (bf16), w_i = -(G_i . y_i) / den_i.  Eight elements per thread, D/8
// consecutive lanes per token.
// ------------------------------------------------------------------------------------
template <int D>
__global__ void __launch_bounds__(256)
prep_kernel(PrepArgs a) {
  constexpr int LPT = D / 8;  // lanes per token
  const int64_t gid = (int64_t)blockIdx.x * 256 + threadIdx.x;
  int64_t tok = gid / LPT;
  const int part = (int)(gid % LPT);
  const bool live = tok < a.tokens;
  if (!live) tok = a.tokens - 1;  // keep the lane in the shuffles below
  const int64_t off = tok * D + 8 * part;
  const u32x4 gr = *reinterpret_cast<const u32x4*>(a.g + off);
  const u32x4 yr = *reinterpret_cast<const u32x4*>(a.y + off);
  const float inv = 1.0f / (a.nS[tok] + a.nL[tok]);
  float dot = 0.f;
  u32x4 ur;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const float g0 = __builtin_bit_cast(float, gr[i] << 16), g1 = __builtin_bit_cast(float, gr[i] & 0xffff0000u);
    const float y0 = __builtin_bit_cast(float, yr[i] << 16), y1 = __builtin_bit_cast(float, yr[i] & 0xffff0000u);
    dot += g0 * y0 + g1 * y1;
    ur[i] = pack_bf16(g0 * inv, g1 * inv);
  }
#pragma unroll
  for (int m = 1; m < LPT; m <<= 1) dot += __shfl_xor(dot, m);
  if (live) {
    *reinterpret_cast<u32x4*>(a.u + off) = ur;
    if (part == 0) a.tokw[tok] = -dot * inv;
  }
}

hipError_t launch_prep(const PrepArgs& a, hipStream_t stream) {
  const int lpt = a.d / 8;
  const int64_t threads = a.tokens * lpt;
  const unsigned grid = (unsigned)((threads + 255) / 256);
  if (a.d == 128) hipLaunchKernelGGL(prep_kernel<128>, dim3(grid), dim3(256), 0, stream, a);
  else hipLaunchKernelGGL(prep_kernel<64>, dim3(grid), dim3(256), 0, stream, a);
  return hipGetLastError();
}

// ------------------------------------------------------------------------------------
// R_tau = sum over segments s >= tau of the chunk-state gradient partials (segment s holds
// dL/dS of chunk s+1, so this is the sum over chunks t > tau), r_tau likewise.  Each thread
// owns four consecutive elements and walks the segments from the last to the first (fixed
// order: bit-reproducible).
// ------------------------------------------------------------------------------------
__global__ void __launch_bounds__(256)
suffix_kernel(SuffixArgs a) {
  const int bh = blockIdx.y;
  const int idx = (blockIdx.x * 256 + threadIdx.x) * 4;
  if (idx >= a.elems) return;
  const bool is_s = idx < a.s_elems;
  f32x4 acc = {0.f, 0.f, 0.f, 0.f};
  for (int c = a.n_seg - 1; c >= 0; --c) {
    if (is_s) {
      const float* p = a.s_part + ((int64_t)bh * a.s_slots + (int64_t)c * a.s_nsplit) * a.elems + idx;
      for (int sp = 0; sp < a.s_nsplit; ++sp) acc += *reinterpret_cast<const f32x4*>(p + (int64_t)sp * a.elems);
      u32x2 pk;
      pk[0] = pack_bf16(acc[0], acc[1]);
      pk[1] = pack_bf16(acc[2], acc[3]);
      *reinterpret_cast<u32x2*>(a.Rt + ((int64_t)bh * a.slots + c) * a.s_elems + idx) = pk;
    } else {
      const int zi = idx - a.s_elems;
      const float* p = a.z_part + (((int64_t)bh * a.n_seg + c) * a.z_nsplit) * a.dp + zi;
      for (int sp = 0; sp < a.z_nsplit; ++sp) acc += *reinterpret_cast<const f32x4*>(p + (int64_t)sp * a.dp);
      *reinterpret_cast<f32x4*>(a.r + ((int64_t)bh * a.slots + c) * a.dp + zi) = acc;
    }
  }
}

hipError_t launch_suffix(const SuffixArgs& a, hipStream_t stream) {
  dim3 grid((a.elems / 4 + 255) / 256, a.BH);
  hipLaunchKernelGGL(suffix_kernel, grid, dim3(256), 0, stream, a);
  return hipGetLastError();
}

// ------------------------------------------------------------------------------------
// bf16 [n][R][C] -> [n][C][R] through a padded 32 x 32 LDS tile; optionally a second batch of n
// matrices of the same shape in the same launch.
// ------------------------------------------------------------------------------------
__global__ void __launch_bounds__(256)
transpose_kernel(TransposeArgs a) {
  __shared__ bf16_t tile[32][33];
  int m = blockIdx.z;
  const bf16_t* in = a.in;
  bf16_t* out = a.out;
  if (m >= a.n) {   // second batch of matrices
    m -= a.n;
    in = a.in2;
    out = a.out2;
  }
  const int r0 = blockIdx.y * 32, c0 = blockIdx.x * 32;
  const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;  // 32 x 8
  in += (int64_t)m * a.R * a.C;
  out += (int64_t)m * a.R * a.C;
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int rr = r0 + ty + 8 * j, cc = c0 + tx;
    if (rr < a.R && cc < a.C) tile[ty + 8 * j][tx] = in[(int64_t)rr * a.C + cc];
  }
  __syncthreads();
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int cc = c0 + ty + 8 * j, rr = r0 + tx;
    if (rr < a.R && cc < a.C) out[(int64_t)cc * a.R + rr] = tile[tx][ty + 8 * j];
  }
}

hipError_t launch_transpose(const TransposeArgs& a, hipStream_t stream) {
  dim3 grid((a.C + 31) / 32, (a.R + 31) / 32, a.in2 ? 2 * a.n : a.n);
  hipLaunchKernelGGL(transpose_kernel, grid, dim3(256), 0, stream, a);
  return hipGetLastError();
}

// ------------------------------------------------------------------------------------
// Activation gradients.  Wave w owns hidden units and features [32w, 32w + 32); its rows of
// W1, W2 and of the segment's matrix M stay in registers as MFMA operands for the whole token
// range.  Per tile of 64 tokens:
//   first half   U^T slice = relu(W1[slice] X^T + b1[slice]) -> LDS as U[token][hidden];
//   second half  psi slice = U W2[slice]^T + b2 and dPhi slice = Vec M[slice]^T, both with
//                tokens in accumulator rows and the wave's 32 features in lanes;
//                dpsi = dPhi + w zv, times 2 psi in the squared half, zero where psi = 0;
//                dpsi goes through a wave-private LDS patch so that it leaves in 16-byte stores.
// The x and vec tiles (and the 64 token weights) of tile t+2 are requested when tile t is
// finished, into the buffers tile t used; they are ordered against the reads by counted
// waits.  Vector memory operations of a wave complete in the order issued, stores included,
// so "at most n outstanding" after n younger stores means every older load has landed.
// ------------------------------------------------------------------------------------
template <int D, int NW, bool TW>
__global__ void __launch_bounds__(64 * NW)
act_grad_kernel(ActGradArgs a) {
  constexpr int HID = 2 * D, DP = 2 * D;
  constexpr int KS = D / 16;
  constexpr int KS2 = HID / 16;
  constexpr int TB = 64 * 2 * D;  // bytes of an x or vec tile
  constexpr int UROW = HID * 2;
  constexpr int LPT = TB / (1024 * NW);
  constexpr int LG = 2 * LPT + (TW ? 1 : 0);  // direct loads per wave per tile
  constexpr int SROW = 80;        // bytes per token row of the dpsi patch: 32 features + padding
  constexpr int NST = 4;          // dpsi stores per lane per full tile
  // U[token][hidden] with 16 bytes of padding per row: consecutive rows start four banks apart,
  // so fragment reads and writes are conflict-free without a chunk permutation and every
  // k-step is an immediate offset from one per-lane address
  constexpr int UPAD = UROW + 16;
  static_assert(DP / NW == 32, "each wave owns 32 features");

  __shared__ __attribute__((aligned(1024))) char XV[4 * TB];   // x tiles 0/1, then vec tiles 0/1
  __shared__ __attribute__((aligned(1024))) char Us[64 * UPAD];
  __shared__ __attribute__((aligned(1024))) char Stg[NW * 32 * SROW];
  __shared__ __attribute__((aligned(256))) float Tws[2 * 64];
  __shared__ __attribute__((aligned(256))) float B1s[HID];

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int g = lane >> 5;
  const int r = lane & 31;

  const int item = xcd_swizzle(blockIdx.x, a.items_per_xcd);
  if (item >= a.n_items) return;
  const int sp = item % a.nsplit;
  const int rest = item / a.nsplit;
  const int seg = rest % a.n_seg;
  const int bh = rest / a.n_seg;
  const int h = bh % a.H;

  int64_t seg_lo, seg_hi;
  int slot;
  if (a.query_side) {
    const ChunkRange cr = chunk_range(a.T, a.HW, a.chunk, a.overlap, seg + 1);
    seg_lo = cr.q_lo;
    seg_hi = cr.q_hi;
    slot = seg + 1;
  } else {  // keys that enter the linear set between chunk seg and chunk seg + 1 (Eq. 13)
    seg_lo = chunk_range(a.T, a.HW, a.chunk, a.overlap, seg).s_lo;
    seg_hi = chunk_range(a.T, a.HW, a.chunk, a.overlap, seg + 1).s_lo;
    slot = seg;
  }
  const int64_t N = (int64_t)a.T * a.HW;
  const int64_t len = seg_hi - seg_lo;
  const int64_t lo = seg_lo + (len * sp) / a.nsplit;
  const int64_t hi = seg_lo + (len * (sp + 1)) / a.nsplit;
  const int n_full = (int)((hi - lo) / 64);
  const int rem = (int)((hi - lo) - 64 * (int64_t)n_full);
  const int n_tiles = n_full + (rem > 0 ? 1 : 0);

  const int64_t row0 = (int64_t)bh * N + lo;  // first token of this piece, over all (b, h)
  char* Pg = reinterpret_cast<char*>(a.dpsi + row0 * DP);

  // ---- resident operands ----------------------------------------------------
  // first-layer bias in LDS: accumulator register 4i+j is hidden unit 32w + 8i + 4g + j, so a
  // lane reads its four rows of block i with one 16-byte read
  if (tid < HID) B1s[tid] = a.b1[(int64_t)h * HID + tid];
  const float* const b1rows = B1s + wave * 32 + 4 * g;
  const int unit = wave * 32 + r;  // this lane's hidden unit (first half) and feature (second half)
  const float b2v = a.b2[(int64_t)h * DP + unit];
  const float zvv = a.zv[((int64_t)bh * a.slots + slot) * DP + unit];
  bf16x8 w1f[KS];   // A operands: row = hidden unit, k = head dimension
  {
    const bf16_t* p = a.w1 + ((int64_t)h * HID + unit) * D + 8 * g;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) w1f[ks] = *reinterpret_cast<const bf16x8*>(p + 16 * ks);
  }
  bf16x8 w2f[KS2];  // B operands: column = feature, k = hidden
  {
    const bf16_t* p = a.w2 + ((int64_t)h * DP + unit) * HID + 8 * g;
#pragma unroll
    for (int ks = 0; ks < KS2; ++ks) w2f[ks] = *reinterpret_cast<const bf16x8*>(p + 16 * ks);
  }
  bf16x8 mf[KS];    // B operands: column = feature, k = head dimension (row `unit` of M)
  {
    // M is stored transposed ([d][dprime], the layout of the forward chunk states): the eight
    // values of a fragment are gathered one by one -- once per workgroup
    const bf16_t* p = a.M + ((int64_t)bh * a.slots + slot) * D * DP + unit;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      u32x4 w;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const uint32_t lo = p[(int64_t)(16 * ks + 8 * g + 2 * j) * DP];
        const uint32_t hi = p[(int64_t)(16 * ks + 8 * g + 2 * j + 1) * DP];
        w[j] = lo | (hi << 16);
      }
      mf[ks] = __builtin_bit_cast(bf16x8, w);
    }
  }

  const u32x4 Xr = make_rsrc_words(a.x + row0 * D), Vr = make_rsrc_words(a.vec + row0 * D);
  const u32x4 Twr = make_rsrc_words(TW ? (const void*)(a.tokw + row0) : (const void*)a.x);
  const uint32_t xv_lds = lds_address(XV), tw_lds = lds_address(Tws);
  const int voff_full = tile_voff_full<2 * D, NW>(wave, lane);
  auto issue = [&](int it) {   // tile `it` into the buffers of its parity
    const int valid = it < n_full ? 64 : rem;
    const int soff = __builtin_amdgcn_readfirstlane(it * TB);
    tile_load_fast<2 * D, TB, NW>(Xr, soff, xv_lds + (it & 1) * TB, wave, lane, valid, voff_full);
    if (TW) {
      const int t = lane < valid ? lane : valid - 1;
      direct_load_4(Twr, 4 * t, __builtin_amdgcn_readfirstlane(it * 256), tw_lds + (it & 1) * 256);
    }
    tile_load_fast<2 * D, TB, NW>(Vr, soff, xv_lds + (2 + (it & 1)) * TB, wave, lane, valid, voff_full);
  };

  // ---- per-lane LDS byte offsets (as in the chunk-state kernel) -----------------
  // fragment of token row r, k-step ks inside an x or vec tile: chunk 2 ks + g, permuted by the
  // row -- the chunk bits do not overlap the row bits, so the offset is one XOR away from a
  // per-lane constant
  // (derived per tile from an opaque copy of the lane index: held across the loop, the eight
  // offsets and the addresses of the dpsi patch would push resident operands out of registers)
  const int uwbase = r * UPAD + wave * 64 + 8 * g;   // write: token r, units 32w + 8i + 4g .. +3 at + 16 i
  const int urbase = r * UPAD + 16 * g;              // read: A fragment of token r, k-step ks at + 32 ks
  char* const Sg = Stg + wave * (32 * SROW);   // this wave's patch: [32 tokens][32 features]

  float db2acc = 0.f, dzacc = 0.f;
  const bool squared = (wave * 32 >= DP / 2);
  const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};

  if (n_tiles > 0) issue(0);
  if (n_tiles > 1) {
    issue(1);
    wait_loads_and_barrier<LG>();   // tile 0 has landed, tile 1 may be in flight
  } else {
    wait_loads_and_barrier<0>();
  }

  for (int it = 0; it < n_tiles; ++it) {
    const int valid = it < n_full ? 64 : rem;
    const char* const Xs = XV + (it & 1) * TB;
    const char* const Vs = XV + (2 + (it & 1)) * TB;
    const float* const tws = Tws + (it & 1) * 64;
    int ln = lane;
    asm volatile("" : "+v"(ln));
    const int xbase = tile_off<2 * D>(ln & 31, 8 * (ln >> 5));

    // ---- first half ----------------------------------------------------------
#pragma unroll
    for (int tb = 0; tb < 2; ++tb) {
      f32x16 u = zero;
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        bf16x8 xf = *reinterpret_cast<const bf16x8*>(Xs + (xbase ^ (32 * ks)) + tb * (32 * 2 * D));
        u = mfma(w1f[ks], xf, u);
      }
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const f32x4 bb = *reinterpret_cast<const f32x4*>(b1rows + 8 * i);
        u32x2 pk;
        pk[0] = pack_bf16(fmaxf(u[4 * i] + bb[0], 0.f), fmaxf(u[4 * i + 1] + bb[1], 0.f));
        pk[1] = pack_bf16(fmaxf(u[4 * i + 2] + bb[2], 0.f), fmaxf(u[4 * i + 3] + bb[3], 0.f));
        *reinterpret_cast<u32x2*>(Us + uwbase + 16 * i + tb * (32 * UPAD)) = pk;
      }
    }
    lds_barrier();   // U complete

    // ---- second half ---------------------------------------------------------
#pragma unroll
    for (int tb = 0; tb < 2; ++tb) {
      f32x16 ps = zero, dphi = zero;
#pragma unroll
      for (int ks = 0; ks < KS2; ++ks) {
        bf16x8 uf = *reinterpret_cast<const bf16x8*>(Us + urbase + 32 * ks + tb * (32 * UPAD));
        ps = mfma(uf, w2f[ks], ps);
      }
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        bf16x8 vf = *reinterpret_cast<const bf16x8*>(Vs + (xbase ^ (32 * ks)) + tb * (32 * 2 * D));
        dphi = mfma(vf, mf[ks], dphi);
      }
      float pdb = 0.f, pdz = 0.f;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        f32x4 tw = {1.f, 1.f, 1.f, 1.f};   // weights of zv for tokens 32 tb + 8 i + 4 g + j
        if (TW) tw = *reinterpret_cast<const f32x4*>(tws + 32 * tb + 8 * i + 4 * g);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const int e = 4 * i + j;
          const bool live = 32 * tb + 8 * i + 4 * g + j < valid;
          const float psi = fmaxf(ps[e] + b2v, 0.f);
          const float base = dphi[e] + tw[j] * zvv;   // dL/dPhi
          // Phi = psi^2 in the squared half, psi = relu(.) in the other (wave-uniform choice)
          const float dp = squared ? 2.f * psi * base : (psi > 0.f ? base : 0.f);
          const float ph = squared ? psi * psi : psi;
          pdb += live ? dp : 0.f;
          pdz += live ? tw[j] * ph : 0.f;
          *reinterpret_cast<bf16_t*>(Sg + (8 * i + 4 * g + j) * SROW + 2 * r) =
              (bf16_t)(pack_bf16(dp, 0.f) & 0xffffu);
        }
      }
      db2acc += pdb;
      dzacc += pdz;
      // the patch leaves token-major: 4 chunks of 16 bytes per token row, two per lane
#pragma unroll
      for (int n = 0; n < 2; ++n) {
        const int idx = ln + 64 * n;
        const int row = idx >> 2, c = idx & 3;
        const u32x4 val = *reinterpret_cast<const u32x4*>(Sg + row * SROW + 16 * c);
        if (32 * tb + row < valid)
          *reinterpret_cast<u32x4*>(Pg + ((int64_t)it * 64 + 32 * tb + row) * (DP * 2) + wave * 64 + 16 * c) = val;
      }
    }
    if (it + 1 < n_tiles) {
      // tile it+1 has landed: it is older than this (full) tile's NST stores; every wave is done
      // with this tile's buffers and with U
      wait_loads_and_barrier<NST>();
      if (it + 2 < n_tiles) issue(it + 2);
    }
  }

  const float db2 = half_swap_sum(db2acc);
  const float dz = half_swap_sum(dzacc);
  if (g == 0) {
    a.db2_part[(int64_t)item * DP + unit] = db2;
    if (a.dz_part) a.dz_part[(int64_t)item * DP + unit] = dz;
  }
}

hipError_t launch_act_grad(const ActGradArgs& a, int d, int grid, hipStream_t stream) {
  if (d == 128) {
    if (a.tokw) hipLaunchKernelGGL((act_grad_kernel<128, 8, true>), dim3(grid), dim3(512), 0, stream, a);
    else hipLaunchKernelGGL((act_grad_kernel<128, 8, false>), dim3(grid), dim3(512), 0, stream, a);
  } else {
    if (a.tokw) hipLaunchKernelGGL((act_grad_kernel<64, 4, true>), dim3(grid), dim3(256), 0, stream, a);
    else hipLaunchKernelGGL((act_grad_kernel<64, 4, false>), dim3(grid), dim3(256), 0, stream, a);
  }
  return hipGetLastError();
}

// token range of piece sp of nsplit: whole tiles of 64 from `lo`, the last tile ragged
struct Piece {
  int64_t tok0;
  int n_tiles;    // tiles of this piece
  int last_rows;  // valid rows of its last tile (64 unless it is the range's last tile)
};
__device__ __forceinline__ Piece piece_of(int64_t lo, int64_t hi, int sp, int nsplit) {
  const int64_t nt = (hi - lo + 63) / 64;
  const int64_t t0 = nt * sp / nsplit, t1 = nt * (sp + 1) / nsplit;
  Piece p;
  p.tok0 = lo + 64 * t0;
  p.n_tiles = (int)(t1 - t0);
  p.last_rows = 64;
  if (t1 == nt && nt > 0) p.last_rows = (int)((hi - lo) - 64 * (nt - 1));
  return p;
}

// first-layer bias of the wave's accumulator rows: register 4i+j is hidden unit
// 32 wave + 8i + 4g + j, two wave-uniform values per register picked by the lane half
struct BiasRows {
  float lo[16], hi[16];
};
__device__ __forceinline__ BiasRows load_bias_rows(const float* bp) {
  BiasRows b;
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      b.lo[4 * i + j] = __builtin_bit_cast(float, __builtin_amdgcn_readfirstlane(__builtin_bit_cast(int, bp[8 * i + j])));
      b.hi[4 * i + j] = __builtin_bit_cast(float, __builtin_amdgcn_readfirstlane(__builtin_bit_cast(int, bp[8 * i + 4 + j])));
    }
  return b;
}

// ------------------------------------------------------------------------------------
// dW2 partial: part[f][hid] = sum_tok dpsi[tok][f] U[tok][hid].  Per tile the waves first
// rebuild U = relu(W1 x + b1) in LDS (token-major, as the chunk-state kernel does; 16 MFMAs per
// wave against 512 bytes per token that U would cost through HBM); then both operands are
// token-major LDS tiles read with transposing loads (tokens become the contraction index).
// Each wave owns 64 rows f and half of the columns.  The dpsi and x tiles of tile t+1 are
// requested at the start of tile t.
// ------------------------------------------------------------------------------------
template <int D, int NW>
__global__ void __launch_bounds__(64 * NW)
tn_gemm_kernel(TnGemmArgs a) {
  constexpr int W = 2 * D;          // features = hidden units
  constexpr int KS = D / 16;
  constexpr int ROWB = 2 * W;       // bytes per token row of dpsi and of U
  constexpr int TBY = 64 * ROWB;    // dpsi tile
  constexpr int TB = 64 * 2 * D;    // x tile
  constexpr int SET = TBY + TB;
  constexpr int NT = 64 * NW;
  constexpr int HB = W / 64;        // 32-column blocks per wave (half of the columns)
  static_assert(W / 64 == NW / 2, "waves form a (W/64) x 2 grid");
  static_assert(W / NW == 32, "each wave rebuilds 32 hidden units");

  __shared__ __attribute__((aligned(1024))) char Ts[2 * SET];   // (dpsi tile, x tile) x 2
  __shared__ __attribute__((aligned(1024))) char Us[2 * TBY];   // U of the current and of the next tile

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int g = lane >> 5, r = lane & 31, i16 = lane & 15;
  const int wf = wave >> 1, wh = wave & 1;

  const int item = xcd_swizzle(blockIdx.x, a.items_per_xcd);
  if (item >= a.n_items) return;
  const int sp = item % a.nsplit;
  const int bh = item / a.nsplit;
  const int h = bh % a.H;
  const Piece pc = piece_of(a.lo, a.hi, sp, a.nsplit);
  const int64_t row0 = (int64_t)bh * a.N + pc.tok0;
  const u32x4 Pr = make_rsrc_words(a.dpsi + row0 * W), Xr = make_rsrc_words(a.x + row0 * D);

  const BiasRows b1 = load_bias_rows(a.b1 + (int64_t)h * W + wave * 32);
  bf16x8 w1f[KS];   // A operands: row = hidden unit 32 wave + r, k = head dimension
  {
    const bf16_t* p = a.w1 + ((int64_t)h * W + wave * 32 + r) * D + 8 * g;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) w1f[ks] = *reinterpret_cast<const bf16x8*>(p + 16 * ks);
  }
  int xoff[KS];
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) xoff[ks] = tile_off<2 * D>(r, 16 * ks + 8 * g);
  int uwoff[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) uwoff[i] = r * ROWB + (((wave * 4 + i) ^ swz<256>(r)) << 4) + 8 * g;

  int xlo[2], xhi[2], ylo[HB], yhi[HB];
#pragma unroll
  for (int fb = 0; fb < 2; ++fb) {
    const int col = 64 * wf + 32 * fb + 16 * (r >> 4) + 4 * (i16 & 3);
    xlo[fb] = tile_off<ROWB>(4 * g + (i16 >> 2), col);
    xhi[fb] = tile_off<ROWB>(8 + 4 * g + (i16 >> 2), col);
  }
#pragma unroll
  for (int hb = 0; hb < HB; ++hb) {
    const int col = (W / 2) * wh + 32 * hb + 16 * (r >> 4) + 4 * (i16 & 3);
    ylo[hb] = tile_off<ROWB>(4 * g + (i16 >> 2), col);
    yhi[hb] = tile_off<ROWB>(8 + 4 * g + (i16 >> 2), col);
  }

  f32x16 acc[2][HB];
#pragma unroll
  for (int fb = 0; fb < 2; ++fb)
#pragma unroll
    for (int hb = 0; hb < HB; ++hb)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[fb][hb][e] = 0.f;

  const uint32_t ts_lds = lds_address(Ts);
  const int pvoff = tile_voff_full<ROWB, NW>(wave, lane), xvoff = tile_voff_full<2 * D, NW>(wave, lane);
  auto valid_of = [&](int it) { return (it + 1 < pc.n_tiles) ? 64 : pc.last_rows; };
  auto issue_p = [&](int it) {
    tile_load_fast<ROWB, TBY, NW>(Pr, __builtin_amdgcn_readfirstlane(it * TBY), ts_lds + (it & 1) * SET, wave, lane,
                                  valid_of(it), pvoff);
  };
  auto issue_x = [&](int it) {
    tile_load_fast<2 * D, TB, NW>(Xr, __builtin_amdgcn_readfirstlane(it * TB), ts_lds + (it & 1) * SET + TBY, wave,
                                  lane, valid_of(it), xvoff);
  };
  // U^T slice of tile `it` = relu(W1[slice] X^T + b1[slice]) -> U[token][hidden] in the buffer of
  // the tile's parity
  auto build_u = [&](int it) {
    const char* const Xs = Ts + (it & 1) * SET + TBY;
    char* const Ud = Us + (it & 1) * TBY;
#pragma unroll
    for (int tb = 0; tb < 2; ++tb) {
      f32x16 u;
#pragma unroll
      for (int e = 0; e < 16; ++e) u[e] = g ? b1.hi[e] : b1.lo[e];
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        bf16x8 xf = *reinterpret_cast<const bf16x8*>(Xs + xoff[ks] + tb * (32 * 2 * D));
        u = mfma(w1f[ks], xf, u);
      }
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        u32x2 pk;
        pk[0] = pack_bf16(fmaxf(u[4 * i], 0.f), fmaxf(u[4 * i + 1], 0.f));
        pk[1] = pack_bf16(fmaxf(u[4 * i + 2], 0.f), fmaxf(u[4 * i + 3], 0.f));
        *reinterpret_cast<u32x2*>(Ud + uwoff[i] + tb * (32 * ROWB)) = pk;
      }
    }
  };
  // One barrier per tile: in step `it` the waves rebuild U of tile it+1 while they multiply
  // tile it, so the two phases overlap inside every wave.  x runs one tile ahead of dpsi.
  if (pc.n_tiles > 0) {
    issue_x(0);
    issue_p(0);
    wait_loads_and_barrier<0>();
    if (pc.n_tiles > 1) issue_x(1);
    build_u(0);
  }
  for (int it = 0; it < pc.n_tiles; ++it) {
    const int valid = valid_of(it);
    char* const Ps = Ts + (it & 1) * SET;
    const char* const Uc = Us + (it & 1) * TBY;
    // dpsi of tile `it` and x of tile it+1 have landed (the only loads in flight); U of tile
    // `it` is complete; every wave is done with tile it-1
    wait_loads_and_barrier<0>();
    if (it + 1 < pc.n_tiles) issue_p(it + 1);
    if (it + 2 < pc.n_tiles) issue_x(it + 2);
    if (valid < 64) {  // rows past the range hold copies of the last row: clear them in dpsi
      const u32x4 z4 = {0u, 0u, 0u, 0u};
      for (int o = valid * ROWB + tid * 16; o < TBY; o += NT * 16) *reinterpret_cast<u32x4*>(Ps + o) = z4;
      lds_barrier();
    }
    if (it + 1 < pc.n_tiles) build_u(it + 1);
#pragma unroll
    for (int s = 0; s < 4; ++s) {
      const int so = s * 16 * ROWB;
      bf16x8 af[2], bfr[HB];
#pragma unroll
      for (int fb = 0; fb < 2; ++fb)
        af[fb] = join_tr(lds_read_tr(reinterpret_cast<const bf16_t*>(Ps + xlo[fb] + so)),
                         lds_read_tr(reinterpret_cast<const bf16_t*>(Ps + xhi[fb] + so)));
#pragma unroll
      for (int hb = 0; hb < HB; ++hb)
        bfr[hb] = join_tr(lds_read_tr(reinterpret_cast<const bf16_t*>(Uc + ylo[hb] + so)),
                          lds_read_tr(reinterpret_cast<const bf16_t*>(Uc + yhi[hb] + so)));
#pragma unroll
      for (int fb = 0; fb < 2; ++fb)
#pragma unroll
        for (int hb = 0; hb < HB; ++hb) acc[fb][hb] = mfma(af[fb], bfr[hb], acc[fb][hb]);
    }
  }

  float* P = a.part + (int64_t)item * W * W;
#pragma unroll
  for (int fb = 0; fb < 2; ++fb)
#pragma unroll
    for (int hb = 0; hb < HB; ++hb)
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int f = 64 * wf + 32 * fb + 8 * (e >> 2) + 4 * g + (e & 3);
        P[f * W + (W / 2) * wh + 32 * hb + r] = acc[fb][hb][e];
      }
}

hipError_t launch_tn_gemm(const TnGemmArgs& a, int d, int grid, hipStream_t stream) {
  if (d == 128) hipLaunchKernelGGL((tn_gemm_kernel<128, 8>), dim3(grid), dim3(512), 0, stream, a);
  else hipLaunchKernelGGL((tn_gemm_kernel<64, 4>), dim3(grid), dim3(256), 0, stream, a);
  return hipGetLastError();
}

// ------------------------------------------------------------------------------------
// First-layer gradients.  Wave w owns hidden units [32w, 32w + 32): its rows of W1 and of
// W2^T stay in registers as B operands.  Per tile, with tokens in accumulator rows and the
// wave's hidden units in lanes: U slice = X W1[slice]^T + b1 (only its sign is needed),
// dU slice = dpsi W2[:, slice], zero where U <= 0; then x^T dU into the wave's [d][32] slice
// of dW1^T, exactly as the chunk-state kernel accumulates V^T phi.
// ------------------------------------------------------------------------------------
template <int D, int NW>
__global__ void __launch_bounds__(64 * NW)
hid_grad_kernel(HidGradArgs a) {
  constexpr int HID = 2 * D, DP = 2 * D;
  constexpr int KS = D / 16;
  constexpr int KS2 = DP / 16;      // k-steps across the features
  constexpr int DB = D / 32;
  constexpr int TB = 64 * 2 * D;    // x tile
  constexpr int UROW = DP * 2;      // bytes of a dpsi row
  constexpr int TBU = 64 * UROW;
  constexpr int SET = TBU + TB;
  static_assert(HID / NW == 32, "each wave owns 32 hidden units");

  __shared__ __attribute__((aligned(1024))) char Ts[2 * SET];   // (dpsi tile, x tile) x 2

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int g = lane >> 5, r = lane & 31, i16 = lane & 15;

  const int item = xcd_swizzle(blockIdx.x, a.items_per_xcd);
  if (item >= a.n_items) return;
  const int sp = item % a.nsplit;
  const int bh = item / a.nsplit;
  const int h = bh % a.H;
  const Piece pc = piece_of(a.lo, a.hi, sp, a.nsplit);
  const int64_t row0 = (int64_t)bh * a.N + pc.tok0;
  const u32x4 Pr = make_rsrc_words(a.dpsi + row0 * DP), Xr = make_rsrc_words(a.x + row0 * D);

  const int unit = wave * 32 + r;   // this lane's hidden unit
  const float b1v = a.b1[(int64_t)h * HID + unit];
  bf16x8 w1f[KS];                   // B operands: column = hidden unit, k = head dimension
  {
    const bf16_t* p = a.w1 + ((int64_t)h * HID + unit) * D + 8 * g;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) w1f[ks] = *reinterpret_cast<const bf16x8*>(p + 16 * ks);
  }
  bf16x8 w2tf[KS2];                 // B operands: column = hidden unit, k = feature
  {
    const bf16_t* p = a.w2t + ((int64_t)h * HID + unit) * DP + 8 * g;
#pragma unroll
    for (int ks = 0; ks < KS2; ++ks) w2tf[ks] = *reinterpret_cast<const bf16x8*>(p + 16 * ks);
  }
  // Fragment offsets inside the tiles are one XOR away from a per-lane constant (the chunk bits
  // do not overlap the row bits).  They are derived per tile from an opaque copy of the lane
  // index: held across the loop they would push resident operands out of registers.

  f32x16 acc[DB];
#pragma unroll
  for (int db = 0; db < DB; ++db)
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[db][e] = 0.f;
  float dbacc = 0.f;
  const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};

  const uint32_t ts_lds = lds_address(Ts);
  const int pvoff = tile_voff_full<UROW, NW>(wave, lane), xvoff = tile_voff_full<2 * D, NW>(wave, lane);
  auto issue = [&](int it) {   // requested one tile step ahead of its use
    const int valid = (it + 1 < pc.n_tiles) ? 64 : pc.last_rows;
    const uint32_t base = ts_lds + (it & 1) * SET;
    tile_load_fast<UROW, TBU, NW>(Pr, __builtin_amdgcn_readfirstlane(it * TBU), base, wave, lane, valid, pvoff);
    tile_load_fast<2 * D, TB, NW>(Xr, __builtin_amdgcn_readfirstlane(it * TB), base + TBU, wave, lane, valid, xvoff);
  };
  if (pc.n_tiles > 0) issue(0);
  for (int it = 0; it < pc.n_tiles; ++it) {
    const int valid = (it + 1 < pc.n_tiles) ? 64 : pc.last_rows;
    const char* const Ps = Ts + (it & 1) * SET;
    const char* const Xs = Ps + TBU;
    // tile `it` has landed (the only loads in flight) and every wave is done with tile it-1
    wait_loads_and_barrier<0>();
    if (it + 1 < pc.n_tiles) issue(it + 1);
    int ln = lane;
    asm volatile("" : "+v"(ln));
    const int lr = ln & 31, lg = ln >> 5, li = ln & 15;
    const int pbase = lr * UROW + ((lg ^ swz<256>(lr)) << 4);   // dpsi row lr, chunk 2 ks + g at ^ 32 ks
    const int xbase = tile_off<2 * D>(lr, 8 * lg);             // x row lr, k-step ks at ^ 32 ks
    int voff_lo[DB], voff_hi[DB];                              // transposing reads of x
#pragma unroll
    for (int db = 0; db < DB; ++db) {
      const int col = 32 * db + 16 * (lr >> 4) + 4 * (li & 3);
      voff_lo[db] = tile_off<2 * D>(4 * lg + (li >> 2), col);
      voff_hi[db] = tile_off<2 * D>(8 + 4 * lg + (li >> 2), col);
    }
#pragma unroll
    for (int tb = 0; tb < 2; ++tb) {
      f32x16 uu, du = zero;
#pragma unroll
      for (int e = 0; e < 16; ++e) uu[e] = b1v;
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        bf16x8 xf = *reinterpret_cast<const bf16x8*>(Xs + (xbase ^ (32 * ks)) + tb * (32 * 2 * D));
        uu = mfma(xf, w1f[ks], uu);
      }
#pragma unroll
      for (int ks = 0; ks < KS2; ++ks) {
        bf16x8 pf = *reinterpret_cast<const bf16x8*>(Ps + (pbase ^ (32 * ks)) + tb * (32 * UROW));
        du = mfma(pf, w2tf[ks], du);
      }
      float part = 0.f;
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int t = 32 * tb + 8 * (e >> 2) + 4 * g + (e & 3);
        float x = du[e];
        if (!(uu[e] > 0.f) || t >= valid) x = 0.f;
        x = bf16_round(x);
        du[e] = x;
        part += x;
      }
      dbacc += part;
#pragma unroll
      for (int s = 0; s < 2; ++s) {
        bf16x8 fb = acc_to_operand(du, s);
#pragma unroll
        for (int db = 0; db < DB; ++db) {
          const int so = (2 * tb + s) * (16 * 2 * D);
          i16x4 vlo = lds_read_tr(reinterpret_cast<const bf16_t*>(Xs + voff_lo[db] + so));
          i16x4 vhi = lds_read_tr(reinterpret_cast<const bf16_t*>(Xs + voff_hi[db] + so));
          acc[db] = mfma(join_tr(vlo, vhi), fb, acc[db]);
        }
      }
    }
  }

  float* P = a.part + (int64_t)item * (D * HID + HID);
#pragma unroll
  for (int db = 0; db < DB; ++db)
#pragma unroll
    for (int e = 0; e < 16; ++e) {
      const int row = 32 * db + 8 * (e >> 2) + 4 * g + (e & 3);
      P[row * HID + unit] = acc[db][e];
    }
  const float tot = half_swap_sum(dbacc);
  if (g == 0) P[D * HID + unit] = tot;
}

hipError_t launch_hid_grad(const HidGradArgs& a, int d, int grid, hipStream_t stream) {
  if (d == 128) hipLaunchKernelGGL((hid_grad_kernel<128, 8>), dim3(grid), dim3(512), 0, stream, a);
  else hipLaunchKernelGGL((hid_grad_kernel<64, 4>), dim3(grid), dim3(256), 0, stream, a);
  return hipGetLastError();
}

// ------------------------------------------------------------------------------------
// Sum of the per-workgroup partials over batch and pieces, in a fixed order.
// ------------------------------------------------------------------------------------
// A block owns 64 consecutive elements; four groups of 64 threads each sum every fourth
// partial, and the four sums are combined in a fixed order.
__global__ void __launch_bounds__(256)
reduce_kernel(ReduceJobs jobs) {
  __shared__ float sums[4][64];
  const ReduceArgs& a = jobs.job[blockIdx.z];
  const int h = blockIdx.y;
  const int q = threadIdx.x >> 6;
  const int i = blockIdx.x * 64 + (threadIdx.x & 63);
  const int n = a.R * a.C;
  if (blockIdx.x * 64 >= n) return;
  float acc = 0.f;
  if (i < n) {
    const int total = a.B * a.per_bh;
#pragma unroll 8
    for (int m = q; m < total; m += 4) {
      const int b = m / a.per_bh, sidx = m - b * a.per_bh;
      acc += a.part[((int64_t)(b * a.H + h) * a.per_bh + sidx) * a.part_stride + a.part_off + i];
    }
  }
  sums[q][threadIdx.x & 63] = acc;
  __syncthreads();
  if (q == 0 && i < n) {
    const int e = threadIdx.x;
    const float tot = ((sums[0][e] + sums[1][e]) + sums[2][e]) + sums[3][e];
    int o = i;
    if (a.transpose) o = (i % a.C) * a.R + i / a.C;
    a.out[(int64_t)h * n + o] = tot;
  }
}

hipError_t launch_reduce(const ReduceJobs& jobs, hipStream_t stream) {
  int most = 0;
  for (int j = 0; j < jobs.n; ++j)
    if (jobs.job[j].R * jobs.job[j].C > most) most = jobs.job[j].R * jobs.job[j].C;
  dim3 grid((most + 63) / 64, jobs.job[0].H, jobs.n);
  hipLaunchKernelGGL(reduce_kernel, grid, dim3(256), 0, stream, jobs);
  return hipGetLastError();
}

__global__ void __launch_bounds__(256)
fill_zero_kernel(float* p, int64_t n) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i < n) p[i] = 0.f;
}

hipError_t launch_fill_zero(float* p, int64_t n, hipStream_t stream) {
  if (n <= 0) return hipSuccess;
  hipLaunchKernelGGL(fill_zero_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, stream, p, n);
  return hipGetLastError();
}

}  // namespace rehyat
