// Chunk-state kernel for gfx950: for a range of key/value tokens of one
// (batch, head) computes the partial sums of the linear-attention state,
//   dS^T = V^T phi_k(K)   (d x D', fp32)      dz = sum_rows phi_k(K)   (D')
// i.e. the increments of Eq. 17-18, with the feature map phi_k (two-layer MLP,
// second half of the output squared) evaluated on the fly from K -- phi_k(K)
// never goes to HBM.
//
// One workgroup of NW waves walks its token range in tiles of 64 tokens.  Wave
// w owns hidden units and output features [32w, 32w+32): it produces that slice
// of U = relu(K W1^T + b1) for the tile (W1 resident in LDS), the waves
// exchange U through LDS, then each wave forms its feature slice
// psi = relu(U W2^T + b2) with its W2 rows resident in registers, squares it if
// it lies in the upper half, and accumulates V^T phi into its d x 32 slice of
// the state, held in MFMA accumulators for the whole token range.
//
// K and V tiles arrive by direct global->LDS loads (chunk-swizzled rows) into two
// buffers each, picked by the parity of the tile, and are requested two tile
// steps ahead of their use: K and V are read exactly once, so every tile comes
// from HBM, whose latency is far longer than the half tile step a single buffer
// allows.  The K tile of step t+2 is requested once every wave is past the first
// half of step t (its buffer is free then), the V tile of step t+2 once step t
// is complete.  The loads are issued through tile_load_asm (see there: with
// buffers picked at run time the compiler must not see them) and ordered
// against the reads by counted waits.  With W1 and U the four tile buffers fill
// the 160 KB of LDS exactly; the first-layer bias is therefore read through
// scalar loads (it is wave-uniform up to the lane half).
#include <type_traits>

#include "rehyat_device.h"
#include "rehyat_kernels.h"

namespace rehyat {

template <int D, int NW>
__global__ void __launch_bounds__(64 * NW)
state_kernel(StateArgs a) {
  constexpr int HID = 2 * D, DP = 2 * D;
  constexpr int KS = D / 16;      // k-steps across the head dimension
  constexpr int KS2 = HID / 16;   // k-steps across the hidden layer
  constexpr int DB = D / 32;      // 32-row blocks of the head dimension
  constexpr int NT = 64 * NW;
  constexpr int TB = 64 * 2 * D;  // bytes of a K, V or W1 tile (64 rows of 2D bytes)
  constexpr int UROW = HID * 2;   // bytes of a row of U
  static_assert(DP / NW == 32, "each wave owns 32 features");

  __shared__ __attribute__((aligned(1024))) char W1s[(HID / 64) * TB];
  __shared__ __attribute__((aligned(1024))) char XV[4 * TB];   // K tiles 0/1, then V tiles 0/1
  __shared__ __attribute__((aligned(1024))) char Us[64 * UROW];

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave-uniform for the compiler too
  const int g = lane >> 5;
  const int r = lane & 31;
  const int i16 = lane & 15;

  const int item = xcd_swizzle(blockIdx.x, a.items_per_xcd);
  if (item >= a.n_items) return;
  const int sp = item % a.nsplit;
  const int rest = item / a.nsplit;
  const int seg = rest % a.n_seg;
  const int bh = rest / a.n_seg;
  const int h = bh % a.H;

  // token range of this piece
  int64_t seg_lo = 0, seg_hi = a.step_n;
  if (a.step_n <= 0) {
    const int tt = a.chunk0 + seg;
    const int nchunks = num_chunks(a.T, a.chunk);
    const ChunkRange cr = chunk_range(a.T, a.HW, a.chunk, a.overlap, tt);
    if (a.query_segments) {   // the queries of chunk tt (gradient of the chunk state)
      seg_lo = cr.q_lo;
      seg_hi = cr.q_hi;
    } else {
      seg_lo = cr.s_lo;
      seg_hi = (tt + 1 < nchunks) ? chunk_range(a.T, a.HW, a.chunk, a.overlap, tt + 1).s_lo
                                  : (int64_t)a.T * a.HW;
    }
  }
  const int64_t len = seg_hi - seg_lo;
  const int64_t lo = seg_lo + (len * sp) / a.nsplit;
  const int64_t hi = seg_lo + (len * (sp + 1)) / a.nsplit;
  const int n_full = (int)((hi - lo) / 64);
  const int rem = (int)((hi - lo) - 64 * (int64_t)n_full);

  const char* Kb = reinterpret_cast<const char*>(a.k + (int64_t)bh * a.kv_bh_stride + lo * D);
  const char* Vb = reinterpret_cast<const char*>(a.v + (int64_t)bh * a.kv_bh_stride + lo * D);
  const char* W1 = reinterpret_cast<const char*>(a.w1_k + (int64_t)h * HID * D);
  const bf16_t* W2 = a.w2_k + (int64_t)h * DP * HID;

  // ---- resident operands ----------------------------------------------------
  // first-layer bias of accumulator register 4i+j: hidden unit 32w + 8i + 4g + j -- two
  // wave-uniform values per register, picked by the lane half
  float b1lo[16], b1hi[16];
  {
    const float* bp = a.b1_k + (int64_t)h * HID + wave * 32;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        b1lo[4 * i + j] = __builtin_bit_cast(float, __builtin_amdgcn_readfirstlane(__builtin_bit_cast(int, bp[8 * i + j])));
        b1hi[4 * i + j] = __builtin_bit_cast(float, __builtin_amdgcn_readfirstlane(__builtin_bit_cast(int, bp[8 * i + 4 + j])));
      }
  }
  const int unit = wave * 32 + r;  // this lane's feature (a column of the wave's products)
  const float b2v = a.b2_k[(int64_t)h * DP + unit];
  // W2 rows of this wave's features as B operands: column = feature, k = hidden
  bf16x8 w2f[KS2];
  {
    const bf16_t* p = W2 + (int64_t)unit * HID + 8 * g;
#pragma unroll
    for (int ks = 0; ks < KS2; ++ks) w2f[ks] = *reinterpret_cast<const bf16x8*>(p + 16 * ks);
  }
  // tile `it` of K or V into the buffer of its parity; rows at or beyond the end of the range
  // re-read the last valid row
  const u32x4 Kr = make_rsrc_words(Kb), Vr = make_rsrc_words(Vb), W1r = make_rsrc_words(W1);
  const uint32_t xv_lds = lds_address(XV);
  const int n_tiles = n_full + (rem > 0 ? 1 : 0);
  constexpr int LPT = TB / (1024 * NW);   // load instructions per wave per tile
  auto issue_k = [&](int it) {
    tile_load_asm<2 * D, TB, NW>(Kr, __builtin_amdgcn_readfirstlane(it * TB), xv_lds + (it & 1) * TB, wave, lane,
                                 it < n_full ? 64 : rem);
  };
  auto issue_v = [&](int it) {
    tile_load_asm<2 * D, TB, NW>(Vr, __builtin_amdgcn_readfirstlane(it * TB), xv_lds + (2 + (it & 1)) * TB, wave,
                                 lane, it < n_full ? 64 : rem);
  };
#pragma unroll
  for (int j = 0; j < HID / 64; ++j)
    tile_load_asm<2 * D, TB, NW>(W1r, j * TB, lds_address(W1s) + j * TB, wave, lane, 64);
  if (n_tiles > 0) {
    issue_k(0);
    issue_v(0);
  }
  if (n_tiles > 1) {
    issue_k(1);
    issue_v(1);
  }

  // ---- per-lane LDS byte offsets ----------------------------------------------
  const int hrow = wave * 32 + r;                      // W1 row of this lane's A fragment
  int w1off[KS], xoff[KS];
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) {
    w1off[ks] = (hrow >> 6) * TB + tile_off<2 * D>(hrow & 63, 16 * ks + 8 * g);
    xoff[ks] = tile_off<2 * D>(r, 16 * ks + 8 * g);    // + 32 rows for the second token block
  }
  // U[token][hidden], rows of UROW bytes, 16-byte chunks swizzled by swz<256>(token)
  int uwoff[4];                                        // write: token r, units 32w + 8i + 4g .. +3
#pragma unroll
  for (int i = 0; i < 4; ++i) uwoff[i] = r * UROW + (((wave * 4 + i) ^ swz<256>(r)) << 4) + 8 * g;
  int uroff[KS2];                                      // read: A fragment, token r, k-step ks2
#pragma unroll
  for (int ks = 0; ks < KS2; ++ks) uroff[ks] = r * UROW + (((2 * ks + g) ^ swz<256>(r)) << 4);
  int voff_lo[DB], voff_hi[DB];                        // transposing reads of V, see softmax kernel
#pragma unroll
  for (int db = 0; db < DB; ++db) {
    const int col = 32 * db + 16 * (r >> 4) + 4 * (i16 & 3);
    voff_lo[db] = tile_off<2 * D>(4 * g + (i16 >> 2), col);
    voff_hi[db] = tile_off<2 * D>(8 + 4 * g + (i16 >> 2), col);
  }

  // state slice: acc[db] register 4i+j = (row d = 32db+8i+4g+j, feature 32w+r)
  f32x16 acc[DB];
#pragma unroll
  for (int db = 0; db < DB; ++db)
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[db][e] = 0.f;
  float zacc = 0.f;
  const bool squared = (wave * 32 >= DP / 2);
  const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};

  // W1 and the first K and V tiles (the second pair may still be in flight).  A wave's loads
  // complete in the order issued, so "at most the n newest outstanding" means that every
  // older one has landed.
  if (n_tiles > 1) wait_loads_and_barrier<2 * LPT>();
  else wait_loads_and_barrier<0>();

  auto tile_step = [&](auto TAILC, int it) {
    constexpr bool TAIL = decltype(TAILC)::value;
    const char* const Xs = XV + (it & 1) * TB;
    const char* const Vs = XV + (2 + (it & 1)) * TB;
    // ---- first half: U^T slice = relu(W1[slice] X^T + b1[slice]) -> LDS as U[token][hidden]
#pragma unroll
    for (int tb = 0; tb < 2; ++tb) {
      f32x16 u;
#pragma unroll
      for (int e = 0; e < 16; ++e) u[e] = g ? b1hi[e] : b1lo[e];
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        bf16x8 wf = *reinterpret_cast<const bf16x8*>(W1s + w1off[ks]);
        bf16x8 xf = *reinterpret_cast<const bf16x8*>(Xs + xoff[ks] + tb * (32 * 2 * D));
        u = mfma(wf, xf, u);
      }
      // register 4i+j = (hidden 32w+8i+4g+j, token 32tb+r)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        u32x2 pk;
        pk[0] = pack_bf16(fmaxf(u[4 * i], 0.f), fmaxf(u[4 * i + 1], 0.f));
        pk[1] = pack_bf16(fmaxf(u[4 * i + 2], 0.f), fmaxf(u[4 * i + 3], 0.f));
        *reinterpret_cast<u32x2*>(Us + uwoff[i] + tb * (32 * UROW)) = pk;
      }
    }
    // U complete; this tile's V has landed (newer: K and V of the next tile); this tile's K
    // buffer is free
    if (it + 1 < n_tiles) wait_loads_and_barrier<2 * LPT>();
    else wait_loads_and_barrier<0>();
    if (it + 2 < n_tiles) issue_k(it + 2);
    // ---- second half ---------------------------------------------------------------
#pragma unroll
    for (int tb = 0; tb < 2; ++tb) {
      // psi slice = relu(U W2[slice]^T + b2): rows = tokens, columns = features
      f32x16 ps = zero;
#pragma unroll
      for (int ks = 0; ks < KS2; ++ks) {
        bf16x8 uf = *reinterpret_cast<const bf16x8*>(Us + uroff[ks] + tb * (32 * UROW));
        ps = mfma(uf, w2f[ks], ps);
      }
      float part = 0.f;
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        float x = fmaxf(ps[e] + b2v, 0.f);
        if (squared) x = x * x;
        if (TAIL) {
          if (32 * tb + 8 * (e >> 2) + 4 * g + (e & 3) >= rem) x = 0.f;   // token beyond the range
        }
        x = bf16_round(x);
        ps[e] = x;
        part += x;
      }
      zacc += part;
      // state slice += V^T phi, two 16-token steps
#pragma unroll
      for (int s = 0; s < 2; ++s) {
        bf16x8 fb = acc_to_operand(ps, s);
#pragma unroll
        for (int db = 0; db < DB; ++db) {
          const int so = (2 * tb + s) * (16 * 2 * D);
          i16x4 vlo = lds_read_tr(reinterpret_cast<const bf16_t*>(Vs + voff_lo[db] + so));
          i16x4 vhi = lds_read_tr(reinterpret_cast<const bf16_t*>(Vs + voff_hi[db] + so));
          acc[db] = mfma(join_tr(vlo, vhi), fb, acc[db]);
        }
      }
    }
    // the next K tile has landed (newer: V of the next tile, K of the one after); U and this
    // tile's V buffer are free
    if (it + 2 < n_tiles) wait_loads_and_barrier<2 * LPT>();
    else if (it + 1 < n_tiles) wait_loads_and_barrier<LPT>();
    else wait_loads_and_barrier<0>();
    if (it + 2 < n_tiles) issue_v(it + 2);
  };

  for (int it = 0; it < n_full; ++it) tile_step(std::false_type{}, it);
  if (rem > 0) tile_step(std::true_type{}, n_full);

  // ---- write the partial: S^T [d][DP] fp32, then z [DP] ---------------------------
  float* P = a.partial + ((int64_t)bh * a.partial_slots + (int64_t)seg * a.nsplit + sp) * (int64_t)(D * DP + DP);
#pragma unroll
  for (int db = 0; db < DB; ++db)
#pragma unroll
    for (int e = 0; e < 16; ++e) {
      const int row = 32 * db + 8 * (e >> 2) + 4 * g + (e & 3);
      P[row * DP + unit] = acc[db][e];
    }
  const float ztot = half_swap_sum(zacc);
  if (g == 0) P[D * DP + unit] = ztot;
}

hipError_t launch_state(const StateArgs& a, int d, int grid, hipStream_t stream) {
  if (d == 128) {
    hipLaunchKernelGGL((state_kernel<128, 8>), dim3(grid), dim3(512), 0, stream, a);
  } else {
    hipLaunchKernelGGL((state_kernel<64, 4>), dim3(grid), dim3(256), 0, stream, a);
  }
  return hipGetLastError();
}

}  // namespace rehyat
