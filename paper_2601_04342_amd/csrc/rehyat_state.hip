// Chunk-state kernel for gfx950: for a range of key/value tokens of one
// (batch, head) computes the partial sums of the linear-attention state,
//   dS^T = V^T phi_k(K)   (d x D', fp32)      dz = sum_rows phi_k(K)   (D')
// i.e. the increments of Eq. 17-18, with the feature map phi_k (two-layer MLP,
// second half of the output squared) evaluated on the fly from K -- phi_k(K)
// never goes to HBM.
//
// One workgroup of NW waves walks its token range in tiles of 64 tokens.  Wave
// w owns hidden units and output features [32w, 32w+32): it produces that slice
// of U = relu(K W1^T + b1) for the tile, the waves exchange U through LDS, then
// each wave forms its feature slice psi = relu(U W2^T + b2), squares it if it
// lies in the upper half, and accumulates V^T phi into its d x 32 slice of the
// state, held in MFMA accumulators for the whole token range.  The wave's rows
// of W1 and W2 stay in registers as MFMA operands; what makes room for them is
// that no per-lane LDS offset is held across the tile loop (U rows are padded so
// that k-steps are immediate offsets; offsets into the permuted K and V tiles
// are one XOR away from a per-lane base and are derived per tile).
//
// K and V tiles arrive by direct global->LDS loads (chunk-swizzled rows) into two
// buffers each, picked by the parity of the tile, and are requested two tile
// steps ahead of their use: K and V are read exactly once, so every tile comes
// from HBM, whose latency is far longer than the half tile step a single buffer
// allows.  The K tile of step t+2 is requested once every wave is past the first
// half of step t (its buffer is free then), the V tile of step t+2 once step t
// is complete.  The loads are issued through tile_load_fast (see tile_load_asm:
// with buffers picked at run time the compiler must not see them) and ordered
// against the reads by counted waits.
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
  constexpr int TB = 64 * 2 * D;  // bytes of a K, V or W1 tile (64 rows of 2D bytes)
  constexpr int UROW = HID * 2;   // bytes of a row of U
  static_assert(DP / NW == 32, "each wave owns 32 features");

  // U[token][hidden] with 16 bytes of padding per row: consecutive rows start four banks
  // apart, so fragment reads and writes are conflict-free without a chunk permutation
  constexpr int UPAD = UROW + 16;
  __shared__ __attribute__((aligned(1024))) char XV[4 * TB];   // K tiles 0/1, then V tiles 0/1
  __shared__ __attribute__((aligned(1024))) char Us[2 * 64 * UPAD];   // U of the current and of the next tile
  __shared__ __attribute__((aligned(256))) float B1s[HID];

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave-uniform for the compiler too
  const int g = lane >> 5;
  const int r = lane & 31;

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

  // ---- resident operands ----------------------------------------------------
  // first-layer bias in LDS: accumulator register 4i+j is hidden unit 32w + 8i + 4g + j, so a
  // lane reads its four rows of block i with one 16-byte read
  if (tid < HID) B1s[tid] = a.b1_k[(int64_t)h * HID + tid];
  const float* const b1rows = B1s + wave * 32 + 4 * g;
  const int unit = wave * 32 + r;  // this lane's hidden unit (first half) and feature (second half)
  const float b2v = a.b2_k[(int64_t)h * DP + unit];
  bf16x8 w1f[KS];   // A operands: row = hidden unit, k = head dimension
  {
    const bf16_t* p = a.w1_k + ((int64_t)h * HID + unit) * D + 8 * g;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) w1f[ks] = *reinterpret_cast<const bf16x8*>(p + 16 * ks);
  }
  bf16x8 w2f[KS2];  // B operands: column = feature, k = hidden
  {
    const bf16_t* p = a.w2_k + ((int64_t)h * DP + unit) * HID + 8 * g;
#pragma unroll
    for (int ks = 0; ks < KS2; ++ks) w2f[ks] = *reinterpret_cast<const bf16x8*>(p + 16 * ks);
  }
  // tile `it` of K or V into the buffer of its parity; rows at or beyond the end of the range
  // re-read the last valid row
  const u32x4 Kr = make_rsrc_words(Kb), Vr = make_rsrc_words(Vb);
  const uint32_t xv_lds = lds_address(XV);
  const int n_tiles = n_full + (rem > 0 ? 1 : 0);
  const int voff_full = tile_voff_full<2 * D, NW>(wave, lane);
  auto issue_k = [&](int it) {
    tile_load_fast<2 * D, TB, NW>(Kr, __builtin_amdgcn_readfirstlane(it * TB), xv_lds + (it & 1) * TB, wave, lane,
                                  it < n_full ? 64 : rem, voff_full);
  };
  auto issue_v = [&](int it) {
    tile_load_fast<2 * D, TB, NW>(Vr, __builtin_amdgcn_readfirstlane(it * TB), xv_lds + (2 + (it & 1)) * TB, wave,
                                  lane, it < n_full ? 64 : rem, voff_full);
  };
  const int uwbase = r * UPAD + wave * 64 + 8 * g;   // write: token r, units 32w + 8i + 4g .. +3 at + 16 i
  const int urbase = r * UPAD + 16 * g;              // read: A fragment of token r, k-step ks at + 32 ks

  // state slice: acc[db] register 4i+j = (row d = 32db+8i+4g+j, feature 32w+r)
  f32x16 acc[DB];
#pragma unroll
  for (int db = 0; db < DB; ++db)
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[db][e] = 0.f;
  float zacc = 0.f;
  const bool squared = (wave * 32 >= DP / 2);
  const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};

  // fragment of row lr, k-step ks of a K tile = xbase ^ 32 ks (the chunk bits of the permuted
  // layout do not overlap the row bits)
  // first half of tile `it`: U^T slice = relu(W1[slice] X^T + b1[slice]) -> U[token][hidden] in
  // the buffer of the tile's parity
  auto first_half = [&](int it, int xbase) {
    const char* const Xs = XV + (it & 1) * TB;
    char* const Ud = Us + (it & 1) * (64 * UPAD);
#pragma unroll
    for (int tb = 0; tb < 2; ++tb) {
      f32x16 u = zero;
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        bf16x8 xf = *reinterpret_cast<const bf16x8*>(Xs + (xbase ^ (32 * ks)) + tb * (32 * 2 * D));
        u = mfma(w1f[ks], xf, u);
      }
      // register 4i+j = (hidden 32w+8i+4g+j, token 32tb+r)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const f32x4 bb = *reinterpret_cast<const f32x4*>(b1rows + 8 * i);
        u32x2 pk;
        pk[0] = pack_bf16(fmaxf(u[4 * i] + bb[0], 0.f), fmaxf(u[4 * i + 1] + bb[1], 0.f));
        pk[1] = pack_bf16(fmaxf(u[4 * i + 2] + bb[2], 0.f), fmaxf(u[4 * i + 3] + bb[3], 0.f));
        *reinterpret_cast<u32x2*>(Ud + uwbase + 16 * i + tb * (32 * UPAD)) = pk;
      }
    }
  };
  auto opaque_lane = [&]() {   // offsets derived from it are recomputed per tile, not held in registers
    int ln = lane;
    asm volatile("" : "+v"(ln));
    return ln;
  };

  // Step `it` runs the second half of tile `it` together with the first half of tile it+1
  // (independent instruction streams inside every wave), so one barrier per tile is enough:
  // it publishes U of tile it+1 and frees the buffers of tile `it`.  K runs two tiles ahead
  // of V's use, both are requested one step before they are read.
  if (n_tiles > 0) {
    issue_k(0);
    issue_v(0);
    wait_loads_and_barrier<0>();   // also: the bias is in LDS
    if (n_tiles > 1) issue_k(1);
    const int ln = opaque_lane();
    first_half(0, tile_off<2 * D>(ln & 31, 8 * (ln >> 5)));
  }

  auto tile_step = [&](auto TAILC, int it) {
    constexpr bool TAIL = decltype(TAILC)::value;
    const char* const Vs = XV + (2 + (it & 1)) * TB;
    const char* const Uc = Us + (it & 1) * (64 * UPAD);
    // K of tile it+1 and V of tile `it` have landed (the only loads in flight); U of tile `it`
    // is complete; every wave is done with tile it-1
    wait_loads_and_barrier<0>();
    if (it + 2 < n_tiles) issue_k(it + 2);
    if (it + 1 < n_tiles) issue_v(it + 1);
    const int ln = opaque_lane();
    const int lr = ln & 31, lg = ln >> 5, li = ln & 15;
    int voff_lo[DB], voff_hi[DB];                        // transposing reads of V, see softmax kernel
#pragma unroll
    for (int db = 0; db < DB; ++db) {
      const int col = 32 * db + 16 * (lr >> 4) + 4 * (li & 3);
      voff_lo[db] = tile_off<2 * D>(4 * lg + (li >> 2), col);
      voff_hi[db] = tile_off<2 * D>(8 + 4 * lg + (li >> 2), col);
    }
    if (it + 1 < n_tiles) first_half(it + 1, tile_off<2 * D>(lr, 8 * lg));
    // ---- second half ---------------------------------------------------------------
#pragma unroll
    for (int tb = 0; tb < 2; ++tb) {
      // psi slice = relu(U W2[slice]^T + b2): rows = tokens, columns = features
      f32x16 ps = zero;
#pragma unroll
      for (int ks = 0; ks < KS2; ++ks) {
        bf16x8 uf = *reinterpret_cast<const bf16x8*>(Uc + urbase + 32 * ks + tb * (32 * UPAD));
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
