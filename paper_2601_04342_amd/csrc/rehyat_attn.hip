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
#include "rehyat_device.h"
#include "rehyat_kernels.h"

namespace rehyat {

template <int D>
struct AttnShape {
  static constexpr int HID = 2 * D;
  static constexpr int DP = 2 * D;
  static constexpr int KS = D / 16;    // k-steps across the head dimension
  static constexpr int DB = D / 32;    // 32-row blocks across the head dimension
  static constexpr int NT = 256;       // threads
  static constexpr int QW = 64;        // queries per wave
  static constexpr int QT = 256;       // queries per workgroup
  static constexpr int KT = 64;        // keys per tile
  static constexpr int LDK = D + 8;    // K / W1 tile row stride
  static constexpr int LDV = D + 8;    // V tile row stride
  static constexpr int LDW2 = HID + 8; // W2 slab row stride
  static constexpr int LDS_S = 32 + 8; // state slab row stride
  // tile buffer A: K tile [64][LDK], W1 slab [64][LDK], W2 slab [32][LDW2]
  static constexpr int BUFA = (64 * LDK > 32 * LDW2) ? 64 * LDK : 32 * LDW2;
  // tile buffer B: V tile [64][LDV], state slab [D][LDS_S]
  static constexpr int BUFB = (64 * LDV > D * LDS_S) ? 64 * LDV : D * LDS_S;
};

template <int D>
__global__ void __launch_bounds__(256)
attn_kernel(AttnArgs a) {
  using C = AttnShape<D>;
  constexpr int HID = C::HID, DP = C::DP, KS = C::KS, DB = C::DB, NT = C::NT;
  __shared__ __attribute__((aligned(16))) bf16_t bufA[C::BUFA];
  __shared__ __attribute__((aligned(16))) bf16_t bufB[C::BUFB];
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
  bf16x8 Qr[2][KS];
#pragma unroll
  for (int qb = 0; qb < 2; ++qb) {
    int64_t row = qw0 + 32 * qb + r;
    if (row > cr.q_hi - 1) row = cr.q_hi - 1;
    const bf16_t* p = Qg + row * D + 8 * g;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks)
      Qr[qb][ks] = *reinterpret_cast<const bf16x8*>(p + 16 * ks);
  }

  // numerator: O[db][qb] register 4i+j = (row d = 32db + 8i + 4g + j, query 32qb + r)
  f32x16 O[DB][2];
#pragma unroll
  for (int db = 0; db < DB; ++db)
#pragma unroll
    for (int qb = 0; qb < 2; ++qb)
#pragma unroll
      for (int e = 0; e < 16; ++e) O[db][qb][e] = 0.f;
  float mrun[2] = {-INFINITY, -INFINITY};  // running max of exponent * log2(e)
  float lrun[2] = {0.f, 0.f};              // this lane half's share of the sum

  const float sc = a.scale_log2e;

  // =========================== phase S =====================================
  {
    TileRegs<64, D, NT> kreg, vreg;
    const int64_t s_lo = cr.s_lo, s_hi = cr.s_hi;
    {
      int valid = (int)((s_hi - s_lo) < 64 ? (s_hi - s_lo) : 64);
      tile_load<64, D, NT>(kreg, Kg + s_lo * D, D, valid, tid);
      tile_load<64, D, NT>(vreg, Vg + s_lo * D, D, valid, tid);
    }
    for (int64_t kt = s_lo; kt < s_hi; kt += 64) {
      __syncthreads();  // previous tile fully consumed
      tile_store<64, D, NT, false>(kreg, bufA, C::LDK, tid);
      tile_store<64, D, NT, false>(vreg, bufB, C::LDV, tid);
      __syncthreads();
      if (kt + 64 < s_hi) {  // prefetch the next tile into registers
        int64_t rem = s_hi - (kt + 64);
        int valid = (int)(rem < 64 ? rem : 64);
        tile_load<64, D, NT>(kreg, Kg + (kt + 64) * D, D, valid, tid);
        tile_load<64, D, NT>(vreg, Vg + (kt + 64) * D, D, valid, tid);
      }
      // exponents, transposed: E[kb][qb] register 4i+j = (key 32kb+8i+4g+j, query)
      f32x16 E[2][2];
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int qb = 0; qb < 2; ++qb)
#pragma unroll
          for (int e = 0; e < 16; ++e) E[kb][qb][e] = 0.f;
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) {
          bf16x8 kf = lds_read_frag(bufA + (32 * kb + r) * C::LDK + 16 * ks + 8 * g);
          E[kb][0] = mfma(kf, Qr[0][ks], E[kb][0]);
          E[kb][1] = mfma(kf, Qr[1][ks], E[kb][1]);
        }
      }
      const bool tail = (kt + 64 > s_hi);
#pragma unroll
      for (int qb = 0; qb < 2; ++qb) {
        float mx = -INFINITY;
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
          for (int e = 0; e < 16; ++e) {
            float x = E[kb][qb][e] * sc;
            if (tail) {
              int64_t key = kt + 32 * kb + 8 * (e >> 2) + 4 * g + (e & 3);
              if (key >= s_hi) x = -INFINITY;
            }
            E[kb][qb][e] = x;
            mx = fmaxf(mx, x);
          }
        }
        mx = fmaxf(mx, __shfl_xor(mx, 32));
        const float mnew = fmaxf(mrun[qb], mx);
        const float alpha = __builtin_amdgcn_exp2f(mrun[qb] - mnew);
        mrun[qb] = mnew;
        float sum = 0.f;
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
          for (int e = 0; e < 16; ++e) {
            float p = __builtin_amdgcn_exp2f(E[kb][qb][e] - mnew);
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
      // numerator += V^T P
#pragma unroll
      for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
        for (int s = 0; s < 2; ++s) {
          bf16x8 p0 = acc_to_operand(E[kb][0], s);
          bf16x8 p1 = acc_to_operand(E[kb][1], s);
#pragma unroll
          for (int db = 0; db < DB; ++db) {
            bf16x8 vf = lds_read_frag_transposed(bufB, C::LDV, 32 * kb + 16 * s, 32 * db, lane);
            O[db][0] = mfma(vf, p0, O[db][0]);
            O[db][1] = mfma(vf, p1, O[db][1]);
          }
        }
      }
    }
  }

  // complete the softmax normaliser across the two lane halves
  float nS[2], mtrue[2];
#pragma unroll
  for (int qb = 0; qb < 2; ++qb) {
    nS[qb] = lrun[qb] + __shfl_xor(lrun[qb], 32);
    mtrue[qb] = mrun[qb] * 0.6931471805599453f;  // back from base 2
  }

  // debug: softmax components
  if (a.dbg_m || a.dbg_nS || a.dbg_aS) {
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
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
  float nL[2] = {0.f, 0.f};
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
    float lin_scale[2] = {1.f, 1.f};
    if (a.stab_mode == 1) {
      lin_scale[0] = __builtin_amdgcn_exp2f(-mrun[0]);
      lin_scale[1] = __builtin_amdgcn_exp2f(-mrun[1]);
    }

    // ---- U^T = relu(W1 Q^T + b1), kept as bf16 B operands -------------------
    bf16x8 Ub[2][HID / 16];
    {
      TileRegs<64, D, NT> wreg;
      tile_load<64, D, NT>(wreg, W1, D, 64, tid);
      constexpr int NSLAB = HID / 64;
#pragma unroll
      for (int sl = 0; sl < NSLAB; ++sl) {
        __syncthreads();
        tile_store<64, D, NT, false>(wreg, bufA, C::LDK, tid);
        __syncthreads();
        if (sl + 1 < NSLAB) tile_load<64, D, NT>(wreg, W1 + (int64_t)(sl + 1) * 64 * D, D, 64, tid);
#pragma unroll
        for (int hb2 = 0; hb2 < 2; ++hb2) {
          const int hb = 2 * sl + hb2;  // 32-row block of hidden units
          f32x16 acc[2];
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            f32x4 bias = *reinterpret_cast<const f32x4*>(sb1 + 32 * hb + 8 * i + 4 * g);
#pragma unroll
            for (int j = 0; j < 4; ++j) {
              acc[0][4 * i + j] = bias[j];
              acc[1][4 * i + j] = bias[j];
            }
          }
#pragma unroll
          for (int ks = 0; ks < KS; ++ks) {
            bf16x8 wf = lds_read_frag(bufA + (32 * hb2 + r) * C::LDK + 16 * ks + 8 * g);
            acc[0] = mfma(wf, Qr[0][ks], acc[0]);
            acc[1] = mfma(wf, Qr[1][ks], acc[1]);
          }
#pragma unroll
          for (int qb = 0; qb < 2; ++qb) {
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
      tile_load<32, HID, NT>(wreg, W2, HID, 32, tid);
      tile_load<D, 32, NT>(sreg, St, DP, D, tid);
      constexpr int NPB = DP / 32;
#pragma unroll 1
      for (int pb = 0; pb < NPB; ++pb) {
        __syncthreads();
        tile_store<32, HID, NT, true>(wreg, bufA, C::LDW2, tid);
        tile_store<D, 32, NT, true>(sreg, bufB, C::LDS_S, tid);
        __syncthreads();
        if (pb + 1 < NPB) {
          tile_load<32, HID, NT>(wreg, W2 + (int64_t)(pb + 1) * 32 * HID, HID, 32, tid);
          tile_load<D, 32, NT>(sreg, St + (pb + 1) * 32, DP, D, tid);
        }
        f32x16 acc[2];
        float zv[16];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          f32x4 bias = *reinterpret_cast<const f32x4*>(sb2 + 32 * pb + 8 * i + 4 * g);
          f32x4 zz = *reinterpret_cast<const f32x4*>(sz + 32 * pb + 8 * i + 4 * g);
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            acc[0][4 * i + j] = bias[j];
            acc[1][4 * i + j] = bias[j];
            zv[4 * i + j] = zz[j];
          }
        }
#pragma unroll
        for (int ks = 0; ks < HID / 16; ++ks) {
          bf16x8 wf = lds_read_frag(bufA + r * C::LDW2 + 16 * ks + 8 * g);
          acc[0] = mfma(wf, Ub[0][ks], acc[0]);
          acc[1] = mfma(wf, Ub[1][ks], acc[1]);
        }
        const bool squared = (32 * pb >= DP / 2);
        bf16x8 Fb[2][2];
#pragma unroll
        for (int qb = 0; qb < 2; ++qb) {
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
            O[db][0] = mfma(sf, Fb[0][s], O[db][0]);
            O[db][1] = mfma(sf, Fb[1][s], O[db][1]);
          }
        }
      }
    }
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) nL[qb] += __shfl_xor(nL[qb], 32);
  }

  // =========================== merge (Eq. 5) ================================
#pragma unroll
  for (int qb = 0; qb < 2; ++qb) {
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

template __global__ void attn_kernel<64>(AttnArgs);
template __global__ void attn_kernel<128>(AttnArgs);

hipError_t launch_attn(const AttnArgs& a, int d, int grid, hipStream_t stream) {
  if (d == 128) {
    hipLaunchKernelGGL(attn_kernel<128>, dim3(grid), dim3(256), 0, stream, a);
  } else {
    hipLaunchKernelGGL(attn_kernel<64>, dim3(grid), dim3(256), 0, stream, a);
  }
  return hipGetLastError();
}

}  // namespace rehyat
