// Prefix pass over chunk states for gfx950 (Eq. 14-18): turns the per-segment
// partial sums written by the state kernel into the state S_t, z_t seen by each
// chunk of the window, s_0 = z_0 = 0, s_{t+1} = s_t + (tokens that entered the
// linear set between chunk t and chunk t+1).  Purely HBM-bound: each thread
// owns four consecutive state elements and walks the window's chunks in order
// (fixed summation order, so results are bit-reproducible).  S_t is written in
// bf16, transposed ([d][D']), ready to be an MFMA operand of the read-out; z_t
// stays fp32.  The running total is left in `carry` for the next window.
#include "rehyat_device.h"
#include "rehyat_kernels.h"

namespace rehyat {

__global__ void __launch_bounds__(256)
prefix_kernel(PrefixArgs a) {
  const int bh = blockIdx.y;
  const int idx = (blockIdx.x * 256 + threadIdx.x) * 4;
  if (idx >= a.elems) return;
  const float* part = a.partial + (int64_t)bh * a.partial_slots * a.elems + idx;
  float* carry = a.carry + (int64_t)bh * a.elems + idx;
  f32x4 acc = {0.f, 0.f, 0.f, 0.f};
  if (!a.first_window) acc = *reinterpret_cast<const f32x4*>(carry);
  const bool is_s = idx < a.s_elems;
  const int n_steps = a.n_chunks > a.n_seg ? a.n_chunks : a.n_seg;
  for (int c = 0; c < n_steps; ++c) {
    if (c < a.n_chunks) {
      if (is_s) {
        u32x2 pk;
        pk[0] = pack_bf16(acc[0], acc[1]);
        pk[1] = pack_bf16(acc[2], acc[3]);
        *reinterpret_cast<u32x2*>(a.state_s + ((int64_t)bh * a.state_slots + c) * a.s_elems + idx) = pk;
      } else {
        *reinterpret_cast<f32x4*>(a.state_z + ((int64_t)bh * a.state_slots + c) * (a.elems - a.s_elems) +
                                  (idx - a.s_elems)) = acc;
      }
    }
    if (c < a.n_seg) {
      for (int sp = 0; sp < a.nsplit; ++sp) {
        f32x4 x = *reinterpret_cast<const f32x4*>(part + (int64_t)(c * a.nsplit + sp) * a.elems);
        acc += x;
      }
    }
  }
  *reinterpret_cast<f32x4*>(carry) = acc;
}

__global__ void __launch_bounds__(256)
bidir_state_kernel(BidirArgs a) {
  const int bh = blockIdx.y;
  const int idx = (blockIdx.x * 256 + threadIdx.x) * 4;
  if (idx >= a.elems) return;
  const float* part = a.partial + (int64_t)bh * a.partial_slots * a.elems + idx;
  const f32x4 total = *reinterpret_cast<const f32x4*>(a.total + (int64_t)bh * a.elems + idx);
  const bool is_s = idx < a.s_elems;
  for (int c = 0; c < a.n_chunks; ++c) {
    const int t = a.chunk0 + c;
    // frames of the softmax window of chunk t (Eq. 12)
    int f_lo = t * a.chunk - a.overlap;
    if (f_lo < 0) f_lo = 0;
    int f_hi = (t + 1) * a.chunk;
    if (f_hi > a.T) f_hi = a.T;
    f32x4 w = {0.f, 0.f, 0.f, 0.f};
    for (int f = f_lo; f < f_hi; ++f)
      for (int sp = 0; sp < a.nsplit; ++sp)
        w += *reinterpret_cast<const f32x4*>(part + (int64_t)((f - a.frame0) * a.nsplit + sp) * a.elems);
    const f32x4 acc = total - w;
    if (is_s) {
      u32x2 pk;
      pk[0] = pack_bf16(acc[0], acc[1]);
      pk[1] = pack_bf16(acc[2], acc[3]);
      *reinterpret_cast<u32x2*>(a.state_s + ((int64_t)bh * a.state_slots + c) * a.s_elems + idx) = pk;
    } else {
      *reinterpret_cast<f32x4*>(a.state_z + ((int64_t)bh * a.state_slots + c) * (a.elems - a.s_elems) +
                                (idx - a.s_elems)) = acc;
    }
  }
}

__global__ void __launch_bounds__(256)
state_out_kernel(StateOutArgs a) {
  const int bh = blockIdx.y;
  const int i = blockIdx.x * 256 + threadIdx.x;  // index into S_out [dprime][d]
  const int n = a.d * a.dprime;
  const float* c = a.carry + (int64_t)bh * (n + a.dprime);
  if (i < n) {
    const int e = i / a.d, col = i % a.d;
    a.S_out[(int64_t)bh * n + i] = c[col * a.dprime + e];
  }
  if (i < a.dprime) a.z_out[(int64_t)bh * a.dprime + i] = c[n + i];
}

// One tile of 64 features x 16 head-dimension columns of S per block, transposed through LDS
// both ways: the pieces -- the bulk of the bytes -- and the state slot are moved in 16-byte
// accesses along the workspace's [d][dprime] rows, the caller's [dprime][d] rows in 64-byte runs.
__global__ void __launch_bounds__(256)
step_state_kernel(StepStateArgs a) {
  __shared__ float tile[64][17];
  const int bh = blockIdx.z;
  const int f0 = blockIdx.x * 64, e0 = blockIdx.y * 16;
  const int tid = threadIdx.x;
  const int n = a.d * a.dprime, elems = n + a.dprime;
  float* S = a.S + (int64_t)bh * n;
#pragma unroll
  for (int m = 0; m < 4; ++m) {
    const int idx = tid + 256 * m, row = idx >> 4, col = idx & 15;
    tile[row][col] = S[(int64_t)(f0 + row) * a.d + e0 + col];
  }
  __syncthreads();
  const float* part = a.partial + (int64_t)bh * a.partial_slots * elems;
  bf16_t* slot = a.state_s + (int64_t)bh * a.state_slots * n;
  {
    const int f4 = tid & 15, el = tid >> 4;   // features 4 f4 .. 4 f4 + 3 of row e0 + el of S^T
    const int64_t o = (int64_t)(e0 + el) * a.dprime + f0 + 4 * f4;
    f32x4 v = {tile[4 * f4][el], tile[4 * f4 + 1][el], tile[4 * f4 + 2][el], tile[4 * f4 + 3][el]};
    if (a.write_slot) {
      u32x2 pk;
      pk[0] = pack_bf16(v[0], v[1]);
      pk[1] = pack_bf16(v[2], v[3]);
      *reinterpret_cast<u32x2*>(slot + o) = pk;
    }
#pragma unroll 8
    for (int sp = 0; sp < a.nsplit; ++sp) v += *reinterpret_cast<const f32x4*>(part + (int64_t)sp * elems + o);
#pragma unroll
    for (int i = 0; i < 4; ++i) tile[4 * f4 + i][el] = v[i];
  }
  __syncthreads();
  if (a.nsplit > 0) {   // nothing added: the caller's state stays as it is
#pragma unroll
    for (int m = 0; m < 4; ++m) {
      const int idx = tid + 256 * m, row = idx >> 4, col = idx & 15;
      S[(int64_t)(f0 + row) * a.d + e0 + col] = tile[row][col];
    }
  }
  if (blockIdx.y == 0 && tid < 64) {   // z of this block's 64 features
    const int f = f0 + tid;
    float v = a.z[(int64_t)bh * a.dprime + f];
    if (a.write_slot) a.state_z[(int64_t)bh * a.state_slots * a.dprime + f] = v;
    for (int sp = 0; sp < a.nsplit; ++sp) v += part[(int64_t)sp * elems + n + f];
    if (a.nsplit > 0) a.z[(int64_t)bh * a.dprime + f] = v;
  }
}

// s_0 = 0, z_0 = 0 (Eq. 14-15) in the layout of the public state hook
__global__ void __launch_bounds__(256)
zero_state_kernel(float* S, float* z, int64_t n_s, int64_t n_z) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i < n_s) S[i] = 0.f;
  if (i < n_z) z[i] = 0.f;
}

hipError_t launch_zero_state(float* S, float* z, int BH, int d, int dprime, hipStream_t stream) {
  const int64_t n_s = (int64_t)BH * d * dprime, n_z = (int64_t)BH * dprime;
  hipLaunchKernelGGL(zero_state_kernel, dim3((unsigned)((n_s + 255) / 256)), dim3(256), 0, stream, S, z,
                     n_s, n_z);
  return hipGetLastError();
}

hipError_t launch_prefix(const PrefixArgs& a, hipStream_t stream) {
  dim3 grid((a.elems / 4 + 255) / 256, a.BH);
  hipLaunchKernelGGL(prefix_kernel, grid, dim3(256), 0, stream, a);
  return hipGetLastError();
}

hipError_t launch_state_out(const StateOutArgs& a, hipStream_t stream) {
  dim3 grid((a.d * a.dprime + 255) / 256, a.BH);
  hipLaunchKernelGGL(state_out_kernel, grid, dim3(256), 0, stream, a);
  return hipGetLastError();
}

hipError_t launch_bidir_state(const BidirArgs& a, hipStream_t stream) {
  dim3 grid((a.elems / 4 + 255) / 256, a.BH);
  hipLaunchKernelGGL(bidir_state_kernel, grid, dim3(256), 0, stream, a);
  return hipGetLastError();
}

hipError_t launch_step_state(const StepStateArgs& a, hipStream_t stream) {
  dim3 grid(a.dprime / 64, a.d / 16, a.BH);
  hipLaunchKernelGGL(step_state_kernel, grid, dim3(256), 0, stream, a);
  return hipGetLastError();
}

}  // namespace rehyat
