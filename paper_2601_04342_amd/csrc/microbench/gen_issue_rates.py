"""Writes issue_rates.hip: instruction-issue micro-benchmarks for gfx950, each pattern one
inline-asm block so that the order is exactly what is measured.  Patterns: 16 bf16
32x32x16 MFMAs (M16); k x 16 independent v_fma_f32 (Vk); one MFMA followed by k vector
instructions, 16 times (MVk; accumulators in VGPRs or AGPRs); v_exp_f32, v_max3_f32,
v_cvt_pk_bf16_f32, v_mov_b32 streams; MFMA mixed with exponentials and FMAs (ME*).  One
workgroup per CU, 256 threads (one wave per SIMD) and 512 threads (two waves per SIMD).
Prints, per pattern, the shader-clock cycles per iteration seen by a wave (clock64) and the
wall time per iteration in cycles of the nominal 2.4 GHz clock.

    python gen_issue_rates.py && hipcc --offload-arch=gfx950 -O3 -o issue_rates issue_rates.hip && ./issue_rates
"""
pats = {}
def mfma(i, acc='v'):
    return f"v_mfma_f32_32x32x16_bf16 %{i}, %4, %5, %{i}"
def fma(j):   # x_j = x_j * k + x_j  (registers %8..%15)
    return f"v_fma_f32 %{8+j}, %{8+j}, %6, %{8+j}"
def vexp(j):
    return f"v_exp_f32 %{8+j}, %{8+j}"
def vmax3(j):
    return f"v_max3_f32 %{8+j}, %{8+j}, %6, %7"
def vcvt(j):
    return f"v_cvt_pk_bf16_f32 %{8+j}, %{8+j}, %6"
def vmov(j):
    return f"v_mov_b32 %{8+j}, %6"
def body_mv(k, op=fma, nm=16):
    lines=[]; j=0
    for m in range(nm):
        lines.append(mfma(m%4))
        for _ in range(k):
            lines.append(op(j%8)); j+=1
    return lines
pats['M16'] = [mfma(m%4) for m in range(16)]
for k in (1,2,3,4,5,6,7,8): pats[f'V{k}x16'] = [fma(j%8) for j in range(16*k)]
for k in (1,2,3,4,5,6,7,8): pats[f'MV{k}'] = body_mv(k)
pats['E64'] = [vexp(j%8) for j in range(64)]
pats['E32F96'] = sum([[vexp(j%8), fma((j+1)%8), fma((j+2)%8), fma((j+3)%8)] for j in range(32)], [])
pats['ME2'] = body_mv(2, vexp)
pats['ME1F3'] = sum([[mfma(m%4), vexp((4*m)%8), fma((4*m+1)%8), fma((4*m+2)%8), fma((4*m+3)%8)] for m in range(16)], [])
pats['ME2F6'] = sum([[mfma(m%4), vexp((m)%8), fma((m+1)%8), fma((m+2)%8), fma((m+3)%8), vexp((m+4)%8), fma((m+5)%8), fma((m+6)%8), fma((m+7)%8)] for m in range(16)], [])
pats['MAX3_64'] = [vmax3(j%8) for j in range(64)]
pats['CVT64'] = [vcvt(j%8) for j in range(64)]
pats['MOV64'] = [vmov(j%8) for j in range(64)]
names = list(pats)
src = r'''#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdlib>
#define CK(x) do { hipError_t e = (x); if (e != hipSuccess) { printf("HIP error %s at %d\n", hipGetErrorString(e), __LINE__); exit(1);} } while (0)
typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
template <int PAT, bool AGPR>
__global__ void __launch_bounds__(512) k(float* out, long long* cyc, int iters) {
  bf16x8 a, b;
  for (int e = 0; e < 8; ++e) { a[e] = (__bf16)(1.0f + threadIdx.x * 0.001f); b[e] = (__bf16)(0.5f); }
  f32x16 c0 = {0}, c1 = {0}, c2 = {0}, c3 = {0};
  float x0 = threadIdx.x * 1e-3f, x1 = x0 + 1, x2 = x0 + 2, x3 = x0 + 3, x4 = x0 + 4, x5 = x0 + 5, x6 = x0 + 6, x7 = x0 + 7;
  float kk = 0.25f, k2 = 0.5f;
  long long t0 = clock64();
  for (int i = 0; i < iters; ++i) {
'''
for pi, n in enumerate(names):
    body = "\\n\\t".join(pats[n])
    for ag in (False, True):
        c = 'a' if ag else 'v'
        src += f'''    if (PAT == {pi} && AGPR == {'true' if ag else 'false'}) asm volatile("{body}"
      : "+{c}"(c0), "+{c}"(c1), "+{c}"(c2), "+{c}"(c3) : "v"(a), "v"(b), "v"(kk), "v"(k2), "v"(x0), "v"(x1), "v"(x2), "v"(x3), "v"(x4), "v"(x5), "v"(x6), "v"(x7));
'''
src += r'''  }
  long long t1 = clock64();
  float s = 0;
  for (int r = 0; r < 16; ++r) s += c0[r] + c1[r] + c2[r] + c3[r];
  s += x0 + x1 + x2 + x3 + x4 + x5 + x6 + x7;
  out[blockIdx.x * blockDim.x + threadIdx.x] = s;
  if ((threadIdx.x & 63) == 0) cyc[blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6)] = t1 - t0;
}
template <int PAT, bool AGPR>
void run(const char* name, float* d, long long* dc, int threads) {
  const int iters = 2000, blocks = 256;
  hipEvent_t e0, e1; CK(hipEventCreate(&e0)); CK(hipEventCreate(&e1));
  float ms = 0;
  for (int rep = 0; rep < 2; ++rep) {
    CK(hipEventRecord(e0));
    k<PAT, AGPR><<<blocks, threads>>>(d, dc, iters);
    CK(hipEventRecord(e1)); CK(hipEventSynchronize(e1));
    CK(hipEventElapsedTime(&ms, e0, e1));
  }
  static long long h[256 * 8];
  const int nw = blocks * threads / 64;
  CK(hipMemcpy(h, dc, nw * sizeof(long long), hipMemcpyDeviceToHost));
  double avg = 0; for (int i = 0; i < nw; ++i) avg += h[i]; avg /= nw;
  printf("%-10s %s waves/SIMD %d : clock64/iter %8.1f   wall cycles@2.4/iter %8.1f   (ratio %.3f)\n", name, AGPR ? "agpr" : "vgpr",
         threads / 256, avg / iters, ms * 2.4e6 / iters, (avg / iters) / (ms * 2.4e6 / iters));
}
int main() {
  float* d; long long* dc;
  CK(hipMalloc(&d, 256 * 512 * 4)); CK(hipMalloc(&dc, 256 * 8 * 8));
'''
for pi, n in enumerate(names):
    for ag in (False, True):
        if ag and not n.startswith('M'): continue
        if n.startswith('MAX') or n.startswith('MOV'):
            if ag: continue
        for th in (256, 512):
            src += f'  run<{pi}, {"true" if ag else "false"}>("{n}", d, dc, {th});\n'
src += '  printf("issue done\\n");\n  return 0;\n}\n'
import os
open(os.path.join(os.path.dirname(os.path.abspath(__file__)), 'issue_rates.hip'), 'w').write(src)
