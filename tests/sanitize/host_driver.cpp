// Runs the host layer of the library (argument validation, chunk plan, workspace rules)
// under AddressSanitizer / UndefinedBehaviorSanitizer.  No call below reaches the GPU: every
// one is rejected, or answered, before the first HIP call.  Pointers are fake, aligned,
// non-null values that are never dereferenced.
#include <climits>
#include <cstdint>
#include <cstdio>
#include <cstring>
#include <vector>

#include "../../include/rehyat.h"

#define CHECK(c) do { if (!(c)) { printf("FAILED line %d: %s\n", __LINE__, #c); return 1; } } while (0)

int main() {
  void* const A = (void*)0x1000;
  rehyat_phi_params phi;
  phi.w1_q = phi.b1_q = phi.w2_q = phi.b2_q = phi.w1_k = phi.b1_k = phi.w2_k = phi.b2_k = A;
  phi.hidden = 256; phi.dprime = 256; phi.degree = 2; phi.act = 0;

  // chunk plans over a sweep of shapes, into an exactly sized table (ASan guards its ends)
  for (int T : {1, 2, 5, 21, 41, 161})
    for (int HW : {1, 7, 600, 1560})
      for (int chunk : {1, 2, 3, 7, 22, INT_MAX})
        for (int overlap : {0, 1, 3, INT_MAX}) {
          int n = -1;
          CHECK(rehyat_chunk_plan(T, HW, chunk, overlap, nullptr, &n) == REHYAT_OK);
          const int c = chunk > T ? T : chunk;
          CHECK(n == (T + c - 1) / c);
          std::vector<int64_t> table((size_t)n * 5);
          CHECK(rehyat_chunk_plan(T, HW, chunk, overlap, table.data(), &n) == REHYAT_OK);
          CHECK(table[0] == 0 && table[(size_t)(n - 1) * 5 + 1] == (int64_t)T * HW);
          for (int t = 0; t < n; ++t) {
            const int64_t* r = &table[(size_t)t * 5];
            CHECK(r[0] < r[1] && r[2] <= r[0] && r[3] == r[1] && r[4] == r[2] && r[2] >= 0);
          }
        }
  int n = 0;
  CHECK(rehyat_chunk_plan(0, 1, 1, 0, nullptr, &n) == REHYAT_E_SHAPE);
  CHECK(rehyat_chunk_plan(1, 1, 1, 0, nullptr, nullptr) == REHYAT_E_NULL);

  // workspace sizes
  CHECK(rehyat_workspace_bytes(1, 12, 128, 256) > 0);
  CHECK(rehyat_workspace_bytes(1, 12, 128, 256) % 256 == 0);
  CHECK(rehyat_workspace_bytes(1, 12, 96, 192) == 0);
  CHECK(rehyat_workspace_bytes(65535, 65535, 128, 256) > 0);   // no overflow in size_t arithmetic

  // forward: every kind of rejection
  CHECK(rehyat_forward(nullptr, A, A, &phi, A, 1, 12, 21, 1560, 128, 1, nullptr) == REHYAT_E_NULL);
  CHECK(rehyat_forward(A, A, A, nullptr, A, 1, 12, 21, 1560, 128, 1, nullptr) == REHYAT_E_NULL);
  CHECK(rehyat_forward(A, A, A, &phi, A, 0, 12, 21, 1560, 128, 1, nullptr) == REHYAT_E_SHAPE);
  CHECK(rehyat_forward(A, A, A, &phi, A, 1, 12, 21, 1560, 128, 0, nullptr) == REHYAT_E_SHAPE);
  CHECK(rehyat_forward(A, A, A, &phi, A, 1, 12, INT_MAX, INT_MAX, 128, 1, nullptr) == REHYAT_E_SHAPE);
  CHECK(rehyat_forward(A, A, A, &phi, A, INT_MAX, INT_MAX, 21, 1560, 128, 1, nullptr) == REHYAT_E_SHAPE);
  CHECK(rehyat_forward(A, A, A, &phi, A, 1, 12, 21, 1560, 96, 1, nullptr) == REHYAT_E_UNSUPPORTED);
  CHECK(rehyat_forward((char*)A + 2, A, A, &phi, A, 1, 12, 21, 1560, 128, 1, nullptr) == REHYAT_E_SHAPE);
  CHECK(rehyat_forward_ex(A, A, A, &phi, A, 1, 12, 21, 1560, 128, 1, -1, 1, 0, nullptr, nullptr) == REHYAT_E_SHAPE);
  CHECK(rehyat_forward_ex(A, A, A, &phi, A, 1, 12, 21, 1560, 128, 1, 0, 3, 0, nullptr, nullptr) == REHYAT_E_SHAPE);
  CHECK(rehyat_forward_ex(A, A, A, &phi, A, 1, 12, 21, 1560, 128, 1, 0, 1, 9, nullptr, nullptr) == REHYAT_E_SHAPE);
  {
    rehyat_phi_params bad = phi;
    bad.hidden = 128;
    CHECK(rehyat_forward(A, A, A, &bad, A, 1, 12, 21, 1560, 128, 1, nullptr) == REHYAT_E_UNSUPPORTED);
    bad = phi;
    bad.degree = 3;
    CHECK(rehyat_forward(A, A, A, &bad, A, 1, 12, 21, 1560, 128, 1, nullptr) == REHYAT_E_SHAPE);
    bad = phi;
    bad.w2_k = nullptr;
    CHECK(rehyat_forward(A, A, A, &bad, A, 1, 12, 21, 1560, 128, 1, nullptr) == REHYAT_E_NULL);
  }
  // per-call workspace rules
  const size_t need = rehyat_workspace_bytes(1, 12, 128, 256);
  CHECK(rehyat_forward_ws(A, A, A, &phi, A, 1, 12, 21, 1560, 128, 1, 0, 1, 0, nullptr, need, nullptr) == REHYAT_E_NULL);
  CHECK(rehyat_forward_ws(A, A, A, &phi, A, 1, 12, 21, 1560, 128, 1, 0, 1, 0, (char*)A + 16, need, nullptr) == REHYAT_E_WORKSPACE);
  CHECK(rehyat_forward_ws(A, A, A, &phi, A, 1, 12, 21, 1560, 128, 1, 0, 1, 0, A, need - 1, nullptr) == REHYAT_E_WORKSPACE);
  // a caller-set workspace that is too small is never replaced
  CHECK(rehyat_set_workspace((char*)A + 8, 1 << 20) == REHYAT_E_WORKSPACE);
  CHECK(rehyat_set_workspace(A, 4096) == REHYAT_OK);
  CHECK(rehyat_forward(A, A, A, &phi, A, 1, 12, 21, 1560, 128, 1, nullptr) == REHYAT_E_WORKSPACE);
  float* const F = (float*)A;
  CHECK(rehyat_step(A, A, A, &phi, F, F, A, 1, 12, 128, 1560, 1560, 1560, 0, nullptr) == REHYAT_E_WORKSPACE);
  CHECK(rehyat_state(A, A, &phi, F, F, 1, 12, 21, 1560, 128, 3, nullptr) == REHYAT_E_WORKSPACE);
  CHECK(rehyat_set_workspace(nullptr, 0) == REHYAT_OK);
  // the allocation-free entry point: more (batch, head) pairs than its fixed array holds
  CHECK(rehyat_forward_noalloc(A, A, A, &phi, A, 17, 12, 2, 8, 128, 1, nullptr) == REHYAT_E_WORKSPACE);
  // streaming step and state hook validation
  CHECK(rehyat_step(A, A, A, &phi, nullptr, F, A, 1, 12, 128, 8, 16, 8, 0, nullptr) == REHYAT_E_NULL);
  CHECK(rehyat_step(A, A, A, &phi, F, F, A, 1, 12, 128, 8, 16, 17, 0, nullptr) == REHYAT_E_SHAPE);
  CHECK(rehyat_state(A, A, &phi, F, F, 1, 12, 21, 1560, 128, 22, nullptr) == REHYAT_E_SHAPE);
  // feature-map gradient: workspace plan arithmetic over a sweep of shapes, then rejections
  for (int T : {1, 2, 21, 41, 1024})
    for (int HW : {1, 600, 1560})
      for (int chunk : {1, 3, INT_MAX})
        for (int B : {1, 2, 64}) {
          const size_t wb = rehyat_phi_backward_workspace_bytes(B, 12, T, HW, 128, chunk);
          CHECK(wb > 0 && wb % 256 == 0);
          CHECK(wb >= rehyat_phi_backward_workspace_bytes(B, 12, T, HW, 64, chunk));
        }
  CHECK(rehyat_phi_backward_workspace_bytes(1, 12, 1025, 1, 128, 1) == 0);
  CHECK(rehyat_phi_backward_workspace_bytes(1, 12, INT_MAX, INT_MAX, 128, 1) == 0);
  CHECK(rehyat_phi_backward_workspace_bytes(65535, 65535, 21, 1560, 128, 1) == 0);
  {
    rehyat_phi_grads g;
    g.w1_q = g.b1_q = g.w2_q = g.b2_q = g.w1_k = g.b1_k = g.w2_k = g.b2_k = A;
    const size_t wb = rehyat_phi_backward_workspace_bytes(1, 12, 21, 1560, 128, 1);
    CHECK(rehyat_phi_backward(A, A, A, &phi, nullptr, A, nullptr, &g, 1, 12, 21, 1560, 128, 1, 0, A, wb, nullptr) == REHYAT_E_NULL);
    CHECK(rehyat_phi_backward(A, A, A, &phi, A, nullptr, nullptr, nullptr, 1, 12, 21, 1560, 128, 1, 0, A, wb, nullptr) == REHYAT_E_NULL);
    CHECK(rehyat_phi_backward(A, A, A, &phi, A, nullptr, nullptr, &g, 1, 12, 21, 1560, 128, 1, 0, nullptr, wb, nullptr) == REHYAT_E_NULL);
    CHECK(rehyat_phi_backward(A, A, A, &phi, A, nullptr, nullptr, &g, 1, 12, 21, 1560, 128, 1, 0, A, wb - 1, nullptr) == REHYAT_E_WORKSPACE);
    CHECK(rehyat_phi_backward(A, A, A, &phi, A, nullptr, nullptr, &g, 1, 12, 21, 1560, 128, 1, 0, (char*)A + 64, wb, nullptr) == REHYAT_E_WORKSPACE);
    CHECK(rehyat_phi_backward(A, A, A, &phi, A, nullptr, nullptr, &g, 1, 12, 2000, 1, 128, 1, 0, A, (size_t)1 << 40, nullptr) == REHYAT_E_UNSUPPORTED);
    CHECK(rehyat_phi_backward(A, A, A, &phi, A, nullptr, nullptr, &g, 1, 12, 21, 1560, 128, 1, -1, A, wb, nullptr) == REHYAT_E_SHAPE);
    rehyat_forward_saved sv;
    sv.nS = (const float*)A;
    sv.nL = nullptr;
    CHECK(rehyat_phi_backward(A, A, A, &phi, A, A, &sv, &g, 1, 12, 21, 1560, 128, 1, 0, A, wb, nullptr) == REHYAT_E_NULL);
    sv.nL = (const float*)A;
    CHECK(rehyat_phi_backward(A, A, A, &phi, A, nullptr, &sv, &g, 1, 12, 21, 1560, 128, 1, 0, A, wb, nullptr) == REHYAT_E_NULL);
    g.b1_k = nullptr;
    CHECK(rehyat_phi_backward(A, A, A, &phi, A, nullptr, nullptr, &g, 1, 12, 21, 1560, 128, 1, 0, A, wb, nullptr) == REHYAT_E_NULL);
  }
  CHECK(rehyat_profile_read(nullptr, nullptr) == REHYAT_E_NULL);
  for (int code = 1; code >= -7; --code) CHECK(std::strlen(rehyat_status_string(code)) > 0);
  CHECK(rehyat_version() >= 200);
  CHECK(std::strlen(rehyat_attn_kernel_name(128)) > 0 && std::strlen(rehyat_attn_kernel_name(7)) == 0);
  CHECK(rehyat_shutdown() == REHYAT_OK);
  printf("host sanitize ok\n");
  return 0;
}
