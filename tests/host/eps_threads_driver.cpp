// Host-only driver for sanitizer builds of the EPS (csrc/eps.cpp): two threads call into one store at the same
// time, the way the trainer's eager-update thread and its main thread do (Section 2.1: the EPS updates "eagerly",
// in parallel with the device), and the results must equal those of the same calls made one after the other.
// Built by tests/test_host_logic.py with -fsanitize=address,undefined and with -fsanitize=thread; exits 0 when
// everything matched (the sanitizers make the process fail on their own findings).
//
// The four HIP runtime functions eps.cpp uses are defined here as "no GPU": the store then takes its pageable
// path, and the sanitized process needs no GPU runtime.
#include <hip/hip_runtime_api.h>

#include <cmath>
#include <cstdio>
#include <cstring>
#include <thread>
#include <vector>

#include "../../include/l2l.h"

extern "C" {
hipError_t hipGetDeviceCount(int* n) { if (n) *n = 0; return hipErrorNoDevice; }
hipError_t hipGetLastError(void) { return hipSuccess; }
hipError_t hipHostMalloc(void**, size_t, unsigned int) { return hipErrorOutOfMemory; }
hipError_t hipHostFree(void*) { return hipSuccess; }
}

namespace {

const size_t kElems[3] = {70000 + 7, 200000 + 3, 1000};   // two blocks large enough for the thread pool, one small

void fill(eps_store* e) {
  for (int b = 0; b < 3; ++b) {
    float* w = eps_master(e, b);
    float* g = eps_grad(e, b);
    uint16_t* g16 = (uint16_t*)eps_grad16(e, b);
    for (size_t i = 0; i < kElems[b]; ++i) {
      w[i] = 0.02f * std::sin(0.37f * (float)i + (float)b);
      g[i] = 1e-3f * std::cos(0.11f * (float)i - (float)b);
      float h = 2e-3f * std::sin(0.05f * (float)i);
      uint32_t u;
      std::memcpy(&u, &h, 4);
      g16[i] = (uint16_t)(u >> 16);   // a bf16 pattern (truncated: any pattern will do)
    }
  }
}

// the calls of thread A and of thread B touch different blocks, so their order does not matter for the result
void work_a(eps_store* e) {
  for (int t = 1; t <= 3; ++t) {
    eps_adam_step(e, 0, 0, t, 1e-3, 0.9, 0.999, 1e-8);
    int bad = 0;
    eps_grad_unscale(e, 0, 0, 0.5, &bad);
  }
  eps_refresh_ship(e, 0, 0);
}
void work_b(eps_store* e) {
  const long long seg_b[2] = {0, 150000}, seg_e[2] = {150000, (long long)kElems[1]};
  const double decay[2] = {1.0, 0.0};
  for (int t = 1; t <= 3; ++t) {
    eps_grad_widen(e, 1, 2, L2L_BF16);
    eps_lamb_step(e, 1, 1, t, 1e-3, 0.9, 0.999, 1e-6, 0.01, 2, seg_b, seg_e, decay);
    eps_adam_step_range16(e, 2, 0, (long long)kElems[2], t, 1e-3, 0.9, 0.999, 1e-8, L2L_BF16);
    eps_adam_step_range(e, 1, 128, 70000, t, 1e-4, 0.9, 0.999, 1e-8);
  }
}

}  // namespace

int main() {
  eps_store *par = nullptr, *ser = nullptr;
  if (eps_create(3, kElems, L2L_BF16, 4, &par) != L2L_OK || eps_create(3, kElems, L2L_BF16, 4, &ser) != L2L_OK) return 2;
  if (eps_enable_grad16(par) != L2L_OK || eps_enable_grad16(ser) != L2L_OK) return 2;
  fill(par);
  fill(ser);
  std::thread a(work_a, par), b(work_b, par);
  a.join();
  b.join();
  work_a(ser);
  work_b(ser);
  // LAMB's norms are sums over per-thread partial sums added under a mutex in arrival order: the trust ratio may
  // differ in its last bits between two runs, so block 1 is compared to a tolerance and the others exactly
  bool ok = true;
  for (int blk = 0; blk < 3; ++blk) {
    const float *p = eps_master(par, blk), *s = eps_master(ser, blk);
    for (size_t i = 0; i < kElems[blk]; ++i) {
      const float tol = blk == 1 ? 1e-6f * (std::fabs(s[i]) + 1e-3f) : 0.f;
      if (!(std::fabs(p[i] - s[i]) <= tol)) { std::printf("block %d element %zu: %g vs %g\n", blk, i, p[i], s[i]); ok = false; break; }
    }
  }
  eps_destroy(par);
  eps_destroy(ser);
  std::printf(ok ? "eps threads driver: ok\n" : "eps threads driver: MISMATCH\n");
  return ok ? 0 : 1;
}
