// Host eager param-server (EPS): the model and the optimizer live in host DRAM (Section 2.1); the
// device only ever sees one layer's shipping copy.  fp32 master weights and Adam moments stay on the
// host, the optimizer runs on host cores, and a reduced-precision copy is what gets shipped
// (cross mixed precision, Section 2.3, with bf16 in place of FP16).
#include <hip/hip_runtime_api.h>

#include <immintrin.h>

#include <atomic>
#include <cmath>
#include <condition_variable>
#include <cstdlib>
#include <cstring>
#include <functional>
#include <mutex>
#include <thread>
#include <vector>

#include "../../include/l2l.h"

namespace {

// Persistent worker pool: run(n, f) calls f(begin, end) on disjoint chunks of [0, n).
class Pool {
 public:
  explicit Pool(int threads) : n_(threads) {
    for (int i = 1; i < n_; ++i) workers_.emplace_back([this, i] { loop(i); });
  }
  ~Pool() {
    {
      std::lock_guard<std::mutex> l(mu_);
      stop_ = true;
      ++epoch_;
    }
    cv_.notify_all();
    for (auto& t : workers_) t.join();
  }
  int size() const { return n_; }
  void run(size_t n, const std::function<void(size_t, size_t)>& f) {
    if (n_ == 1 || n < 65536) { f(0, n); return; }
    // one job at a time: a second caller (the eager-update thread and the training thread may both get here) waits
    // for the first to finish instead of overwriting its job
    std::lock_guard<std::mutex> serial(run_mu_);
    {
      std::lock_guard<std::mutex> l(mu_);
      fn_ = &f;
      total_ = n;
      pending_ = n_ - 1;
      ++epoch_;
    }
    cv_.notify_all();
    chunk(0);
    std::unique_lock<std::mutex> l(mu_);
    done_.wait(l, [this] { return pending_ == 0; });
    fn_ = nullptr;
  }

 private:
  void chunk(int i) {
    // chunk boundaries on multiples of 16 elements so that vector loops stay aligned
    const size_t per = ((total_ + n_ - 1) / n_ + 15) / 16 * 16;
    const size_t b = std::min(total_, per * i), e = std::min(total_, b + per);
    if (b < e) (*fn_)(b, e);
  }
  void loop(int i) {
    unsigned seen = 0;
    for (;;) {
      {
        std::unique_lock<std::mutex> l(mu_);
        cv_.wait(l, [&] { return epoch_ != seen; });
        seen = epoch_;
        if (stop_) return;
      }
      chunk(i);
      std::lock_guard<std::mutex> l(mu_);
      if (--pending_ == 0) done_.notify_one();
    }
  }
  int n_;
  std::vector<std::thread> workers_;
  std::mutex mu_, run_mu_;
  std::condition_variable cv_, done_;
  const std::function<void(size_t, size_t)>* fn_ = nullptr;
  size_t total_ = 0;
  int pending_ = 0;
  unsigned epoch_ = 0;
  bool stop_ = false;
};

struct Block {
  size_t n = 0;
  bool pinned = false;
  float *w = nullptr, *m = nullptr, *v = nullptr;  // pageable
  void* ship = nullptr;                             // pinned
  float* grad = nullptr;                            // pinned
  uint16_t* grad16 = nullptr;                       // pinned, optional: landing buffer of 16-bit drains
};

inline uint16_t f32_to_bf16_rne(float f) {
  uint32_t u;
  std::memcpy(&u, &f, 4);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40);  // quiet NaN
  return (uint16_t)((u + 0x7fffu + ((u >> 16) & 1u)) >> 16);
}

}  // namespace

struct eps_store {
  std::vector<Block> blocks;
  int ship_dtype = L2L_BF16;
  Pool* pool = nullptr;
  size_t host_bytes = 0;
  bool pinned = false;
};

static void ship_range(const eps_store* e, const Block& b, size_t lo, size_t hi) {
  if (e->ship_dtype == L2L_BF16) {
    uint16_t* d = (uint16_t*)b.ship;
    for (size_t i = lo; i < hi; ++i) d[i] = f32_to_bf16_rne(b.w[i]);
  } else if (e->ship_dtype == L2L_FP16) {
    uint16_t* d = (uint16_t*)b.ship;
    for (size_t i = lo; i < hi; ++i) d[i] = _cvtss_sh(b.w[i], _MM_FROUND_TO_NEAREST_INT | _MM_FROUND_NO_EXC);   // IEEE half, ties to even
  } else {
    std::memcpy((float*)b.ship + lo, b.w + lo, (hi - lo) * sizeof(float));
  }
}

// bias-corrected Adam on elements [lo, hi) of a block with the gradients at g[k - lo0 ...]: g points at the gradient of
// element `lo` (the fp32 gradient buffer, or a widened run of the 16-bit landing buffer)
static void adam_run(const Block& b, size_t lo, size_t hi, const float* __restrict g, float lr, float beta1, float beta2,
                     float eps_a, float omb1, float omb2, float c1, float c2) {
  float* __restrict w = b.w + lo;
  float* __restrict m = b.m + lo;
  float* __restrict v = b.v + lo;
  const size_t n = hi - lo;
#pragma omp simd   // the arrays are distinct allocations: iterations are independent
  for (size_t k = 0; k < n; ++k) {
    const float gk = g[k];
    const float mk = beta1 * m[k] + omb1 * gk;
    const float vk = beta2 * v[k] + omb2 * gk * gk;
    m[k] = mk;
    v[k] = vk;
    w[k] -= lr * (mk * c1) / (std::sqrt(vk * c2) + eps_a);
  }
}

static void widen_run(const uint16_t* __restrict s, float* __restrict d, size_t n, int dtype) {
  if (dtype == L2L_BF16) {
#pragma omp simd
    for (size_t k = 0; k < n; ++k) {
      const uint32_t u = (uint32_t)s[k] << 16;
      float f;
      std::memcpy(&f, &u, 4);
      d[k] = f;
    }
  } else {
    size_t k = 0;
    for (; k + 8 <= n; k += 8) _mm256_storeu_ps(d + k, _mm256_cvtph_ps(_mm_loadu_si128((const __m128i*)(s + k))));
    for (; k < n; ++k) d[k] = _cvtsh_ss(s[k]);
  }
}

// Adam on elements [e0, e0 + n) of a block, master -> shipping copy included.  gd: where the gradients are read from:
// the fp32 buffer (L2L_F32) or the 16-bit landing buffer (L2L_BF16 / L2L_FP16), widened a cache-resident run at a time
// (a loop that mixes 16- and 32-bit lanes does not vectorise; two loops over a run that stays in L1 do).
static void adam_range(eps_store* e, const Block& b, size_t e0, size_t n, int gd, float lr, float beta1, float beta2,
                       float eps_a, float omb1, float omb2, float c1, float c2) {
  e->pool->run(n, [&](size_t lo, size_t hi) {
    if (gd == L2L_F32) {
      adam_run(b, e0 + lo, e0 + hi, b.grad + e0 + lo, lr, beta1, beta2, eps_a, omb1, omb2, c1, c2);
    } else {
      constexpr size_t RUN = 2048;
      alignas(64) float tmp[RUN];
      for (size_t k0 = e0 + lo; k0 < e0 + hi; k0 += RUN) {
        const size_t k1 = std::min(e0 + hi, k0 + RUN);
        widen_run(b.grad16 + k0, tmp, k1 - k0, gd);
        adam_run(b, k0, k1, tmp, lr, beta1, beta2, eps_a, omb1, omb2, c1, c2);
      }
    }
    ship_range(e, b, e0 + lo, e0 + hi);
  });
}

extern "C" {

int eps_create(int n_blocks, const size_t* elems, int ship_dtype, int threads, eps_store** out) {
  if (!out || !elems || n_blocks <= 0 || (ship_dtype != L2L_F32 && ship_dtype != L2L_BF16 && ship_dtype != L2L_FP16)) return L2L_E_ARG;
  *out = nullptr;
  if (threads <= 0) threads = (int)std::thread::hardware_concurrency();
  if (threads <= 0) threads = 1;
  eps_store* e = new eps_store;
  e->ship_dtype = ship_dtype;
  e->blocks.resize(n_blocks);
  {
    int ndev = 0;
    e->pinned = hipGetDeviceCount(&ndev) == hipSuccess && ndev > 0;
    if (!e->pinned) (void)hipGetLastError();
  }
  const size_t se = ship_dtype == L2L_F32 ? 4 : 2;
  for (int i = 0; i < n_blocks; ++i) {
    Block& b = e->blocks[i];
    b.n = elems[i];
    const size_t fb = (b.n * 4 + 63) / 64 * 64;
    b.w = (float*)aligned_alloc(64, fb);
    b.m = (float*)aligned_alloc(64, fb);
    b.v = (float*)aligned_alloc(64, fb);
    bool ok = b.w && b.m && b.v;
    if (ok && e->pinned) {
      ok = hipHostMalloc(&b.ship, b.n * se, hipHostMallocDefault) == hipSuccess;
      if (ok) ok = hipHostMalloc((void**)&b.grad, b.n * 4, hipHostMallocDefault) == hipSuccess;
      b.pinned = true;
    } else if (ok) {  // no GPU in this process: plain host memory (host-side logic still works)
      b.ship = aligned_alloc(64, (b.n * se + 63) / 64 * 64);
      b.grad = (float*)aligned_alloc(64, fb);
      ok = b.ship && b.grad;
    }
    if (!ok) {
      (void)hipGetLastError();
      eps_destroy(e);
      return L2L_E_NOMEM;
    }
    std::memset(b.w, 0, b.n * 4);
    std::memset(b.m, 0, b.n * 4);
    std::memset(b.v, 0, b.n * 4);
    std::memset(b.ship, 0, b.n * se);
    std::memset(b.grad, 0, b.n * 4);
    e->host_bytes += 3 * fb + b.n * se + b.n * 4;
  }
  e->pool = new Pool(threads);
  *out = e;
  return L2L_OK;
}

int eps_destroy(eps_store* e) {
  if (!e) return L2L_E_ARG;
  delete e->pool;
  for (Block& b : e->blocks) {
    free(b.w);
    free(b.m);
    free(b.v);
    if (b.pinned) {
      if (b.ship) (void)hipHostFree(b.ship);
      if (b.grad) (void)hipHostFree(b.grad);
      if (b.grad16) (void)hipHostFree(b.grad16);
    } else {
      free(b.ship);
      free(b.grad);
      free(b.grad16);
    }
  }
  delete e;
  return L2L_OK;
}

static Block* blk(eps_store* e, int i) {
  if (!e || i < 0 || i >= (int)e->blocks.size()) return nullptr;
  return &e->blocks[i];
}
float* eps_master(eps_store* e, int i) { Block* b = blk(e, i); return b ? b->w : nullptr; }
void* eps_ship(eps_store* e, int i) { Block* b = blk(e, i); return b ? b->ship : nullptr; }
float* eps_grad(eps_store* e, int i) { Block* b = blk(e, i); return b ? b->grad : nullptr; }
float* eps_moment(eps_store* e, int i, int which) {
  Block* b = blk(e, i);
  if (!b || (which != 0 && which != 1)) return nullptr;
  return which == 0 ? b->m : b->v;
}
size_t eps_host_bytes(const eps_store* e) { return e ? e->host_bytes : 0; }
int eps_is_pinned(const eps_store* e) { return e && e->pinned ? 1 : 0; }

int eps_refresh_ship(eps_store* e, int first, int last) {
  if (!e || first < 0 || last >= (int)e->blocks.size() || first > last) return L2L_E_ARG;
  for (int i = first; i <= last; ++i) {
    const Block& b = e->blocks[i];
    e->pool->run(b.n, [&](size_t lo, size_t hi) { ship_range(e, b, lo, hi); });
  }
  return L2L_OK;
}

int eps_adam_step(eps_store* e, int first, int last, int t, double lr_d, double beta1_d, double beta2_d, double eps_a_d) {
  if (!e || first < 0 || last >= (int)e->blocks.size() || first > last || t < 1) return L2L_E_ARG;
  // hyper-parameters arrive in double so that 1 - beta is rounded once, not computed in fp32
  const float lr = (float)lr_d, beta1 = (float)beta1_d, beta2 = (float)beta2_d, eps_a = (float)eps_a_d;
  const float omb1 = (float)(1.0 - beta1_d), omb2 = (float)(1.0 - beta2_d);
  const float c1 = (float)(1.0 / (1.0 - std::pow(beta1_d, t)));
  const float c2 = (float)(1.0 / (1.0 - std::pow(beta2_d, t)));
  for (int i = first; i <= last; ++i) adam_range(e, e->blocks[i], 0, e->blocks[i].n, L2L_F32, lr, beta1, beta2, eps_a, omb1, omb2, c1, c2);
  return L2L_OK;
}

int eps_adam_step_range(eps_store* e, int block, long long first_elem, long long count, int t, double lr_d, double beta1_d,
                        double beta2_d, double eps_a_d) {
  if (!e || block < 0 || block >= (int)e->blocks.size() || t < 1) return L2L_E_ARG;
  if (first_elem < 0 || count <= 0 || (size_t)(first_elem + count) > e->blocks[block].n) return L2L_E_ARG;
  const float lr = (float)lr_d, beta1 = (float)beta1_d, beta2 = (float)beta2_d, eps_a = (float)eps_a_d;
  const float omb1 = (float)(1.0 - beta1_d), omb2 = (float)(1.0 - beta2_d);
  const float c1 = (float)(1.0 / (1.0 - std::pow(beta1_d, t)));
  const float c2 = (float)(1.0 / (1.0 - std::pow(beta2_d, t)));
  adam_range(e, e->blocks[block], (size_t)first_elem, (size_t)count, L2L_F32, lr, beta1, beta2, eps_a, omb1, omb2, c1, c2);
  return L2L_OK;
}

int eps_adam_step_range16(eps_store* e, int block, long long first_elem, long long count, int t, double lr_d, double beta1_d,
                          double beta2_d, double eps_a_d, int grad_dtype) {
  if (!e || block < 0 || block >= (int)e->blocks.size() || t < 1 || (grad_dtype != L2L_BF16 && grad_dtype != L2L_FP16)) return L2L_E_ARG;
  const Block& b = e->blocks[block];
  if (!b.grad16) return L2L_E_STATE;
  if (first_elem < 0 || count <= 0 || (size_t)(first_elem + count) > b.n) return L2L_E_ARG;
  const float lr = (float)lr_d, beta1 = (float)beta1_d, beta2 = (float)beta2_d, eps_a = (float)eps_a_d;
  const float omb1 = (float)(1.0 - beta1_d), omb2 = (float)(1.0 - beta2_d);
  const float c1 = (float)(1.0 / (1.0 - std::pow(beta1_d, t)));
  const float c2 = (float)(1.0 / (1.0 - std::pow(beta2_d, t)));
  adam_range(e, b, (size_t)first_elem, (size_t)count, grad_dtype, lr, beta1, beta2, eps_a, omb1, omb2, c1, c2);
  return L2L_OK;
}

int eps_enable_grad16(eps_store* e) {
  if (!e) return L2L_E_ARG;
  for (Block& b : e->blocks) {
    if (b.grad16) continue;
    const size_t bytes = (b.n * 2 + 63) / 64 * 64;
    if (b.pinned) {   // as the block's other host-link buffers
      if (hipHostMalloc((void**)&b.grad16, bytes, hipHostMallocDefault) != hipSuccess) { b.grad16 = nullptr; return L2L_E_NOMEM; }
    } else {
      b.grad16 = (uint16_t*)aligned_alloc(64, bytes);
      if (!b.grad16) return L2L_E_NOMEM;
    }
    std::memset(b.grad16, 0, bytes);
    e->host_bytes += bytes;
  }
  return L2L_OK;
}

void* eps_grad16(eps_store* e, int i) { Block* b = blk(e, i); return b ? b->grad16 : nullptr; }

static void widen_range(const Block& b, size_t lo, size_t hi, int dtype) { widen_run(b.grad16 + lo, b.grad + lo, hi - lo, dtype); }

int eps_grad_widen_range(eps_store* e, int block, long long first_elem, long long count, int dtype) {
  if (!e || block < 0 || block >= (int)e->blocks.size() || (dtype != L2L_BF16 && dtype != L2L_FP16)) return L2L_E_ARG;
  const Block& b = e->blocks[block];
  if (!b.grad16) return L2L_E_STATE;
  if (first_elem < 0 || count <= 0 || (size_t)(first_elem + count) > b.n) return L2L_E_ARG;
  const size_t e0 = (size_t)first_elem;
  e->pool->run((size_t)count, [&](size_t lo, size_t hi) { widen_range(b, e0 + lo, e0 + hi, dtype); });
  return L2L_OK;
}

int eps_grad_widen(eps_store* e, int first, int last, int dtype) {
  if (!e || first < 0 || last >= (int)e->blocks.size() || first > last) return L2L_E_ARG;
  for (int i = first; i <= last; ++i) {
    const int rc = eps_grad_widen_range(e, i, 0, (long long)e->blocks[i].n, dtype);
    if (rc != L2L_OK) return rc;
  }
  return L2L_OK;
}

int eps_grad_unscale(eps_store* e, int first, int last, double inv_scale, int* nonfinite) {
  if (!e || first < 0 || last >= (int)e->blocks.size() || first > last || !std::isfinite(inv_scale)) return L2L_E_ARG;
  const float s = (float)inv_scale;
  std::atomic<int> bad{0};
  for (int i = first; i <= last; ++i) {
    const Block& b = e->blocks[i];
    float* __restrict g = b.grad;
    e->pool->run(b.n, [&](size_t lo, size_t hi) {
      float worst = 0.f;   // a NaN or inf anywhere turns this sum of |g| * 0 into NaN
      for (size_t k = lo; k < hi; ++k) {
        const float v = g[k] * s;
        g[k] = v;
        worst += v * 0.f;
      }
      if (!(worst == 0.f)) bad.store(1);
    });
  }
  if (nonfinite) *nonfinite = bad.load();
  return L2L_OK;
}

int eps_grad_unscale_range(eps_store* e, int block, long long first_elem, long long count, double inv_scale, int* nonfinite) {
  if (!e || block < 0 || block >= (int)e->blocks.size() || !std::isfinite(inv_scale)) return L2L_E_ARG;
  if (first_elem < 0 || count <= 0 || (size_t)(first_elem + count) > e->blocks[block].n) return L2L_E_ARG;
  const float s = (float)inv_scale;
  std::atomic<int> bad{0};
  float* __restrict g = e->blocks[block].grad + first_elem;
  e->pool->run((size_t)count, [&](size_t lo, size_t hi) {
    float worst = 0.f;   // as in eps_grad_unscale
    for (size_t k = lo; k < hi; ++k) {
      const float v = g[k] * s;
      g[k] = v;
      worst += v * 0.f;
    }
    if (!(worst == 0.f)) bad.store(1);
  });
  if (nonfinite) *nonfinite = bad.load();
  return L2L_OK;
}

int eps_lamb_step(eps_store* e, int first, int last, int t, double lr_d, double beta1_d, double beta2_d, double eps_a_d,
                  double weight_decay, int n_seg, const long long* seg_begin, const long long* seg_end,
                  const double* seg_decay) {
  if (!e || first < 0 || last >= (int)e->blocks.size() || first > last || t < 1) return L2L_E_ARG;
  if (n_seg < 0 || (n_seg > 0 && (!seg_begin || !seg_end))) return L2L_E_ARG;
  for (int i = first; i <= last; ++i) {
    long long prev = 0;
    for (int s = 0; s < n_seg; ++s) {
      if (seg_begin[s] < prev || seg_end[s] < seg_begin[s] || (size_t)seg_end[s] > e->blocks[i].n) return L2L_E_ARG;
      prev = seg_end[s];
    }
  }
  const float beta1 = (float)beta1_d, beta2 = (float)beta2_d, eps_a = (float)eps_a_d;
  const float omb1 = (float)(1.0 - beta1_d), omb2 = (float)(1.0 - beta2_d);
  const float c1 = (float)(1.0 / (1.0 - std::pow(beta1_d, t)));
  const float c2 = (float)(1.0 / (1.0 - std::pow(beta2_d, t)));
  std::mutex sum_mu;
  for (int i = first; i <= last; ++i) {
    const Block& b = e->blocks[i];
    for (int s = 0; s < n_seg; ++s) {
      const size_t s0 = (size_t)seg_begin[s], len = (size_t)(seg_end[s] - seg_begin[s]);
      if (len == 0) continue;
      const float wd = (float)(weight_decay * (seg_decay ? seg_decay[s] : 1.0));
      float* __restrict w = b.w + s0;
      float* __restrict m = b.m + s0;
      float* __restrict v = b.v + s0;
      const float* __restrict g = b.grad + s0;
      // pass 1: moments, and the two norms of the tensor (u is formed again in pass 2: w has not moved yet)
      double wn2 = 0.0, un2 = 0.0;
      e->pool->run(len, [&](size_t lo, size_t hi) {
        double a = 0.0, c = 0.0;
        // the squares are summed in fp32 over runs of 256 elements (a loop the compiler vectorises) and the runs in double
        for (size_t k0 = lo; k0 < hi; k0 += 256) {
          const size_t k1 = std::min(hi, k0 + 256);
          float fa = 0.f, fc = 0.f;
#pragma omp simd reduction(+ : fa, fc)
          for (size_t k = k0; k < k1; ++k) {
            const float gk = g[k];
            const float mk = beta1 * m[k] + omb1 * gk;
            const float vk = beta2 * v[k] + omb2 * gk * gk;
            m[k] = mk;
            v[k] = vk;
            const float u = (mk * c1) / (std::sqrt(vk * c2) + eps_a) + wd * w[k];
            fa += w[k] * w[k];
            fc += u * u;
          }
          a += fa;
          c += fc;
        }
        std::lock_guard<std::mutex> l(sum_mu);
        wn2 += a;
        un2 += c;
      });
      const double trust = (wn2 > 0.0 && un2 > 0.0) ? std::sqrt(wn2) / std::sqrt(un2) : 1.0;
      const float step = (float)(lr_d * trust);
      e->pool->run(len, [&](size_t lo, size_t hi) {
        for (size_t k = lo; k < hi; ++k) {
          const float u = (m[k] * c1) / (std::sqrt(v[k] * c2) + eps_a) + wd * w[k];
          w[k] -= step * u;
        }
        ship_range(e, b, s0 + lo, s0 + hi);
      });
    }
  }
  return L2L_OK;
}

}  // extern "C"
