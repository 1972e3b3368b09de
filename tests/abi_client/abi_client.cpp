// A client of the C ABI with no Python and no torch in the process: loads libcorm.so with dlopen, takes
// device memory from the HIP runtime, drives corm_decode_step for a few dozen steps and checks the results
// against closed forms worked out on the host in fp64.  TEST CODE: built by build(), run by the GPU tests.
//
//   c = 0     nothing is ever evicted: out equals full softmax attention over every key so far, lens = t.
//   c = 1e9   nothing is ever important: once w queries are recorded the cache is exactly the last r keys,
//             and out of a step equals attention over the r + 1 keys that were live when it ran.
//
// usage: abi_client /path/to/libcorm.so        exit status 0 = every check passed
#include <hip/hip_runtime.h>
#include <dlfcn.h>

#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "corm.h"

#define HIP_OK(x)                                                                      \
  do {                                                                                 \
    hipError_t e_ = (x);                                                               \
    if (e_ != hipSuccess) {                                                            \
      std::printf("HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__);      \
      std::exit(2);                                                                    \
    }                                                                                  \
  } while (0)

namespace {

using workspace_bytes_fn = int (*)(const corm_desc*, size_t*);
using workspace_init_fn = int (*)(const corm_desc*, void*, size_t, void*);
using decode_step_fn = int (*)(const corm_desc*, const void*, const void*, const void*, void*, void*, int32_t*,
                               int32_t*, int32_t*, const int32_t*, const int32_t*, void*, float*, uint8_t*,
                               int32_t*, void*, size_t, int32_t*, const corm_launch_opts*, void*);
using strerror_fn = const char* (*)(int);

// deterministic inputs: a small linear congruential generator mapped to (-1, 1)
struct Lcg {
  uint64_t s;
  float next() {
    s = s * 6364136223846793005ull + 1442695040888963407ull;
    return (float)((double)(s >> 11) / (double)(1ull << 53) * 2.0 - 1.0);
  }
};

template <typename T>
T* dev_alloc(size_t n) {
  T* p = nullptr;
  HIP_OK(hipMalloc(&p, n * sizeof(T)));
  HIP_OK(hipMemset(p, 0, n * sizeof(T)));
  return p;
}

int failures = 0;
void expect(bool ok, const char* what, int step, double got, double want) {
  if (!ok) {
    std::printf("FAIL %s at step %d: got %.9g, want %.9g\n", what, step, got, want);
    ++failures;
  }
}

// softmax attention of one query over keys [lo, hi) of the history, fp64
void attention(const std::vector<float>& q, const std::vector<float>& Kh, const std::vector<float>& Vh, int lo, int hi,
               int d, std::vector<double>& out) {
  std::vector<double> s(hi - lo);
  double m = -1e300;
  for (int i = lo; i < hi; ++i) {
    double acc = 0;
    for (int c = 0; c < d; ++c) acc += (double)q[c] * (double)Kh[(size_t)i * d + c];
    s[i - lo] = acc / std::sqrt((double)d);
    m = std::fmax(m, s[i - lo]);
  }
  double z = 0;
  for (double& v : s) {
    v = std::exp(v - m);
    z += v;
  }
  out.assign(d, 0.0);
  for (int i = lo; i < hi; ++i)
    for (int c = 0; c < d; ++c) out[c] += s[i - lo] / z * (double)Vh[(size_t)i * d + c];
}

int run(void* lib, float c, int P, int steps) {
  auto ws_bytes = (workspace_bytes_fn)dlsym(lib, "corm_workspace_bytes");
  auto ws_init = (workspace_init_fn)dlsym(lib, "corm_workspace_init");
  auto step_fn = (decode_step_fn)dlsym(lib, "corm_decode_step");
  auto err_str = (strerror_fn)dlsym(lib, "corm_strerror");
  if (!ws_bytes || !ws_init || !step_fn || !err_str) {
    std::printf("FAIL: symbol missing\n");
    return 1;
  }
  const int B = 2, Hq = 2, Hkv = 2, d = 64, w = 4, r = 3;
  const int Lcap = P + steps, Tcap = P + steps;
  corm_desc desc{B, Hq, Hkv, d, Lcap, Tcap, w, r, CORM_F32, CORM_F32, c, 0.0f};
  size_t wsb = 0;
  int rc = ws_bytes(&desc, &wsb);
  if (rc != CORM_OK) {
    std::printf("FAIL corm_workspace_bytes: %s\n", err_str(rc));
    return 1;
  }
  const int units = B * Hkv;
  // history of every unit on the host (unit u = b * Hkv + h; one query head per KV head here)
  Lcg rng{12345u + (uint64_t)(c > 1.f)};
  std::vector<std::vector<float>> Kh(units), Vh(units);
  std::vector<float> hK((size_t)units * Lcap * d, 0.f), hV((size_t)units * Lcap * d, 0.f);
  std::vector<int32_t> hlens(units, P), hpos((size_t)units * Lcap, 0);
  for (int u = 0; u < units; ++u) {
    for (int i = 0; i < P; ++i) {
      for (int cc = 0; cc < d; ++cc) {
        const float kx = rng.next() * 1.5f, vx = rng.next();
        Kh[u].push_back(kx);
        Vh[u].push_back(vx);
        hK[((size_t)u * Lcap + i) * d + cc] = kx;
        hV[((size_t)u * Lcap + i) * d + cc] = vx;
      }
      hpos[(size_t)u * Lcap + i] = i;
    }
  }
  float* K = dev_alloc<float>(hK.size());
  float* V = dev_alloc<float>(hV.size());
  int32_t* lens = dev_alloc<int32_t>(units);
  int32_t* pos = dev_alloc<int32_t>((size_t)units * Lcap);
  int32_t* last_hit = dev_alloc<int32_t>((size_t)units * Lcap);
  float* ring = dev_alloc<float>((size_t)B * Hq * w * Tcap);
  float* out = dev_alloc<float>((size_t)B * Hq * d);
  float* q = dev_alloc<float>((size_t)B * Hq * d);
  float* kn = dev_alloc<float>((size_t)units * d);
  float* vn = dev_alloc<float>((size_t)units * d);
  int32_t* t = dev_alloc<int32_t>(B);
  int32_t* tf = dev_alloc<int32_t>(B);
  int32_t* status = dev_alloc<int32_t>(1);
  void* ws = nullptr;
  HIP_OK(hipMalloc(&ws, wsb));
  HIP_OK(hipMemcpy(K, hK.data(), hK.size() * 4, hipMemcpyHostToDevice));
  HIP_OK(hipMemcpy(V, hV.data(), hV.size() * 4, hipMemcpyHostToDevice));
  HIP_OK(hipMemcpy(lens, hlens.data(), units * 4, hipMemcpyHostToDevice));
  HIP_OK(hipMemcpy(pos, hpos.data(), hpos.size() * 4, hipMemcpyHostToDevice));
  rc = ws_init(&desc, ws, wsb, nullptr);
  if (rc != CORM_OK) {
    std::printf("FAIL corm_workspace_init: %s\n", err_str(rc));
    return 1;
  }
  std::vector<int32_t> ht(B), htf(B, P + 1);   // the first recorded query is step P + 1
  HIP_OK(hipMemcpy(tf, htf.data(), B * 4, hipMemcpyHostToDevice));
  std::vector<float> hq((size_t)B * Hq * d), hkn((size_t)units * d), hvn((size_t)units * d), hout((size_t)B * Hq * d);
  std::vector<double> ref;

  for (int sidx = 0; sidx < steps; ++sidx) {
    const int tcur = P + sidx + 1;   // number of tokens including the current one
    for (auto& x : hq) x = rng.next() * 2.0f;
    for (int u = 0; u < units; ++u)
      for (int cc = 0; cc < d; ++cc) {
        hkn[(size_t)u * d + cc] = rng.next() * 1.5f;
        hvn[(size_t)u * d + cc] = rng.next();
        Kh[u].push_back(hkn[(size_t)u * d + cc]);
        Vh[u].push_back(hvn[(size_t)u * d + cc]);
      }
    for (int b = 0; b < B; ++b) ht[b] = tcur;
    HIP_OK(hipMemcpy(q, hq.data(), hq.size() * 4, hipMemcpyHostToDevice));
    HIP_OK(hipMemcpy(kn, hkn.data(), hkn.size() * 4, hipMemcpyHostToDevice));
    HIP_OK(hipMemcpy(vn, hvn.data(), hvn.size() * 4, hipMemcpyHostToDevice));
    HIP_OK(hipMemcpy(t, ht.data(), B * 4, hipMemcpyHostToDevice));
    rc = step_fn(&desc, q, kn, vn, K, V, lens, pos, last_hit, t, tf, ring, out, nullptr, nullptr, ws, wsb, status,
                 nullptr, nullptr);
    if (rc != CORM_OK) {
      std::printf("FAIL corm_decode_step: %s\n", err_str(rc));
      return 1;
    }
    HIP_OK(hipDeviceSynchronize());
    HIP_OK(hipMemcpy(hout.data(), out, hout.size() * 4, hipMemcpyDeviceToHost));
    HIP_OK(hipMemcpy(hlens.data(), lens, units * 4, hipMemcpyDeviceToHost));
    int32_t hstatus = 0;
    HIP_OK(hipMemcpy(&hstatus, status, 4, hipMemcpyDeviceToHost));
    expect(hstatus == 0, "device status word", sidx, hstatus, 0);
    // the keys that were live when this step attended, and how many remain after it
    const bool sliding = c > 1.f;
    const bool full_before = sidx >= w;        // the window was already full at the previous step
    const bool full_now = sidx + 1 >= w;
    const int lo = (sliding && full_before) ? tcur - 1 - r : 0;
    const int want_len = (sliding && full_now) ? r : tcur;
    for (int u = 0; u < units; ++u) {
      expect(hlens[u] == want_len, "lens", sidx, hlens[u], want_len);
      std::vector<float> qu(hq.begin() + (size_t)u * d, hq.begin() + (size_t)(u + 1) * d);   // Hq == Hkv: head u
      attention(qu, Kh[u], Vh[u], lo, tcur, d, ref);
      double worst = 0, scale = 1e-30;
      for (int cc = 0; cc < d; ++cc) {
        worst = std::fmax(worst, std::fabs((double)hout[(size_t)u * d + cc] - ref[cc]));
        scale = std::fmax(scale, std::fabs(ref[cc]));
      }
      expect(worst / scale <= 1e-5, "out (max error relative to the row's largest component)", sidx, worst / scale, 0);
    }
  }
  // the recorded row of the last step: the normalized scores of the keys it saw sum to one (columns of keys
  // evicted earlier keep what an older query wrote there; nothing reads them)
  std::vector<float> hring((size_t)B * Hq * w * Tcap);
  HIP_OK(hipMemcpy(hring.data(), ring, hring.size() * 4, hipMemcpyDeviceToHost));
  const int tlast = P + steps;
  const int lo_last = (c > 1.f && steps - 1 >= w) ? tlast - 1 - r : 0;
  for (int head = 0; head < B * Hq; ++head) {
    const float* row = &hring[((size_t)head * w + (size_t)((tlast - 1) % w)) * Tcap];
    double sum = 0;
    for (int i = lo_last; i < tlast; ++i) sum += row[i];
    expect(std::fabs(sum - 1.0) < 1e-5, "recorded row sums to one", steps - 1, sum, 1.0);
  }
  for (void* p : {(void*)K, (void*)V, (void*)lens, (void*)pos, (void*)last_hit, (void*)ring, (void*)out, (void*)q,
                  (void*)kn, (void*)vn, (void*)t, (void*)tf, (void*)status, ws})
    HIP_OK(hipFree(p));
  return failures;
}

}  // namespace

int main(int argc, char** argv) {
  if (argc < 2) {
    std::printf("usage: %s /path/to/libcorm.so\n", argv[0]);
    return 2;
  }
  void* lib = dlopen(argv[1], RTLD_NOW | RTLD_LOCAL);
  if (!lib) {
    std::printf("FAIL dlopen: %s\n", dlerror());
    return 2;
  }
  auto version = (int (*)(void))dlsym(lib, "corm_version");
  if (!version || version() < 100) {
    std::printf("FAIL corm_version\n");
    return 1;
  }
  int bad = run(lib, 0.0f, 37, 24);      // nothing evicted
  bad += run(lib, 1e9f, 37, 24);         // sliding window of r keys
  std::printf(bad ? "abi_client: %d checks FAILED\n" : "abi_client: all checks passed\n", bad);
  return bad ? 1 : 0;
}
