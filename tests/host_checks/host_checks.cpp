// Host-side checks of the C ABI under AddressSanitizer and UndefinedBehaviorSanitizer (CPU only, no GPU in
// the process): the library's translation unit is compiled into this program with its HOST code
// instrumented, and the code that runs before any launch -- descriptor validation, workspace layout
// arithmetic, pointer and option checks, path selection, the static-scratch limit -- is driven with shapes
// at and beyond the interface limits, from two threads at once.  Every call here must be refused (or
// answered) on the host; nothing reaches a device.
#include <cstdint>
#include <cstdio>
#include <cstring>
#include <thread>
#include <vector>

#include "corm.h"

static int failures = 0;
#define EXPECT(cond)                                                  \
  do {                                                                \
    if (!(cond)) {                                                    \
      std::printf("FAIL %s:%d: %s\n", __FILE__, __LINE__, #cond);     \
      ++failures;                                                     \
    }                                                                 \
  } while (0)

static corm_desc desc(int B, int Hq, int Hkv, int d, int Lcap, int Tcap, int w, int r, int kv, int sc) {
  corm_desc x;
  std::memset(&x, 0, sizeof x);
  x.B = B; x.Hq = Hq; x.Hkv = Hkv; x.d = d; x.Lcap = Lcap; x.Tcap = Tcap; x.w = w; x.r = r;
  x.kv_dtype = kv; x.score_dtype = sc; x.thr_scale = 1.0f; x.sm_scale = 0.0f;
  return x;
}

static void limits() {
  size_t n = 0;
  // the largest unit: byte offsets inside a unit are 32-bit, so Lcap * 512 must stay below 2^31
  corm_desc longest = desc(1, 1, 1, 128, 4194303, 4194303, 4, 4, CORM_F32, CORM_F32);
  EXPECT(corm_workspace_bytes(&longest, &n) == CORM_OK && n > (size_t)4194303 * 512 * 2);
  longest.Lcap = 4194304;
  EXPECT(corm_workspace_bytes(&longest, &n) == CORM_EUNSUPPORTED);
  longest.Lcap = 2147483647;
  EXPECT(corm_workspace_bytes(&longest, &n) == CORM_EUNSUPPORTED);
  // the most units: the launch grid has 65535 rows
  corm_desc most = desc(4095, 16, 16, 64, 64, 64, 8, 4, CORM_F32, CORM_F32);
  EXPECT(corm_workspace_bytes(&most, &n) == CORM_OK && n > 0);
  most.B = 4096;
  EXPECT(corm_workspace_bytes(&most, &n) == CORM_EUNSUPPORTED);
  // sizes whose products overflow 32 bits must be computed in 64 bits or refused: B * Hq beyond 2^30
  corm_desc huge = desc(2147483647, 8, 8, 128, 1024, 1024, 8, 8, CORM_BF16, CORM_BF16);
  EXPECT(corm_workspace_bytes(&huge, &n) == CORM_EINVAL);
  huge = desc(65535, 32768, 1, 128, 1024, 1024, 8, 8, CORM_BF16, CORM_BF16);   // group of 32768
  EXPECT(corm_workspace_bytes(&huge, &n) != CORM_OK);
  // the full-size workloads: the layout must be monotone and 256-byte aligned in total
  const int shapes[5][6] = {{1, 4, 4, 64, 576, 32}, {1, 32, 32, 128, 4352, 1024}, {16, 32, 32, 128, 4608, 1024},
                            {4, 32, 32, 128, 33024, 2048}, {16, 32, 8, 128, 8704, 1024}};
  size_t prev = 0;
  for (int i = 0; i < 5; ++i) {
    corm_desc s = desc(shapes[i][0], shapes[i][1], shapes[i][2], shapes[i][3], shapes[i][4], shapes[i][4],
                       shapes[i][5], shapes[i][5], i == 0 ? CORM_F32 : CORM_BF16, i == 0 ? CORM_F32 : CORM_BF16);
    EXPECT(corm_workspace_bytes(&s, &n) == CORM_OK && n % 256 == 0 && n > 0);
    EXPECT(corm_selected_path(&s, nullptr) == (i == 2 ? 2 : 1));   // 256 compute units are assumed without a device
    corm_desc bits = s;
    bits.score_dtype = CORM_BIT;
    size_t nb = 0;
    EXPECT(corm_workspace_bytes(&bits, &nb) == CORM_OK && nb == n);   // the workspace does not depend on the ring
    prev = n;
  }
  (void)prev;
  EXPECT(corm_workspace_bytes(nullptr, &n) == CORM_EINVAL);
  EXPECT(corm_workspace_bytes(&most, nullptr) != CORM_OK);
}

static void arguments() {
  corm_desc d = desc(2, 8, 2, 128, 1024, 1024, 16, 16, CORM_BF16, CORM_BF16);
  alignas(256) static unsigned char fake[4096];   // never dereferenced: every call below fails validation first
  void* a = fake;
  int32_t* i = reinterpret_cast<int32_t*>(fake);
  float* f = reinterpret_cast<float*>(fake);
  const size_t big = (size_t)1 << 40;
  EXPECT(corm_decode_step(&d, nullptr, a, a, a, a, i, i, i, i, i, a, f, nullptr, nullptr, a, big, nullptr, nullptr, nullptr) == CORM_EINVAL);
  EXPECT(corm_decode_step(&d, a, a, a, fake + 8, a, i, i, i, i, i, a, f, nullptr, nullptr, a, big, nullptr, nullptr, nullptr) == CORM_EINVAL);
  EXPECT(corm_decode_step(&d, a, a, a, a, a, i, i, i, i, i, a, f, nullptr, nullptr, a, 64, nullptr, nullptr, nullptr) == CORM_ECAPACITY);
  EXPECT(corm_decode_step(&d, a, a, a, a, a, i, i, i, i, i, a, f, nullptr, nullptr, fake + 16, big, nullptr, nullptr, nullptr) == CORM_EINVAL);
  corm_launch_opts bad_path = {4, 0, nullptr, nullptr}, one_event = {0, 0, a, nullptr};
  EXPECT(corm_decode_step(&d, a, a, a, a, a, i, i, i, i, i, a, f, nullptr, nullptr, a, big, nullptr, &bad_path, nullptr) == CORM_EINVAL);
  EXPECT(corm_decode_attend(&d, a, a, a, i, i, i, a, i, f, a, big, nullptr, &one_event, nullptr) == CORM_EINVAL);
  EXPECT(corm_selected_path(&d, &bad_path) == CORM_EINVAL);
  EXPECT(corm_decode_step_lazy(&d, a, a, a, a, a, i, nullptr, i, i, i, i, a, f, nullptr, nullptr, 1, 4, a, big, nullptr, nullptr, nullptr) == CORM_EINVAL);
  EXPECT(corm_decode_step_lazy(&d, a, a, a, a, a, i, reinterpret_cast<uint64_t*>(fake), i, i, i, i, a, f, nullptr, nullptr, 5, 4, a, big, nullptr, nullptr, nullptr) == CORM_EINVAL);
  EXPECT(corm_prefill_seed(&d, a, 0, a, a, i, i, i, i, i, a, nullptr, nullptr, a, big, nullptr, nullptr) == CORM_EINVAL);
  EXPECT(corm_prefill_seed(&d, a, 17, a, a, i, i, i, i, i, a, nullptr, nullptr, a, big, nullptr, nullptr) == CORM_EINVAL);
  EXPECT(corm_compact(&d, a, a, i, i, i, nullptr, nullptr, a, big, nullptr) == CORM_EINVAL);
  EXPECT(corm_evict_mask(&d, nullptr, i, i, i, i, fake, nullptr) == CORM_EINVAL);
  EXPECT(corm_threshold(-1.0f, i, 4, f, nullptr) == CORM_EINVAL);
  EXPECT(corm_threshold(1.0f, i, 0, f, nullptr) == CORM_OK);   // nothing to do: no launch
  // the static scratch: a shape beyond the array is refused before any device call
  corm_desc wide = desc(16, 32, 32, 128, 32768, 32768, 16, 16, CORM_BF16, CORM_BF16);
  EXPECT(corm_decode_attend_static(&wide, a, a, a, i, i, i, a, i, f, nullptr, nullptr, nullptr) == CORM_ECAPACITY);
  EXPECT(corm_decode_attend_static(&d, a, a, a, i, i, i, a, nullptr, f, nullptr, nullptr, nullptr) == CORM_EINVAL);
  for (int s = 1; s >= -6; --s) EXPECT(corm_strerror(s) != nullptr && std::strlen(corm_strerror(s)) > 0);
  EXPECT(corm_version() >= 100);
}

int main() {
  limits();
  arguments();
  // the same checks from two threads at once: the library keeps no mutable state of its own
  std::vector<std::thread> th;
  for (int k = 0; k < 2; ++k)
    th.emplace_back([] {
      for (int rep = 0; rep < 200; ++rep) {
        limits();
        arguments();
      }
    });
  for (auto& t : th) t.join();
  if (failures) {
    std::printf("host checks: %d failure(s)\n", failures);
    return 1;
  }
  std::printf("host checks ok\n");
  return 0;
}
