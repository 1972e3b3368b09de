// small standalone kernels: append, literal and summary masks, threshold, fill.
// Part of one translation unit: included by corm_kernels.hip, in this order, after <hip/hip_runtime.h> and corm.h.
#ifndef CORM_STANDALONE_HPP
#define CORM_STANDALONE_HPP

namespace {

// ---------------------------------------------------------------- standalone kernels

__global__ __launch_bounds__(64) void corm_append_kernel(char* K, char* V, int32_t* lens, int32_t* pos,
                                                         int32_t* last_hit, const char* k_new, const char* v_new,
                                                         const int32_t* t, int32_t* status, int Hkv, int Lcap,
                                                         int rowb) {
  const int unit = blockIdx.x;
  const int b = unit / Hkv;
  const int L0 = lens[unit];
  if (L0 < 0 || L0 >= Lcap) {
    if (threadIdx.x == 0 && status) atomicOr(status, L0 == Lcap ? CORM_DEV_UNIT_FULL : CORM_DEV_BAD_LENS);
    return;
  }
  const int lane = threadIdx.x;
  if (lane * 16 < rowb) {
    size_t dst = ((size_t)unit * Lcap + L0) * rowb + (size_t)lane * 16;
    size_t src = (size_t)unit * rowb + (size_t)lane * 16;
    *reinterpret_cast<uint4*>(K + dst) = *reinterpret_cast<const uint4*>(k_new + src);
    *reinterpret_cast<uint4*>(V + dst) = *reinterpret_cast<const uint4*>(v_new + src);
  }
  if (lane == 0) {
    pos[(size_t)unit * Lcap + L0] = t[b] - 1;
    last_hit[(size_t)unit * Lcap + L0] = 0;
    lens[unit] = L0 + 1;
  }
}

// literal windowed OR over the ring (Def. 4.1 + recent r + group rule)
__global__ __launch_bounds__(WG) void corm_evict_mask_kernel(const void* ring, int ring_mode, const int32_t* lens,
                                                             const int32_t* pos, const int32_t* t,
                                                             const int32_t* t_first, uint8_t* keep, int Hq, int Hkv,
                                                             int Lcap, int Tcap, int w, int r, float c) {
  const int unit = blockIdx.y;
  const int b = unit / Hkv, hkv = unit - b * Hkv;
  const int G = Hq / Hkv;
  int L = lens[unit];
  L = L < 0 ? 0 : (L > Lcap ? Lcap : L);
  const int i = blockIdx.x * WG + threadIdx.x;
  if (i >= L) return;
  const int tcur = t[b];
  const int tf = t_first[b];
  bool k = i >= L - r;
  const bool full = tcur - tf + 1 >= w;
  if (!full) k = true;
  const int pi = pos[(size_t)unit * Lcap + i];
  if (!k && pi >= 0 && pi < Tcap) {
    const int lo = max(max(tf, tcur - w + 1), 1);
    for (int tau = tcur; tau >= lo && !k; --tau) {
      if (pi > tau - 1) break;  // the key did not exist at step tau (nor earlier): minor there
      const float thr = importance_threshold(c, tau);
      const int slot = (tau - 1) % w;
      for (int g = 0; g < G; ++g) {
        const size_t row = (size_t)(b * Hq + hkv * G + g) * w + slot;
        if (ring_mode == CORM_BIT) {   // the recorded boolean itself
          const uint32_t word = reinterpret_cast<const uint32_t*>(ring)[row * ((Tcap + 31) >> 5) + (size_t)(pi >> 5)];
          k |= ((word >> (pi & 31)) & 1u) != 0;
        } else {
          const size_t ri = row * Tcap + (size_t)pi;
          const float v = ring_mode == CORM_BF16
                              ? __uint_as_float((uint32_t) reinterpret_cast<const uint16_t*>(ring)[ri] << 16)
                              : reinterpret_cast<const float*>(ring)[ri];
          k |= (v >= thr);
        }
      }
    }
  }
  keep[(size_t)unit * Lcap + i] = k ? 1 : 0;
}

__global__ __launch_bounds__(WG) void corm_evict_mask_summary_kernel(const int32_t* last_hit, const int32_t* lens,
                                                                     const int32_t* t, const int32_t* t_first,
                                                                     uint8_t* keep, int Hkv, int Lcap, int w, int r) {
  const int unit = blockIdx.y;
  const int b = unit / Hkv;
  int L = lens[unit];
  L = L < 0 ? 0 : (L > Lcap ? Lcap : L);
  const int i = blockIdx.x * WG + threadIdx.x;
  if (i >= L) return;
  const int tcur = t[b];
  const bool full = tcur - t_first[b] + 1 >= w;
  const bool k = !full || last_hit[(size_t)unit * Lcap + i] > tcur - w || i >= L - r;
  keep[(size_t)unit * Lcap + i] = k ? 1 : 0;
}

// Diagnostic (Section 3, attention sparsity): per query head, the share of the unit's live keys whose
// recorded score of step t reaches c/t.  One workgroup per head.
__global__ __launch_bounds__(WG) void corm_row_density_kernel(const void* ring, int ring_mode, const int32_t* lens,
                                                              const int32_t* pos, const int32_t* t, float* density,
                                                              int Hq, int Hkv, int Lcap, int Tcap, int w, float c) {
  __shared__ int sh_cnt[WAVES];
  const int head = blockIdx.x;
  const int b = head / Hq, hq = head - b * Hq;
  const int unit = b * Hkv + hq / (Hq / Hkv);
  int L = lens[unit];
  L = L < 0 ? 0 : (L > Lcap ? Lcap : L);
  const int tcur = t[b];
  const bool step_ok = tcur >= 1 && tcur <= Tcap;
  const float thr = importance_threshold(c, step_ok ? tcur : 1);
  const size_t row = (size_t)head * w + (size_t)(step_ok ? (tcur - 1) % w : 0);
  int cnt = 0;
  for (int i0 = 0; i0 < L; i0 += WG) {
    const int i = i0 + (int)threadIdx.x;
    bool hit = false;
    if (i < L && step_ok) {
      const int pi = pos[(size_t)unit * Lcap + i];
      if (pi >= 0 && pi < Tcap && pi <= tcur - 1) {
        if (ring_mode == CORM_BIT) {
          hit = ((reinterpret_cast<const uint32_t*>(ring)[row * ((Tcap + 31) >> 5) + (size_t)(pi >> 5)] >> (pi & 31)) & 1u) != 0;
        } else {
          const size_t ri = row * Tcap + (size_t)pi;
          const float v = ring_mode == CORM_BF16
                              ? __uint_as_float((uint32_t) reinterpret_cast<const uint16_t*>(ring)[ri] << 16)
                              : reinterpret_cast<const float*>(ring)[ri];
          hit = v >= thr;
        }
      }
    }
    cnt += __popcll(__ballot(hit));
  }
  if ((threadIdx.x & 63) == 0) sh_cnt[threadIdx.x >> 6] = cnt;
  __syncthreads();
  if (threadIdx.x == 0) {
    int tot = 0;
#pragma unroll
    for (int i = 0; i < WAVES; ++i) tot += sh_cnt[i];
    density[head] = L > 0 ? (float)tot / (float)L : 0.f;
  }
}

__global__ void corm_threshold_kernel(float c, const int32_t* t, int n, float* thr) {
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) thr[i] = importance_threshold(c, t[i]);
}

__global__ void corm_fill_i32_kernel(int32_t* p, size_t n, int32_t v) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = v;
}

}  // namespace

#endif  // CORM_STANDALONE_HPP
