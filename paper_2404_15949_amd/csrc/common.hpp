// constants, the kernel parameter block and small device helpers shared by every kernel.
// Part of one translation unit: included by corm_kernels.hip, in this order, after <hip/hip_runtime.h> and corm.h.
#ifndef CORM_COMMON_HPP
#define CORM_COMMON_HPP

namespace {

constexpr int WG = 256;          // threads per workgroup
constexpr int WAVES = WG / 64;   // waves per workgroup
constexpr int CHUNK = 512;       // keys per split
constexpr int UNROLL = 4;        // 16-byte K loads (and V loads) per lane and pipeline stage
constexpr int MAX_PARTS_PER_CHUNK = 4;   // split path: a chunk may be shared by up to 4 attend workgroups
constexpr float LOG2E = 1.4426950408889634f;

struct Params {
  const void* q;
  const void* k_new;
  const void* v_new;
  void* K;
  void* V;
  int32_t* lens;
  int32_t* pos;
  int32_t* last_hit;
  const int32_t* t;
  const int32_t* t_first;
  void* ring;
  float* out;
  uint8_t* keep;       // optional: the caller's keep flags [B,Hkv,Lcap], one byte per slot
  unsigned long long* keepbits;  // keep flags as wave ballots [B*Hkv, ceil(Lcap/64)] (workspace)
  int32_t* kept_idx;   // optional
  int32_t* counts;     // survivors per (unit, split)
  int32_t* unit_dirty; // [units] words of the workspace: a step launch sets a unit's word to the call's dirty_tag
                       // if the unit has to be compacted; while it differs from the tag the compaction
                       // launches know, from one load, that only the unit's bookkeeping is left to do.  A stale
                       // or foreign value that happens to equal the tag only sends them down the ordinary path.
  float* partials;     // [B*Hq, nsplit, d+2]
  float* logits;       // [B*Hq, Lcap], log2 domain
  int32_t* status;
  int32_t B, Hq, Hkv, Lcap, Tcap, w, r, nsplit;
  float thr_scale, scale_log2;
  int32_t do_append, do_evict, ring_bf16;
  int32_t ring_bits;    // the ring holds the boolean message: one bit per (row, position), 32 positions per word
  int32_t ring_words;   // words per ring row in that case: ceil(Tcap / 32)
  int32_t part_keys;    // split path: keys per attend workgroup (CHUNK, or a fraction of it when the launch has few units)
  int32_t npart;        // partials per head in the workspace: nsplit * (CHUNK / smallest part)
  int32_t kb_stride;    // 64-bit words per unit in keepbits
  int32_t lazy;         // lazy mode: keepbits are the caller's persistent live masks; dead slots are skipped
  int32_t dead_num, dead_den;   // lazy mode: the compaction policy (a unit is compacted once dead_num/dead_den of its slots are dead)
};

// ---------------------------------------------------------------- small device helpers

__device__ __forceinline__ float bf16_lo(uint32_t x) { return __uint_as_float(x << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t x) { return __uint_as_float(x & 0xffff0000u); }

// fp32 -> bf16 bits, round to nearest even (NaN stays NaN)
__device__ __forceinline__ uint16_t f32_to_bf16_rne(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40u);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}

typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));

__device__ __forceinline__ float dot2_bf16(uint32_t a, uint32_t b, float c) {
  return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, a), __builtin_bit_cast(bf16x2_t, b), c,
                                         false);
}

template <int CTRL>
__device__ __forceinline__ float dpp_f32(float v) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xf, 0xf, true));
}

// sum over the LPR lanes that share a row; every lane of the group gets the total
template <int LPR>
__device__ __forceinline__ float row_allreduce_sum(float v) {
  v += dpp_f32<0xB1>(v);                    // quad_perm [1,0,3,2]
  v += dpp_f32<0x4E>(v);                    // quad_perm [2,3,0,1]
  v += dpp_f32<0x141>(v);                   // row_half_mirror: lanes 0..7 of each 16 are now equal
  if (LPR >= 16) v += dpp_f32<0x140>(v);    // row_mirror
  if (LPR >= 32) v += __shfl_xor(v, 16);
  return v;
}

// All-reduce over the four 16-lane rows of a wave (lanes l, l^16, l^32, l^48) on the vector ALU:
// v_permlane16_swap exchanges the odd rows of its first operand with the even rows of its second,
// v_permlane32_swap the upper half of the first with the lower half of the second; applied to two copies
// of a value, the two results hold in every lane the value of the lane itself and of its partner.
__device__ __forceinline__ float rows_allreduce_max(float v) {
  const unsigned u = __float_as_uint(v);
  const auto a = __builtin_amdgcn_permlane16_swap(u, u, false, false);
  const float m = fmaxf(__uint_as_float(a[0]), __uint_as_float(a[1]));
  const unsigned w = __float_as_uint(m);
  const auto b = __builtin_amdgcn_permlane32_swap(w, w, false, false);
  return fmaxf(__uint_as_float(b[0]), __uint_as_float(b[1]));
}
__device__ __forceinline__ float rows_allreduce_sum(float v) {
  const unsigned u = __float_as_uint(v);
  const auto a = __builtin_amdgcn_permlane16_swap(u, u, false, false);
  const float m = __uint_as_float(a[0]) + __uint_as_float(a[1]);
  const unsigned w = __float_as_uint(m);
  const auto b = __builtin_amdgcn_permlane32_swap(w, w, false, false);
  return __uint_as_float(b[0]) + __uint_as_float(b[1]);
}

__device__ __forceinline__ uint32_t rows_allreduce_or(uint32_t u) {
  const auto a = __builtin_amdgcn_permlane16_swap(u, u, false, false);
  const uint32_t w = a[0] | a[1];
  const auto b = __builtin_amdgcn_permlane32_swap(w, w, false, false);
  return b[0] | b[1];
}

struct F32 {
  static constexpr int EPL = 4;  // elements per 16-byte lane slice
  static constexpr int ESZ = 4;
  __device__ static __forceinline__ float dot(const uint4& k, const uint4& q) {
    float s = __uint_as_float(k.x) * __uint_as_float(q.x);
    s = fmaf(__uint_as_float(k.y), __uint_as_float(q.y), s);
    s = fmaf(__uint_as_float(k.z), __uint_as_float(q.z), s);
    s = fmaf(__uint_as_float(k.w), __uint_as_float(q.w), s);
    return s;
  }
  __device__ static __forceinline__ void axpy(float* acc, float p, const uint4& v) {
    acc[0] = fmaf(p, __uint_as_float(v.x), acc[0]);
    acc[1] = fmaf(p, __uint_as_float(v.y), acc[1]);
    acc[2] = fmaf(p, __uint_as_float(v.z), acc[2]);
    acc[3] = fmaf(p, __uint_as_float(v.w), acc[3]);
  }
};

struct BF16 {
  static constexpr int EPL = 8;
  static constexpr int ESZ = 2;
  __device__ static __forceinline__ float dot(const uint4& k, const uint4& q) {
    float s = dot2_bf16(k.x, q.x, 0.f);
    s = dot2_bf16(k.y, q.y, s);
    s = dot2_bf16(k.z, q.z, s);
    s = dot2_bf16(k.w, q.w, s);
    return s;
  }
  __device__ static __forceinline__ void axpy(float* acc, float p, const uint4& v) {
    acc[0] = fmaf(p, bf16_lo(v.x), acc[0]);
    acc[1] = fmaf(p, bf16_hi(v.x), acc[1]);
    acc[2] = fmaf(p, bf16_lo(v.y), acc[2]);
    acc[3] = fmaf(p, bf16_hi(v.y), acc[3]);
    acc[4] = fmaf(p, bf16_lo(v.z), acc[4]);
    acc[5] = fmaf(p, bf16_hi(v.z), acc[5]);
    acc[6] = fmaf(p, bf16_lo(v.w), acc[6]);
    acc[7] = fmaf(p, bf16_hi(v.w), acc[7]);
  }
};

__device__ __forceinline__ float neg_inf() { return -__builtin_inff(); }

// Def. 3.1 threshold: IEEE fp32 quotient c / t
__device__ __forceinline__ float importance_threshold(float c, int32_t t) { return __fdiv_rn(c, (float)t); }

// vmcnt(0), expcnt and lgkmcnt left at their maxima (gfx9 encoding)
__device__ __forceinline__ void wait_vm_loads() { __builtin_amdgcn_s_waitcnt(0x0F70); }

// Live length of a unit for this launch: lens clamped to [0, Lcap], plus one if a row is appended.
struct UnitLen {
  int L0;         // live keys before the step
  int L;          // keys the step attends over
  bool appended;
  int flags;      // CORM_DEV_* conditions seen
};

// lens_value: what lens holds for the unit
__device__ __forceinline__ UnitLen unit_len_of(const Params& p, int lens_value) {
  UnitLen u;
  u.flags = 0;
  int L0 = lens_value;
  if (L0 < 0 || L0 > p.Lcap) {
    u.flags |= CORM_DEV_BAD_LENS;
    L0 = L0 < 0 ? 0 : p.Lcap;
  }
  u.L0 = L0;
  u.L = L0;
  u.appended = false;
  if (p.do_append) {
    if (L0 < p.Lcap) {
      u.L = L0 + 1;
      u.appended = true;
    } else {
      u.flags |= CORM_DEV_UNIT_FULL;
    }
  }
  return u;
}

__device__ __forceinline__ UnitLen unit_len(const Params& p, int unit) { return unit_len_of(p, p.lens[unit]); }

// Does a unit with L slots in use, T of them live after this step, get compacted in this step?  Exact mode:
// whenever a key went.  Lazy mode: once its dead slots reach dead_num / dead_den of its slots, or its slots
// are about to run out.
// What marks a unit's dirty word for one call: its step and the cache it works on.  Layers that share a
// workspace run the same step one after the other: the word a layer left must not look set to the next one.
__device__ __forceinline__ int32_t dirty_tag(const int32_t* t, const void* K) {
  return (int32_t)((uint32_t)t[0] * 0x9E3779B1u ^ (uint32_t)(reinterpret_cast<uintptr_t>(K) >> 8));
}

__device__ __forceinline__ bool compact_policy(int lazy, int dead_num, int dead_den, int Lcap, int L, int T) {
  if (T == L) return false;
  if (!lazy) return true;
  return (long long)(L - T) * dead_den >= (long long)L * dead_num || L + 1 >= Lcap;
}

// ---------------------------------------------------------------- boolean message (bit ring)
//
// score_dtype CORM_BIT: the ring holds what Algorithm 1 itself keeps, one bit per (recorded query, key
// position): [B, Hq, w, ceil(Tcap/32)] words, bit pos % 32 of word pos / 32.  The row of a step is
// cleared before the step's keys are recorded into it (the positions a step can touch are < t).

__device__ __forceinline__ void clear_bit_rows(const Params& p, int b, int hq0, int G, int nthreads) {
  const int tcur = p.t[b];
  if (!p.ring_bits || !p.ring || tcur < 1 || tcur > p.Tcap) return;
  const int slot = (tcur - 1) % p.w;
  const int nw = min((tcur + 31) >> 5, p.ring_words);
  for (int g = 0; g < G; ++g) {
    uint32_t* row = reinterpret_cast<uint32_t*>(p.ring) + ((size_t)(b * p.Hq + hq0 + g) * p.w + slot) * p.ring_words;
    for (int i = threadIdx.x; i < nw; i += nthreads) row[i] = 0u;
  }
}

// Sets the bits of the keys this wave found important for one head.  pos: this lane's key position
// (any value where !valid); hit implies valid.  When the valid lanes hold consecutive positions
// (lane l: base + l) the wave's ballot is shifted into at most three words and three lanes issue one
// atomic each; otherwise every hit lane sets its own bit.
__device__ __forceinline__ void record_bits(uint32_t* row, int ring_words, int pos, bool valid, bool hit) {
  const int lane = threadIdx.x & 63;
  const unsigned long long vmask = __ballot(valid);
  if (vmask == 0ull) return;
  const int first = __ffsll((long long)vmask) - 1;
  const int base = __shfl(pos, first) - first;
  const bool run = __all(!valid || pos == base + lane) && base >= 0;
  const unsigned long long hmask = __ballot(hit);
  if (hmask == 0ull) return;
  if (run) {
    const int sh = base & 31;
    const unsigned long long lo = hmask << sh;                        // bits 0..63 of the shifted mask
    const uint32_t hi = sh ? (uint32_t)(hmask >> (64 - sh)) : 0u;     // bits 64..95
    if (lane < 3) {
      const uint32_t part = lane == 0 ? (uint32_t)lo : (lane == 1 ? (uint32_t)(lo >> 32) : hi);
      const int w = (base >> 5) + lane;
      if (part && w < ring_words) atomicOr(&row[w], part);
    }
  } else if (hit) {
    atomicOr(&row[pos >> 5], 1u << (pos & 31));
  }
}

}  // namespace

#endif  // CORM_COMMON_HPP
