// HIP kernels (gfx950 / CDNA4, wave64) and C ABI of the CORM decode hot path.
//
// One decode step of one layer is three launches on one stream (kernel boundaries are the only
// cross-workgroup synchronization: no fences, atomics or spinning inside the kernels):
//
//   attend   grid (splits, units).  Workgroup (s, u) streams keys [s*CHUNK, (s+1)*CHUNK) of unit u
//            once: q.k logits (numerator of Eq. 2), an online-softmax partial (max, sum, sum p*v) in
//            fp32, raw logits to scratch.  The owner of the chunk that holds slot lens[u] also
//            writes the step's new key/value row into the cache (the append).
//   record   grid (splits, units).  Merges the split partials (every workgroup recomputes the few
//            numbers it needs) -> out (Eq. 1, by split 0); turns its chunk's logits into normalized
//            scores (Eq. 2), writes them to the ring row of this step, updates last_hit (Def. 3.1)
//            and, when evicting, the keep flag of every key (Def. 4.1 + recent r) and the number of
//            survivors of the chunk.
//   compact  grid (units).  If the unit lost no key: lens = l, done.  Otherwise a stable in-place
//            compaction in ascending tile order (the gather of Algorithm 1).
//
// Row geometry: a K/V row is d*sizeof(T) bytes (256 B for bf16 d=128 and fp32 d=64); each lane
// owns 16 bytes of a row, so LPR = row_bytes/16 lanes share a row and one wave-wide 16-byte
// load covers 64/LPR consecutive rows = 1 KiB of contiguous memory.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <math.h>
#include <cmath>

#include "corm.h"

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

__device__ __forceinline__ UnitLen unit_len(const Params& p, int unit) {
  UnitLen u;
  u.flags = 0;
  int L0 = p.lens[unit];
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

// ---------------------------------------------------------------- attend

typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));

// Raw buffer descriptor (gfx9 family): hardware range checking makes a 16-byte load that does not
// lie entirely below num_bytes return zeros without touching memory.
__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* base, uint32_t num_bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, (int)num_bytes, 0x00020000);
}

__device__ __forceinline__ uint4 buffer_load16(__amdgpu_buffer_rsrc_t r, uint32_t byte_offset) {
  const u32x4_t v = __builtin_amdgcn_raw_buffer_load_b128(r, (int)byte_offset, 0, 0);
  return make_uint4(v.x, v.y, v.z, v.w);
}

// byte offset beyond any descriptor: the load returns zeros without touching memory
constexpr uint32_t DEAD_OFFSET = 0x7ffffff0u;

// 2^x by the hardware instruction alone (results below the normal range flush to zero: such
// probabilities vanish against a sum that is >= 1)
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

template <typename DT, int D, int G, int NW>
struct Attend {
  static constexpr int EPL = DT::EPL;
  static constexpr int ROWB = D * DT::ESZ;
  static constexpr int LPR = ROWB / 16;   // lanes per row
  static constexpr int RPL = 64 / LPR;    // rows per wave-wide load
  static constexpr int U = UNROLL;
  static constexpr int LOAD_ROWS = NW * RPL;          // consecutive rows one unrolled load of the workgroup covers
  static constexpr int STAGE_ROWS = LOAD_ROWS * U;    // rows one pipeline stage of the workgroup covers
  static_assert(U <= LPR, "logit store uses one lane per unrolled load");

  struct Stage {
    uint4 k[U];
    uint4 v[U];
    uint32_t live;   // lazy mode: bit j = the row of load j holds a live key
  };

  // Unrolled load j of a stage: the workgroup reads LOAD_ROWS consecutive rows per load.
  // off = byte offset of this lane's slice in its row of load 0.  Lazy mode: sh_live holds the live
  // masks (LDS), lrow is this lane's row of load 0 relative to the first slot sh_live covers; the
  // loads of dead rows get an out-of-range offset (zeros, no memory traffic).
  template <bool LAZY>
  __device__ static __forceinline__ void load(Stage& st, __amdgpu_buffer_rsrc_t rk, __amdgpu_buffer_rsrc_t rv,
                                              uint32_t off, const unsigned long long* sh_live, int lrow) {
    st.live = (1u << U) - 1u;
    if (LAZY) {
      st.live = 0u;
#pragma unroll
      for (int j = 0; j < U; ++j) {
        const int r = lrow + j * LOAD_ROWS;
        st.live |= (uint32_t)((sh_live[r >> 6] >> (r & 63)) & 1ull) << j;
      }
    }
#pragma unroll
    for (int j = 0; j < U; ++j) {
      const uint32_t o = (!LAZY || ((st.live >> j) & 1u)) ? off + (uint32_t)(j * LOAD_ROWS * ROWB) : DEAD_OFFSET;
      st.k[j] = buffer_load16(rk, o);
    }
#pragma unroll
    for (int j = 0; j < U; ++j) {
      const uint32_t o = (!LAZY || ((st.live >> j) & 1u)) ? off + (uint32_t)(j * LOAD_ROWS * ROWB) : DEAD_OFFSET;
      st.v[j] = buffer_load16(rv, o);
    }
  }

  // row0 = this lane's row in unrolled load 0, lrel0 = its index in the logit staging array
  // sh_logit (LDS, `lstride` floats per head)
  __device__ static __forceinline__ void compute(const Stage& st, int row0, int lrel0, int cend, int cl,
                                                 const uint4 (&qreg)[G], float scale_log2, float* sh_logit,
                                                 int lstride, float (&m_run)[G], float (&z_run)[G],
                                                 float (&acc)[G][EPL]) {
#pragma unroll
    for (int g = 0; g < G; ++g) {
      float s[U];
      float my_logit = 0.f;
#pragma unroll
      for (int j = 0; j < U; ++j) {
        const int row = row0 + j * LOAD_ROWS;
        const float part = DT::dot(st.k[j], qreg[g]);
        const float tot = row_allreduce_sum<LPR>(part) * scale_log2;
        s[j] = (row < cend && ((st.live >> j) & 1u)) ? tot : neg_inf();
        if (cl == j) my_logit = tot;
      }
      // lane cl == j keeps the logit of the row of load j: staged in LDS, written out once per chunk
      if (cl < U) sh_logit[g * lstride + lrel0 + cl * LOAD_ROWS] = my_logit;

      float mnew = m_run[g];
#pragma unroll
      for (int j = 0; j < U; ++j) mnew = fmaxf(mnew, s[j]);
      const float msafe = mnew == neg_inf() ? 0.f : mnew;
      const float a = fast_exp2(m_run[g] - msafe);
      float pj[U];
      float zs = 0.f;
#pragma unroll
      for (int j = 0; j < U; ++j) {
        pj[j] = fast_exp2(s[j] - msafe);
        zs += pj[j];
      }
      z_run[g] = fmaf(z_run[g], a, zs);
#pragma unroll
      for (int e = 0; e < EPL; ++e) acc[g][e] *= a;
#pragma unroll
      for (int j = 0; j < U; ++j) DT::axpy(acc[g], pj[j], st.v[j]);
      m_run[g] = mnew;
    }
  }
};

// Lazy mode, shared by the attend kernels: the live masks of slots [first, first + 64*nwords) go to
// LDS; the appended slot's bit is set there and, by its owner, in the caller's array.  Bits at or
// above the unit's length read as dead.  Ends with a barrier.
__device__ __forceinline__ void stage_live_masks(const Params& p, int unit, const UnitLen& ul, int first, int nwords,
                                                 bool owns_new_slot, unsigned long long* sh_live) {
  unsigned long long* bitsb = p.keepbits + (size_t)unit * p.kb_stride;
  for (int wd = threadIdx.x; wd < nwords; wd += blockDim.x) {
    const int lo = first + wd * 64;   // first slot of this word
    unsigned long long w = 0ull;
    if (lo < ul.L0) {
      w = bitsb[lo >> 6];
      if (ul.L0 - lo < 64) w &= (1ull << (ul.L0 - lo)) - 1ull;   // slots that never held a key
    }
    if (ul.appended && ul.L0 >= lo && ul.L0 < lo + 64) {
      w |= 1ull << (ul.L0 - lo);
      if (owns_new_slot) bitsb[lo >> 6] = w;
    }
    sh_live[wd] = w;
  }
  __syncthreads();
}

template <typename DT, int D, int G, bool LAZY>
__global__ __launch_bounds__(WG) void corm_attend_kernel(const Params p) {
  using A = Attend<DT, D, G, WAVES>;
  constexpr int EPL = A::EPL, ROWB = A::ROWB, LPR = A::LPR, RPL = A::RPL;

  const int split = blockIdx.x;
  const int unit = blockIdx.y;
  const UnitLen ul = unit_len(p, unit);
  const int L = ul.L;
  // (boolean message) the row of this step is cleared here, one launch before the record kernel sets bits
  if (split == 0) clear_bit_rows(p, unit / p.Hkv, (unit % p.Hkv) * G, G, WG);
  if (split * p.part_keys >= L) return;   // no live key in this part

  const int b = unit / p.Hkv;
  const int hkv = unit - b * p.Hkv;
  const int tid = threadIdx.x;
  const int lane = tid & 63, wv = tid >> 6;
  const int sub = lane / LPR, cl = lane % LPR;

  __shared__ float sh_m[G][WAVES];
  __shared__ float sh_z[G][WAVES];
  __shared__ float sh_acc[G][WAVES][D];
  __shared__ float sh_logit[G][CHUNK];   // raw logits of the chunk, stored to the workspace at the end
  __shared__ unsigned long long sh_live[LAZY ? CHUNK / 64 : 1];

  char* Kb = reinterpret_cast<char*>(p.K) + (size_t)unit * p.Lcap * ROWB;
  char* Vb = reinterpret_cast<char*>(p.V) + (size_t)unit * p.Lcap * ROWB;
  const int hq0 = hkv * G;
  // this workgroup's keys: a whole 512-key chunk, or (launches with few units) a fraction of one; the
  // unrolled pipeline below simply ends early
  const int cbeg = split * p.part_keys;
  const int cend = min(cbeg + p.part_keys, L);

  // The append: the owner of the chunk that holds the new slot writes the row and its metadata into the
  // cache first; after the barrier every wave of this workgroup reads it back like any other row.
  if (ul.appended && ul.L0 >= cbeg && ul.L0 < cend) {   // this workgroup owns the new slot
    if (wv == 0) {
      if (lane < LPR) {
        const char* knew = reinterpret_cast<const char*>(p.k_new) + (size_t)unit * ROWB;
        const char* vnew = reinterpret_cast<const char*>(p.v_new) + (size_t)unit * ROWB;
        const uint4 kx = *reinterpret_cast<const uint4*>(knew + (size_t)lane * 16);
        const uint4 vx = *reinterpret_cast<const uint4*>(vnew + (size_t)lane * 16);
        *reinterpret_cast<uint4*>(Kb + (size_t)ul.L0 * ROWB + (size_t)lane * 16) = kx;
        *reinterpret_cast<uint4*>(Vb + (size_t)ul.L0 * ROWB + (size_t)lane * 16) = vx;
      }
      if (lane == 0) {
        p.pos[(size_t)unit * p.Lcap + ul.L0] = p.t[b] - 1;
        p.last_hit[(size_t)unit * p.Lcap + ul.L0] = 0;
      }
    }
    __syncthreads();
  }

  if (LAZY) stage_live_masks(p, unit, ul, cbeg, CHUNK / 64, ul.appended && ul.L0 >= cbeg && ul.L0 < cend, sh_live);

  // this lane's slice of the G queries
  uint4 qreg[G];
#pragma unroll
  for (int g = 0; g < G; ++g)
    qreg[g] = *reinterpret_cast<const uint4*>(reinterpret_cast<const char*>(p.q) +
                                              ((size_t)(b * p.Hq + hq0 + g) * ROWB + (size_t)cl * 16));

  float m_run[G], z_run[G], acc[G][EPL];
#pragma unroll
  for (int g = 0; g < G; ++g) {
    m_run[g] = neg_inf();
    z_run[g] = 0.f;
#pragma unroll
    for (int e = 0; e < EPL; ++e) acc[g][e] = 0.f;
  }
  float* logit_u = p.logits + (size_t)(b * p.Hq + hq0) * p.Lcap;

  // Rows of this chunk only: the descriptors end at row cend, so the pipeline may run past the end of
  // the chunk (those loads return zeros and cost no memory traffic; their scores are masked).
  const __amdgpu_buffer_rsrc_t rk = make_rsrc(Kb, (uint32_t)cend * ROWB);
  const __amdgpu_buffer_rsrc_t rv = make_rsrc(Vb, (uint32_t)cend * ROWB);
  const int lane_row = wv * RPL + sub;                            // this lane's row inside a load
  uint32_t off = (uint32_t)(cbeg + lane_row) * ROWB + (uint32_t)cl * 16;
  constexpr uint32_t STAGE_BYTES = (uint32_t)A::STAGE_ROWS * ROWB;

  // Two register stages, loads always issued one stage ahead.  The chunk loop is fully unrolled
  // (CHUNK is a compile-time constant): no loop-carried registers, no branch around a load, so each
  // stage is consumed while the next one is still in flight and the wait counts are exact.
  constexpr int PAIRS = CHUNK / (2 * A::STAGE_ROWS);
  static_assert(PAIRS >= 1 && CHUNK % (2 * A::STAGE_ROWS) == 0, "CHUNK must hold whole stage pairs");
  typename A::Stage s0, s1;
  A::template load<LAZY>(s0, rk, rv, off, sh_live, lane_row);
#pragma unroll
  for (int i = 0; i < PAIRS; ++i) {
    const int it = cbeg + i * 2 * A::STAGE_ROWS;
    if (it >= cend) break;
    A::template load<LAZY>(s1, rk, rv, off + (uint32_t)(2 * i + 1) * STAGE_BYTES, sh_live,
                           (2 * i + 1) * A::STAGE_ROWS + lane_row);
    A::compute(s0, it + lane_row, it - cbeg + lane_row, cend, cl, qreg, p.scale_log2, &sh_logit[0][0], CHUNK, m_run,
               z_run, acc);
    if (i + 1 < PAIRS)
      A::template load<LAZY>(s0, rk, rv, off + (uint32_t)(2 * i + 2) * STAGE_BYTES, sh_live,
                             (2 * i + 2) * A::STAGE_ROWS + lane_row);
    A::compute(s1, it + A::STAGE_ROWS + lane_row, it - cbeg + A::STAGE_ROWS + lane_row, cend, cl, qreg,
               p.scale_log2, &sh_logit[0][0], CHUNK, m_run, z_run, acc);
  }

  // merge the row groups of the wave (lanes differing in bits >= log2(LPR)), then the waves
#pragma unroll
  for (int g = 0; g < G; ++g) {
#pragma unroll
    for (int o = LPR; o < 64; o <<= 1) {
      const float mo = __shfl_xor(m_run[g], o);
      const float zo = __shfl_xor(z_run[g], o);
      const float mn = fmaxf(m_run[g], mo);
      const float ms = mn == neg_inf() ? 0.f : mn;
      const float a0 = fast_exp2(m_run[g] - ms), a1 = fast_exp2(mo - ms);
      z_run[g] = z_run[g] * a0 + zo * a1;
#pragma unroll
      for (int e = 0; e < EPL; ++e) {
        const float ao = __shfl_xor(acc[g][e], o);
        acc[g][e] = acc[g][e] * a0 + ao * a1;
      }
      m_run[g] = mn;
    }
    if (sub == 0) {
#pragma unroll
      for (int e = 0; e < EPL; ++e) sh_acc[g][wv][cl * EPL + e] = acc[g][e];
      if (cl == 0) {
        sh_m[g][wv] = m_run[g];
        sh_z[g][wv] = z_run[g];
      }
    }
  }
  __syncthreads();

  // the chunk's logits, coalesced
  for (int idx = tid; idx < G * CHUNK; idx += WG) {
    const int g = idx / CHUNK, i = idx - g * CHUNK;
    if (cbeg + i < cend) logit_u[(size_t)g * p.Lcap + cbeg + i] = sh_logit[g][i];
  }

  // partial of this split: [max, sum, acc[D]] per query head
  constexpr int PSTRIDE = D + 2;
  for (int idx = tid; idx < G * D; idx += WG) {
    const int g = idx / D, c = idx - g * D;
    float mw[WAVES];
    float mx = neg_inf();
#pragma unroll
    for (int i = 0; i < WAVES; ++i) {
      mw[i] = sh_m[g][i];
      mx = fmaxf(mx, mw[i]);
    }
    const float ms = mx == neg_inf() ? 0.f : mx;
    float zt = 0.f, at = 0.f;
#pragma unroll
    for (int i = 0; i < WAVES; ++i) {
      const float a = fast_exp2(mw[i] - ms);
      zt = fmaf(sh_z[g][i], a, zt);
      at = fmaf(sh_acc[g][i][c], a, at);
    }
    float* part = p.partials + ((size_t)(b * p.Hq + hq0 + g) * p.npart + split) * PSTRIDE;
    part[2 + c] = at;
    if (c == 0) {
      part[0] = mx;
      part[1] = zt;
    }
  }
}

// ---------------------------------------------------------------- attend, grouped queries: q.K^T on MFMA
//
// bf16, d = 128, G query heads per KV head.  Per stage a wave owns a tile of 16 consecutive keys.
// K is loaded straight into the A-operand layout of v_mfma_f32_16x16x32_bf16 (lane l: key l%16, the 8
// elements 32*kb + 8*(l/16) .. +8 of block kb: 64 contiguous bytes of a row per load), the G queries
// sit in columns 0..G-1 of the B operand (the other columns are zero), and four MFMAs give the 16 x G
// logits of the tile without any cross-lane reduction: lane (n = l%16 < G, lg = l/16) holds the logits
// of head n for keys 4*lg .. 4*lg+3.  The softmax bookkeeping runs in those lanes (all heads at once),
// the probabilities go through a per-wave LDS tile to the lanes that hold V in the row layout
// (lane l: row l/16 of a load, 16-byte column slice l%16), and p.V stays on the vector ALU.

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));

template <int G>
struct AttendGqa {
  static constexpr int D = 128, ROWB = 256, EPL = 8;
  static constexpr int TILE = 16;                    // keys per wave and stage
  static constexpr int STAGE_ROWS = WAVES * TILE;    // keys per workgroup and stage

  struct Stage {
    uint4 k[4];  // A operand, k-blocks 0..3
    uint4 v[4];  // rows 4*j + lane/16 of the tile, this lane's 16-byte column slice
    uint32_t live;   // lazy mode: bit i = key i of the tile is live
  };

  // Lazy mode: sh_live holds the live masks (LDS), trow is the tile's first key relative to the first
  // slot sh_live covers (a multiple of 16); the loads of dead keys get an out-of-range offset.
  template <bool LAZY>
  __device__ static __forceinline__ void load(Stage& st, __amdgpu_buffer_rsrc_t rk, __amdgpu_buffer_rsrc_t rv,
                                              uint32_t koff, uint32_t voff, const unsigned long long* sh_live,
                                              int trow, int n, int lg) {
    st.live = 0xffffu;
    if (LAZY) st.live = (uint32_t)(sh_live[trow >> 6] >> (trow & 63)) & 0xffffu;
    const bool klive = !LAZY || ((st.live >> n) & 1u);
#pragma unroll
    for (int kb = 0; kb < 4; ++kb) st.k[kb] = buffer_load16(rk, klive ? koff + (uint32_t)(64 * kb) : DEAD_OFFSET);
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const bool vlive = !LAZY || ((st.live >> (4 * j + lg)) & 1u);
      st.v[j] = buffer_load16(rv, vlive ? voff + (uint32_t)(j * 4 * ROWB) : DEAD_OFFSET);
    }
  }

  // row0: first key of this wave's tile; lrel0: its index in the logit staging array
  __device__ static __forceinline__ void compute(const Stage& st, int row0, int lrel0, int cend, int n, int lg,
                                                 const uint4 (&qb)[4], float scale_log2, float* sh_logit,
                                                 int lstride, float* sh_p, float* sh_alpha, float& m_run,
                                                 float& z_run, float (&acc)[G][EPL]) {
    f32x4_t d = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int kb = 0; kb < 4; ++kb)
      d = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, st.k[kb]),
                                                  __builtin_bit_cast(bf16x8_t, qb[kb]), d, 0, 0, 0);
    float s[4];
    float tmax = neg_inf();
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const float v = d[r] * scale_log2;
      d[r] = v;
      s[r] = ((row0 + 4 * lg + r) < cend && ((st.live >> (4 * lg + r)) & 1u)) ? v : neg_inf();
      tmax = fmaxf(tmax, s[r]);
    }
    // the 16 keys of head n are spread over the four lane groups
    tmax = rows_allreduce_max(tmax);
    const float mnew = fmaxf(m_run, tmax);
    const float msafe = mnew == neg_inf() ? 0.f : mnew;
    const float a = fast_exp2(m_run - msafe);
    float pr[4];
    float zs = 0.f;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      pr[r] = fast_exp2(s[r] - msafe);
      zs += pr[r];
    }
    z_run = fmaf(z_run, a, zs);
    m_run = mnew;
    if (n < G) {
      *reinterpret_cast<float4*>(&sh_logit[n * lstride + lrel0 + 4 * lg]) = make_float4(d[0], d[1], d[2], d[3]);
#pragma unroll
      for (int r = 0; r < 4; ++r) sh_p[(4 * lg + r) * G + n] = pr[r];
      if (lg == 0) sh_alpha[n] = a;
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");   // LDS is in order within a wave: compiler fence only
    // p.V for the rows this lane holds: row 4*j + lg of the tile in load j
#pragma unroll
    for (int g = 0; g < G; ++g) {
      const float ag = sh_alpha[g];
#pragma unroll
      for (int e = 0; e < EPL; ++e) acc[g][e] *= ag;
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) {
#pragma unroll
      for (int g = 0; g < G; ++g) BF16::axpy(acc[g], sh_p[(4 * j + lg) * G + g], st.v[j]);
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
  }
};

template <int G, bool LAZY>
__global__ __launch_bounds__(WG) void corm_attend_gqa_kernel(const Params p) {
  using A = AttendGqa<G>;
  constexpr int D = A::D, ROWB = A::ROWB, EPL = A::EPL, LPR = 16;

  const int split = blockIdx.x;
  const int unit = blockIdx.y;
  const UnitLen ul = unit_len(p, unit);
  const int L = ul.L;
  if (split == 0) clear_bit_rows(p, unit / p.Hkv, (unit % p.Hkv) * G, G, WG);
  if (split * p.part_keys >= L) return;

  const int b = unit / p.Hkv;
  const int hkv = unit - b * p.Hkv;
  const int tid = threadIdx.x;
  const int lane = tid & 63, wv = tid >> 6;
  const int n = lane & 15, lg = lane >> 4;   // MFMA column / lane group; also: 16-byte column slice / row in a V load

  __shared__ float sh_m[G][WAVES];
  __shared__ float sh_z[G][WAVES];
  __shared__ float sh_acc[G][WAVES][D];
  __shared__ float sh_logit[G][CHUNK];
  __shared__ __attribute__((aligned(16))) float sh_p[WAVES][A::TILE * G];
  __shared__ __attribute__((aligned(16))) float sh_alpha[WAVES][G];
  __shared__ unsigned long long sh_live[LAZY ? CHUNK / 64 : 1];

  char* Kb = reinterpret_cast<char*>(p.K) + (size_t)unit * p.Lcap * ROWB;
  char* Vb = reinterpret_cast<char*>(p.V) + (size_t)unit * p.Lcap * ROWB;
  const int hq0 = hkv * G;
  // this workgroup's keys: a whole 512-key chunk, or (launches with few units) a fraction of one; the
  // unrolled pipeline below simply ends early
  const int cbeg = split * p.part_keys;
  const int cend = min(cbeg + p.part_keys, L);

  if (ul.appended && ul.L0 >= cbeg && ul.L0 < cend) {   // this workgroup owns the new slot: write it, then read it back
    if (wv == 0) {
      if (lane < LPR) {
        const char* knew = reinterpret_cast<const char*>(p.k_new) + (size_t)unit * ROWB;
        const char* vnew = reinterpret_cast<const char*>(p.v_new) + (size_t)unit * ROWB;
        const uint4 kx = *reinterpret_cast<const uint4*>(knew + (size_t)lane * 16);
        const uint4 vx = *reinterpret_cast<const uint4*>(vnew + (size_t)lane * 16);
        *reinterpret_cast<uint4*>(Kb + (size_t)ul.L0 * ROWB + (size_t)lane * 16) = kx;
        *reinterpret_cast<uint4*>(Vb + (size_t)ul.L0 * ROWB + (size_t)lane * 16) = vx;
      }
      if (lane == 0) {
        p.pos[(size_t)unit * p.Lcap + ul.L0] = p.t[b] - 1;
        p.last_hit[(size_t)unit * p.Lcap + ul.L0] = 0;
      }
    }
    __syncthreads();
  }

  if (LAZY) stage_live_masks(p, unit, ul, cbeg, CHUNK / 64, ul.appended && ul.L0 >= cbeg && ul.L0 < cend, sh_live);

  // B operand: column n < G holds query head n, elements 32*kb + 8*lg .. +8 in block kb
  uint4 qb[4];
#pragma unroll
  for (int kb = 0; kb < 4; ++kb) {
    qb[kb] = make_uint4(0u, 0u, 0u, 0u);
    if (n < G)
      qb[kb] = *reinterpret_cast<const uint4*>(reinterpret_cast<const char*>(p.q) +
                                               ((size_t)(b * p.Hq + hq0 + n) * ROWB + (size_t)(64 * kb + 16 * lg)));
  }

  float m_run = neg_inf(), z_run = 0.f;   // of head n, in the lanes with n < G (equal across lane groups)
  float acc[G][EPL];
#pragma unroll
  for (int g = 0; g < G; ++g)
#pragma unroll
    for (int e = 0; e < EPL; ++e) acc[g][e] = 0.f;
  float* logit_u = p.logits + (size_t)(b * p.Hq + hq0) * p.Lcap;

  const __amdgpu_buffer_rsrc_t rk = make_rsrc(Kb, (uint32_t)cend * ROWB);
  const __amdgpu_buffer_rsrc_t rv = make_rsrc(Vb, (uint32_t)cend * ROWB);
  const int tile0 = cbeg + wv * A::TILE;   // first key of this wave's tile in stage 0
  const uint32_t koff = (uint32_t)(tile0 + n) * ROWB + (uint32_t)(16 * lg);
  const uint32_t voff = (uint32_t)(tile0 + lg) * ROWB + (uint32_t)(16 * n);
  constexpr uint32_t STAGE_BYTES = (uint32_t)A::STAGE_ROWS * ROWB;
  constexpr int PAIRS = CHUNK / (2 * A::STAGE_ROWS);
  static_assert(PAIRS >= 1 && CHUNK % (2 * A::STAGE_ROWS) == 0, "CHUNK must hold whole stage pairs");

  typename A::Stage s0, s1;
  A::template load<LAZY>(s0, rk, rv, koff, voff, sh_live, wv * A::TILE, n, lg);
#pragma unroll
  for (int i = 0; i < PAIRS; ++i) {
    const int it = cbeg + i * 2 * A::STAGE_ROWS;
    if (it >= cend) break;
    A::template load<LAZY>(s1, rk, rv, koff + (uint32_t)(2 * i + 1) * STAGE_BYTES,
                           voff + (uint32_t)(2 * i + 1) * STAGE_BYTES, sh_live,
                           (2 * i + 1) * A::STAGE_ROWS + wv * A::TILE, n, lg);
    A::compute(s0, it + wv * A::TILE, it - cbeg + wv * A::TILE, cend, n, lg, qb, p.scale_log2, &sh_logit[0][0],
               CHUNK, sh_p[wv], sh_alpha[wv], m_run, z_run, acc);
    if (i + 1 < PAIRS)
      A::template load<LAZY>(s0, rk, rv, koff + (uint32_t)(2 * i + 2) * STAGE_BYTES,
                             voff + (uint32_t)(2 * i + 2) * STAGE_BYTES, sh_live,
                             (2 * i + 2) * A::STAGE_ROWS + wv * A::TILE, n, lg);
    A::compute(s1, it + A::STAGE_ROWS + wv * A::TILE, it - cbeg + A::STAGE_ROWS + wv * A::TILE, cend, n, lg, qb,
               p.scale_log2, &sh_logit[0][0], CHUNK, sh_p[wv], sh_alpha[wv], m_run, z_run, acc);
  }

  // the wave's sum of head n is spread over the lane groups; its accumulators over the rows of a load.
  // All lanes of a wave share one running max per head, so these are plain sums.
  z_run += __shfl_xor(z_run, 16);
  z_run += __shfl_xor(z_run, 32);
#pragma unroll
  for (int g = 0; g < G; ++g) {
#pragma unroll
    for (int e = 0; e < EPL; ++e) {
      acc[g][e] += __shfl_xor(acc[g][e], 16);
      acc[g][e] += __shfl_xor(acc[g][e], 32);
    }
    if (lg == 0) {
#pragma unroll
      for (int e = 0; e < EPL; ++e) sh_acc[g][wv][n * EPL + e] = acc[g][e];
    }
  }
  if (lg == 0 && n < G) {
    sh_m[n][wv] = m_run;
    sh_z[n][wv] = z_run;
  }
  __syncthreads();

  for (int idx = tid; idx < G * CHUNK; idx += WG) {
    const int g = idx / CHUNK, i = idx - g * CHUNK;
    if (cbeg + i < cend) logit_u[(size_t)g * p.Lcap + cbeg + i] = sh_logit[g][i];
  }

  constexpr int PSTRIDE = D + 2;
  for (int idx = tid; idx < G * D; idx += WG) {
    const int g = idx / D, c = idx - g * D;
    float mw[WAVES];
    float mx = neg_inf();
#pragma unroll
    for (int i = 0; i < WAVES; ++i) {
      mw[i] = sh_m[g][i];
      mx = fmaxf(mx, mw[i]);
    }
    const float ms = mx == neg_inf() ? 0.f : mx;
    float zt = 0.f, at = 0.f;
#pragma unroll
    for (int i = 0; i < WAVES; ++i) {
      const float a = fast_exp2(mw[i] - ms);
      zt = fmaf(sh_z[g][i], a, zt);
      at = fmaf(sh_acc[g][i][c], a, at);
    }
    float* part = p.partials + ((size_t)(b * p.Hq + hq0 + g) * p.npart + split) * PSTRIDE;
    part[2 + c] = at;
    if (c == 0) {
      part[0] = mx;
      part[1] = zt;
    }
  }
}

// ---------------------------------------------------------------- fused unit kernel (no split)
//
// When a launch has at least as many units as the chip has compute units, splitting units buys
// nothing: one workgroup of 512 threads streams a whole unit, keeps the raw logits in LDS, and,
// knowing the unit's max and sum itself, writes out, the ring row, last_hit and the keep flags in
// the same launch.  No partials, no logits round trip through memory, no second kernel.  Only the
// (rare) compaction remains for the two compaction launches.

constexpr int UNIT_WG = 512;
constexpr int UNIT_WAVES = UNIT_WG / 64;
constexpr int UNIT_XCDS = 8;         // accelerator dies of the device; the grid is a multiple of it
constexpr int UNIT_MAX_TILES = 24;   // 48 KiB of logits hold at most 12288 slots = 24 tiles of 512
static_assert(UNIT_WG == CHUNK, "the unit kernel reports survivors per CHUNK slots, one tile each");

template <typename DT, int D, int G, bool LAZY>
__global__ __launch_bounds__(UNIT_WG) void corm_unit_kernel(const Params p, const int lstride) {
  using A = Attend<DT, D, G, UNIT_WAVES>;
  constexpr int EPL = A::EPL, ROWB = A::ROWB, LPR = A::LPR, RPL = A::RPL;

  extern __shared__ float sh_logit[];   // [G][lstride] raw logits of the unit (log2 domain)
  __shared__ float sh_m[G][UNIT_WAVES];
  __shared__ float sh_z[G][UNIT_WAVES];
  __shared__ float sh_acc[G][UNIT_WAVES][D];
  __shared__ float sh_M[G], sh_Z[G];
  __shared__ int sh_tilecnt[UNIT_MAX_TILES];
  // live masks of every slot the pipeline may touch: it runs up to one super-chunk past the unit's end
  constexpr int LIVE_WORDS = (UNIT_MAX_TILES * CHUNK + 2048) / 64;
  __shared__ unsigned long long sh_live[LAZY ? LIVE_WORDS : 1];

  // Workgroups are dealt round-robin to the 8 XCDs, so workgroup id % 8 names the XCD.  Each XCD gets a
  // contiguous range of units: unit lengths often follow the head index with a small period (heads differ,
  // sequences less so), and a strided assignment would put all the long units on one or two XCDs, which
  // then finish the launch alone.
  const int units = p.B * p.Hkv;
  const int per_xcd = (units + UNIT_XCDS - 1) / UNIT_XCDS;
  const int unit = (int)(blockIdx.x % UNIT_XCDS) * per_xcd + (int)(blockIdx.x / UNIT_XCDS);
  if (unit >= units) return;
  const UnitLen ul = unit_len(p, unit);
  const int L = ul.L;
  const int b = unit / p.Hkv;
  const int hkv = unit - b * p.Hkv;
  const int tid = threadIdx.x;
  const int lane = tid & 63, wv = tid >> 6;
  const int sub = lane / LPR, cl = lane % LPR;
  const int hq0 = hkv * G;
  if (tid == 0 && ul.flags && p.status) atomicOr(p.status, ul.flags);

  char* Kb = reinterpret_cast<char*>(p.K) + (size_t)unit * p.Lcap * ROWB;
  char* Vb = reinterpret_cast<char*>(p.V) + (size_t)unit * p.Lcap * ROWB;
  int32_t* posb = p.pos + (size_t)unit * p.Lcap;
  int32_t* lhb = p.last_hit + (size_t)unit * p.Lcap;
  const int tcur = p.t[b];

  clear_bit_rows(p, b, hq0, G, UNIT_WG);   // (ordered before the record phase by the barriers of the merge)
  if (L == 0) {   // empty unit: out = 0, nothing to record
    for (int idx = tid; idx < G * D; idx += UNIT_WG) p.out[(size_t)(b * p.Hq + hq0) * D + idx] = 0.f;
    return;
  }

  // the append: the row and its metadata go into the cache first, then everybody reads them back
  if (ul.appended) {
    if (wv == 0) {
      if (lane < LPR) {
        const char* knew = reinterpret_cast<const char*>(p.k_new) + (size_t)unit * ROWB;
        const char* vnew = reinterpret_cast<const char*>(p.v_new) + (size_t)unit * ROWB;
        const uint4 kx = *reinterpret_cast<const uint4*>(knew + (size_t)lane * 16);
        const uint4 vx = *reinterpret_cast<const uint4*>(vnew + (size_t)lane * 16);
        *reinterpret_cast<uint4*>(Kb + (size_t)ul.L0 * ROWB + (size_t)lane * 16) = kx;
        *reinterpret_cast<uint4*>(Vb + (size_t)ul.L0 * ROWB + (size_t)lane * 16) = vx;
      }
      if (lane == 0) {
        posb[ul.L0] = tcur - 1;
        lhb[ul.L0] = 0;
      }
    }
    __syncthreads();
  }

  if (LAZY) stage_live_masks(p, unit, ul, 0, LIVE_WORDS, true, sh_live);

  if (tid < UNIT_MAX_TILES) sh_tilecnt[tid] = 0;

  uint4 qreg[G];
#pragma unroll
  for (int g = 0; g < G; ++g)
    qreg[g] = *reinterpret_cast<const uint4*>(reinterpret_cast<const char*>(p.q) +
                                              ((size_t)(b * p.Hq + hq0 + g) * ROWB + (size_t)cl * 16));
  float m_run[G], z_run[G], acc[G][EPL];
#pragma unroll
  for (int g = 0; g < G; ++g) {
    m_run[g] = neg_inf();
    z_run[g] = 0.f;
#pragma unroll
    for (int e = 0; e < EPL; ++e) acc[g][e] = 0.f;
  }

  // stream the unit: descriptors end at row L, loads past it return zeros and cost no traffic
  const __amdgpu_buffer_rsrc_t rk = make_rsrc(Kb, (uint32_t)L * ROWB);
  const __amdgpu_buffer_rsrc_t rv = make_rsrc(Vb, (uint32_t)L * ROWB);
  const int lane_row = wv * RPL + sub;
  uint32_t off = (uint32_t)lane_row * ROWB + (uint32_t)cl * 16;
  constexpr uint32_t STAGE_BYTES = (uint32_t)A::STAGE_ROWS * ROWB;
  // Super-chunks of PAIRS_U stage pairs, each fully unrolled (two register stages, the next stage's
  // loads in flight while one is consumed; straight-line code keeps the wait counts exact).  The
  // pipeline drains between super-chunks; the other waves of the compute unit cover that gap.
  constexpr int PAIRS_U = 4;
  constexpr int SUPER_ROWS = 2 * PAIRS_U * A::STAGE_ROWS;
  static_assert(SUPER_ROWS <= 2048, "sh_live covers one super-chunk past the last tile");
  typename A::Stage s0, s1;
  for (int c0 = 0; c0 < L; c0 += SUPER_ROWS) {
    A::template load<LAZY>(s0, rk, rv, off, sh_live, c0 + lane_row);
#pragma unroll
    for (int i = 0; i < PAIRS_U; ++i) {
      const int it = c0 + i * 2 * A::STAGE_ROWS;
      if (it >= L) break;
      A::template load<LAZY>(s1, rk, rv, off + (uint32_t)(2 * i + 1) * STAGE_BYTES, sh_live,
                             it + A::STAGE_ROWS + lane_row);
      A::compute(s0, it + lane_row, it + lane_row, L, cl, qreg, p.scale_log2, sh_logit, lstride, m_run, z_run, acc);
      if (i + 1 < PAIRS_U)
        A::template load<LAZY>(s0, rk, rv, off + (uint32_t)(2 * i + 2) * STAGE_BYTES, sh_live,
                               it + 2 * A::STAGE_ROWS + lane_row);
      A::compute(s1, it + A::STAGE_ROWS + lane_row, it + A::STAGE_ROWS + lane_row, L, cl, qreg, p.scale_log2,
                 sh_logit, lstride, m_run, z_run, acc);
    }
    off += (uint32_t)(2 * PAIRS_U) * STAGE_BYTES;
  }

  // The record phase's metadata (this thread's key of every 512-slot tile), requested in one batch as
  // soon as the stream ends: one memory latency for the whole unit, hidden behind the merge, instead of
  // one per tile.  The registers of the stream's stages are free by now.
  int pos_r[UNIT_MAX_TILES], lh_r[UNIT_MAX_TILES];
#pragma unroll
  for (int kt = 0; kt < UNIT_MAX_TILES; ++kt) {
    pos_r[kt] = 0;
    lh_r[kt] = 0;
    if (kt * UNIT_WG < L) {   // uniform over the workgroup
      const int in = min(kt * UNIT_WG + tid, L - 1);
      pos_r[kt] = posb[in];
      lh_r[kt] = lhb[in];
    }
  }

  // merge the row groups of each wave, then the waves
#pragma unroll
  for (int g = 0; g < G; ++g) {
#pragma unroll
    for (int o = LPR; o < 64; o <<= 1) {
      const float mo = __shfl_xor(m_run[g], o);
      const float zo = __shfl_xor(z_run[g], o);
      const float mn = fmaxf(m_run[g], mo);
      const float ms = mn == neg_inf() ? 0.f : mn;
      const float a0 = fast_exp2(m_run[g] - ms), a1 = fast_exp2(mo - ms);
      z_run[g] = z_run[g] * a0 + zo * a1;
#pragma unroll
      for (int e = 0; e < EPL; ++e) {
        const float ao = __shfl_xor(acc[g][e], o);
        acc[g][e] = acc[g][e] * a0 + ao * a1;
      }
      m_run[g] = mn;
    }
    if (sub == 0) {
#pragma unroll
      for (int e = 0; e < EPL; ++e) sh_acc[g][wv][cl * EPL + e] = acc[g][e];
      if (cl == 0) {
        sh_m[g][wv] = m_run[g];
        sh_z[g][wv] = z_run[g];
      }
    }
  }
  __syncthreads();

  // out (Eq. 1) and the unit's max / sum (Eq. 2)
  for (int idx = tid; idx < G * D; idx += UNIT_WG) {
    const int g = idx / D, c = idx - g * D;
    float mx = neg_inf();
#pragma unroll
    for (int i = 0; i < UNIT_WAVES; ++i) mx = fmaxf(mx, sh_m[g][i]);
    float zt = 0.f, at = 0.f;
#pragma unroll
    for (int i = 0; i < UNIT_WAVES; ++i) {
      const float a = fast_exp2(sh_m[g][i] - mx);
      zt = fmaf(sh_z[g][i], a, zt);
      at = fmaf(sh_acc[g][i][c], a, at);
    }
    p.out[(size_t)(b * p.Hq + hq0 + g) * D + c] = at / zt;
    if (c == 0) {
      sh_M[g] = mx;
      sh_Z[g] = zt;
    }
  }
  __syncthreads();

  // record (Def. 3.1) and decide (Def. 4.1 + recent r).  Survivors per tile are summed with LDS
  // atomics, so the loop has no barrier.
  const bool step_ok = tcur >= 1 && tcur <= p.Tcap;
  if (!step_ok && tid == 0 && p.status) atomicOr(p.status, CORM_DEV_BAD_STEP);
  const int slot = step_ok ? (tcur - 1) % p.w : 0;
  const float thr = importance_threshold(p.thr_scale, step_ok ? tcur : 1);
  const int tfirst = p.do_evict ? p.t_first[b] : tcur;
  const bool full = p.do_evict && step_ok && (tcur - tfirst + 1 >= p.w);
  uint8_t* keepb = p.keep ? p.keep + (size_t)unit * p.Lcap : nullptr;
  unsigned long long* bitsb = p.keepbits + (size_t)unit * p.kb_stride;
  // Boolean message (score_dtype CORM_BIT): a plain loop of its own, so that the unrolled loop below
  // keeps its register budget.  The fp32 score itself is compared; bits are set wave by wave.
  if (p.ring_bits) {
#pragma unroll 1
    for (int tile = 0; tile < L; tile += UNIT_WG) {
      const int i = tile + tid;
      const bool live = i < L && (!LAZY || ((sh_live[i >> 6] >> (i & 63)) & 1ull));
      const int my_pos = posb[min(i, L - 1)];
      int lh = lhb[min(i, L - 1)];
      const bool pos_ok = live && my_pos >= 0 && my_pos < p.Tcap;
      if (live && !pos_ok && p.status) atomicOr(p.status, CORM_DEV_BAD_STEP);
      bool hit = false;
#pragma unroll
      for (int g = 0; g < G; ++g) {
        const float sc = live ? fast_exp2(sh_logit[g * lstride + i] - sh_M[g]) / sh_Z[g] : 0.f;
        const bool hg = live && sc >= thr;
        hit |= hg;
        if (p.ring && step_ok)
          record_bits(reinterpret_cast<uint32_t*>(p.ring) + ((size_t)(b * p.Hq + hq0 + g) * p.w + slot) * p.ring_words,
                      p.ring_words, my_pos, pos_ok, hg && pos_ok);
      }
      bool keep = false;
      if (live) {
        if (hit && step_ok) {
          lh = tcur;
          lhb[i] = tcur;
        }
        const bool recent = LAZY ? (my_pos >= tcur - p.r) : (i >= L - p.r);
        keep = !full || (lh > tcur - p.w) || recent;
      }
      if (p.do_evict && keepb && i < L) keepb[i] = keep ? 1 : 0;
      if (p.do_evict) {
        const unsigned long long bal = __ballot(keep);
        if (lane == 0 && tile + wv * 64 < L) {
          bitsb[(tile >> 6) + wv] = bal;
          atomicAdd(&sh_tilecnt[tile / CHUNK], __popcll(bal));
        }
      }
    }
  }
  // (fully unrolled up to the largest tile count the LDS budget allows: straight-line code keeps the
  // wait counts exact, so a tile's stores are never waited for before the next tile starts)
#pragma unroll
  for (int kt = 0; kt < UNIT_MAX_TILES; ++kt) {
    const int tile = kt * UNIT_WG;
    if (tile >= L || p.ring_bits) break;
    const int i = tile + tid;
    // (lazy mode: a slot whose key was evicted earlier takes no part: nothing recorded, stays dead)
    const bool live = i < L && (!LAZY || ((sh_live[i >> 6] >> (i & 63)) & 1ull));
    const int my_pos = pos_r[kt];
    int lh = lh_r[kt];
    bool keep = false;
    if (live) {
      const bool pos_ok = my_pos >= 0 && my_pos < p.Tcap;
      if (!pos_ok && p.status) atomicOr(p.status, CORM_DEV_BAD_STEP);
      bool hit = false;
#pragma unroll
      for (int g = 0; g < G; ++g) {
        const float sc = fast_exp2(sh_logit[g * lstride + i] - sh_M[g]) / sh_Z[g];
        float stored;
        const size_t ri = ((size_t)(b * p.Hq + hq0 + g) * p.w + slot) * p.Tcap + (size_t)my_pos;
        if (p.ring_bf16) {
          const uint16_t hb = f32_to_bf16_rne(sc);
          stored = __uint_as_float((uint32_t)hb << 16);
          if (step_ok && pos_ok && p.ring) reinterpret_cast<uint16_t*>(p.ring)[ri] = hb;
        } else {
          stored = sc;
          if (step_ok && pos_ok && p.ring) reinterpret_cast<float*>(p.ring)[ri] = sc;
        }
        hit |= (stored >= thr);
      }
      if (hit && step_ok) {
        lh = tcur;
        lhb[i] = tcur;
      }
      // the r newest keys: the last r slots, or (lazy mode, where dead slots lie between) by position
      const bool recent = LAZY ? (my_pos >= tcur - p.r) : (i >= L - p.r);
      keep = !full || (lh > tcur - p.w) || recent;
    }
    if (p.do_evict && keepb && i < L) keepb[i] = keep ? 1 : 0;
    if (p.do_evict) {
      const unsigned long long bal = __ballot(keep);
      if (lane == 0 && tile + wv * 64 < L) {
        bitsb[(tile >> 6) + wv] = bal;
        atomicAdd(&sh_tilecnt[tile / CHUNK], __popcll(bal));
      }
    }
  }
  if (p.do_evict) {
    __syncthreads();
    const int ntile = (L + CHUNK - 1) / CHUNK;
    if (tid < ntile) p.counts[(size_t)unit * p.nsplit + tid] = sh_tilecnt[tid];
  }
}

// ---------------------------------------------------------------- record (+ keep flags)

// RECORD_CHUNKS: 512-slot chunks per workgroup (more keys per workgroup amortize its fixed chain of
// dependent loads; fewer keep the chip full when the launch has few units)
template <int G, int RECORD_CHUNKS>
__global__ __launch_bounds__(WG) void corm_record_kernel(const Params p, const int D) {
  constexpr int RECORD_ROWS = RECORD_CHUNKS * CHUNK;  // keys per workgroup
  constexpr int KPT = RECORD_ROWS / WG;  // keys per thread
  constexpr int KPC = CHUNK / WG;        // of which per chunk
  const int rsplit = blockIdx.x;         // this workgroup covers chunks [rsplit*RECORD_CHUNKS, +RECORD_CHUNKS)
  const int unit = blockIdx.y;
  const UnitLen ul = unit_len(p, unit);
  const int L = ul.L;
  const int tid = threadIdx.x;
  if (rsplit == 0 && tid == 0 && ul.flags && p.status) atomicOr(p.status, ul.flags);
  const int nlive = (L + CHUNK - 1) / CHUNK;                        // chunks that hold keys
  const int nparts = (L + p.part_keys - 1) / p.part_keys;           // attend partials that hold keys
  const int nwg = max((L + RECORD_ROWS - 1) / RECORD_ROWS, 1);      // record workgroups that have work
  if (rsplit >= nwg) return;

  const int b = unit / p.Hkv;
  const int hkv = unit - b * p.Hkv;
  const int hq0 = hkv * G;
  const int lane = tid & 63, wv = tid >> 6;
  const int PSTRIDE = D + 2;
  const int rbeg = rsplit * RECORD_ROWS;
  const int rend = min(rbeg + RECORD_ROWS, L);

  __shared__ float sh_M[G], sh_Z[G];
  __shared__ float sh_out[WAVES][64];
  __shared__ int sh_cnt[RECORD_CHUNKS][WAVES];

  // this thread's keys: issue their loads first, they are consumed after the merge below
  const int32_t* posb = p.pos + (size_t)unit * p.Lcap;
  int32_t* lhb = p.last_hit + (size_t)unit * p.Lcap;
  const float* logit_u = p.logits + (size_t)(b * p.Hq + hq0) * p.Lcap;
  unsigned long long* bitsb = p.keepbits + (size_t)unit * p.kb_stride;
  int my_pos[KPT], my_lh[KPT];
  bool my_live[KPT];   // lazy mode: the slot holds a key that was not evicted earlier
  float lg[KPT][G];
#pragma unroll
  for (int k = 0; k < KPT; ++k) {
    const int i = min(rbeg + k * WG + tid, max(rend - 1, 0));   // clamped: a live slot (or 0 in an empty unit)
    my_pos[k] = posb[i];
    my_lh[k] = lhb[i];
    my_live[k] = p.lazy ? ((bitsb[i >> 6] >> (i & 63)) & 1ull) != 0 : true;
#pragma unroll
    for (int g = 0; g < G; ++g) lg[k][g] = logit_u[(size_t)g * p.Lcap + i];
  }
  const int tcur = p.t[b];
  const int tfirst = p.do_evict ? p.t_first[b] : tcur;

  // global max and sum of Eq. 2 from the split partials (wave g handles head g, g + WAVES, ...)
  for (int g = wv; g < G; g += WAVES) {
    const float* part0 = p.partials + (size_t)(b * p.Hq + hq0 + g) * p.npart * PSTRIDE;
    float mx = neg_inf();
    for (int s = lane; s < nparts; s += 64) mx = fmaxf(mx, part0[(size_t)s * PSTRIDE]);
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off));
    const float ms = mx == neg_inf() ? 0.f : mx;
    float zt = 0.f;
    for (int s = lane; s < nparts; s += 64) {
      const float* ps = part0 + (size_t)s * PSTRIDE;
      zt = fmaf(ps[1], exp2f(ps[0] - ms), zt);
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) zt += __shfl_xor(zt, off);
    if (lane == 0) {
      sh_M[g] = ms;
      sh_Z[g] = zt;
    }
  }
  __syncthreads();

  // out (Eq. 1): (head, block of 64 columns) items of the unit are dealt round-robin to its
  // workgroups; lane = column, so every split's partial row is read as one contiguous 256-byte piece
  // and the loads of all splits are independent (no cross-lane reduction, one memory latency per item)
  // An item belongs to one workgroup; its waves take the splits round-robin and meet in LDS.
  const int cblocks = D / 64;
  for (int item = rsplit; item < G * cblocks; item += nwg) {   // (uniform over the workgroup)
    const int g = item / cblocks, c = (item - g * cblocks) * 64 + lane;
    const float* part0 = p.partials + (size_t)(b * p.Hq + hq0 + g) * p.npart * PSTRIDE;
    const float ms = sh_M[g];
    float at = 0.f;
#pragma unroll 4
    for (int s = wv; s < nparts; s += WAVES) {
      const float* ps = part0 + (size_t)s * PSTRIDE;
      at = fmaf(ps[2 + c], exp2f(ps[0] - ms), at);
    }
    sh_out[wv][lane] = at;
    __syncthreads();
    if (wv == 0) {
      float tot = 0.f;
#pragma unroll
      for (int i = 0; i < WAVES; ++i) tot += sh_out[i][lane];
      p.out[(size_t)(b * p.Hq + hq0 + g) * D + c] = L > 0 ? tot / sh_Z[g] : 0.f;
    }
    __syncthreads();
  }
  if (L == 0) return;  // an empty unit: nothing to record

  // record (Def. 3.1) and decide (Def. 4.1 + recent r) for the keys of this workgroup
  const bool step_ok = tcur >= 1 && tcur <= p.Tcap;
  if (!step_ok && rsplit == 0 && tid == 0 && p.status) atomicOr(p.status, CORM_DEV_BAD_STEP);
  const int slot = step_ok ? (tcur - 1) % p.w : 0;
  const float thr = importance_threshold(p.thr_scale, step_ok ? tcur : 1);
  const bool full = p.do_evict && step_ok && (tcur - tfirst + 1 >= p.w);
  uint8_t* keepb = p.keep ? p.keep + (size_t)unit * p.Lcap : nullptr;

  int kept[RECORD_CHUNKS];
#pragma unroll
  for (int c = 0; c < RECORD_CHUNKS; ++c) kept[c] = 0;
#pragma unroll
  for (int k = 0; k < KPT; ++k) {
    const int i = rbeg + k * WG + tid;
    const bool live = i < rend && my_live[k];
    bool keep = false;
    if (p.ring_bits) {   // (uniform) boolean message: compare the fp32 score, set bits wave by wave
      const bool pos_ok = live && my_pos[k] >= 0 && my_pos[k] < p.Tcap;
      if (live && !pos_ok && p.status) atomicOr(p.status, CORM_DEV_BAD_STEP);
      bool hit = false;
#pragma unroll
      for (int g = 0; g < G; ++g) {
        const float sc = live ? exp2f(lg[k][g] - sh_M[g]) / sh_Z[g] : 0.f;
        const bool hg = live && sc >= thr;
        hit |= hg;
        if (p.ring && step_ok)
          record_bits(reinterpret_cast<uint32_t*>(p.ring) + ((size_t)(b * p.Hq + hq0 + g) * p.w + slot) * p.ring_words,
                      p.ring_words, my_pos[k], pos_ok, hg && pos_ok);
      }
      if (live) {
        int lh = my_lh[k];
        if (hit && step_ok) {
          lh = tcur;
          lhb[i] = tcur;
        }
        const bool recent = p.lazy ? (my_pos[k] >= tcur - p.r) : (i >= L - p.r);
        keep = !full || (lh > tcur - p.w) || recent;
      }
    } else if (live) {
      const bool pos_ok = my_pos[k] >= 0 && my_pos[k] < p.Tcap;
      if (!pos_ok && p.status) atomicOr(p.status, CORM_DEV_BAD_STEP);
      bool hit = false;
#pragma unroll
      for (int g = 0; g < G; ++g) {
        const float sc = exp2f(lg[k][g] - sh_M[g]) / sh_Z[g];
        float stored;
        const size_t ri = ((size_t)(b * p.Hq + hq0 + g) * p.w + slot) * p.Tcap + (size_t)my_pos[k];
        if (p.ring_bf16) {
          const uint16_t hb = f32_to_bf16_rne(sc);
          stored = __uint_as_float((uint32_t)hb << 16);
          if (step_ok && pos_ok && p.ring) reinterpret_cast<uint16_t*>(p.ring)[ri] = hb;
        } else {
          stored = sc;
          if (step_ok && pos_ok && p.ring) reinterpret_cast<float*>(p.ring)[ri] = sc;
        }
        hit |= (stored >= thr);
      }
      int lh = my_lh[k];
      if (hit && step_ok) {
        lh = tcur;
        lhb[i] = tcur;
      }
      // the r newest keys: the last r slots, or (lazy mode, where dead slots lie between) by position
      const bool recent = p.lazy ? (my_pos[k] >= tcur - p.r) : (i >= L - p.r);
      keep = !full || (lh > tcur - p.w) || recent;
    }
    if (p.do_evict && keepb && i < rend) keepb[i] = keep ? 1 : 0;
    const unsigned long long bal = __ballot(keep);
    if (p.do_evict && lane == 0 && rbeg + k * WG + wv * 64 < rend) bitsb[((rbeg + k * WG) >> 6) + wv] = bal;
    kept[k / KPC] += __popcll(bal);
  }
  if (p.do_evict) {
    if (lane == 0) {
#pragma unroll
      for (int c = 0; c < RECORD_CHUNKS; ++c) sh_cnt[c][wv] = kept[c];
    }
    __syncthreads();
    if (tid < RECORD_CHUNKS && rsplit * RECORD_CHUNKS + tid < nlive) {
      int tot = 0;
#pragma unroll
      for (int i = 0; i < WAVES; ++i) tot += sh_cnt[tid][i];
      p.counts[(size_t)unit * p.nsplit + rsplit * RECORD_CHUNKS + tid] = tot;
    }
  }
}

// ---------------------------------------------------------------- stable in-place compaction
//
// Survivor number rho of a unit (in slot order) must end in slot rho.  Two launches, no
// cross-workgroup synchronization inside either:
//
//   local     grid (splits, units).  R_c = survivors before chunk c (from the per-split counts).
//             The workgroup of chunk c = slots [a_c, a_c + CHUNK) moves its survivors with rho >= a_c
//             to slot rho -- inside its own chunk, so it reads and writes only its own slots -- in
//             ascending tiles (every destination <= its source; inside a tile all loads complete
//             before any store).  Its first survivors, those with rho < a_c ("boundary rows", at most
//             as many as slots were freed before the chunk), belong in earlier chunks, whose owners
//             may not have read those slots yet: they go to the chunk's staging area instead.
//   boundary  grid (splits, units).  Workgroup c copies its staged rows to slots
//             [R_c, min(a_c, R_{c+1})): slots no local workgroup writes, and whose old contents were
//             consumed in the previous launch.  Workgroup 0 writes lens, the live count and, in lazy
//             mode, the reset live masks.  The unit's length is handed over through the workspace so
//             that no workgroup of this launch reads lens.
//
// Policy (lazy mode): a unit is compacted only when its dead slots reach dead_num/dead_den of its
// slots (or its slots are about to run out); otherwise both launches leave it alone, its dead rows
// stay in place and the attend kernels skip them by their live masks.  Exact mode: dead_num = 0.

struct CompactShared {
  int32_t wave_count[WAVES];
  int32_t src_of[WG];
};

struct CompactArgs {
  char* K;
  char* V;
  int32_t* pos;
  int32_t* last_hit;
  int32_t* lens;
  const uint8_t* keep;           // caller's byte mask (corm_compact only)
  unsigned long long* keepbits;  // [units, kb_stride] wave ballots: workspace, or the caller's live masks (lazy mode)
  int32_t* kept_idx;             // optional
  const int32_t* counts;         // [units, nsplit]
  int32_t* unit_len;             // [units] slots of the unit in this step (written by local, read by boundary)
  int32_t* nlive;                // optional [units]: live keys after the step
  char* stage_k;                 // [units, nsplit, CHUNK, ROWB]
  char* stage_v;
  int32_t* stage_meta;           // [units, nsplit, CHUNK, 2] (pos, last_hit)
  int32_t nsplit, Lcap, do_append, kb_stride;
  int32_t lazy, dead_num, dead_den;
};

// does this unit get compacted in this step?  L slots, T survivors
__device__ __forceinline__ bool compact_now(const CompactArgs& a, int L, int T) {
  if (T == L) return false;
  if (!a.lazy) return true;
  return (long long)(L - T) * a.dead_den >= (long long)L * a.dead_num || L + 1 >= a.Lcap;
}

// Moves the n_rows survivors listed in src_of (ascending) to consecutive destinations starting at
// survivor number rho0: slot rho if rho >= own_begin, else staging row (rho - stage_rho0).
template <int ROWB>
__device__ __forceinline__ void move_rows(char* Kb, char* Vb, char* sk, char* sv, const int32_t* src_of, int n_rows,
                                          int rho0, int own_begin, int stage_rho0) {
  constexpr int LPR = ROWB / 16;
  constexpr int RPP = WG / LPR;  // rows per pass of the workgroup
  const int tid = threadIdx.x;
  const int sub = tid / LPR;
  const size_t col = (size_t)(tid % LPR) * 16;
  // four passes are in flight together (named registers: an indexed array would be demoted to scratch)
  for (int base = 0; base < n_rows; base += RPP * 4) {
    const int j0 = base + sub, j1 = j0 + RPP, j2 = j1 + RPP, j3 = j2 + RPP;
    const int last = n_rows - 1;
    // clamped row numbers: every load reads a valid row, stores are predicated
    const size_t o0 = (size_t)src_of[min(j0, last)] * ROWB + col;
    const size_t o1 = (size_t)src_of[min(j1, last)] * ROWB + col;
    const size_t o2 = (size_t)src_of[min(j2, last)] * ROWB + col;
    const size_t o3 = (size_t)src_of[min(j3, last)] * ROWB + col;
    const uint4 k0 = *reinterpret_cast<const uint4*>(Kb + o0);
    const uint4 k1 = *reinterpret_cast<const uint4*>(Kb + o1);
    const uint4 k2 = *reinterpret_cast<const uint4*>(Kb + o2);
    const uint4 k3 = *reinterpret_cast<const uint4*>(Kb + o3);
    const uint4 v0 = *reinterpret_cast<const uint4*>(Vb + o0);
    const uint4 v1 = *reinterpret_cast<const uint4*>(Vb + o1);
    const uint4 v2 = *reinterpret_cast<const uint4*>(Vb + o2);
    const uint4 v3 = *reinterpret_cast<const uint4*>(Vb + o3);
    wait_vm_loads();
    __syncthreads();
#define CORM_STORE_ROW(J, KR, VR)                                              \
    if ((J) < n_rows) {                                                          \
      const int rho = rho0 + (J);                                                \
      if (rho >= own_begin) {                                                    \
        const size_t d = (size_t)rho * ROWB + col;                               \
        *reinterpret_cast<uint4*>(Kb + d) = (KR);                                \
        *reinterpret_cast<uint4*>(Vb + d) = (VR);                                \
      } else {                                                                   \
        const size_t d = (size_t)(rho - stage_rho0) * ROWB + col;                \
        *reinterpret_cast<uint4*>(sk + d) = (KR);                                \
        *reinterpret_cast<uint4*>(sv + d) = (VR);                                \
      }                                                                          \
    }
    CORM_STORE_ROW(j0, k0, v0)
    CORM_STORE_ROW(j1, k1, v1)
    CORM_STORE_ROW(j2, k2, v2)
    CORM_STORE_ROW(j3, k3, v3)
#undef CORM_STORE_ROW
  }
}

// One tile step of the scan.  keep: this thread's flag (0 for slots >= L).  Returns this thread's
// rank among the tile's survivors and the tile's survivor count (via *tile_kept).
__device__ __forceinline__ int tile_scan(bool keep, CompactShared& sh, int* tile_kept) {
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
  const unsigned long long bal = __ballot(keep);
  const int rank = __popcll(bal & ((1ull << lane) - 1ull));
  if (lane == 0) sh.wave_count[wv] = __popcll(bal);
  __syncthreads();
  int before = 0, total = 0;
#pragma unroll
  for (int i = 0; i < WAVES; ++i) {
    const int c = sh.wave_count[i];
    if (i < wv) before += c;
    total += c;
  }
  *tile_kept = total;
  return before + rank;
}

__device__ __forceinline__ int compact_unit_len(const CompactArgs& a, int unit) {
  int L = a.lens[unit];
  L = L < 0 ? 0 : (L > a.Lcap ? a.Lcap : L);
  if (a.do_append && L < a.Lcap) L += 1;
  return L;
}

// survivors before chunk `split` (R) and of the whole unit (T), by one wave-wide pass over the counts
__device__ __forceinline__ void unit_counts(const int32_t* cnt, int nlive, int split, int* R, int* T) {
  int r = 0, t = 0;
  for (int s = (threadIdx.x & 63); s < nlive; s += 64) {
    const int c = cnt[s];
    if (s < split) r += c;
    t += c;
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) {
    r += __shfl_xor(r, off);
    t += __shfl_xor(t, off);
  }
  *R = r;
  *T = t;
}

// a caller's byte mask (corm_compact) -> wave ballots and survivors per split
__global__ __launch_bounds__(WG) void corm_count_kernel(const CompactArgs a, int32_t* counts) {
  __shared__ int sh_cnt[WAVES];
  const int split = blockIdx.x, unit = blockIdx.y;
  const int L = compact_unit_len(a, unit);
  const int cbeg = split * CHUNK;
  if (cbeg >= L) return;
  const int cend = min(cbeg + CHUNK, L);
  const uint8_t* keepb = a.keep + (size_t)unit * a.Lcap;
  unsigned long long* bitsb = a.keepbits + (size_t)unit * a.kb_stride;
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
  int kept = 0;
  for (int i0 = cbeg; i0 < cbeg + CHUNK; i0 += WG) {
    const int i = i0 + threadIdx.x;
    const unsigned long long bal = __ballot(i < cend && keepb[i] != 0);
    if (lane == 0 && i0 + wv * 64 < cend) bitsb[(i0 >> 6) + wv] = bal;
    kept += __popcll(bal);
  }
  if (lane == 0) sh_cnt[wv] = kept;
  __syncthreads();
  if (threadIdx.x == 0) {
    int tot = 0;
#pragma unroll
    for (int i = 0; i < WAVES; ++i) tot += sh_cnt[i];
    counts[(size_t)unit * a.nsplit + split] = tot;
  }
}

template <int ROWB>
__global__ __launch_bounds__(WG) void corm_compact_local_kernel(const CompactArgs a) {
  __shared__ CompactShared sh_c;
  const int split = blockIdx.x, unit = blockIdx.y;
  const int tid = threadIdx.x;
  const int L = compact_unit_len(a, unit);
  if (split == 0 && tid == 0) a.unit_len[unit] = L;
  const int nlive = (L + CHUNK - 1) / CHUNK;
  if (split >= nlive) return;
  const int32_t* cnt = a.counts + (size_t)unit * a.nsplit;
  int R, T;   // survivors before this chunk, survivors of the unit
  unit_counts(cnt, nlive, split, &R, &T);
  int32_t* idxb = a.kept_idx ? a.kept_idx + (size_t)unit * a.Lcap : nullptr;
  const int cbeg = split * CHUNK;
  const int cend = min(cbeg + CHUNK, L);
  if (!compact_now(a, L, T)) {   // nothing evicted, or (lazy mode) not enough dead slots yet
    if (idxb && T == L)
      for (int i = cbeg + tid; i < cend; i += WG) idxb[i] = i;
    return;
  }
  const int my_cnt = cnt[split];
  if (R == cbeg && my_cnt == cend - cbeg) {   // no hole before or inside this chunk
    if (idxb)
      for (int i = cbeg + tid; i < cend; i += WG) idxb[i] = i;
    return;
  }
  char* Kb = a.K + (size_t)unit * a.Lcap * ROWB;
  char* Vb = a.V + (size_t)unit * a.Lcap * ROWB;
  int32_t* posb = a.pos + (size_t)unit * a.Lcap;
  int32_t* lhb = a.last_hit + (size_t)unit * a.Lcap;
  const unsigned long long* bitsb = a.keepbits + (size_t)unit * a.kb_stride;
  const size_t stage_row0 = ((size_t)unit * a.nsplit + split) * CHUNK;
  char* sk = a.stage_k + stage_row0 * ROWB;
  char* sv = a.stage_v + stage_row0 * ROWB;
  int32_t* sm = a.stage_meta + stage_row0 * 2;
  // a chunk whose count equals its size lost nothing: its flags are implied (and may be unwritten)
  const bool chunk_full = my_cnt == cend - cbeg;

  int rho_base = R;  // survivor number of the first survivor of the current tile
  for (int tile = cbeg; tile < cend; tile += WG) {
    const int i = tile + tid;
    const bool kp = i < cend && (chunk_full || ((bitsb[i >> 6] >> (i & 63)) & 1ull) != 0);
    int my_pos = 0, my_lh = 0;
    if (kp) {
      my_pos = posb[i];
      my_lh = lhb[i];
    }
    wait_vm_loads();
    int tile_kept;
    const int rank = tile_scan(kp, sh_c, &tile_kept);
    const int rho = rho_base + rank;
    if (kp) {
      sh_c.src_of[rank] = i;
      if (idxb) idxb[rho] = i;
      if (rho >= cbeg) {
        if (rho != i) {
          posb[rho] = my_pos;
          lhb[rho] = my_lh;
        }
      } else {
        sm[(rho - R) * 2] = my_pos;
        sm[(rho - R) * 2 + 1] = my_lh;
      }
    }
    __syncthreads();
    const int tile_n = min(WG, cend - tile);
    if (!(rho_base == tile && tile_kept == tile_n))
      move_rows<ROWB>(Kb, Vb, sk, sv, sh_c.src_of, tile_kept, rho_base, cbeg, R);
    rho_base += tile_kept;
    __syncthreads();
  }
}

template <int ROWB>
__global__ __launch_bounds__(WG) void corm_compact_boundary_kernel(const CompactArgs a) {
  constexpr int LPR = ROWB / 16;
  const int split = blockIdx.x, unit = blockIdx.y;
  const int tid = threadIdx.x;
  const int L = a.unit_len[unit];
  const int nlive = (L + CHUNK - 1) / CHUNK;
  if (split >= nlive && split != 0) return;
  const int32_t* cnt = a.counts + (size_t)unit * a.nsplit;
  int R, T;
  unit_counts(cnt, nlive, split, &R, &T);
  const bool compacted = compact_now(a, L, T);
  if (compacted && split > 0) {
    const int nb = min(split * CHUNK, R + cnt[split]) - R;   // boundary rows of this chunk: survivors [R, R + nb)
    if (nb > 0) {
      char* Kb = a.K + (size_t)unit * a.Lcap * ROWB;
      char* Vb = a.V + (size_t)unit * a.Lcap * ROWB;
      int32_t* posb = a.pos + (size_t)unit * a.Lcap;
      int32_t* lhb = a.last_hit + (size_t)unit * a.Lcap;
      const size_t stage_row0 = ((size_t)unit * a.nsplit + split) * CHUNK;
      const size_t col = (size_t)(tid % LPR) * 16;
      for (int j = tid / LPR; j < nb; j += WG / LPR) {
        const size_t s = (stage_row0 + j) * ROWB + col;
        const size_t d = (size_t)(R + j) * ROWB + col;
        *reinterpret_cast<uint4*>(Kb + d) = *reinterpret_cast<const uint4*>(a.stage_k + s);
        *reinterpret_cast<uint4*>(Vb + d) = *reinterpret_cast<const uint4*>(a.stage_v + s);
      }
      for (int j = tid; j < nb; j += WG) {
        posb[R + j] = a.stage_meta[(stage_row0 + j) * 2];
        lhb[R + j] = a.stage_meta[(stage_row0 + j) * 2 + 1];
      }
    }
  }
  if (split == 0) {
    const int Lnew = compacted ? T : L;
    if (tid == 0) {
      a.lens[unit] = Lnew;
      if (a.nlive) a.nlive[unit] = T;
    }
    if (a.lazy && compacted) {   // every slot below T is live again
      unsigned long long* bitsb = a.keepbits + (size_t)unit * a.kb_stride;
      for (int wd = tid; wd < a.kb_stride; wd += WG) {
        const int lo = wd * 64;
        bitsb[wd] = T >= lo + 64 ? ~0ull : (T > lo ? ((1ull << (T - lo)) - 1ull) : 0ull);
      }
    }
  }
}

// ---------------------------------------------------------------- prompt seeding (dense, matrix cores)
//
// The prompt's last m queries (steps tau_j = t - m + 1 + j) against all its keys: the causal rows of
// Eq. 2, thresholded (Def. 3.1) into last_hit and stored in the ring exactly where m decode steps would
// have put them.  [m x L] logits per head are a dense contraction, so q.K^T runs on the MFMA units; the
// elementwise tail (exp, rounding, compare) and the ring store bound the rest.
//
// Key-major decomposition, the same inner loop twice:
//   pass 1   workgroup = 256 (128) keys of a unit, loops over all query tiles: per query the max and the
//            sum of exp over its keys -> partials [head, key block, query]
//   merge    per query: max and 1/sum over the key blocks
//   pass 2   same loop; p = exp2(s - max) / sum, stored to the ring row of the query's step at the key's
//            position, and per key the latest step whose stored score reaches the threshold
// The workgroup keeps its keys in registers as the A operand (lane l: key l%16 of a 16-key tile, the
// 16 bytes 64*c + 16*(l/16) .. of each 64-byte chunk c of the row); a tile of 16 queries is the B
// operand, loaded the same way.  D: lane l holds query l%16, keys 4*(l/16) .. +3 of the tile.

struct PrefillArgs {
  const void* q_tail;   // [B, Hq, m, d]
  const void* K;
  const int32_t* lens;
  const int32_t* pos;
  int32_t* last_hit;
  const int32_t* t;
  void* ring;
  float2* part;    // [B*Hq, nkb, w]  (max, sum) per key block
  float4* stats;   // [B*Hq, w]       (max, 1/sum, threshold of the query's step, unused)
  int32_t* status;
  int32_t Hq, Hkv, Lcap, Tcap, w, m, nkb, ring_bf16;
  int32_t ring_bits, ring_words;   // boolean message: one bit per (row, position), words per row
  float thr_scale, scale_log2;
};

template <typename DT> struct PrefillMma;
template <> struct PrefillMma<BF16> {
  __device__ static __forceinline__ f32x4_t mma(const uint4& a, const uint4& b, f32x4_t c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, a), __builtin_bit_cast(bf16x8_t, b), c,
                                                   0, 0, 0);
  }
};
template <> struct PrefillMma<F32> {
  // four k-steps of v_mfma_f32_16x16x4_f32: lane group l/16 supplies element 4*(l/16) + e of the chunk in step e
  __device__ static __forceinline__ f32x4_t mma(const uint4& a, const uint4& b, f32x4_t c) {
    c = __builtin_amdgcn_mfma_f32_16x16x4f32(__uint_as_float(a.x), __uint_as_float(b.x), c, 0, 0, 0);
    c = __builtin_amdgcn_mfma_f32_16x16x4f32(__uint_as_float(a.y), __uint_as_float(b.y), c, 0, 0, 0);
    c = __builtin_amdgcn_mfma_f32_16x16x4f32(__uint_as_float(a.z), __uint_as_float(b.z), c, 0, 0, 0);
    c = __builtin_amdgcn_mfma_f32_16x16x4f32(__uint_as_float(a.w), __uint_as_float(b.w), c, 0, 0, 0);
    return c;
  }
};

typedef float f32x2_t __attribute__((ext_vector_type(2)));

// two fp32 -> two bf16 (round to nearest even) in one word, first value in the low half
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  const f32x2_t v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
}

// Pass 1 on one wave tile (16 queries x 16*T keys): per query, max of the scaled logits and the sum of
// exp2 relative to it, over the keys the query sees.  MASKED = false when every query sees every key.
template <bool MASKED, int T>
__device__ __forceinline__ void prefill_stats_tile(const f32x4_t (&d)[T], const int (&kp)[T][4], int vis,
                                                   float scale_log2, float& mx_out, float& z_out) {
  float mx = neg_inf();   // of the raw logits: the scale is positive and keeps their order
#pragma unroll
  for (int tl = 0; tl < T; ++tl)
#pragma unroll
    for (int r = 0; r < 4; ++r) mx = fmaxf(mx, (!MASKED || kp[tl][r] <= vis) ? d[tl][r] : neg_inf());
  mx = rows_allreduce_max(mx);
  const float ms = mx == neg_inf() ? 0.f : mx * scale_log2;
  float z = 0.f;
#pragma unroll
  for (int tl = 0; tl < T; ++tl)
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const float e = fast_exp2(fmaf(d[tl][r], scale_log2, -ms));
      z += (!MASKED || kp[tl][r] <= vis) ? e : 0.f;
    }
  z = rows_allreduce_sum(z);
  mx_out = mx == neg_inf() ? mx : ms;
  z_out = z;
}

// Pass 2 on one wave tile, bf16 ring: the stored scores (packed) and, per key, the step of this query
// where its stored score reaches the threshold.  st = (max, 1/sum) of this lane's query.
template <bool MASKED, int T>
__device__ __forceinline__ void prefill_scores_bf16(const f32x4_t (&d)[T], const int (&kp)[T][4], int vis,
                                                    float scale_log2, float4 st, float thr, int tau,
                                                    uint32_t (&pk)[T][2], int (&hmg)[T][4]) {
#pragma unroll
  for (int tl = 0; tl < T; ++tl) {
    float pv[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const float e = fast_exp2(fmaf(d[tl][r], scale_log2, -st.x)) * st.y;
      pv[r] = (!MASKED || kp[tl][r] <= vis) ? e : 0.f;
    }
    pk[tl][0] = pack_bf16x2(pv[0], pv[1]);
    pk[tl][1] = pack_bf16x2(pv[2], pv[3]);
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const uint32_t w = pk[tl][r >> 1];
      const float stored = __uint_as_float((r & 1) ? (w & 0xffff0000u) : (w << 16));
      const bool hit = stored >= thr && (!MASKED || kp[tl][r] <= vis);
      hmg[tl][r] = hit ? tau : hmg[tl][r];
    }
  }
}

constexpr int PREFILL_SEG = 1024;   // queries whose pass-1 partials a workgroup holds in LDS at a time

template <int ROWB>
struct PrefillGeom {
  static constexpr int NCH = ROWB / 64;            // 64-byte chunks of a row
  static constexpr int T = NCH <= 4 ? 4 : 2;       // 16-key tiles per wave
  static constexpr int KB = WAVES * T * 16;        // keys per workgroup
  static constexpr int QBLK = ROWB <= 256 ? 64 : 32;   // queries staged in LDS at a time
  static constexpr int QROW = ROWB + 16;           // LDS row pitch (padded against bank conflicts)
  static constexpr int QLOADS = QBLK * ROWB / (WG * 16);   // 16-byte loads per thread and block
  static_assert(QBLK * ROWB % (WG * 16) == 0 && QBLK <= WG, "a block is loaded in whole passes of the workgroup");
};

template <typename DT, int D, int PASS, bool BITS>
__global__ __launch_bounds__(WG) void corm_prefill_kernel(const PrefillArgs a) {
  constexpr int ROWB = D * DT::ESZ;
  using Geo = PrefillGeom<ROWB>;
  constexpr int NCH = Geo::NCH, T = Geo::T, KB = Geo::KB;
  constexpr int NEVER = 0x7fffffff;   // position of a slot that holds no key: visible to no query

  const int kb = blockIdx.x, unit = blockIdx.y;
  const int b = unit / a.Hkv, hkv = unit - b * a.Hkv;
  const int G = a.Hq / a.Hkv;
  int L = a.lens[unit];
  L = L < 0 ? 0 : (L > a.Lcap ? a.Lcap : L);
  const int key_blk = kb * KB;
  if (key_blk >= L) return;
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const int n = lane & 15, lg = lane >> 4;
  const int tcur = a.t[b];
  const int tau0 = tcur - a.m + 1;   // step of tail query 0
  if (tau0 < 1 || tcur > a.Tcap) {
    if (tid == 0 && a.status) atomicOr(a.status, CORM_DEV_BAD_STEP);
    return;
  }
  const int s0 = (tau0 - 1) % a.w;   // ring slot of tail query 0

  const char* Kb = reinterpret_cast<const char*>(a.K) + (size_t)unit * a.Lcap * ROWB;
  const int32_t* posb = a.pos + (size_t)unit * a.Lcap;
  const __amdgpu_buffer_rsrc_t rk = make_rsrc(Kb, (uint32_t)L * ROWB);
  const int wkey0 = key_blk + wv * (T * 16);   // first key of this wave

  uint4 ka[T][NCH];
  int kp[T][4];      // positions of this lane's keys 4*lg .. 4*lg+3 of each tile
  bool quad[T];      // the four are consecutive positions: one vector store per query
#pragma unroll
  for (int tl = 0; tl < T; ++tl) {
#pragma unroll
    for (int c = 0; c < NCH; ++c)
      ka[tl][c] = buffer_load16(rk, (uint32_t)(wkey0 + tl * 16 + n) * ROWB + (uint32_t)(c * 64 + 16 * lg));
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int key = wkey0 + tl * 16 + 4 * lg + r;
      int pk = key < L ? posb[key] : NEVER;
      if (key < L && (pk < 0 || pk >= a.Tcap)) {
        if (a.status) atomicOr(a.status, CORM_DEV_BAD_STEP);
        pk = NEVER;
      }
      kp[tl][r] = pk;
    }
    quad[tl] = kp[tl][3] != NEVER && kp[tl][1] == kp[tl][0] + 1 && kp[tl][2] == kp[tl][0] + 2 &&
               kp[tl][3] == kp[tl][0] + 3;
  }
  // Positions ascend with the slot, so queries before the one that sees the block's first key see none of it.
  const int pfirst = posb[key_blk];
  const int jt_first = max(pfirst - tau0 + 1, 0) / 16;

  constexpr int QBLK = Geo::QBLK, QROW = Geo::QROW, QLOADS = Geo::QLOADS;
  __shared__ float2 sh_part[PASS == 1 ? WAVES : 1][PASS == 1 ? PREFILL_SEG : 1];
  __shared__ __attribute__((aligned(16))) char sh_q[2][QBLK * QROW];     // query blocks, double buffered
  __shared__ __attribute__((aligned(16))) float4 sh_st[2][PASS == 2 ? QBLK : 1];   // (max, 1/sum, threshold, -) per query
  // Pass 2, bf16 ring: a wave's 16 x 64 tile of stored scores is turned through LDS so that every query's
  // 64 consecutive positions leave as one 128-byte piece of its ring row (16 bytes per lane) instead of
  // sixteen 8-byte pieces.  Rows are padded to 144 bytes.
  constexpr int TROW = 72;
  __shared__ __attribute__((aligned(16))) uint16_t sh_t[PASS == 2 ? WAVES : 1][PASS == 2 ? 16 : 1][TROW];
  // ... possible when the wave's 64 slots hold consecutive positions starting at a multiple of 8 (and rows
  // of the ring start at multiples of 8 elements), for query tiles that see all of them
  bool wave_rows = false, wave_bitrows = false;
  // every slot of the wave holds a key (then pos_wlast is the largest position among them)
  const bool wave_whole = wkey0 + T * 16 <= L;
  const int pos_w0 = __shfl(kp[0][0], 0);
  const int pos_wlast = __shfl(kp[T - 1][3], 63);
  if (PASS == 2 && T == 4) {
    bool ok = true;
#pragma unroll
    for (int tl = 0; tl < T; ++tl) ok = ok && quad[tl] && kp[tl][0] == pos_w0 + tl * 16 + 4 * lg;
    wave_rows = __all(ok) && a.ring_bf16 && (pos_w0 & 7) == 0 && (a.Tcap & 7) == 0;
    // boolean message: the wave's 64 consecutive positions are exactly two words of a row
    wave_bitrows = BITS && __all(ok) && (pos_w0 & 31) == 0;
  }
  int hm[T][4];   // pass 2: latest step at which one of the group's queries found the key important
#pragma unroll
  for (int tl = 0; tl < T; ++tl)
#pragma unroll
    for (int r = 0; r < 4; ++r) hm[tl][r] = 0;

  for (int g = 0; g < G; ++g) {
    const int head = b * a.Hq + hkv * G + g;
    int hmg[T][4];   // the same for this head alone (its steps ascend, so the last hit is the latest)
#pragma unroll
    for (int tl = 0; tl < T; ++tl)
#pragma unroll
      for (int r = 0; r < 4; ++r) hmg[tl][r] = 0;
    const char* qh = reinterpret_cast<const char*>(a.q_tail) + (size_t)head * a.m * ROWB;
    const __amdgpu_buffer_rsrc_t rq = make_rsrc(qh, (uint32_t)a.m * ROWB);
    const float4* stats = a.stats + (size_t)head * a.w;

    for (int seg0 = 0; seg0 < a.m; seg0 += PREFILL_SEG) {
      const int seg1 = min(seg0 + PREFILL_SEG, a.m);
      if (PASS == 1) {
        for (int i = tid; i < WAVES * PREFILL_SEG; i += WG) (&sh_part[0][0])[i] = make_float2(neg_inf(), 0.f);
        __syncthreads();
      }
      // Queries reach the waves through LDS, QBLK at a time: the block after the current one is in flight
      // (registers) while the current one is worked on, so the loop never waits on a load it has just
      // issued -- nor, with it, on the acknowledgement of the ring stores of the tile before (loads and
      // stores share one in-order counter).  Two LDS buffers, one barrier per block.
      const int blk_first = max(jt_first * 16, seg0) / QBLK * QBLK;
      uint4 qr[QLOADS];
      float4 str = make_float4(0.f, 0.f, 0.f, 0.f);
      if (blk_first < seg1) {
#pragma unroll
        for (int i = 0; i < QLOADS; ++i)   // (past the last query the descriptor's range check returns zeros)
          qr[i] = buffer_load16(rq, (uint32_t)blk_first * ROWB + (uint32_t)((i * WG + tid) * 16));
        if (PASS == 2 && tid < QBLK && blk_first + tid < a.m) str = stats[blk_first + tid];
      }
      __syncthreads();   // the last block of the previous head / segment has been read by every wave
      for (int blk = blk_first; blk < seg1; blk += QBLK) {
        const int cur = (blk / QBLK) & 1;
#pragma unroll
        for (int i = 0; i < QLOADS; ++i) {
          const int o = (i * WG + tid) * 16;   // byte offset inside the block: row o / ROWB, column o % ROWB
          *reinterpret_cast<uint4*>(&sh_q[cur][(o / ROWB) * QROW + (o % ROWB)]) = qr[i];
        }
        if (PASS == 2 && tid < QBLK) sh_st[cur][tid] = str;
        __syncthreads();
        if (blk + QBLK < seg1) {
#pragma unroll
          for (int i = 0; i < QLOADS; ++i)
            qr[i] = buffer_load16(rq, (uint32_t)(blk + QBLK) * ROWB + (uint32_t)((i * WG + tid) * 16));
          str = make_float4(0.f, 0.f, 0.f, 0.f);
          if (PASS == 2 && tid < QBLK && blk + QBLK + tid < a.m) str = stats[blk + QBLK + tid];
        }
#pragma unroll
       for (int ti = 0; ti < QBLK / 16; ++ti) {   // unrolled: the next tile's MFMAs can start under this tile's tail
        const int jt = blk / 16 + ti;
        if (jt < jt_first || jt * 16 >= seg1) continue;   // (uniform) no key of this workgroup is visible / past the end
        uint4 qb[NCH];
#pragma unroll
        for (int c = 0; c < NCH; ++c)
          qb[c] = *reinterpret_cast<const uint4*>(&sh_q[cur][(jt * 16 - blk + n) * QROW + c * 64 + 16 * lg]);
        float4 st = make_float4(0.f, 0.f, 0.f, 0.f);
        if (PASS == 2) st = sh_st[cur][jt * 16 - blk + n];

        f32x4_t d[T];
#pragma unroll
        for (int tl = 0; tl < T; ++tl) {
          d[tl] = f32x4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
          for (int c = 0; c < NCH; ++c) d[tl] = PrefillMma<DT>::mma(ka[tl][c], qb[c], d[tl]);
        }
        const int j = jt * 16 + n;                 // this lane's query
        const int tau = tau0 + j;
        const int vis = j < a.m ? tau - 1 : -1;   // the query sees positions <= vis
        // (uniform over the wave) every query of the tile exists and sees every key of the wave: no masking
        const bool all_seen = wave_whole && jt * 16 + 15 < a.m && pos_wlast <= tau0 + jt * 16 - 1;

        if (PASS == 1) {
          float mx, z;
          if (all_seen) prefill_stats_tile<false, T>(d, kp, vis, a.scale_log2, mx, z);
          else prefill_stats_tile<true, T>(d, kp, vis, a.scale_log2, mx, z);
          if (lg == 0 && j < seg1) sh_part[wv][j - seg0] = make_float2(mx, z);
        } else {
          const float thr = st.z;
          int slot = s0 + j;
          if (slot >= a.w) slot -= a.w;
          const size_t rowbase = ((size_t)head * a.w + (size_t)(j < a.m ? slot : 0)) * a.Tcap;
          const bool rows_now = wave_rows && all_seen;
          if (BITS) {
            // boolean message: the fp32 score itself is compared; bit tl*16 + 4*lg + r of the wave's 64 positions
            uint32_t hbits = 0u;
#pragma unroll
            for (int tl = 0; tl < T; ++tl)
#pragma unroll
              for (int r = 0; r < 4; ++r) {
                const float e = fast_exp2(fmaf(d[tl][r], a.scale_log2, -st.x)) * st.y;
                const bool hit = kp[tl][r] <= vis && e >= thr;
                hmg[tl][r] = hit ? tau : hmg[tl][r];
                hbits |= (uint32_t)hit << (tl * 4 + r);
              }
            if (a.ring) {
              uint32_t* roww = reinterpret_cast<uint32_t*>(a.ring) +
                               ((size_t)head * a.w + (size_t)(j < a.m ? slot : 0)) * a.ring_words;
              if (wave_bitrows) {   // (uniform) the wave owns two whole words of every query's row: plain stores
                uint32_t w0 = (((hbits >> 0) & 0xfu) << (4 * lg)) | (((hbits >> 4) & 0xfu) << (16 + 4 * lg));
                uint32_t w1 = 0u;
                if (T == 4) w1 = (((hbits >> 8) & 0xfu) << (4 * lg)) | (((hbits >> 12) & 0xfu) << (16 + 4 * lg));
                w0 = rows_allreduce_or(w0);
                w1 = rows_allreduce_or(w1);
                if (j < a.m && lg < 2) roww[(pos_w0 >> 5) + lg] = lg == 0 ? w0 : w1;
              } else {              // rows were cleared by the launch before: set single bits
#pragma unroll
                for (int tl = 0; tl < T; ++tl)
#pragma unroll
                  for (int r = 0; r < 4; ++r)
                    if ((hbits >> (tl * 4 + r)) & 1u) atomicOr(&roww[kp[tl][r] >> 5], 1u << (kp[tl][r] & 31));
              }
            }
          } else if (a.ring_bf16) {
            uint32_t pk[T][2];   // stored scores, two bf16 per word
            if (all_seen) prefill_scores_bf16<false, T>(d, kp, vis, a.scale_log2, st, thr, tau, pk, hmg);
            else prefill_scores_bf16<true, T>(d, kp, vis, a.scale_log2, st, thr, tau, pk, hmg);
            uint16_t* row = reinterpret_cast<uint16_t*>(a.ring) + rowbase;
            if (!a.ring) {
              // summary-only state: nothing is recorded but last_hit
            } else if (rows_now) {
#pragma unroll
              for (int tl = 0; tl < T; ++tl)
                *reinterpret_cast<uint2*>(&sh_t[wv][n][tl * 16 + 4 * lg]) = make_uint2(pk[tl][0], pk[tl][1]);
              __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");   // LDS is in order within a wave
#pragma unroll
              for (int hh = 0; hh < 2; ++hh) {
                const int qi = hh * 8 + (lane >> 3), ch = lane & 7;   // query of the tile, 16-byte piece of its row
                const uint4 v = *reinterpret_cast<const uint4*>(&sh_t[wv][qi][ch * 8]);
                int sl = s0 + jt * 16 + qi;
                if (sl >= a.w) sl -= a.w;
                uint16_t* dst =
                    reinterpret_cast<uint16_t*>(a.ring) + ((size_t)head * a.w + sl) * a.Tcap + pos_w0 + ch * 8;
                *reinterpret_cast<uint4*>(dst) = v;
              }
              __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
            } else {
#pragma unroll
              for (int tl = 0; tl < T; ++tl) {
                if (quad[tl] && kp[tl][3] <= vis && ((rowbase + (size_t)kp[tl][0]) & 3) == 0) {
                  *reinterpret_cast<uint2*>(row + kp[tl][0]) = make_uint2(pk[tl][0], pk[tl][1]);
                } else {
#pragma unroll
                  for (int r = 0; r < 4; ++r)
                    if (kp[tl][r] <= vis) row[kp[tl][r]] = (uint16_t)(pk[tl][r >> 1] >> (16 * (r & 1)));
                }
              }
            }
          } else {
            float* row = reinterpret_cast<float*>(a.ring) + rowbase;
#pragma unroll
            for (int tl = 0; tl < T; ++tl) {
              float pv[4];
#pragma unroll
              for (int r = 0; r < 4; ++r) {
                const bool seen = kp[tl][r] <= vis;
                const float e = fast_exp2(fmaf(d[tl][r], a.scale_log2, -st.x)) * st.y;
                pv[r] = seen ? e : 0.f;
                hmg[tl][r] = (seen && pv[r] >= thr) ? tau : hmg[tl][r];
              }
              if (!a.ring) {
              } else if (quad[tl] && kp[tl][3] <= vis && ((rowbase + (size_t)kp[tl][0]) & 3) == 0) {
                *reinterpret_cast<float4*>(row + kp[tl][0]) = make_float4(pv[0], pv[1], pv[2], pv[3]);
              } else {
#pragma unroll
                for (int r = 0; r < 4; ++r)
                  if (kp[tl][r] <= vis) row[kp[tl][r]] = pv[r];
              }
            }
          }
        }
       }
      }
      if (PASS == 1) {
        __syncthreads();
        float2* part = a.part + ((size_t)head * a.nkb + kb) * a.w;
        for (int j = seg0 + tid; j < seg1; j += WG) {
          float mx = neg_inf();
#pragma unroll
          for (int i = 0; i < WAVES; ++i) mx = fmaxf(mx, sh_part[i][j - seg0].x);
          const float ms = mx == neg_inf() ? 0.f : mx;
          float z = 0.f;
#pragma unroll
          for (int i = 0; i < WAVES; ++i) z = fmaf(sh_part[i][j - seg0].y, fast_exp2(sh_part[i][j - seg0].x - ms), z);
          part[j] = make_float2(mx, z);
        }
        __syncthreads();
      }
    }
#pragma unroll
    for (int tl = 0; tl < T; ++tl)
#pragma unroll
      for (int r = 0; r < 4; ++r) hm[tl][r] = max(hm[tl][r], hmg[tl][r]);
  }

  if (PASS == 2) {
    int32_t* lhb = a.last_hit + (size_t)unit * a.Lcap;
#pragma unroll
    for (int tl = 0; tl < T; ++tl)
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        int v = hm[tl][r];
        v = max(v, __shfl_xor(v, 1));
        v = max(v, __shfl_xor(v, 2));
        v = max(v, __shfl_xor(v, 4));
        v = max(v, __shfl_xor(v, 8));
        const int key = wkey0 + tl * 16 + 4 * lg + r;
        if (n == 0 && key < L && v > lhb[key]) lhb[key] = v;
      }
  }
}

// boolean message: zero the words of the rows of steps tau_0 .. tau_{m-1} that pass 2 may set bits in
// (positions < tau); workgroup = 16 rows of one head
__global__ __launch_bounds__(256) void corm_prefill_clear_bits_kernel(const PrefillArgs a) {
  const int head = blockIdx.y;
  const int tcur = a.t[head / a.Hq];
  const int tau0 = tcur - a.m + 1;
  if (tau0 < 1 || tcur > a.Tcap) return;
  const int s0 = (tau0 - 1) % a.w;
  for (int jr = 0; jr < 16; ++jr) {
    const int j = blockIdx.x * 16 + jr;
    if (j >= a.m) break;
    int slot = s0 + j;
    if (slot >= a.w) slot -= a.w;
    uint32_t* row = reinterpret_cast<uint32_t*>(a.ring) + ((size_t)head * a.w + slot) * a.ring_words;
    const int nw = min((tau0 + j + 31) >> 5, a.ring_words);
    for (int i = threadIdx.x; i < nw; i += 256) row[i] = 0u;
  }
}

// per query: max and 1/sum over the key blocks of its unit
__global__ __launch_bounds__(256) void corm_prefill_merge_kernel(const PrefillArgs a, const int KB) {
  const int head = blockIdx.y;
  const int j = blockIdx.x * 256 + threadIdx.x;
  if (j >= a.m) return;
  const int unit = (head / a.Hq) * a.Hkv + (head % a.Hq) / (a.Hq / a.Hkv);
  int L = a.lens[unit];
  L = L < 0 ? 0 : (L > a.Lcap ? a.Lcap : L);
  const int nblk = (L + KB - 1) / KB;
  const float2* part = a.part + (size_t)head * a.nkb * a.w + j;
  float mx = neg_inf();
  for (int k = 0; k < nblk; ++k) mx = fmaxf(mx, part[(size_t)k * a.w].x);
  const float ms = mx == neg_inf() ? 0.f : mx;
  float z = 0.f;
  for (int k = 0; k < nblk; ++k) {
    const float2 pk = part[(size_t)k * a.w];
    z = fmaf(pk.y, exp2f(pk.x - ms), z);
  }
  const int tau = a.t[head / a.Hq] - a.m + 1 + j;
  a.stats[(size_t)head * a.w + j] =
      make_float4(ms, z > 0.f ? 1.0f / z : 0.f, importance_threshold(a.thr_scale, tau >= 1 ? tau : 1), 0.f);
}

// Def. 4.1 + recent r from last_hit for whole units (no append): wave ballots and survivors per chunk
// for the compaction launches, optionally one byte per slot; writes t_first.
__global__ __launch_bounds__(WG) void corm_decide_kernel(const int32_t* lens, const int32_t* last_hit, const int32_t* t,
                                                         int32_t* t_first, unsigned long long* keepbits,
                                                         int32_t* counts, uint8_t* keep, int Hkv, int Lcap, int nsplit,
                                                         int kb_stride, int w, int r, int m) {
  __shared__ int sh_cnt[WAVES];
  const int split = blockIdx.x, unit = blockIdx.y;
  const int b = unit / Hkv;
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const int tcur = t[b];
  if (split == 0 && unit % Hkv == 0 && tid == 0) t_first[b] = tcur - m + 1;
  int L = lens[unit];
  L = L < 0 ? 0 : (L > Lcap ? Lcap : L);
  const int cbeg = split * CHUNK;
  if (cbeg >= L) return;
  const int cend = min(cbeg + CHUNK, L);
  const bool full = m >= w;
  const int32_t* lhb = last_hit + (size_t)unit * Lcap;
  unsigned long long* bitsb = keepbits + (size_t)unit * kb_stride;
  int kept = 0;
  for (int i0 = cbeg; i0 < cbeg + CHUNK; i0 += WG) {
    const int i = i0 + tid;
    bool k = false;
    if (i < cend) {
      k = !full || lhb[i] > tcur - w || i >= L - r;
      if (keep) keep[(size_t)unit * Lcap + i] = k ? 1 : 0;
    }
    const unsigned long long bal = __ballot(k);
    if (lane == 0 && i0 + wv * 64 < cend) bitsb[(i0 >> 6) + wv] = bal;
    kept += __popcll(bal);
  }
  if (lane == 0) sh_cnt[wv] = kept;
  __syncthreads();
  if (tid == 0) {
    int tot = 0;
#pragma unroll
    for (int i = 0; i < WAVES; ++i) tot += sh_cnt[i];
    counts[(size_t)unit * nsplit + split] = tot;
  }
}

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

__global__ void corm_threshold_kernel(float c, const int32_t* t, int n, float* thr) {
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) thr[i] = importance_threshold(c, t[i]);
}

__global__ void corm_fill_i32_kernel(int32_t* p, size_t n, int32_t v) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = v;
}

// ---------------------------------------------------------------- host side

struct WorkspaceLayout {
  size_t counts_off, unit_len_off, keepbits_off, partials_off, logits_off, stage_meta_off, stage_k_off, stage_v_off;
  size_t seed_part_off, seed_stats_off, total;
  int nsplit, kb_stride;
  int seed_kb, seed_nkb;   // prompt seeding: keys per workgroup, key blocks per unit
};

size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

int row_bytes(const corm_desc* d) { return d->d * (d->kv_dtype == CORM_F32 ? 4 : 2); }

WorkspaceLayout workspace_layout(const corm_desc& d) {
  WorkspaceLayout w;
  w.nsplit = (d.Lcap + CHUNK - 1) / CHUNK;
  const size_t units = (size_t)d.B * d.Hkv, heads = (size_t)d.B * d.Hq;
  const size_t stage_rows = units * w.nsplit * CHUNK;   // every survivor of a chunk may be a boundary row
  w.counts_off = 0;
  w.kb_stride = (d.Lcap + 63) / 64;
  w.unit_len_off = align_up(units * w.nsplit * sizeof(int32_t), 256);
  w.keepbits_off = align_up(w.unit_len_off + units * sizeof(int32_t), 256);
  w.partials_off = align_up(w.keepbits_off + units * w.kb_stride * sizeof(unsigned long long), 256);
  w.logits_off = align_up(w.partials_off + heads * w.nsplit * MAX_PARTS_PER_CHUNK * (d.d + 2) * sizeof(float), 256);
  w.stage_meta_off = align_up(w.logits_off + heads * d.Lcap * sizeof(float), 256);
  w.stage_k_off = align_up(w.stage_meta_off + stage_rows * 2 * sizeof(int32_t), 256);
  w.stage_v_off = align_up(w.stage_k_off + stage_rows * row_bytes(&d), 256);
  w.seed_kb = row_bytes(&d) / 64 <= 4 ? PrefillGeom<256>::KB : PrefillGeom<512>::KB;
  w.seed_nkb = (d.Lcap + w.seed_kb - 1) / w.seed_kb;
  w.seed_part_off = align_up(w.stage_v_off + stage_rows * row_bytes(&d), 256);
  w.seed_stats_off = align_up(w.seed_part_off + heads * w.seed_nkb * d.w * sizeof(float2), 256);
  w.total = align_up(w.seed_stats_off + heads * d.w * sizeof(float4), 256);
  return w;
}

int validate_desc(const corm_desc* d) {
  if (!d) return CORM_EINVAL;
  if (d->B < 1 || d->Hq < 1 || d->Hkv < 1 || d->Lcap < 1 || d->Tcap < 1 || d->w < 1 || d->r < 1) return CORM_EINVAL;
  if (d->Hq % d->Hkv != 0) return CORM_EINVAL;
  if (!(d->thr_scale >= 0.f) || !std::isfinite(d->thr_scale)) return CORM_EINVAL;
  if (!(d->sm_scale >= 0.f) || !std::isfinite(d->sm_scale)) return CORM_EINVAL;
  if ((long long)d->B * d->Hkv > 2147483647LL / 2 || (long long)d->B * d->Hq > 2147483647LL / 2) return CORM_EINVAL;
  if (d->B * d->Hkv > 65535) return CORM_EUNSUPPORTED;  // grid.y limit
  if ((long long)d->Lcap * 512 >= (1LL << 31)) return CORM_EUNSUPPORTED;  // byte offsets inside a unit are 32-bit
  if (d->kv_dtype != CORM_F32 && d->kv_dtype != CORM_BF16) return CORM_EUNSUPPORTED;
  if (d->score_dtype != CORM_F32 && d->score_dtype != CORM_BF16 && d->score_dtype != CORM_BIT) return CORM_EUNSUPPORTED;
  if (d->d != 64 && d->d != 128) return CORM_EUNSUPPORTED;
  const int G = d->Hq / d->Hkv;
  if (G != 1 && G != 2 && G != 4 && G != 8) return CORM_EUNSUPPORTED;
  return CORM_OK;
}

bool misaligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) != 0; }
bool misaligned4(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 3u) != 0; }

int launch_status() { return hipGetLastError() == hipSuccess ? CORM_OK : CORM_EHIP; }

// optional events recorded around the attend launch of the next step call (corm_profile_attend)
hipEvent_t g_prof_start = nullptr, g_prof_stop = nullptr;

int check_workspace(const corm_desc* d, void* workspace, size_t workspace_bytes, WorkspaceLayout* wl) {
  *wl = workspace_layout(*d);
  if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255u)) return CORM_EINVAL;
  if (workspace_bytes < wl->total) return CORM_ECAPACITY;
  return CORM_OK;
}

// fills the descriptor- and workspace-derived fields of p
void bind_params(const corm_desc* d, const WorkspaceLayout& wl, void* workspace, Params& p) {
  char* ws = reinterpret_cast<char*>(workspace);
  p.counts = reinterpret_cast<int32_t*>(ws + wl.counts_off);
  p.keepbits = reinterpret_cast<unsigned long long*>(ws + wl.keepbits_off);
  p.kb_stride = wl.kb_stride;
  p.partials = reinterpret_cast<float*>(ws + wl.partials_off);
  p.logits = reinterpret_cast<float*>(ws + wl.logits_off);
  p.B = d->B; p.Hq = d->Hq; p.Hkv = d->Hkv; p.Lcap = d->Lcap; p.Tcap = d->Tcap; p.w = d->w; p.r = d->r;
  p.nsplit = wl.nsplit;
  p.npart = wl.nsplit * MAX_PARTS_PER_CHUNK;
  p.part_keys = CHUNK;
  p.thr_scale = d->thr_scale;
  const float sm = d->sm_scale > 0.f ? d->sm_scale : 1.0f / sqrtf((float)d->d);
  p.scale_log2 = sm * LOG2E;
  p.ring_bf16 = d->score_dtype == CORM_BF16;
  p.ring_bits = d->score_dtype == CORM_BIT;
  p.ring_words = (d->Tcap + 31) / 32;
}

// 0 = choose by shape, 1 = split kernels (attend + record), 2 = fused unit kernel,
// 3 = split kernels with q.K^T on the vector ALU even where the MFMA kernel applies
int g_force_path = 0;
int g_num_cus = 0;

template <typename DT, int D, bool LAZY>
int launch_attend_g(const Params& p, int G, dim3 grid, hipStream_t s) {
  switch (G) {
    case 1: hipLaunchKernelGGL((corm_attend_kernel<DT, D, 1, LAZY>), grid, dim3(WG), 0, s, p); break;
    case 2: hipLaunchKernelGGL((corm_attend_kernel<DT, D, 2, LAZY>), grid, dim3(WG), 0, s, p); break;
    case 4: hipLaunchKernelGGL((corm_attend_kernel<DT, D, 4, LAZY>), grid, dim3(WG), 0, s, p); break;
    case 8: hipLaunchKernelGGL((corm_attend_kernel<DT, D, 8, LAZY>), grid, dim3(WG), 0, s, p); break;
    default: return CORM_EUNSUPPORTED;
  }
  return launch_status();
}

template <bool LAZY>
int launch_attend_gqa(const Params& p, int G, dim3 grid, hipStream_t s) {
  switch (G) {
    case 2: hipLaunchKernelGGL((corm_attend_gqa_kernel<2, LAZY>), grid, dim3(WG), 0, s, p); break;
    case 4: hipLaunchKernelGGL((corm_attend_gqa_kernel<4, LAZY>), grid, dim3(WG), 0, s, p); break;
    case 8: hipLaunchKernelGGL((corm_attend_gqa_kernel<8, LAZY>), grid, dim3(WG), 0, s, p); break;
    default: return CORM_EUNSUPPORTED;
  }
  return launch_status();
}

template <bool LAZY>
int launch_attend_dt(const corm_desc* d, const Params& p, int G, dim3 grid, hipStream_t s) {
  if (d->kv_dtype == CORM_F32)
    return d->d == 64 ? launch_attend_g<F32, 64, LAZY>(p, G, grid, s) : launch_attend_g<F32, 128, LAZY>(p, G, grid, s);
  // grouped queries, bf16, d = 128: q.K^T on the matrix cores
  if (d->d == 128 && G > 1 && g_force_path != 3) return launch_attend_gqa<LAZY>(p, G, grid, s);
  return d->d == 64 ? launch_attend_g<BF16, 64, LAZY>(p, G, grid, s) : launch_attend_g<BF16, 128, LAZY>(p, G, grid, s);
}

int launch_attend(const corm_desc* d, const Params& p, hipStream_t s) {
  const int G = d->Hq / d->Hkv;
  const dim3 grid((d->Lcap + p.part_keys - 1) / p.part_keys, d->B * d->Hkv);
  const hipEvent_t ev0 = g_prof_start, ev1 = g_prof_stop;
  g_prof_start = g_prof_stop = nullptr;
  if (ev0 && hipEventRecord(ev0, s) != hipSuccess) return CORM_EHIP;
  const int rc = p.lazy ? launch_attend_dt<true>(d, p, G, grid, s) : launch_attend_dt<false>(d, p, G, grid, s);
  if (rc) return rc;
  if (ev1 && hipEventRecord(ev1, s) != hipSuccess) return CORM_EHIP;
  return CORM_OK;
}


size_t unit_lds_bytes(const corm_desc* d, int* lstride) {
  const int rowb = row_bytes(d);
  const int stage_rows = UNIT_WAVES * (64 / (rowb / 16)) * UNROLL;
  *lstride = (d->Lcap + 2 * stage_rows - 1) / (2 * stage_rows) * (2 * stage_rows);
  return (size_t)(d->Hq / d->Hkv) * (size_t)(*lstride) * sizeof(float);
}

// The unit kernel needs the unit's logits in LDS (48 KiB of dynamic LDS at most here, so that two
// workgroups fit a compute unit) and pays off once there are at least as many units as compute units.
bool use_unit_path(const corm_desc* d) {
  int lstride;
  const bool fits = unit_lds_bytes(d, &lstride) <= 48 * 1024 && d->Hq / d->Hkv <= 4;  // G = 8 exceeds the register file
  if (g_force_path == 1 || g_force_path == 3 || !fits) return false;
  if (g_force_path == 2) return true;
  if (g_num_cus == 0) {
    int dev = 0, n = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0)
      n = 256;
    g_num_cus = n;
  }
  return d->B * d->Hkv >= g_num_cus;
}

template <typename DT, int D, bool LAZY>
int launch_unit_g(const Params& p, int G, int units, size_t lds, int lstride, hipStream_t s) {
  switch (G) {
    case 1:
      hipLaunchKernelGGL((corm_unit_kernel<DT, D, 1, LAZY>), dim3(units), dim3(UNIT_WG), lds, s, p, lstride);
      break;
    case 2:
      hipLaunchKernelGGL((corm_unit_kernel<DT, D, 2, LAZY>), dim3(units), dim3(UNIT_WG), lds, s, p, lstride);
      break;
    case 4:
      hipLaunchKernelGGL((corm_unit_kernel<DT, D, 4, LAZY>), dim3(units), dim3(UNIT_WG), lds, s, p, lstride);
      break;
    default: return CORM_EUNSUPPORTED;
  }
  return launch_status();
}

template <bool LAZY>
int launch_unit_dt(const corm_desc* d, const Params& p, int G, int units, size_t lds, int lstride, hipStream_t s) {
  if (d->kv_dtype == CORM_F32)
    return d->d == 64 ? launch_unit_g<F32, 64, LAZY>(p, G, units, lds, lstride, s)
                      : launch_unit_g<F32, 128, LAZY>(p, G, units, lds, lstride, s);
  return d->d == 64 ? launch_unit_g<BF16, 64, LAZY>(p, G, units, lds, lstride, s)
                    : launch_unit_g<BF16, 128, LAZY>(p, G, units, lds, lstride, s);
}

int launch_unit(const corm_desc* d, const Params& p, hipStream_t s) {
  int lstride;
  const size_t lds = unit_lds_bytes(d, &lstride);
  const int G = d->Hq / d->Hkv;
  const int units = (d->B * d->Hkv + UNIT_XCDS - 1) / UNIT_XCDS * UNIT_XCDS;   // grid: whole rounds over the XCDs
  const hipEvent_t ev0 = g_prof_start, ev1 = g_prof_stop;
  g_prof_start = g_prof_stop = nullptr;
  if (ev0 && hipEventRecord(ev0, s) != hipSuccess) return CORM_EHIP;
  const int rc = p.lazy ? launch_unit_dt<true>(d, p, G, units, lds, lstride, s)
                        : launch_unit_dt<false>(d, p, G, units, lds, lstride, s);
  if (rc) return rc;
  if (ev1 && hipEventRecord(ev1, s) != hipSuccess) return CORM_EHIP;
  return CORM_OK;
}

// append (if p.do_append) + attend + record: one fused launch or the attend / record pair
int launch_attend_record(const corm_desc* d, const Params& p, hipStream_t s);

template <int RC>
int launch_record_rc(const corm_desc* d, const Params& p, hipStream_t s) {
  const int G = d->Hq / d->Hkv;
  const dim3 grid((p.nsplit + RC - 1) / RC, d->B * d->Hkv);
  switch (G) {
    case 1: hipLaunchKernelGGL((corm_record_kernel<1, RC>), grid, dim3(WG), 0, s, p, d->d); break;
    case 2: hipLaunchKernelGGL((corm_record_kernel<2, RC>), grid, dim3(WG), 0, s, p, d->d); break;
    case 4: hipLaunchKernelGGL((corm_record_kernel<4, RC>), grid, dim3(WG), 0, s, p, d->d); break;
    case 8: hipLaunchKernelGGL((corm_record_kernel<8, RC>), grid, dim3(WG), 0, s, p, d->d); break;
    default: return CORM_EUNSUPPORTED;
  }
  return launch_status();
}

int launch_record(const corm_desc* d, const Params& p, hipStream_t s) {
  // the largest workgroup that still leaves about four workgroups per compute unit
  const long units = (long)d->B * d->Hkv;
  const long want = 4L * (g_num_cus > 0 ? g_num_cus : 256);
  if (units * ((p.nsplit + 3) / 4) >= want) return launch_record_rc<4>(d, p, s);
  if (units * ((p.nsplit + 1) / 2) >= want) return launch_record_rc<2>(d, p, s);
  return launch_record_rc<1>(d, p, s);
}

// Keys per attend workgroup on the split path: a whole chunk, or a half / a quarter of one while the
// launch would otherwise have fewer than about two workgroups per compute unit.  A part must hold whole
// pairs of pipeline stages of the kernel that runs.
int attend_part_keys(const corm_desc* d) {
  const int G = d->Hq / d->Hkv;
  const bool mfma = d->kv_dtype == CORM_BF16 && d->d == 128 && G > 1 && g_force_path != 3;
  const int stage_rows = mfma ? WAVES * 16 : WAVES * (64 / (row_bytes(d) / 16)) * UNROLL;
  const long want = 2L * (g_num_cus > 0 ? g_num_cus : 256);
  const long wgs = (long)d->B * d->Hkv * ((d->Lcap + CHUNK - 1) / CHUNK);
  int part = CHUNK;
  while (part / 2 >= 2 * stage_rows && CHUNK / (part / 2) <= MAX_PARTS_PER_CHUNK && wgs * (CHUNK / part) < want) part /= 2;
  return part;
}

int launch_attend_record(const corm_desc* d, const Params& p0, hipStream_t s) {
  if (use_unit_path(d)) return launch_unit(d, p0, s);
  Params p = p0;
  p.part_keys = attend_part_keys(d);
  const int rc = launch_attend(d, p, s);
  if (rc) return rc;
  return launch_record(d, p, s);
}

// Policy of the compaction launches: exact mode compacts every unit that lost a key; lazy mode only
// units whose dead slots reach dead_num / dead_den of their slots.
struct CompactPolicy {
  int lazy = 0, dead_num = 0, dead_den = 1;
  unsigned long long* live = nullptr;   // lazy mode: the caller's live masks take the place of the keep masks
  int32_t* nlive = nullptr;             // optional output: live keys per unit
};

// local + boundary launches of the compaction; count_first: derive the per-split counts from the mask
int launch_compact(const corm_desc* d, const WorkspaceLayout& wl, void* workspace, void* K, void* V, int32_t* pos,
                   int32_t* last_hit, int32_t* lens, const uint8_t* keep, int32_t* kept_idx, int do_append,
                   bool count_first, const CompactPolicy& pol, hipStream_t s) {
  char* ws = reinterpret_cast<char*>(workspace);
  CompactArgs a;
  a.K = reinterpret_cast<char*>(K);
  a.V = reinterpret_cast<char*>(V);
  a.pos = pos; a.last_hit = last_hit; a.lens = lens; a.keep = keep; a.kept_idx = kept_idx;
  a.keepbits = pol.live ? pol.live : reinterpret_cast<unsigned long long*>(ws + wl.keepbits_off);
  a.kb_stride = wl.kb_stride;
  int32_t* counts = reinterpret_cast<int32_t*>(ws + wl.counts_off);
  a.counts = counts;
  a.unit_len = reinterpret_cast<int32_t*>(ws + wl.unit_len_off);
  a.nlive = pol.nlive;
  a.stage_k = ws + wl.stage_k_off;
  a.stage_v = ws + wl.stage_v_off;
  a.stage_meta = reinterpret_cast<int32_t*>(ws + wl.stage_meta_off);
  a.nsplit = wl.nsplit; a.Lcap = d->Lcap; a.do_append = do_append;
  a.lazy = pol.lazy; a.dead_num = pol.dead_num; a.dead_den = pol.dead_den;
  const dim3 grid(wl.nsplit, d->B * d->Hkv);
  if (count_first) {
    hipLaunchKernelGGL(corm_count_kernel, grid, dim3(WG), 0, s, a, counts);
    if (launch_status()) return CORM_EHIP;
  }
  switch (row_bytes(d)) {
    case 128:
      hipLaunchKernelGGL((corm_compact_local_kernel<128>), grid, dim3(WG), 0, s, a);
      hipLaunchKernelGGL((corm_compact_boundary_kernel<128>), grid, dim3(WG), 0, s, a);
      break;
    case 256:
      hipLaunchKernelGGL((corm_compact_local_kernel<256>), grid, dim3(WG), 0, s, a);
      hipLaunchKernelGGL((corm_compact_boundary_kernel<256>), grid, dim3(WG), 0, s, a);
      break;
    case 512:
      hipLaunchKernelGGL((corm_compact_local_kernel<512>), grid, dim3(WG), 0, s, a);
      hipLaunchKernelGGL((corm_compact_boundary_kernel<512>), grid, dim3(WG), 0, s, a);
      break;
    default: return CORM_EUNSUPPORTED;
  }
  return launch_status();
}

template <typename DT, int D>
int launch_prefill_dt(const PrefillArgs& a, dim3 grid, dim3 mgrid, int KB, hipStream_t s) {
  hipLaunchKernelGGL((corm_prefill_kernel<DT, D, 1, false>), grid, dim3(WG), 0, s, a);
  hipLaunchKernelGGL(corm_prefill_merge_kernel, mgrid, dim3(256), 0, s, a, KB);
  if (a.ring_bits) hipLaunchKernelGGL((corm_prefill_kernel<DT, D, 2, true>), grid, dim3(WG), 0, s, a);
  else hipLaunchKernelGGL((corm_prefill_kernel<DT, D, 2, false>), grid, dim3(WG), 0, s, a);
  return launch_status();
}

int check_step_pointers(const void* q, const void* k_new, const void* v_new, const void* K, const void* V,
                        const int32_t* lens, const int32_t* pos, const int32_t* last_hit, const int32_t* t,
                        const int32_t* t_first, const void* score_ring, const float* out, const int32_t* kept_idx,
                        const int32_t* status) {
  if (!q || !k_new || !v_new || !K || !V || !lens || !pos || !last_hit || !t || !t_first || !out)
    return CORM_EINVAL;   // (score_ring may be null: summary-only state)
  if (misaligned16(q) || misaligned16(k_new) || misaligned16(v_new) || misaligned16(K) || misaligned16(V) ||
      misaligned4(out) || misaligned4(score_ring))
    return CORM_EINVAL;
  if (misaligned4(lens) || misaligned4(pos) || misaligned4(last_hit) || misaligned4(t) || misaligned4(t_first) ||
      misaligned4(kept_idx) || misaligned4(status))
    return CORM_EINVAL;
  return CORM_OK;
}

}  // namespace

// ---------------------------------------------------------------- C ABI

extern "C" {

int corm_version(void) { return 100; }

const char* corm_strerror(int status) {
  switch (status) {
    case CORM_OK: return "ok";
    case CORM_EINVAL: return "invalid argument (null or misaligned pointer, bad shape, w < 1, r < 1, c < 0)";
    case CORM_EUNSUPPORTED: return "unsupported configuration (d not in {64,128}, group size not in {1,2,4,8}, dtype)";
    case CORM_ECAPACITY: return "capacity exceeded (workspace too small)";
    case CORM_EHIP: return "HIP launch failed";
    default: return "unknown status";
  }
}

int corm_workspace_bytes(const corm_desc* desc, size_t* bytes) {
  int rc = validate_desc(desc);
  if (rc) return rc;
  if (!bytes) return CORM_EINVAL;
  *bytes = workspace_layout(*desc).total;
  return CORM_OK;
}

int corm_workspace_init(const corm_desc* desc, void* workspace, size_t workspace_bytes, void* stream) {
  int rc = validate_desc(desc);
  if (rc) return rc;
  if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255u)) return CORM_EINVAL;
  const WorkspaceLayout wl = workspace_layout(*desc);
  if (workspace_bytes < wl.total) return CORM_ECAPACITY;
  const size_t n = (size_t)desc->B * desc->Hkv * wl.nsplit;
  hipLaunchKernelGGL(corm_fill_i32_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, (hipStream_t)stream,
                     reinterpret_cast<int32_t*>(reinterpret_cast<char*>(workspace) + wl.counts_off), n, 0);
  return launch_status();
}

int corm_append(const corm_desc* desc, void* K, void* V, int32_t* lens, int32_t* pos, int32_t* last_hit,
                const void* k_new, const void* v_new, const int32_t* t, int32_t* status, void* stream) {
  int rc = validate_desc(desc);
  if (rc) return rc;
  if (!K || !V || !lens || !pos || !last_hit || !k_new || !v_new || !t) return CORM_EINVAL;
  if (misaligned16(K) || misaligned16(V) || misaligned16(k_new) || misaligned16(v_new)) return CORM_EINVAL;
  if (misaligned4(lens) || misaligned4(pos) || misaligned4(last_hit) || misaligned4(t) || misaligned4(status))
    return CORM_EINVAL;
  hipLaunchKernelGGL(corm_append_kernel, dim3(desc->B * desc->Hkv), dim3(64), 0, (hipStream_t)stream,
                     reinterpret_cast<char*>(K), reinterpret_cast<char*>(V), lens, pos, last_hit,
                     reinterpret_cast<const char*>(k_new), reinterpret_cast<const char*>(v_new), t, status, desc->Hkv,
                     desc->Lcap, row_bytes(desc));
  return launch_status();
}

int corm_decode_attend(const corm_desc* desc, const void* q, const void* K, const void* V, const int32_t* lens,
                       const int32_t* pos, const int32_t* t, void* score_ring, int32_t* last_hit, float* out,
                       void* workspace, size_t workspace_bytes, int32_t* status, void* stream) {
  int rc = validate_desc(desc);
  if (rc) return rc;
  rc = check_step_pointers(q, K, V, K, V, lens, pos, last_hit, t, t, score_ring, out, nullptr, status);
  if (rc) return rc;
  WorkspaceLayout wl;
  rc = check_workspace(desc, workspace, workspace_bytes, &wl);
  if (rc) return rc;
  Params p = {};
  p.q = q; p.k_new = K; p.v_new = V;  // k_new/v_new are not read without an append; kept non-null
  p.K = const_cast<void*>(K); p.V = const_cast<void*>(V);
  p.lens = const_cast<int32_t*>(lens); p.pos = const_cast<int32_t*>(pos); p.last_hit = last_hit;
  p.t = t; p.t_first = t; p.ring = score_ring; p.out = out; p.status = status;
  p.do_append = 0; p.do_evict = 0;
  bind_params(desc, wl, workspace, p);
  return launch_attend_record(desc, p, (hipStream_t)stream);
}

int corm_evict_mask(const corm_desc* desc, const void* score_ring, const int32_t* lens, const int32_t* pos,
                    const int32_t* t, const int32_t* t_first, uint8_t* keep, void* stream) {
  int rc = validate_desc(desc);
  if (rc) return rc;
  if (!score_ring || !lens || !pos || !t || !t_first || !keep) return CORM_EINVAL;
  if (misaligned4(score_ring) || misaligned4(lens) || misaligned4(pos) || misaligned4(t) || misaligned4(t_first))
    return CORM_EINVAL;
  dim3 grid((desc->Lcap + WG - 1) / WG, desc->B * desc->Hkv);
  hipLaunchKernelGGL(corm_evict_mask_kernel, grid, dim3(WG), 0, (hipStream_t)stream, score_ring,
                     (int)desc->score_dtype, lens, pos, t, t_first, keep, desc->Hq, desc->Hkv,
                     desc->Lcap, desc->Tcap, desc->w, desc->r, desc->thr_scale);
  return launch_status();
}

int corm_evict_mask_summary(const corm_desc* desc, const int32_t* last_hit, const int32_t* lens, const int32_t* t,
                            const int32_t* t_first, uint8_t* keep, void* stream) {
  int rc = validate_desc(desc);
  if (rc) return rc;
  if (!last_hit || !lens || !t || !t_first || !keep) return CORM_EINVAL;
  if (misaligned4(last_hit) || misaligned4(lens) || misaligned4(t) || misaligned4(t_first)) return CORM_EINVAL;
  dim3 grid((desc->Lcap + WG - 1) / WG, desc->B * desc->Hkv);
  hipLaunchKernelGGL(corm_evict_mask_summary_kernel, grid, dim3(WG), 0, (hipStream_t)stream, last_hit, lens, t,
                     t_first, keep, desc->Hkv, desc->Lcap, desc->w, desc->r);
  return launch_status();
}

int corm_compact(const corm_desc* desc, void* K, void* V, int32_t* pos, int32_t* last_hit, int32_t* lens,
                 const uint8_t* keep, int32_t* kept_idx, void* workspace, size_t workspace_bytes, void* stream) {
  int rc = validate_desc(desc);
  if (rc) return rc;
  if (!K || !V || !pos || !last_hit || !lens || !keep) return CORM_EINVAL;
  if (misaligned16(K) || misaligned16(V) || misaligned4(pos) || misaligned4(last_hit) || misaligned4(lens) ||
      misaligned4(kept_idx))
    return CORM_EINVAL;
  WorkspaceLayout wl;
  rc = check_workspace(desc, workspace, workspace_bytes, &wl);
  if (rc) return rc;
  return launch_compact(desc, wl, workspace, K, V, pos, last_hit, lens, keep, kept_idx, 0, true, CompactPolicy(),
                        (hipStream_t)stream);
}

int corm_step_attend(const corm_desc* desc, const void* q, const void* k_new, const void* v_new, void* K, void* V,
                     const int32_t* lens, int32_t* pos, int32_t* last_hit, const int32_t* t, const int32_t* t_first,
                     void* score_ring, float* out, uint8_t* keep, void* workspace, size_t workspace_bytes,
                     int32_t* status, void* stream) {
  int rc = validate_desc(desc);
  if (rc) return rc;
  rc = check_step_pointers(q, k_new, v_new, K, V, lens, pos, last_hit, t, t_first, score_ring, out, nullptr, status);
  if (rc) return rc;
  WorkspaceLayout wl;
  rc = check_workspace(desc, workspace, workspace_bytes, &wl);
  if (rc) return rc;
  Params p = {};
  p.q = q; p.k_new = k_new; p.v_new = v_new; p.K = K; p.V = V; p.lens = const_cast<int32_t*>(lens); p.pos = pos;
  p.last_hit = last_hit; p.t = t; p.t_first = t_first; p.ring = score_ring; p.out = out; p.keep = keep;
  p.status = status;
  p.do_append = 1; p.do_evict = 1;
  bind_params(desc, wl, workspace, p);
  return launch_attend_record(desc, p, (hipStream_t)stream);
}

int corm_step_evict(const corm_desc* desc, void* K, void* V, int32_t* lens, int32_t* pos, int32_t* last_hit,
                    int32_t* kept_idx, void* workspace, size_t workspace_bytes, void* stream) {
  int rc = validate_desc(desc);
  if (rc) return rc;
  if (!K || !V || !pos || !last_hit || !lens) return CORM_EINVAL;
  if (misaligned16(K) || misaligned16(V) || misaligned4(pos) || misaligned4(last_hit) || misaligned4(lens) ||
      misaligned4(kept_idx))
    return CORM_EINVAL;
  WorkspaceLayout wl;
  rc = check_workspace(desc, workspace, workspace_bytes, &wl);
  if (rc) return rc;
  return launch_compact(desc, wl, workspace, K, V, pos, last_hit, lens, nullptr, kept_idx, 1, false, CompactPolicy(),
                        (hipStream_t)stream);
}

int corm_decode_step(const corm_desc* desc, const void* q, const void* k_new, const void* v_new, void* K, void* V,
                     int32_t* lens, int32_t* pos, int32_t* last_hit, const int32_t* t, const int32_t* t_first,
                     void* score_ring, float* out, uint8_t* keep, int32_t* kept_idx, void* workspace,
                     size_t workspace_bytes, int32_t* status, void* stream) {
  int rc = validate_desc(desc);
  if (rc) return rc;
  if (misaligned4(kept_idx)) return CORM_EINVAL;
  rc = corm_step_attend(desc, q, k_new, v_new, K, V, lens, pos, last_hit, t, t_first, score_ring, out, keep,
                        workspace, workspace_bytes, status, stream);
  if (rc) return rc;
  return corm_step_evict(desc, K, V, lens, pos, last_hit, kept_idx, workspace, workspace_bytes, stream);
}

int corm_decode_step_lazy(const corm_desc* desc, const void* q, const void* k_new, const void* v_new, void* K, void* V,
                          int32_t* lens, uint64_t* live, int32_t* pos, int32_t* last_hit, const int32_t* t,
                          const int32_t* t_first, void* score_ring, float* out, uint8_t* keep, int32_t* nlive,
                          int32_t dead_num, int32_t dead_den, void* workspace, size_t workspace_bytes,
                          int32_t* status, void* stream) {
  int rc = validate_desc(desc);
  if (rc) return rc;
  rc = check_step_pointers(q, k_new, v_new, K, V, lens, pos, last_hit, t, t_first, score_ring, out, nlive, status);
  if (rc) return rc;
  if (!live || (reinterpret_cast<uintptr_t>(live) & 7u)) return CORM_EINVAL;
  if (dead_num < 0 || dead_den < 1 || dead_num > dead_den) return CORM_EINVAL;
  WorkspaceLayout wl;
  rc = check_workspace(desc, workspace, workspace_bytes, &wl);
  if (rc) return rc;
  Params p = {};
  p.q = q; p.k_new = k_new; p.v_new = v_new; p.K = K; p.V = V; p.lens = lens; p.pos = pos;
  p.last_hit = last_hit; p.t = t; p.t_first = t_first; p.ring = score_ring; p.out = out; p.keep = keep;
  p.status = status;
  p.do_append = 1; p.do_evict = 1;
  bind_params(desc, wl, workspace, p);
  p.lazy = 1;
  p.keepbits = reinterpret_cast<unsigned long long*>(live);   // the live masks are read, then replaced by the new ones
  rc = launch_attend_record(desc, p, (hipStream_t)stream);
  if (rc) return rc;
  CompactPolicy pol;
  pol.lazy = 1; pol.dead_num = dead_num; pol.dead_den = dead_den;
  pol.live = reinterpret_cast<unsigned long long*>(live);
  pol.nlive = nlive;
  return launch_compact(desc, wl, workspace, K, V, pos, last_hit, lens, nullptr, nullptr, 1, false, pol,
                        (hipStream_t)stream);
}

int corm_prefill_seed(const corm_desc* desc, const void* q_tail, int32_t m, void* K, void* V, int32_t* lens,
                      int32_t* pos, int32_t* last_hit, const int32_t* t, int32_t* t_first, void* score_ring,
                      uint8_t* keep, int32_t* kept_idx, void* workspace, size_t workspace_bytes, int32_t* status,
                      void* stream) {
  int rc = validate_desc(desc);
  if (rc) return rc;
  if (!q_tail || !K || !V || !lens || !pos || !last_hit || !t || !t_first) return CORM_EINVAL;
  if (misaligned16(q_tail) || misaligned16(K) || misaligned16(V) || misaligned16(score_ring)) return CORM_EINVAL;
  if (misaligned4(lens) || misaligned4(pos) || misaligned4(last_hit) || misaligned4(t) || misaligned4(t_first) ||
      misaligned4(kept_idx) || misaligned4(status))
    return CORM_EINVAL;
  if (m < 1 || m > desc->w) return CORM_EINVAL;
  WorkspaceLayout wl;
  rc = check_workspace(desc, workspace, workspace_bytes, &wl);
  if (rc) return rc;
  char* ws = reinterpret_cast<char*>(workspace);
  hipStream_t s = (hipStream_t)stream;
  PrefillArgs a;
  a.q_tail = q_tail; a.K = K; a.lens = lens; a.pos = pos; a.last_hit = last_hit; a.t = t; a.ring = score_ring;
  a.part = reinterpret_cast<float2*>(ws + wl.seed_part_off);
  a.stats = reinterpret_cast<float4*>(ws + wl.seed_stats_off);
  a.status = status;
  a.Hq = desc->Hq; a.Hkv = desc->Hkv; a.Lcap = desc->Lcap; a.Tcap = desc->Tcap; a.w = desc->w; a.m = m;
  a.nkb = wl.seed_nkb; a.ring_bf16 = desc->score_dtype == CORM_BF16;
  a.ring_bits = desc->score_dtype == CORM_BIT; a.ring_words = (desc->Tcap + 31) / 32;
  a.thr_scale = desc->thr_scale;
  a.scale_log2 = (desc->sm_scale > 0.f ? desc->sm_scale : 1.0f / sqrtf((float)desc->d)) * LOG2E;
  const int units = desc->B * desc->Hkv;
  const dim3 grid(wl.seed_nkb, units), mgrid((m + 255) / 256, desc->B * desc->Hq);
  if (a.ring_bits && score_ring) {
    hipLaunchKernelGGL(corm_prefill_clear_bits_kernel, dim3((m + 15) / 16, desc->B * desc->Hq), dim3(256), 0, s, a);
    if (launch_status()) return CORM_EHIP;
  }
  if (desc->kv_dtype == CORM_F32)
    rc = desc->d == 64 ? launch_prefill_dt<F32, 64>(a, grid, mgrid, wl.seed_kb, s)
                       : launch_prefill_dt<F32, 128>(a, grid, mgrid, wl.seed_kb, s);
  else
    rc = desc->d == 64 ? launch_prefill_dt<BF16, 64>(a, grid, mgrid, wl.seed_kb, s)
                       : launch_prefill_dt<BF16, 128>(a, grid, mgrid, wl.seed_kb, s);
  if (rc) return rc;
  hipLaunchKernelGGL(corm_decide_kernel, dim3(wl.nsplit, units), dim3(WG), 0, s, lens, last_hit, t, t_first,
                     reinterpret_cast<unsigned long long*>(ws + wl.keepbits_off),
                     reinterpret_cast<int32_t*>(ws + wl.counts_off), keep, desc->Hkv, desc->Lcap, wl.nsplit,
                     wl.kb_stride, desc->w, desc->r, m);
  if (launch_status()) return CORM_EHIP;
  return launch_compact(desc, wl, workspace, K, V, pos, last_hit, lens, nullptr, kept_idx, 0, false, CompactPolicy(), s);
}

int corm_selected_path(const corm_desc* desc) {
  const int rc = validate_desc(desc);
  if (rc) return rc;
  return use_unit_path(desc) ? 2 : 1;
}

int corm_force_path(int path) {
  if (path < 0 || path > 3) return CORM_EINVAL;
  g_force_path = path;
  return CORM_OK;
}

int corm_profile_attend(void* start_event, void* stop_event) {
  if ((start_event == nullptr) != (stop_event == nullptr)) return CORM_EINVAL;
  g_prof_start = (hipEvent_t)start_event;
  g_prof_stop = (hipEvent_t)stop_event;
  return CORM_OK;
}

int corm_threshold(float c, const int32_t* t, int32_t n, float* thr, void* stream) {
  if (!t || !thr || n < 0 || !(c >= 0.f)) return CORM_EINVAL;
  if (n == 0) return CORM_OK;
  hipLaunchKernelGGL(corm_threshold_kernel, dim3((n + 255) / 256), dim3(256), 0, (hipStream_t)stream, c, t, n, thr);
  return launch_status();
}

}  // extern "C"
