// split path, first launch: the attend kernels (vector-ALU dot, and q.K^T on MFMA for grouped bf16 queries).
// Part of one translation unit: included by corm_kernels.hip, in this order, after <hip/hip_runtime.h> and corm.h.
#ifndef CORM_ATTEND_HPP
#define CORM_ATTEND_HPP

namespace {

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

// The same with the non-temporal cache policy (the `nt` bit of the instruction): for the K and V rows of
// a decode step, which are read exactly once per launch and not again before gigabytes of other rows have
// passed.  Measured on the unit kernel (config 3 shape): 207 -> 186 us per launch.
__device__ __forceinline__ uint4 buffer_load16_stream(__amdgpu_buffer_rsrc_t r, uint32_t byte_offset) {
  const u32x4_t v = __builtin_amdgcn_raw_buffer_load_b128(r, (int)byte_offset, 0, 2);
  return make_uint4(v.x, v.y, v.z, v.w);
}

// byte offset beyond any descriptor: the load returns zeros without touching memory
constexpr uint32_t DEAD_OFFSET = 0x7ffffff0u;

// 2^x by the hardware instruction alone (results below the normal range flush to zero: such
// probabilities vanish against a sum that is >= 1)
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

template <typename DT, int D, int G, int NW, int UU = UNROLL>
struct Attend {
  static constexpr int EPL = DT::EPL;
  static constexpr int ROWB = D * DT::ESZ;
  static constexpr int LPR = ROWB / 16;   // lanes per row
  static constexpr int RPL = 64 / LPR;    // rows per wave-wide load
  static constexpr int U = UU;          // 16-byte K loads (and V loads) per lane and pipeline stage
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
      st.k[j] = buffer_load16_stream(rk, o);
    }
#pragma unroll
    for (int j = 0; j < U; ++j) {
      const uint32_t o = (!LAZY || ((st.live >> j) & 1u)) ? off + (uint32_t)(j * LOAD_ROWS * ROWB) : DEAD_OFFSET;
      st.v[j] = buffer_load16_stream(rv, o);
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
// K and V are both loaded in the row layout (lane l: row l/16 of a load, 16-byte column slice l%16, so
// 16 lanes read one whole 256-byte row and a load covers four full rows).  The A operand of
// v_mfma_f32_16x16x32_bf16 wants lane l to hold key l%16, elements 32*kb + 8*(l/16) .. +8 of block kb;
// loading K that way straight from memory would fetch 64-byte pieces of 16 rows per instruction (half
// cache lines: measurably slower), so the tile takes a turn through a wave-private 4 KiB LDS tile
// instead, its 16-byte pieces XOR-swizzled by the row so that neither the writes nor the reads
// conflict.  The G queries sit in columns 0..G-1 of the B operand (the other columns are zero), and
// four MFMAs give the 16 x G logits of the tile without any cross-lane reduction: lane (n = l%16 < G,
// lg = l/16) holds the logits of head n for keys 4*lg .. 4*lg+3.  The softmax bookkeeping runs in those
// lanes (all heads at once), the probabilities go through a per-wave LDS tile to the lanes that hold V,
// and p.V stays on the vector ALU.

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));

template <int G>
struct AttendGqa {
  static constexpr int D = 128, ROWB = 256, EPL = 8;
  static constexpr int TILE = 16;                    // keys per wave and stage
  static constexpr int STAGE_ROWS = WAVES * TILE;    // keys per workgroup and stage

  struct Stage {
    uint4 k[4];  // rows 4*j + lane/16 of the tile, this lane's 16-byte column slice
    uint4 v[4];  // the same rows and slice of V
    uint32_t live;   // lazy mode: bit i = key i of the tile is live
  };

  // Lazy mode: sh_live holds the live masks (LDS), trow is the tile's first key relative to the first
  // slot sh_live covers (a multiple of 16); the loads of dead keys get an out-of-range offset.
  template <bool LAZY>
  __device__ static __forceinline__ void load(Stage& st, __amdgpu_buffer_rsrc_t rk, __amdgpu_buffer_rsrc_t rv,
                                              uint32_t off, const unsigned long long* sh_live, int trow,
                                              int lg) {
    st.live = 0xffffu;
    if (LAZY) st.live = (uint32_t)(sh_live[trow >> 6] >> (trow & 63)) & 0xffffu;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const bool rlive = !LAZY || ((st.live >> (4 * j + lg)) & 1u);
      st.k[j] = buffer_load16_stream(rk, rlive ? off + (uint32_t)(j * 4 * ROWB) : DEAD_OFFSET);
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const bool rlive = !LAZY || ((st.live >> (4 * j + lg)) & 1u);
      st.v[j] = buffer_load16_stream(rv, rlive ? off + (uint32_t)(j * 4 * ROWB) : DEAD_OFFSET);
    }
  }

  // row0: first key of this wave's tile; lrel0: its index in the logit staging array;
  // sh_kt: this wave's 16 x 16 tile of 16-byte pieces (piece c of key r at [r][c ^ (r & 7)])
  __device__ static __forceinline__ void compute(const Stage& st, int row0, int lrel0, int cend, int n, int lg,
                                                 const uint4 (&qb)[4], float scale_log2, float* sh_logit,
                                                 int lstride, uint4* sh_kt, float* sh_p, float* sh_alpha,
                                                 float& m_run, float& z_run, float (&acc)[G][EPL]) {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int r = 4 * j + lg;
      sh_kt[r * 16 + (n ^ (r & 7))] = st.k[j];
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");   // LDS is in order within a wave: compiler fence only
    f32x4_t d = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int kb = 0; kb < 4; ++kb) {
      const uint4 a = sh_kt[n * 16 + ((4 * kb + lg) ^ (n & 7))];   // key n, elements 32*kb + 8*lg .. +8
      d = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, a),
                                                  __builtin_bit_cast(bf16x8_t, qb[kb]), d, 0, 0, 0);
    }
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
__global__ __launch_bounds__(WG) __attribute__((amdgpu_waves_per_eu(G <= 4 ? 3 : 2)))
void corm_attend_gqa_kernel(const Params p) {
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
  __shared__ uint4 sh_kt[WAVES][A::TILE * 16];
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
  const uint32_t off = (uint32_t)(tile0 + lg) * ROWB + (uint32_t)(16 * n);
  constexpr uint32_t STAGE_BYTES = (uint32_t)A::STAGE_ROWS * ROWB;
  constexpr int PAIRS = CHUNK / (2 * A::STAGE_ROWS);
  static_assert(PAIRS >= 1 && CHUNK % (2 * A::STAGE_ROWS) == 0, "CHUNK must hold whole stage pairs");

  typename A::Stage s0, s1;
  A::template load<LAZY>(s0, rk, rv, off, sh_live, wv * A::TILE, lg);
#pragma unroll
  for (int i = 0; i < PAIRS; ++i) {
    const int it = cbeg + i * 2 * A::STAGE_ROWS;
    if (it >= cend) break;
    A::template load<LAZY>(s1, rk, rv, off + (uint32_t)(2 * i + 1) * STAGE_BYTES, sh_live,
                           (2 * i + 1) * A::STAGE_ROWS + wv * A::TILE, lg);
    A::compute(s0, it + wv * A::TILE, it - cbeg + wv * A::TILE, cend, n, lg, qb, p.scale_log2, &sh_logit[0][0],
               CHUNK, sh_kt[wv], sh_p[wv], sh_alpha[wv], m_run, z_run, acc);
    if (i + 1 < PAIRS)
      A::template load<LAZY>(s0, rk, rv, off + (uint32_t)(2 * i + 2) * STAGE_BYTES, sh_live,
                             (2 * i + 2) * A::STAGE_ROWS + wv * A::TILE, lg);
    A::compute(s1, it + A::STAGE_ROWS + wv * A::TILE, it - cbeg + A::STAGE_ROWS + wv * A::TILE, cend, n, lg, qb,
               p.scale_log2, &sh_logit[0][0], CHUNK, sh_kt[wv], sh_p[wv], sh_alpha[wv], m_run, z_run, acc);
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

}  // namespace

#endif  // CORM_ATTEND_HPP
