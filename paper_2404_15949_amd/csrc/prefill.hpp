// prompt seeding: the dense [m x L] causal rows on the matrix cores, merge, decision.
// Part of one translation unit: included by corm_kernels.hip, in this order, after <hip/hip_runtime.h> and corm.h.
#ifndef CORM_PREFILL_HPP
#define CORM_PREFILL_HPP

namespace {

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
// operand in the same layout, read from LDS, where the workgroup stages the queries in double-buffered
// blocks.  D: lane l holds query l%16, keys 4*(l/16) .. +3 of the tile.

constexpr int PREFILL_XCDS = 8;   // accelerator dies of the device

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
  int32_t units;                   // B * Hkv
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

constexpr int PREFILL_SEG = 512;   // queries whose pass-1 partials a workgroup holds in LDS at a time

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
__device__ __forceinline__ void prefill_pass(const PrefillArgs& a) {
  constexpr int ROWB = D * DT::ESZ;
  using Geo = PrefillGeom<ROWB>;
  constexpr int NCH = Geo::NCH, T = Geo::T, KB = Geo::KB;
  constexpr int NEVER = 0x7fffffff;   // position of a slot that holds no key: visible to no query

  // One-dimensional grid of 8 * ceil(units / 8) * nkb workgroups.  Workgroups are dealt round-robin to the 8
  // XCDs, so id % 8 names the XCD; each XCD takes a contiguous range of units and runs the key blocks of a unit
  // one after the other: they all read the same tail queries, which then stay in that XCD's L2.
  const int per_xcd = (a.units + PREFILL_XCDS - 1) / PREFILL_XCDS;
  const int li = (int)(blockIdx.x / PREFILL_XCDS);
  const int unit = (int)(blockIdx.x % PREFILL_XCDS) * per_xcd + li / a.nkb;
  const int kb = li % a.nkb;
  if (li / a.nkb >= per_xcd || unit >= a.units) return;
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
                __builtin_nontemporal_store(u32x4_t{v.x, v.y, v.z, v.w}, reinterpret_cast<u32x4_t*>(dst));
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

// Pass 1 has a light tail (max, exp, sum) and is latency-bound at two waves per SIMD: held to the registers
// and LDS of three (0.91 -> 0.64 ms per layer on config 3).  Pass 2 needs its registers.
template <typename DT, int D>
__global__ __launch_bounds__(WG) __attribute__((amdgpu_waves_per_eu(3, 3))) void corm_prefill_stats_kernel(
    const PrefillArgs a) {
  prefill_pass<DT, D, 1, false>(a);
}

template <typename DT, int D, bool BITS>
__global__ __launch_bounds__(WG) void corm_prefill_scores_kernel(const PrefillArgs a) {
  prefill_pass<DT, D, 2, BITS>(a);
}

// boolean message: zero the words of the rows of steps tau_0 .. tau_{m-1} that pass 2 may set bits in
// (positions < tau); workgroup = 16 rows of one head
__global__ __launch_bounds__(256) void corm_prefill_clear_bits_kernel(const PrefillArgs a) {
  const int head = blockIdx.x;   // (heads in x: B * Hq may exceed the 65535 rows a grid has in y)
  const int tcur = a.t[head / a.Hq];
  const int tau0 = tcur - a.m + 1;
  if (tau0 < 1 || tcur > a.Tcap) return;
  const int s0 = (tau0 - 1) % a.w;
  for (int jr = 0; jr < 16; ++jr) {
    const int j = blockIdx.y * 16 + jr;
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
  const int head = blockIdx.x;   // (heads in x: B * Hq may exceed the 65535 rows a grid has in y)
  const int j = blockIdx.y * 256 + threadIdx.x;
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

}  // namespace

#endif  // CORM_PREFILL_HPP
