// the fused unit kernel: append + attend + record + decide by one workgroup per unit.
// Part of one translation unit: included by corm_kernels.hip, in this order, after <hip/hip_runtime.h> and corm.h.
#ifndef CORM_UNIT_HPP
#define CORM_UNIT_HPP

namespace {

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

// UU: 16-byte K (and V) loads per lane and pipeline stage.  UNROLL for one query head per KV head.  Grouped
// queries have two instances: UNROLL (146-224 registers: one workgroup per compute unit, deep stages) for
// launches that have about one unit per compute unit anyway, and a small stage (UNROLL / G) that keeps the G
// accumulator sets and two stages within 128 registers, so that two workgroups share a compute unit, for
// launches with at least two units per compute unit.
template <typename DT, int D, int G, bool LAZY, int UU>
__global__ __launch_bounds__(UNIT_WG) void corm_unit_kernel(const Params p, const int lstride) {
  using A = Attend<DT, D, G, UNIT_WAVES, UU>;
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
  // Inside an XCD the first 32 workgroups land on its 32 compute units one each and the next 32 join them in
  // the same order (two workgroups per compute unit), so workgroups i and i + 32 of a block of 64 share a
  // compute unit and its memory pipeline.  A unit's length is a property of its head, and the same head of
  // the next sequence sits exactly 32 (or 64, ...) units further on: the plain order pairs like with like, and
  // the compute units holding two long units finish the launch alone.  Instead every block of 64 units is
  // ranked by length and the longest is paired with the shortest, the second longest with the second
  // shortest, and so on -- unless the block's lengths differ by less than an eighth, where there is nothing
  // to balance.  (A guess at the placement only costs balance, never correctness: the map is a permutation
  // of the block whatever the hardware does.)
  const int units = p.B * p.Hkv;
  const int per_xcd = (units + UNIT_XCDS - 1) / UNIT_XCDS;
  constexpr int XCD_CUS = 32, BLK = 2 * XCD_CUS;
  static_assert(BLK == 64, "one lane of a wave per unit of a block");
  const int li = (int)(blockIdx.x / UNIT_XCDS);   // index inside the XCD's range
  const int blk0 = (int)(blockIdx.x % UNIT_XCDS) * per_xcd + (li / BLK) * BLK;   // first unit of the block
  const int nblk = min(BLK, min(per_xcd - (li / BLK) * BLK, units - blk0));      // units in it
  const int jblk = li % BLK;
  if (jblk >= nblk) return;
  __shared__ int sh_unit, sh_lens;
  if (threadIdx.x < 64) {   // one wave, one unit of the block per lane
    const int k = threadIdx.x;
    int Lk = -1, raw = 0;
    if (k < nblk) {
      raw = p.lens[blk0 + k];
      Lk = raw < 0 ? 0 : (raw > p.Lcap ? p.Lcap : raw);
    }
    int lmax = Lk, lmin = k < nblk ? Lk : 0x7fffffff;
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
      lmax = max(lmax, __shfl_xor(lmax, o));
      lmin = min(lmin, __shfl_xor(lmin, o));
    }
    // A block of (nearly) equal lengths keeps the plain order: there is nothing to balance there.
    int rank = k, want = jblk;
    if ((lmax - lmin) * 8 > lmax) {   // (uniform)
      rank = 0;   // units of the block that come before this one: longer, or as long and earlier
      for (int m = 0; m < BLK; ++m) {
        const int Lm = __shfl(Lk, m);
        rank += (Lm > Lk || (Lm == Lk && m < k)) ? 1 : 0;
      }
      want = jblk < XCD_CUS ? jblk : nblk - 1 - (jblk - XCD_CUS);
    }
    if (k < nblk && rank == want) {   // exactly one lane
      sh_unit = blk0 + k;
      sh_lens = raw;
    }
  }
  __syncthreads();
  // (the same for every thread; said so explicitly, or the K and V descriptors would count as divergent)
  const int unit = __builtin_amdgcn_readfirstlane(sh_unit);
  const UnitLen ul = unit_len_of(p, __builtin_amdgcn_readfirstlane(sh_lens));
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
    if (kt * UNIT_WG < L && !p.ring_bits) {   // uniform over the workgroup (the bit-ring loop loads its own)
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
    // (rolled, so the metadata of the next tile is requested while the current one is worked on: the loop
    // must not pay one memory latency per tile)
    int pos_nx = posb[min(tid, L - 1)], lh_nx = lhb[min(tid, L - 1)];
#pragma unroll 1
    for (int tile = 0; tile < L; tile += UNIT_WG) {
      const int i = tile + tid;
      const bool live = i < L && (!LAZY || ((sh_live[i >> 6] >> (i & 63)) & 1ull));
      const int my_pos = pos_nx;
      int lh = lh_nx;
      if (tile + UNIT_WG < L) {   // (uniform; slots of the next tile: nobody writes them in this one)
        pos_nx = posb[min(i + UNIT_WG, L - 1)];
        lh_nx = lhb[min(i + UNIT_WG, L - 1)];
      }
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
    if (tid == 0) {   // tell the compaction launches, in one word, whether this unit needs them
      int T = 0;
      for (int k = 0; k < ntile; ++k) T += sh_tilecnt[k];
      if (compact_policy(LAZY, p.dead_num, p.dead_den, p.Lcap, L, T)) p.unit_dirty[unit] = dirty_tag(p.t, p.K);
    }
  }
}

}  // namespace

#endif  // CORM_UNIT_HPP
