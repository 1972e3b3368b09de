// split path, second launch: merge of the partials, record and decide.
// Part of one translation unit: included by corm_kernels.hip, in this order, after <hip/hip_runtime.h> and corm.h.
#ifndef CORM_RECORD_HPP
#define CORM_RECORD_HPP

namespace {

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
      const int chunk = rsplit * RECORD_CHUNKS + tid;
      p.counts[(size_t)unit * p.nsplit + chunk] = tot;
      // exact mode: a chunk that lost a key means the compaction launches have work (see Params::unit_dirty)
      if (!p.lazy && tot != min(CHUNK, L - chunk * CHUNK)) p.unit_dirty[unit] = dirty_tag(p.t, p.K);
    }
  }
}

}  // namespace

#endif  // CORM_RECORD_HPP
