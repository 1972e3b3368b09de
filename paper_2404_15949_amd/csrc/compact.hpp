// stable in-place compaction: count, local and boundary launches.
// Part of one translation unit: included by corm_kernels.hip, in this order, after <hip/hip_runtime.h> and corm.h.
#ifndef CORM_COMPACT_HPP
#define CORM_COMPACT_HPP

namespace {

// ---------------------------------------------------------------- stable in-place compaction
//
// Survivor number rho of a unit (in slot order) must end in slot rho.  Two launches, no
// cross-workgroup synchronization inside either:
//
//   local     grid (splits, units).  R_c = survivors before chunk c (from the per-split counts).
//             The workgroup of chunk c = slots [a_c, a_c + CHUNK) moves its survivors with rho >= a_c
//             to slot rho -- inside its own chunk, so it reads and writes only its own slots -- in
//             ascending batches (every destination <= its source; inside a batch all loads complete
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

// The local launch runs one thread per slot of a chunk: a chunk is scanned in one step and its rows are requested
// 64 to 256 at a time (four passes of the workgroup), so a unit that lost a single key (the common case of a
// dense cache) costs a few memory latencies.
constexpr int CWG = CHUNK;
constexpr int CWAVES = CWG / 64;

struct CompactShared {
  int32_t wave_count[CWAVES];
  int32_t first_hole;   // first slot of the chunk (relative) that does not survive
  int32_t src_of[CWG];
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
  const int32_t* unit_dirty;     // optional (with t) [units]: a value other than dirty_tag(t, K) means the unit is not compacted
  const int32_t* t;
};

// The unit does not have to be compacted (told by the step launch before, in one word): only its first
// workgroup still has the bookkeeping to do (the unit's length, lens, the live count).
__device__ __forceinline__ bool nothing_to_compact(const CompactArgs& a, int unit) {
  return a.unit_dirty != nullptr && a.unit_dirty[unit] != dirty_tag(a.t, a.K);
}

__device__ __forceinline__ bool compact_now(const CompactArgs& a, int L, int T) {
  return compact_policy(a.lazy, a.dead_num, a.dead_den, a.Lcap, L, T);
}

// Moves the n_rows survivors listed in src_of (ascending) to consecutive destinations starting at
// survivor number rho0: slot rho if rho >= own_begin, else staging row (rho - stage_rho0).  Every destination
// is <= its source; all loads of a batch complete before any of its stores.
template <int ROWB>
__device__ __forceinline__ void move_rows(char* Kb, char* Vb, char* sk, char* sv, const int32_t* src_of, int n_rows,
                                          int rho0, int own_begin, int stage_rho0) {
  constexpr int LPR = ROWB / 16;
  constexpr int RPP = CWG / LPR;  // rows per pass of the workgroup
  // Four passes in flight together, in named registers (an indexed array would be demoted to scratch).  Eight
  // (94 registers, two workgroups per compute unit) moved a full launch 2 % faster and made the launches that
  // find nothing to do slower: the workgroups that only look at their unit's word then come in more rounds.
  constexpr int NP = 4;
  const int tid = threadIdx.x;
  const int sub = tid / LPR;
  const size_t col = (size_t)(tid % LPR) * 16;
  const int last = n_rows - 1;
  for (int base = 0; base < n_rows; base += RPP * NP) {
    // clamped row numbers: every load reads a valid row, stores are predicated
#define CORM_LOAD_ROW(U)                                                                          \
    const size_t o##U = (size_t)src_of[min(base + sub + (U) * RPP, last)] * ROWB + col;            \
    const uint4 k##U = *reinterpret_cast<const uint4*>(Kb + o##U);                                \
    const uint4 v##U = *reinterpret_cast<const uint4*>(Vb + o##U);
    CORM_LOAD_ROW(0) CORM_LOAD_ROW(1) CORM_LOAD_ROW(2) CORM_LOAD_ROW(3)
#undef CORM_LOAD_ROW
    wait_vm_loads();
    __syncthreads();
#define CORM_STORE_ROW(U)                                                      \
    {                                                                            \
      const int j = base + sub + (U) * RPP;                                      \
      if (j < n_rows) {                                                          \
        const int rho = rho0 + j;                                                \
        if (rho >= own_begin) {                                                  \
          const size_t d = (size_t)rho * ROWB + col;                             \
          *reinterpret_cast<uint4*>(Kb + d) = k##U;                              \
          *reinterpret_cast<uint4*>(Vb + d) = v##U;                              \
        } else {                                                                 \
          const size_t d = (size_t)(rho - stage_rho0) * ROWB + col;              \
          *reinterpret_cast<uint4*>(sk + d) = k##U;                              \
          *reinterpret_cast<uint4*>(sv + d) = v##U;                              \
        }                                                                        \
      }                                                                          \
    }
    CORM_STORE_ROW(0) CORM_STORE_ROW(1) CORM_STORE_ROW(2) CORM_STORE_ROW(3)
#undef CORM_STORE_ROW
  }
  static_assert(NP == 4, "four named passes");
}

// The scan of a chunk.  keep: this thread's flag (0 for slots >= L).  Returns this thread's rank among the
// chunk's survivors and their number (via *kept).
__device__ __forceinline__ int chunk_scan(bool keep, CompactShared& sh, int* kept) {
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
  const unsigned long long bal = __ballot(keep);
  const int rank = __popcll(bal & ((1ull << lane) - 1ull));
  if (lane == 0) sh.wave_count[wv] = __popcll(bal);
  __syncthreads();
  int before = 0, total = 0;
#pragma unroll
  for (int i = 0; i < CWAVES; ++i) {
    const int c = sh.wave_count[i];
    if (i < wv) before += c;
    total += c;
  }
  *kept = total;
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
__global__ __launch_bounds__(CWG) void corm_compact_local_kernel(const CompactArgs a) {
  __shared__ CompactShared sh_c;
  const int split = blockIdx.x, unit = blockIdx.y;
  const int tid = threadIdx.x;
  if (split != 0 && nothing_to_compact(a, unit)) return;
  const int L = compact_unit_len(a, unit);
  if (split == 0 && tid == 0) a.unit_len[unit] = L;
  // (a unit that is not compacted: handing its length on was all its first workgroup had to do; lens and the unit's
  // word are loaded together, nothing waits for the counts)
  if (split == 0 && nothing_to_compact(a, unit)) return;
  const int nlive = (L + CHUNK - 1) / CHUNK;
  if (split >= nlive) return;
  const int32_t* cnt = a.counts + (size_t)unit * a.nsplit;
  int R, T;   // survivors before this chunk, survivors of the unit
  unit_counts(cnt, nlive, split, &R, &T);
  int32_t* idxb = a.kept_idx ? a.kept_idx + (size_t)unit * a.Lcap : nullptr;
  const int cbeg = split * CHUNK;
  const int cend = min(cbeg + CHUNK, L);
  const int i = cbeg + tid;   // this thread's slot
  if (!compact_now(a, L, T)) {   // nothing evicted, or (lazy mode) not enough dead slots yet
    if (idxb && T == L && i < cend) idxb[i] = i;
    return;
  }
  const int my_cnt = cnt[split];
  if (R == cbeg && my_cnt == cend - cbeg) {   // no hole before or inside this chunk
    if (idxb && i < cend) idxb[i] = i;
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

  const bool kp = i < cend && (chunk_full || ((bitsb[i >> 6] >> (i & 63)) & 1ull) != 0);
  int my_pos = 0, my_lh = 0;
  if (kp) {
    my_pos = posb[i];
    my_lh = lhb[i];
  }
  if (tid == 0) sh_c.first_hole = CWG;
  wait_vm_loads();
  int kept;
  const int rank = chunk_scan(kp, sh_c, &kept);
  const int rho = R + rank;   // survivor number of this thread's key
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
  } else if (i < cend) {
    atomicMin(&sh_c.first_hole, tid);
  }
  __syncthreads();
  // with no hole before the chunk, the survivors in front of its first hole already lie where they belong
  const int fixed = R == cbeg ? min(sh_c.first_hole, kept) : 0;
  move_rows<ROWB>(Kb, Vb, sk, sv, sh_c.src_of + fixed, kept - fixed, R + fixed, cbeg, R);
}

template <int ROWB>
__global__ __launch_bounds__(WG) void corm_compact_boundary_kernel(const CompactArgs a) {
  constexpr int LPR = ROWB / 16;
  const int split = blockIdx.x, unit = blockIdx.y;
  const int tid = threadIdx.x;
  if (split != 0 && nothing_to_compact(a, unit)) return;
  const int L = a.unit_len[unit];
  if (split == 0 && !a.nlive && nothing_to_compact(a, unit)) {   // not compacted and nobody asks for the live count
    if (tid == 0) a.lens[unit] = L;
    return;
  }
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

}  // namespace

#endif  // CORM_COMPACT_HPP
