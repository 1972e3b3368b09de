// HIP kernels (gfx950 / CDNA4, wave64) and C ABI of the CORM decode hot path: one translation unit.
//
// One decode step of one layer, on one stream, with kernel boundaries as the only cross-workgroup
// synchronization (no device-wide fences, no spinning inside the kernels):
//
//   many units (>= compute units, logits fit LDS):   unit kernel | compact local | compact boundary
//   few units:                       attend | record | compact local | compact boundary
//
//   unit     one workgroup per unit streams its K and V once, keeps the logits in LDS, writes the new
//            row (append), out (Eq. 1), the ring row and last_hit (Eq. 2, Def. 3.1), the keep masks
//            (Def. 4.1 + recent r) and the survivors per 512-slot chunk.                     unit.hpp
//   attend   grid (parts, units): online-softmax partials and raw logits per part of a unit; the
//            owner of slot lens[u] writes the new row.                                     attend.hpp
//   record   merges the partials -> out; scores, ring row, last_hit, keep masks, counts.   record.hpp
//   compact  stable in-place gather of Algorithm 1, chunk-parallel, in two launches; skipped per unit
//            when nothing was evicted, or deferred by policy (lazy mode).                 compact.hpp
//   prefill  the prompt's last w queries in one dense call (MFMA), then the bulk eviction. prefill.hpp
//
// Row geometry: a K/V row is d*sizeof(T) bytes (256 B for bf16 d=128 and fp32 d=64); each lane
// owns 16 bytes of a row, so LPR = row_bytes/16 lanes share a row and one wave-wide 16-byte
// load covers 64/LPR consecutive rows = 1 KiB of contiguous memory.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <math.h>
#include <cmath>
#include <algorithm>
#include <mutex>

#include "corm.h"

#include "common.hpp"
#include "attend.hpp"
#include "unit.hpp"
#include "record.hpp"
#include "compact.hpp"
#include "prefill.hpp"
#include "standalone.hpp"
#include "host.hpp"

// ---- corm_decode_attend_static: the attend call for callers that cannot allocate
//
// The split partials and raw logits that corm_decode_attend keeps in the caller's workspace live in this
// file-scope device array instead.  In host code the array's name is only a stand-in: its device address
// is asked for once per device (with that device current) and kept; only that address is ever used.
static __device__ __align__(256) unsigned char scratch[CORM_STATIC_SCRATCH_BYTES];

namespace {
std::mutex g_scratch_mutex;
void* g_scratch_ptr[MAX_DEVICES] = {};

// device address of `scratch` on the current device
int static_scratch(void** ptr) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess) return CORM_EHIP;
  if (dev < 0 || dev >= MAX_DEVICES) return CORM_EUNSUPPORTED;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return CORM_EHIP;
    if (reinterpret_cast<uintptr_t>(p) & 255u) return CORM_EHIP;
    g_scratch_ptr[dev] = p;
  }
  *ptr = g_scratch_ptr[dev];
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
    case CORM_ECAPACITY: return "capacity exceeded (workspace too small, or shape beyond the static scratch)";
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
                       void* workspace, size_t workspace_bytes, int32_t* status, const corm_launch_opts* opts,
                       void* stream) {
  int rc = validate_desc(desc);
  if (rc) return rc;
  rc = check_step_pointers(q, K, V, K, V, lens, pos, last_hit, t, t, score_ring, out, nullptr, status);
  if (rc) return rc;
  WorkspaceLayout wl;
  rc = check_workspace(desc, workspace, workspace_bytes, &wl);
  if (rc) return rc;
  LaunchCtx ctx;
  rc = make_ctx(opts, &ctx);
  if (rc) return rc;
  Params p = {};
  p.q = q; p.k_new = K; p.v_new = V;  // k_new/v_new are not read without an append; kept non-null
  p.K = const_cast<void*>(K); p.V = const_cast<void*>(V);
  p.lens = const_cast<int32_t*>(lens); p.pos = const_cast<int32_t*>(pos); p.last_hit = last_hit;
  p.t = t; p.t_first = t; p.ring = score_ring; p.out = out; p.status = status;
  p.do_append = 0; p.do_evict = 0;
  bind_params(desc, wl, workspace, p);
  return launch_attend_record(desc, p, ctx, (hipStream_t)stream);
}

int corm_decode_attend_static(const corm_desc* desc, const void* q, const void* K, const void* V,
                              const int32_t* lens, const int32_t* pos, const int32_t* t, void* score_ring,
                              int32_t* last_hit, float* out, int32_t* status, const corm_launch_opts* opts,
                              void* stream) {
  int rc = validate_desc(desc);
  if (rc) return rc;
  rc = check_step_pointers(q, K, V, K, V, lens, pos, last_hit, t, t, score_ring, out, nullptr, status);
  if (rc) return rc;
  // what attend + record keep in scratch memory: everything in front of the compaction's staging area
  const WorkspaceLayout wl = workspace_layout(*desc);
  if (wl.stage_meta_off > CORM_STATIC_SCRATCH_BYTES) return CORM_ECAPACITY;
  LaunchCtx ctx;
  rc = make_ctx(opts, &ctx);
  if (rc) return rc;
  void* ws = nullptr;
  rc = static_scratch(&ws);
  if (rc) return rc;
  Params p = {};
  p.q = q; p.k_new = K; p.v_new = V;
  p.K = const_cast<void*>(K); p.V = const_cast<void*>(V);
  p.lens = const_cast<int32_t*>(lens); p.pos = const_cast<int32_t*>(pos); p.last_hit = last_hit;
  p.t = t; p.t_first = t; p.ring = score_ring; p.out = out; p.status = status;
  p.do_append = 0; p.do_evict = 0;
  bind_params(desc, wl, ws, p);
  return launch_attend_record(desc, p, ctx, (hipStream_t)stream);
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

int corm_row_density(const corm_desc* desc, const void* score_ring, const int32_t* lens, const int32_t* pos,
                     const int32_t* t, float* density, void* stream) {
  int rc = validate_desc(desc);
  if (rc) return rc;
  if (!score_ring || !lens || !pos || !t || !density) return CORM_EINVAL;
  if (misaligned4(score_ring) || misaligned4(lens) || misaligned4(pos) || misaligned4(t) || misaligned4(density))
    return CORM_EINVAL;
  hipLaunchKernelGGL(corm_row_density_kernel, dim3(desc->B * desc->Hq), dim3(WG), 0, (hipStream_t)stream, score_ring,
                     (int)desc->score_dtype, lens, pos, t, density, desc->Hq, desc->Hkv, desc->Lcap, desc->Tcap,
                     desc->w, desc->thr_scale);
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
                     int32_t* status, const corm_launch_opts* opts, void* stream) {
  int rc = validate_desc(desc);
  if (rc) return rc;
  rc = check_step_pointers(q, k_new, v_new, K, V, lens, pos, last_hit, t, t_first, score_ring, out, nullptr, status);
  if (rc) return rc;
  WorkspaceLayout wl;
  rc = check_workspace(desc, workspace, workspace_bytes, &wl);
  if (rc) return rc;
  LaunchCtx ctx;
  rc = make_ctx(opts, &ctx);
  if (rc) return rc;
  Params p = {};
  p.q = q; p.k_new = k_new; p.v_new = v_new; p.K = K; p.V = V; p.lens = const_cast<int32_t*>(lens); p.pos = pos;
  p.last_hit = last_hit; p.t = t; p.t_first = t_first; p.ring = score_ring; p.out = out; p.keep = keep;
  p.status = status;
  p.do_append = 1; p.do_evict = 1;
  bind_params(desc, wl, workspace, p);
  return launch_attend_record(desc, p, ctx, (hipStream_t)stream);
}

// t: the step's t array when the attend launch of the same step maintained the workspace's dirty word (the
// compaction launches then leave at once where nothing is to be compacted); NULL: no such shortcut
static int step_evict_impl(const corm_desc* desc, void* K, void* V, int32_t* lens, int32_t* pos, int32_t* last_hit,
                           int32_t* kept_idx, void* workspace, size_t workspace_bytes, const int32_t* t, void* stream) {
  int rc = validate_desc(desc);
  if (rc) return rc;
  if (!K || !V || !pos || !last_hit || !lens) return CORM_EINVAL;
  if (misaligned16(K) || misaligned16(V) || misaligned4(pos) || misaligned4(last_hit) || misaligned4(lens) ||
      misaligned4(kept_idx))
    return CORM_EINVAL;
  WorkspaceLayout wl;
  rc = check_workspace(desc, workspace, workspace_bytes, &wl);
  if (rc) return rc;
  CompactPolicy pol;
  pol.t = t;
  return launch_compact(desc, wl, workspace, K, V, pos, last_hit, lens, nullptr, kept_idx, 1, false, pol,
                        (hipStream_t)stream);
}

int corm_step_evict(const corm_desc* desc, void* K, void* V, int32_t* lens, int32_t* pos, int32_t* last_hit,
                    int32_t* kept_idx, void* workspace, size_t workspace_bytes, void* stream) {
  return step_evict_impl(desc, K, V, lens, pos, last_hit, kept_idx, workspace, workspace_bytes, nullptr, stream);
}

int corm_decode_step(const corm_desc* desc, const void* q, const void* k_new, const void* v_new, void* K, void* V,
                     int32_t* lens, int32_t* pos, int32_t* last_hit, const int32_t* t, const int32_t* t_first,
                     void* score_ring, float* out, uint8_t* keep, int32_t* kept_idx, void* workspace,
                     size_t workspace_bytes, int32_t* status, const corm_launch_opts* opts, void* stream) {
  int rc = validate_desc(desc);
  if (rc) return rc;
  if (misaligned4(kept_idx)) return CORM_EINVAL;
  rc = corm_step_attend(desc, q, k_new, v_new, K, V, lens, pos, last_hit, t, t_first, score_ring, out, keep,
                        workspace, workspace_bytes, status, opts, stream);
  if (rc) return rc;
  return step_evict_impl(desc, K, V, lens, pos, last_hit, kept_idx, workspace, workspace_bytes, t, stream);
}

int corm_decode_step_lazy(const corm_desc* desc, const void* q, const void* k_new, const void* v_new, void* K, void* V,
                          int32_t* lens, uint64_t* live, int32_t* pos, int32_t* last_hit, const int32_t* t,
                          const int32_t* t_first, void* score_ring, float* out, uint8_t* keep, int32_t* nlive,
                          int32_t dead_num, int32_t dead_den, void* workspace, size_t workspace_bytes,
                          int32_t* status, const corm_launch_opts* opts, void* stream) {
  int rc = validate_desc(desc);
  if (rc) return rc;
  rc = check_step_pointers(q, k_new, v_new, K, V, lens, pos, last_hit, t, t_first, score_ring, out, nlive, status);
  if (rc) return rc;
  if (!live || (reinterpret_cast<uintptr_t>(live) & 7u)) return CORM_EINVAL;
  if (dead_num < 0 || dead_den < 1 || dead_num > dead_den) return CORM_EINVAL;
  WorkspaceLayout wl;
  rc = check_workspace(desc, workspace, workspace_bytes, &wl);
  if (rc) return rc;
  LaunchCtx ctx;
  rc = make_ctx(opts, &ctx);
  if (rc) return rc;
  Params p = {};
  p.q = q; p.k_new = k_new; p.v_new = v_new; p.K = K; p.V = V; p.lens = lens; p.pos = pos;
  p.last_hit = last_hit; p.t = t; p.t_first = t_first; p.ring = score_ring; p.out = out; p.keep = keep;
  p.status = status;
  p.do_append = 1; p.do_evict = 1;
  bind_params(desc, wl, workspace, p);
  p.lazy = 1;
  p.dead_num = dead_num; p.dead_den = dead_den;
  p.keepbits = reinterpret_cast<unsigned long long*>(live);   // the live masks are read, then replaced by the new ones
  rc = launch_attend_record(desc, p, ctx, (hipStream_t)stream);
  if (rc) return rc;
  CompactPolicy pol;
  pol.lazy = 1; pol.dead_num = dead_num; pol.dead_den = dead_den;
  pol.live = reinterpret_cast<unsigned long long*>(live);
  pol.nlive = nlive;
  pol.t = use_unit_path(desc, ctx) ? t : nullptr;   // (the unit kernel evaluates the policy per unit; the split kernels cannot)
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
  if ((m + 15) / 16 > 65535) return CORM_EUNSUPPORTED;   // grid rows of the clear / merge launches
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
  a.units = units;
  if ((long long)PREFILL_XCDS * ((units + PREFILL_XCDS - 1) / PREFILL_XCDS) * wl.seed_nkb > 2147483647LL)
    return CORM_EUNSUPPORTED;
  const dim3 grid((unsigned)(PREFILL_XCDS * ((units + PREFILL_XCDS - 1) / PREFILL_XCDS) * wl.seed_nkb));
  const dim3 mgrid(desc->B * desc->Hq, (m + 255) / 256);
  if (a.ring_bits && score_ring) {
    hipLaunchKernelGGL(corm_prefill_clear_bits_kernel, dim3(desc->B * desc->Hq, (m + 15) / 16), dim3(256), 0, s, a);
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

int corm_selected_path(const corm_desc* desc, const corm_launch_opts* opts) {
  int rc = validate_desc(desc);
  if (rc) return rc;
  LaunchCtx ctx;
  rc = make_ctx(opts, &ctx);
  if (rc) return rc;
  return use_unit_path(desc, ctx) ? 2 : 1;
}

int corm_threshold(float c, const int32_t* t, int32_t n, float* thr, void* stream) {
  if (!t || !thr || n < 0 || !(c >= 0.f)) return CORM_EINVAL;
  if (n == 0) return CORM_OK;
  hipLaunchKernelGGL(corm_threshold_kernel, dim3((n + 255) / 256), dim3(256), 0, (hipStream_t)stream, c, t, n, thr);
  return launch_status();
}

}  // extern "C"
