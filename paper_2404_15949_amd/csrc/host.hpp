// host side: workspace layout, validation, path selection and launches.
// Part of one translation unit: included by corm_kernels.hip, in this order, after <hip/hip_runtime.h> and corm.h.
#ifndef CORM_HOST_HPP
#define CORM_HOST_HPP

namespace {

// ---------------------------------------------------------------- host side

struct WorkspaceLayout {
  size_t counts_off, unit_len_off, dirty_off, keepbits_off, partials_off, logits_off, stage_meta_off, stage_k_off, stage_v_off;
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
  w.dirty_off = w.unit_len_off + units * sizeof(int32_t);   // one word per unit: see Params::unit_dirty
  w.keepbits_off = align_up(w.dirty_off + units * sizeof(int32_t), 256);
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

// Per-call launch context: what corm_launch_opts asks for, plus the compute-unit count of the current
// device.  Nothing here outlives the call.
struct LaunchCtx {
  int path = 0;                               // 0 = choose by shape, 1 = split kernels (attend + record), 2 = fused
                                              // unit kernel, 3 = split kernels with q.K^T on the vector ALU even
                                              // where the MFMA kernel applies
  hipEvent_t ev0 = nullptr, ev1 = nullptr;    // recorded around the launch that streams K and V
  int cus = 256;
};

// Compute units of the current device, asked once per device (thread safe); 256 where no device answers.
constexpr int MAX_DEVICES = 64;
std::mutex g_device_mutex;
int g_device_cus[MAX_DEVICES] = {};

int device_cus() {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) return 256;
  std::lock_guard<std::mutex> lock(g_device_mutex);
  if (g_device_cus[dev] == 0) {
    int n = 0;
    if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) n = 256;
    g_device_cus[dev] = n;
  }
  return g_device_cus[dev];
}

int make_ctx(const corm_launch_opts* o, LaunchCtx* c) {
  *c = LaunchCtx();
  if (o) {
    if (o->path < 0 || o->path > 3) return CORM_EINVAL;
    if ((o->attend_start_event == nullptr) != (o->attend_stop_event == nullptr)) return CORM_EINVAL;
    c->path = o->path;
    c->ev0 = (hipEvent_t)o->attend_start_event;
    c->ev1 = (hipEvent_t)o->attend_stop_event;
  }
  c->cus = device_cus();
  return CORM_OK;
}

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
  p.unit_dirty = reinterpret_cast<int32_t*>(ws + wl.dirty_off);
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
int launch_attend_dt(const corm_desc* d, const Params& p, const LaunchCtx& c, int G, dim3 grid, hipStream_t s) {
  if (d->kv_dtype == CORM_F32)
    return d->d == 64 ? launch_attend_g<F32, 64, LAZY>(p, G, grid, s) : launch_attend_g<F32, 128, LAZY>(p, G, grid, s);
  // grouped queries, bf16, d = 128: q.K^T on the matrix cores
  if (d->d == 128 && G > 1 && c.path != 3) return launch_attend_gqa<LAZY>(p, G, grid, s);
  return d->d == 64 ? launch_attend_g<BF16, 64, LAZY>(p, G, grid, s) : launch_attend_g<BF16, 128, LAZY>(p, G, grid, s);
}

int launch_attend(const corm_desc* d, const Params& p, const LaunchCtx& c, hipStream_t s) {
  const int G = d->Hq / d->Hkv;
  const dim3 grid((d->Lcap + p.part_keys - 1) / p.part_keys, d->B * d->Hkv);
  if (c.ev0 && hipEventRecord(c.ev0, s) != hipSuccess) return CORM_EHIP;
  const int rc = p.lazy ? launch_attend_dt<true>(d, p, c, G, grid, s) : launch_attend_dt<false>(d, p, c, G, grid, s);
  if (rc) return rc;
  if (c.ev1 && hipEventRecord(c.ev1, s) != hipSuccess) return CORM_EHIP;
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
bool use_unit_path(const corm_desc* d, const LaunchCtx& c) {
  int lstride;
  const bool fits = unit_lds_bytes(d, &lstride) <= 48 * 1024 && d->Hq / d->Hkv <= 4;  // G = 8 exceeds the register file
  if (c.path == 1 || c.path == 3 || !fits) return false;
  if (c.path == 2) return true;
  return d->B * d->Hkv >= c.cus;
}

template <typename DT, int D, bool LAZY>
int launch_unit_g(const Params& p, const LaunchCtx& c, int G, int units, size_t lds, int lstride, hipStream_t s) {
  // grouped queries: the small-stage instance (two workgroups per compute unit) once there are two units per
  // compute unit; measured on 32 query / 8 KV heads: 1024 units 161 -> 134 us per step, 512 units 139 -> 133 us,
  // but 256 units 81 -> 91 us
  const bool small = (long)p.B * p.Hkv >= 2L * c.cus;
  const dim3 grid(units), wg(UNIT_WG);
  switch (G) {
    case 1: hipLaunchKernelGGL((corm_unit_kernel<DT, D, 1, LAZY, UNROLL>), grid, wg, lds, s, p, lstride); break;
    case 2:
      if (small) hipLaunchKernelGGL((corm_unit_kernel<DT, D, 2, LAZY, UNROLL / 2>), grid, wg, lds, s, p, lstride);
      else hipLaunchKernelGGL((corm_unit_kernel<DT, D, 2, LAZY, UNROLL>), grid, wg, lds, s, p, lstride);
      break;
    case 4:
      if (small) hipLaunchKernelGGL((corm_unit_kernel<DT, D, 4, LAZY, UNROLL / 4>), grid, wg, lds, s, p, lstride);
      else hipLaunchKernelGGL((corm_unit_kernel<DT, D, 4, LAZY, UNROLL>), grid, wg, lds, s, p, lstride);
      break;
    default: return CORM_EUNSUPPORTED;
  }
  return launch_status();
}

template <bool LAZY>
int launch_unit_dt(const corm_desc* d, const Params& p, const LaunchCtx& c, int G, int units, size_t lds, int lstride,
                   hipStream_t s) {
  if (d->kv_dtype == CORM_F32)
    return d->d == 64 ? launch_unit_g<F32, 64, LAZY>(p, c, G, units, lds, lstride, s)
                      : launch_unit_g<F32, 128, LAZY>(p, c, G, units, lds, lstride, s);
  return d->d == 64 ? launch_unit_g<BF16, 64, LAZY>(p, c, G, units, lds, lstride, s)
                    : launch_unit_g<BF16, 128, LAZY>(p, c, G, units, lds, lstride, s);
}

int launch_unit(const corm_desc* d, const Params& p, const LaunchCtx& c, hipStream_t s) {
  int lstride;
  const size_t lds = unit_lds_bytes(d, &lstride);
  const int G = d->Hq / d->Hkv;
  const int units = (d->B * d->Hkv + UNIT_XCDS - 1) / UNIT_XCDS * UNIT_XCDS;   // grid: whole rounds over the XCDs
  if (c.ev0 && hipEventRecord(c.ev0, s) != hipSuccess) return CORM_EHIP;
  const int rc = p.lazy ? launch_unit_dt<true>(d, p, c, G, units, lds, lstride, s)
                        : launch_unit_dt<false>(d, p, c, G, units, lds, lstride, s);
  if (rc) return rc;
  if (c.ev1 && hipEventRecord(c.ev1, s) != hipSuccess) return CORM_EHIP;
  return CORM_OK;
}

// append (if p.do_append) + attend + record: one fused launch or the attend / record pair
int launch_attend_record(const corm_desc* d, const Params& p, const LaunchCtx& c, hipStream_t s);

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

int launch_record(const corm_desc* d, const Params& p, const LaunchCtx& c, hipStream_t s) {
  // the largest workgroup that still leaves about four workgroups per compute unit
  const long units = (long)d->B * d->Hkv;
  const long want = 4L * c.cus;
  if (units * ((p.nsplit + 3) / 4) >= want) return launch_record_rc<4>(d, p, s);
  if (units * ((p.nsplit + 1) / 2) >= want) return launch_record_rc<2>(d, p, s);
  return launch_record_rc<1>(d, p, s);
}

// Keys per attend workgroup on the split path: a whole chunk, or a half / a quarter of one while the
// launch would otherwise have fewer than about two workgroups per compute unit.  A part must hold whole
// pairs of pipeline stages of the kernel that runs.
int attend_part_keys(const corm_desc* d, const LaunchCtx& c) {
  const int G = d->Hq / d->Hkv;
  const bool mfma = d->kv_dtype == CORM_BF16 && d->d == 128 && G > 1 && c.path != 3;
  const int stage_rows = mfma ? WAVES * 16 : WAVES * (64 / (row_bytes(d) / 16)) * UNROLL;
  const long want = 2L * c.cus;
  const long wgs = (long)d->B * d->Hkv * ((d->Lcap + CHUNK - 1) / CHUNK);
  int part = CHUNK;
  while (part / 2 >= 2 * stage_rows && CHUNK / (part / 2) <= MAX_PARTS_PER_CHUNK && wgs * (CHUNK / part) < want) part /= 2;
  return part;
}

int launch_attend_record(const corm_desc* d, const Params& p0, const LaunchCtx& c, hipStream_t s) {
  if (use_unit_path(d, c)) return launch_unit(d, p0, c, s);
  Params p = p0;
  p.part_keys = attend_part_keys(d, c);
  const int rc = launch_attend(d, p, c, s);
  if (rc) return rc;
  return launch_record(d, p, c, s);
}

// Policy of the compaction launches: exact mode compacts every unit that lost a key; lazy mode only
// units whose dead slots reach dead_num / dead_den of their slots.
struct CompactPolicy {
  int lazy = 0, dead_num = 0, dead_den = 1;
  unsigned long long* live = nullptr;   // lazy mode: the caller's live masks take the place of the keep masks
  int32_t* nlive = nullptr;             // optional output: live keys per unit
  const int32_t* t = nullptr;           // the step's t array, if the launch before maintains the workspace's dirty words
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
  // (a caller who wants kept_idx gets the identity written for untouched units: every workgroup has work then)
  a.unit_dirty = pol.t && !kept_idx ? reinterpret_cast<const int32_t*>(ws + wl.dirty_off) : nullptr;
  a.t = pol.t;
  const dim3 grid(wl.nsplit, d->B * d->Hkv);
  if (count_first) {
    hipLaunchKernelGGL(corm_count_kernel, grid, dim3(WG), 0, s, a, counts);
    if (launch_status()) return CORM_EHIP;
  }
  switch (row_bytes(d)) {
    case 128:
      hipLaunchKernelGGL((corm_compact_local_kernel<128>), grid, dim3(CWG), 0, s, a);
      hipLaunchKernelGGL((corm_compact_boundary_kernel<128>), grid, dim3(WG), 0, s, a);
      break;
    case 256:
      hipLaunchKernelGGL((corm_compact_local_kernel<256>), grid, dim3(CWG), 0, s, a);
      hipLaunchKernelGGL((corm_compact_boundary_kernel<256>), grid, dim3(WG), 0, s, a);
      break;
    case 512:
      hipLaunchKernelGGL((corm_compact_local_kernel<512>), grid, dim3(CWG), 0, s, a);
      hipLaunchKernelGGL((corm_compact_boundary_kernel<512>), grid, dim3(WG), 0, s, a);
      break;
    default: return CORM_EUNSUPPORTED;
  }
  return launch_status();
}

template <typename DT, int D>
int launch_prefill_dt(const PrefillArgs& a, dim3 grid, dim3 mgrid, int KB, hipStream_t s) {
  hipLaunchKernelGGL((corm_prefill_stats_kernel<DT, D>), grid, dim3(WG), 0, s, a);
  hipLaunchKernelGGL(corm_prefill_merge_kernel, mgrid, dim3(256), 0, s, a, KB);
  if (a.ring_bits) hipLaunchKernelGGL((corm_prefill_scores_kernel<DT, D, true>), grid, dim3(WG), 0, s, a);
  else hipLaunchKernelGGL((corm_prefill_scores_kernel<DT, D, false>), grid, dim3(WG), 0, s, a);
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

#endif  // CORM_HOST_HPP
