/*
 * corm.h -- C ABI of the MI355X (gfx950) decode hot path of CORM
 * ("Cache Optimization with Recent Message", arXiv 2404.15949).
 *
 * One decode step, per layer, for every (sequence b, KV head h) "unit":
 *   append  k_t, v_t                         (shapes of Algorithm 1: keys [l,d] include the current token)
 *   attend  out = softmax(q K^T / sqrt(d)) V (Eq. 1) over the l LIVE keys of the unit only,
 *           alpha_{t,i} the normalized scores (Eq. 2)
 *   record  the scores of this query into row (t-1) mod w of a ring of the last w queries
 *           (Section 4.2 "Approach": a recent window of size w records what each query finds important)
 *   evict   a key survives iff some recorded query of the window (any query head of its group,
 *           Section 5.3) gave it a score >= c/t_j (Def. 3.1, c = 1), or it is among the r newest
 *           slots (Def. 4.1 and the recent-r protection of Section 4.2); nothing is evicted
 *           while fewer than w rows are recorded (Algorithm 1)
 *   compact K, V (and the per-key metadata) are gathered in ascending slot order
 *           (the nonzero()/index step of Algorithm 1): a STABLE stream compaction.
 *
 * Conventions
 * -----------
 * Every pointer is a DEVICE pointer to caller-owned memory unless it says "host".  The library
 * allocates and frees nothing; scratch lives in a caller-provided workspace (one call,
 * corm_decode_attend_static, keeps it in a device array of the library instead).  Calls are
 * asynchronous on `stream` (a hipStream_t passed as void*, NULL = the default stream) and never
 * synchronize.  Every call returns 0 (CORM_OK) or a negative corm_status; argument errors are
 * detected on the host before anything is launched.  Conditions only the device can see
 * (a full unit, a step beyond the ring's columns) never fault: the kernel skips the offending
 * write and ORs a bit into the optional `status` word.
 * Calls that overlap in time (other streams, other host threads) need a workspace each and must not share
 * any array a call writes; beyond that the library keeps no mutable state: what a call does depends on its
 * arguments alone (the only things remembered are, per device, the number of compute units and the address
 * of the static scratch array, both looked up once under a lock), so every call may be made from any thread.
 *
 * Layouts (row-major, sizes in elements)
 *   q              [B, Hq, d]            kv_dtype        query of the current token per head
 *   k_new, v_new   [B, Hkv, d]           kv_dtype        key/value of the current token
 *   K, V           [B, Hkv, Lcap, d]     kv_dtype        slot i of a unit is one contiguous row; only
 *                                                        slots < lens[b,h] are live; 16-byte aligned
 *   lens           [B, Hkv]              int32           live keys per unit
 *   pos            [B, Hkv, Lcap]        int32           absolute 0-based token position of each slot,
 *                                                        strictly increasing within a unit
 *   last_hit       [B, Hkv, Lcap]        int32           last step at which some head of the group found
 *                                                        the key important; 0 = never
 *   t              [B]                   int32           absolute 1-based step of the current query
 *                                                        (tokens of the sequence so far, incl. this one)
 *   t_first        [B]                   int32           step of the oldest row ever recorded in the ring;
 *                                                        the window is full iff t - t_first + 1 >= w
 *   score_ring     [B, Hq, w, Tcap]      score_dtype     row (tau-1) mod w holds the scores of step tau,
 *                                                        column = ABSOLUTE position of the key, so rows
 *                                                        never need compaction.  A step writes the columns
 *                                                        of the keys live at that step; the columns of keys
 *                                                        evicted earlier keep what an older query left
 *                                                        there, and columns of positions a row's query
 *                                                        had not reached hold whatever the buffer held:
 *                                                        no call reads either
 *   out            [B, Hq, d]            float32
 *   keep           [B, Hkv, Lcap]        uint8           1 = survives; entries >= lens are unspecified
 *   kept_idx       [B, Hkv, Lcap]        int32           old slot of the j-th survivor, ascending
 * Slots >= lens' after a compaction hold unspecified data.
 *
 * Arithmetic: logits and all accumulation in fp32; scores are rounded (nearest-even) to
 * score_dtype when stored, and the importance test compares the STORED value, widened to fp32,
 * against fp32(c) / fp32(t) (IEEE division) with >=.
 *
 * score_dtype CORM_BIT: the ring holds the boolean message of Algorithm 1 instead of scores:
 *   score_ring     [B, Hq, w, ceil(Tcap/32)]  uint32     bit (pos % 32) of word (pos / 32) of row (tau-1) mod w
 *                                                        = the key at position pos was important at step tau
 * (1/16 of a bf16 ring).  The test then compares the fp32 score itself; the row of a step is cleared
 * before its bits are set.
 */
#ifndef CORM_H
#define CORM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum corm_dtype { CORM_F32 = 0, CORM_BF16 = 1, CORM_BIT = 2 /* score_dtype only */ };

enum corm_status {
  CORM_OK = 0,
  CORM_EINVAL = -1,       /* null / misaligned pointer, bad shape, w < 1, r < 1, c < 0 ...      */
  CORM_EUNSUPPORTED = -2, /* d not in {64,128}, group size not in {1,2,4,8}, unknown dtype      */
  CORM_ECAPACITY = -3,    /* workspace too small (host); device: see CORM_DEV_* bits             */
  CORM_EHIP = -4          /* a HIP call or launch failed                                         */
};

/* bits ORed into the optional device status word */
enum corm_dev_status {
  CORM_DEV_UNIT_FULL = 1, /* append skipped: lens == Lcap                                        */
  CORM_DEV_BAD_STEP = 2,  /* t < 1 or t > Tcap or a position outside [0,Tcap): record skipped   */
  CORM_DEV_BAD_LENS = 4   /* lens outside [0,Lcap]: clamped                                      */
};

typedef struct corm_desc {
  int32_t B, Hq, Hkv, d; /* d in {64,128}; Hq % Hkv == 0; G = Hq/Hkv in {1,2,4,8}                */
  int32_t Lcap;          /* slots per unit                                                        */
  int32_t Tcap;          /* ring columns = largest absolute position + 1                          */
  int32_t w, r;          /* recent-query window, protected newest slots; both >= 1                */
  int32_t kv_dtype;      /* corm_dtype of q, K, V, k_new, v_new                                   */
  int32_t score_dtype;   /* corm_dtype of score_ring                                              */
  float thr_scale;       /* c in the threshold c/t; 1 = Def. 3.1; 0 = everything important        */
  float sm_scale;        /* logit scale; 0 selects 1/sqrt(d) (Eq. 1)                              */
} corm_desc;

/* Optional per-call launch options of the attend / step calls (NULL = all defaults).
 *   path   how attend + record are launched: 0 = chosen by shape (default); 1 = split kernels (several
 *          workgroups per unit, partials merged by a second launch; grouped bf16 d=128 queries take q.K^T on
 *          the matrix cores); 2 = one workgroup per unit with the logits in LDS (taken only if they fit);
 *          3 = as 1 but q.K^T always on the vector ALU.  Every path produces the same keep mask, indices
 *          and cache; out and the recorded scores agree within fp32 rounding.  A tuning and test knob.
 *   attend_start_event, attend_stop_event   hipEvent_t handles (as void*), both or neither: recorded on the
 *          call's stream immediately before and after the launch that streams K and V (the split attend
 *          kernel or the fused unit kernel), so that its duration can be measured in place.  Not for use
 *          under graph capture.
 * CORM_EINVAL for a path outside 0..3 or a single event. */
typedef struct corm_launch_opts {
  int32_t path;
  int32_t reserved;            /* 0 */
  void* attend_start_event;
  void* attend_stop_event;
} corm_launch_opts;

int corm_version(void);
const char* corm_strerror(int status);

/* Bytes of workspace the attend/step calls need for this descriptor (host call). */
int corm_workspace_bytes(const corm_desc* desc, size_t* bytes);

/* Prepare a freshly allocated workspace (clears its per-split survivor counts).  Optional: every
 * call writes what it later reads. */
int corm_workspace_init(const corm_desc* desc, void* workspace, size_t workspace_bytes, void* stream);

/* Append (shapes of Algorithm 1): K[b,h,lens] = k_new, V likewise, pos = t-1, last_hit = 0, lens += 1.
 * A full unit is left unchanged and flagged in *status (may be NULL). */
int corm_append(const corm_desc* desc, void* K, void* V, int32_t* lens, int32_t* pos, int32_t* last_hit,
                const void* k_new, const void* v_new, const int32_t* t, int32_t* status, void* stream);

/* Attend + record (Eq. 1, Eq. 2, Def. 3.1): for every query head, exact softmax attention over the
 * live keys of its unit -> out; the normalized scores are written to ring row (t-1) mod w at the
 * keys' absolute positions, and last_hit[i] = t for keys some head of the group scores >= c/t.
 * Reads K, V, lens, pos; writes out, score_ring, last_hit, workspace.  A unit with lens == 0
 * yields out = 0 and records nothing. */
int corm_decode_attend(const corm_desc* desc, const void* q, const void* K, const void* V,
                       const int32_t* lens, const int32_t* pos, const int32_t* t, void* score_ring,
                       int32_t* last_hit, float* out, void* workspace, size_t workspace_bytes,
                       int32_t* status, const corm_launch_opts* opts, void* stream);

/* For callers that cannot allocate device memory (code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc): corm_decode_attend without a workspace argument.  The split partials
 * and raw logits live in a device array inside the library, CORM_STATIC_SCRATCH_BYTES large, which every
 * GPU the library runs on holds until the process ends.  The call allocates and frees nothing; arguments,
 * results, errors and status flags are those of corm_decode_attend, bit for bit.
 * Limit: the scratch the shape needs -- per-unit survivor counts and keep words, B*Hq*ceil(Lcap/512)*4*(d+2)
 * floats of partials and B*Hq*Lcap floats of logits, each part rounded up to 256 bytes -- must fit, else
 * CORM_ECAPACITY and nothing is launched (d = 128: 32 heads x 4352 slots need 1.2 MB, 512 heads x 4608 slots
 * 19 MB, 512 query / 128 KV heads x 8704 slots 36 MB; 128 heads x 66000 slots, 70 MB, are refused).
 * Every call on a GPU shares that GPU's array: calls that overlap in time on one GPU (other streams, other
 * threads) race; calls on one stream are ordered.  Nothing in the array has to start at zero or survive
 * between calls (a call writes every partial and logit it later reads).  The first call on a device looks
 * the array's address up once: make one call eagerly before capturing a graph. */
#define CORM_STATIC_SCRATCH_BYTES (40u << 20)
int corm_decode_attend_static(const corm_desc* desc, const void* q, const void* K, const void* V,
                              const int32_t* lens, const int32_t* pos, const int32_t* t, void* score_ring,
                              int32_t* last_hit, float* out, int32_t* status, const corm_launch_opts* opts,
                              void* stream);

/* Eviction decision from the ring alone (Def. 4.1 + recent-r rule + Section 5.3 group rule),
 * evaluated literally: keep[i] = OR over the recorded rows tau in [max(t_first, t-w+1), t] and the
 * G heads of the group of (ring[tau][pos_i] >= c/tau), OR i >= lens - r.  If fewer than w rows are
 * recorded every live key is kept (Algorithm 1). */
int corm_evict_mask(const corm_desc* desc, const void* score_ring, const int32_t* lens, const int32_t* pos,
                    const int32_t* t, const int32_t* t_first, uint8_t* keep, void* stream);

/* Diagnostic (Section 3, the sparsity measurement): density[b,hq] = share of the unit's live keys whose
 * recorded score of the current step t reaches c/t (Def. 3.1), read from the ring row of step t after
 * corm_decode_attend / a step call recorded it (before a compaction moves pos).  density: device float32
 * [B, Hq]; 1 - density is the share of minor keys of that head at that step.  Works on score and bit rings. */
int corm_row_density(const corm_desc* desc, const void* score_ring, const int32_t* lens, const int32_t* pos,
                     const int32_t* t, float* density, void* stream);

/* The same decision from the per-key summary: keep[i] = last_hit[i] > t - w  OR  i >= lens - r
 * (equal to corm_evict_mask when last_hit was maintained by corm_decode_attend over the window). */
int corm_evict_mask_summary(const corm_desc* desc, const int32_t* last_hit, const int32_t* lens,
                            const int32_t* t, const int32_t* t_first, uint8_t* keep, void* stream);

/* Stable per-unit compaction (the gather of Algorithm 1), in place: survivors keep their order;
 * K, V, pos, last_hit rows move to slot (number of survivors before them); lens = survivors.
 * kept_idx (may be NULL) receives the old slot of each survivor.  Uses the workspace for staging. */
int corm_compact(const corm_desc* desc, void* K, void* V, int32_t* pos, int32_t* last_hit, int32_t* lens,
                 const uint8_t* keep, int32_t* kept_idx, void* workspace, size_t workspace_bytes, void* stream);

/* One fused decode step = append, attend, record, evict, compact, in Algorithm 1's order (the
 * current query attends over ALL l keys, eviction takes effect from the next step).  Same bits
 * as corm_append + corm_decode_attend + corm_evict_mask + corm_compact.  keep and kept_idx may
 * be NULL; when given they describe the slots as they were after the append. */
int corm_decode_step(const corm_desc* desc, const void* q, const void* k_new, const void* v_new,
                     void* K, void* V, int32_t* lens, int32_t* pos, int32_t* last_hit,
                     const int32_t* t, const int32_t* t_first, void* score_ring, float* out,
                     uint8_t* keep, int32_t* kept_idx, void* workspace, size_t workspace_bytes,
                     int32_t* status, const corm_launch_opts* opts, void* stream);

/* The fused step in two phases, for callers that overlap the compaction with other work (another
 * layer's attention, the model's GEMMs) on a second stream:
 *   corm_step_attend  append + attend + record + decide (Eq. 1, Eq. 2, Def. 3.1, Def. 4.1): reads the cache
 *                     and lens; writes the new row (K, V, pos, last_hit at slot lens), out, the ring row,
 *                     last_hit of important keys, the keep flags (bit masks in the workspace; also one
 *                     byte per slot in `keep` if given) and per-chunk survivor counts.  Does NOT change lens.
 *   corm_step_evict   compact (Algorithm 1's gather) from the workspace's keep masks: moves K, V, pos,
 *                     last_hit rows, writes lens and, if given, kept_idx.
 * corm_decode_step == corm_step_attend then corm_step_evict on one stream, with the same workspace.
 * The caller orders: evict after attend of the same step; the next step's attend of the same cache
 * after evict; no other call may use the workspace between the two phases. */
int corm_step_attend(const corm_desc* desc, const void* q, const void* k_new, const void* v_new, void* K, void* V,
                     const int32_t* lens, int32_t* pos, int32_t* last_hit, const int32_t* t, const int32_t* t_first,
                     void* score_ring, float* out, uint8_t* keep, void* workspace, size_t workspace_bytes,
                     int32_t* status, const corm_launch_opts* opts, void* stream);
int corm_step_evict(const corm_desc* desc, void* K, void* V, int32_t* lens, int32_t* pos, int32_t* last_hit,
                    int32_t* kept_idx, void* workspace, size_t workspace_bytes, void* stream);

/* The fused step with deferred compaction.  Algorithm 1 gathers the surviving keys after every step;
 * the gather only changes where keys lie, not which keys the next step attends to (Sec. 4.2, Eq. 1 over
 * the kept set), so it may be postponed: evicted keys stay in their slots as dead rows, marked in
 * `live`, and a unit is compacted (stably, as in corm_decode_step) only once its dead slots reach
 * dead_num/dead_den of its slots or its slots are about to run out.  The live keys of a unit, read in
 * slot order, and out, the ring and last_hit are what corm_decode_step produces; only the slot numbers
 * differ.  Dead rows are neither loaded nor scored.
 *   live       device uint64 [B, Hkv, ceil(Lcap/64)], in/out: bit (i % 64) of word (i / 64) = slot i holds a
 *              live key.  Bits at or above lens are ignored on input.  Initialise to all ones.
 *   lens       slots in use (live + dead); after a compaction, the number of live keys.
 *   keep       optional byte mask [B, Hkv, Lcap] of the slots as they were after the append: 1 = live after
 *              this step.
 *   nlive      optional device int32 [B, Hkv]: live keys after the step.
 *   dead_num, dead_den   0 <= dead_num <= dead_den, dead_den >= 1; dead_num = 0 compacts at every
 *              eviction and reproduces corm_decode_step slot for slot.
 * The recent-r rule is taken by position (pos >= t - r), which equals the last r live keys whenever
 * the cache was filled by consecutive steps (Sec. 4.2).  Other arguments, errors and status flags as
 * corm_decode_step.  CORM_EINVAL for a null or misaligned (8 bytes) live, or a bad fraction. */
int corm_decode_step_lazy(const corm_desc* desc, const void* q, const void* k_new, const void* v_new, void* K, void* V,
                          int32_t* lens, uint64_t* live, int32_t* pos, int32_t* last_hit, const int32_t* t,
                          const int32_t* t_first, void* score_ring, float* out, uint8_t* keep, int32_t* nlive,
                          int32_t dead_num, int32_t dead_den, void* workspace, size_t workspace_bytes,
                          int32_t* status, const corm_launch_opts* opts, void* stream);

/* Seeds the recent-query window from a prompt, in place of replaying its last m tokens through
 * corm_decode_step.  The paper starts Algorithm 1 from an existing message and does not say how a prompt
 * fills it; the reading taken is that prompt tokens are ordinary steps: the query at step tau (1-based)
 * attends causally to positions 0..tau-1 (Eq. 2), its scores are thresholded at c/tau (Def. 3.1) and
 * recorded, and the first eviction (Def. 4.1 + recent r, Algorithm 1's gather) fires once w rows exist.
 * Only the last m <= w queries can still be in the window when the prompt ends, so only they are needed.
 *   q_tail     device [B, Hq, m, d], kv_dtype: the prompt's last m queries, oldest first; query j belongs to
 *              step tau_j = t[b] - m + 1 + j.
 *   K, V, lens, pos   the cache already holding every prompt key (lens[b,h] slots, ascending positions);
 *              a key is visible to query j iff pos <= tau_j - 1.
 *   t          device int32 [B]: step of the last prompt token (the prompt's length, plus any offset).
 *   t_first    device int32 [B], OUT: t[b] - m + 1, as the decode calls expect it afterwards.
 *   last_hit   in/out: raised to the latest step at which a recorded score of the key reached the threshold.
 *   score_ring the rows of steps tau_0..tau_{m-1} are written at the keys' positions (16-byte aligned base).
 *   keep, kept_idx   optional, as in corm_compact: the decision per slot and the old slot of each survivor.
 * If m == w the units are then compacted exactly as corm_decode_step would after its w-th recorded step;
 * if m < w nothing is evicted yet.  Result: the state m calls of corm_decode_step would leave (same keep
 * decisions for the same recorded scores; the scores themselves agree within fp32 rounding), without `out`.
 * q.K^T runs on the matrix cores (bf16: v_mfma_f32_16x16x32_bf16, fp32: v_mfma_f32_16x16x4_f32).
 * Errors: CORM_EINVAL also for m < 1 or m > w; device status CORM_DEV_BAD_STEP if t[b] - m < 0,
 * t[b] > Tcap, or a position lies outside [0, Tcap). */
int corm_prefill_seed(const corm_desc* desc, const void* q_tail, int32_t m, void* K, void* V, int32_t* lens,
                      int32_t* pos, int32_t* last_hit, const int32_t* t, int32_t* t_first, void* score_ring,
                      uint8_t* keep, int32_t* kept_idx, void* workspace, size_t workspace_bytes, int32_t* status,
                      void* stream);

/* HIP graph capture.  The step, seeding and standalone calls enqueue kernels only (no allocation, no memset,
 * no host synchronization), so a caller may capture them in a HIP graph on `stream` and replay it with the
 * inputs refreshed in place.  The first call on a device queries it once (number of compute units): make one
 * call eagerly before capturing, and pass no events in corm_launch_opts while capturing. */

/* Summary-only state.  corm_decode_attend, corm_step_attend, corm_decode_step, corm_decode_step_lazy and
 * corm_prefill_seed accept score_ring == NULL: the scores are still formed, rounded to score_dtype and
 * compared with c/t (Def. 3.1), and last_hit is updated, but no row is recorded.  last_hit alone decides
 * Def. 4.1 (a key is kept iff its last important step lies inside the window), so every later decision,
 * lens, K, V and out are bit for bit what the same calls produce with a ring; only corm_evict_mask, which
 * reads the ring, is then unavailable.  Saves B*Hq*w*Tcap score elements of memory (the paper's own
 * message is w x l booleans; this keeps one int32 per key instead). */

/* The path (1 or 2, see corm_launch_opts) the attend / step calls take for this descriptor and these options
 * (NULL = defaults) on the current device; a negative corm_status for a bad descriptor or bad options. */
int corm_selected_path(const corm_desc* desc, const corm_launch_opts* opts);

/* Diagnostic: thr[i] = fp32(c) / fp32(t[i]) exactly as the kernels compute it (Def. 3.1). */
int corm_threshold(float c, const int32_t* t, int32_t n, float* thr, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* CORM_H */
