// C ABI of libsparq (see include/sparq.h): argument validation, launch planning, enqueue.
// No allocation, no synchronisation (sparq_async_error excepted), no host-side arithmetic of
// the method.
#include "../../include/sparq.h"

#include <hip/hip_runtime.h>

#include "params.h"

namespace {

using namespace sparq;

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

int check_shape(const sparq_shape* s) {
  if (!s) return SPARQ_EINVAL;
  if (s->B < 1 || s->H < 1 || s->H_kv < 1 || s->S_max < 1 || s->d_h < 1) return SPARQ_EINVAL;
  if (s->H % s->H_kv != 0) return SPARQ_EINVAL;
  if (s->r < 1 || s->r > s->d_h || s->k < 1) return SPARQ_EINVAL;
  if (s->dtype != SPARQ_F16 && s->dtype != SPARQ_BF16) return SPARQ_EINVAL;
  if (s->S_max % 64 != 0) return SPARQ_EINVAL;
  if (s->flags & ~(uint32_t)(SPARQ_FLAG_NO_REALLOC | SPARQ_FLAG_GQA_SHARED | SPARQ_FLAG_RAGGED_BATCH |
                             SPARQ_FLAG_TAU_SQRT_DH | SPARQ_FLAG_TAU_SQRT_R | SPARQ_FLAG_SINGLE_K | SPARQ_FLAG_TILED_K)) return SPARQ_EINVAL;
  if ((s->flags & SPARQ_FLAG_SINGLE_K) && (s->flags & SPARQ_FLAG_TILED_K)) return SPARQ_EINVAL;
  if ((s->flags & SPARQ_FLAG_TAU_SQRT_DH) && (s->flags & SPARQ_FLAG_TAU_SQRT_R)) return SPARQ_EINVAL;
  if (s->local_window < 0) return SPARQ_EINVAL;
  if (s->S_bound < 0 || s->S_bound > s->S_max || s->S_bound % 64 != 0) return SPARQ_EINVAL;
  if (s->d_h != 64 && s->d_h != 128 && s->d_h != 256) return SPARQ_EUNSUPPORTED;
  // element offsets inside one tensor are formed in size_t; the counts themselves stay in int32
  if ((int64_t)s->B * s->H > (int64_t)1 << 30) return SPARQ_EUNSUPPORTED;
  return SPARQ_OK;
}

int check_cache(const sparq_cache* c, const sparq_shape* s) {
  if (!c || !c->K || !c->V || !c->v_mean || !c->seq_lens) return SPARQ_EINVAL;
  if (!aligned16(c->K) || !aligned16(c->V) || !aligned16(c->v_mean)) return SPARQ_EINVAL;
  if (!(s->flags & SPARQ_FLAG_SINGLE_K) && (!c->Kt || !aligned16(c->Kt))) return SPARQ_EINVAL;
  return SPARQ_OK;
}

// split-sequence plan of dense_decode: enough workgroups to fill 256 CUs several times over,
// runs of at least 256 rows
void dense_plan(const sparq_shape* s, int* n_split, int* rows_per_split) {
  const int64_t heads = (int64_t)s->B * s->H_kv;
  int64_t want = (2048 + heads - 1) / heads;
  const int64_t cap = s->S_max / 256 > 0 ? s->S_max / 256 : 1;
  if (want > cap) want = cap;
  if (want < 1) want = 1;
  int rows = (int)((s->S_max + want - 1) / want);
  rows = (rows + 63) / 64 * 64;
  *rows_per_split = rows;
  *n_split = (s->S_max + rows - 1) / rows;
}

// The shape that plans, LDS and workspace are sized for: the caller's bound on the lengths (S_bound), where one is
// given, stands in for S_max; the buffers keep the strides of the shape's own S_max.
sparq_shape bounded(const sparq_shape* s) {
  sparq_shape e = *s;
  if (s->S_bound > 0) e.S_max = s->S_bound;
  e.S_bound = 0;
  return e;
}

size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

// LDS a workgroup may use: the device's, or gfx950's 160 KiB where no device can be asked (sizing
// queries on a machine without a GPU)
int max_lds_bytes() {
  static int cached = -1;   // same for every device of one machine; benign race
  if (cached < 0) {
    int dev = 0, v = 0;
    if (hipGetDevice(&dev) != hipSuccess) return 160 * 1024;
    if (hipDeviceGetAttribute(&v, hipDeviceAttributeMaxSharedMemoryPerBlock, dev) != hipSuccess) return 160 * 1024;
    cached = v;
  }
  return cached;
}

// the paper's grouped-query rule is a kernel of its own; with one query head per KV head it is
// the ordinary rule
bool wants_shared(const sparq_shape* shape) {
  return (shape->flags & SPARQ_FLAG_GQA_SHARED) && shape->H != shape->H_kv;
}

bool single_k(const sparq_shape* shape) { return (shape->flags & SPARQ_FLAG_SINGLE_K) != 0; }
bool tiled_k(const sparq_shape* shape) { return (shape->flags & SPARQ_FLAG_TILED_K) != 0; }

// Which kernels serve a shape.  Every plan keeps one 4-byte key per position (or per candidate) of its
// unit of work in LDS; that decides what fits.
enum Plan { kPlanNone, kPlanFused, kPlanLong, kPlanShared, kPlanSharedSplit, kPlanSingleK, kPlanBucket, kPlanSharedBucket };
struct PlanInfo { Plan plan; int n_split, n_span, span_len, cand_cap, n1, span1; };

// The two-level plan: spans of `span` positions select their own top-k, one workgroup per unit merges at
// most n_span * min(k, span) candidates.  It serves what no single workgroup can hold (S_max beyond the LDS)
// for batches with more units than the digit-bucket plan takes.
bool two_level_plan(const sparq_shape* s, int span, size_t lds_max, PlanInfo* p) {
  const int64_t n_span = ((int64_t)s->S_max + span - 1) / span;
  if (n_span > kMaxSpans) return false;
  const int cap = s->k < span ? s->k : span;
  if (long_scores_lds_bytes(span, s->d_h) > lds_max || long_merge_lds_bytes((int)n_span, cap) > lds_max) return false;
  const int64_t units = (int64_t)s->B * s->H;
  int64_t n = 512 / units;                      // gather workgroups per unit: fill the chip, >= 64 rows each
  if (n > kMaxSplit) n = kMaxSplit;
  if (n > s->k / 64) n = s->k / 64;
  if (n < 1) n = 1;
  p->n_span = (int)n_span; p->span_len = span; p->cand_cap = cap; p->n_split = (int)n;
  return true;
}

// The digit-bucket plan for few units with long caches: about 512 workgroups in all, spans of 1024 to 8192
// positions (a multiple of 64), at most kMaxSpans of them.
bool bucket_plan(const sparq_shape* s, size_t lds_max, PlanInfo* p) {
  const int64_t units = (int64_t)s->B * s->H;
  int64_t n_span = 512 / units;
  if (n_span < 2) n_span = 2;
  // (units x n_span <= 512: both kernels hold two workgroups per CU, and a second round of workgroups costs
  // more than longer spans do)
  if (n_span > kMaxSpans) n_span = kMaxSpans;
  int64_t span = (s->S_max + n_span - 1) / n_span;
  if (span < 1024) span = 1024;
  span = (span + 63) / 64 * 64;
  if (span > kLongSpan) span = kLongSpan;
  n_span = (s->S_max + span - 1) / span;
  if (n_span > kMaxSpans) return false;
  // the keys that share the threshold digit are a few percent of the sequence unless many keys are identical
  const int cap = s->S_max <= 40000 ? 2048 : (s->S_max <= 100000 ? 4096 : 8192);
  if (bk_scores_lds_bytes((int)span, s->d_h) > lds_max ||
      bk_select_lds_bytes((int)span, s->d_h, (int)n_span, cap) > lds_max) return false;
  p->n_span = (int)n_span; p->span_len = (int)span; p->cand_cap = cap;
  return true;
}

// The grouped-query rule over several workgroups per KV unit: n1 spans for the logits (at most 256 workgroups,
// at least 1024 positions each), spans of 4096 / 8192 positions for the two-level selection.
bool shared_split_plan(const sparq_shape* s, size_t lds_max, PlanInfo* p) {
  const int64_t ukv = (int64_t)s->B * s->H_kv;
  // (gs_logits with 4 heads' accumulators runs one workgroup per CU: more than 256 workgroups would come in two
  // rounds, which was measured as 58 instead of 47 us per decode just above S = 32768 with 8 KV units)
  int64_t n1 = 256 / ukv;
  if (n1 > kMaxSpans) n1 = kMaxSpans;
  if (n1 < 1) n1 = 1;
  int64_t span1 = (s->S_max + n1 - 1) / n1;
  if (span1 < 1024) span1 = 1024;
  span1 = (span1 + 63) / 64 * 64;
  n1 = (s->S_max + span1 - 1) / span1;
  const int span2 = s->S_max >= 32768 ? kLongSpan : kLongSpan / 2;
  const int64_t n2 = ((int64_t)s->S_max + span2 - 1) / span2;
  if (n1 > kMaxSpans || n2 > kMaxSpans) return false;
  const int cap = s->k < span2 ? s->k : span2;
  if (gs_select_lds_bytes(span2) > lds_max || gs_merge_lds_bytes((int)n2, cap) > lds_max) return false;
  int64_t n = 512 / ukv;
  if (n > kMaxSplit) n = kMaxSplit;
  if (n > s->k / 64) n = s->k / 64;
  if (n < 1) n = 1;
  p->n1 = (int)n1; p->span1 = (int)span1; p->n_span = (int)n2; p->span_len = span2; p->cand_cap = cap; p->n_split = (int)n;
  return true;
}

// The grouped-query rule on the digit-bucket plan: gs_logits over n1 spans per KV unit (at most 256 workgroups, at
// least 1024 positions each), then the bucket plan's spans for the selection.
bool shared_bucket_plan(const sparq_shape* s, size_t lds_max, PlanInfo* p) {
  const int64_t ukv = (int64_t)s->B * s->H_kv;
  int64_t n1 = 256 / ukv;                   // one round of gs_logits workgroups, as above
  if (n1 > kMaxSpans) n1 = kMaxSpans;
  if (n1 < 1) n1 = 1;
  int64_t span1 = (s->S_max + n1 - 1) / n1;
  if (span1 < 1024) span1 = 1024;
  span1 = (span1 + 63) / 64 * 64;
  n1 = (s->S_max + span1 - 1) / span1;
  if (n1 > kMaxSpans) return false;
  if (!bucket_plan(s, lds_max, p)) return false;
  if (bk_group_scores_lds_bytes(p->span_len) > lds_max) return false;
  p->n1 = (int)n1; p->span1 = (int)span1;
  return true;
}

PlanInfo choose_plan(const sparq_shape* s) {
  PlanInfo p{kPlanNone, 0, 0, 0, 0, 0, 0};
  const size_t lds_max = (size_t)max_lds_bytes();
  if (single_k(s)) {
    const size_t need = wants_shared(s) ? 0 : decode_single_k_lds_bytes(s->S_max, s->d_h);
    if (need != 0 && need <= lds_max) p.plan = kPlanSingleK;
    return p;
  }
  if (tiled_k(s)) {            // one kernel reads the tiled layout: one workgroup per head
    if (!wants_shared(s) && decode_lds_bytes(s->S_max, s->d_h) <= lds_max) p.plan = kPlanFused;
    return p;
  }
  if (wants_shared(s)) {
    const size_t need = decode_shared_lds_bytes(s->S_max, s->d_h, s->H / s->H_kv);
    if (need == 0) return p;                                    // no kernel for this group size
    const bool one_wg = need <= lds_max;
    // measured: the one-workgroup kernel is faster from about 64 KV units on (116 vs 123 us at 128 units,
    // S = 8192) and far slower below (230 vs 70 us at 8 units, S = 32768)
    const int64_t ukv = (int64_t)s->B * s->H_kv;
    const bool few = (ukv <= 32 && s->S_max >= 8192) || (ukv <= 64 && s->S_max >= 16384);
    // few heads with long caches: the digit-bucket selection, one for the group (measured against the two-level
    // selection per KV head: 59 vs 87 us at 8 KV units, S = 32768; 107 vs 166 us at S = 131072)
    if ((few || !one_wg) && (int64_t)s->B * s->H <= kSplitMaxUnits && s->S_max >= 8192 && shared_bucket_plan(s, lds_max, &p)) {
      p.plan = kPlanSharedBucket;
      return p;
    }
    if ((few || !one_wg) && shared_split_plan(s, lds_max, &p)) { p.plan = kPlanSharedSplit; return p; }
    if (one_wg) p.plan = kPlanShared;
    return p;
  }
  // Few units with long caches: the digit-bucket plan, where it was measured faster than one workgroup per unit
  // (H = 32, r = 32, k = S / 16, bucket / one-workgroup us per decode; S = 8192: 29/27, 32/29, 36/31, 41/32 at 32, 64,
  // 96, 128 units; 12 288: 30/37, 36/39, 43/43, 49/43; 16 384: 33/46, 41/51, 49/55, 59/59; 24 576: 36/65, 48/70,
  // 63/77, 95/79; 32 768: 41/82, 59/89, 94/98, 116/103), and whatever one workgroup's LDS cannot hold.
  const int64_t units = (int64_t)s->B * s->H;
  const bool one_wg_fits = decode_lds_bytes(s->S_max, s->d_h) <= lds_max;
  const bool bucket_faster = (s->S_max >= 16384 && units <= 96) || (s->S_max >= 12288 && units <= 64);
  if (units <= kSplitMaxUnits && s->S_max >= 8192 && (bucket_faster || !one_wg_fits) && bucket_plan(s, lds_max, &p)) {
    p.plan = kPlanBucket;
    return p;
  }
  if (one_wg_fits) { p.plan = kPlanFused; return p; }
  if (two_level_plan(s, kLongSpan, lds_max, &p)) p.plan = kPlanLong;
  return p;
}

struct GsLayout { size_t z, stat, esc, alpha, cnt, ckey, cpos, list, part, end; int list_stride; };

GsLayout gs_layout(const sparq_shape* s, const PlanInfo& p) {
  const size_t units = (size_t)s->B * s->H, ukv = (size_t)s->B * s->H_kv, g = (size_t)(s->H / s->H_kv);
  GsLayout l;
  const int kk = s->k < s->S_max ? s->k : s->S_max;
  l.list_stride = (kk + 7) & ~7;
  size_t off = kControlBytes;
  l.z = off; off = align256(off + units * s->S_max * sizeof(float));
  l.stat = off; off = align256(off + ukv * p.n1 * g * 2 * sizeof(float));
  l.esc = off; off = align256(off + units * sizeof(float));
  l.alpha = off; off = align256(off + units * sizeof(float));
  l.cnt = off; off = align256(off + ukv * p.n_span * sizeof(int32_t));
  l.ckey = off; off = align256(off + ukv * p.n_span * p.cand_cap * sizeof(uint32_t));
  l.cpos = off; off = align256(off + ukv * p.n_span * p.cand_cap * sizeof(int32_t));
  l.list = off; off = align256(off + ukv * l.list_stride * sizeof(int32_t));
  l.part = off; off = align256(off + units * p.n_split * (s->d_h + 2) * sizeof(float));
  l.end = off;
  return l;
}

struct BucketLayout { size_t tmax, zsum, anum, tau, zden, coarse, fine, skey, spos, part, z, stat, esc, end; };

BucketLayout bucket_layout(const sparq_shape* s, const PlanInfo& p) {
  const size_t units = (size_t)s->B * s->H, slots = units * p.n_span;
  BucketLayout l;
  size_t off = kControlBytes;
  l.tmax = off; off = align256(off + slots * sizeof(float));
  l.zsum = off; off = align256(off + slots * sizeof(float));
  l.anum = off; off = align256(off + slots * sizeof(float));
  l.tau = off; off = align256(off + units * sizeof(float));
  l.zden = off; off = align256(off + units * sizeof(float));
  l.coarse = off; off = align256(off + slots * 64 * sizeof(uint16_t));
  l.fine = off; off = align256(off + slots * bk_fine_len() * sizeof(uint16_t));
  l.skey = off; off = align256(off + slots * p.span_len * sizeof(uint32_t));
  l.spos = off; off = align256(off + slots * p.span_len * sizeof(uint32_t));
  l.part = off; off = align256(off + slots * (s->d_h + 2) * sizeof(float));
  l.z = l.stat = l.esc = off;
  if (p.plan == kPlanSharedBucket) {      // what gs_logits hands on: logit numerators, span statistics, temperatures
    const size_t ukv = (size_t)s->B * s->H_kv, g = (size_t)(s->H / s->H_kv);
    l.z = off; off = align256(off + units * s->S_max * sizeof(float));
    l.stat = off; off = align256(off + ukv * p.n1 * g * 2 * sizeof(float));
    l.esc = off; off = align256(off + units * sizeof(float));
  }
  l.end = off;
  return l;
}

struct LongLayout { size_t tmax, zsum, cnt, tau, alpha, ckey, cpos, list, part, end; };

LongLayout long_layout(const sparq_shape* s, const PlanInfo& p) {
  const size_t units = (size_t)s->B * s->H;
  LongLayout l;
  size_t off = kControlBytes;
  l.tmax = off; off = align256(off + units * p.n_span * sizeof(float));
  l.zsum = off; off = align256(off + units * p.n_span * sizeof(float));
  l.cnt = off; off = align256(off + units * p.n_span * sizeof(int32_t));
  l.tau = off; off = align256(off + units * sizeof(float));
  l.alpha = off; off = align256(off + units * sizeof(float));
  l.ckey = off; off = align256(off + units * p.n_span * p.cand_cap * sizeof(uint32_t));
  l.cpos = off; off = align256(off + units * p.n_span * p.cand_cap * sizeof(int32_t));
  l.list = off; off = align256(off + units * s->S_max * sizeof(int32_t));
  l.part = off; off = align256(off + units * p.n_split * (s->d_h + 2) * sizeof(float));
  l.end = off;
  return l;
}

size_t workspace_need(const sparq_shape* s) {
  int n_split, rows;
  dense_plan(s, &n_split, &rows);
  size_t need = (size_t)kControlBytes + (size_t)s->B * s->H * n_split * (s->d_h + 2) * sizeof(float);
  const PlanInfo p = choose_plan(s);
  size_t e = 0;
  if (p.plan == kPlanLong) e = long_layout(s, p).end;
  if (p.plan == kPlanBucket || p.plan == kPlanSharedBucket) e = bucket_layout(s, p).end;
  if (p.plan == kPlanShared) e = (size_t)kControlBytes + (size_t)s->B * s->H * s->S_max * sizeof(float);
  if (p.plan == kPlanSharedSplit) e = gs_layout(s, p).end;
#ifdef SPARQ_STAGE_CLOCKS
  if (p.plan == kPlanFused) e = (size_t)kControlBytes + (size_t)s->B * s->H * kStageStamps * sizeof(unsigned long long);
#endif
  return e > need ? e : need;
}

int check_workspace(const sparq_shape* s, const void* ws, size_t bytes) {
  if (!ws || !aligned16(ws) || bytes < workspace_need(s)) return SPARQ_EWORKSPACE;
  return SPARQ_OK;
}

// enqueue one decode over `a` with the plan the shape calls for
hipError_t enqueue_decode(const sparq_shape* shape, const DecodeArgs& a, void* workspace, hipStream_t s) {
  const PlanInfo p = choose_plan(shape);
  if (p.plan == kPlanNone) return hipErrorInvalidValue;
#ifdef SPARQ_STAGE_CLOCKS
  if (p.plan == kPlanFused) {
    DecodeArgs c = a;
    c.clocks = reinterpret_cast<unsigned long long*>(static_cast<char*>(workspace) + kControlBytes);
    return launch_decode(c, shape->dtype, s);
  }
#endif
  if (p.plan == kPlanFused) return launch_decode(a, shape->dtype, s);
  const bool one_k = p.plan == kPlanSingleK;
  DecodeArgs d = a;
  if (a.k_new && p.plan != kPlanBucket && p.plan != kPlanSharedBucket) {
    // the one-workgroup-per-head kernel and the digit-bucket plans have the append built in; the other plans
    // append into the *_next state with the append kernel, then decode from that state
    AppendArgs ap;
    ap.K = a.K; ap.Kt = one_k ? nullptr : a.Kt; ap.V = a.V; ap.v_mean = const_cast<float*>(a.v_mean); ap.seq_lens = const_cast<int32_t*>(a.seq_lens);
    ap.v_mean_out = a.v_mean_next; ap.seq_lens_out = a.seq_lens_next;
    ap.k_new = a.k_new; ap.v_new = a.v_new; ap.n_new_per_seq = nullptr; ap.err = a.err;
    ap.B = a.B; ap.H_kv = a.H_kv; ap.S_max = a.S_max; ap.S_stride = a.S_stride; ap.d_h = a.d_h; ap.n_new = 1; ap.tiled = tiled_k(shape) ? 1 : 0;
    hipError_t e = launch_append(ap, shape->dtype, s);
    if (e != hipSuccess) return e;
    d.v_mean = a.v_mean_next; d.seq_lens = a.seq_lens_next;
    d.k_new = nullptr; d.v_new = nullptr; d.v_mean_next = nullptr; d.seq_lens_next = nullptr;
  }
  if (one_k) return launch_decode_single_k(d, shape->dtype, s);
  if (p.plan == kPlanShared)
    return launch_decode_shared(d, reinterpret_cast<float*>(static_cast<char*>(workspace) + kControlBytes), shape->dtype, s);
  char* w = static_cast<char*>(workspace);
  if (p.plan == kPlanSharedSplit) {
    const GsLayout l = gs_layout(shape, p);
    GsArgs ga;
    ga.d = d;
    ga.n1 = p.n1; ga.span1 = p.span1; ga.n2 = p.n_span; ga.span2 = p.span_len; ga.cand_cap = p.cand_cap;
    ga.n_split = p.n_split; ga.list_stride = l.list_stride;
    ga.z_ws = reinterpret_cast<float*>(w + l.z);
    ga.stat_ws = reinterpret_cast<float*>(w + l.stat);
    ga.esc_ws = reinterpret_cast<float*>(w + l.esc);
    ga.alpha_ws = reinterpret_cast<float*>(w + l.alpha);
    ga.cnt_ws = reinterpret_cast<int32_t*>(w + l.cnt);
    ga.cand_key_ws = reinterpret_cast<uint32_t*>(w + l.ckey);
    ga.cand_pos_ws = reinterpret_cast<int32_t*>(w + l.cpos);
    ga.list_ws = reinterpret_cast<int32_t*>(w + l.list);
    ga.part_ws = reinterpret_cast<float*>(w + l.part);
    return launch_decode_shared_split(ga, shape->dtype, s);
  }
  if (p.plan == kPlanBucket || p.plan == kPlanSharedBucket) {
    const BucketLayout l = bucket_layout(shape, p);
    BucketArgs ba;
    ba.d = d;
    ba.n_span = p.n_span; ba.span_len = p.span_len; ba.cand_cap = p.cand_cap;
    ba.tmax_ws = reinterpret_cast<float*>(w + l.tmax);
    ba.zsum_ws = reinterpret_cast<float*>(w + l.zsum);
    ba.anum_ws = reinterpret_cast<float*>(w + l.anum);
    ba.tau_ws = reinterpret_cast<float*>(w + l.tau);
    ba.zden_ws = reinterpret_cast<float*>(w + l.zden);
    ba.coarse_ws = reinterpret_cast<uint16_t*>(w + l.coarse);
    ba.fine_ws = reinterpret_cast<uint16_t*>(w + l.fine);
    ba.skey_ws = reinterpret_cast<uint32_t*>(w + l.skey);
    ba.spos_ws = reinterpret_cast<uint32_t*>(w + l.spos);
    ba.part_ws = reinterpret_cast<float*>(w + l.part);
    if (p.plan == kPlanSharedBucket) {
      GsArgs ga{};
      ga.d = d;
      ga.n1 = p.n1; ga.span1 = p.span1;
      ga.z_ws = reinterpret_cast<float*>(w + l.z);
      ga.stat_ws = reinterpret_cast<float*>(w + l.stat);
      ga.esc_ws = reinterpret_cast<float*>(w + l.esc);
      hipError_t e = launch_group_logits(ga, shape->dtype, s);
      if (e != hipSuccess) return e;
      ba.group = shape->H / shape->H_kv; ba.n1 = p.n1;
      ba.z_ws = ga.z_ws; ba.stat_ws = ga.stat_ws; ba.esc_ws = ga.esc_ws;
      return launch_decode_bucket_group(ba, shape->dtype, s);
    }
    return launch_decode_bucket(ba, shape->dtype, s);
  }
  if (p.plan == kPlanLong) {
    const LongLayout l = long_layout(shape, p);
    LongArgs la;
    la.d = d;
    la.n_span = p.n_span; la.span_len = p.span_len; la.cand_cap = p.cand_cap; la.n_split = p.n_split;
    la.tmax_ws = reinterpret_cast<float*>(w + l.tmax);
    la.zsum_ws = reinterpret_cast<float*>(w + l.zsum);
    la.cnt_ws = reinterpret_cast<int32_t*>(w + l.cnt);
    la.tau_ws = reinterpret_cast<float*>(w + l.tau);
    la.alpha_ws = reinterpret_cast<float*>(w + l.alpha);
    la.cand_key_ws = reinterpret_cast<uint32_t*>(w + l.ckey);
    la.cand_pos_ws = reinterpret_cast<int32_t*>(w + l.cpos);
    la.list_ws = reinterpret_cast<int32_t*>(w + l.list);
    la.part_ws = reinterpret_cast<float*>(w + l.part);
    return launch_decode_long(la, shape->dtype, s);
  }
  return hipErrorInvalidValue;
}

bool decode_supported(const sparq_shape* shape) { return choose_plan(shape).plan != kPlanNone; }

// ---- library-owned scratch for sparq_decode_noalloc ----
// One array per GPU (each device that loads this code object holds its own copy at its own address), kept
// until the process ends.  In host code the array's name is only a handle for hipGetSymbolAddress: kernels,
// fills and copies take the device address looked up below, never the name.
constexpr size_t kStaticScratchBytes = (size_t)32 << 20;
constexpr int kMaxDevices = 64;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

// Device address of `scratch` on the current device; looked up (and the control block cleared by a fill
// kernel on `s`) on the first call per device.  Returns nullptr if the runtime refuses.
void* static_scratch(hipStream_t s) {
  static void* ptr[kMaxDevices] = {};      // benign race: every thread computes the same value
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
  if (!ptr[dev]) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return nullptr;
    if (launch_clear(p, kControlBytes, s) != hipSuccess) return nullptr;
    ptr[dev] = p;
  }
  return ptr[dev];
}

}  // namespace

extern "C" {

int sparq_workspace_bytes(const sparq_shape* caller_shape, size_t* out_bytes) {
  int rc = check_shape(caller_shape);
  if (rc != SPARQ_OK) return rc;
  if (!out_bytes) return SPARQ_EINVAL;
  const sparq_shape sized = bounded(caller_shape);
  const sparq_shape* shape = &sized;
  *out_bytes = workspace_need(shape);
  return SPARQ_OK;
}

int sparq_workspace_init(void* workspace, size_t workspace_bytes, void* hip_stream) {
  if (!workspace || !aligned16(workspace) || workspace_bytes < (size_t)kControlBytes) return SPARQ_EWORKSPACE;
  return launch_clear(workspace, kControlBytes, static_cast<hipStream_t>(hip_stream)) == hipSuccess ? SPARQ_OK : SPARQ_ELAUNCH;
}

int sparq_kv_append(const sparq_shape* caller_shape, const sparq_cache* cache, const void* k_new,
                    const void* v_new, int32_t n_new, const int32_t* n_new_per_seq,
                    void* workspace, size_t workspace_bytes, void* hip_stream) {
  int rc = check_shape(caller_shape);
  if (rc == SPARQ_OK) rc = check_cache(cache, caller_shape);
  if (rc != SPARQ_OK) return rc;
  const sparq_shape sized = bounded(caller_shape);
  const sparq_shape* shape = &sized;
  if (!k_new || !v_new || !aligned16(k_new) || !aligned16(v_new) || n_new < 1 || n_new > caller_shape->S_max) return SPARQ_EINVAL;
  rc = check_workspace(shape, workspace, workspace_bytes);
  if (rc != SPARQ_OK) return rc;
  AppendArgs a;
  a.K = cache->K; a.Kt = single_k(shape) ? nullptr : cache->Kt; a.V = cache->V; a.v_mean = cache->v_mean; a.seq_lens = cache->seq_lens;
  a.v_mean_out = cache->v_mean; a.seq_lens_out = cache->seq_lens;
  a.k_new = k_new; a.v_new = v_new; a.n_new_per_seq = n_new_per_seq; a.err = static_cast<int32_t*>(workspace);
  a.B = shape->B; a.H_kv = shape->H_kv; a.S_max = a.S_stride = caller_shape->S_max;   // S_bound does not limit an append
  a.d_h = shape->d_h; a.n_new = n_new; a.tiled = tiled_k(shape) ? 1 : 0;
  return launch_append(a, shape->dtype, static_cast<hipStream_t>(hip_stream)) == hipSuccess ? SPARQ_OK : SPARQ_ELAUNCH;
}

int sparq_decode(const sparq_shape* caller_shape, const sparq_cache* cache, const void* q,
                 const int32_t* k_per_seq, void* out, float* alpha_out, int32_t* idx_out,
                 int32_t idx_stride, int32_t* chan_out, void* workspace, size_t workspace_bytes,
                 void* hip_stream) {
  int rc = check_shape(caller_shape);
  if (rc == SPARQ_OK) rc = check_cache(cache, caller_shape);
  if (rc != SPARQ_OK) return rc;
  const sparq_shape sized = bounded(caller_shape);
  const sparq_shape* shape = &sized;
  if (!q || !out || !aligned16(q) || !aligned16(out)) return SPARQ_EINVAL;
  if (idx_out && idx_stride < 1) return SPARQ_EINVAL;
  rc = check_workspace(shape, workspace, workspace_bytes);
  if (rc != SPARQ_OK) return rc;
  if (!decode_supported(shape)) return SPARQ_EUNSUPPORTED;
  DecodeArgs a;
  a.K = cache->K; a.Kt = cache->Kt; a.V = cache->V; a.v_mean = cache->v_mean; a.seq_lens = cache->seq_lens;
  a.q = q; a.k_per_seq = k_per_seq; a.out = out; a.alpha_out = alpha_out; a.idx_out = idx_out;
  a.k_new = nullptr; a.v_new = nullptr; a.v_mean_next = nullptr; a.seq_lens_next = nullptr;
  a.chan_out = chan_out; a.err = static_cast<int32_t*>(workspace);
  a.B = shape->B; a.H = shape->H; a.H_kv = shape->H_kv; a.S_max = shape->S_max; a.S_stride = caller_shape->S_max; a.d_h = shape->d_h;
  a.r = shape->r; a.k = shape->k; a.idx_stride = idx_out ? idx_stride : 0; a.flags = shape->flags;
  a.local_window = shape->local_window;
  return enqueue_decode(shape, a, workspace, static_cast<hipStream_t>(hip_stream)) == hipSuccess ? SPARQ_OK : SPARQ_ELAUNCH;
}

int sparq_decode_noalloc(const sparq_shape* caller_shape, const sparq_cache* cache, const void* q,
                         const int32_t* k_per_seq, void* out, float* alpha_out, int32_t* idx_out,
                         int32_t idx_stride, int32_t* chan_out, int32_t* error_word, void* hip_stream) {
  int rc = check_shape(caller_shape);
  if (rc == SPARQ_OK) rc = check_cache(cache, caller_shape);
  if (rc != SPARQ_OK) return rc;
  const sparq_shape sized = bounded(caller_shape);
  const sparq_shape* shape = &sized;
  if (!q || !out || !aligned16(q) || !aligned16(out)) return SPARQ_EINVAL;
  if (idx_out && idx_stride < 1) return SPARQ_EINVAL;
  if (!decode_supported(shape)) return SPARQ_EUNSUPPORTED;
  if (workspace_need(shape) > kStaticScratchBytes) return SPARQ_ETOOLARGE;
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  void* ws = static_scratch(s);
  if (!ws) return SPARQ_ELAUNCH;
  DecodeArgs a;
  a.K = cache->K; a.Kt = cache->Kt; a.V = cache->V; a.v_mean = cache->v_mean; a.seq_lens = cache->seq_lens;
  a.q = q; a.k_per_seq = k_per_seq; a.out = out; a.alpha_out = alpha_out; a.idx_out = idx_out;
  a.k_new = nullptr; a.v_new = nullptr; a.v_mean_next = nullptr; a.seq_lens_next = nullptr;
  a.chan_out = chan_out; a.err = error_word ? error_word : static_cast<int32_t*>(ws);
  a.B = shape->B; a.H = shape->H; a.H_kv = shape->H_kv; a.S_max = shape->S_max; a.S_stride = caller_shape->S_max; a.d_h = shape->d_h;
  a.r = shape->r; a.k = shape->k; a.idx_stride = idx_out ? idx_stride : 0; a.flags = shape->flags;
  a.local_window = shape->local_window;
  return enqueue_decode(shape, a, ws, s) == hipSuccess ? SPARQ_OK : SPARQ_ELAUNCH;
}

int sparq_decode_step(const sparq_shape* caller_shape, const sparq_cache* cache, const void* k_new,
                      const void* v_new, float* v_mean_next, int32_t* seq_lens_next, const void* q,
                      const int32_t* k_per_seq, void* out, float* alpha_out, int32_t* idx_out,
                      int32_t idx_stride, int32_t* chan_out, void* workspace, size_t workspace_bytes,
                      void* hip_stream) {
  int rc = check_shape(caller_shape);
  if (rc == SPARQ_OK) rc = check_cache(cache, caller_shape);
  if (rc != SPARQ_OK) return rc;
  const sparq_shape sized = bounded(caller_shape);
  const sparq_shape* shape = &sized;
  if (!q || !out || !aligned16(q) || !aligned16(out)) return SPARQ_EINVAL;
  if (!k_new || !v_new || !aligned16(k_new) || !aligned16(v_new)) return SPARQ_EINVAL;
  if (!v_mean_next || !seq_lens_next || !aligned16(v_mean_next)) return SPARQ_EINVAL;
  if (v_mean_next == cache->v_mean || seq_lens_next == cache->seq_lens) return SPARQ_EINVAL;
  if (idx_out && idx_stride < 1) return SPARQ_EINVAL;
  rc = check_workspace(shape, workspace, workspace_bytes);
  if (rc != SPARQ_OK) return rc;
  if (!decode_supported(shape)) return SPARQ_EUNSUPPORTED;
  DecodeArgs a;
  a.K = cache->K; a.Kt = cache->Kt; a.V = cache->V; a.v_mean = cache->v_mean; a.seq_lens = cache->seq_lens;
  a.q = q; a.k_per_seq = k_per_seq; a.out = out; a.alpha_out = alpha_out; a.idx_out = idx_out;
  a.k_new = k_new; a.v_new = v_new; a.v_mean_next = v_mean_next; a.seq_lens_next = seq_lens_next;
  a.chan_out = chan_out; a.err = static_cast<int32_t*>(workspace);
  a.B = shape->B; a.H = shape->H; a.H_kv = shape->H_kv; a.S_max = shape->S_max; a.S_stride = caller_shape->S_max; a.d_h = shape->d_h;
  a.r = shape->r; a.k = shape->k; a.idx_stride = idx_out ? idx_stride : 0; a.flags = shape->flags;
  a.local_window = shape->local_window;
  return enqueue_decode(shape, a, workspace, static_cast<hipStream_t>(hip_stream)) == hipSuccess ? SPARQ_OK : SPARQ_ELAUNCH;
}

int dense_decode(const sparq_shape* caller_shape, const sparq_cache* cache, const void* q, void* out,
                 void* workspace, size_t workspace_bytes, void* hip_stream) {
  int rc = check_shape(caller_shape);
  if (rc == SPARQ_OK) rc = check_cache(cache, caller_shape);
  if (rc != SPARQ_OK) return rc;
  const sparq_shape sized = bounded(caller_shape);
  const sparq_shape* shape = &sized;
  if (!q || !out || !aligned16(q) || !aligned16(out)) return SPARQ_EINVAL;
  rc = check_workspace(shape, workspace, workspace_bytes);
  if (rc != SPARQ_OK) return rc;
  if (tiled_k(shape)) return SPARQ_EUNSUPPORTED;   // the comparison kernel reads key rows
  DenseArgs a;
  a.K = cache->K; a.V = cache->V; a.seq_lens = cache->seq_lens; a.q = q; a.out = out;
  a.partials = reinterpret_cast<float*>(static_cast<char*>(workspace) + kControlBytes);
  a.err = static_cast<int32_t*>(workspace);
  a.B = shape->B; a.H = shape->H; a.H_kv = shape->H_kv; a.S_max = shape->S_max; a.S_stride = caller_shape->S_max; a.d_h = shape->d_h;
  dense_plan(shape, &a.n_split, &a.rows_per_split);
  return launch_dense(a, shape->dtype, static_cast<hipStream_t>(hip_stream)) == hipSuccess ? SPARQ_OK : SPARQ_ELAUNCH;
}

int sparq_async_error(void* workspace, int32_t* host_flag, void* hip_stream) {
  if (!workspace || !host_flag) return SPARQ_EINVAL;
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  if (hipMemcpyAsync(host_flag, workspace, sizeof(int32_t), hipMemcpyDeviceToHost, s) != hipSuccess) return SPARQ_ELAUNCH;
  if (launch_clear(workspace, kWorkspaceHeader, s) != hipSuccess) return SPARQ_ELAUNCH;
  return hipStreamSynchronize(s) == hipSuccess ? SPARQ_OK : SPARQ_ELAUNCH;
}

int sparq_copy_probe(void* dst, const void* src, size_t n_bytes, void* hip_stream) {
  if (!dst || !src || !aligned16(dst) || !aligned16(src) || n_bytes % 16 != 0) return SPARQ_EINVAL;
  return launch_copy_probe(dst, src, n_bytes, static_cast<hipStream_t>(hip_stream)) == hipSuccess ? SPARQ_OK : SPARQ_ELAUNCH;
}

int sparq_read_probe(const void* src, size_t n_bytes, void* sink, size_t sink_bytes, void* hip_stream) {
  if (!src || !sink || !aligned16(src) || !aligned16(sink) || n_bytes % 16 != 0) return SPARQ_EINVAL;
  if (sink_bytes < (size_t)kProbeBlocks * 256 * sizeof(uint32_t)) return SPARQ_EWORKSPACE;
  return launch_read_probe(src, n_bytes, sink, static_cast<hipStream_t>(hip_stream)) == hipSuccess ? SPARQ_OK : SPARQ_ELAUNCH;
}

const char* sparq_decode_plan(const sparq_shape* caller_shape) {
  if (check_shape(caller_shape) != SPARQ_OK) return "invalid shape";
  const sparq_shape sized = bounded(caller_shape);
  const sparq_shape* shape = &sized;
  switch (choose_plan(shape).plan) {
    case kPlanFused: return "sparq_decode_fused (one workgroup per head, one launch)";
    case kPlanLong: return "long_scores + long_merge + split_gather + split_combine (two-level selection plan)";
    case kPlanBucket: return "bk_scores + bk_select_gather + bk_combine (digit-bucket plan)";
    case kPlanShared: return "sparq_decode_shared (grouped-query rule, one workgroup per KV head)";
    case kPlanSharedBucket: return "gs_logits + bk_group_scores + bk_select_gather + bk_combine (grouped-query rule on the digit-bucket plan)";
    case kPlanSharedSplit: return "gs_logits + gs_select + gs_merge + gs_gather + split_combine (grouped-query rule, several workgroups per KV head)";
    case kPlanSingleK: return "sparq_decode_single_k (key cache stored once)";
    default: return "unsupported";
  }
}

int sparq_stage_clocks(const sparq_shape* caller_shape, size_t* offset_bytes, int32_t* n_workgroups, int32_t* stamps_per_workgroup) {
  if (!offset_bytes || !n_workgroups || !stamps_per_workgroup) return SPARQ_EINVAL;
  const int rc = check_shape(caller_shape);
  if (rc != SPARQ_OK) return rc;
#ifdef SPARQ_STAGE_CLOCKS
  const sparq_shape sized = bounded(caller_shape);
  const sparq_shape* shape = &sized;
  if (choose_plan(shape).plan != kPlanFused) return SPARQ_EUNSUPPORTED;
  *offset_bytes = kControlBytes; *n_workgroups = shape->B * shape->H; *stamps_per_workgroup = kStageStamps;
  return SPARQ_OK;
#else
  return SPARQ_EUNSUPPORTED;
#endif
}

const char* sparq_status_string(int status) {
  switch (status) {
    case SPARQ_OK: return "ok";
    case SPARQ_EINVAL: return "invalid argument";
    case SPARQ_EUNSUPPORTED: return "unsupported shape or mode";
    case SPARQ_EWORKSPACE: return "workspace missing, misaligned or too small";
    case SPARQ_ELAUNCH: return "HIP launch failed";
    case SPARQ_ETOOLARGE: return "shape needs more scratch than the library's built-in buffer holds";
    default: return "unknown status";
  }
}

}  // extern "C"
