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
  if (s->flags & ~(uint32_t)(SPARQ_FLAG_NO_REALLOC | SPARQ_FLAG_GQA_SHARED)) return SPARQ_EINVAL;
  if (s->d_h != 64 && s->d_h != 128 && s->d_h != 256) return SPARQ_EUNSUPPORTED;
  // element offsets inside one tensor are formed in size_t; the counts themselves stay in int32
  if ((int64_t)s->B * s->H > (int64_t)1 << 30) return SPARQ_EUNSUPPORTED;
  return SPARQ_OK;
}

int check_cache(const sparq_cache* c) {
  if (!c || !c->K || !c->Kt || !c->V || !c->v_mean || !c->seq_lens) return SPARQ_EINVAL;
  if (!aligned16(c->K) || !aligned16(c->Kt) || !aligned16(c->V) || !aligned16(c->v_mean)) return SPARQ_EINVAL;
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

size_t workspace_need(const sparq_shape* s) {
  int n_split, rows;
  dense_plan(s, &n_split, &rows);
  return (size_t)kWorkspaceHeader + (size_t)s->B * s->H * n_split * (s->d_h + 2) * sizeof(float);
}

int check_workspace(const sparq_shape* s, const void* ws, size_t bytes) {
  if (!ws || !aligned16(ws) || bytes < workspace_need(s)) return SPARQ_EWORKSPACE;
  return SPARQ_OK;
}

int max_lds_bytes() {
  static int cached = -1;   // same for every device of one machine; benign race
  if (cached < 0) {
    int dev = 0, v = 0;
    if (hipGetDevice(&dev) != hipSuccess) return 0;
    if (hipDeviceGetAttribute(&v, hipDeviceAttributeMaxSharedMemoryPerBlock, dev) != hipSuccess) return 0;
    cached = v;
  }
  return cached;
}

}  // namespace

extern "C" {

int sparq_workspace_bytes(const sparq_shape* shape, size_t* out_bytes) {
  int rc = check_shape(shape);
  if (rc != SPARQ_OK) return rc;
  if (!out_bytes) return SPARQ_EINVAL;
  *out_bytes = workspace_need(shape);
  return SPARQ_OK;
}

int sparq_workspace_init(void* workspace, size_t workspace_bytes, void* hip_stream) {
  if (!workspace || !aligned16(workspace) || workspace_bytes < (size_t)kWorkspaceHeader) return SPARQ_EWORKSPACE;
  return launch_clear_header(workspace, static_cast<hipStream_t>(hip_stream)) == hipSuccess ? SPARQ_OK : SPARQ_ELAUNCH;
}

int sparq_kv_append(const sparq_shape* shape, const sparq_cache* cache, const void* k_new,
                    const void* v_new, int32_t n_new, const int32_t* n_new_per_seq,
                    void* workspace, size_t workspace_bytes, void* hip_stream) {
  int rc = check_shape(shape);
  if (rc == SPARQ_OK) rc = check_cache(cache);
  if (rc != SPARQ_OK) return rc;
  if (!k_new || !v_new || !aligned16(k_new) || !aligned16(v_new) || n_new < 1 || n_new > shape->S_max) return SPARQ_EINVAL;
  rc = check_workspace(shape, workspace, workspace_bytes);
  if (rc != SPARQ_OK) return rc;
  AppendArgs a;
  a.K = cache->K; a.Kt = cache->Kt; a.V = cache->V; a.v_mean = cache->v_mean; a.seq_lens = cache->seq_lens;
  a.k_new = k_new; a.v_new = v_new; a.n_new_per_seq = n_new_per_seq; a.err = static_cast<int32_t*>(workspace);
  a.B = shape->B; a.H_kv = shape->H_kv; a.S_max = shape->S_max; a.d_h = shape->d_h; a.n_new = n_new;
  return launch_append(a, shape->dtype, static_cast<hipStream_t>(hip_stream)) == hipSuccess ? SPARQ_OK : SPARQ_ELAUNCH;
}

int sparq_decode(const sparq_shape* shape, const sparq_cache* cache, const void* q,
                 const int32_t* k_per_seq, void* out, float* alpha_out, int32_t* idx_out,
                 int32_t idx_stride, int32_t* chan_out, void* workspace, size_t workspace_bytes,
                 void* hip_stream) {
  int rc = check_shape(shape);
  if (rc == SPARQ_OK) rc = check_cache(cache);
  if (rc != SPARQ_OK) return rc;
  if (!q || !out || !aligned16(q) || !aligned16(out)) return SPARQ_EINVAL;
  if (idx_out && idx_stride < 1) return SPARQ_EINVAL;
  rc = check_workspace(shape, workspace, workspace_bytes);
  if (rc != SPARQ_OK) return rc;
  if (shape->flags & SPARQ_FLAG_GQA_SHARED) return SPARQ_EUNSUPPORTED;
  // the fused kernel keeps one 4-byte key per cached position in LDS
  if (decode_lds_bytes(shape->S_max, shape->d_h) > (size_t)max_lds_bytes()) return SPARQ_EUNSUPPORTED;
  DecodeArgs a;
  a.K = cache->K; a.Kt = cache->Kt; a.V = cache->V; a.v_mean = cache->v_mean; a.seq_lens = cache->seq_lens;
  a.q = q; a.k_per_seq = k_per_seq; a.out = out; a.alpha_out = alpha_out; a.idx_out = idx_out;
  a.k_new = nullptr; a.v_new = nullptr; a.v_mean_next = nullptr; a.seq_lens_next = nullptr;
  a.chan_out = chan_out; a.err = static_cast<int32_t*>(workspace);
  a.B = shape->B; a.H = shape->H; a.H_kv = shape->H_kv; a.S_max = shape->S_max; a.d_h = shape->d_h;
  a.r = shape->r; a.k = shape->k; a.idx_stride = idx_out ? idx_stride : 0; a.flags = shape->flags;
  return launch_decode(a, shape->dtype, static_cast<hipStream_t>(hip_stream)) == hipSuccess ? SPARQ_OK : SPARQ_ELAUNCH;
}

int sparq_decode_step(const sparq_shape* shape, const sparq_cache* cache, const void* k_new,
                      const void* v_new, float* v_mean_next, int32_t* seq_lens_next, const void* q,
                      const int32_t* k_per_seq, void* out, float* alpha_out, int32_t* idx_out,
                      int32_t idx_stride, int32_t* chan_out, void* workspace, size_t workspace_bytes,
                      void* hip_stream) {
  int rc = check_shape(shape);
  if (rc == SPARQ_OK) rc = check_cache(cache);
  if (rc != SPARQ_OK) return rc;
  if (!q || !out || !aligned16(q) || !aligned16(out)) return SPARQ_EINVAL;
  if (!k_new || !v_new || !aligned16(k_new) || !aligned16(v_new)) return SPARQ_EINVAL;
  if (!v_mean_next || !seq_lens_next || !aligned16(v_mean_next)) return SPARQ_EINVAL;
  if (v_mean_next == cache->v_mean || seq_lens_next == cache->seq_lens) return SPARQ_EINVAL;
  if (idx_out && idx_stride < 1) return SPARQ_EINVAL;
  rc = check_workspace(shape, workspace, workspace_bytes);
  if (rc != SPARQ_OK) return rc;
  if (shape->flags & SPARQ_FLAG_GQA_SHARED) return SPARQ_EUNSUPPORTED;
  if (decode_lds_bytes(shape->S_max, shape->d_h) > (size_t)max_lds_bytes()) return SPARQ_EUNSUPPORTED;
  DecodeArgs a;
  a.K = cache->K; a.Kt = cache->Kt; a.V = cache->V; a.v_mean = cache->v_mean; a.seq_lens = cache->seq_lens;
  a.q = q; a.k_per_seq = k_per_seq; a.out = out; a.alpha_out = alpha_out; a.idx_out = idx_out;
  a.k_new = k_new; a.v_new = v_new; a.v_mean_next = v_mean_next; a.seq_lens_next = seq_lens_next;
  a.chan_out = chan_out; a.err = static_cast<int32_t*>(workspace);
  a.B = shape->B; a.H = shape->H; a.H_kv = shape->H_kv; a.S_max = shape->S_max; a.d_h = shape->d_h;
  a.r = shape->r; a.k = shape->k; a.idx_stride = idx_out ? idx_stride : 0; a.flags = shape->flags;
  return launch_decode(a, shape->dtype, static_cast<hipStream_t>(hip_stream)) == hipSuccess ? SPARQ_OK : SPARQ_ELAUNCH;
}

int dense_decode(const sparq_shape* shape, const sparq_cache* cache, const void* q, void* out,
                 void* workspace, size_t workspace_bytes, void* hip_stream) {
  int rc = check_shape(shape);
  if (rc == SPARQ_OK) rc = check_cache(cache);
  if (rc != SPARQ_OK) return rc;
  if (!q || !out || !aligned16(q) || !aligned16(out)) return SPARQ_EINVAL;
  rc = check_workspace(shape, workspace, workspace_bytes);
  if (rc != SPARQ_OK) return rc;
  DenseArgs a;
  a.K = cache->K; a.V = cache->V; a.seq_lens = cache->seq_lens; a.q = q; a.out = out;
  a.partials = reinterpret_cast<float*>(static_cast<char*>(workspace) + kWorkspaceHeader);
  a.err = static_cast<int32_t*>(workspace);
  a.B = shape->B; a.H = shape->H; a.H_kv = shape->H_kv; a.S_max = shape->S_max; a.d_h = shape->d_h;
  dense_plan(shape, &a.n_split, &a.rows_per_split);
  return launch_dense(a, shape->dtype, static_cast<hipStream_t>(hip_stream)) == hipSuccess ? SPARQ_OK : SPARQ_ELAUNCH;
}

int sparq_async_error(void* workspace, int32_t* host_flag, void* hip_stream) {
  if (!workspace || !host_flag) return SPARQ_EINVAL;
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  if (hipMemcpyAsync(host_flag, workspace, sizeof(int32_t), hipMemcpyDeviceToHost, s) != hipSuccess) return SPARQ_ELAUNCH;
  if (launch_clear_header(workspace, s) != hipSuccess) return SPARQ_ELAUNCH;
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

const char* sparq_status_string(int status) {
  switch (status) {
    case SPARQ_OK: return "ok";
    case SPARQ_EINVAL: return "invalid argument";
    case SPARQ_EUNSUPPORTED: return "unsupported shape or mode";
    case SPARQ_EWORKSPACE: return "workspace missing, misaligned or too small";
    case SPARQ_ELAUNCH: return "HIP launch failed";
    default: return "unknown status";
  }
}

}  // extern "C"
