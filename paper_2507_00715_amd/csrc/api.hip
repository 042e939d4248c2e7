// C ABI of libearn: argument validation on the host, then kernel launches on the caller's stream.
#include <math.h>
#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include <atomic>
#include <vector>

#include "common.h"

namespace earn {

static thread_local char g_err[512] = "";

void set_error(const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
}

RopeTable make_rope_table(float base, int head_dim) {
  // every entry point asks for the table on every call, nearly always for the same model: keep the last one per thread
  // (64 calls of pow() cost about as much host time as a kernel launch)
  static thread_local RopeTable cached;
  static thread_local float cached_base = 0.f;
  static thread_local int cached_dim = 0;
  if (base > 0.f && base == cached_base && head_dim == cached_dim) return cached;
  RopeTable t;
  memset(&t, 0, sizeof(t));
  t.enabled = base > 0.f ? 1 : 0;
  if (!t.enabled) return t;
  const double two_pi = 6.283185307179586476925286766559;
  for (int e = 0; e < head_dim / 2 && e < kMaxHalfDim; ++e) {
    double turns = pow((double)base, -2.0 * (double)e / (double)head_dim) / two_pi;
    float hi = (float)turns;
    t.hi[e] = hi;
    t.lo[e] = (float)(turns - (double)hi);
  }
  cached = t; cached_base = base; cached_dim = head_dim;
  return t;
}

int launch_compact(int n_tensors, const void* const* src, void* const* dst, const int64_t* row_bytes,
                   const int32_t* cu_seqlens, int batch, int total_tokens, int h, int t, int32_t* idx_out,
                   int32_t* pos_out, int32_t* cu_out, hipStream_t stream);
int launch_prefill(const earn_attn_desc* desc, const void* q, const void* k, const void* v, const int32_t* cu_seqlens,
                   const int32_t* positions, int batch, int total_tokens, int max_seqlen, void* out, void* k_rot_out,
                   float* lse_out, void* workspace, size_t workspace_bytes, hipStream_t stream,
                   const PrefillLayers* layers);
size_t prefill_workspace_bytes(const earn_attn_desc* desc, int total_tokens, int have_k_rot_out);
int launch_decode(const earn_attn_desc* desc, const void* q, const void* k_new, const void* v_new,
                  const int32_t* q_pos, const void* shared_k, const void* shared_v, const int32_t* shared_cu,
                  const int32_t* stream_to_seq, void* gen_k, void* gen_v, const int32_t* gen_len, int gen_cap,
                  int n_streams, int batch, int max_shared_len, int shared_total, void* out, void* workspace,
                  size_t workspace_bytes, hipStream_t stream, const DecodeLayers* layers, const int32_t* gen_src);
size_t beam_topk_workspace_bytes(int batch, int beams, int vocab);
int launch_beam_topk(const float* beam_scores, const float* logp, int batch, int beams, int vocab, int32_t* parent,
                     int32_t* token, float* score, void* workspace, hipStream_t stream);
int launch_beam_reorder(const int32_t* parent, const int32_t* src_in, int32_t* src_out, int n_streams, int gen_cap, int step,
                        hipStream_t stream);
int beam_topk_limits(int beams, int vocab, const char** why);
size_t decode_workspace_bytes(int dtype, int hq, int hkv, int d, int n_streams, int batch, int max_shared_len,
                              int gen_cap, int n_layers);
int launch_decode_static(const earn_attn_desc* desc, const void* q, const void* k_new, const void* v_new,
                         const int32_t* q_pos, const void* shared_k, const void* shared_v, const int32_t* shared_cu,
                         const int32_t* stream_to_seq, void* gen_k, void* gen_v, const int32_t* gen_len, int gen_cap,
                         int n_streams, int batch, int max_shared_len, int shared_total, void* out, hipStream_t stream);
int launch_step_positions(const int32_t* cu, const int32_t* stream_to_seq, int n_streams, int batch, int step,
                          int32_t* q_pos, int32_t* gen_len, hipStream_t stream);
int launch_attn_stats(const earn_attn_desc* desc, const void* q_rows, const void* k_rot, const int32_t* cu_seqlens,
                      const int32_t* row_pos, int batch, int total_tokens, int rows_per_seq, float epsilon, int t_head,
                      int tail_back, float* stats_out, hipStream_t stream);
int launch_linear(const void* x, const void* w, int rows, int k, int n, int activation, void* out, void* workspace,
                  size_t workspace_bytes, hipStream_t stream);
size_t linear_workspace_bytes(long long rows, int k, int n);
int launch_qkv_rope_project(const earn_attn_desc* desc, const void* x, const void* w_qkv, int rows, int d_model,
                            const int32_t* cu_seqlens, const int32_t* positions, int batch, void* q_out, void* k_out,
                            void* v_out, void* workspace, size_t workspace_bytes, hipStream_t stream);
size_t attn_backward_workspace_bytes(int hq, int total_tokens);
int launch_attn_backward(const earn_attn_desc* desc, const void* q, const void* k, const void* v, const void* out,
                         const float* lse, const void* d_out, const int32_t* cu_seqlens, int batch, int total_tokens,
                         int max_seqlen, void* dq, void* dk, void* dv, void* workspace, hipStream_t stream);
int launch_rope_keys(const earn_attn_desc* desc, const void* k, void* k_rot, const int32_t* cu_seqlens,
                     const int32_t* positions, int batch, int total_tokens, hipStream_t stream);
int launch_prefill_rows_f32(const earn_attn_desc* desc, const void* q_rows, const void* k_rot, const void* v,
                            const int32_t* cu_seqlens, const int32_t* row_pos, int batch, int total_tokens,
                            int max_seqlen, int rows_per_seq, void* out_rows, hipStream_t stream);
size_t prefill_rows_workspace_bytes(int hq, int hkv, int d, int batch, int max_seqlen, int rows_per_seq);
int launch_prefill_rows(const earn_attn_desc* desc, const void* q_rows, const void* k_rot, const void* v,
                        const int32_t* cu_seqlens, const int32_t* row_pos, int batch, int total_tokens, int max_seqlen,
                        int rows_per_seq, void* out_rows, void* workspace, size_t workspace_bytes, hipStream_t stream);

static std::atomic<int> g_tuning[kTuneCount];
int tuning(Tuning t, int dflt) {
  const int v = g_tuning[t].load(std::memory_order_relaxed);
  return v > 0 ? v : dflt;
}

int make_head_map(const earn_attn_desc* d, HeadMap* m, const char* who) {
  memset(m, 0, sizeof(*m));
  if (!d->q_to_kv) return EARN_OK;
  const int hq = d->n_q_heads, hkv = d->n_kv_heads, gq = hq / hkv;
  if (hq > kMaxMappedHeads) { set_error("%s: an explicit q_to_kv map takes at most %d query heads", who, kMaxMappedHeads); return EARN_ERR_UNSUPPORTED; }
  int count[kMaxMappedHeads] = {0};
  bool identity = true;
  for (int a = 0; a < hq; ++a) {
    const int c = d->q_to_kv[a];
    if (c < 0 || c >= hkv) { set_error("%s: q_to_kv[%d] = %d outside [0, %d)", who, a, c, hkv); return EARN_ERR_INVALID_ARG; }
    if (count[c] >= gq) {
      set_error("%s: q_to_kv gives kv head %d more than Hq/Hkv = %d query heads (groups of unequal size are not supported)", who, c, gq);
      return EARN_ERR_UNSUPPORTED;
    }
    m->q_of_slot[c * gq + count[c]++] = (unsigned char)a;
    identity = identity && c == a / gq;
  }
  m->enabled = identity ? 0 : 1;
  return EARN_OK;
}

static int check_desc(const earn_attn_desc* d, const char* who) {
  if (!d) { set_error("%s: desc is NULL", who); return EARN_ERR_INVALID_ARG; }
  if (d->dtype != EARN_F32 && d->dtype != EARN_BF16) { set_error("%s: unknown dtype %d", who, d->dtype); return EARN_ERR_UNSUPPORTED; }
  if (d->n_q_heads <= 0 || d->n_kv_heads <= 0) { set_error("%s: head counts must be positive", who); return EARN_ERR_INVALID_ARG; }
  if (d->n_q_heads % d->n_kv_heads != 0) {
    set_error("%s: n_q_heads (%d) is not a multiple of n_kv_heads (%d)", who, d->n_q_heads, d->n_kv_heads);
    return d->q_to_kv ? EARN_ERR_UNSUPPORTED : EARN_ERR_INVALID_ARG;
  }
  if (d->head_dim != 64 && d->head_dim != 128) { set_error("%s: head_dim %d not in {64,128}", who, d->head_dim); return EARN_ERR_UNSUPPORTED; }
  HeadMap m;
  return make_head_map(d, &m, who);
}

// ---- debug validation of the preconditions that live in device memory ----
static std::atomic<int> g_validate{0};

// copies n int32 from device to host on the stream and waits for it
static int fetch_i32(const int32_t* dev, size_t n, std::vector<int32_t>& host, hipStream_t stream, const char* who) {
  host.resize(n);
  if (n == 0) return EARN_OK;
  if (hipMemcpyAsync(host.data(), dev, n * sizeof(int32_t), hipMemcpyDeviceToHost, stream) != hipSuccess ||
      hipStreamSynchronize(stream) != hipSuccess) {
    set_error("%s: validation could not read a device array", who);
    return EARN_ERR_HIP;
  }
  return EARN_OK;
}
// cu[0] == 0, non-decreasing, every length <= max_len, cu[batch] == total (total < 0: not checked)
static int validate_cu(const char* who, const char* name, const std::vector<int32_t>& cu, int batch, long long total,
                       int max_len) {
  if (cu[0] != 0) { set_error("%s: %s[0] = %d, must be 0", who, name, cu[0]); return EARN_ERR_INVALID_ARG; }
  for (int s = 0; s < batch; ++s) {
    if (cu[s + 1] < cu[s]) { set_error("%s: %s decreases at %d (%d -> %d)", who, name, s, cu[s], cu[s + 1]); return EARN_ERR_INVALID_ARG; }
    if (cu[s + 1] - cu[s] > max_len) {
      set_error("%s: sequence %d has %d rows, more than the bound %d passed by value", who, s, cu[s + 1] - cu[s], max_len);
      return EARN_ERR_INVALID_ARG;
    }
  }
  if (total >= 0 && cu[batch] != total) { set_error("%s: %s[batch] = %d, expected %lld", who, name, cu[batch], total); return EARN_ERR_INVALID_ARG; }
  return EARN_OK;
}
static int validate_positions(const char* who, const char* name, const std::vector<int32_t>& p) {
  for (size_t i = 0; i < p.size(); ++i)
    if (p[i] < 0 || p[i] >= (1 << 24)) { set_error("%s: %s[%zu] = %d outside [0, 2^24)", who, name, i, p[i]); return EARN_ERR_INVALID_ARG; }
  return EARN_OK;
}

static int validate_decode(const char* who, const int32_t* q_pos, const int32_t* shared_cu, const int32_t* stream_to_seq,
                           const int32_t* gen_len, int gen_cap, int n_streams, int batch, int max_shared_len,
                           int shared_total, hipStream_t stream) {
  std::vector<int32_t> cu, qp, gl, s2s;
  int rc;
  if ((rc = fetch_i32(shared_cu, (size_t)batch + 1, cu, stream, who)) != EARN_OK) return rc;
  if ((rc = validate_cu(who, "shared_cu", cu, batch, -1, max_shared_len)) != EARN_OK) return rc;
  if (cu[batch] > shared_total) {
    set_error("%s: shared_cu[batch] = %d, more than the %d rows of the shared tensors", who, cu[batch], shared_total);
    return EARN_ERR_INVALID_ARG;
  }
  if ((rc = fetch_i32(q_pos, (size_t)n_streams, qp, stream, who)) != EARN_OK) return rc;
  if ((rc = validate_positions(who, "q_pos", qp)) != EARN_OK) return rc;
  if ((rc = fetch_i32(gen_len, (size_t)n_streams, gl, stream, who)) != EARN_OK) return rc;
  for (int u = 0; u < n_streams; ++u)
    if (gl[u] < 0 || gl[u] >= gen_cap) { set_error("%s: gen_len[%d] = %d outside [0, gen_cap = %d)", who, u, gl[u], gen_cap); return EARN_ERR_INVALID_ARG; }
  if (stream_to_seq) {
    if ((rc = fetch_i32(stream_to_seq, (size_t)n_streams, s2s, stream, who)) != EARN_OK) return rc;
    std::vector<int32_t> per_seq((size_t)batch, 0);
    for (int u = 0; u < n_streams; ++u) {
      if (s2s[u] < 0 || s2s[u] >= batch) { set_error("%s: stream_to_seq[%d] = %d outside [0, batch = %d)", who, u, s2s[u], batch); return EARN_ERR_INVALID_ARG; }
      if (++per_seq[s2s[u]] > 1024) { set_error("%s: sequence %d holds more than 1024 streams", who, s2s[u]); return EARN_ERR_INVALID_ARG; }
    }
  }
  return EARN_OK;
}

}  // namespace earn

using namespace earn;

extern "C" {

const char* earn_last_error(void) { return g_err; }

const char* earn_version(void) { return "libearn 0.2 (gfx950)"; }

int earn_set_validation(int enabled) { return g_validate.exchange(enabled ? 1 : 0); }

int earn_set_tuning(const char* key, int32_t value) {
  static const char* const names[kTuneCount] = {"prefill_block_rows", "decode_mfma_min_len", "decode_mfma_short_wgs",
                                                "decode_mfma_wgs", "decode_vec_wgs", "decode_vec_waves", "compact_blocks", "linear_tile", "linear_splits"};
  g_err[0] = 0;
  for (int i = 0; key && i < kTuneCount; ++i)
    if (strcmp(key, names[i]) == 0) { g_tuning[i].store(value > 0 ? value : 0, std::memory_order_relaxed); return EARN_OK; }
  set_error("earn_set_tuning: unknown key '%s'", key ? key : "(null)");
  return EARN_ERR_INVALID_ARG;
}

size_t earn_prefill_workspace_bytes(const earn_attn_desc* desc, int32_t batch, int32_t total_tokens,
                                    int32_t max_seqlen, int32_t have_k_rot_out) {
  (void)batch; (void)max_seqlen;
  if (check_desc(desc, "earn_prefill_workspace_bytes") != EARN_OK || total_tokens < 0) return 0;
  return prefill_workspace_bytes(desc, total_tokens, have_k_rot_out);
}

static int prefill_entry(const char* who, const earn_attn_desc* desc, const void* q, const void* k, const void* v,
                         const int32_t* cu_seqlens, const int32_t* positions, int32_t batch, int32_t total_tokens,
                         int32_t max_seqlen, void* out, void* k_rot_out, float* lse_out, void* workspace,
                         size_t workspace_bytes, void* stream, const PrefillLayers* layers) {
  g_err[0] = 0;
  int rc = check_desc(desc, who);
  if (rc != EARN_OK) return rc;
  if (batch <= 0 || total_tokens < 0 || max_seqlen <= 0) {
    set_error("%s: batch (%d) and max_seqlen (%d) must be positive, total_tokens (%d) non-negative", who, batch, max_seqlen, total_tokens);
    return EARN_ERR_INVALID_ARG;
  }
  if (!cu_seqlens) { set_error("%s: cu_seqlens is NULL", who); return EARN_ERR_INVALID_ARG; }
  if (total_tokens == 0) return EARN_OK;
  if (!q || !k || !v || !out) { set_error("%s: q, k, v and out must not be NULL", who); return EARN_ERR_INVALID_ARG; }
  if (g_validate.load(std::memory_order_relaxed)) {
    std::vector<int32_t> cu, pos;
    if ((rc = fetch_i32(cu_seqlens, (size_t)batch + 1, cu, (hipStream_t)stream, who)) != EARN_OK) return rc;
    if ((rc = validate_cu(who, "cu_seqlens", cu, batch, total_tokens, max_seqlen)) != EARN_OK) return rc;
    if (positions) {
      if ((rc = fetch_i32(positions, (size_t)total_tokens, pos, (hipStream_t)stream, who)) != EARN_OK) return rc;
      if ((rc = validate_positions(who, "positions", pos)) != EARN_OK) return rc;
    }
  }
  if (max_seqlen > total_tokens) max_seqlen = total_tokens;
  return launch_prefill(desc, q, k, v, cu_seqlens, positions, batch, total_tokens, max_seqlen, out, k_rot_out, lse_out,
                        workspace, workspace_bytes, (hipStream_t)stream, layers);
}

int earn_prefill_attn(const earn_attn_desc* desc, const void* q, const void* k, const void* v,
                      const int32_t* cu_seqlens, const int32_t* positions, int32_t batch, int32_t total_tokens,
                      int32_t max_seqlen, void* out, void* k_rot_out, float* lse_out, void* workspace,
                      size_t workspace_bytes, void* stream) {
  return prefill_entry("earn_prefill_attn", desc, q, k, v, cu_seqlens, positions, batch, total_tokens, max_seqlen, out,
                       k_rot_out, lse_out, workspace, workspace_bytes, stream, nullptr);
}

static int check_layer_stride(const char* who, const char* name, int64_t stride, int n_layers, int align = 16) {
  if (n_layers > 1 && (stride <= 0 || stride % align != 0)) {
    set_error("%s: %s = %lld must be a positive multiple of %d bytes", who, name, (long long)stride, align);
    return EARN_ERR_INVALID_ARG;
  }
  return EARN_OK;
}

int earn_prefill_attn_layers(const earn_attn_desc* desc, int32_t n_layers, const void* q, int64_t q_layer_stride,
                             const void* k, const void* v, int64_t kv_layer_stride, const int32_t* cu_seqlens,
                             const int32_t* positions, int32_t batch, int32_t total_tokens, int32_t max_seqlen,
                             void* out, int64_t out_layer_stride, void* k_rot_out, int64_t k_rot_layer_stride,
                             float* lse_out, int64_t lse_layer_stride, void* workspace, size_t workspace_bytes,
                             void* stream) {
  const char* who = "earn_prefill_attn_layers";
  g_err[0] = 0;
  if (n_layers <= 0 || n_layers > 65535) { set_error("%s: n_layers (%d) outside [1, 65535]", who, n_layers); return EARN_ERR_INVALID_ARG; }
  if (!k_rot_out) { set_error("%s: k_rot_out is required (every layer keeps its rotated keys)", who); return EARN_ERR_INVALID_ARG; }
  int rc;
  if ((rc = check_layer_stride(who, "q_layer_stride", q_layer_stride, n_layers)) != EARN_OK ||
      (rc = check_layer_stride(who, "kv_layer_stride", kv_layer_stride, n_layers)) != EARN_OK ||
      (rc = check_layer_stride(who, "out_layer_stride", out_layer_stride, n_layers)) != EARN_OK ||
      (rc = check_layer_stride(who, "k_rot_layer_stride", k_rot_layer_stride, n_layers)) != EARN_OK ||
      (lse_out && (rc = check_layer_stride(who, "lse_layer_stride", lse_layer_stride, n_layers, 4)) != EARN_OK))
    return rc;
  const PrefillLayers layers = {n_layers, q_layer_stride, kv_layer_stride, out_layer_stride, k_rot_layer_stride, lse_layer_stride};
  return prefill_entry(who, desc, q, k, v, cu_seqlens, positions, batch, total_tokens, max_seqlen, out, k_rot_out, lse_out,
                       workspace, workspace_bytes, stream, &layers);
}

int earn_compact_registers(int32_t n_tensors, const void* const* src, void* const* dst, const int64_t* row_bytes,
                           const int32_t* cu_seqlens, int32_t batch, int32_t total_tokens, int32_t n_head_reg,
                           int32_t n_tail_reg, int32_t* idx_out, int32_t* pos_out, int32_t* cu_out, void* stream) {
  g_err[0] = 0;
  if (batch <= 0 || total_tokens < 0) { set_error("earn_compact_registers: batch must be positive, total_tokens non-negative"); return EARN_ERR_INVALID_ARG; }
  if (n_head_reg < 0 || n_tail_reg < 0 || n_head_reg + n_tail_reg == 0) {
    set_error("earn_compact_registers: register counts must be non-negative and not both zero (h=%d, t=%d)", n_head_reg, n_tail_reg);
    return EARN_ERR_INVALID_ARG;
  }
  if (n_tensors < 0 || n_tensors > EARN_MAX_COMPACT_TENSORS) {
    set_error("earn_compact_registers: n_tensors %d outside [0, %d]", n_tensors, EARN_MAX_COMPACT_TENSORS);
    return EARN_ERR_INVALID_ARG;
  }
  if (!cu_seqlens) { set_error("earn_compact_registers: cu_seqlens is NULL"); return EARN_ERR_INVALID_ARG; }
  if ((long long)batch * (n_head_reg + n_tail_reg) > 0x7fffffffLL) { set_error("earn_compact_registers: too many rows"); return EARN_ERR_INVALID_ARG; }
  if (n_tensors > 0 && (!src || !dst || !row_bytes)) { set_error("earn_compact_registers: src, dst and row_bytes must not be NULL"); return EARN_ERR_INVALID_ARG; }
  for (int i = 0; i < n_tensors; ++i) {
    if (!src[i] || !dst[i]) { set_error("earn_compact_registers: tensor %d has a NULL pointer", i); return EARN_ERR_INVALID_ARG; }
    if (((uintptr_t)src[i] | (uintptr_t)dst[i]) & 15) { set_error("earn_compact_registers: tensor %d is not 16-byte aligned", i); return EARN_ERR_INVALID_ARG; }
    if (row_bytes[i] <= 0 || row_bytes[i] % 16 != 0 || row_bytes[i] / 16 > 0x7fffffffLL) {
      set_error("earn_compact_registers: row_bytes[%d] = %lld is not a positive multiple of 16", i, (long long)row_bytes[i]);
      return EARN_ERR_INVALID_ARG;
    }
  }
  if (g_validate.load(std::memory_order_relaxed)) {
    const char* who = "earn_compact_registers";
    std::vector<int32_t> cu;
    int rc = fetch_i32(cu_seqlens, (size_t)batch + 1, cu, (hipStream_t)stream, who);
    if (rc != EARN_OK) return rc;
    if ((rc = validate_cu(who, "cu_seqlens", cu, batch, -1, 0x7fffffff)) != EARN_OK) return rc;
    for (int s = 0; s < batch; ++s)
      if (cu[s + 1] - cu[s] < n_head_reg + n_tail_reg) {
        set_error("%s: sequence %d has %d rows, fewer than h + t = %d", who, s, cu[s + 1] - cu[s], n_head_reg + n_tail_reg);
        return EARN_ERR_INVALID_ARG;
      }
  }
  return launch_compact(n_tensors, src, dst, row_bytes, cu_seqlens, batch, total_tokens, n_head_reg, n_tail_reg, idx_out,
                        pos_out, cu_out, (hipStream_t)stream);
}

int earn_decode_step_positions(const int32_t* cu_seqlens, const int32_t* stream_to_seq, int32_t n_streams,
                               int32_t batch, int32_t step, int32_t* q_pos, int32_t* gen_len, void* stream) {
  g_err[0] = 0;
  if (!cu_seqlens || n_streams <= 0 || batch <= 0 || step < 0) {
    set_error("earn_decode_step_positions: cu_seqlens must not be NULL, n_streams (%d) and batch (%d) positive, step (%d) non-negative", n_streams, batch, step);
    return EARN_ERR_INVALID_ARG;
  }
  if (!stream_to_seq && n_streams != batch) {
    set_error("earn_decode_step_positions: stream_to_seq is NULL but n_streams (%d) != batch (%d)", n_streams, batch);
    return EARN_ERR_INVALID_ARG;
  }
  if (!q_pos && !gen_len) return EARN_OK;
  return launch_step_positions(cu_seqlens, stream_to_seq, n_streams, batch, step, q_pos, gen_len, (hipStream_t)stream);
}

size_t earn_decode_workspace_bytes(const earn_attn_desc* desc, int32_t n_streams, int32_t batch,
                                   int32_t max_shared_len, int32_t gen_cap) {
  if (check_desc(desc, "earn_decode_workspace_bytes") != EARN_OK || n_streams <= 0 || batch <= 0 || max_shared_len < 0 || gen_cap <= 0) return 0;
  return decode_workspace_bytes(desc->dtype, desc->n_q_heads, desc->n_kv_heads, desc->head_dim, n_streams, batch,
                                max_shared_len, gen_cap, 1);
}

// the host-side checks earn_decode_attn and earn_decode_attn_static share
static int check_decode_args(const char* who, const earn_attn_desc* desc, const void* q, const void* k_new,
                             const void* v_new, const int32_t* q_pos, const void* shared_k, const void* shared_v,
                             const int32_t* shared_cu, const int32_t* stream_to_seq, void* gen_k, void* gen_v,
                             const int32_t* gen_len, int32_t gen_cap, int32_t n_streams, int32_t batch,
                             int32_t max_shared_len, int32_t shared_total, void* out, void* stream) {
  g_err[0] = 0;
  int rc = check_desc(desc, who);
  if (rc != EARN_OK) return rc;
  if (n_streams <= 0 || batch <= 0 || gen_cap <= 0 || max_shared_len < 0 || shared_total < 0) {
    set_error("%s: n_streams (%d), batch (%d), gen_cap (%d) must be positive, max_shared_len (%d) and shared_total (%d) non-negative",
              who, n_streams, batch, gen_cap, max_shared_len, shared_total);
    return EARN_ERR_INVALID_ARG;
  }
  if (!q || !k_new || !v_new || !q_pos || !shared_cu || !gen_k || !gen_v || !gen_len || !out) {
    set_error("%s: a required pointer is NULL", who);
    return EARN_ERR_INVALID_ARG;
  }
  if (max_shared_len > 0 && (!shared_k || !shared_v)) { set_error("%s: shared_k/shared_v are NULL but max_shared_len > 0", who); return EARN_ERR_INVALID_ARG; }
  if (!stream_to_seq && n_streams != batch) { set_error("%s: stream_to_seq is NULL but n_streams (%d) != batch (%d)", who, n_streams, batch); return EARN_ERR_INVALID_ARG; }
  if (g_validate.load(std::memory_order_relaxed) &&
      (rc = validate_decode(who, q_pos, shared_cu, stream_to_seq, gen_len, gen_cap, n_streams, batch, max_shared_len,
                            shared_total, (hipStream_t)stream)) != EARN_OK)
    return rc;
  return EARN_OK;
}

int earn_decode_attn_static(const earn_attn_desc* desc, const void* q, const void* k_new, const void* v_new,
                            const int32_t* q_pos, const void* shared_k, const void* shared_v,
                            const int32_t* shared_cu, const int32_t* stream_to_seq, void* gen_k, void* gen_v,
                            const int32_t* gen_len, int32_t gen_cap, int32_t n_streams, int32_t batch,
                            int32_t max_shared_len, int32_t shared_total, void* out, void* stream) {
  const int rc = check_decode_args("earn_decode_attn_static", desc, q, k_new, v_new, q_pos, shared_k, shared_v, shared_cu,
                                   stream_to_seq, gen_k, gen_v, gen_len, gen_cap, n_streams, batch, max_shared_len, shared_total, out,
                                   stream);
  if (rc != EARN_OK) return rc;
  return launch_decode_static(desc, q, k_new, v_new, q_pos, shared_k, shared_v, shared_cu, stream_to_seq, gen_k, gen_v,
                              gen_len, gen_cap, n_streams, batch, max_shared_len, shared_total, out, (hipStream_t)stream);
}

int earn_decode_attn(const earn_attn_desc* desc, const void* q, const void* k_new, const void* v_new,
                     const int32_t* q_pos, const void* shared_k, const void* shared_v, const int32_t* shared_cu,
                     const int32_t* stream_to_seq, void* gen_k, void* gen_v, const int32_t* gen_len, int32_t gen_cap,
                     int32_t n_streams, int32_t batch, int32_t max_shared_len, int32_t shared_total, void* out, void* workspace,
                     size_t workspace_bytes, void* stream) {
  const int rc = check_decode_args("earn_decode_attn", desc, q, k_new, v_new, q_pos, shared_k, shared_v, shared_cu,
                                   stream_to_seq, gen_k, gen_v, gen_len, gen_cap, n_streams, batch, max_shared_len, shared_total, out,
                                   stream);
  if (rc != EARN_OK) return rc;
  return launch_decode(desc, q, k_new, v_new, q_pos, shared_k, shared_v, shared_cu, stream_to_seq, gen_k, gen_v, gen_len,
                       gen_cap, n_streams, batch, max_shared_len, shared_total, out, workspace, workspace_bytes, (hipStream_t)stream,
                       nullptr, nullptr);
}

int earn_decode_attn_beams(const earn_attn_desc* desc, const void* q, const void* k_new, const void* v_new,
                           const int32_t* q_pos, const void* shared_k, const void* shared_v, const int32_t* shared_cu,
                           const int32_t* stream_to_seq, void* gen_k, void* gen_v, const int32_t* gen_len,
                           const int32_t* gen_src, int32_t gen_cap, int32_t n_streams, int32_t batch,
                           int32_t max_shared_len, int32_t shared_total, void* out, void* workspace, size_t workspace_bytes, void* stream) {
  const int rc = check_decode_args("earn_decode_attn_beams", desc, q, k_new, v_new, q_pos, shared_k, shared_v, shared_cu,
                                   stream_to_seq, gen_k, gen_v, gen_len, gen_cap, n_streams, batch, max_shared_len, shared_total, out,
                                   stream);
  if (rc != EARN_OK) return rc;
  if (gen_src && g_validate.load(std::memory_order_relaxed)) {
    std::vector<int32_t> src;
    int rc2 = fetch_i32(gen_src, (size_t)n_streams * gen_cap, src, (hipStream_t)stream, "earn_decode_attn_beams");
    if (rc2 != EARN_OK) return rc2;
    for (size_t i = 0; i < src.size(); ++i)
      if (src[i] < 0 || src[i] >= n_streams) {
        set_error("earn_decode_attn_beams: gen_src[%zu] = %d outside [0, n_streams = %d)", i, src[i], n_streams);
        return EARN_ERR_INVALID_ARG;
      }
  }
  return launch_decode(desc, q, k_new, v_new, q_pos, shared_k, shared_v, shared_cu, stream_to_seq, gen_k, gen_v, gen_len,
                       gen_cap, n_streams, batch, max_shared_len, shared_total, out, workspace, workspace_bytes, (hipStream_t)stream,
                       nullptr, gen_src);
}

size_t earn_beam_topk_workspace_bytes(int32_t batch, int32_t beams, int32_t vocab) {
  const char* why;
  if (batch <= 0 || beams <= 0 || vocab <= 0 || !beam_topk_limits(beams, vocab, &why)) return 0;
  return beam_topk_workspace_bytes(batch, beams, vocab);
}

int earn_beam_topk(const float* beam_scores, const float* token_logprobs, int32_t batch, int32_t beams, int32_t vocab,
                   int32_t* parent_out, int32_t* token_out, float* score_out, void* workspace, size_t workspace_bytes,
                   void* stream) {
  g_err[0] = 0;
  if (!token_logprobs || !parent_out || !token_out || !score_out || batch <= 0 || beams <= 0 || vocab <= 0 || batch > 65535) {
    set_error("earn_beam_topk: NULL pointer or non-positive size (batch %d, beams %d, vocab %d)", batch, beams, vocab);
    return EARN_ERR_INVALID_ARG;
  }
  const char* why = "";
  if (!beam_topk_limits(beams, vocab, &why)) { set_error("earn_beam_topk: %s", why); return EARN_ERR_UNSUPPORTED; }
  const size_t need = beam_topk_workspace_bytes(batch, beams, vocab);
  if (need > workspace_bytes || (need > 0 && !workspace)) {
    set_error("earn_beam_topk: workspace too small (%zu bytes given, %zu needed)", workspace_bytes, need);
    return EARN_ERR_WORKSPACE_TOO_SMALL;
  }
  return launch_beam_topk(beam_scores, token_logprobs, batch, beams, vocab, parent_out, token_out, score_out, workspace,
                          (hipStream_t)stream);
}

int earn_beam_reorder(const int32_t* parent, const int32_t* gen_src_in, int32_t* gen_src_out, int32_t n_streams,
                      int32_t gen_cap, int32_t step, void* stream) {
  g_err[0] = 0;
  if (!parent || !gen_src_out || gen_src_out == gen_src_in || n_streams <= 0 || gen_cap <= 0 || step < 0 || step >= gen_cap) {
    set_error("earn_beam_reorder: NULL or aliased table, or sizes out of range (n_streams %d, gen_cap %d, step %d)", n_streams, gen_cap, step);
    return EARN_ERR_INVALID_ARG;
  }
  return launch_beam_reorder(parent, gen_src_in, gen_src_out, n_streams, gen_cap, step, (hipStream_t)stream);
}

size_t earn_decode_layers_workspace_bytes(const earn_attn_desc* desc, int32_t n_layers, int32_t n_streams, int32_t batch,
                                          int32_t max_shared_len, int32_t gen_cap) {
  if (check_desc(desc, "earn_decode_layers_workspace_bytes") != EARN_OK || n_layers <= 0 || n_layers > 65535 ||
      n_streams <= 0 || batch <= 0 || max_shared_len < 0 || gen_cap <= 0)
    return 0;
  return decode_workspace_bytes(desc->dtype, desc->n_q_heads, desc->n_kv_heads, desc->head_dim, n_streams, batch,
                                max_shared_len, gen_cap, n_layers);
}

int earn_decode_attn_layers(const earn_attn_desc* desc, int32_t n_layers, const void* q, int64_t q_layer_stride,
                            const void* k_new, const void* v_new, int64_t kv_new_layer_stride, const int32_t* q_pos,
                            const void* shared_k, const void* shared_v, int64_t shared_layer_stride,
                            const int32_t* shared_cu, const int32_t* stream_to_seq, void* gen_k, void* gen_v,
                            int64_t gen_layer_stride, const int32_t* gen_len, int32_t gen_cap, int32_t n_streams,
                            int32_t batch, int32_t max_shared_len, int32_t shared_total, void* out, int64_t out_layer_stride, void* workspace,
                            size_t workspace_bytes, void* stream) {
  const char* who = "earn_decode_attn_layers";
  int rc = check_decode_args(who, desc, q, k_new, v_new, q_pos, shared_k, shared_v, shared_cu, stream_to_seq, gen_k,
                             gen_v, gen_len, gen_cap, n_streams, batch, max_shared_len, shared_total, out, stream);
  if (rc != EARN_OK) return rc;
  if (n_layers <= 0 || n_layers > 65535) { set_error("%s: n_layers (%d) outside [1, 65535]", who, n_layers); return EARN_ERR_INVALID_ARG; }
  if ((rc = check_layer_stride(who, "q_layer_stride", q_layer_stride, n_layers)) != EARN_OK ||
      (rc = check_layer_stride(who, "kv_new_layer_stride", kv_new_layer_stride, n_layers)) != EARN_OK ||
      (max_shared_len > 0 && (rc = check_layer_stride(who, "shared_layer_stride", shared_layer_stride, n_layers)) != EARN_OK) ||
      (rc = check_layer_stride(who, "gen_layer_stride", gen_layer_stride, n_layers)) != EARN_OK ||
      (rc = check_layer_stride(who, "out_layer_stride", out_layer_stride, n_layers)) != EARN_OK)
    return rc;
  const DecodeLayers layers = {n_layers, q_layer_stride, kv_new_layer_stride, shared_layer_stride, gen_layer_stride, out_layer_stride};
  return launch_decode(desc, q, k_new, v_new, q_pos, shared_k, shared_v, shared_cu, stream_to_seq, gen_k, gen_v, gen_len,
                       gen_cap, n_streams, batch, max_shared_len, shared_total, out, workspace, workspace_bytes, (hipStream_t)stream,
                       &layers, nullptr);
}

size_t earn_prefill_register_rows_workspace_bytes(const earn_attn_desc* desc, int32_t batch, int32_t max_seqlen,
                                                  int32_t rows_per_seq) {
  if (check_desc(desc, "earn_prefill_register_rows_workspace_bytes") != EARN_OK || batch <= 0 || max_seqlen < 0 ||
      rows_per_seq <= 0)
    return 0;
  if (desc->dtype == EARN_F32) return 0;
  return prefill_rows_workspace_bytes(desc->n_q_heads, desc->n_kv_heads, desc->head_dim, batch, max_seqlen, rows_per_seq);
}

int earn_prefill_register_rows(const earn_attn_desc* desc, const void* q_rows, const void* k, const void* v,
                               const int32_t* cu_seqlens, const int32_t* row_pos, int32_t batch, int32_t total_tokens,
                               int32_t max_seqlen, int32_t rows_per_seq, void* out_rows, void* k_rot_out,
                               void* workspace, size_t workspace_bytes, void* stream) {
  g_err[0] = 0;
  int rc = check_desc(desc, "earn_prefill_register_rows");
  if (rc != EARN_OK) return rc;
  if (batch <= 0 || total_tokens <= 0 || max_seqlen <= 0 || rows_per_seq <= 0) {
    set_error("earn_prefill_register_rows: batch (%d), total_tokens (%d), max_seqlen (%d) and rows_per_seq (%d) must be positive", batch, total_tokens, max_seqlen, rows_per_seq);
    return EARN_ERR_INVALID_ARG;
  }
  if (rows_per_seq > max_seqlen) {
    set_error("earn_prefill_register_rows: rows_per_seq (%d) exceeds max_seqlen (%d)", rows_per_seq, max_seqlen);
    return EARN_ERR_INVALID_ARG;
  }
  if (!q_rows || !k || !v || !cu_seqlens || !row_pos || !out_rows || !k_rot_out) {
    set_error("earn_prefill_register_rows: a required pointer is NULL");
    return EARN_ERR_INVALID_ARG;
  }
  if (g_validate.load(std::memory_order_relaxed)) {
    const char* who = "earn_prefill_register_rows";
    std::vector<int32_t> cu, rp;
    if ((rc = fetch_i32(cu_seqlens, (size_t)batch + 1, cu, (hipStream_t)stream, who)) != EARN_OK) return rc;
    if ((rc = validate_cu(who, "cu_seqlens", cu, batch, total_tokens, max_seqlen)) != EARN_OK) return rc;
    if ((rc = fetch_i32(row_pos, (size_t)batch * rows_per_seq, rp, (hipStream_t)stream, who)) != EARN_OK) return rc;
    for (int s = 0; s < batch; ++s)
      for (int m = 0; m < rows_per_seq; ++m) {
        const int p = rp[(size_t)s * rows_per_seq + m], n = cu[s + 1] - cu[s];
        if (p < 0 || p >= n || (m > 0 && p <= rp[(size_t)s * rows_per_seq + m - 1])) {
          set_error("%s: row_pos[%d] = %d (row %d of sequence %d, %d tokens) is outside the sequence or not ascending", who, s * rows_per_seq + m, p, m, s, n);
          return EARN_ERR_INVALID_ARG;
        }
      }
  }
  if (desc->dtype == EARN_F32) {
    rc = launch_rope_keys(desc, k, k_rot_out, cu_seqlens, nullptr, batch, total_tokens, (hipStream_t)stream);
    if (rc != EARN_OK) return rc;
    return launch_prefill_rows_f32(desc, q_rows, k_rot_out, v, cu_seqlens, row_pos, batch, total_tokens, max_seqlen,
                                   rows_per_seq, out_rows, (hipStream_t)stream);
  }
  const size_t need = prefill_rows_workspace_bytes(desc->n_q_heads, desc->n_kv_heads, desc->head_dim, batch, max_seqlen, rows_per_seq);
  if (need > workspace_bytes || (need > 0 && !workspace)) {
    set_error("earn_prefill_register_rows: workspace too small (%zu bytes given, %zu needed)", workspace_bytes, need);
    return EARN_ERR_WORKSPACE_TOO_SMALL;
  }
  rc = launch_rope_keys(desc, k, k_rot_out, cu_seqlens, nullptr, batch, total_tokens, (hipStream_t)stream);
  if (rc != EARN_OK) return rc;
  return launch_prefill_rows(desc, q_rows, k_rot_out, v, cu_seqlens, row_pos, batch, total_tokens, max_seqlen, rows_per_seq,
                             out_rows, workspace, workspace_bytes, (hipStream_t)stream);
}

int earn_attn_stats(const earn_attn_desc* desc, const void* q_rows, const void* k_rot, const int32_t* cu_seqlens,
                    const int32_t* row_pos, int32_t batch, int32_t total_tokens, int32_t rows_per_seq, float epsilon,
                    int32_t t_head, int32_t tail_back, float* stats_out, void* stream) {
  g_err[0] = 0;
  int rc = check_desc(desc, "earn_attn_stats");
  if (rc != EARN_OK) return rc;
  if (batch <= 0 || total_tokens < 0 || rows_per_seq <= 0 || !(epsilon >= 0.f) || t_head < 0 || tail_back < 0 ||
      (long long)batch * rows_per_seq > 0x7fffffffLL || desc->n_q_heads > 65535) {
    set_error("earn_attn_stats: batch (%d) and rows_per_seq (%d) must be positive, epsilon, t_head (%d) and tail_back (%d) non-negative", batch, rows_per_seq, t_head, tail_back);
    return EARN_ERR_INVALID_ARG;
  }
  if (!q_rows || !k_rot || !cu_seqlens || !row_pos || !stats_out) {
    set_error("earn_attn_stats: a required pointer is NULL");
    return EARN_ERR_INVALID_ARG;
  }
  return launch_attn_stats(desc, q_rows, k_rot, cu_seqlens, row_pos, batch, total_tokens, rows_per_seq, epsilon, t_head,
                           tail_back, stats_out, (hipStream_t)stream);
}

int earn_qkv_rope_project(const earn_attn_desc* desc, const void* x, const void* w_qkv, int32_t rows, int32_t d_model,
                          const int32_t* cu_seqlens, const int32_t* positions, int32_t batch, void* q_out, void* k_out,
                          void* v_out, void* workspace, size_t workspace_bytes, void* stream) {
  g_err[0] = 0;
  int rc = check_desc(desc, "earn_qkv_rope_project");
  if (rc != EARN_OK) return rc;
  if (desc->dtype != EARN_BF16) { set_error("earn_qkv_rope_project: bf16 only"); return EARN_ERR_UNSUPPORTED; }
  if (!x || !w_qkv || !q_out || !k_out || !v_out || rows <= 0 || d_model <= 0) {
    set_error("earn_qkv_rope_project: NULL pointer or non-positive size (rows %d, d_model %d)", rows, d_model);
    return EARN_ERR_INVALID_ARG;
  }
  if (desc->rope_base > 0.f && !positions && (!cu_seqlens || batch <= 0)) {
    set_error("earn_qkv_rope_project: positions is NULL and no cu_seqlens / batch to derive them from");
    return EARN_ERR_INVALID_ARG;
  }
  return launch_qkv_rope_project(desc, x, w_qkv, rows, d_model, cu_seqlens, positions, batch, q_out, k_out, v_out,
                                 workspace, workspace_bytes, (hipStream_t)stream);
}

size_t earn_linear_workspace_bytes(int32_t rows, int32_t k, int32_t n) { return linear_workspace_bytes(rows, k, n); }

int earn_linear(const void* x, const void* w, int32_t rows, int32_t k, int32_t n, int32_t activation, void* out,
                void* workspace, size_t workspace_bytes, void* stream) {
  g_err[0] = 0;
  if (!x || !w || !out || rows <= 0 || k <= 0 || n <= 0 || activation < 0 || activation > 1) {
    set_error("earn_linear: NULL pointer, non-positive size or unknown activation %d", activation);
    return EARN_ERR_INVALID_ARG;
  }
  return launch_linear(x, w, rows, k, n, activation, out, workspace, workspace_bytes, (hipStream_t)stream);
}

size_t earn_attn_backward_workspace_bytes(const earn_attn_desc* desc, int32_t total_tokens) {
  if (check_desc(desc, "earn_attn_backward_workspace_bytes") != EARN_OK || total_tokens <= 0) return 0;
  return attn_backward_workspace_bytes(desc->n_q_heads, total_tokens);
}

int earn_attn_backward(const earn_attn_desc* desc, const void* q, const void* k, const void* v, const void* out,
                       const float* lse, const void* d_out, const int32_t* cu_seqlens, int32_t batch,
                       int32_t total_tokens, int32_t max_seqlen, void* dq, void* dk, void* dv, void* workspace,
                       size_t workspace_bytes, void* stream) {
  g_err[0] = 0;
  int rc = check_desc(desc, "earn_attn_backward");
  if (rc != EARN_OK) return rc;
  if (desc->rope_base > 0.f) {
    set_error("earn_attn_backward: takes rotated q and k and rotates nothing: set rope_base <= 0");
    return EARN_ERR_UNSUPPORTED;
  }
  if (!q || !k || !v || !out || !lse || !d_out || !cu_seqlens || !dq || !dk || !dv || batch <= 0 || total_tokens <= 0 ||
      max_seqlen <= 0) {
    set_error("earn_attn_backward: NULL pointer or non-positive size (batch %d, total_tokens %d, max_seqlen %d)", batch, total_tokens, max_seqlen);
    return EARN_ERR_INVALID_ARG;
  }
  const size_t need = attn_backward_workspace_bytes(desc->n_q_heads, total_tokens);
  if (need > workspace_bytes || !workspace) {
    set_error("earn_attn_backward: workspace too small (%zu bytes given, %zu needed)", workspace_bytes, need);
    return EARN_ERR_WORKSPACE_TOO_SMALL;
  }
  if (g_validate.load(std::memory_order_relaxed)) {
    std::vector<int32_t> cu;
    if ((rc = fetch_i32(cu_seqlens, (size_t)batch + 1, cu, (hipStream_t)stream, "earn_attn_backward")) != EARN_OK) return rc;
    if ((rc = validate_cu("earn_attn_backward", "cu_seqlens", cu, batch, total_tokens, max_seqlen)) != EARN_OK) return rc;
  }
  if (max_seqlen > total_tokens) max_seqlen = total_tokens;
  return launch_attn_backward(desc, q, k, v, out, lse, d_out, cu_seqlens, batch, total_tokens, max_seqlen, dq, dk, dv,
                              workspace, (hipStream_t)stream);
}

int64_t earn_cache_entries(int32_t n_layers, int32_t split_k, int64_t seq_len, int32_t n_registers, int64_t gen) {
  return (int64_t)split_k * seq_len + (int64_t)(n_layers - split_k) * n_registers + (int64_t)n_layers * gen;
}

}  // extern "C"
