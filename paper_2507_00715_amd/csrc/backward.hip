// Backward of the causal attention (paper Section 3.2, Training: the model is trained through the same attention, full
// length for layers l <= k and over register + target tokens for l > k; Eq. 3).  Given the forward's inputs as the
// attention saw them (rotated queries and keys), its output O, the log-sum-exp of every softmax row and dO:
//   D_i  = sum_e dO_ie O_ie                    P_ij = exp(s_ij - lse_i),  s_ij = scale q_i . k_j   (j <= i)
//   dV_j = sum_i P_ij dO_i                     dP_ij = dO_i . v_j          dS_ij = P_ij (dP_ij - D_i)
//   dQ_i = scale sum_j dS_ij k_j               dK_j = scale sum_i dS_ij q_i
// (sums over the query heads of a kv head's group for dK, dV).  A first form on the vector ALU, fp32 arithmetic for both
// storage types, without atomics: one kernel owns query rows (dQ), one owns key rows (dK, dV); each recomputes the
// probabilities it needs from lse.  Four lanes share a row and hold d/4 of its elements each.
#include "common.h"

namespace earn {

struct BwdParams {
  const void* q; const void* k; const void* v; const void* out; const float* lse; const void* d_out;
  const int32_t* cu; float* dsum;  // D [tokens, Hq]
  void* dq; void* dk; void* dv;
  int batch, hq, hkv, total, max_seqlen;
  float scale, scale_log2;
  HeadMap heads;
};

template <typename T> struct B8;
template <> struct B8<float> {
  static __device__ __forceinline__ void load(const float* p, float* x) {
    f32x4 a = *(const f32x4*)p, b = *(const f32x4*)(p + 4);
    x[0] = a[0]; x[1] = a[1]; x[2] = a[2]; x[3] = a[3]; x[4] = b[0]; x[5] = b[1]; x[6] = b[2]; x[7] = b[3];
  }
  static __device__ __forceinline__ void store(float* p, const float* x) {
    *(f32x4*)p = f32x4{x[0], x[1], x[2], x[3]};
    *(f32x4*)(p + 4) = f32x4{x[4], x[5], x[6], x[7]};
  }
};
template <> struct B8<__bf16> {
  static __device__ __forceinline__ void load(const __bf16* p, float* x) {
    u32x4 w = *(const u32x4*)p;
#pragma unroll
    for (int i = 0; i < 4; ++i) { x[2 * i] = bf16_lo(w[i]); x[2 * i + 1] = bf16_hi(w[i]); }
  }
  static __device__ __forceinline__ void store(__bf16* p, const float* x) {
    u32x4 w;
#pragma unroll
    for (int i = 0; i < 4; ++i) w[i] = pack_bf16(x[2 * i], x[2 * i + 1]);
    *(u32x4*)p = w;
  }
};
// the D/4 elements of a row this lane holds: pieces [qt*E, +E) and [D/2 + qt*E, +E), E = D/8
template <typename T, int D>
__device__ __forceinline__ void load_quarter(const T* row, int qt, float* x) {
  constexpr int E = D / 8;
#pragma unroll
  for (int e = 0; e < E; e += 8) { B8<T>::load(row + qt * E + e, x + e); B8<T>::load(row + D / 2 + qt * E + e, x + E + e); }
}
template <typename T, int D>
__device__ __forceinline__ void store_quarter(T* row, int qt, const float* x) {
  constexpr int E = D / 8;
#pragma unroll
  for (int e = 0; e < E; e += 8) { B8<T>::store(row + qt * E + e, x + e); B8<T>::store(row + D / 2 + qt * E + e, x + E + e); }
}
__device__ __forceinline__ float quad_sum(float x) {
  x += __shfl_xor(x, 1, kWave);
  x += __shfl_xor(x, 2, kWave);
  return x;
}

// D_i = dO_i . O_i for every (token, query head): one thread per 8 elements, four... one quad per row
template <typename T, int D>
__global__ __launch_bounds__(256) void bwd_dsum_kernel(const T* __restrict__ out, const T* __restrict__ d_out,
                                                       float* __restrict__ dsum, long long rows) {
  const long long t = (long long)blockIdx.x * 256 + threadIdx.x;
  const long long row = t >> 2;
  const int qt = (int)(t & 3);
  float acc = 0.f;
  if (row < rows) {
    float o[D / 4], g[D / 4];
    load_quarter<T, D>(out + row * D, qt, o);
    load_quarter<T, D>(d_out + row * D, qt, g);
#pragma unroll
    for (int e = 0; e < D / 4; ++e) acc = __builtin_fmaf(o[e], g[e], acc);
  }
  acc = quad_sum(acc);
  if (row < rows && qt == 0) dsum[row] = acc;
}

// dQ: 64 query rows per workgroup (grid: row block, query-head slot, sequence); the rows of a wave walk the keys together
template <typename T, int D>
__global__ __launch_bounds__(256) void bwd_dq_kernel(BwdParams p) {
  constexpr int Q4 = D / 4;
  const int slot = blockIdx.y, s = blockIdx.z;
  const int a = head_of_slot(p.heads, slot), c = slot / (p.hq / p.hkv);
  int b0, n;
  clamped_bounds(p.cu, s, p.total, p.max_seqlen, b0, n);
  const int row0 = blockIdx.x * 64;
  if (row0 >= n) return;
  const int qt = threadIdx.x & 3;
  const int i = row0 + (threadIdx.x >> 2);
  const bool row_ok = i < n;
  const int ic = row_ok ? i : n - 1;
  const long long io = ((long long)(b0 + ic) * p.hq + a);
  float q[Q4], g[Q4], dq[Q4];
  load_quarter<T, D>((const T*)p.q + io * D, qt, q);
  load_quarter<T, D>((const T*)p.d_out + io * D, qt, g);
#pragma unroll
  for (int e = 0; e < Q4; ++e) { q[e] *= p.scale_log2; dq[e] = 0.f; }
  const float lse2 = p.lse[io] * 1.4426950408889634f, dsum = p.dsum[io];
  const int wave_last = min(n - 1, row0 + (int)(threadIdx.x / kWave) * 16 + 15);
  const T* kbase = (const T*)p.k + ((long long)b0 * p.hkv + c) * D;
  const T* vbase = (const T*)p.v + ((long long)b0 * p.hkv + c) * D;
  const long long rs = (long long)p.hkv * D;
  for (int j = 0; j <= wave_last; ++j) {
    float kx[Q4], vx[Q4];
    load_quarter<T, D>(kbase + j * rs, qt, kx);
    load_quarter<T, D>(vbase + j * rs, qt, vx);
    float sc = 0.f, dp = 0.f;
#pragma unroll
    for (int e = 0; e < Q4; ++e) { sc = __builtin_fmaf(q[e], kx[e], sc); dp = __builtin_fmaf(g[e], vx[e], dp); }
    sc = quad_sum(sc);
    dp = quad_sum(dp);
    const float pr = j <= ic ? __builtin_amdgcn_exp2f(sc - lse2) : 0.f;   // causal: keys 0 .. i
    const float ds = pr * (dp - dsum);
#pragma unroll
    for (int e = 0; e < Q4; ++e) dq[e] = __builtin_fmaf(ds, kx[e], dq[e]);
  }
  if (!row_ok) return;
#pragma unroll
  for (int e = 0; e < Q4; ++e) dq[e] *= p.scale;
  store_quarter<T, D>((T*)p.dq + io * D, qt, dq);
}

// dK, dV: 64 key rows per workgroup (grid: key block, kv head, sequence); a quad owns one key row and walks the query
// rows j .. n-1 of every query head of the group
template <typename T, int D>
__global__ __launch_bounds__(256) void bwd_dkv_kernel(BwdParams p) {
  constexpr int Q4 = D / 4;
  const int c = blockIdx.y, s = blockIdx.z;
  const int gq = p.hq / p.hkv;
  int b0, n;
  clamped_bounds(p.cu, s, p.total, p.max_seqlen, b0, n);
  const int key0 = blockIdx.x * 64;
  if (key0 >= n) return;
  const int qt = threadIdx.x & 3;
  const int j = key0 + (threadIdx.x >> 2);
  const bool key_ok = j < n;
  const int jc = key_ok ? j : n - 1;
  const long long jo = ((long long)(b0 + jc) * p.hkv + c);
  float kx[Q4], vx[Q4], dk[Q4], dv[Q4];
  load_quarter<T, D>((const T*)p.k + jo * D, qt, kx);
  load_quarter<T, D>((const T*)p.v + jo * D, qt, vx);
#pragma unroll
  for (int e = 0; e < Q4; ++e) { kx[e] *= p.scale_log2; dk[e] = 0.f; dv[e] = 0.f; }
  const int wave_first = key0 + (int)(threadIdx.x / kWave) * 16;   // the wave's keys are wave_first .. wave_first + 15
  for (int ai = 0; ai < gq; ++ai) {
    const int a = head_of_slot(p.heads, c * gq + ai);
    for (int i = wave_first; i < n; ++i) {
      const long long io = ((long long)(b0 + i) * p.hq + a);
      float q[Q4], g[Q4];
      load_quarter<T, D>((const T*)p.q + io * D, qt, q);
      load_quarter<T, D>((const T*)p.d_out + io * D, qt, g);
      float sc = 0.f, dp = 0.f;
#pragma unroll
      for (int e = 0; e < Q4; ++e) { sc = __builtin_fmaf(q[e], kx[e], sc); dp = __builtin_fmaf(g[e], vx[e], dp); }
      sc = quad_sum(sc);
      dp = quad_sum(dp);
      const float pr = jc <= i ? __builtin_amdgcn_exp2f(sc - p.lse[io] * 1.4426950408889634f) : 0.f;   // query i sees keys 0 .. i
      const float ds = pr * (dp - p.dsum[io]);
#pragma unroll
      for (int e = 0; e < Q4; ++e) { dv[e] = __builtin_fmaf(pr, g[e], dv[e]); dk[e] = __builtin_fmaf(ds, q[e], dk[e]); }
    }
  }
  if (!key_ok) return;
#pragma unroll
  for (int e = 0; e < Q4; ++e) dk[e] *= p.scale;
  store_quarter<T, D>((T*)p.dk + jo * D, qt, dk);
  store_quarter<T, D>((T*)p.dv + jo * D, qt, dv);
}

size_t attn_backward_workspace_bytes(int hq, int total_tokens) { return ((size_t)total_tokens * hq * sizeof(float) + 255) / 256 * 256; }

template <typename T, int D>
static void launch_bwd_t(const BwdParams& p, int total_tokens, int max_seqlen, hipStream_t stream) {
  const long long rows = (long long)total_tokens * p.hq;
  hipLaunchKernelGGL((bwd_dsum_kernel<T, D>), dim3((unsigned)((rows * 4 + 255) / 256)), dim3(256), 0, stream, (const T*)p.out,
                     (const T*)p.d_out, p.dsum, rows);
  const unsigned blocks = (unsigned)((max_seqlen + 63) / 64);
  hipLaunchKernelGGL((bwd_dq_kernel<T, D>), dim3(blocks, p.hq, p.batch), dim3(256), 0, stream, p);
  hipLaunchKernelGGL((bwd_dkv_kernel<T, D>), dim3(blocks, p.hkv, p.batch), dim3(256), 0, stream, p);
}

int launch_attn_backward(const earn_attn_desc* desc, const void* q, const void* k, const void* v, const void* out,
                         const float* lse, const void* d_out, const int32_t* cu_seqlens, int batch, int total_tokens,
                         int max_seqlen, void* dq, void* dk, void* dv, void* workspace, hipStream_t stream) {
  BwdParams p;
  p.q = q; p.k = k; p.v = v; p.out = out; p.lse = lse; p.d_out = d_out; p.cu = cu_seqlens; p.dsum = (float*)workspace;
  p.dq = dq; p.dk = dk; p.dv = dv; p.batch = batch; p.hq = desc->n_q_heads; p.hkv = desc->n_kv_heads;
  p.total = total_tokens; p.max_seqlen = max_seqlen;
  const int d = desc->head_dim;
  p.scale = desc->softmax_scale > 0.f ? desc->softmax_scale : 1.0f / sqrtf((float)d);
  p.scale_log2 = p.scale * 1.4426950408889634f;
  if (make_head_map(desc, &p.heads, "earn_attn_backward") != EARN_OK) return EARN_ERR_UNSUPPORTED;
  if (batch > 65535 || p.hq > 65535) { set_error("earn_attn_backward: batch or head count beyond 65535"); return EARN_ERR_UNSUPPORTED; }
  if (desc->dtype == EARN_F32) {
    if (d == 64) launch_bwd_t<float, 64>(p, total_tokens, max_seqlen, stream); else launch_bwd_t<float, 128>(p, total_tokens, max_seqlen, stream);
  } else {
    if (d == 64) launch_bwd_t<__bf16, 64>(p, total_tokens, max_seqlen, stream); else launch_bwd_t<__bf16, 128>(p, total_tokens, max_seqlen, stream);
  }
  return hipGetLastError() == hipSuccess ? EARN_OK : EARN_ERR_HIP;
}

}  // namespace earn
