// Attention-score statistics of chosen query rows (paper Appendix, "Quantitative Measurements of Attention Score
// Distributions"): for the causal softmax row p_1..p_n of a query (Eq. 3)
//   Sparsity = (1/n) #{ j : p_j > epsilon },  Sink_head = sum_{j <= T_h} p_j,  Sink_tail = sum_{j >= n - tail_back} p_j.
// The flash-style attention kernels never hold a softmax row, so this kernel recomputes the scores of the chosen rows in
// two passes over the row's keys (the layer's cache: rotated keys): pass 1 finds the row maximum and the normaliser,
// pass 2 forms each probability once, compares it with epsilon and adds it to the window sums.  Bound by reading the keys
// (once from HBM, the second pass from L2); one workgroup per (row, kv head).
#include "common.h"

namespace earn {

struct StatsParams {
  const void* q_rows; const void* k_rot; const int32_t* cu; const int32_t* row_pos; float* out;
  int batch, total, rows_per_seq, hq, hkv, t_head, tail_back;
  float scale_log2, epsilon;
  RopeTable rope;
  HeadMap heads;
};

template <typename T> struct Ld8;
template <> struct Ld8<float> {
  static __device__ __forceinline__ void load(const float* p, float* x) {
    f32x4 a = *(const f32x4*)p, b = *(const f32x4*)(p + 4);
    x[0] = a[0]; x[1] = a[1]; x[2] = a[2]; x[3] = a[3]; x[4] = b[0]; x[5] = b[1]; x[6] = b[2]; x[7] = b[3];
  }
};
template <> struct Ld8<__bf16> {
  static __device__ __forceinline__ void load(const __bf16* p, float* x) {
    u32x4 w = *(const u32x4*)p;
#pragma unroll
    for (int i = 0; i < 4; ++i) { x[2 * i] = bf16_lo(w[i]); x[2 * i + 1] = bf16_hi(w[i]); }
  }
};

// One workgroup per (row, kv head): the GQ query heads that share the kv head are served together, so a key row is read
// once for all of them (GQ = the smallest of 1, 2, 4, 8 that covers Hq / Hkv).
template <typename T, int D, int GQ>
__global__ __launch_bounds__(256) void attn_stats_kernel(StatsParams p) {
  constexpr int LPK = D / 8;        // lanes per key row, 8 elements each
  constexpr int KPW = kWave / LPK;  // keys per wave instruction
  constexpr int WAVES = 4;
  __shared__ float red[WAVES][GQ][3];
  const int m = blockIdx.x, c = blockIdx.y;
  const int gq = p.hq / p.hkv;
  const int s = m / p.rows_per_seq;
  int b0, n_seq;
  clamped_bounds(p.cu, s, p.total, p.total, b0, n_seq);
  if (n_seq <= 0) {  // an empty sequence has no keys: its rows report zeros
    const int gq0 = p.hq / p.hkv;
    if ((int)threadIdx.x < gq0) {
      float* o = p.out + ((long long)m * p.hq + head_of_slot(p.heads, c * gq0 + threadIdx.x)) * 3;
      o[0] = 0.f; o[1] = 0.f; o[2] = 0.f;
    }
    return;
  }
  const int pos = max(min(p.row_pos[m], n_seq - 1), 0);  // the row's token index = rotary position: keys 0 .. pos
  const int n = pos + 1;
  const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
  const int sub = lane % LPK, kk = lane / LPK;

  // this lane's 8 elements of every query head of the group, rotated at the row's position, scaled by scale * log2(e)
  float qv[GQ][8];
  {
    float cs[8], sn[8];
    const bool upper = sub * 8 >= D / 2;
    const int e0 = (sub * 8) % (D / 2);
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      sn[i] = 0.f; cs[i] = 1.f;
      if (p.rope.enabled) {
        const float t = rope_turns((float)pos, p.rope.hi[e0 + i], p.rope.lo[e0 + i]);
        if (sizeof(T) == 2) sincos_turns_fast(t, &sn[i], &cs[i]); else sincos_turns_precise(t, &sn[i], &cs[i]);
      }
    }
#pragma unroll
    for (int a = 0; a < GQ; ++a) {
      const int head = head_of_slot(p.heads, c * gq + min(a, gq - 1));
      const T* qrow = (const T*)p.q_rows + ((long long)m * p.hq + head) * D;
      float own[8], other[8];
      Ld8<T>::load(qrow + sub * 8, own);
      Ld8<T>::load(qrow + (sub ^ (LPK / 2)) * 8, other);
#pragma unroll
      for (int i = 0; i < 8; ++i)
        qv[a][i] = (upper ? own[i] * cs[i] + other[i] * sn[i] : own[i] * cs[i] - other[i] * sn[i]) * p.scale_log2;
    }
  }
  const T* Kc = (const T*)p.k_rot + ((long long)b0 * p.hkv + c) * D + sub * 8;
  const long long row_stride = (long long)p.hkv * D;
  // base-2 scores of keys j, j + STEP, ... (NB of them, requested together: the walk is otherwise one memory round trip
  // per key) for the GQ heads, in every lane of each key's group; keys past the row's last one get -inf
  constexpr int NB = 4, STEP = WAVES * KPW;
  auto scores = [&](int j, float (&sc)[NB][GQ]) {
    float kx[NB][8];
#pragma unroll
    for (int b = 0; b < NB; ++b) Ld8<T>::load(Kc + (long long)min(j + b * STEP, n - 1) * row_stride, kx[b]);
#pragma unroll
    for (int b = 0; b < NB; ++b)
#pragma unroll
      for (int a = 0; a < GQ; ++a) {
        float d = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) d = __builtin_fmaf(qv[a][e], kx[b][e], d);
#pragma unroll
        for (int off = 1; off < LPK; off <<= 1) d += __shfl_xor(d, off, kWave);
        sc[b][a] = j + b * STEP < n ? d : -INFINITY;
      }
  };
  // combines the lane groups of a wave (lanes with equal `sub`) and the waves; every thread gets the result
  auto wg_reduce = [&](float x, int a, int slot_, bool take_max) {
#pragma unroll
    for (int off = LPK; off < kWave; off <<= 1) {
      const float y = __shfl_xor(x, off, kWave);
      x = take_max ? fmaxf(x, y) : x + y;
    }
    if (lane == 0) red[wave][a][slot_] = x;
    __syncthreads();
    float r = red[0][a][slot_];
#pragma unroll
    for (int w = 1; w < WAVES; ++w) r = take_max ? fmaxf(r, red[w][a][slot_]) : r + red[w][a][slot_];
    __syncthreads();
    return r;
  };

  // pass 1: running maximum and the normaliser against it (rescaled when the maximum moves)
  float mx[GQ], l[GQ];
#pragma unroll
  for (int a = 0; a < GQ; ++a) { mx[a] = -INFINITY; l[a] = 0.f; }
  for (int j = wave * KPW + kk; j < n; j += NB * STEP) {
    float sc[NB][GQ];
    scores(j, sc);
#pragma unroll
    for (int a = 0; a < GQ; ++a) {
      float mn = mx[a];
#pragma unroll
      for (int b = 0; b < NB; ++b) mn = fmaxf(mn, sc[b][a]);   // finite: the first key of the batch is in range
      float add = 0.f;
#pragma unroll
      for (int b = 0; b < NB; ++b) add += __builtin_amdgcn_exp2f(sc[b][a] - mn);  // exp2(-inf) = 0 for keys past the end
      l[a] = l[a] * __builtin_amdgcn_exp2f(mx[a] - mn) + add;  // exp2(-inf) = 0 at the start
      mx[a] = mn;
    }
  }
  float inv[GQ];
#pragma unroll
  for (int a = 0; a < GQ; ++a) {
    const float mall = wg_reduce(mx[a], a, 0, true);   // finite: key 0 is visible to every row
    const float mine = mx[a] == -INFINITY ? 0.f : l[a] * __builtin_amdgcn_exp2f(mx[a] - mall);
    inv[a] = 1.f / wg_reduce(mine, a, 1, false);
    mx[a] = mall;
  }
  // pass 2 (the keys come from L2 now): one probability per key and head, counted by the first lane of the key's group
  float count[GQ], head[GQ], tail[GQ];
#pragma unroll
  for (int a = 0; a < GQ; ++a) { count[a] = 0.f; head[a] = 0.f; tail[a] = 0.f; }
  for (int j = wave * KPW + kk; j < n; j += NB * STEP) {
    float sc[NB][GQ];
    scores(j, sc);
    if (sub == 0) {
#pragma unroll
      for (int b = 0; b < NB; ++b) {
        const int jb = j + b * STEP;                        // keys past the end carry -inf: probability 0
#pragma unroll
        for (int a = 0; a < GQ; ++a) {
          const float pj = __builtin_amdgcn_exp2f(sc[b][a] - mx[a]) * inv[a];
          count[a] += pj > p.epsilon ? 1.f : 0.f;
          if (jb + 1 <= p.t_head) head[a] += pj;            // 1-based key index j + 1 <= T_h
          if (jb + 1 >= n - p.tail_back && jb < n) tail[a] += pj;  // j + 1 >= T_t = n - tail_back
        }
      }
    }
  }
#pragma unroll
  for (int a = 0; a < GQ; ++a) {
    // lanes with sub != 0 hold zeros; the reduction over the lane groups leaves them out of lane 0's total anyway
    const float cn = wg_reduce(count[a], a, 0, false), hd = wg_reduce(head[a], a, 1, false), tl = wg_reduce(tail[a], a, 2, false);
    if (threadIdx.x == 0 && a < gq) {
      float* o = p.out + ((long long)m * p.hq + head_of_slot(p.heads, c * gq + a)) * 3;
      o[0] = cn / (float)n;
      o[1] = hd;
      o[2] = tl;
    }
  }
}

template <typename T, int D>
static void launch_stats_t(const StatsParams& p, dim3 grid, hipStream_t stream) {
  const int gq = p.hq / p.hkv;
  if (gq == 1) hipLaunchKernelGGL((attn_stats_kernel<T, D, 1>), grid, dim3(256), 0, stream, p);
  else if (gq == 2) hipLaunchKernelGGL((attn_stats_kernel<T, D, 2>), grid, dim3(256), 0, stream, p);
  else if (gq <= 4) hipLaunchKernelGGL((attn_stats_kernel<T, D, 4>), grid, dim3(256), 0, stream, p);
  else hipLaunchKernelGGL((attn_stats_kernel<T, D, 8>), grid, dim3(256), 0, stream, p);
}

int launch_attn_stats(const earn_attn_desc* desc, const void* q_rows, const void* k_rot, const int32_t* cu_seqlens,
                      const int32_t* row_pos, int batch, int total_tokens, int rows_per_seq, float epsilon, int t_head,
                      int tail_back, float* stats_out, hipStream_t stream) {
  StatsParams p;
  p.q_rows = q_rows; p.k_rot = k_rot; p.cu = cu_seqlens; p.row_pos = row_pos; p.out = stats_out;
  p.batch = batch; p.total = total_tokens; p.rows_per_seq = rows_per_seq; p.hq = desc->n_q_heads; p.hkv = desc->n_kv_heads;
  p.t_head = t_head; p.tail_back = tail_back; p.epsilon = epsilon;
  const int d = desc->head_dim;
  const float scale = desc->softmax_scale > 0.f ? desc->softmax_scale : 1.0f / sqrtf((float)d);
  p.scale_log2 = scale * 1.4426950408889634f;
  p.rope = make_rope_table(desc->rope_base, d);
  if (make_head_map(desc, &p.heads, "earn_attn_stats") != EARN_OK) return EARN_ERR_UNSUPPORTED;
  if (p.hq / p.hkv > 8) { set_error("earn_attn_stats: more than 8 query heads per kv head is not supported"); return EARN_ERR_UNSUPPORTED; }
  const dim3 grid((unsigned)(batch * rows_per_seq), (unsigned)p.hkv);
  if (desc->dtype == EARN_F32) {
    if (d == 64) launch_stats_t<float, 64>(p, grid, stream); else launch_stats_t<float, 128>(p, grid, stream);
  } else {
    if (d == 64) launch_stats_t<__bf16, 64>(p, grid, stream); else launch_stats_t<__bf16, 128>(p, grid, stream);
  }
  return hipGetLastError() == hipSuccess ? EARN_OK : EARN_ERR_HIP;
}

}  // namespace earn
