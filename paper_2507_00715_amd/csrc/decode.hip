// Decode-step attention (paper Section 2.2, Eq. 4; Section 3.2 decoding bullet): each stream appends its rotated key
// and its value to its generated cache and attends over the sequence's shared cache rows plus its own generated rows.
// The step is bound by streaming K/V from HBM, so:
//   * one workgroup serves ALL query heads that share a kv head (grouped-query attention): K/V bytes are read once
//     per group, not once per query head;
//   * a key row is spread over d/8 lanes holding 8 elements (16 bytes of bf16) each, so a wave reads whole rows with
//     full-width loads; the dot product is finished with log2(d/8) wavefront shuffles;
//   * every lane keeps an online-softmax state (max, sum, 8 output elements per head) for its share of the keys; the
//     states of the lanes that hold the same output elements are merged with shuffles inside the wave and through LDS
//     across the 4 waves;
//   * the key range of a long cache is split over several workgroups (split-K); partial (max, sum, out) triples go to
//     the workspace and a second kernel merges them.
#include "common.h"

namespace earn {

constexpr int kDecThreads = 256;
constexpr int kDecWaves = kDecThreads / kWave;

template <typename T>
struct Row8;  // 8 consecutive elements of a row as floats
template <>
struct Row8<float> {
  static __device__ __forceinline__ void load(const float* p, float* x) {
    f32x4 a = *(const f32x4*)p, b = *(const f32x4*)(p + 4);
    x[0] = a[0]; x[1] = a[1]; x[2] = a[2]; x[3] = a[3]; x[4] = b[0]; x[5] = b[1]; x[6] = b[2]; x[7] = b[3];
  }
  static __device__ __forceinline__ void store(float* p, const float* x) {
    f32x4 a = {x[0], x[1], x[2], x[3]}, b = {x[4], x[5], x[6], x[7]};
    *(f32x4*)p = a;
    *(f32x4*)(p + 4) = b;
  }
  // value as it will be read back from storage
  static __device__ __forceinline__ float round(float x) { return x; }
};
template <>
struct Row8<__bf16> {
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
  static __device__ __forceinline__ float round(float x) { return bf16_lo(pack_bf16(x, 0.f) & 0xffffu); }
};

struct DecodeParams {
  const void* q; const void* k_new; const void* v_new; const int32_t* q_pos;
  const void* shared_k; const void* shared_v; const int32_t* shared_cu; const int32_t* stream_to_seq;
  void* gen_k; void* gen_v; const int32_t* gen_len;
  void* out; float* part_o; float* part_ml;
  int gen_cap, n_streams, batch, hq, hkv, n_splits, chunk;  // chunk: keys per split (multiple of 64)
  float scale_log2;
  RopeTable rope;
};

// merge (m2,l2,o2) into (m,l,o); all in base-2 exponent units
template <int N>
__device__ __forceinline__ void merge_state(float& m, float& l, float* o, float m2, float l2, const float* o2) {
  float mn = fmaxf(m, m2);
  float a = (m == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(m - mn);
  float b = (m2 == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(m2 - mn);
  l = l * a + l2 * b;
#pragma unroll
  for (int i = 0; i < N; ++i) o[i] = o[i] * a + o2[i] * b;
  m = mn;
}

template <typename T, int D, int GQ>
__global__ __launch_bounds__(kDecThreads) void decode_kernel(DecodeParams p) {
  constexpr int LPK = D / 8;         // lanes per key row
  constexpr int KPW = kWave / LPK;   // key rows per wave instruction
  const int c = blockIdx.x, u = blockIdx.y, z = blockIdx.z;
  const int gq = p.hq / p.hkv;       // query heads per kv head
  const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
  const int sub = lane % LPK, kk = lane / LPK;
  const int s = p.stream_to_seq ? p.stream_to_seq[u] : u;
  const int b0 = p.shared_cu[s], ns = p.shared_cu[s + 1] - b0;
  const int g = p.gen_len[u];
  const int m_total = ns + g + 1;    // shared rows, earlier generated rows, the new token
  const float pos = (float)p.q_pos[u];

  const T* Kc = (const T*)p.shared_k + ((long long)b0 * p.hkv + c) * D + sub * 8;
  const T* Vc = (const T*)p.shared_v + ((long long)b0 * p.hkv + c) * D + sub * 8;
  T* Gk = (T*)p.gen_k + (((long long)u * p.gen_cap) * p.hkv + c) * D + sub * 8;
  T* Gv = (T*)p.gen_v + (((long long)u * p.gen_cap) * p.hkv + c) * D + sub * 8;
  const long long row_stride = (long long)p.hkv * D;

  // rotary factors of this lane's 8 elements (pairs (e, e + D/2): this lane holds one side, the partner lane the other)
  float cs[8], sn[8];
  {
    const int e0 = (sub * 8) % (D / 2);
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      if (p.rope.enabled) {
        float t = rope_turns(pos, p.rope.hi[e0 + i], p.rope.lo[e0 + i]);
        sincos_turns_precise(t, &sn[i], &cs[i]);
      } else { cs[i] = 1.f; sn[i] = 0.f; }
    }
  }
  const bool upper = sub * 8 >= D / 2;  // this lane holds elements e + D/2
  // rotate a row held as 8 elements per lane across LPK lanes: partner lane is sub ^ (LPK/2)
  auto rotate = [&](float* x) {
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      float other = __shfl_xor(x[i], LPK / 2, kWave);
      // lower half: x*c - partner*s ; upper half: x*c + partner*s
      x[i] = upper ? x[i] * cs[i] + other * sn[i] : x[i] * cs[i] - other * sn[i];
    }
  };

  // queries of the group, rotated and pre-scaled (scale * log2 e), 8 elements per lane per head
  float qv[GQ][8];
#pragma unroll
  for (int a = 0; a < GQ; ++a) {
    if (a < gq) {
      Row8<T>::load((const T*)p.q + ((long long)u * p.hq + c * gq + a) * D + sub * 8, qv[a]);
      rotate(qv[a]);
#pragma unroll
      for (int i = 0; i < 8; ++i) qv[a][i] *= p.scale_log2;
    } else {
#pragma unroll
      for (int i = 0; i < 8; ++i) qv[a][i] = 0.f;
    }
  }

  // the new token's key (rotated, rounded as stored) and value
  float kn[8], vn[8];
  Row8<T>::load((const T*)p.k_new + ((long long)u * p.hkv + c) * D + sub * 8, kn);
  Row8<T>::load((const T*)p.v_new + ((long long)u * p.hkv + c) * D + sub * 8, vn);
  rotate(kn);
#pragma unroll
  for (int i = 0; i < 8; ++i) kn[i] = Row8<T>::round(kn[i]);

  const int j_begin = z * p.chunk;
  const int j_end = min(m_total, j_begin + p.chunk);
  // cache append (Eq. 4): done by the one workgroup whose key range holds the new token
  if (m_total - 1 >= j_begin && m_total - 1 < j_end && wave == 0 && kk == 0) {
    Row8<T>::store(Gk + (long long)g * row_stride, kn);
    Row8<T>::store(Gv + (long long)g * row_stride, vn);
  }

  float mx[GQ], ls[GQ], o[GQ][8];
#pragma unroll
  for (int a = 0; a < GQ; ++a) {
    mx[a] = -INFINITY; ls[a] = 0.f;
#pragma unroll
    for (int i = 0; i < 8; ++i) o[a][i] = 0.f;
  }

  for (int j0 = j_begin + wave * KPW; j0 < j_end; j0 += kDecWaves * KPW) {
    const int j = j0 + kk;
    const bool valid = j < j_end;
    float kx[8], vx[8];
    if (valid) {
      if (j < ns) {
        Row8<T>::load(Kc + (long long)j * row_stride, kx);
        Row8<T>::load(Vc + (long long)j * row_stride, vx);
      } else if (j < m_total - 1) {
        Row8<T>::load(Gk + (long long)(j - ns) * row_stride, kx);
        Row8<T>::load(Gv + (long long)(j - ns) * row_stride, vx);
      } else {
#pragma unroll
        for (int i = 0; i < 8; ++i) { kx[i] = kn[i]; vx[i] = vn[i]; }
      }
    } else {
#pragma unroll
      for (int i = 0; i < 8; ++i) { kx[i] = 0.f; vx[i] = 0.f; }
    }
#pragma unroll
    for (int a = 0; a < GQ; ++a) {
      float sc = 0.f;
#pragma unroll
      for (int i = 0; i < 8; ++i) sc = __builtin_fmaf(qv[a][i], kx[i], sc);
#pragma unroll
      for (int off = LPK / 2; off >= 1; off >>= 1) sc += __shfl_xor(sc, off, kWave);
      if (!valid) sc = -INFINITY;
      float mn = fmaxf(mx[a], sc);
      float corr = (mx[a] == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(mx[a] - mn);
      float pr = valid ? __builtin_amdgcn_exp2f(sc - mn) : 0.f;
      ls[a] = ls[a] * corr + pr;
#pragma unroll
      for (int i = 0; i < 8; ++i) o[a][i] = __builtin_fmaf(pr, vx[i], o[a][i] * corr);
      mx[a] = mn;
    }
  }

  // merge the KPW lane groups of the wave (lanes with equal `sub`)
#pragma unroll
  for (int a = 0; a < GQ; ++a) {
#pragma unroll
    for (int off = LPK; off < kWave; off <<= 1) {
      float m2 = __shfl_xor(mx[a], off, kWave), l2 = __shfl_xor(ls[a], off, kWave), o2[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) o2[i] = __shfl_xor(o[a][i], off, kWave);
      merge_state<8>(mx[a], ls[a], o[a], m2, l2, o2);
    }
  }
  // merge the waves through LDS
  __shared__ float sm[kDecWaves][GQ][LPK][10];
  if (kk == 0) {
#pragma unroll
    for (int a = 0; a < GQ; ++a) {
      sm[wave][a][sub][0] = mx[a];
      sm[wave][a][sub][1] = ls[a];
#pragma unroll
      for (int i = 0; i < 8; ++i) sm[wave][a][sub][2 + i] = o[a][i];
    }
  }
  __syncthreads();
  // thread t < gq*LPK finishes head a = t / LPK, element group t % LPK
  const int t = threadIdx.x;
  if (t < gq * LPK) {
    const int a = t / LPK, sb = t % LPK;
    float m = sm[0][a][sb][0], l = sm[0][a][sb][1], oo[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) oo[i] = sm[0][a][sb][2 + i];
#pragma unroll
    for (int w = 1; w < kDecWaves; ++w) merge_state<8>(m, l, oo, sm[w][a][sb][0], sm[w][a][sb][1], &sm[w][a][sb][2]);
    const int head = c * gq + a;
    if (p.n_splits == 1) {
      float inv = 1.f / l;
#pragma unroll
      for (int i = 0; i < 8; ++i) oo[i] *= inv;
      Row8<T>::store((T*)p.out + ((long long)u * p.hq + head) * D + sb * 8, oo);
    } else {
      const long long slot = ((long long)u * p.hq + head) * p.n_splits + z;
      float* po = p.part_o + slot * D + sb * 8;
#pragma unroll
      for (int i = 0; i < 8; ++i) po[i] = oo[i];
      if (sb == 0) { p.part_ml[slot * 2] = m; p.part_ml[slot * 2 + 1] = l; }
    }
  }
}

// merge the split-K partials: one thread per (stream, head, 8-element group)
template <typename T, int D>
__global__ __launch_bounds__(256) void decode_combine_kernel(const float* __restrict__ part_o,
                                                             const float* __restrict__ part_ml, T* __restrict__ out,
                                                             int rows /* n_streams*hq */, int n_splits) {
  constexpr int LPK = D / 8;
  const int t = blockIdx.x * 256 + threadIdx.x;
  if (t >= rows * LPK) return;
  const int row = t / LPK, sb = t % LPK;
  float m = -INFINITY, l = 0.f, o[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) o[i] = 0.f;
  for (int z = 0; z < n_splits; ++z) {
    const long long slot = (long long)row * n_splits + z;
    float m2 = part_ml[slot * 2], l2 = part_ml[slot * 2 + 1];
    if (l2 == 0.f) continue;  // a split with no keys
    float o2[8];
    f32x4 a = *(const f32x4*)(part_o + slot * D + sb * 8), b = *(const f32x4*)(part_o + slot * D + sb * 8 + 4);
    o2[0] = a[0]; o2[1] = a[1]; o2[2] = a[2]; o2[3] = a[3]; o2[4] = b[0]; o2[5] = b[1]; o2[6] = b[2]; o2[7] = b[3];
    merge_state<8>(m, l, o, m2, l2, o2);
  }
  float inv = 1.f / l;
#pragma unroll
  for (int i = 0; i < 8; ++i) o[i] *= inv;
  Row8<T>::store(out + (long long)row * D + sb * 8, o);
}

static int choose_splits(int hkv, int n_streams, int max_len) {
  // aim at >= 1024 workgroups (4 per CU) while keeping at least 256 keys per split
  long long base = (long long)hkv * n_streams;
  int want = (int)((1024 + base - 1) / base);
  int cap = (max_len + 255) / 256;
  int n = want < cap ? want : cap;
  if (n < 1) n = 1;
  if (n > 64) n = 64;
  return n;
}

size_t decode_workspace_bytes(int hq, int hkv, int d, int n_streams, int max_total_len) {
  int n = choose_splits(hkv, n_streams, max_total_len);
  if (n == 1) return 0;
  size_t rows = (size_t)n_streams * hq * n;
  return rows * d * sizeof(float) + rows * 2 * sizeof(float);
}

template <typename T, int D>
static void launch_decode_t(DecodeParams& p, int gq, hipStream_t stream) {
  dim3 grid(p.hkv, p.n_streams, p.n_splits), block(kDecThreads);
  if (gq == 1) hipLaunchKernelGGL((decode_kernel<T, D, 1>), grid, block, 0, stream, p);
  else if (gq == 2) hipLaunchKernelGGL((decode_kernel<T, D, 2>), grid, block, 0, stream, p);
  else if (gq <= 4) hipLaunchKernelGGL((decode_kernel<T, D, 4>), grid, block, 0, stream, p);
  else hipLaunchKernelGGL((decode_kernel<T, D, 8>), grid, block, 0, stream, p);
  if (p.n_splits > 1) {
    int rows = p.n_streams * p.hq;
    int threads = rows * (D / 8);
    hipLaunchKernelGGL((decode_combine_kernel<T, D>), dim3((threads + 255) / 256), dim3(256), 0, stream, p.part_o,
                       p.part_ml, (T*)p.out, rows, p.n_splits);
  }
}

int launch_decode(const earn_attn_desc* desc, const void* q, const void* k_new, const void* v_new,
                  const int32_t* q_pos, const void* shared_k, const void* shared_v, const int32_t* shared_cu,
                  const int32_t* stream_to_seq, void* gen_k, void* gen_v, const int32_t* gen_len, int gen_cap,
                  int n_streams, int batch, int max_shared_len, void* out, void* workspace, size_t workspace_bytes,
                  hipStream_t stream) {
  const int hq = desc->n_q_heads, hkv = desc->n_kv_heads, d = desc->head_dim, gq = hq / hkv;
  if (gq > 8) { set_error("earn_decode_attn: more than 8 query heads per kv head is not supported"); return EARN_ERR_UNSUPPORTED; }
  DecodeParams p;
  p.q = q; p.k_new = k_new; p.v_new = v_new; p.q_pos = q_pos;
  p.shared_k = shared_k; p.shared_v = shared_v; p.shared_cu = shared_cu; p.stream_to_seq = stream_to_seq;
  p.gen_k = gen_k; p.gen_v = gen_v; p.gen_len = gen_len; p.out = out;
  p.gen_cap = gen_cap; p.n_streams = n_streams; p.batch = batch; p.hq = hq; p.hkv = hkv;
  const int max_total = max_shared_len + gen_cap;
  p.n_splits = choose_splits(hkv, n_streams, max_total);
  p.chunk = (((max_total + p.n_splits - 1) / p.n_splits) + 63) / 64 * 64;
  const size_t need = decode_workspace_bytes(hq, hkv, d, n_streams, max_total);
  if (need > workspace_bytes || (need > 0 && !workspace)) {
    set_error("earn_decode_attn: workspace too small (%zu bytes given, %zu needed)", workspace_bytes, need);
    return EARN_ERR_WORKSPACE_TOO_SMALL;
  }
  p.part_o = (float*)workspace;
  p.part_ml = p.part_o + (size_t)n_streams * hq * p.n_splits * d;
  const float scale = desc->softmax_scale > 0.f ? desc->softmax_scale : 1.0f / sqrtf((float)d);
  p.scale_log2 = scale * 1.4426950408889634f;
  p.rope = make_rope_table(desc->rope_base, d);
  if (desc->dtype == EARN_F32) {
    if (d == 64) launch_decode_t<float, 64>(p, gq, stream); else launch_decode_t<float, 128>(p, gq, stream);
  } else {
    if (d == 64) launch_decode_t<__bf16, 64>(p, gq, stream); else launch_decode_t<__bf16, 128>(p, gq, stream);
  }
  return hipGetLastError() == hipSuccess ? EARN_OK : EARN_ERR_HIP;
}

}  // namespace earn
