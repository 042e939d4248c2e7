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
#include <mutex>
#include <type_traits>

#include "common.h"
#include "mfma_tiles.h"

namespace earn {


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
  // the 8 elements as loaded, converted on use: lets several rows be in flight without holding their floats
  struct Raw { f32x4 a, b; };
  static __device__ __forceinline__ Raw load_raw(const float* p) { return Raw{*(const f32x4*)p, *(const f32x4*)(p + 4)}; }
  static __device__ __forceinline__ void unpack(const Raw& r, float* x) {
    x[0] = r.a[0]; x[1] = r.a[1]; x[2] = r.a[2]; x[3] = r.a[3]; x[4] = r.b[0]; x[5] = r.b[1]; x[6] = r.b[2]; x[7] = r.b[3];
  }
  static constexpr int kRowsInFlight = 2;
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
  typedef u32x4 Raw;
  static __device__ __forceinline__ Raw load_raw(const __bf16* p) { return *(const u32x4*)p; }
  static __device__ __forceinline__ void unpack(const Raw& w, float* x) {
#pragma unroll
    for (int i = 0; i < 4; ++i) { x[2 * i] = bf16_lo(w[i]); x[2 * i + 1] = bf16_hi(w[i]); }
  }
  static constexpr int kRowsInFlight = 4;
};

struct DecodeParams {
  const void* q; const void* k_new; const void* v_new; const int32_t* q_pos;
  const void* shared_k; const void* shared_v; const int32_t* shared_cu; const int32_t* stream_to_seq;
  void* gen_k; void* gen_v; const int32_t* gen_len;
  // Beam search without cache copies (NULL = every stream reads its own rows): row g < gen_len[u] of stream u's generated
  // cache lives in the physical slot (gen_src[u * gen_cap + g], g), i.e. in the cache rows of the stream that wrote it
  // at step g, an ancestor of u; the append of this call still goes to the stream's own slot (u, gen_len[u]).
  const int32_t* gen_src;
  void* out; float* part_o; float* part_ml;
  int gen_cap, n_streams, batch, hq, hkv, n_splits, chunk;  // chunk: keys per split (multiple of 64)
  int shared_total, max_shared_len;  // rows of shared_k / shared_v; the longest cache the launch was sized for
  int n_slots;    // partial-result slots per (stream, head) in the workspace (one per key split)
  // Prefill of chosen rows with the decode machinery (0 = decode).  r > 0: the "streams" are r query rows per sequence
  // (stream s*r + i belongs to sequence s), q_pos[u] is the row's token index in its sequence, a row sees shared keys
  // 0 .. q_pos[u] (causal), and there is no generated part and no new token.
  int causal_rows;
  // Query rows beyond one pass (32 rows per wave group) are normally taken in further passes of the same workgroup over
  // its keys.  n_pass > 1 gives every pass a workgroup of its own instead (pass index in the grid, last pass first):
  // used with causal rows, where passes differ widely in length and the long ones of a (sequence, kv head) then run
  // side by side on one XCD, sharing the keys in its L2.
  int n_pass;
  float scale_log2;
  // byte strides between the layers of a layer-batched launch (grid row y = layer); all zero for a single layer
  long long ls_q, ls_kv_new, ls_shared, ls_gen, ls_out, ls_part_o, ls_part_ml;
  RopeTable rope;
  HeadMap heads;
};

// Bounds of sequence s's shared cache as the kernels use them: whatever shared_cu holds, rows [b0, b0 + ns) lie inside
// the shared tensors and ns within the length the launch was sized (and its 32-bit offsets checked) for.  A corrupt or
// not yet written shared_cu gives wrong values, never an access outside the tensors.
__device__ __forceinline__ void shared_bounds(const DecodeParams& p, int s, int& b0, int& ns) {
  b0 = min(max(p.shared_cu[s], 0), p.shared_total);
  ns = min(min(max(p.shared_cu[s + 1] - b0, 0), p.shared_total - b0), p.max_shared_len);
}

template <typename P>
__device__ __forceinline__ P* layer_ptr(P* base, long long stride, int layer) {
  return (P*)((const char*)base + stride * layer);
}
// The per-layer pointers of this grid row's layer.  (A view beside the parameter block, not a modified copy of it: the
// block holds arrays that are indexed at run time, so a modified copy would live in scratch memory and nothing read
// from it would count as wave-uniform any more.)
struct DecodeLayer {
  const void* q; const void* k_new; const void* v_new; const void* shared_k; const void* shared_v;
  void* gen_k; void* gen_v; void* out; float* part_o; float* part_ml;
};
__device__ __forceinline__ DecodeLayer layer_view(const DecodeParams& p, int layer) {
  DecodeLayer v;
  v.q = layer_ptr(p.q, p.ls_q, layer);
  v.k_new = layer_ptr(p.k_new, p.ls_kv_new, layer);
  v.v_new = layer_ptr(p.v_new, p.ls_kv_new, layer);
  v.shared_k = layer_ptr(p.shared_k, p.ls_shared, layer);
  v.shared_v = layer_ptr(p.shared_v, p.ls_shared, layer);
  v.gen_k = layer_ptr(p.gen_k, p.ls_gen, layer);
  v.gen_v = layer_ptr(p.gen_v, p.ls_gen, layer);
  v.out = layer_ptr(p.out, p.ls_out, layer);
  v.part_o = layer_ptr(p.part_o, p.ls_part_o, layer);
  v.part_ml = layer_ptr(p.part_ml, p.ls_part_ml, layer);
  return v;
}

// gen_len as the kernels use it: inside [0, gen_cap), so that a violated precondition cannot move the cache append or
// the walk over the generated rows outside the stream's cache
__device__ __forceinline__ int clamp_gen_len(int g, int gen_cap) { return max(min(g, gen_cap - 1), 0); }

// Sum over the LPK (8 or 16) adjacent lanes that hold one key row, left in every lane of the group.  Data-parallel
// primitives instead of shuffles through LDS: pairs, quads, the mirrored half (lane i <-> 7-i: the other quad), the
// mirrored row (lane i <-> 15-i: the other half).
template <int CTRL>
__device__ __forceinline__ float dpp_move(float x) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), CTRL, 0xf, 0xf, true));
}
template <int LPK>
__device__ __forceinline__ float group_sum(float x) {
  static_assert(LPK == 8 || LPK == 16);
  x += dpp_move<0xB1>(x);   // quad_perm [1,0,3,2]
  x += dpp_move<0x4E>(x);   // quad_perm [2,3,0,1]
  x += dpp_move<0x141>(x);  // row_half_mirror
  if (LPK == 16) x += dpp_move<0x140>(x);  // row_mirror
  return x;
}

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

// Attention of one (stream u, kv head c) over the key range `z` of its key list, by WAVES cooperating waves
// (WAVES > 1: states merged through `sm`; WAVES = 1: a single wave, no LDS, no barrier — used for short key lists,
// where the per-wave prologue dominates).
template <typename T, int D, int GQ, int WAVES>
__device__ __forceinline__ void decode_rows(const DecodeParams& p, const DecodeLayer& lv, const int c, const int u,
                                            const int z, const int wave, const int lane, const int chunk,
                                            float* sm_base) {
  constexpr int LPK = D / 8;         // lanes per key row
  constexpr int KPW = kWave / LPK;   // key rows per wave instruction
  const int gq = p.hq / p.hkv;       // query heads per kv head
  const int sub = lane % LPK, kk = lane / LPK;
  const int s = p.stream_to_seq ? max(min(p.stream_to_seq[u], p.batch - 1), 0) : u;
  int b0, ns;
  shared_bounds(p, s, b0, ns);
  const int g = clamp_gen_len(p.gen_len[u], p.gen_cap);
  const int m_total = ns + g + 1;    // shared rows, earlier generated rows, the new token
  const float pos = (float)p.q_pos[u];

  const T* Kc = (const T*)lv.shared_k + ((long long)b0 * p.hkv + c) * D + sub * 8;
  const T* Vc = (const T*)lv.shared_v + ((long long)b0 * p.hkv + c) * D + sub * 8;
  T* Gk = (T*)lv.gen_k + (((long long)u * p.gen_cap) * p.hkv + c) * D + sub * 8;
  T* Gv = (T*)lv.gen_v + (((long long)u * p.gen_cap) * p.hkv + c) * D + sub * 8;
  const long long row_stride = (long long)p.hkv * D;

  // The wave's keys are j_begin + wave*KPW + kk + i*WAVES*KPW.  NP iterations' rows are requested together, then
  // consumed: a short key list (register-only caches) is one memory round trip instead of one per iteration, and
  // the first batch is requested here, ahead of the query rotation, which then runs in its shadow.
  constexpr int NP = GQ >= 8 ? 2 : Row8<T>::kRowsInFlight;  // fewer with many heads: their accumulators need the registers
  const int j_begin = z * chunk;
  const int j_end = min(m_total, j_begin + chunk);
  typename Row8<T>::Raw kr[NP], vr[NP];
  auto load_batch = [&](int jb) {
#pragma unroll
    for (int i = 0; i < NP; ++i) {
      const int j = jb + i * WAVES * KPW + kk;
      if (j < ns && j < j_end) {
        kr[i] = Row8<T>::load_raw(Kc + (long long)j * row_stride);
        vr[i] = Row8<T>::load_raw(Vc + (long long)j * row_stride);
      } else if (j < m_total - 1 && j < j_end) {
        // the physical stream that holds logical row j - ns (an ancestor's slot under beam search)
        long long from = 0;
        if (p.gen_src) {
          const int src = max(min(p.gen_src[(long long)u * p.gen_cap + (j - ns)], p.n_streams - 1), 0);
          from = (long long)(src - u) * p.gen_cap * row_stride;
        }
        kr[i] = Row8<T>::load_raw(Gk + from + (long long)(j - ns) * row_stride);
        vr[i] = Row8<T>::load_raw(Gv + from + (long long)(j - ns) * row_stride);
      } else {
        kr[i] = typename Row8<T>::Raw{};
        vr[i] = typename Row8<T>::Raw{};
      }
    }
  };
  const int jb_first = j_begin + wave * KPW;
  if (jb_first < j_end) load_batch(jb_first);

  // rotary factors of this lane's 8 elements (pairs (e, e + D/2): this lane holds one side, the partner lane the other)
  float cs[8], sn[8];
  {
    const int e0 = (sub * 8) % (D / 2);
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      if (p.rope.enabled) {
        float t = rope_turns(pos, p.rope.hi[e0 + i], p.rope.lo[e0 + i]);
        if (sizeof(T) == 2) sincos_turns_fast(t, &sn[i], &cs[i]);   // hardware sin/cos: error far below bf16 resolution
        else sincos_turns_precise(t, &sn[i], &cs[i]);
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
      Row8<T>::load((const T*)lv.q + ((long long)u * p.hq + head_of_slot(p.heads, c * gq + a)) * D + sub * 8, qv[a]);
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
  Row8<T>::load((const T*)lv.k_new + ((long long)u * p.hkv + c) * D + sub * 8, kn);
  Row8<T>::load((const T*)lv.v_new + ((long long)u * p.hkv + c) * D + sub * 8, vn);
  rotate(kn);
#pragma unroll
  for (int i = 0; i < 8; ++i) kn[i] = Row8<T>::round(kn[i]);

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

  for (int jb = jb_first; jb < j_end; jb += NP * WAVES * KPW) {
    if (jb != jb_first) load_batch(jb);
    // scores of the batch first, then one reference update per head for the whole batch, then the weighted values:
    // the running maximum and the rescale of the accumulators are paid once per NP keys instead of once per key
    float sc[NP][GQ];
#pragma unroll
    for (int i = 0; i < NP; ++i) {
      const int j = jb + i * WAVES * KPW + kk;
      const bool valid = j < j_end;
      float kx[8];
      Row8<T>::unpack(kr[i], kx);
      if (valid && j == m_total - 1) {
#pragma unroll
        for (int e = 0; e < 8; ++e) kx[e] = kn[e];
      }
#pragma unroll
      for (int a = 0; a < GQ; ++a) {
        float d = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) d = __builtin_fmaf(qv[a][e], kx[e], d);
        sc[i][a] = valid ? group_sum<LPK>(d) : -INFINITY;
      }
    }
#pragma unroll
    for (int a = 0; a < GQ; ++a) {
      float mn = mx[a];
#pragma unroll
      for (int i = 0; i < NP; ++i) mn = fmaxf(mn, sc[i][a]);
      const float corr = (mx[a] == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(mx[a] - mn);
      float sum = 0.f;
#pragma unroll
      for (int i = 0; i < NP; ++i) {
        sc[i][a] = (sc[i][a] == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(sc[i][a] - mn);  // a finite score makes mn finite
        sum += sc[i][a];
      }
      ls[a] = ls[a] * corr + sum;
#pragma unroll
      for (int e = 0; e < 8; ++e) o[a][e] *= corr;
      mx[a] = mn;
    }
#pragma unroll
    for (int i = 0; i < NP; ++i) {
      const int j = jb + i * WAVES * KPW + kk;
      float vx[8];
      Row8<T>::unpack(vr[i], vx);
      if (j == m_total - 1) {
#pragma unroll
        for (int e = 0; e < 8; ++e) vx[e] = vn[e];
      }
#pragma unroll
      for (int a = 0; a < GQ; ++a)
#pragma unroll
        for (int e = 0; e < 8; ++e) o[a][e] = __builtin_fmaf(sc[i][a], vx[e], o[a][e]);
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
  // write one finished (head, 8-element group) state: final output or a partial slot
  auto finish = [&](int a, int sb, float m, float l, float* oo) {
    const int head = head_of_slot(p.heads, c * gq + a);
    if (p.n_slots == 1) {
      float inv = 1.f / l;
#pragma unroll
      for (int i = 0; i < 8; ++i) oo[i] *= inv;
      Row8<T>::store((T*)lv.out + ((long long)u * p.hq + head) * D + sb * 8, oo);
    } else {
      const long long slot = ((long long)u * p.hq + head) * p.n_slots + z;
      float* po = lv.part_o + slot * D + sb * 8;
#pragma unroll
      for (int i = 0; i < 8; ++i) po[i] = oo[i];
      if (sb == 0) { lv.part_ml[slot * 2] = m; lv.part_ml[slot * 2 + 1] = l; }
    }
  };
  if constexpr (WAVES == 1) {
    if (kk == 0) {
#pragma unroll
      for (int a = 0; a < GQ; ++a)
        if (a < gq) finish(a, sub, mx[a], ls[a], o[a]);
    }
  } else {
    // merge the waves through LDS
    typedef float MergeBuf[GQ][LPK][10];
    MergeBuf* sm = (MergeBuf*)sm_base;
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
    const int t = wave * kWave + lane;
    if (t < gq * LPK) {
      const int a = t / LPK, sb = t % LPK;
      float m = sm[0][a][sb][0], l = sm[0][a][sb][1], oo[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) oo[i] = sm[0][a][sb][2 + i];
#pragma unroll
      for (int w = 1; w < WAVES; ++w) merge_state<8>(m, l, oo, sm[w][a][sb][0], sm[w][a][sb][1], &sm[w][a][sb][2]);
      finish(a, sb, m, l, oo);
    }
  }
}

template <typename T, int D, int GQ, int WAVES>
__global__ __launch_bounds__(kWave * WAVES) void decode_kernel(DecodeParams p) {
  __shared__ float sm[WAVES > 1 ? WAVES * GQ * (D / 8) * 10 : 1];
  // Work item -> (kv head c, stream u, key split z).  Linear ids go to the 8 XCDs round-robin.  The hkv items that read
  // the interleaved head slices of the same cache rows (one (u, z), all c) get ids 8 apart, i.e. the same XCD.
  const int n_uz = p.n_streams * p.n_splits, n_uz8 = (n_uz + 7) / 8 * 8;
  const int L = blockIdx.x;
  const int uz = (L / (8 * p.hkv)) * 8 + L % 8;
  const int c = (L / 8) % p.hkv;
  if (uz >= n_uz || L >= n_uz8 * p.hkv) return;
  const DecodeLayer lv = layer_view(p, blockIdx.y);
  decode_rows<T, D, GQ, WAVES>(p, lv, c, uz % p.n_streams, uz / p.n_streams, threadIdx.x / kWave, threadIdx.x % kWave,
                               p.chunk, sm);
}

// merge the partial results of the slots: one thread per (stream, head, 8-element group)
template <typename T, int D>
__global__ __launch_bounds__(256) void decode_combine_kernel(const float* __restrict__ part_o,
                                                             const float* __restrict__ part_ml, T* __restrict__ out,
                                                             int rows /* n_streams*hq */, int n_slots,
                                                             long long ls_part_o, long long ls_part_ml, long long ls_out) {
  constexpr int LPK = D / 8;
  const int t = blockIdx.x * 256 + threadIdx.x;
  if (t >= rows * LPK) return;
  part_o = layer_ptr(part_o, ls_part_o, blockIdx.y);   // grid row y = layer
  part_ml = layer_ptr(part_ml, ls_part_ml, blockIdx.y);
  out = layer_ptr(out, ls_out, blockIdx.y);
  const int row = t / LPK, sb = t % LPK;
  float m = -INFINITY, l = 0.f, o[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) o[i] = 0.f;
  for (int z = 0; z < n_slots; ++z) {
    const long long slot = (long long)row * n_slots + z;
    float m2 = part_ml[slot * 2], l2 = part_ml[slot * 2 + 1];
    if (l2 == 0.f) continue;  // a slot with no keys
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

// ------------------------------------------------------------------------------------------------------------------
// Shared-cache part on the matrix cores.  All query rows that read the same (sequence, kv head) cache — the gq query
// heads of the group times the W beams of the sequence — form the M columns of S^T = K Q^T, so the shared K/V rows are
// streamed from HBM ONCE per sequence, not once per beam or per query head.  Same register-level scheme as the prefill
// kernel (S^T accumulators feed V^T P^T directly; V^T fragments come from transposing LDS reads), without a mask.
//
// A workgroup has C groups of 4 waves; group g serves query rows [32g, 32g+32) of the cache (C = 2 covers the 40 rows of
// 4 grouped heads x 10 beams) at <= 256 registers per wave, i.e. two waves per SIMD.  The workgroup walks its key range
// in tiles of 64 keys that stream from global memory straight into a ring of four LDS buffers (three tiles on their
// way while one is used), so every K/V byte is fetched once.  Wave (ksub, dh) of a group works on the 32-key sub-tile
// ksub of the tile and accumulates half dh of the head dimension (both waves of a sub-tile compute its scores: the
// matrix core has time to spare here, LDS space has not) with a private softmax state; the states of the two
// sub-tiles are merged through LDS at the end.
// Key ranges of long caches are split over workgroups; every (row, split) partial goes to the workspace and
// decode_combine_kernel merges them.  The per-stream generated rows and the new token differ per beam.  They are laid
// out as one more key list, stream after stream at a common pitch, cut into the same 64-key tiles and multiplied
// against ALL query rows with a mask that lets a query row see only its own stream's rows: a few tiles more for a
// workgroup that walks dozens, instead of a second, latency-bound pass in vector code.  The workgroup that owns such a
// tile also rotates the new token's key and appends key and value to the stream's cache (Eq. 4).
// Without key splits (enough (sequence, kv head) pairs to fill the GPU) the kernel normalises and stores the outputs.
//
// The same kernel computes prefill attention at chosen rows (DecodeParams::causal_rows): the r register rows of a
// sequence against the sequence's full-length keys (Section 3.2: the input of layer k keeps only those rows of layer
// k-1's output) are r "beams" with a causal limit each and without a generated part.
// ------------------------------------------------------------------------------------------------------------------
constexpr int kDsTile = 32;              // keys per wave sub-tile
constexpr int kDsGroupWaves = 4;         // waves per 32-row group: 2 key sub-tiles x 2 halves of the head dimension
constexpr int kDsRing = 4;               // K/V tiles (kTileKeys = 64 keys each) in LDS: one in use, three on their way
constexpr int kDsSuper = 128;            // key ranges of the splits are multiples of this
constexpr float kDecSumLimit = kSumLimit;  // per lane: 16 exponentials of one query row and tile
constexpr int kMaxStreamsPerSeq = 1024;  // beams of one sequence the stream list holds
constexpr int kDsTabStreams = 16;        // streams whose rotary factors are tabulated in LDS

// Workgroup barrier for data exchanged through LDS only: waits for this wave's LDS traffic, not for its global loads.
// (__syncthreads() also drains the vector-memory queue, which would cut the depth of the K/V stream below to the one
// super-tile a single iteration can cover.)  The empty asm statements keep the compiler from moving memory accesses
// across the barrier.
__device__ __forceinline__ void lds_barrier() {
  asm volatile("" ::: "memory");
  __builtin_amdgcn_s_waitcnt(0xC07F);  // lgkmcnt(0)
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
}

template <int D>
struct DsSmem {
  // [ring slot][K, V][64 keys x D], rows unpadded, 16-byte chunks swizzled as in the prefill kernels (the loads
  // deposit them directly); reused as the merge buffers once the key loop is done
  __bf16 tile[kDsRing][2][kTileKeys * D];
  int streams[kMaxStreamsPerSeq];
  int glen[kMaxStreamsPerSeq];  // rows already in the generated cache of each listed stream
  float qpos[kMaxStreamsPerSeq];  // position of each listed stream's new token
  int n_streams_of_seq;
  int gen_pitch;                // 1 + the largest of them: generated key e is row e % gen_pitch of listed stream e / gen_pitch
  // (cos, sin) of the rotary angles of the first kDsTabStreams streams of the list, [stream][d/2]: computed once by
  // the workgroup instead of once per query row (the gq heads of a stream share them)
  f32x2 cs[kDsTabStreams][D / 2];
};

template <int D, int C>
__global__ __launch_bounds__(256 * C, 1) void decode_shared_mfma_kernel(DecodeParams p) {
  constexpr int KSTEPS = D / 16, DB = D / 32;
  constexpr int ROWS = 32 * C;
  constexpr int DBH = DB / 2;                      // d blocks per wave: each wave accumulates half of the head dimension
  constexpr int STATE = DBH * 16 + 2;              // floats per lane in a merge
  using Sm = DsSmem<D>;
  static_assert(sizeof(Sm::tile) >= (size_t)C * 2 * STATE * kWave * sizeof(float), "merge buffers");
  __shared__ Sm sm;

  // Workgroup -> (kv head c, sequence s, key split z).  Linear ids go to the 8 XCDs round-robin; the hkv workgroups that
  // read the interleaved head slices of the SAME cache rows (one (s, z), all c) get ids 8 apart, i.e. the same XCD and
  // neighbouring dispatch slots, so that their requests for one DRAM row arrive together.
  int c, s, z, own_pass;
  {
    const int n_sz = p.batch * p.n_splits * p.n_pass, n_sz8 = (n_sz + 7) / 8 * 8;
    const int L = blockIdx.x;
    const int sz = (L / (8 * p.hkv)) * 8 + L % 8;
    c = (L / 8) % p.hkv;
    if (sz >= n_sz || L >= n_sz8 * p.hkv) return;
    s = sz % p.batch; z = (sz / p.batch) % p.n_splits; own_pass = p.n_pass - 1 - sz / (p.batch * p.n_splits);
  }
  const DecodeLayer lv = layer_view(p, blockIdx.y);
  const int gq = p.hq / p.hkv;
  // the wave index is the same in all 64 lanes: saying so keeps the key loop and everything derived from the wave's
  // place in the workgroup in scalar registers
  const int lane = threadIdx.x % kWave, wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
  const int grp = wave / kDsGroupWaves, sub = wave % kDsGroupWaves;
  const int ksub = sub & 1, dh = sub >> 1;   // key sub-tile of the tile, half of the head dimension
  const int r32 = lane & 31, hf = lane >> 5;
  // Wave 0 builds the list of this sequence's streams below.  Its first look at the per-stream arrays is requested
  // here, ahead of everything else that goes to memory, so the lists, the sequence bounds and the first K/V tiles share
  // one round trip instead of queueing behind each other.
  int seq_of[4], gl[4], qp[4];
  auto fetch_lists = [&](int base) {
#pragma unroll
    for (int k4 = 0; k4 < 4; ++k4) {
      const int u = base + k4 * kWave + lane;
      const bool in = u < p.n_streams;
      seq_of[k4] = in ? p.stream_to_seq[u] : -1;
      gl[k4] = in ? clamp_gen_len(p.gen_len[u], p.gen_cap) : 0;
      qp[k4] = in ? p.q_pos[u] : 0;
    }
  };
  const bool causal = p.causal_rows > 0;
  if (wave == 0 && p.stream_to_seq && !causal) fetch_lists(0);
  int b0, ns;
  shared_bounds(p, s, b0, ns);
  const int j_begin = z * p.chunk;
  const int j_end = min(ns, j_begin + p.chunk);
  const int n_keys = max(j_end - j_begin, 0);
  const int n_tiles = (n_keys + kTileKeys - 1) / kTileKeys;

  const __bf16* Kg = (const __bf16*)lv.shared_k + ((long long)b0 * p.hkv + c) * D;
  const __bf16* Vg = (const __bf16*)lv.shared_v + ((long long)b0 * p.hkv + c) * D;
  const long long kv_stride = (long long)p.hkv * D;
  FragOffsets<D> fo;
  fo.init(lane);
  float* mbuf = (float*)&sm.tile[0][0][0] + (size_t)grp * 2 * STATE * kWave;
  // Staging: the 64-key tiles of this workgroup's key range stream from global memory straight into a ring of LDS
  // buffers, all waves sharing the instructions; the buffer descriptors cover exactly the rows of the range, so rows
  // past its end read as zeros (no clamping code, finite data for the masked tail).  Three tiles are on their way while
  // one is used: the stream is bound by memory latency times bytes in flight, so the kernel keeps as much of its LDS
  // in flight as it can and consumes in small pieces.
  using Stager = TileStager<D, 4 * C, kTileKeys>;
  constexpr int LPT = 2 * Stager::NI;  // loads per wave and tile (K and V)
  Stager stager;
  stager.init(Kg + j_begin * kv_stride, Vg + j_begin * kv_stride, n_keys, p.hkv, wave, lane);
  const unsigned lds_tiles = (unsigned)(size_t)(lds_void_ptr)&sm.tile[0][0][0];
  auto issue_tile = [&](int t) {
    const unsigned at = lds_tiles + (unsigned)((t % kDsRing) * 2 * kTileKeys * D * 2);
    stager.issue(stager.k_rsrc, at, t);
    stager.issue(stager.v_rsrc, at + (unsigned)(kTileKeys * D * 2), t);
  };
  auto issue_first_tiles = [&](int nt) {
#pragma unroll
    for (int t = 0; t < kDsRing - 1; ++t)
      if (t < nt) issue_tile(t);
  };
  // the first tiles are requested before anything else: they fly while the stream list is built and the queries are
  // rotated
  issue_first_tiles(n_tiles);

  // ---- streams (beams) of this sequence, ascending ----
  if (wave == 0) {
    int count = 0, gmax = 0;
    if (causal) {
      count = p.causal_rows;
      for (int i = lane; i < count; i += kWave) {
        sm.streams[i] = s * count + i;
        sm.glen[i] = 0;
        sm.qpos[i] = (float)p.q_pos[s * count + i];
      }
    } else if (!p.stream_to_seq) {
      gmax = clamp_gen_len(p.gen_len[s], p.gen_cap);
      if (lane == 0) { sm.streams[0] = s; sm.glen[0] = gmax; sm.qpos[0] = (float)p.q_pos[s]; }
      count = 1;
    } else {
      for (int base = 0; base < p.n_streams; base += 4 * kWave) {
        if (base > 0) fetch_lists(base);  // four chunks of the three lists per memory round trip
#pragma unroll
        for (int k4 = 0; k4 < 4; ++k4) {
          const bool hit = seq_of[k4] == s;
          const unsigned long long mask = __ballot(hit);
          const int idx = count + __popcll(mask & ((1ull << lane) - 1ull));
          if (hit && idx < kMaxStreamsPerSeq) {
            sm.streams[idx] = base + k4 * kWave + lane;
            sm.glen[idx] = gl[k4];
            sm.qpos[idx] = (float)qp[k4];
            gmax = max(gmax, gl[k4]);
          }
          count += __popcll(mask);
        }
      }
      if (count > kMaxStreamsPerSeq) count = kMaxStreamsPerSeq;
#pragma unroll
      for (int off = 1; off < kWave; off <<= 1) gmax = max(gmax, __shfl_xor(gmax, off, kWave));
    }
    if (lane == 0) { sm.n_streams_of_seq = count; sm.gen_pitch = gmax + 1; }
  }
  __syncthreads();
  const int n_st = sm.n_streams_of_seq;
  const int M = n_st * gq;  // query rows sharing this cache
  // the generated part as a key list of its own: n_st streams x gp rows (rows past a stream's own length are masked)
  const int gp = sm.gen_pitch;
  const int n_gen_keys = causal ? 0 : n_st * gp;
  const int n_gen_tiles = (n_gen_keys + kTileKeys - 1) / kTileKeys;
  const int tg0 = p.n_splits - 1 - z;  // this workgroup takes generated tiles tg0, tg0 + n_splits, ...: the last split,
                                       // whose key range is the shortest, takes the first
  // ---- the queries of the first 32 * C rows are requested before the rotary table is worked out, and rotated after ----
  // row m of the cache's query rows is head c*gq + m % gq of listed stream m / gq; a group's lane holds row r32 and,
  // per k-step, elements [16 ks + 8 hf, + 8) of both rotary halves
  u32x4 q_lo[KSTEPS / 2], q_hi[KSTEPS / 2];
  auto load_q_raw = [&](int row0) {
    const int m = min(row0 + 32 * grp + r32, M - 1);
    const __bf16* qrow = (const __bf16*)lv.q + ((long long)sm.streams[m / gq] * p.hq + head_of_slot(p.heads, c * gq + m % gq)) * D + 8 * hf;
#pragma unroll
    for (int ks = 0; ks < KSTEPS / 2; ++ks) {
      q_lo[ks] = *(const u32x4*)(qrow + 16 * ks);
      q_hi[ks] = *(const u32x4*)(qrow + 16 * ks + D / 2);
    }
  };
  if (M > 0) load_q_raw(p.n_pass > 1 ? min(own_pass * ROWS, M - 1) : 0);
  // rotary factors of the tabulated streams, one (stream, pair) per thread and pass
  if (p.rope.enabled) {
    const int n_tab = min(sm.n_streams_of_seq, kDsTabStreams);
    for (int i = threadIdx.x; i < n_tab * (D / 2); i += 256 * C) {
      const int e = i % (D / 2);
      float sn, cs;
      sincos_turns_fast(rope_turns(sm.qpos[i / (D / 2)], p.rope.hi[e], p.rope.lo[e]), &sn, &cs);
      sm.cs[i / (D / 2)][e] = f32x2{cs, sn};
    }
  }

  lds_barrier();  // the table of rotary factors is complete

  // ---- a tile of the generated key list, fetched into registers (one 16-byte unit of K and of V per thread and pass):
  // rows of the streams' generated caches as stored; the row after a stream's last one is its new token, whose key is
  // rotated and rounded here and, with `append`, written to its cache slot together with the value ----
  constexpr int UPR = D / 8, NCH = kTileKeys * UPR / (256 * C);
  static_assert(NCH >= 1 && NCH * 256 * C == kTileKeys * UPR);
  u32x4 gk[NCH], gv[NCH];
  auto load_gen_tile = [&](int tg, bool append) {
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
      const int unit = threadIdx.x + i * 256 * C;
      const int row = unit / UPR, ch = unit % UPR;
      const int e = tg * kTileKeys + row;
      const int si = e / gp, ri = e - si * gp;
      u32x4 kx = {0u, 0u, 0u, 0u}, vx = {0u, 0u, 0u, 0u};
      if (si < n_st) {
        const int u = sm.streams[si], g = sm.glen[si];
        const long long row0_of_u = (((long long)u * p.gen_cap) * p.hkv + c) * D + ch * 8;
        if (ri < g) {
          long long from = row0_of_u;  // the physical stream that holds logical row ri (an ancestor's slot under beam search)
          if (p.gen_src) {
            const int src = max(min(p.gen_src[(long long)u * p.gen_cap + ri], p.n_streams - 1), 0);
            from += (long long)(src - u) * p.gen_cap * kv_stride;
          }
          kx = *(const u32x4*)((const __bf16*)lv.gen_k + from + ri * kv_stride);
          vx = *(const u32x4*)((const __bf16*)lv.gen_v + from + ri * kv_stride);
        } else if (ri == g) {
          const long long tok = ((long long)u * p.hkv + c) * D;
          float x[8], y[8];  // this unit's elements and their rotary partners (the unit half a row away)
          Row8<__bf16>::load((const __bf16*)lv.k_new + tok + ch * 8, x);
          Row8<__bf16>::load((const __bf16*)lv.k_new + tok + (ch ^ (UPR / 2)) * 8, y);
          vx = *(const u32x4*)((const __bf16*)lv.v_new + tok + ch * 8);
          const bool upper = ch >= UPR / 2;
          const float pos = sm.qpos[si];
#pragma unroll
          for (int j = 0; j < 8; ++j) {
            const int pe = (ch % (UPR / 2)) * 8 + j;
            float sn = 0.f, cs = 1.f;
            if (p.rope.enabled) {
              if (si < kDsTabStreams) { const f32x2 t = sm.cs[si][pe]; cs = t[0]; sn = t[1]; }
              else sincos_turns_fast(rope_turns(pos, p.rope.hi[pe], p.rope.lo[pe]), &sn, &cs);
            }
            x[j] = upper ? x[j] * cs + y[j] * sn : x[j] * cs - y[j] * sn;
          }
#pragma unroll
          for (int j = 0; j < 4; ++j) kx[j] = pack_bf16(x[2 * j], x[2 * j + 1]);
          if (append) {
            *(u32x4*)((__bf16*)lv.gen_k + row0_of_u + g * kv_stride) = kx;
            *(u32x4*)((__bf16*)lv.gen_v + row0_of_u + g * kv_stride) = vx;
          }
        }
      }
      gk[i] = kx;
      gv[i] = vx;
    }
  };
  auto store_gen_tile = [&](int slot) {
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
      const int unit = threadIdx.x + i * 256 * C;
      const int row = unit / UPR, ch = unit % UPR;
      const int off = row * D + ((ch ^ swz<D>(row)) << 3);
      *(u32x4*)(sm.tile[slot][0] + off) = gk[i];
      *(u32x4*)(sm.tile[slot][1] + off) = gv[i];
    }
  };
  // the first generated tile of this workgroup is requested now, in the shadow of the first K/V tiles, and waits in
  // registers until the key loop is through
  bool gen_tile_in_regs = tg0 < n_gen_tiles;
  if (gen_tile_in_regs) load_gen_tile(tg0, own_pass == 0);  // one pass appends the new tokens

  const int row_begin = p.n_pass > 1 ? own_pass * ROWS : 0;
  const int row_end = p.n_pass > 1 && own_pass < p.n_pass - 1 ? min(M, row_begin + ROWS) : M;
  for (int row0 = row_begin; row0 < row_end; row0 += ROWS) {
    // ---- Q fragments of this group's rows, rotated and pre-scaled ----
    const bool grp_active = row0 + 32 * grp < M;
    bf16x8 qf[KSTEPS];
    int row_u, row_a;
    if (row0 > row_begin) load_q_raw(row0);
    {
      const int m = min(row0 + 32 * grp + r32, M - 1);
      row_u = sm.streams[m / gq]; row_a = head_of_slot(p.heads, c * gq + m % gq);
      const float pos = sm.qpos[m / gq];
#pragma unroll
      for (int ks = 0; ks < KSTEPS / 2; ++ks) {
        float lo[8], hi[8];
        Row8<__bf16>::unpack(q_lo[ks], lo);
        Row8<__bf16>::unpack(q_hi[ks], hi);
        u32x4 wl, wh;
#pragma unroll
        for (int j = 0; j < 8; j += 2) {
          float x[2], y[2];
#pragma unroll
          for (int jj = 0; jj < 2; ++jj) {
            float sn = 0.f, cs = 1.f;
            const int e = 16 * ks + 8 * hf + j + jj;
            if (p.rope.enabled) {
              if (m / gq < kDsTabStreams) { const f32x2 t = sm.cs[m / gq][e]; cs = t[0]; sn = t[1]; }
              else sincos_turns_fast(rope_turns(pos, p.rope.hi[e], p.rope.lo[e]), &sn, &cs);
            }
            x[jj] = (lo[j + jj] * cs - hi[j + jj] * sn) * p.scale_log2;
            y[jj] = (hi[j + jj] * cs + lo[j + jj] * sn) * p.scale_log2;
          }
          wl[j / 2] = pack_bf16(x[0], x[1]);
          wh[j / 2] = pack_bf16(y[0], y[1]);
        }
        qf[ks] = __builtin_bit_cast(bf16x8, wl);
        qf[ks + KSTEPS / 2] = __builtin_bit_cast(bf16x8, wh);
      }
    }

    f32x16 o[DBH];  // d blocks dh * DBH + (0 .. DBH-1)
#pragma unroll
    for (int db = 0; db < DBH; ++db)
#pragma unroll
      for (int i = 0; i < 16; ++i) o[db][i] = 0.f;
    float mrow = -INFINITY, lrow = 0.f;
    f32x16 neg_m;  // -m in every register; +inf while there is no reference yet, which sends the first tile down the exact path
#pragma unroll
    for (int i = 0; i < 16; ++i) neg_m[i] = INFINITY;

    // S^T = K Q^T of this wave's sub-tile (the two waves that share a sub-tile both compute it: the matrix core has
    // time to spare here, LDS space has not); keys past the range end get zero weight
    // SHIFTED: the accumulator starts at -m in every register (the steady state: no subtraction on the vector ALU),
    // else at 0 (the exact path, which needs the raw scores)
    const int q_si = min(row0 + 32 * grp + r32, M - 1) / gq;
    // causal rows: this lane's row sees keys 0 .. my_pos, the wave's rows at least 0 .. wave_min_pos
    int my_pos = 0, wave_min_pos = 0, wave_max_pos = 0;
    int nt = n_tiles;  // tiles of the key range this pass walks: with causal rows, those holding a key some row sees
    if (causal) {
      my_pos = (int)sm.qpos[q_si];
      wave_min_pos = wave_max_pos = my_pos;
#pragma unroll
      for (int off = 1; off < 32; off <<= 1) {
        wave_min_pos = min(wave_min_pos, __shfl_xor(wave_min_pos, off, kWave));
        wave_max_pos = max(wave_max_pos, __shfl_xor(wave_max_pos, off, kWave));
      }
      wave_min_pos = __builtin_amdgcn_readfirstlane(wave_min_pos);
      wave_max_pos = __builtin_amdgcn_readfirstlane(wave_max_pos);
      int pass_max_pos = 0;
      for (int i = row0 / gq; i <= min(M - 1, row0 + ROWS - 1) / gq; ++i) pass_max_pos = max(pass_max_pos, (int)sm.qpos[i]);
      pass_max_pos = __builtin_amdgcn_readfirstlane(pass_max_pos);
      nt = min(n_tiles, (max(pass_max_pos + 1 - j_begin, 0) + kTileKeys - 1) / kTileKeys);
    }
    // `mask` sets the scores of keys this lane's query row must not see to -inf
    auto scores = [&](int slot, f32x16& sc, auto shifted, auto mask) {
      const __bf16* my_k = sm.tile[slot][0] + ksub * kDsTile * D;
      if constexpr (decltype(shifted)::value) {
        sc = neg_m;
      } else {
#pragma unroll
        for (int i = 0; i < 16; ++i) sc[i] = 0.f;
      }
      // all K fragments of the sub-tile are requested before the first MFMA: the products form one dependent chain, and
      // a read per step would put the LDS latency into every link
      bf16x8 kf[KSTEPS];
#pragma unroll
      for (int ks = 0; ks < KSTEPS; ++ks) kf[ks] = *(const bf16x8*)(my_k + fo.k(ks));
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int ks = 0; ks < KSTEPS; ++ks) sc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[ks], qf[ks], sc, 0, 0, 0);
      mask(sc);
    };
    // register i of a score tile is key 8 (i / 4) + 4 hf + i % 4 of the wave's 32-key sub-tile
    // shared rows: keys past the end of the workgroup's key range
    auto range_mask = [&](int it) {
      return [&, it](f32x16& sc) {
        const int key0 = j_begin + it * kTileKeys + ksub * kDsTile;
        if (key0 + kDsTile > j_end) {
#pragma unroll
          for (int i = 0; i < 16; ++i)
            if (key0 + 8 * (i >> 2) + 4 * hf + (i & 3) >= j_end) sc[i] = -INFINITY;
        }
        if (causal && key0 + kDsTile - 1 > wave_min_pos) {
#pragma unroll
          for (int i = 0; i < 16; ++i)
            if (key0 + 8 * (i >> 2) + 4 * hf + (i & 3) > my_pos) sc[i] = -INFINITY;
        }
      };
    };
    // generated rows: a query row sees keys [gen_lo, gen_hi] of the generated key list, its own stream's rows
    // including the new token
    const int gen_lo = q_si * gp, gen_hi = gen_lo + sm.glen[q_si];
    auto gen_mask = [&](int tg) {
      return [&, tg](f32x16& sc) {
        const int e0 = tg * kTileKeys + ksub * kDsTile + 4 * hf;
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const int e = e0 + 8 * (i >> 2) + (i & 3);
          if (e < gen_lo || e > gen_hi) sc[i] = -INFINITY;
        }
      };
    };
    // P = exp2(S - m) of scores that already carry -m, as the bf16 B operands of the second product, and the lane's
    // share of the row sum (over the rounded probabilities, two per instruction)
    auto softmax_tile = [&](const f32x16& sc, bf16x8 (&pf)[2], float& lsum) {
      float s0 = 0.f, s1 = 0.f;
#pragma unroll
      for (int kk = 0; kk < 2; ++kk) {
        u32x4 w;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          w[j] = pack_bf16(__builtin_amdgcn_exp2f(sc[8 * kk + 2 * j]), __builtin_amdgcn_exp2f(sc[8 * kk + 2 * j + 1]));
          add_pair(j & 1 ? s1 : s0, w[j]);
        }
        pf[kk] = __builtin_bit_cast(bf16x8, w);
      }
      lsum = add_chains(s0, s1);
    };
    // V^T fragments of this wave's sub-tile and half of the head dimension, requested ahead of the exponentials
    auto fetch_v = [&](int slot, bf16x8 (&vf)[2][DBH]) {
      const __bf16* my_v = sm.tile[slot][1] + ksub * kDsTile * D;
#pragma unroll
      for (int kk = 0; kk < 2; ++kk)
#pragma unroll
        for (int db = 0; db < DBH; ++db) vf[kk][db] = read_v_fragment<D>(my_v, fo, dh * DBH + db, kk);
      __builtin_amdgcn_sched_barrier(0);
    };
    auto accumulate = [&](const bf16x8 (&pf)[2], float lsum, const bf16x8 (&vf)[2][DBH]) {
      lrow += lsum;
#pragma unroll
      for (int kk = 0; kk < 2; ++kk)
#pragma unroll
        for (int db = 0; db < DBH; ++db)
          o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[kk][db], pf[kk], o[db], 0, 0, 0);
    };
    // A new reference for the rows of a tile whose raw scores are in `sc` (the exact path): the exact row maxima enter
    // the running ones, sums and outputs are rescaled, and the scores leave relative to the new reference.  A row that
    // has not met a visible key yet (every score so far masked) keeps "no reference".
    auto rebase = [&](f32x16& sc) {
      float m = sc[0];
#pragma unroll
      for (int i = 1; i < 16; ++i) m = fmaxf(m, sc[i]);
      m = fmaxf(m, __shfl_xor(m, 32, kWave));
      const float mnew = fmaxf(mrow, m);
      const float ref = mnew == -INFINITY ? 0.f : mnew;
      const float alpha = __builtin_amdgcn_exp2f(mrow - ref);  // 0 for a row without a reference: its sums are 0
      mrow = mnew;
      lrow *= alpha;
#pragma unroll
      for (int db = 0; db < DBH; ++db)
#pragma unroll
        for (int i = 0; i < 16; ++i) o[db][i] *= alpha;
      const float nm = mnew == -INFINITY ? INFINITY : -mnew;
#pragma unroll
      for (int i = 0; i < 16; ++i) { neg_m[i] = nm; sc[i] -= ref; }
    };
    // does this wave have keys in super-tile `it`?
    auto has_keys = [&](int it) {
      const int k0 = it * kTileKeys + ksub * kDsTile;
      return grp_active && k0 < n_keys && (!causal || j_begin + k0 <= wave_max_pos);
    };

    // Every tile iteration opens with exactly one barrier, whichever path a wave takes.  The steady-state loop takes
    // exponentials against the reference maximum it has and never touches the output accumulators with the vector
    // ALU; a reference is stale exactly when some exponential is large, which shows in the partial row sums
    // (+inf / NaN on the first tile, whose reference is -inf).  A wave that sees a stale reference leaves the loop,
    // takes the exact maxima of the tile, rescales, finishes the tile and re-enters.
    if (row0 > row_begin) issue_first_tiles(nt);  // further passes over the same keys for more query rows
    // Iteration `it` opens with the barrier behind which tile `it` is complete (every wave has waited for its own part:
    // loads complete in order, so that means at most the younger tiles' loads are still in flight) and nobody reads
    // tile it-1 any more, whose ring slot the loads of tile it+3 then start to fill.
    auto sync_and_stage = [&](int it) {
      const int younger = min(nt - 1 - it, kDsRing - 2);  // tiles issued after tile `it` (at least)
      if (younger >= 2) wait_vmcnt<2 * LPT>();
      else if (younger == 1) wait_vmcnt<LPT>();
      else wait_vmcnt<0>();
      lds_barrier();
      if (it + kDsRing - 1 < nt) issue_tile(it + kDsRing - 1);
    };
    int it = 0;
    while (it < nt) {
      bool rescale = false;
      for (; it < nt; ++it) {
        sync_and_stage(it);
        if (has_keys(it)) {
          f32x16 sc;
          float lsum;
          bf16x8 vf[2][DBH], pf[2];
          scores(it % kDsRing, sc, std::true_type{}, range_mask(it));
          fetch_v(it % kDsRing, vf);
          softmax_tile(sc, pf, lsum);
          if (__any(!(lsum <= kDecSumLimit))) { rescale = true; break; }
          accumulate(pf, lsum, vf);
        }
      }
      if (!rescale) break;
      {
        f32x16 sc;
        float lsum;
        bf16x8 vf[2][DBH], pf[2];
        scores(it % kDsRing, sc, std::false_type{}, range_mask(it));  // the tile is still staged
        fetch_v(it % kDsRing, vf);
        rebase(sc);
        softmax_tile(sc, pf, lsum);
        accumulate(pf, lsum, vf);
        ++it;
      }
    }

    // Tiles requested before the pass knew how few it needs (causal rows) may still be on their way into the ring;
    // nothing may be, past this point: the ring's memory is about to be written by the workgroup itself.
    wait_vmcnt<0>();

    // ---- the generated key list: this workgroup's tiles of it, one at a time through ring slot 0 ----
    for (int tg = tg0; tg < n_gen_tiles; tg += p.n_splits) {
      if (!gen_tile_in_regs) load_gen_tile(tg, row0 == row_begin && own_pass == 0);
      gen_tile_in_regs = false;
      __syncthreads();  // nobody reads the slot any more (all of the workgroup's loads into LDS have landed long ago)
      store_gen_tile(0);
      __syncthreads();
      if (grp_active && tg * kTileKeys + ksub * kDsTile < n_gen_keys) {
        f32x16 sc;
        float lsum;
        bf16x8 vf[2][DBH], pf[2];
        scores(0, sc, std::true_type{}, gen_mask(tg));
        fetch_v(0, vf);
        softmax_tile(sc, pf, lsum);
        if (__any(!(lsum <= kDecSumLimit))) {
          scores(0, sc, std::false_type{}, gen_mask(tg));
          rebase(sc);
          softmax_tile(sc, pf, lsum);
        }
        accumulate(pf, lsum, vf);
      }
    }
    __syncthreads();  // every wave is done with the tiles: their memory becomes the merge buffers

    // ---- merge the two key sub-tiles of each half of the head dimension: wave (ksub 1, dh) -> wave (ksub 0, dh);
    // lane-wise, the layouts are identical ----
    auto put = [&](int slot) {
      float* dst = mbuf + (size_t)slot * STATE * kWave + lane;
      int r = 0;
      dst[(r++) * kWave] = mrow;
      dst[(r++) * kWave] = lrow;
#pragma unroll
      for (int db = 0; db < DBH; ++db)
#pragma unroll
        for (int i = 0; i < 16; ++i) dst[(r++) * kWave] = o[db][i];
    };
    auto take = [&](int slot) {
      const float* src = mbuf + (size_t)slot * STATE * kWave + lane;
      int r = 0;
      const float m2 = src[(r++) * kWave], l2 = src[(r++) * kWave];
      const float mn = fmaxf(mrow, m2);
      const float a = mrow == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(mrow - mn);
      const float b = m2 == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(m2 - mn);
      lrow = lrow * a + l2 * b;
      mrow = mn;
#pragma unroll
      for (int db = 0; db < DBH; ++db)
#pragma unroll
        for (int i = 0; i < 16; ++i) o[db][i] = o[db][i] * a + src[(r++) * kWave] * b;
    };
    if (ksub == 1) put(dh);
    __syncthreads();
    if (ksub == 0) {
      take(dh);
      // ---- partial results of this key range: unnormalised O (this wave's half of the head dimension), running max
      // and sum (base-2 units; both halves hold the same ones) ----
      const float ltot = lrow + __shfl_xor(lrow, 32, kWave);
      const int m = row0 + 32 * grp + r32;
      if (m < M && p.n_slots == 1) {
        // nothing was split: this is the whole key list of the row (the new token is always among the keys, so the
        // sum is positive); normalise and store the final output
        const float inv = 1.f / ltot;
        __bf16* po = (__bf16*)lv.out + ((long long)row_u * p.hq + row_a) * D + dh * (D / 2) + 4 * hf;
#pragma unroll
        for (int db = 0; db < DBH; ++db)
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            u32x2 w = {pack_bf16(o[db][4 * j] * inv, o[db][4 * j + 1] * inv),
                       pack_bf16(o[db][4 * j + 2] * inv, o[db][4 * j + 3] * inv)};
            *(u32x2*)(po + 32 * db + 8 * j) = w;
          }
      } else if (m < M) {
        const long long slot = ((long long)row_u * p.hq + row_a) * p.n_slots + z;
        float* po = lv.part_o + slot * D + dh * (D / 2) + 4 * hf;
#pragma unroll
        for (int db = 0; db < DBH; ++db)
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            f32x4 w = {o[db][4 * j], o[db][4 * j + 1], o[db][4 * j + 2], o[db][4 * j + 3]};
            *(f32x4*)(po + 32 * db + 8 * j) = w;
          }
        if (hf == 0 && dh == 0) { lv.part_ml[slot * 2] = mrow; lv.part_ml[slot * 2 + 1] = ltot; }
      }
    }
    __syncthreads();  // the merge buffers are tile memory again in the next row chunk
  }
  wait_vmcnt<0>();  // a workgroup without query rows still has its first tiles on their way into LDS
}

// ------------------------------------------------------------------------------------------------------------------
// host side
// ------------------------------------------------------------------------------------------------------------------
struct DecodePlan {
  bool mfma;      // shared and generated rows on the matrix cores + combine
  int n_splits;   // key-range splits of the shared (mfma) or whole (vector) key list
  int n_slots;    // partial slots per (stream, head)
  int chunk;      // keys per split
  int n_pass;     // matrix-core kernel: passes of 64 query rows that get workgroups of their own (1: the rows of a cache
                  // beyond the first 64, if any, are taken in further passes of the same workgroup)
};

static DecodePlan plan_decode(int dtype, int hq, int hkv, int n_streams, int batch, int max_shared_len, int gen_cap,
                              int n_layers = 1) {
  DecodePlan pl;
  const int gq = hq / hkv;
  // several query rows per cache (grouped heads or beams) make the shared part a matrix product
  // (short caches are launch-latency bound: the single-launch vector kernel wins there)
  const int mfma_min = tuning(kTuneDecMfmaMinLen, 128);
  // ... unless all its workgroups (one per CU: they hold most of the LDS) fit on the GPU at once, or beams share the
  // caches (measured on 28 layers of 64-row caches in one launch: 10 beams x 4 grouped heads per cache, 194 us against
  // 372 us for the vector kernel, which reads a cache once per beam; 7 grouped heads without beams, 37 against 23 us)
  const int mfma_wgs = tuning(kTuneDecMfmaShortWgs, 256);
  pl.mfma = dtype == EARN_BF16 && (gq > 1 || n_streams > batch) &&
            (max_shared_len >= mfma_min || (long long)hkv * batch * n_layers <= mfma_wgs || n_streams >= 2 * batch);
  pl.n_pass = 1;
  if (pl.mfma) {
    // Beams beyond 64 query rows per cache (say 20 beams of 7 grouped heads) would make a workgroup walk its keys once
    // per 64 rows.  Planned from the average beam count, every such pass gets workgroups of its own, with fewer key
    // splits: the passes of a (sequence, kv head) then run side by side on one XCD and share the keys in its L2.  (The
    // last pass takes whatever rows a sequence has beyond the plan.)
    const long long rows_bound = (long long)gq * (n_streams - batch + 1), rows_avg = (long long)gq * ((n_streams + batch - 1) / batch);
    if (rows_bound > 32 && rows_avg > 64) pl.n_pass = (int)((rows_avg + 63) / 64);
    long long base = (long long)hkv * batch * pl.n_pass * n_layers;
    const int wg_env = tuning(kTuneDecMfmaWgs, 256);
    int want = (int)((wg_env + base - 1) / base);               // one workgroup per CU: it holds 8 waves and most of the LDS
    int cap = (max_shared_len + kDsSuper - 1) / kDsSuper;  // at least one super-tile per workgroup
    int n = want < cap ? want : cap;
    if (n < 1) n = 1;
    if (n > 64) n = 64;
    pl.n_splits = n;
    pl.n_slots = n;
    pl.chunk = (((max_shared_len + n - 1) / n) + kDsSuper - 1) / kDsSuper * kDsSuper;
  } else {
    const int max_total = max_shared_len + gen_cap;
    // aim at >= 1024 workgroups (4 per CU) while keeping at least 256 keys per split
    long long base = (long long)hkv * n_streams * n_layers;
    const int wgs_env = tuning(kTuneDecVecWgs, 1024);
    int want = (int)((wgs_env + base - 1) / base);
    int cap = (max_total + 255) / 256;
    int n = want < cap ? want : cap;
    if (n < 1) n = 1;
    if (n > 64) n = 64;
    pl.n_splits = n;
    pl.n_slots = n;
    pl.chunk = (((max_total + n - 1) / n) + 63) / 64 * 64;
  }
  return pl;
}

// partial results: [layers][rows][d] floats, then [layers][rows][2] floats
size_t decode_workspace_bytes(int dtype, int hq, int hkv, int d, int n_streams, int batch, int max_shared_len,
                              int gen_cap, int n_layers) {
  DecodePlan pl = plan_decode(dtype, hq, hkv, n_streams, batch, max_shared_len, gen_cap, n_layers);
  if (pl.n_slots == 1) return 0;  // nothing is split: the kernels write the final outputs themselves
  size_t rows = (size_t)n_streams * hq * pl.n_slots * n_layers;
  return rows * d * sizeof(float) + rows * 2 * sizeof(float);
}

template <typename T, int D, int WAVES>
static void launch_vector_w(const DecodeParams& p, int gq, dim3 grid, hipStream_t stream) {
  dim3 block(kWave * WAVES);
  if (gq == 1) hipLaunchKernelGGL((decode_kernel<T, D, 1, WAVES>), grid, block, 0, stream, p);
  else if (gq == 2) hipLaunchKernelGGL((decode_kernel<T, D, 2, WAVES>), grid, block, 0, stream, p);
  else if (gq <= 4) hipLaunchKernelGGL((decode_kernel<T, D, 4, WAVES>), grid, block, 0, stream, p);
  else hipLaunchKernelGGL((decode_kernel<T, D, 8, WAVES>), grid, block, 0, stream, p);
}
template <typename T, int D>
static void launch_vector(const DecodeParams& p, int gq, dim3 grid, hipStream_t stream) {
  // Short key lists are latency bound: every wave repeats the prologue (query rotation), and what counts is that all
  // workgroups are resident at once.  One wave per (stream, kv head) for a single query head, two for grouped heads
  // (more arithmetic per key); long key lists take four.
  const int waves_env = tuning(kTuneDecVecWaves, 0);
  const int waves = waves_env ? waves_env : (p.chunk > 128 ? 4 : (gq == 1 ? 1 : 2));
  if (waves == 1) launch_vector_w<T, D, 1>(p, gq, grid, stream);
  else if (waves == 2) launch_vector_w<T, D, 2>(p, gq, grid, stream);
  else launch_vector_w<T, D, 4>(p, gq, grid, stream);
}

template <typename T, int D>
static void launch_combine(const DecodeParams& p, hipStream_t stream, int n_layers = 1) {
  const int rows = p.n_streams * p.hq;
  const int threads = rows * (D / 8);
  hipLaunchKernelGGL((decode_combine_kernel<T, D>), dim3((threads + 255) / 256, n_layers), dim3(256), 0, stream, p.part_o,
                     p.part_ml, (T*)p.out, rows, p.n_slots, p.ls_part_o, p.ls_part_ml, p.ls_out);
}

template <typename T, int D>
static void launch_decode_t(DecodeParams& p, const DecodePlan& pl, int gq, hipStream_t stream, int n_layers) {
  if (!pl.mfma) {
    launch_vector<T, D>(p, gq, dim3((unsigned)(((long long)p.n_streams * p.n_splits + 7) / 8 * 8 * p.hkv), n_layers, 1), stream);
    if (p.n_slots > 1) launch_combine<T, D>(p, stream, n_layers);
    return;
  }
  if constexpr (sizeof(T) == 2) {
    dim3 grid((unsigned)(((long long)p.batch * p.n_splits * p.n_pass + 7) / 8 * 8 * p.hkv), n_layers, 1);
    // one 32-row group is enough when a cache serves at most 32 query rows; with beams the host only has an upper bound
    const bool one_group = (long long)gq * (p.n_streams - p.batch + 1) <= 32;
    if (one_group) hipLaunchKernelGGL((decode_shared_mfma_kernel<D, 1>), grid, dim3(256), 0, stream, p);
    else hipLaunchKernelGGL((decode_shared_mfma_kernel<D, 2>), grid, dim3(512), 0, stream, p);
    if (p.n_slots > 1) launch_combine<T, D>(p, stream, n_layers);
  }
}

int launch_decode(const earn_attn_desc* desc, const void* q, const void* k_new, const void* v_new,
                  const int32_t* q_pos, const void* shared_k, const void* shared_v, const int32_t* shared_cu,
                  const int32_t* stream_to_seq, void* gen_k, void* gen_v, const int32_t* gen_len, int gen_cap,
                  int n_streams, int batch, int max_shared_len, int shared_total, void* out, void* workspace,
                  size_t workspace_bytes, hipStream_t stream, const DecodeLayers* layers, const int32_t* gen_src) {
  const int hq = desc->n_q_heads, hkv = desc->n_kv_heads, d = desc->head_dim, gq = hq / hkv;
  const int n_layers = layers ? layers->n_layers : 1;
  if (gq > 8) { set_error("earn_decode_attn: more than 8 query heads per kv head is not supported"); return EARN_ERR_UNSUPPORTED; }
  const DecodePlan pl = plan_decode(desc->dtype, hq, hkv, n_streams, batch, max_shared_len, gen_cap, n_layers);
  if (pl.mfma && (long long)(max_shared_len + kDsSuper) * hkv * d * 2 >= (1ll << 31)) {
    set_error("earn_decode_attn: a shared cache of %d rows exceeds the 2 GiB addressing range of one sequence", max_shared_len);
    return EARN_ERR_UNSUPPORTED;
  }
  // (what the host can tell without reading stream_to_seq: with more than 1024 streams per sequence ON AVERAGE some
  // sequence must exceed the limit; the exact check is part of the validation mode)
  if (pl.mfma && n_streams > (long long)kMaxStreamsPerSeq * batch) {
    set_error("earn_decode_attn: more than %d streams would share one sequence", kMaxStreamsPerSeq);
    return EARN_ERR_UNSUPPORTED;
  }
  DecodeParams p;
  p.q = q; p.k_new = k_new; p.v_new = v_new; p.q_pos = q_pos;
  p.shared_k = shared_k; p.shared_v = shared_v; p.shared_cu = shared_cu; p.stream_to_seq = stream_to_seq;
  p.gen_k = gen_k; p.gen_v = gen_v; p.gen_len = gen_len; p.out = out; p.gen_src = gen_src;
  p.gen_cap = gen_cap; p.n_streams = n_streams; p.batch = batch; p.hq = hq; p.hkv = hkv;
  p.shared_total = shared_total; p.max_shared_len = max_shared_len;
  p.n_splits = pl.n_splits; p.n_slots = pl.n_slots; p.chunk = pl.chunk; p.causal_rows = 0; p.n_pass = pl.n_pass;
  const size_t need = decode_workspace_bytes(desc->dtype, hq, hkv, d, n_streams, batch, max_shared_len, gen_cap, n_layers);
  if (need > workspace_bytes || (need > 0 && !workspace)) {
    set_error("earn_decode_attn: workspace too small (%zu bytes given, %zu needed)", workspace_bytes, need);
    return EARN_ERR_WORKSPACE_TOO_SMALL;
  }
  const size_t part_rows = (size_t)n_streams * hq * p.n_slots;  // per layer
  p.part_o = (float*)workspace;
  p.part_ml = p.part_o + part_rows * d * n_layers;
  p.ls_part_o = (long long)(part_rows * d * sizeof(float));
  p.ls_part_ml = (long long)(part_rows * 2 * sizeof(float));
  p.ls_q = layers ? layers->q : 0; p.ls_kv_new = layers ? layers->kv_new : 0; p.ls_shared = layers ? layers->shared : 0;
  p.ls_gen = layers ? layers->gen : 0; p.ls_out = layers ? layers->out : 0;
  const float scale = desc->softmax_scale > 0.f ? desc->softmax_scale : 1.0f / sqrtf((float)d);
  p.scale_log2 = scale * 1.4426950408889634f;
  p.rope = make_rope_table(desc->rope_base, d);
  if (make_head_map(desc, &p.heads, "earn_decode_attn") != EARN_OK) return EARN_ERR_UNSUPPORTED;
  if (desc->dtype == EARN_F32) {
    if (d == 64) launch_decode_t<float, 64>(p, pl, gq, stream, n_layers); else launch_decode_t<float, 128>(p, pl, gq, stream, n_layers);
  } else {
    if (d == 64) launch_decode_t<__bf16, 64>(p, pl, gq, stream, n_layers); else launch_decode_t<__bf16, 128>(p, pl, gq, stream, n_layers);
  }
  return hipGetLastError() == hipSuccess ? EARN_OK : EARN_ERR_HIP;
}

// ---- the entry point that allocates nothing: split-key partials in a buffer inside the library ----
// One copy of the array exists per GPU, each at its own address; in host code its name is only a handle for
// hipGetSymbolAddress, never a pointer a kernel could take.
constexpr size_t kStaticScratchBytes = EARN_STATIC_SCRATCH_BYTES;
constexpr int kMaxDevices = 64;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

// device address of `scratch` on the current GPU, looked up on the first call made with that GPU current
static int static_scratch_of_current_device(void** ptr) {
  static std::mutex mu;
  static void* address[kMaxDevices] = {};
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) {
    set_error("earn_decode_attn_static: no current GPU (device %d)", dev);
    return EARN_ERR_HIP;
  }
  std::lock_guard<std::mutex> lock(mu);
  if (!address[dev]) {
    void* p = nullptr;
    const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !p) {
      set_error("earn_decode_attn_static: hipGetSymbolAddress failed on device %d: %s", dev, hipGetErrorString(e));
      return EARN_ERR_HIP;
    }
    address[dev] = p;
  }
  *ptr = address[dev];
  return EARN_OK;
}

int launch_decode_static(const earn_attn_desc* desc, const void* q, const void* k_new, const void* v_new,
                         const int32_t* q_pos, const void* shared_k, const void* shared_v, const int32_t* shared_cu,
                         const int32_t* stream_to_seq, void* gen_k, void* gen_v, const int32_t* gen_len, int gen_cap,
                         int n_streams, int batch, int max_shared_len, int shared_total, void* out, hipStream_t stream) {
  const size_t need = decode_workspace_bytes(desc->dtype, desc->n_q_heads, desc->n_kv_heads, desc->head_dim, n_streams,
                                             batch, max_shared_len, gen_cap, 1);
  if (need > kStaticScratchBytes) {
    set_error("earn_decode_attn_static: the partial results of this problem need %zu bytes, the library's buffer holds "
              "%zu; use earn_decode_attn with a workspace", need, kStaticScratchBytes);
    return EARN_ERR_WORKSPACE_TOO_SMALL;
  }
  void* ptr = nullptr;
  const int rc = static_scratch_of_current_device(&ptr);
  if (rc != EARN_OK) return rc;
  return launch_decode(desc, q, k_new, v_new, q_pos, shared_k, shared_v, shared_cu, stream_to_seq, gen_k, gen_v, gen_len,
                       gen_cap, n_streams, batch, max_shared_len, shared_total, out, ptr, kStaticScratchBytes, stream, nullptr,
                       nullptr);
}

// ---- causal attention of r chosen rows per sequence over the sequence's full-length keys, on the shared-cache kernel:
// the rows of a (sequence, kv head) are its "beams" ----
// Every pass of 32 * C query rows gets workgroups of its own.  About half of the passes (the suffix registers' rows)
// walk the whole sequence, the others (prefix registers) a tile or two: the key range is split so that the long ones
// make about one workgroup per CU.
static DecodePlan plan_rows(int hkv, int batch, int max_seqlen, int rows_per_seq, int gq, int* n_pass) {
  DecodePlan pl;
  pl.mfma = true;
  const int m = rows_per_seq * gq, rows = m <= 32 ? 32 : 64;
  *n_pass = (m + rows - 1) / rows;
  const long long base = (long long)hkv * batch * ((*n_pass + 1) / 2);
  int n = (int)((256 + base - 1) / base);
  const int cap = (max_seqlen + kDsSuper - 1) / kDsSuper;
  if (n > cap) n = cap;
  if (n < 1) n = 1;
  if (n > 64) n = 64;
  pl.n_splits = pl.n_slots = n;
  pl.chunk = (((max_seqlen + n - 1) / n) + kDsSuper - 1) / kDsSuper * kDsSuper;
  return pl;
}

size_t prefill_rows_workspace_bytes(int hq, int hkv, int d, int batch, int max_seqlen, int rows_per_seq) {
  int n_pass;
  const DecodePlan pl = plan_rows(hkv, batch, max_seqlen, rows_per_seq, hq / hkv, &n_pass);
  if (pl.n_slots == 1) return 0;
  const size_t rows = (size_t)batch * rows_per_seq * hq * pl.n_slots;
  return rows * d * sizeof(float) + rows * 2 * sizeof(float);
}

int launch_prefill_rows(const earn_attn_desc* desc, const void* q_rows, const void* k_rot, const void* v,
                        const int32_t* cu_seqlens, const int32_t* row_pos, int batch, int total_tokens, int max_seqlen,
                        int rows_per_seq, void* out_rows, void* workspace, size_t workspace_bytes, hipStream_t stream) {
  const int hq = desc->n_q_heads, hkv = desc->n_kv_heads, d = desc->head_dim, gq = hq / hkv;
  if (desc->dtype != EARN_BF16) { set_error("earn_prefill_register_rows: bf16 only"); return EARN_ERR_UNSUPPORTED; }
  if (rows_per_seq > kMaxStreamsPerSeq) {
    set_error("earn_prefill_register_rows: more than %d rows per sequence", kMaxStreamsPerSeq);
    return EARN_ERR_UNSUPPORTED;
  }
  if ((long long)(max_seqlen + kDsSuper) * hkv * d * 2 >= (1ll << 31)) {
    set_error("earn_prefill_register_rows: a sequence of %d rows exceeds the 2 GiB addressing range of one sequence", max_seqlen);
    return EARN_ERR_UNSUPPORTED;
  }
  int n_pass;
  const DecodePlan pl = plan_rows(hkv, batch, max_seqlen, rows_per_seq, gq, &n_pass);
  const size_t need = prefill_rows_workspace_bytes(hq, hkv, d, batch, max_seqlen, rows_per_seq);
  if (need > workspace_bytes || (need > 0 && !workspace)) {
    set_error("earn_prefill_register_rows: workspace too small (%zu bytes given, %zu needed)", workspace_bytes, need);
    return EARN_ERR_WORKSPACE_TOO_SMALL;
  }
  DecodeParams p;
  p.q = q_rows; p.k_new = nullptr; p.v_new = nullptr; p.q_pos = row_pos;
  p.shared_k = k_rot; p.shared_v = v; p.shared_cu = cu_seqlens; p.stream_to_seq = nullptr;
  p.gen_k = nullptr; p.gen_v = nullptr; p.gen_len = nullptr; p.out = out_rows; p.gen_src = nullptr;
  p.gen_cap = 0; p.n_streams = batch * rows_per_seq; p.batch = batch; p.hq = hq; p.hkv = hkv;
  p.shared_total = total_tokens; p.max_shared_len = max_seqlen;
  p.n_splits = pl.n_splits; p.n_slots = pl.n_slots; p.chunk = pl.chunk; p.causal_rows = rows_per_seq; p.n_pass = n_pass;
  p.part_o = (float*)workspace;
  p.part_ml = p.part_o + (size_t)p.n_streams * hq * p.n_slots * d;
  p.ls_q = p.ls_kv_new = p.ls_shared = p.ls_gen = p.ls_out = p.ls_part_o = p.ls_part_ml = 0;
  const float scale = desc->softmax_scale > 0.f ? desc->softmax_scale : 1.0f / sqrtf((float)d);
  p.scale_log2 = scale * 1.4426950408889634f;
  p.rope = make_rope_table(desc->rope_base, d);
  if (make_head_map(desc, &p.heads, "earn_prefill_register_rows") != EARN_OK) return EARN_ERR_UNSUPPORTED;
  const dim3 grid((unsigned)(((long long)batch * p.n_splits * n_pass + 7) / 8 * 8 * hkv), 1, 1);
  const bool one_group = rows_per_seq * gq <= 32;
  if (d == 64) {
    if (one_group) hipLaunchKernelGGL((decode_shared_mfma_kernel<64, 1>), grid, dim3(256), 0, stream, p);
    else hipLaunchKernelGGL((decode_shared_mfma_kernel<64, 2>), grid, dim3(512), 0, stream, p);
    if (p.n_slots > 1) launch_combine<__bf16, 64>(p, stream);
  } else {
    if (one_group) hipLaunchKernelGGL((decode_shared_mfma_kernel<128, 1>), grid, dim3(256), 0, stream, p);
    else hipLaunchKernelGGL((decode_shared_mfma_kernel<128, 2>), grid, dim3(512), 0, stream, p);
    if (p.n_slots > 1) launch_combine<__bf16, 128>(p, stream);
  }
  return hipGetLastError() == hipSuccess ? EARN_OK : EARN_ERR_HIP;
}

}  // namespace earn
