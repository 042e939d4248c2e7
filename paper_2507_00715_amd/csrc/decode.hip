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
  int n_slots;    // partial-result slots per (stream, head) in the workspace: n_splits (+1 for the generated rows)
  int gen_only;   // 1: this launch covers only the stream's generated rows and the new token (slot n_slots-1)
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
  const int b0 = p.shared_cu[s];
  const int ns = p.gen_only ? 0 : p.shared_cu[s + 1] - b0;  // shared rows this launch walks
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
    if (p.n_slots == 1) {
      float inv = 1.f / l;
#pragma unroll
      for (int i = 0; i < 8; ++i) oo[i] *= inv;
      Row8<T>::store((T*)p.out + ((long long)u * p.hq + head) * D + sb * 8, oo);
    } else {
      const long long slot = ((long long)u * p.hq + head) * p.n_slots + (p.gen_only ? p.n_slots - 1 : z);
      float* po = p.part_o + slot * D + sb * 8;
#pragma unroll
      for (int i = 0; i < 8; ++i) po[i] = oo[i];
      if (sb == 0) { p.part_ml[slot * 2] = m; p.part_ml[slot * 2 + 1] = l; }
    }
  }
}

// merge the partial results of the slots: one thread per (stream, head, 8-element group)
template <typename T, int D>
__global__ __launch_bounds__(256) void decode_combine_kernel(const float* __restrict__ part_o,
                                                             const float* __restrict__ part_ml, T* __restrict__ out,
                                                             int rows /* n_streams*hq */, int n_slots) {
  constexpr int LPK = D / 8;
  const int t = blockIdx.x * 256 + threadIdx.x;
  if (t >= rows * LPK) return;
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
// The 4 waves of a workgroup walk disjoint 32-key tiles of the workgroup's key range with private LDS staging and
// private softmax states, which are merged through LDS at the end; key ranges of long caches are split over
// workgroups and every (row, split) partial goes to the workspace.  The per-stream generated rows and the new token
// are handled by decode_kernel in gen_only mode (they differ per beam, so they are not a shared matrix product).
// ------------------------------------------------------------------------------------------------------------------
constexpr int kDsTile = 32;              // keys per wave tile
constexpr int kMaxStreamsPerSeq = 1024;  // beams of one sequence the stream list holds

typedef __attribute__((address_space(3))) s16x4* lds_s16x4_ptr;

template <int D>
struct DsSmem {
  static constexpr int KS = D + 8;
  static constexpr int VS = D + 32;
  struct WaveTile { __bf16 k[kDsTile * KS]; __bf16 v[kDsTile * VS]; };
  WaveTile tile[kDecWaves];   // reused as the merge buffer once the key loop is done
  int streams[kMaxStreamsPerSeq];
  int n_streams_of_seq;
};

template <int D, int QB>
__global__ __launch_bounds__(kDecThreads, 1) void decode_shared_mfma_kernel(DecodeParams p) {
  constexpr int KSTEPS = D / 16, DB = D / 32, UPR = D / 8;
  constexpr int UNITS = kDsTile * UPR / kWave;  // 16-byte units per lane per tile and tensor
  constexpr int ROWS = 32 * QB;
  constexpr int STATE = DB * QB * 16 + 2 * QB;  // floats per lane in a merge
  using Sm = DsSmem<D>;
  static_assert(sizeof(typename Sm::WaveTile) * kDecWaves >= 2 * STATE * kWave * sizeof(float), "merge buffer");
  __shared__ Sm sm;

  const int c = blockIdx.x, s = blockIdx.y, z = blockIdx.z;
  const int gq = p.hq / p.hkv;
  const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
  const int r32 = lane & 31, hf = lane >> 5;
  const int b0 = p.shared_cu[s], ns = p.shared_cu[s + 1] - b0;
  const int j_begin = z * p.chunk;
  const int j_end = min(ns, j_begin + p.chunk);
  const int n_tiles = j_end > j_begin ? (j_end - j_begin + kDsTile - 1) / kDsTile : 0;

  // ---- streams (beams) of this sequence, ascending ----
  if (wave == 0) {
    int count = 0;
    if (!p.stream_to_seq) {
      if (lane == 0) sm.streams[0] = s;
      count = 1;
    } else {
      for (int base = 0; base < p.n_streams; base += kWave) {
        const int u = base + lane;
        const bool hit = u < p.n_streams && p.stream_to_seq[u] == s;
        const unsigned long long mask = __ballot(hit);
        const int idx = count + __popcll(mask & ((1ull << lane) - 1ull));
        if (hit && idx < kMaxStreamsPerSeq) sm.streams[idx] = u;
        count += __popcll(mask);
      }
      if (count > kMaxStreamsPerSeq) count = kMaxStreamsPerSeq;
    }
    if (lane == 0) sm.n_streams_of_seq = count;
  }
  __syncthreads();
  const int M = sm.n_streams_of_seq * gq;  // query rows sharing this cache

  const __bf16* Kg = (const __bf16*)p.shared_k + ((long long)b0 * p.hkv + c) * D;
  const __bf16* Vg = (const __bf16*)p.shared_v + ((long long)b0 * p.hkv + c) * D;
  const long long kv_stride = (long long)p.hkv * D;
  __bf16* my_k = sm.tile[wave].k;
  __bf16* my_v = sm.tile[wave].v;
  const int k_off = r32 * Sm::KS + 8 * hf;
  const int v_off = (4 * hf + ((lane & 15) >> 2)) * Sm::VS + 16 * ((lane >> 4) & 1) + 4 * (lane & 3);
  float* mbuf = (float*)&sm.tile[0];

  for (int row0 = 0; row0 < M; row0 += ROWS) {
    // ---- Q fragments of rows row0 .. row0+ROWS-1: row m -> (stream list[m / gq], head c*gq + m % gq) ----
    bf16x8 qf[QB][KSTEPS];
    int row_u[QB], row_a[QB];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
      const int m = min(row0 + 32 * qb + r32, M - 1);
      const int u = sm.streams[m / gq], a = c * gq + m % gq;
      row_u[qb] = u; row_a[qb] = a;
      const float pos = (float)p.q_pos[u];
      const __bf16* qrow = (const __bf16*)p.q + ((long long)u * p.hq + a) * D + 8 * hf;
#pragma unroll
      for (int ks = 0; ks < KSTEPS / 2; ++ks) {
        float lo[8], hi[8];
        Row8<__bf16>::load(qrow + 16 * ks, lo);
        Row8<__bf16>::load(qrow + 16 * ks + D / 2, hi);
        u32x4 wl, wh;
#pragma unroll
        for (int j = 0; j < 8; j += 2) {
          float x[2], y[2];
#pragma unroll
          for (int jj = 0; jj < 2; ++jj) {
            float sn = 0.f, cs = 1.f;
            const int e = 16 * ks + 8 * hf + j + jj;
            if (p.rope.enabled) sincos_turns_precise(rope_turns(pos, p.rope.hi[e], p.rope.lo[e]), &sn, &cs);
            x[jj] = (lo[j + jj] * cs - hi[j + jj] * sn) * p.scale_log2;
            y[jj] = (hi[j + jj] * cs + lo[j + jj] * sn) * p.scale_log2;
          }
          wl[j / 2] = pack_bf16(x[0], x[1]);
          wh[j / 2] = pack_bf16(y[0], y[1]);
        }
        qf[qb][ks] = __builtin_bit_cast(bf16x8, wl);
        qf[qb][ks + KSTEPS / 2] = __builtin_bit_cast(bf16x8, wh);
      }
    }

    f32x16 o[DB][QB];
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int qb = 0; qb < QB; ++qb)
#pragma unroll
        for (int i = 0; i < 16; ++i) o[db][qb][i] = 0.f;
    float mrow[QB], lrow[QB];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) { mrow[qb] = -INFINITY; lrow[qb] = 0.f; }

    u32x4 kreg[UNITS], vreg[UNITS];
    auto load_tile = [&](int t) {
#pragma unroll
      for (int i = 0; i < UNITS; ++i) {
        const int un = i * kWave + lane;
        const int row = un / UPR, cu8 = un % UPR;
        const int key = min(j_begin + t * kDsTile + row, j_end - 1);  // tail rows repeat the last valid row
        kreg[i] = *(const u32x4*)(Kg + key * kv_stride + cu8 * 8);
        vreg[i] = *(const u32x4*)(Vg + key * kv_stride + cu8 * 8);
      }
    };
    if (wave < n_tiles) load_tile(wave);
    for (int t = wave; t < n_tiles; t += kDecWaves) {
      // wave-private staging: LDS operations of one wave execute in order, the fences only pin the compiler
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
#pragma unroll
      for (int i = 0; i < UNITS; ++i) {
        const int un = i * kWave + lane;
        const int row = un / UPR, cu8 = un % UPR;
        *(u32x4*)(my_k + row * Sm::KS + cu8 * 8) = kreg[i];
        *(u32x4*)(my_v + row * Sm::VS + cu8 * 8) = vreg[i];
      }
      __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
      __builtin_amdgcn_wave_barrier();
      if (t + kDecWaves < n_tiles) load_tile(t + kDecWaves);

      f32x16 sc[QB];
#pragma unroll
      for (int qb = 0; qb < QB; ++qb)
#pragma unroll
        for (int i = 0; i < 16; ++i) sc[qb][i] = 0.f;
#pragma unroll
      for (int ks = 0; ks < KSTEPS; ++ks) {
        const bf16x8 kf = *(const bf16x8*)(my_k + k_off + 16 * ks);
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) sc[qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[qb][ks], sc[qb], 0, 0, 0);
      }
      const int key0 = j_begin + t * kDsTile;
      if (key0 + kDsTile > j_end) {  // ragged last tile: keys past the range get zero weight
#pragma unroll
        for (int qb = 0; qb < QB; ++qb)
#pragma unroll
          for (int i = 0; i < 16; ++i)
            if (key0 + 8 * (i >> 2) + 4 * hf + (i & 3) >= j_end) sc[qb][i] = -INFINITY;
      }
      bf16x8 pf[QB][2];
#pragma unroll
      for (int qb = 0; qb < QB; ++qb) {
        float mloc = sc[qb][0];
#pragma unroll
        for (int i = 1; i < 16; ++i) mloc = fmaxf(mloc, sc[qb][i]);
        mloc = fmaxf(mloc, __shfl_xor(mloc, 32, kWave));
        const float mnew = fmaxf(mrow[qb], mloc);   // finite: every tile holds at least one valid key
        const float alpha = __builtin_amdgcn_exp2f(mrow[qb] - mnew);
        mrow[qb] = mnew;
        float lsum = 0.f;
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const float e = __builtin_amdgcn_exp2f(sc[qb][i] - mnew);
          sc[qb][i] = e;
          lsum += e;
        }
        lrow[qb] = lrow[qb] * alpha + lsum;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
          for (int i = 0; i < 16; ++i) o[db][qb][i] *= alpha;
#pragma unroll
        for (int kk = 0; kk < 2; ++kk) {
          u32x4 w;
#pragma unroll
          for (int j = 0; j < 4; ++j) w[j] = pack_bf16(sc[qb][8 * kk + 2 * j], sc[qb][8 * kk + 2 * j + 1]);
          pf[qb][kk] = __builtin_bit_cast(bf16x8, w);
        }
      }
#pragma unroll
      for (int kk = 0; kk < 2; ++kk) {
#pragma unroll
        for (int db = 0; db < DB; ++db) {
          const __bf16* vp = my_v + v_off + 16 * kk * Sm::VS + 32 * db;
          s16x4 v0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(vp));
          s16x4 v1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(vp + 8 * Sm::VS));
          typedef short s16x8 __attribute__((ext_vector_type(8)));
          s16x8 vv = __builtin_shufflevector(v0, v1, 0, 1, 2, 3, 4, 5, 6, 7);
          const bf16x8 vf = __builtin_bit_cast(bf16x8, vv);
#pragma unroll
          for (int qb = 0; qb < QB; ++qb)
            o[db][qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf[qb][kk], o[db][qb], 0, 0, 0);
        }
      }
      __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
      __builtin_amdgcn_wave_barrier();
    }

    // ---- merge the 4 waves: (2,3) -> (0,1), then 1 -> 0; lane-wise, the layouts are identical ----
    auto put = [&](int slot) {
      float* dst = mbuf + (size_t)slot * STATE * kWave + lane;
      int r = 0;
#pragma unroll
      for (int qb = 0; qb < QB; ++qb) { dst[(r++) * kWave] = mrow[qb]; dst[(r++) * kWave] = lrow[qb]; }
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int qb = 0; qb < QB; ++qb)
#pragma unroll
          for (int i = 0; i < 16; ++i) dst[(r++) * kWave] = o[db][qb][i];
    };
    auto take = [&](int slot) {
      const float* src = mbuf + (size_t)slot * STATE * kWave + lane;
      float a[QB], b[QB];
      int r = 0;
#pragma unroll
      for (int qb = 0; qb < QB; ++qb) {
        const float m2 = src[(r++) * kWave], l2 = src[(r++) * kWave];
        const float mn = fmaxf(mrow[qb], m2);
        a[qb] = mrow[qb] == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(mrow[qb] - mn);
        b[qb] = m2 == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(m2 - mn);
        lrow[qb] = lrow[qb] * a[qb] + l2 * b[qb];
        mrow[qb] = mn;
      }
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int qb = 0; qb < QB; ++qb)
#pragma unroll
          for (int i = 0; i < 16; ++i) o[db][qb][i] = o[db][qb][i] * a[qb] + src[(r++) * kWave] * b[qb];
    };
    __syncthreads();
    if (wave >= 2) put(wave - 2);
    __syncthreads();
    if (wave < 2) take(wave);
    __syncthreads();
    if (wave == 1) put(0);
    __syncthreads();
    if (wave == 0) {
      take(0);
      // ---- partial results of this key range: unnormalised O, running max and sum (base-2 units) ----
#pragma unroll
      for (int qb = 0; qb < QB; ++qb) {
        const float ltot = lrow[qb] + __shfl_xor(lrow[qb], 32, kWave);
        const int m = row0 + 32 * qb + r32;
        if (m >= M) continue;
        const long long slot = ((long long)row_u[qb] * p.hq + row_a[qb]) * p.n_slots + z;
        float* po = p.part_o + slot * D + 4 * hf;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            f32x4 w = {o[db][qb][4 * j], o[db][qb][4 * j + 1], o[db][qb][4 * j + 2], o[db][qb][4 * j + 3]};
            *(f32x4*)(po + 32 * db + 8 * j) = w;
          }
        if (hf == 0) { p.part_ml[slot * 2] = mrow[qb]; p.part_ml[slot * 2 + 1] = ltot; }
      }
    }
    __syncthreads();  // the merge buffer is tile memory again in the next row chunk
  }
}

// ------------------------------------------------------------------------------------------------------------------
// host side
// ------------------------------------------------------------------------------------------------------------------
struct DecodePlan {
  bool mfma;      // shared rows on the matrix cores + generated rows on the vector ALU + combine
  int n_splits;   // key-range splits of the shared (mfma) or whole (vector) key list
  int n_slots;    // partial slots per (stream, head)
  int chunk;      // keys per split
};

static DecodePlan plan_decode(int dtype, int hq, int hkv, int n_streams, int batch, int max_shared_len, int gen_cap) {
  DecodePlan pl;
  const int gq = hq / hkv;
  // several query rows per cache (grouped heads or beams) make the shared part a matrix product
  // (short caches are launch-latency bound: the single-launch vector kernel wins there)
  pl.mfma = dtype == EARN_BF16 && (gq > 1 || n_streams > batch) && max_shared_len >= 128;
  if (pl.mfma) {
    long long base = (long long)hkv * batch;
    int want = (int)((512 + base - 1) / base);               // >= 2 workgroups per CU
    int cap = (max_shared_len + 4 * kDsTile - 1) / (4 * kDsTile);  // at least one tile per wave
    int n = want < cap ? want : cap;
    if (n < 1) n = 1;
    if (n > 64) n = 64;
    pl.n_splits = n;
    pl.n_slots = n + 1;
    pl.chunk = (((max_shared_len + n - 1) / n) + kDsTile - 1) / kDsTile * kDsTile;
  } else {
    const int max_total = max_shared_len + gen_cap;
    // aim at >= 1024 workgroups (4 per CU) while keeping at least 256 keys per split
    long long base = (long long)hkv * n_streams;
    int want = (int)((1024 + base - 1) / base);
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

size_t decode_workspace_bytes(int dtype, int hq, int hkv, int d, int n_streams, int batch, int max_shared_len,
                              int gen_cap) {
  DecodePlan pl = plan_decode(dtype, hq, hkv, n_streams, batch, max_shared_len, gen_cap);
  if (pl.n_slots == 1) return 0;
  size_t rows = (size_t)n_streams * hq * pl.n_slots;
  return rows * d * sizeof(float) + rows * 2 * sizeof(float);
}

template <typename T, int D>
static void launch_vector(const DecodeParams& p, int gq, dim3 grid, hipStream_t stream) {
  dim3 block(kDecThreads);
  if (gq == 1) hipLaunchKernelGGL((decode_kernel<T, D, 1>), grid, block, 0, stream, p);
  else if (gq == 2) hipLaunchKernelGGL((decode_kernel<T, D, 2>), grid, block, 0, stream, p);
  else if (gq <= 4) hipLaunchKernelGGL((decode_kernel<T, D, 4>), grid, block, 0, stream, p);
  else hipLaunchKernelGGL((decode_kernel<T, D, 8>), grid, block, 0, stream, p);
}

template <typename T, int D>
static void launch_combine(const DecodeParams& p, hipStream_t stream) {
  const int rows = p.n_streams * p.hq;
  const int threads = rows * (D / 8);
  hipLaunchKernelGGL((decode_combine_kernel<T, D>), dim3((threads + 255) / 256), dim3(256), 0, stream, p.part_o,
                     p.part_ml, (T*)p.out, rows, p.n_slots);
}

template <typename T, int D>
static void launch_decode_t(DecodeParams& p, const DecodePlan& pl, int gq, hipStream_t stream) {
  if (!pl.mfma) {
    launch_vector<T, D>(p, gq, dim3(p.hkv, p.n_streams, p.n_splits), stream);
    if (p.n_slots > 1) launch_combine<T, D>(p, stream);
    return;
  }
  if constexpr (sizeof(T) == 2) {
    dim3 grid(p.hkv, p.batch, p.n_splits), block(kDecThreads);
    // one 32-row block is enough when a cache serves at most 32 query rows; beams need the host's upper bound
    const bool one_block = (long long)gq * (p.n_streams - p.batch + 1) <= 32;
    if (one_block) hipLaunchKernelGGL((decode_shared_mfma_kernel<D, 1>), grid, block, 0, stream, p);
    else hipLaunchKernelGGL((decode_shared_mfma_kernel<D, 2>), grid, block, 0, stream, p);
    DecodeParams pg = p;
    pg.gen_only = 1;
    pg.chunk = (p.gen_cap + 1 + 63) / 64 * 64;
    launch_vector<T, D>(pg, gq, dim3(p.hkv, p.n_streams, 1), stream);
    launch_combine<T, D>(p, stream);
  }
}

int launch_decode(const earn_attn_desc* desc, const void* q, const void* k_new, const void* v_new,
                  const int32_t* q_pos, const void* shared_k, const void* shared_v, const int32_t* shared_cu,
                  const int32_t* stream_to_seq, void* gen_k, void* gen_v, const int32_t* gen_len, int gen_cap,
                  int n_streams, int batch, int max_shared_len, void* out, void* workspace, size_t workspace_bytes,
                  hipStream_t stream) {
  const int hq = desc->n_q_heads, hkv = desc->n_kv_heads, d = desc->head_dim, gq = hq / hkv;
  if (gq > 8) { set_error("earn_decode_attn: more than 8 query heads per kv head is not supported"); return EARN_ERR_UNSUPPORTED; }
  const DecodePlan pl = plan_decode(desc->dtype, hq, hkv, n_streams, batch, max_shared_len, gen_cap);
  if (pl.mfma && n_streams - batch + 1 > kMaxStreamsPerSeq) {
    set_error("earn_decode_attn: more than %d streams may share one sequence", kMaxStreamsPerSeq);
    return EARN_ERR_UNSUPPORTED;
  }
  DecodeParams p;
  p.q = q; p.k_new = k_new; p.v_new = v_new; p.q_pos = q_pos;
  p.shared_k = shared_k; p.shared_v = shared_v; p.shared_cu = shared_cu; p.stream_to_seq = stream_to_seq;
  p.gen_k = gen_k; p.gen_v = gen_v; p.gen_len = gen_len; p.out = out;
  p.gen_cap = gen_cap; p.n_streams = n_streams; p.batch = batch; p.hq = hq; p.hkv = hkv;
  p.n_splits = pl.n_splits; p.n_slots = pl.n_slots; p.chunk = pl.chunk; p.gen_only = 0;
  const size_t need = decode_workspace_bytes(desc->dtype, hq, hkv, d, n_streams, batch, max_shared_len, gen_cap);
  if (need > workspace_bytes || (need > 0 && !workspace)) {
    set_error("earn_decode_attn: workspace too small (%zu bytes given, %zu needed)", workspace_bytes, need);
    return EARN_ERR_WORKSPACE_TOO_SMALL;
  }
  p.part_o = (float*)workspace;
  p.part_ml = p.part_o + (size_t)n_streams * hq * p.n_slots * d;
  const float scale = desc->softmax_scale > 0.f ? desc->softmax_scale : 1.0f / sqrtf((float)d);
  p.scale_log2 = scale * 1.4426950408889634f;
  p.rope = make_rope_table(desc->rope_base, d);
  if (desc->dtype == EARN_F32) {
    if (d == 64) launch_decode_t<float, 64>(p, pl, gq, stream); else launch_decode_t<float, 128>(p, pl, gq, stream);
  } else {
    if (d == 64) launch_decode_t<__bf16, 64>(p, pl, gq, stream); else launch_decode_t<__bf16, 128>(p, pl, gq, stream);
  }
  return hipGetLastError() == hipSuccess ? EARN_OK : EARN_ERR_HIP;
}

}  // namespace earn
