// Causal prefill attention over a packed ragged batch (paper Section 2.2, Eq. 3; used at full length for the first
// k layers and on the compacted register rows, with their original positions, for the remaining N-k layers —
// Section 3.2, Inference).
//
// Kernels:
//   rope_k_kernel        rotates K once per layer into the buffer the KV cache keeps (k_rot_out); every query block
//                        then reads rotated keys, so the sin/cos work is O(T), not O(T * blocks).
//   prefill_pipe_kernel  bf16 flash-style attention on the matrix cores (v_mfma_f32_32x32x16_bf16), software pipelined:
//                        long sequences.
//   prefill_mfma_kernel  the same arithmetic in a plain per-tile schedule with smaller workgroups: medium sequences and
//                        the register-only layers.
//   prefill_rows_kernel  fp32 attention on the vector ALU: one query row per 4 lanes. Used for the fp32
//                        configuration, where the 1e-4 tolerance rules out bf16 operands.
//
// MFMA kernel layout (all shapes in the 32x32x16 tile of the instruction, 64 lanes, lane = (r32 = lane%32, hf = lane/32)):
//   The kernels compute the TRANSPOSED score tile S^T = K Q^T (keys x queries).  Its accumulator layout gives every lane
//   ONE query column (r32) and 16 of the 32 keys of a block, so the softmax row statistics are a private loop plus one
//   exchange with lane^32, and the rescaling of the output accumulator is lane-private as well.
//   The accumulator registers of S^T, converted to bf16, are exactly the B operand (keys x queries, 8 keys per lane)
//   of the second product O^T = V^T P^T, so P never leaves registers.  The 8 key slots of a lane are keys
//   {4hf..4hf+3, 8+4hf..8+4hf+3} of a 16-key step; the A operand V^T uses the same key order, which is what two
//   transposing LDS reads (ds_read_b64_tr_b16: 4 consecutive keys of one d column) deliver from a V tile kept in its
//   natural [key][d] layout.
//   Each wave owns 32 query rows; the 64-key K/V tile in LDS is shared by the waves of a workgroup.
#include "common.h"
#include "mfma_tiles.h"

namespace earn {

struct PrefillParams {
  const void* q; const void* k_rot; const void* v; const int32_t* cu; const int32_t* positions;
  const f32x2* cs;  // [tokens][d/2] (cos, sin) of every token's rotary angles, written by rope_k_kernel (bf16 paths)
  void* out; float* lse;
  int batch, hq, hkv, max_seqlen;
  int total;   // rows of the packed tensors
  int n_qblk;  // query blocks of the longest sequence
  // chosen-rows mode of the vector kernel (rows_per_seq > 0): q and out hold rows_per_seq rows per sequence in
  // compacted order, row m of sequence s being token row_pos[s * rows_per_seq + m] (ascending) of the sequence
  const int32_t* row_pos;
  int rows_per_seq;
  float scale_log2;
  // byte strides between the layers of a layer-batched launch (one grid dimension indexes the layer); zero otherwise.
  // The sequence bounds, the positions and the cos/sin table are shared by the layers.
  long long ls_q, ls_k_rot, ls_v, ls_out, ls_lse;
  RopeTable rope;
  HeadMap heads;
};

// Bounds of sequence s as the kernels use them: whatever cu_seqlens holds, rows [b0, b0 + n) lie inside the packed
// tensors and n within the length the launch was sized (and its 32-bit offsets checked) for.  A corrupt or not yet
// written cu_seqlens then gives wrong values, never an access outside the tensors.
__device__ __forceinline__ void pf_seq_bounds(const PrefillParams& p, int s, int& b0, int& n) {
  b0 = min(max(p.cu[s], 0), p.total);
  n = min(min(max(p.cu[s + 1] - b0, 0), p.total - b0), p.max_seqlen);
}

template <typename P>
__device__ __forceinline__ P* pf_layer_ptr(P* base, long long stride, int layer) {
  return (P*)((const char*)base + stride * layer);
}
// The per-layer pointers of one layer, as a view beside the parameter block (a modified copy of the block would live
// in scratch memory: it holds arrays indexed at run time).
struct PfLayer { const void* q; const void* k_rot; const void* v; void* out; float* lse; };
__device__ __forceinline__ PfLayer pf_layer_view(const PrefillParams& p, int layer) {
  PfLayer v;
  v.q = pf_layer_ptr(p.q, p.ls_q, layer);
  v.k_rot = pf_layer_ptr(p.k_rot, p.ls_k_rot, layer);
  v.v = pf_layer_ptr(p.v, p.ls_v, layer);
  v.out = pf_layer_ptr(p.out, p.ls_out, layer);
  v.lse = p.lse ? pf_layer_ptr(p.lse, p.ls_lse, layer) : nullptr;
  return v;
}

// ------------------------------------------------------------------------------------------------------------------
// K rotation
// ------------------------------------------------------------------------------------------------------------------
template <typename T> struct Vec8;
template <> struct Vec8<float> {
  static __device__ __forceinline__ void load(const float* p, float* x) {
    f32x4 a = *(const f32x4*)p, b = *(const f32x4*)(p + 4);
    x[0] = a[0]; x[1] = a[1]; x[2] = a[2]; x[3] = a[3]; x[4] = b[0]; x[5] = b[1]; x[6] = b[2]; x[7] = b[3];
  }
  static __device__ __forceinline__ void store(float* p, const float* x) {
    f32x4 a = {x[0], x[1], x[2], x[3]}, b = {x[4], x[5], x[6], x[7]};
    *(f32x4*)p = a; *(f32x4*)(p + 4) = b;
  }
};
template <> struct Vec8<__bf16> {
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

// One thread per (token, group of 8 rotary pairs): the sin/cos of the group are computed once and applied to every kv
// head of the token.  bf16 rows use the hardware sin/cos (error ~1e-6, far below bf16 resolution).
// cs_out (optional): the (cos, sin) pairs themselves, [token][d/2].  The attention kernels rotate their query rows with
// them: a workgroup per query head would otherwise recompute the same angles once per head, and on short sequences
// that prologue costs as much as the attention itself.
template <typename T, int D>
__global__ __launch_bounds__(256) void rope_k_kernel(const T* __restrict__ k, T* __restrict__ k_rot,
                                                     const int32_t* __restrict__ cu,
                                                     const int32_t* __restrict__ positions, int batch, int total,
                                                     int hkv, RopeTable rope, f32x2* __restrict__ cs_out,
                                                     int heads_per_thread, long long ls_k, long long ls_k_rot) {
  constexpr int G = D / 16;  // groups of 8 pairs per head
  const long long t = (long long)blockIdx.x * 256 + threadIdx.x;
  if (t >= (long long)total * G) return;
  k = pf_layer_ptr(k, ls_k, blockIdx.z);           // grid layer z = layer of a layer-batched launch
  k_rot = pf_layer_ptr(k_rot, ls_k_rot, blockIdx.z);
  const int g = (int)(t % G);
  const int token = (int)(t / G);
  float sn[8], cs[8];
  if (rope.enabled) {
    int pos;
    if (positions) pos = positions[token];
    else pos = token - cu[find_seq(cu, batch, token)];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const float turns = rope_turns((float)pos, rope.hi[g * 8 + i], rope.lo[g * 8 + i]);
      if (sizeof(T) == 2) sincos_turns_fast(turns, &sn[i], &cs[i]);
      else sincos_turns_precise(turns, &sn[i], &cs[i]);
    }
  } else {
#pragma unroll
    for (int i = 0; i < 8; ++i) { sn[i] = 0.f; cs[i] = 1.f; }
  }
  if (cs_out && blockIdx.y == 0 && blockIdx.z == 0) {
    f32x4* dst4 = (f32x4*)(cs_out + (long long)token * (D / 2) + g * 8);
#pragma unroll
    for (int i = 0; i < 8; i += 2) dst4[i / 2] = f32x4{cs[i], sn[i], cs[i + 1], sn[i + 1]};
  }
  const T* src = k + (long long)token * hkv * D + g * 8;
  T* dst = k_rot + (long long)token * hkv * D + g * 8;
  // grid row y takes kv heads [y * heads_per_thread, + heads_per_thread): all of them when there are tokens enough to
  // fill the GPU, a few when there are not (the loop over heads is a chain of memory round trips)
  const int h_begin = blockIdx.y * heads_per_thread, h_end = min(hkv, h_begin + heads_per_thread);
  for (int h = h_begin; h < h_end; ++h) {
    float lo[8], hi[8];
    Vec8<T>::load(src + h * D, lo);
    Vec8<T>::load(src + h * D + D / 2, hi);
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const float a = lo[i], b = hi[i];
      lo[i] = a * cs[i] - b * sn[i];
      hi[i] = b * cs[i] + a * sn[i];
    }
    Vec8<T>::store(dst + h * D, lo);
    Vec8<T>::store(dst + h * D + D / 2, hi);
  }
}

// ------------------------------------------------------------------------------------------------------------------
// vector-ALU attention: 64 query rows per workgroup, 4 lanes per row (each holds D/4 elements of q and of the output)
// ------------------------------------------------------------------------------------------------------------------
template <typename T, int D>
__global__ __launch_bounds__(256) void prefill_rows_kernel(PrefillParams p) {
  constexpr int E = D / 8;  // elements per contiguous piece; a lane holds pieces [qt*E, +E) and [D/2 + qt*E, +E)
  const int slot = blockIdx.y, s = blockIdx.z % p.batch;  // slot: the query heads in kv-head order
  const PfLayer lv = pf_layer_view(p, blockIdx.z / p.batch);
  const int a = head_of_slot(p.heads, slot);
  int b0, n;
  pf_seq_bounds(p, s, b0, n);
  const int row0 = blockIdx.x * 64;
  const int r = p.rows_per_seq;           // 0: every row of the sequence
  const int n_rows = r > 0 ? r : n;
  if (row0 >= n_rows || n <= 0) return;
  const int qt = threadIdx.x & 3;
  const int mrow = row0 + (threadIdx.x >> 2);                  // row of the sequence's row list
  const bool row_ok = mrow < n_rows;
  const int mc = row_ok ? mrow : n_rows - 1;
  // its token index: it sees keys 0 .. ic (a row_pos outside the sequence is held inside it: wrong values, no stray access)
  const int ic = r > 0 ? min(max(p.row_pos[s * r + mc], 0), n - 1) : mc;
  const long long io = r > 0 ? (long long)s * r + mc : (long long)b0 + mc;  // its row in q / out / lse
  const int c = slot / (p.hq / p.hkv);
  const T* qrow = (const T*)lv.q + (io * p.hq + a) * D;
  float ql[E], qh[E];
#pragma unroll
  for (int e = 0; e < E; e += 8) { Vec8<T>::load(qrow + qt * E + e, ql + e); Vec8<T>::load(qrow + D / 2 + qt * E + e, qh + e); }
  const int pos = (p.positions && r == 0) ? p.positions[b0 + ic] : ic;
#pragma unroll
  for (int e = 0; e < E; ++e) {
    float sn = 0.f, cs = 1.f;
    if (p.rope.enabled) sincos_turns_precise(rope_turns((float)pos, p.rope.hi[qt * E + e], p.rope.lo[qt * E + e]), &sn, &cs);
    float x = ql[e], y = qh[e];
    ql[e] = (x * cs - y * sn) * p.scale_log2;
    qh[e] = (y * cs + x * sn) * p.scale_log2;
  }
  float ol[E], oh[E], m = -INFINITY, l = 0.f;
#pragma unroll
  for (int e = 0; e < E; ++e) { ol[e] = 0.f; oh[e] = 0.f; }
  // all rows of a wave walk the keys together up to the wave's last row
  const int wave_last_row = min(n_rows - 1, row0 + (int)(threadIdx.x / kWave) * 16 + 15);
  const int wave_last = r > 0 ? min(max(p.row_pos[s * r + wave_last_row], 0), n - 1) : wave_last_row;
  const T* kbase = (const T*)lv.k_rot + ((long long)b0 * p.hkv + c) * D;
  const T* vbase = (const T*)lv.v + ((long long)b0 * p.hkv + c) * D;
  const long long rs = (long long)p.hkv * D;
  // NB keys per step: their rows are requested together and their scores formed side by side (the walk is otherwise a
  // chain of memory round trips); the softmax state still takes them one after the other, in key order
  constexpr int NB = D == 64 ? 4 : 2;
  for (int j0 = 0; j0 <= wave_last; j0 += NB) {
    float kl[NB][E], kh[NB][E], vl[NB][E], vh[NB][E], sc[NB];
#pragma unroll
    for (int b = 0; b < NB; ++b) {
      const int j = min(j0 + b, wave_last);
#pragma unroll
      for (int e = 0; e < E; e += 8) {
        Vec8<T>::load(kbase + j * rs + qt * E + e, kl[b] + e);
        Vec8<T>::load(kbase + j * rs + D / 2 + qt * E + e, kh[b] + e);
        Vec8<T>::load(vbase + j * rs + qt * E + e, vl[b] + e);
        Vec8<T>::load(vbase + j * rs + D / 2 + qt * E + e, vh[b] + e);
      }
    }
#pragma unroll
    for (int b = 0; b < NB; ++b) {
      float d = 0.f;
#pragma unroll
      for (int e = 0; e < E; ++e) d = __builtin_fmaf(ql[e], kl[b][e], __builtin_fmaf(qh[e], kh[b][e], d));
      d += __shfl_xor(d, 1, kWave);
      d += __shfl_xor(d, 2, kWave);
      sc[b] = d;
    }
#pragma unroll
    for (int b = 0; b < NB; ++b) {
      if (j0 + b <= ic && j0 + b <= wave_last) {  // causal: keys 0..i
        float mn = fmaxf(m, sc[b]);
        float corr = __builtin_amdgcn_exp2f(m - mn);  // exp2(-inf) = 0 on the first key
        float pr = __builtin_amdgcn_exp2f(sc[b] - mn);
        l = l * corr + pr;
#pragma unroll
        for (int e = 0; e < E; ++e) { ol[e] = __builtin_fmaf(pr, vl[b][e], ol[e] * corr); oh[e] = __builtin_fmaf(pr, vh[b][e], oh[e] * corr); }
        m = mn;
      }
    }
  }
  if (!row_ok) return;
  const float inv = 1.f / l;
#pragma unroll
  for (int e = 0; e < E; ++e) { ol[e] *= inv; oh[e] *= inv; }
  T* orow = (T*)lv.out + (io * p.hq + a) * D;
#pragma unroll
  for (int e = 0; e < E; e += 8) { Vec8<T>::store(orow + qt * E + e, ol + e); Vec8<T>::store(orow + D / 2 + qt * E + e, oh + e); }
  if (lv.lse && qt == 0) lv.lse[io * p.hq + a] = (m + __builtin_log2f(l)) * 0.6931471805599453f;
}

// ------------------------------------------------------------------------------------------------------------------
// bf16 MFMA flash attention
// ------------------------------------------------------------------------------------------------------------------

// ---- workgroup -> (sequence, kv head, query block, head of the group), XCD aware ----
// Workgroups are handed to the 8 XCDs round-robin by linear id, and every XCD has its own L2.  Id (x, k) = the k-th
// workgroup of XCD x.  Each XCD walks its own list of (sequence, kv head) pairs (pair % 8 == x) one pair at a time:
// all query blocks of the pair (long, late blocks first) and all query heads of the group, so the workgroups that
// are resident on an XCD at any moment stream the SAME K/V rows and find them in that XCD's L2.
struct PfBlock {
  int c, a;     // kv head, query head
  int b0, n;    // first packed row and length of the sequence
  int q0;       // first query row of the workgroup inside the sequence
  bool valid;
};
__device__ __forceinline__ PfBlock pf_map_block(const PrefillParams& p, int block_rows) {
  PfBlock b;
  b.valid = false;
  const int gq = p.hq / p.hkv;
  const int xcd = blockIdx.x % kXcds, k_in_xcd = blockIdx.x / kXcds;
  const int per_pair = p.n_qblk * gq;
  const int pair = (k_in_xcd / per_pair) * kXcds + xcd;
  if (pair >= p.batch * p.hkv) return b;
  const int rem = k_in_xcd % per_pair;
  const int qblk = p.n_qblk - 1 - rem / gq;
  const int s = pair / p.hkv;
  b.c = pair % p.hkv;
  b.a = head_of_slot(p.heads, b.c * gq + rem % gq);
  pf_seq_bounds(p, s, b.b0, b.n);
  b.q0 = qblk * block_rows;
  b.valid = b.q0 < b.n;
  return b;
}

// ---- Q fragments: rotate at the original position (tabulated cos/sin), fold in scale*log2(e), keep as bf16 B operands ----
// lane (r32, hf) holds, for k-step ks, dims 16 ks + 8 hf + (0..7) of query r32
template <int D>
__device__ __forceinline__ void pf_load_q(const PrefillParams& p, const __bf16* qrow /* row + 8 hf */,
                                          const f32x2* csrow /* token's table row + 8 hf */, bf16x8 (&qf)[D / 16]) {
  constexpr int KSTEPS = D / 16;
#pragma unroll
  for (int ks = 0; ks < KSTEPS / 2; ++ks) {
    float lo[8], hi[8];
    Vec8<__bf16>::load(qrow + 16 * ks, lo);
    Vec8<__bf16>::load(qrow + 16 * ks + D / 2, hi);
    const f32x4* cs4 = (const f32x4*)(csrow + 16 * ks);  // pairs 16 ks + 8 hf + (0..7)
    u32x4 wl, wh;
#pragma unroll
    for (int j = 0; j < 8; j += 2) {
      const f32x4 c = p.cs ? cs4[j / 2] : f32x4{1.f, 0.f, 1.f, 0.f};  // (cos, sin) of pairs j, j + 1; no table: no rotation
      const float x0 = (lo[j] * c[0] - hi[j] * c[1]) * p.scale_log2, y0 = (hi[j] * c[0] + lo[j] * c[1]) * p.scale_log2;
      const float x1 = (lo[j + 1] * c[2] - hi[j + 1] * c[3]) * p.scale_log2, y1 = (hi[j + 1] * c[2] + lo[j + 1] * c[3]) * p.scale_log2;
      wl[j / 2] = pack_bf16(x0, x1);
      wh[j / 2] = pack_bf16(y0, y1);
    }
    qf[ks] = __builtin_bit_cast(bf16x8, wl);
    qf[ks + KSTEPS / 2] = __builtin_bit_cast(bf16x8, wh);
  }
}

// S^T (+)= K Q^T for the K tile at smk: two 32-key blocks, K fragments requested AHEAD k-steps before the MFMAs that use
// them.  ZERO: start from 0, else from `init` in every register (the steady state starts at -m, which takes the
// subtraction of the reference maximum off the vector ALU).
template <int D, bool ZERO>
__device__ __forceinline__ void score_tile(const __bf16* smk, const FragOffsets<D>& fo, const bf16x8 (&qf)[D / 16],
                                           const f32x16& init, f32x16 (&sc)[2]) {
  constexpr int KSTEPS = D / 16;
  constexpr int AHEAD = ZERO ? 1 : (2 < KSTEPS ? 2 : KSTEPS);  // the exact paths are short of registers, not of time
  const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  bf16x8 kf[2][KSTEPS];
#pragma unroll
  for (int ks = 0; ks < AHEAD; ++ks)
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) kf[kb][ks] = *(const bf16x8*)(smk + fo.k(ks) + kb * 32 * D);
#pragma unroll
  for (int ks = 0; ks < KSTEPS; ++ks) {
    if (ks + AHEAD < KSTEPS) {
#pragma unroll
      for (int kb = 0; kb < 2; ++kb) kf[kb][ks + AHEAD] = *(const bf16x8*)(smk + fo.k(ks + AHEAD) + kb * 32 * D);
    }
    __builtin_amdgcn_sched_barrier(0);  // the fragment requests stay ahead of the MFMAs that hide their latency
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
      sc[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[kb][ks], qf[ks], ks == 0 ? (ZERO ? zero : init) : sc[kb], 0, 0, 0);
    __builtin_amdgcn_sched_barrier(0);
  }
}
// causal mask of the wave's diagonal tile, in place: lane (r32, hf) holds keys 32 kb + 8 (i/4) + 4 hf + i%4 of query
// q_in_tile + r32 (keys beyond the sequence end are beyond every valid query too)
__device__ __forceinline__ void mask_diagonal(f32x16 (&sc)[2], int q_in_tile, int r32, int hf) {
  const int bound = q_in_tile + r32 - 4 * hf;
#pragma unroll
  for (int kb = 0; kb < 2; ++kb)
#pragma unroll
    for (int i = 0; i < 16; ++i)
      if (32 * kb + 8 * (i >> 2) + (i & 3) > bound) sc[kb][i] = -INFINITY;
}
// Softmax unit u (0..15) of a score tile: two exponentials (the scores already carry -m), the bf16 word that holds
// them, and the word's contribution to the lane's row sum.  Word (kk, j) of the B operand P^T packs accumulator
// registers 8 (kk & 1) + 2 j, + 1 of key block kk >> 1; u = 4 kk + j.
__device__ __forceinline__ void softmax_unit(const f32x16 (&sc)[2], int u, u32x4 (&w)[4], float& s0, float& s1) {
  const int kk = u >> 2, j = u & 3, r = 8 * (kk & 1) + 2 * j;
  w[kk][j] = pack_bf16(__builtin_amdgcn_exp2f(sc[kk >> 1][r]), __builtin_amdgcn_exp2f(sc[kk >> 1][r + 1]));
  add_pair(j & 1 ? s1 : s0, w[kk][j]);
}
// normalise and store one query row's share: lane holds d = 32 db + 8 j + 4 hf + (0..3)
template <int D>
__device__ __forceinline__ void pf_store_row(__bf16* orow /* row + 4 hf */, const f32x16 (&o)[D / 32], float inv) {
#pragma unroll
  for (int db = 0; db < D / 32; ++db)
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      u32x2 w;
      w[0] = pack_bf16(o[db][4 * j] * inv, o[db][4 * j + 1] * inv);
      w[1] = pack_bf16(o[db][4 * j + 2] * inv, o[db][4 * j + 3] * inv);
      *(u32x2*)(orow + 32 * db + 8 * j) = w;
    }
}

// ------------------------------------------------------------------------------------------------------------------
// Plain schedule: per tile  barrier -> S^T -> exponentials -> O^T.  One 32-query column block per wave.
//   WAVES = 4: 128 query rows per workgroup, two workgroups per CU: less idle time on the causal diagonal of medium
//              sequences than 256-row workgroups, at the price of staging every K/V tile twice as often.
//   WAVES = 2, STAGES = 1: the register-only-layer variant: every sequence fits one K/V tile, so there is nothing to
//              double buffer, and the small footprint lets 4 workgroups share a CU, which is what hides the
//              load -> rotate -> multiply latency chain of these tiny problems.
// ------------------------------------------------------------------------------------------------------------------
//
// Life-cycle timers, compiled in only with -DEARN_PF_TIMELINE (paper_2507_00715_amd/timeline.py builds that variant
// into a library of its own and prints where a workgroup's life goes).  Thread 0 of every workgroup stamps the 100 MHz
// wall clock into 8 words of a caller-provided buffer: 0 entry, 1 block known, 2 queries, cos/sin rows and first K/V
// tile arrived (this stamp waits for them, which the normal build does only at the first barrier), 3 first tile done,
// 4 all tiles done, 5 output stores issued; 6 the CU, 7 the block's tile count (0: block beyond its sequence).  In the
// normal build the macros are empty.
#ifdef EARN_PF_TIMELINE
__device__ long long* g_pf_timeline;
__device__ int g_pf_timeline_slots;
#define PF_TIMELINE(code) code
#define PF_STAMP(i)                                                                                    \
  do {                                                                                                 \
    const long long pf_wg = (long long)blockIdx.y * gridDim.x + blockIdx.x;                            \
    if (threadIdx.x == 0 && g_pf_timeline && pf_wg < g_pf_timeline_slots) g_pf_timeline[pf_wg * 8 + (i)] = wall_clock64(); \
  } while (0)
#else
#define PF_TIMELINE(code)
#define PF_STAMP(i)
#endif
template <int D, int WAVES, int STAGES>
__global__ __launch_bounds__(64 * WAVES, WAVES == 8 ? 1 : 2) void prefill_mfma_kernel(PrefillParams p) {
  constexpr int kBlockRows = 32 * WAVES;
  constexpr int DB = D / 32;             // 32-row blocks of O^T
  __shared__ __bf16 smk[STAGES][kTileKeys * D];  // tile t+1 arrives while tile t is read
  __shared__ __bf16 smv[STAGES][kTileKeys * D];
  PF_STAMP(0);

  const PfBlock blk = pf_map_block(p, kBlockRows);
  PF_TIMELINE({
    const long long pf_wg = (long long)blockIdx.y * gridDim.x + blockIdx.x;
    if (threadIdx.x == 0 && g_pf_timeline && pf_wg < g_pf_timeline_slots) {
      g_pf_timeline[pf_wg * 8 + 6] = __smid();
      g_pf_timeline[pf_wg * 8 + 7] = blk.valid ? (min(blk.q0 + kBlockRows, blk.n) + kTileKeys - 1) / kTileKeys : 0;
    }
  })
  if (!blk.valid) return;
  PF_STAMP(1);
  const PfLayer lv = pf_layer_view(p, blockIdx.y);
  const int b0 = blk.b0, n = blk.n;
  // the wave index is the same in all 64 lanes: say so, and everything derived from it (the wave's query window, its
  // diagonal tile, the tile loop) lives in scalar registers and branches without touching the execution mask
  const int lane = threadIdx.x % kWave, wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
  const int r32 = lane & 31, hf = lane >> 5;
  const int qw = blk.q0 + wave * 32;             // first query row of this wave
  const bool wave_active = qw < n;
  const int t_diag = qw / kTileKeys;             // last (diagonal) tile of this wave
  const int q_in_tile = qw - t_diag * kTileKeys; // offset of the wave's first query inside that tile
  const int n_tiles = (min(blk.q0 + kBlockRows, n) + kTileKeys - 1) / kTileKeys;

  TileStager<D, WAVES> stager;
  stager.init((const __bf16*)lv.k_rot + ((long long)b0 * p.hkv + blk.c) * D, (const __bf16*)lv.v + ((long long)b0 * p.hkv + blk.c) * D,
              n, p.hkv, wave, lane);
  const unsigned lds_k = (unsigned)(size_t)(lds_void_ptr)&smk[0][0], lds_v = (unsigned)(size_t)(lds_void_ptr)&smv[0][0];
  auto issue_tile = [&](int t) {
    const unsigned at = (unsigned)((t % STAGES) * kTileKeys * D * 2);
    stager.issue(stager.k_rsrc, lds_k + at, t);
    stager.issue(stager.v_rsrc, lds_v + at, t);
  };
  // Barrier t: every wave has waited for its own part of tile t, so behind the barrier tile t is complete and visible;
  // the wave then starts its part of tile t+1 into the other buffer, which every wave has finished reading (tile t-1).
  auto sync_and_stage = [&](int t) {
    drain_loads_and_barrier();
    if constexpr (STAGES > 1) {
      if (t + 1 < n_tiles) issue_tile(t + 1);
    }
  };
  issue_tile(0);  // in flight while the queries are loaded and rotated

  bf16x8 qf[D / 16];
  {
    const int qi = min(qw + r32, n - 1);
    pf_load_q<D>(p, (const __bf16*)lv.q + ((long long)(b0 + qi) * p.hq + blk.a) * D + 8 * hf,
                 p.cs + (long long)(b0 + qi) * (D / 2) + 8 * hf, qf);
  }
  FragOffsets<D> fo;
  fo.init(lane);
  PF_TIMELINE(__builtin_amdgcn_s_waitcnt(0x0F70);)  // vmcnt(0)
  PF_STAMP(2);

  f32x16 o[DB], neg_m;  // neg_m: -m in every register, the start value of the steady-state score accumulators
#pragma unroll
  for (int db = 0; db < DB; ++db)
#pragma unroll
    for (int i = 0; i < 16; ++i) o[db][i] = 0.f;
#pragma unroll
  for (int i = 0; i < 16; ++i) neg_m[i] = 0.f;
  float mrow = -INFINITY, lrow = 0.f;

  // exponentials of a whole score tile (already shifted by -m), packed, with the lane's row sum
  auto softmax_tile = [&](const f32x16 (&sc)[2], u32x4 (&w)[4], float& lsum) {
    float s0 = 0.f, s1 = 0.f;
#pragma unroll
    for (int u = 0; u < 16; ++u) softmax_unit(sc, u, w, s0, s1);
    lsum = add_chains(s0, s1);
  };
  // O^T += V^T P^T; the V^T fragments are requested up front so that their latency hides behind whatever the caller
  // does between fetch and use
  auto fetch_v = [&](const __bf16* smv_t, bf16x8 (&vf)[4][DB]) {
#pragma unroll
    for (int kk = 0; kk < 4; ++kk)
#pragma unroll
      for (int db = 0; db < DB; ++db) vf[kk][db] = read_v_fragment<D>(smv_t, fo, db, kk);
    __builtin_amdgcn_sched_barrier(0);
  };
  auto accumulate = [&](const u32x4 (&w)[4], float lsum, const bf16x8 (&vf)[4][DB]) {
    lrow += lsum;
#pragma unroll
    for (int kk = 0; kk < 4; ++kk)
#pragma unroll
      for (int db = 0; db < DB; ++db)
        o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[kk][db], __builtin_bit_cast(bf16x8, w[kk]), o[db], 0, 0, 0);
  };
  // The exact path: raw scores, exact row maxima, rescale of everything accumulated so far.
  // synced = the tile fell out of the steady-state loop, which has passed the tile's barrier already.
  auto exact_tile = [&](int t, bool synced) {
    if (!synced) sync_and_stage(t);
    f32x16 sc[2];
    bf16x8 vf[4][DB];
    u32x4 w[4];
    float lsum;
    score_tile<D, true>(smk[t % STAGES], fo, qf, neg_m, sc);
    if (t == t_diag) mask_diagonal(sc, q_in_tile, r32, hf);
    float m = sc[0][0];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int i = 0; i < 16; ++i) m = fmaxf(m, sc[kb][i]);
    const float mnew = fmaxf(mrow, half_max(m));  // finite: tile 0 holds key 0, visible to every query
    const float alpha = __builtin_amdgcn_exp2f(mrow - mnew);
    mrow = mnew;
    lrow *= alpha;
#pragma unroll
    for (int i = 0; i < 16; ++i) neg_m[i] = -mnew;
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int i = 0; i < 16; ++i) o[db][i] *= alpha;
    fetch_v(smv[t % STAGES], vf);
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int i = 0; i < 16; ++i) sc[kb][i] -= mnew;
    softmax_tile(sc, w, lsum);
    accumulate(w, lsum, vf);
  };

  // Every wave passes exactly one barrier per tile, whichever path it takes.  The steady-state loop takes the
  // exponentials against the reference maxima it already has and never touches the output accumulators with the
  // vector ALU.  It does not even compute row maxima: a reference is stale exactly when some exponential is large, so
  // the (already needed) partial row sums are compared with kSumLimit instead.  A wave that fails leaves the loop,
  // recomputes the tile's scores, takes the exact maxima, rescales, finishes the tile and re-enters.  Tile 0 (reference
  // still -inf) always takes the exact path; the wave's diagonal tile is the only one that needs the causal mask.
  int t = 0;
  while (t < n_tiles) {
    bool exact = wave_active && t == 0, synced = false;
    if (!exact)
    for (; t < n_tiles; ++t) {
      const bool work = wave_active && t <= t_diag;  // else rows past the sequence end or a tile past the diagonal: only stage
      sync_and_stage(t);
      if (work) {
        f32x16 sc[2];
        bf16x8 vf[4][DB];
        u32x4 w[4];
        float lsum;
        score_tile<D, false>(smk[t % STAGES], fo, qf, neg_m, sc);
        if (t == t_diag) mask_diagonal(sc, q_in_tile, r32, hf);  // masked scores give weight 0 on this path as well
        fetch_v(smv[t % STAGES], vf);
        softmax_tile(sc, w, lsum);
        if (__any(!(lsum <= kSumLimit))) { exact = synced = true; break; }
        accumulate(w, lsum, vf);
      }
    }
    if (!exact) break;
    exact_tile(t, synced);
    ++t;
    PF_TIMELINE(if (t == 1) PF_STAMP(3);)
  }
  PF_STAMP(4);

  if (!wave_active) return;
  const int qi = qw + r32;
  const float ltot = half_sum(lrow);
  if (qi >= n) return;
  pf_store_row<D>((__bf16*)lv.out + ((long long)(b0 + qi) * p.hq + blk.a) * D + 4 * hf, o, 1.f / ltot);
  if (lv.lse && hf == 0) lv.lse[(long long)(b0 + qi) * p.hq + blk.a] = (mrow + __builtin_log2f(ltot)) * 0.6931471805599453f;
  PF_STAMP(5);
}

// ------------------------------------------------------------------------------------------------------------------
// Software-pipelined schedule for long sequences (instantiated with 8 waves: 256 query rows per workgroup, one
// workgroup per CU, two waves per SIMD).
//
// A single wave cannot hide its exponentials behind its own matrix products when the two alternate, and two waves of a
// SIMD that meet at a barrier every tile fall into step, so they do not hide them for each other either.  Here every
// wave overlaps them itself: while the matrix core accumulates the scores of tile t+1, the vector ALU takes the
// exponentials of tile t, instruction by instruction in one stream; then O^T += V^T P^T of tile t follows at once.  The
// matrix core always has the next product queued.
//
//   iteration t:  barrier t (K(t+1) and V(t) have landed; start K(t+2), V(t+1))
//                 S(t+1) = K(t+1) Q^T - m   interleaved with   P(t) = exp2(S(t)), row sums
//                 [sums too large -> reference stale: recompute S(t) exactly from K(t), which is still in LDS]
//                 O += V(t) P(t)
//
// K tiles live in a ring of 3 (t: kept for the exact path, t+1: being multiplied, t+2: in flight), V tiles in a ring
// of 2 (t: being multiplied, t+1: in flight).  The two score tiles swap roles every iteration; the loop is unrolled by
// two so that the swap costs no register moves.
// ------------------------------------------------------------------------------------------------------------------
template <int D, int WAVES>
__global__ __launch_bounds__(64 * WAVES, WAVES == 8 ? 1 : 2) void prefill_pipe_kernel(PrefillParams p) {
  constexpr int kBlockRows = 32 * WAVES;
  constexpr int KSTEPS = D / 16, DB = D / 32;
  constexpr int UPM = 16 / (2 * KSTEPS);  // softmax units per score MFMA: 1 (D = 128) or 2 (D = 64)
  __shared__ __bf16 smk[3][kTileKeys * D];
  __shared__ __bf16 smv[2][kTileKeys * D];

  const PfBlock blk = pf_map_block(p, kBlockRows);
  if (!blk.valid) return;
  const PfLayer lv = pf_layer_view(p, blockIdx.y);
  const int b0 = blk.b0, n = blk.n;
  const int lane = threadIdx.x % kWave, wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
  const int r32 = lane & 31, hf = lane >> 5;
  const int qw = blk.q0 + wave * 32;
  const bool wave_active = qw < n;
  const int t_diag = qw / kTileKeys;
  const int q_in_tile = qw - t_diag * kTileKeys;
  const int n_tiles = (min(blk.q0 + kBlockRows, n) + kTileKeys - 1) / kTileKeys;

  TileStager<D, WAVES> stager;
  stager.init((const __bf16*)lv.k_rot + ((long long)b0 * p.hkv + blk.c) * D, (const __bf16*)lv.v + ((long long)b0 * p.hkv + blk.c) * D,
              n, p.hkv, wave, lane);
  const unsigned lds_k = (unsigned)(size_t)(lds_void_ptr)&smk[0][0], lds_v = (unsigned)(size_t)(lds_void_ptr)&smv[0][0];
  auto issue_k = [&](int t) { stager.issue(stager.k_rsrc, lds_k + (unsigned)((t % 3) * kTileKeys * D * 2), t); };
  auto issue_v = [&](int t) { stager.issue(stager.v_rsrc, lds_v + (unsigned)((t & 1) * kTileKeys * D * 2), t); };
  // Barrier t.  Before it every wave has waited for its own loads, i.e. its parts of K(t+1) and V(t), issued behind
  // barrier t-1.  Behind it nobody reads K(t-1) (last use: the exact path of iteration t-1) or V(t-1) any more, which is
  // where K(t+2) and V(t+1) go.
  auto sync_and_stage = [&](int t) {
    drain_loads_and_barrier();
    if (t + 2 < n_tiles) issue_k(t + 2);
    if (t + 1 < n_tiles) issue_v(t + 1);
  };
  issue_k(0);
  issue_v(0);
  if (n_tiles > 1) issue_k(1);

  bf16x8 qf[KSTEPS];
  {
    const int qi = min(qw + r32, n - 1);
    pf_load_q<D>(p, (const __bf16*)lv.q + ((long long)(b0 + qi) * p.hq + blk.a) * D + 8 * hf,
                 p.cs + (long long)(b0 + qi) * (D / 2) + 8 * hf, qf);
  }
  FragOffsets<D> fo;
  fo.init(lane);

  f32x16 o[DB], neg_m;
#pragma unroll
  for (int db = 0; db < DB; ++db)
#pragma unroll
    for (int i = 0; i < 16; ++i) o[db][i] = 0.f;
#pragma unroll
  for (int i = 0; i < 16; ++i) neg_m[i] = 0.f;
  float mrow = 0.f, lrow = 0.f;
  f32x16 sa[2], sb[2];  // score tiles (minus m): one has its exponentials taken while the other is accumulated

  // ---- tile 0: exact maxima, so that the pipeline starts from a finite reference ----
  drain_loads_and_barrier();  // K(0), V(0), K(1)
  if (wave_active) {
    score_tile<D, true>(smk[0], fo, qf, neg_m, sa);
    if (t_diag == 0) mask_diagonal(sa, q_in_tile, r32, hf);
    float m = sa[0][0];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int i = 0; i < 16; ++i) m = fmaxf(m, sa[kb][i]);
    mrow = half_max(m);  // finite: key 0 is visible to every query
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int i = 0; i < 16; ++i) sa[kb][i] -= mrow;
  }
#pragma unroll
  for (int i = 0; i < 16; ++i) neg_m[i] = -mrow;

  // The reference of tile t turned out stale (or its sums overflowed): redo the tile exactly.  K(t) is still in LDS.
  // The next tile's scores were started from the old reference and move with it.
  auto exact_redo = [&](int t, f32x16 (&nxt)[2], bool have_next, u32x4 (&w)[4], float& lsum, bf16x8 (&vf0)[DB]) {
    f32x16 sc[2];
    score_tile<D, true>(smk[t % 3], fo, qf, neg_m, sc);
    if (t == t_diag) mask_diagonal(sc, q_in_tile, r32, hf);
    float m = sc[0][0];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int i = 0; i < 16; ++i) m = fmaxf(m, sc[kb][i]);
    const float mnew = fmaxf(mrow, half_max(m));
    const float shift = mrow - mnew;  // <= 0
    const float alpha = __builtin_amdgcn_exp2f(shift);
    mrow = mnew;
    lrow *= alpha;
#pragma unroll
    for (int i = 0; i < 16; ++i) neg_m[i] = -mnew;
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int i = 0; i < 16; ++i) o[db][i] *= alpha;
    if (have_next) {
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int i = 0; i < 16; ++i) nxt[kb][i] += shift;
    }
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int i = 0; i < 16; ++i) sc[kb][i] -= mnew;
    float s0 = 0.f, s1 = 0.f;
#pragma unroll
    for (int u = 0; u < 16; ++u) softmax_unit(sc, u, w, s0, s1);
    lsum = add_chains(s0, s1);
    // requested again rather than kept: this path is short of registers, not of time
#pragma unroll
    for (int db = 0; db < DB; ++db) vf0[db] = read_v_fragment<D>(smv[t & 1], fo, db, 0);
  };

  // one iteration; cur = S(t) - m (consumed), nxt = S(t+1) - m (produced)
  auto iteration = [&](int t, f32x16 (&cur)[2], f32x16 (&nxt)[2]) {
    sync_and_stage(t);
    if (!(wave_active && t <= t_diag)) return;  // rows past the sequence end, tiles past the diagonal: only stage
    const bool have_next = t < t_diag;
    const __bf16* smv_t = smv[t & 1];
    u32x4 w[4];
    bf16x8 vf[2][DB];  // V^T fragments of two 16-key steps: one feeding the MFMAs, one arriving
    float lsum, s0 = 0.f, s1 = 0.f;
    if (have_next) {
      // S(t+1) on the matrix core, exponentials of S(t) on the vector ALU, in ONE instruction stream laid out by hand:
      // slot i = [K fragment requests two k-steps ahead] + MFMA i + exponentials of softmax unit(s) i + packing and row
      // sum of unit(s) i-1 (whose exponentials have had a slot's time to finish).  The scheduling barriers keep the
      // compiler from regrouping the slots; the last slots also request the first V^T fragments of the second product.
      const __bf16* smk_n = smk[(t + 1) % 3];
      constexpr int AHEAD = 2 < KSTEPS ? 2 : KSTEPS;
      constexpr int SLOTS = 2 * KSTEPS;
      bf16x8 kf[2][KSTEPS];
      float e[2][UPM][2];  // exponentials of the units of slot i (parity i & 1)
#pragma unroll
      for (int ks = 0; ks < AHEAD; ++ks)
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) kf[kb][ks] = *(const bf16x8*)(smk_n + fo.k(ks) + kb * 32 * D);
#pragma unroll
      for (int i = 0; i <= SLOTS; ++i) {
        const int ks = i >> 1, kb = i & 1;
        if (i < SLOTS) {
          if (kb == 0 && ks + AHEAD < KSTEPS) {
#pragma unroll
            for (int b = 0; b < 2; ++b) kf[b][ks + AHEAD] = *(const bf16x8*)(smk_n + fo.k(ks + AHEAD) + b * 32 * D);
          }
          if (i >= SLOTS - DB) vf[0][i - (SLOTS - DB)] = read_v_fragment<D>(smv_t, fo, i - (SLOTS - DB), 0);
          nxt[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[kb][ks], qf[ks], ks == 0 ? neg_m : nxt[kb], 0, 0, 0);
#pragma unroll
          for (int x = 0; x < UPM; ++x) {
            const int u = i * UPM + x, kk = u >> 2, j = u & 3, r = 8 * (kk & 1) + 2 * j;
            e[i & 1][x][0] = __builtin_amdgcn_exp2f(cur[kk >> 1][r]);
            e[i & 1][x][1] = __builtin_amdgcn_exp2f(cur[kk >> 1][r + 1]);
          }
        }
        if (i > 0) {
#pragma unroll
          for (int x = 0; x < UPM; ++x) {
            const int u = (i - 1) * UPM + x, kk = u >> 2, j = u & 3;
            w[kk][j] = pack_bf16(e[(i - 1) & 1][x][0], e[(i - 1) & 1][x][1]);
            add_pair(j & 1 ? s1 : s0, w[kk][j]);
          }
        }
        __builtin_amdgcn_sched_barrier(0);
      }
      if (t + 1 == t_diag) {
        asm volatile("" ::: "memory");  // keeps this a branch: only one tile per wave needs the mask
        mask_diagonal(nxt, q_in_tile, r32, hf);
      }
    } else {
      // the wave's last tile: nothing to overlap with
#pragma unroll
      for (int u = 0; u < 16; ++u) {
        const int kk = u >> 2, j = u & 3, r = 8 * (kk & 1) + 2 * j;
        float x0 = cur[kk >> 1][r], x1 = cur[kk >> 1][r + 1];
        asm("" : "+v"(x0), "+v"(x1));  // keeps these exponentials apart from the ones in the other branch, which must stay in their slots
        w[kk][j] = pack_bf16(__builtin_amdgcn_exp2f(x0), __builtin_amdgcn_exp2f(x1));
        add_pair(j & 1 ? s1 : s0, w[kk][j]);
      }
#pragma unroll
      for (int db = 0; db < DB; ++db) vf[0][db] = read_v_fragment<D>(smv_t, fo, db, 0);
    }
    lsum = add_chains(s0, s1);
    if (__any(!(lsum <= kSumLimit))) exact_redo(t, nxt, have_next, w, lsum, vf[0]);
    lrow += lsum;
    // O^T += V^T P^T, the fragments of the next 16-key step requested while this step's MFMAs run
#pragma unroll
    for (int kk = 0; kk < 4; ++kk)
#pragma unroll
      for (int db = 0; db < DB; ++db) {
        if (kk + 1 < 4) vf[(kk + 1) & 1][db] = read_v_fragment<D>(smv_t, fo, db, kk + 1);
        o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[kk & 1][db], __builtin_bit_cast(bf16x8, w[kk]), o[db], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
      }
  };
  // unrolled by two; an odd tile count ends in an iteration past the last tile, which only meets the barrier
  for (int t = 0; t < n_tiles; t += 2) {
    iteration(t, sa, sb);
    iteration(t + 1, sb, sa);
  }

  if (!wave_active) return;
  const int qi = qw + r32;
  const float ltot = half_sum(lrow);
  if (qi >= n) return;
  pf_store_row<D>((__bf16*)lv.out + ((long long)(b0 + qi) * p.hq + blk.a) * D + 4 * hf, o, 1.f / ltot);
  if (lv.lse && hf == 0) lv.lse[(long long)(b0 + qi) * p.hq + blk.a] = (mrow + __builtin_log2f(ltot)) * 0.6931471805599453f;
}

// ------------------------------------------------------------------------------------------------------------------
// host side
// ------------------------------------------------------------------------------------------------------------------
// rotated keys when the caller keeps none
static size_t k_rot_bytes(const earn_attn_desc* desc, int total_tokens) {
  const size_t e = desc->dtype == EARN_F32 ? 4 : 2;
  return ((size_t)total_tokens * desc->n_kv_heads * desc->head_dim * e + 255) / 256 * 256;
}
// (cos, sin) table of the bf16 paths: [tokens][d/2] pairs of floats
static size_t cs_table_bytes(const earn_attn_desc* desc, int total_tokens) {
  if (desc->dtype == EARN_F32) return 0;
  return ((size_t)total_tokens * (desc->head_dim / 2) * sizeof(f32x2) + 255) / 256 * 256;
}
// workspace layout: [rotated keys, unless the caller passes k_rot_out][cos/sin table]
// Without rotation and without k_rot_out nothing is staged at all: the keys are read in place.
size_t prefill_workspace_bytes(const earn_attn_desc* desc, int total_tokens, int have_k_rot_out) {
  if (!(desc->rope_base > 0.f) && !have_k_rot_out) return 0;
  return (have_k_rot_out ? 0 : k_rot_bytes(desc, total_tokens)) + cs_table_bytes(desc, total_tokens);
}

template <typename T, int D>
static void launch_rope_k(const void* k, void* k_rot, const int32_t* cu, const int32_t* positions, int batch, int total,
                          int hkv, const RopeTable& rope, f32x2* cs_out, hipStream_t stream, int n_layers = 1,
                          long long ls_k = 0, long long ls_k_rot = 0) {
  long long threads = (long long)total * (D / 16);
  const unsigned gx = (unsigned)((threads + 255) / 256);
  // fewer than about two workgroups per CU: split the heads over grid rows as well
  const int hpt = (long long)gx * n_layers >= 512 ? hkv : (hkv + 7) / 8;
  hipLaunchKernelGGL((rope_k_kernel<T, D>), dim3(gx, (unsigned)((hkv + hpt - 1) / hpt), n_layers), dim3(256), 0, stream,
                     (const T*)k, (T*)k_rot, cu, positions, batch, total, hkv, rope, cs_out, hpt, ls_k, ls_k_rot);
}

// fp32: the chosen rows of every sequence (q_rows, out_rows: [batch * r, Hq, d]) against the rotated keys, vector kernel
int launch_prefill_rows_f32(const earn_attn_desc* desc, const void* q_rows, const void* k_rot, const void* v,
                            const int32_t* cu_seqlens, const int32_t* row_pos, int batch, int total_tokens,
                            int max_seqlen, int rows_per_seq, void* out_rows, hipStream_t stream) {
  const int d = desc->head_dim;
  PrefillParams p;
  p.cs = nullptr; p.row_pos = row_pos; p.rows_per_seq = rows_per_seq;
  p.q = q_rows; p.k_rot = k_rot; p.v = v; p.cu = cu_seqlens; p.positions = nullptr; p.out = out_rows; p.lse = nullptr;
  p.batch = batch; p.hq = desc->n_q_heads; p.hkv = desc->n_kv_heads; p.max_seqlen = max_seqlen; p.n_qblk = 1;
  p.total = total_tokens;
  p.ls_q = p.ls_k_rot = p.ls_v = p.ls_out = p.ls_lse = 0;
  const float scale = desc->softmax_scale > 0.f ? desc->softmax_scale : 1.0f / sqrtf((float)d);
  p.scale_log2 = scale * 1.4426950408889634f;
  p.rope = make_rope_table(desc->rope_base, d);
  if (make_head_map(desc, &p.heads, "earn_prefill_register_rows") != EARN_OK) return EARN_ERR_UNSUPPORTED;
  dim3 grid((rows_per_seq + 63) / 64, p.hq, batch);
  if (d == 64) hipLaunchKernelGGL((prefill_rows_kernel<float, 64>), grid, dim3(256), 0, stream, p);
  else hipLaunchKernelGGL((prefill_rows_kernel<float, 128>), grid, dim3(256), 0, stream, p);
  return hipGetLastError() == hipSuccess ? EARN_OK : EARN_ERR_HIP;
}

// K rotation on its own (for callers that run the attention with another kernel)
int launch_rope_keys(const earn_attn_desc* desc, const void* k, void* k_rot, const int32_t* cu_seqlens,
                     const int32_t* positions, int batch, int total_tokens, hipStream_t stream) {
  const RopeTable rope = make_rope_table(desc->rope_base, desc->head_dim);
  const int hkv = desc->n_kv_heads;
  if (desc->dtype == EARN_F32) {
    if (desc->head_dim == 64) launch_rope_k<float, 64>(k, k_rot, cu_seqlens, positions, batch, total_tokens, hkv, rope, nullptr, stream);
    else launch_rope_k<float, 128>(k, k_rot, cu_seqlens, positions, batch, total_tokens, hkv, rope, nullptr, stream);
  } else {
    if (desc->head_dim == 64) launch_rope_k<__bf16, 64>(k, k_rot, cu_seqlens, positions, batch, total_tokens, hkv, rope, nullptr, stream);
    else launch_rope_k<__bf16, 128>(k, k_rot, cu_seqlens, positions, batch, total_tokens, hkv, rope, nullptr, stream);
  }
  return hipGetLastError() == hipSuccess ? EARN_OK : EARN_ERR_HIP;
}

int launch_prefill(const earn_attn_desc* desc, const void* q, const void* k, const void* v, const int32_t* cu_seqlens,
                   const int32_t* positions, int batch, int total_tokens, int max_seqlen, void* out, void* k_rot_out,
                   float* lse_out, void* workspace, size_t workspace_bytes, hipStream_t stream,
                   const PrefillLayers* layers) {
  const int d = desc->head_dim;
  const int n_layers = layers ? layers->n_layers : 1;
  const long long ls_k = layers ? layers->kv : 0, ls_kr = layers ? layers->k_rot : 0;
  if ((long long)batch * n_layers > 65535 && desc->dtype == EARN_F32) {
    set_error("earn_prefill_attn_layers: batch * n_layers = %lld exceeds 65535 (fp32 launch shape)", (long long)batch * n_layers);
    return EARN_ERR_UNSUPPORTED;
  }
  const size_t need = prefill_workspace_bytes(desc, total_tokens, k_rot_out != nullptr);
  if (need > workspace_bytes || (need > 0 && !workspace)) {
    set_error("earn_prefill_attn: workspace too small (%zu bytes given, %zu needed)", workspace_bytes, need);
    return EARN_ERR_WORKSPACE_TOO_SMALL;
  }
  // the matrix-core kernels address the K/V rows of ONE sequence with 32-bit byte offsets
  if (desc->dtype == EARN_BF16 && (long long)(max_seqlen + 256) * desc->n_kv_heads * d * 2 >= (1ll << 31)) {
    set_error("earn_prefill_attn: a sequence of %d rows exceeds the 2 GiB addressing range of one sequence", max_seqlen);
    return EARN_ERR_UNSUPPORTED;
  }
  // no rotation and no cache copy asked for: the keys (already rotated by their producer) are read where they are
  const bool in_place = !(desc->rope_base > 0.f) && !k_rot_out;
  const void* k_rot = in_place ? k : (k_rot_out ? k_rot_out : workspace);
  f32x2* cs = !in_place && cs_table_bytes(desc, total_tokens) ? (f32x2*)((char*)workspace + (k_rot_out ? 0 : k_rot_bytes(desc, total_tokens))) : nullptr;
  PrefillParams p;
  p.cs = cs; p.row_pos = nullptr; p.rows_per_seq = 0;
  p.q = q; p.k_rot = k_rot; p.v = v; p.cu = cu_seqlens; p.positions = positions; p.out = out; p.lse = lse_out;
  p.batch = batch; p.hq = desc->n_q_heads; p.hkv = desc->n_kv_heads; p.max_seqlen = max_seqlen;
  p.total = total_tokens;
  p.ls_q = layers ? layers->q : 0; p.ls_k_rot = in_place ? ls_k : ls_kr; p.ls_v = ls_k; p.ls_out = layers ? layers->out : 0;
  p.ls_lse = layers ? layers->lse : 0;
  const float scale = desc->softmax_scale > 0.f ? desc->softmax_scale : 1.0f / sqrtf((float)d);
  p.scale_log2 = scale * 1.4426950408889634f;
  p.rope = make_rope_table(desc->rope_base, d);
  if (make_head_map(desc, &p.heads, "earn_prefill_attn") != EARN_OK) return EARN_ERR_UNSUPPORTED;
  const bool f32 = desc->dtype == EARN_F32;
  if (f32) {
    if (!in_place) {
      if (d == 64) launch_rope_k<float, 64>(k, (void*)k_rot, cu_seqlens, positions, batch, total_tokens, p.hkv, p.rope, cs, stream, n_layers, ls_k, ls_kr);
      else launch_rope_k<float, 128>(k, (void*)k_rot, cu_seqlens, positions, batch, total_tokens, p.hkv, p.rope, cs, stream, n_layers, ls_k, ls_kr);
    }
    dim3 grid((max_seqlen + 63) / 64, p.hq, batch * n_layers);
    if (d == 64) hipLaunchKernelGGL((prefill_rows_kernel<float, 64>), grid, dim3(256), 0, stream, p);
    else hipLaunchKernelGGL((prefill_rows_kernel<float, 128>), grid, dim3(256), 0, stream, p);
  } else if (max_seqlen <= kTileKeys) {
    // register-only layers: every sequence is a single K/V tile
    if (!in_place) {
      if (d == 64) launch_rope_k<__bf16, 64>(k, (void*)k_rot, cu_seqlens, positions, batch, total_tokens, p.hkv, p.rope, cs, stream, n_layers, ls_k, ls_kr);
      else launch_rope_k<__bf16, 128>(k, (void*)k_rot, cu_seqlens, positions, batch, total_tokens, p.hkv, p.rope, cs, stream, n_layers, ls_k, ls_kr);
    }
    p.n_qblk = 1;
    const long long pairs8 = ((long long)batch * p.hkv + kXcds - 1) / kXcds * kXcds;
    dim3 grid((unsigned)(pairs8 * (p.hq / p.hkv)), n_layers, 1);
    if (d == 64) hipLaunchKernelGGL((prefill_mfma_kernel<64, 2, 1>), grid, dim3(128), 0, stream, p);
    else hipLaunchKernelGGL((prefill_mfma_kernel<128, 2, 1>), grid, dim3(128), 0, stream, p);
  } else {
    if (!in_place) {
      if (d == 64) launch_rope_k<__bf16, 64>(k, (void*)k_rot, cu_seqlens, positions, batch, total_tokens, p.hkv, p.rope, cs, stream, n_layers, ls_k, ls_kr);
      else launch_rope_k<__bf16, 128>(k, (void*)k_rot, cu_seqlens, positions, batch, total_tokens, p.hkv, p.rope, cs, stream, n_layers, ls_k, ls_kr);
    }
    // 128-row workgroups (two per CU) in the plain schedule up to medium lengths, where the ends of a workgroup's
    // life (first tile's latency, output store) and the causal diagonal weigh most; the pipelined 256-row kernel beyond.
    // What counts is the length of most sequences, not of the longest: a ragged batch whose mean length is medium
    // takes the 128-row form whatever its longest sequence (lengths spread over 269-4018, mean 1411: 1.18 against
    // 1.27 ms per layer).
    const int rows_set = tuning(kTunePrefillBlockRows, 0);
    const bool medium = max_seqlen <= 3072 || total_tokens / batch <= 2048;
    const int block_rows = rows_set == 128 || rows_set == 256 ? rows_set : (medium ? 128 : 256);
    p.n_qblk = (max_seqlen + block_rows - 1) / block_rows;
    const long long pairs8 = ((long long)batch * p.hkv + kXcds - 1) / kXcds * kXcds;
    dim3 grid((unsigned)(pairs8 * p.n_qblk * (p.hq / p.hkv)), n_layers, 1);
    if (block_rows == 128) {
      if (d == 64) hipLaunchKernelGGL((prefill_mfma_kernel<64, 4, 2>), grid, dim3(256), 0, stream, p);
      else hipLaunchKernelGGL((prefill_mfma_kernel<128, 4, 2>), grid, dim3(256), 0, stream, p);
    } else {
      if (d == 64) hipLaunchKernelGGL((prefill_pipe_kernel<64, 8>), grid, dim3(512), 0, stream, p);
      else hipLaunchKernelGGL((prefill_pipe_kernel<128, 8>), grid, dim3(512), 0, stream, p);
    }
  }
  return hipGetLastError() == hipSuccess ? EARN_OK : EARN_ERR_HIP;
}

}  // namespace earn

#ifdef EARN_PF_TIMELINE
// buf: device memory of slots * 8 64-bit words, zeroed by the caller; NULL switches the timers off
extern "C" int earn_debug_set_timeline(void* buf, int slots) {
  if (hipMemcpyToSymbol(HIP_SYMBOL(earn::g_pf_timeline_slots), &slots, sizeof(slots)) != hipSuccess) return EARN_ERR_HIP;
  return hipMemcpyToSymbol(HIP_SYMBOL(earn::g_pf_timeline), &buf, sizeof(buf)) == hipSuccess ? EARN_OK : EARN_ERR_HIP;
}
#endif
