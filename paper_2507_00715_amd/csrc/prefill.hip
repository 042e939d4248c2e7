// Causal prefill attention over a packed ragged batch (paper Section 2.2, Eq. 3; used at full length for the first
// k layers and on the compacted register rows, with their original positions, for the remaining N-k layers —
// Section 3.2, Inference).
//
// Three kernels:
//   rope_k_kernel        rotates K once per layer into the buffer the KV cache keeps (k_rot_out); every query block
//                        then reads rotated keys, so the sin/cos work is O(T), not O(T * blocks).
//   prefill_mfma_kernel  bf16 flash-style attention on the matrix cores (v_mfma_f32_32x32x16_bf16).
//   prefill_rows_kernel  fp32 (or bf16) attention on the vector ALU: one query row per 4 lanes. Used for the fp32
//                        configuration, where the 1e-4 tolerance rules out bf16 operands.
//
// MFMA kernel layout (all shapes in the 32x32x16 tile of the instruction, 64 lanes, lane = (r32 = lane%32, hf = lane/32)):
//   The kernel computes the TRANSPOSED score tile S^T = K Q^T (keys x queries).  Its accumulator layout gives every lane
//   ONE query column (r32) and 16 of the 32 keys of a block, so the softmax row statistics are a private loop plus one
//   exchange with lane^32, and the rescaling of the output accumulator is lane-private as well.
//   The accumulator registers of S^T, converted to bf16, are exactly the B operand (keys x queries, 8 keys per lane)
//   of the second product O^T = V^T P^T, so P never leaves registers.  The 8 key slots of a lane are keys
//   {4hf..4hf+3, 8+4hf..8+4hf+3} of a 16-key step; the A operand V^T uses the same key order, which is what two
//   transposing LDS reads (ds_read_b64_tr_b16: 4 consecutive keys of one d column) deliver from a V tile kept in its
//   natural [key][d] layout.
//   A workgroup is 4 waves; each wave owns 64 query rows (2 column blocks), so every K/V fragment read from LDS feeds
//   two MFMAs; the 64-key K/V tile in LDS is shared by the 4 waves (256 query rows per tile load).
#include <stdlib.h>

#include "common.h"
#include <type_traits>

namespace earn {

struct PrefillParams {
  const void* q; const void* k_rot; const void* v; const int32_t* cu; const int32_t* positions;
  void* out; float* lse;
  int batch, hq, hkv, max_seqlen;
  int n_qblk;  // query blocks of the longest sequence
  float scale_log2;
  RopeTable rope;
};

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
template <typename T, int D>
__global__ __launch_bounds__(256) void rope_k_kernel(const T* __restrict__ k, T* __restrict__ k_rot,
                                                     const int32_t* __restrict__ cu,
                                                     const int32_t* __restrict__ positions, int batch, int total,
                                                     int hkv, RopeTable rope) {
  constexpr int G = D / 16;  // groups of 8 pairs per head
  const long long t = (long long)blockIdx.x * 256 + threadIdx.x;
  if (t >= (long long)total * G) return;
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
  const T* src = k + (long long)token * hkv * D + g * 8;
  T* dst = k_rot + (long long)token * hkv * D + g * 8;
  for (int h = 0; h < hkv; ++h) {
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
  const int a = blockIdx.y, s = blockIdx.z;
  const int b0 = p.cu[s], n = p.cu[s + 1] - b0;
  const int row0 = blockIdx.x * 64;
  if (row0 >= n) return;
  const int qt = threadIdx.x & 3;
  const int i = row0 + (threadIdx.x >> 2);
  const bool row_ok = i < n;
  const int ic = row_ok ? i : n - 1;
  const int c = a / (p.hq / p.hkv);
  const T* qrow = (const T*)p.q + ((long long)(b0 + ic) * p.hq + a) * D;
  float ql[E], qh[E];
#pragma unroll
  for (int e = 0; e < E; e += 8) { Vec8<T>::load(qrow + qt * E + e, ql + e); Vec8<T>::load(qrow + D / 2 + qt * E + e, qh + e); }
  const int pos = p.positions ? p.positions[b0 + ic] : ic;
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
  const int wave_last = min(n - 1, row0 + (int)(threadIdx.x / kWave) * 16 + 15);
  const T* kbase = (const T*)p.k_rot + ((long long)b0 * p.hkv + c) * D;
  const T* vbase = (const T*)p.v + ((long long)b0 * p.hkv + c) * D;
  const long long rs = (long long)p.hkv * D;
  for (int j = 0; j <= wave_last; ++j) {
    float kl[E], kh[E], vl[E], vh[E];
#pragma unroll
    for (int e = 0; e < E; e += 8) {
      Vec8<T>::load(kbase + j * rs + qt * E + e, kl + e);
      Vec8<T>::load(kbase + j * rs + D / 2 + qt * E + e, kh + e);
      Vec8<T>::load(vbase + j * rs + qt * E + e, vl + e);
      Vec8<T>::load(vbase + j * rs + D / 2 + qt * E + e, vh + e);
    }
    float sc = 0.f;
#pragma unroll
    for (int e = 0; e < E; ++e) sc = __builtin_fmaf(ql[e], kl[e], __builtin_fmaf(qh[e], kh[e], sc));
    sc += __shfl_xor(sc, 1, kWave);
    sc += __shfl_xor(sc, 2, kWave);
    if (j <= ic) {  // causal: keys 0..i
      float mn = fmaxf(m, sc);
      float corr = __builtin_amdgcn_exp2f(m - mn);  // exp2(-inf) = 0 on the first key
      float pr = __builtin_amdgcn_exp2f(sc - mn);
      l = l * corr + pr;
#pragma unroll
      for (int e = 0; e < E; ++e) { ol[e] = __builtin_fmaf(pr, vl[e], ol[e] * corr); oh[e] = __builtin_fmaf(pr, vh[e], oh[e] * corr); }
      m = mn;
    }
  }
  if (!row_ok) return;
  const float inv = 1.f / l;
#pragma unroll
  for (int e = 0; e < E; ++e) { ol[e] *= inv; oh[e] *= inv; }
  T* orow = (T*)p.out + ((long long)(b0 + i) * p.hq + a) * D;
#pragma unroll
  for (int e = 0; e < E; e += 8) { Vec8<T>::store(orow + qt * E + e, ol + e); Vec8<T>::store(orow + D / 2 + qt * E + e, oh + e); }
  if (p.lse && qt == 0) p.lse[(long long)(b0 + i) * p.hq + a] = (m + __builtin_log2f(l)) * 0.6931471805599453f;
}

// ------------------------------------------------------------------------------------------------------------------
// bf16 MFMA flash attention
// ------------------------------------------------------------------------------------------------------------------
constexpr int kXcds = 8;         // accelerator complex dies, each with a private L2
constexpr int kTileKeys = 64;    // keys per K/V tile in LDS

typedef __attribute__((address_space(3))) s16x4* lds_s16x4_ptr;

// K/V tiles are written to LDS by the memory pipeline itself (buffer loads with the LDS bit: lane l of a wave
// instruction deposits its 16 bytes at base + 16 l), so rows cannot be padded.  Bank conflicts are avoided by an XOR
// swizzle instead: the 16-byte chunk c of row `row` lives at chunk position c ^ swz(row); each lane simply FETCHES the
// chunk that belongs at its fixed LDS position.  The swizzle makes both read patterns conflict free: the K fragments
// (16 consecutive rows, same chunk) and the transposing V reads (4 consecutive rows x 4 consecutive chunks).
template <int D>
__device__ __forceinline__ int swz(int row) {
  if constexpr (D == 128) return 4 * (row & 3) + ((row >> 2) & 3);     // 16 chunks per row
  else return 4 * ((row >> 1) & 1) + ((row >> 2) & 3);                  // 8 chunks per row (two rows per 256 bytes)
}
template <int D, int STAGES>
struct PfSmem {
  __bf16 k[STAGES][kTileKeys * D];   // ring of STAGES tiles: tiles t+1 .. t+STAGES-1 arrive while tile t is read
  __bf16 v[STAGES][kTileKeys * D];
};
typedef __attribute__((address_space(3))) void* lds_void_ptr;

// One 16-byte-per-lane buffer load that lands directly in LDS: lane l's chunk goes to lds_addr + 16 l (lds_addr, the
// byte address inside LDS, is wave-uniform and travels in M0); a chunk outside the descriptor's range arrives as zeros.
// Written as an instruction rather than through the compiler's builtin on purpose: the compiler cannot tell which LDS
// reads such a load may alias and drains the whole vector-memory queue before every later LDS read, which would allow
// no more than a fraction of one tile's compute time for a tile to arrive.  Here the kernel keeps the order itself
// (sync_and_stage below): a buffer is read only after a counted wait for its loads plus a workgroup barrier.  The kernel
// uses M0 for nothing else.  The wait state between the M0 write and the load is the one the compiler also leaves.
__device__ __forceinline__ void dma16_to_lds(u32x4 rsrc, unsigned lds_addr, int voff, int soff) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds"
               :
               : "s"(lds_addr), "v"(voff), "s"(rsrc), "s"(soff)
               : "memory");
}
// Raw (unstrided, unswizzled) buffer descriptor over [base, base + bytes): accesses are range checked against `bytes`.
__device__ __forceinline__ u32x4 raw_buffer(const void* base, int bytes) {
  const unsigned long long a = (unsigned long long)base;
  u32x4 r;
  r[0] = __builtin_amdgcn_readfirstlane((unsigned)a);
  r[1] = __builtin_amdgcn_readfirstlane((unsigned)(a >> 32) & 0xffffu);
  r[2] = __builtin_amdgcn_readfirstlane((unsigned)bytes);
  r[3] = 0x00020000u;
  return r;
}
template <int N>
__device__ __forceinline__ void wait_vmcnt() {  // wait until at most N vector-memory loads of this wave are in flight
  static_assert(N >= 0 && N < 64);
  __builtin_amdgcn_s_waitcnt(0x0F70 | (N & 15) | ((N >> 4) << 14));
}

// Between rescales the exponentials are taken against a stale row maximum, so they can exceed 1; they are allowed to
// grow until a lane's partial row sum passes this limit.  That is harmless in fp32 sums and in bf16 operands, and the
// final normalisation uses the same reference, so the result is the same function.  Rescaling touches every
// accumulator register of a lane, so doing it only when needed removes most vector-ALU work from the key loop.
constexpr float kSumLimit = 1024.0f;  // per lane: 32 exponentials of one query row

// max / sum of a value with its partner in the other half of the wave (lane ^ 32), without going through LDS
__device__ __forceinline__ float half_max(float x) {
  auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float half_sum(float x) {
  auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

// QB = 32-query column blocks per wave; the workgroup has 8/QB waves (256 query rows either way).
//   QB = 2: 4 waves, one per SIMD, every K/V fragment read from LDS feeds two MFMAs, ~470 registers per lane.
//   QB = 1: 8 waves, two per SIMD (<= 256 registers per lane): while one wave of a SIMD runs its softmax on the
//           vector ALU the other keeps the matrix core busy; LDS traffic per MFMA doubles (fits: LDS reads run at
//           256 B/clk per CU on this part).
// WAVES = waves per workgroup.  8 (or 4 with QB = 2) gives 256 query rows per workgroup; WAVES = 4 with QB = 1 gives
// 128-row workgroups, two of which share a CU: less idle time on the causal diagonal of short sequences, at the price
// of staging every K/V tile twice as often.
// STAGES = 1 (with WAVES = 2: 64 rows) is the register-only-layer variant: every sequence fits one K/V tile, so there is
// nothing to double buffer, and the small footprint (38 KiB LDS, 128 threads) lets 4 workgroups share a CU, which is
// what hides the load -> rotate -> multiply latency chain of these tiny problems.
template <int D, int QB, int WAVES, int STAGES>
__global__ __launch_bounds__(64 * WAVES, (QB == 1 && WAVES <= 4) ? 2 : 1) void prefill_mfma_kernel(PrefillParams p) {
  constexpr int kWaveRows = 32 * QB;
  constexpr int kBlockRows = kWaveRows * WAVES;
  constexpr int KSTEPS = D / 16;         // MFMA k-steps over head_dim for S^T
  constexpr int DB = D / 32;             // 32-row blocks of O^T
  constexpr int UPR = D / 8;             // 16-byte units per K/V row
  constexpr bool PP = STAGES == 3;       // ping-pong schedule of the two waves of a SIMD
  static_assert(!PP || WAVES == 8, "ping-pong pairs wave w with wave w + 4 on one SIMD");
  using Sm = PfSmem<D, STAGES>;
  __shared__ Sm sm;

  // ---- workgroup -> (sequence, kv head, query block, head of the group), XCD aware ----
  // Workgroups are handed to the 8 XCDs round-robin by linear id, and every XCD has its own L2.  Id (x, k) = the k-th
  // workgroup of XCD x.  Each XCD walks its own list of (sequence, kv head) pairs (pair % 8 == x) one pair at a time:
  // all query blocks of the pair (long, late blocks first) and all query heads of the group, so the workgroups that
  // are resident on an XCD at any moment stream the SAME K/V rows and find them in that XCD's L2.
  const int gq = p.hq / p.hkv;
  const int xcd = blockIdx.x % kXcds, k_in_xcd = blockIdx.x / kXcds;
  const int per_pair = p.n_qblk * gq;
  const int pair = (k_in_xcd / per_pair) * kXcds + xcd;
  if (pair >= p.batch * p.hkv) return;
  const int rem = k_in_xcd % per_pair;
  const int qblk = p.n_qblk - 1 - rem / gq;
  const int s = pair / p.hkv, c = pair % p.hkv;
  const int a = c * gq + rem % gq;
  const int b0 = p.cu[s], n = p.cu[s + 1] - b0;
  const int q0 = qblk * kBlockRows;
  if (q0 >= n) return;
  // the wave index is the same in all 64 lanes: say so, and everything derived from it (the wave's query window, its
  // diagonal tile, the tile loop) lives in scalar registers and branches without touching the execution mask
  const int lane = threadIdx.x % kWave, wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
  const int r32 = lane & 31, hf = lane >> 5;
  const int qw = q0 + wave * kWaveRows;          // first query row of this wave
  const bool wave_active = qw < n;
  const int t_diag = qw / kTileKeys;             // last (diagonal) tile of this wave
  const int q_in_tile = qw - t_diag * kTileKeys; // offset of the wave's first query inside that tile
  const int n_tiles = (min(q0 + kBlockRows, n) + kTileKeys - 1) / kTileKeys;

  const __bf16* Qg = (const __bf16*)p.q;
  const __bf16* Kg = (const __bf16*)p.k_rot + ((long long)b0 * p.hkv + c) * D;
  const __bf16* Vg = (const __bf16*)p.v + ((long long)b0 * p.hkv + c) * D;
  const long long kv_stride = (long long)p.hkv * D;

  // ---- tile staging: global -> LDS directly ----
  // A tile is kTileKeys*UPR 16-byte units = UPR wave instructions per tensor; wave w issues instructions w, w+WAVES, ...
  // Instruction I fills LDS units [64 I, 64 I + 64): rows RPI*I + lane/UPR, chunk position lane%UPR.  Rows past the end of
  // the sequence are outside the buffer descriptor and read as zeros (finite data for the masked tail, no clamping).
  constexpr int NI = UPR / WAVES;       // instructions per wave, tile and tensor
  constexpr int RPI = kWave / UPR;      // rows per instruction
  const int row_bytes = (int)kv_stride * 2;
  const int seq_bytes = (n - 1) * row_bytes + D * 2;
  const u32x4 k_rsrc = raw_buffer(Kg, seq_bytes), v_rsrc = raw_buffer(Vg, seq_bytes);
  int st_voff[NI];
#pragma unroll
  for (int i = 0; i < NI; ++i) {
    const int row = RPI * (wave + WAVES * i) + lane / UPR;
    st_voff[i] = row * row_bytes + ((lane % UPR) ^ swz<D>(row)) * 16;
  }
  const unsigned lds_k = (unsigned)(size_t)(lds_void_ptr)&sm.k[0][0], lds_v = (unsigned)(size_t)(lds_void_ptr)&sm.v[0][0];
  auto issue_tile = [&](int t, int buf) {
#if defined(EARN_DBG_NOSTAGE)
    if (t >= STAGES) return;
#endif
    const int soff = t * kTileKeys * row_bytes;
#pragma unroll
    for (int i = 0; i < NI; ++i) {
      const unsigned at = (unsigned)((buf * kTileKeys * D + (wave + WAVES * i) * 512) * 2);
      dma16_to_lds(k_rsrc, lds_k + at, st_voff[i], soff);
      dma16_to_lds(v_rsrc, lds_v + at, st_voff[i], soff);
    }
  };
  // Barrier b (b = 0, 1, ..): every wave has waited for its own part of tile b, so behind the barrier tile b is
  // complete and visible; the wave then starts its part of tile b+1 into the next buffer of the ring.  Waves that run
  // "on time" pass barrier b at the top of iteration b.  With PP (ping-pong, 3 buffers) the upper half of the waves runs
  // "late": it passes barrier b+1 in the MIDDLE of iteration b, between its two matrix products.  The barrier then
  // holds the two waves that share a SIMD half an iteration apart for good, so that one of them is in its matrix
  // products while the other is in its exponentials, instead of both competing for the same unit and leaving the other
  // idle.  Buffer (b+1) % STAGES held tile b+1-STAGES: on-time waves are done with that tile before barrier b+2-STAGES,
  // late waves (STAGES = 3) read its V between barriers b-1 and b; both are behind every wave when barrier b opens.
  auto sync_and_stage = [&](int b) {
#if !defined(EARN_DBG_NOWAIT)
    wait_vmcnt<0>();
#endif
    __syncthreads();
    if constexpr (STAGES > 1) {
      if (b + 1 < n_tiles) issue_tile(b + 1, (b + 1) % STAGES);
    }
  };
  issue_tile(0, 0);  // in flight while the queries are loaded and rotated

  // ---- Q fragments: rotate at the original position, fold in scale*log2(e), keep as bf16 B operands ----
  bf16x8 qf[QB][KSTEPS];
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    const int qi = min(qw + 32 * qb + r32, n - 1);
    const float pos = (float)(p.positions ? p.positions[b0 + qi] : qi);
    const __bf16* qrow = Qg + ((long long)(b0 + qi) * p.hq + a) * D + 8 * hf;
#pragma unroll
    for (int ks = 0; ks < KSTEPS / 2; ++ks) {
      float lo[8], hi[8];
      Vec8<__bf16>::load(qrow + 16 * ks, lo);
      Vec8<__bf16>::load(qrow + 16 * ks + D / 2, hi);
      u32x4 wl, wh;
#pragma unroll
      for (int j = 0; j < 8; j += 2) {
        float x[2], y[2];
#pragma unroll
        for (int jj = 0; jj < 2; ++jj) {
          float sn = 0.f, cs = 1.f;
          const int e = 16 * ks + 8 * hf + j + jj;
          if (p.rope.enabled) sincos_turns_fast(rope_turns(pos, p.rope.hi[e], p.rope.lo[e]), &sn, &cs);
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

  // per-lane LDS element offsets of the MFMA fragments (the swizzle does not depend on kb / kk: those add multiples of 16 rows)
  int k_offs[KSTEPS];      // + kb * 32 * D
#pragma unroll
  for (int ks = 0; ks < KSTEPS; ++ks) k_offs[ks] = r32 * D + (((2 * ks + hf) ^ swz<D>(r32)) << 3);
  int v_offs[DB][2];       // + kk * 16 * D ; [..][1] is the second group of 4 keys (8 rows further)
#pragma unroll
  for (int db = 0; db < DB; ++db)
#pragma unroll
    for (int h2 = 0; h2 < 2; ++h2) {
      const int row = 4 * hf + 8 * h2 + ((lane & 15) >> 2);
      const int chunk = 4 * db + 2 * ((lane >> 4) & 1) + ((lane & 3) >> 1);
      v_offs[db][h2] = row * D + ((chunk ^ swz<D>(row)) << 3) + 4 * (lane & 1);
    }

  // ---- pieces of one key-tile iteration ----
  // S^T = K Q^T for tile t.  All 2*KSTEPS K fragments are requested from LDS before
  // the first MFMA (and before `staging`, the global->LDS traffic of later tiles), so the MFMAs wait on a draining
  // queue instead of paying one LDS round trip each.
  auto scores = [&](int buf, f32x16 (&sc)[2][QB], const f32x16 (&init)[QB]) {
    const __bf16* smk = sm.k[buf];
#ifndef EARN_PF_KAHEAD
#define EARN_PF_KAHEAD 2
#endif
    constexpr int AHEAD = EARN_PF_KAHEAD < KSTEPS ? EARN_PF_KAHEAD : KSTEPS;  // k-steps of K fragments in flight ahead of the MFMAs
    bf16x8 kf[2][KSTEPS];
    auto fetch_k = [&](int ks) {
#pragma unroll
      for (int kb = 0; kb < 2; ++kb) kf[kb][ks] = *(const bf16x8*)(smk + k_offs[ks] + kb * 32 * D);
    };
#pragma unroll
    for (int ks = 0; ks < AHEAD; ++ks) fetch_k(ks);
#pragma unroll
    for (int ks = 0; ks < KSTEPS; ++ks) {
      if (ks + AHEAD < KSTEPS) fetch_k(ks + AHEAD);
      __builtin_amdgcn_sched_barrier(0);  // the fragment requests stay ahead of the MFMAs that hide their latency
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int qb = 0; qb < QB; ++qb)
          sc[kb][qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[kb][ks], qf[qb][ks], ks == 0 ? init[qb] : sc[kb][qb], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
    }
  };
  // causal mask, in place; it only bites on the wave's diagonal tile (keys beyond the sequence end are beyond every
  // valid query too), elsewhere the bound is out of reach
  auto mask_causal = [&](int t, f32x16 (&sc)[2][QB]) {
    const int bound = t == t_diag ? q_in_tile + r32 - 4 * hf : kTileKeys;  // lane's last visible key, less its 4 hf share
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int qb = 0; qb < QB; ++qb)
#pragma unroll
        for (int i = 0; i < 16; ++i)
          sc[kb][qb][i] = (32 * kb + 8 * (i >> 2) + (i & 3) > bound + 32 * qb) ? -INFINITY : sc[kb][qb][i];
  };
  // P = exp2(S - m) in place.  SHIFTED: the scores already carry -m (the steady-state path starts its score
  // accumulators at -m instead of 0, which takes the subtraction off the vector ALU).
  auto exponentials = [&](f32x16 (&sc)[2][QB], auto shifted) {
#pragma unroll
    for (int qb = 0; qb < QB; ++qb)
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
#if defined(EARN_DBG_NOEXP)
          sc[kb][qb][i] = sc[kb][qb][i] * 1e-30f;
#else
          sc[kb][qb][i] = __builtin_amdgcn_exp2f(decltype(shifted)::value ? sc[kb][qb][i] : sc[kb][qb][i] - mrow[qb]);
#endif
        }
  };
  // P as bf16 B operands of the second product, and the lane's share of the row sums.  The sums are taken over the
  // ROUNDED probabilities (two per instruction, exact products with 1 accumulated in fp32): they are the weights the
  // second product really applies, and it halves the additions.
  auto pack_probs = [&](f32x16 (&sc)[2][QB], bf16x8 (&pf)[QB][4], float (&lsum)[QB]) {
    const unsigned ones = 0x3f803f80u;  // (1.0, 1.0) in bf16
    // acc += w.lo + w.hi.  Written as instructions: the compiler's own dot builtin came out wrong in this kernel (half
    // of the words summed twice, the other half not at all).  What the compiler would otherwise look after is done by
    // hand: a dot result may feed the next dot's accumulator at once, but any other vector instruction has to keep
    // three wait states' distance, hence the s_nop in front of the closing addition.
    auto add_pair = [&](float& acc, unsigned w) {
      asm("v_dot2c_f32_bf16 %0, %1, %2" : "+v"(acc) : "s"(ones), "v"(w));
    };
    auto add_chains = [&](float s0, float s1) {
      float r;
      asm("s_nop 2\n\tv_add_f32 %0, %1, %2" : "=v"(r) : "v"(s0), "v"(s1));
      return r;
    };
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
      float s0 = 0.f, s1 = 0.f;  // two chains
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) {
        u32x4 w;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          w[j] = pack_bf16(sc[kk >> 1][qb][8 * (kk & 1) + 2 * j], sc[kk >> 1][qb][8 * (kk & 1) + 2 * j + 1]);
          add_pair(j & 1 ? s1 : s0, w[j]);
        }
        pf[qb][kk] = __builtin_bit_cast(bf16x8, w);
      }
      lsum[qb] = add_chains(s0, s1);
    }
  };
  // V^T fragments of tile t (A operands of the second product): requested before the exponentials so that the LDS
  // latency hides behind the vector-ALU work
  auto fetch_v = [&](int buf, bf16x8 (&vf)[4][DB]) {
    const __bf16* smv = sm.v[buf];
#pragma unroll
    for (int kk = 0; kk < 4; ++kk)
#pragma unroll
      for (int db = 0; db < DB; ++db) {
        s16x4 v0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(smv + v_offs[db][0] + kk * 16 * D));
        s16x4 v1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(smv + v_offs[db][1] + kk * 16 * D));
        typedef short s16x8 __attribute__((ext_vector_type(8)));
        s16x8 vv = __builtin_shufflevector(v0, v1, 0, 1, 2, 3, 4, 5, 6, 7);
        vf[kk][db] = __builtin_bit_cast(bf16x8, vv);
      }
    __builtin_amdgcn_sched_barrier(0);
  };
  // row sums, O^T += V^T P^T
  auto accumulate = [&](bf16x8 (&pf)[QB][4], float (&lsum)[QB], bf16x8 (&vf)[4][DB]) {
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) lrow[qb] += lsum[qb];
#pragma unroll
    for (int kk = 0; kk < 4; ++kk)
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int qb = 0; qb < QB; ++qb)
          o[db][qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[kk][db], pf[qb][kk], o[db][qb], 0, 0, 0);
  };

  // Every wave passes exactly one barrier per tile, whichever path it takes.  The steady-state loop takes the
  // exponentials against the reference maxima it already has and never touches the output accumulators with the
  // vector ALU.  It does not even compute row maxima: a reference is stale exactly when some exponential is large, so
  // the (already needed) partial row sums are compared with kSumLimit instead.  A wave that fails leaves the loop,
  // recomputes the tile's scores, takes the exact maxima, rescales, finishes the tile and re-enters.  Tile 0 (reference
  // still -inf) and the wave's diagonal tile (the only one that needs the causal mask) always take the exact path.
  f32x16 zero16[QB], neg_m[QB];  // score accumulator starts: 0 (exact path), -m in every register (steady state)
#pragma unroll
  for (int qb = 0; qb < QB; ++qb)
#pragma unroll
    for (int i = 0; i < 16; ++i) { zero16[qb][i] = 0.f; neg_m[qb][i] = 0.f; }
  const bool late = PP && wave >= WAVES / 2;
  if (late) sync_and_stage(0);
  // The exact path.  synced = the tile fell out of the steady-state loop, which has passed the tile's barrier already.
  auto exact_tile = [&](int t, int buf, bool synced) {
    if (!late && !synced) sync_and_stage(t);
    f32x16 sc[2][QB];
    float lsum[QB];
    bf16x8 vf[4][DB];
    bf16x8 pf[QB][4];
    scores(buf, sc, zero16);
    mask_causal(t, sc);
    if (late && !synced && t + 1 < n_tiles) sync_and_stage(t + 1);
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
      float m = sc[0][qb][0];
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int i = 0; i < 16; ++i) m = fmaxf(m, sc[kb][qb][i]);
      const float mnew = fmaxf(mrow[qb], half_max(m));  // finite: tile 0 holds key 0, visible to every query
      const float alpha = __builtin_amdgcn_exp2f(mrow[qb] - mnew);
      mrow[qb] = mnew;
#pragma unroll
      for (int i = 0; i < 16; ++i) neg_m[qb][i] = -mnew;
      lrow[qb] *= alpha;
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int i = 0; i < 16; ++i) o[db][qb][i] *= alpha;
    }
    fetch_v(buf, vf);
    exponentials(sc, std::false_type{});
    pack_probs(sc, pf, lsum);
    accumulate(pf, lsum, vf);
  };
#if defined(EARN_DBG_PHASES)  // working instrumentation: cycles per phase of the steady-state loop, written in place of lse
  long long ph[5] = {0, 0, 0, 0, 0};
  int ph_tiles = 0;
#define PH_STAMP(x) { __builtin_amdgcn_sched_barrier(0); x = (long long)__builtin_readcyclecounter(); __builtin_amdgcn_sched_barrier(0); }
#else
#define PH_STAMP(x)
#endif
  int t = 0, buf = 0;  // buf = t % STAGES
  auto next_tile = [&]() { ++t; buf = (buf + 1 == STAGES ? 0 : buf + 1); };
  while (t < n_tiles) {
    bool exact = wave_active && t == 0, synced = false;
    if (!exact)
    for (; t < n_tiles; next_tile()) {
      const bool work = wave_active && t <= t_diag;  // else rows past the sequence end or a tile past the diagonal: only stage
      if (work && t == t_diag) { exact = true; break; }
      [[maybe_unused]] long long c0, c1, c2, c2b, c3, c4;
      PH_STAMP(c0);
      if (!late) sync_and_stage(t);
      PH_STAMP(c1);
      f32x16 sc[2][QB];
      float lsum[QB];
      bf16x8 vf[4][DB];
      bf16x8 pf[QB][4];
      if (work) scores(buf, sc, neg_m);
      PH_STAMP(c2);
      if (late && t + 1 < n_tiles) sync_and_stage(t + 1);
      PH_STAMP(c2b);
      if (work) {
        fetch_v(buf, vf);
#if defined(EARN_DBG_PHASES) && EARN_DBG_PHASES == 2
        { long long cv; PH_STAMP(cv); ph[4] += cv - c2b; }
#endif
        exponentials(sc, std::true_type{});
        pack_probs(sc, pf, lsum);
        PH_STAMP(c3);
        bool stale = false;
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) stale |= !(lsum[qb] <= kSumLimit);
        if (__any(stale)) { exact = synced = true; break; }
        accumulate(pf, lsum, vf);
        PH_STAMP(c4);
#if defined(EARN_DBG_PHASES)
        ph[0] += c1 - c0; ph[1] += c2 - c1; ph[2] += c3 - c2b; ph[3] += c4 - c3; ph[4] += c2b - c2; ++ph_tiles;
#endif
      }
    }
    if (!exact) break;
    exact_tile(t, buf, synced);
    next_tile();
  }

  if (!wave_active) return;
  // ---- epilogue: normalise and store; lane holds d = 32db + 8j + 4hf + (0..3) of query r32 ----
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    const int qi = qw + 32 * qb + r32;
    const float ltot = half_sum(lrow[qb]);
    if (qi >= n) continue;
    const float inv = 1.f / ltot;
    __bf16* orow = (__bf16*)p.out + ((long long)(b0 + qi) * p.hq + a) * D + 4 * hf;
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        u32x2 w;
        w[0] = pack_bf16(o[db][qb][4 * j] * inv, o[db][qb][4 * j + 1] * inv);
        w[1] = pack_bf16(o[db][qb][4 * j + 2] * inv, o[db][qb][4 * j + 3] * inv);
        *(u32x2*)(orow + 32 * db + 8 * j) = w;
      }
#if defined(EARN_DBG_PHASES)
    if (p.lse && hf == 0) p.lse[(long long)(b0 + qi) * p.hq + a] = r32 < 5 ? (float)ph[r32 < 5 ? r32 : 0] / (float)max(ph_tiles, 1) : (float)ph_tiles;
#else
    if (p.lse && hf == 0) p.lse[(long long)(b0 + qi) * p.hq + a] = (mrow[qb] + __builtin_log2f(ltot)) * 0.6931471805599453f;
#endif
  }
}

// ------------------------------------------------------------------------------------------------------------------
// host side
// ------------------------------------------------------------------------------------------------------------------
size_t prefill_workspace_bytes(const earn_attn_desc* desc, int total_tokens, int have_k_rot_out) {
  if (have_k_rot_out) return 0;
  const size_t e = desc->dtype == EARN_F32 ? 4 : 2;
  return ((size_t)total_tokens * desc->n_kv_heads * desc->head_dim * e + 255) / 256 * 256;
}

template <typename T, int D>
static void launch_rope_k(const void* k, void* k_rot, const int32_t* cu, const int32_t* positions, int batch, int total,
                          int hkv, const RopeTable& rope, hipStream_t stream) {
  long long threads = (long long)total * (D / 16);
  hipLaunchKernelGGL((rope_k_kernel<T, D>), dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, stream,
                     (const T*)k, (T*)k_rot, cu, positions, batch, total, hkv, rope);
}

#ifndef EARN_PF_STAGES4
#define EARN_PF_STAGES4 2
#endif
#ifndef EARN_PF_STAGES8
#define EARN_PF_STAGES8 2
#endif
int launch_prefill(const earn_attn_desc* desc, const void* q, const void* k, const void* v, const int32_t* cu_seqlens,
                   const int32_t* positions, int batch, int total_tokens, int max_seqlen, void* out, void* k_rot_out,
                   float* lse_out, void* workspace, size_t workspace_bytes, hipStream_t stream) {
  const int d = desc->head_dim;
  const size_t need = prefill_workspace_bytes(desc, total_tokens, k_rot_out != nullptr);
  if (need > workspace_bytes || (need > 0 && !workspace)) {
    set_error("earn_prefill_attn: workspace too small (%zu bytes given, %zu needed)", workspace_bytes, need);
    return EARN_ERR_WORKSPACE_TOO_SMALL;
  }
  void* k_rot = k_rot_out ? k_rot_out : workspace;
  PrefillParams p;
  p.q = q; p.k_rot = k_rot; p.v = v; p.cu = cu_seqlens; p.positions = positions; p.out = out; p.lse = lse_out;
  p.batch = batch; p.hq = desc->n_q_heads; p.hkv = desc->n_kv_heads; p.max_seqlen = max_seqlen;
  const float scale = desc->softmax_scale > 0.f ? desc->softmax_scale : 1.0f / sqrtf((float)d);
  p.scale_log2 = scale * 1.4426950408889634f;
  p.rope = make_rope_table(desc->rope_base, d);
  const bool f32 = desc->dtype == EARN_F32;
  if (f32) {
    if (d == 64) launch_rope_k<float, 64>(k, k_rot, cu_seqlens, positions, batch, total_tokens, p.hkv, p.rope, stream);
    else launch_rope_k<float, 128>(k, k_rot, cu_seqlens, positions, batch, total_tokens, p.hkv, p.rope, stream);
    dim3 grid((max_seqlen + 63) / 64, p.hq, batch);
    if (d == 64) hipLaunchKernelGGL((prefill_rows_kernel<float, 64>), grid, dim3(256), 0, stream, p);
    else hipLaunchKernelGGL((prefill_rows_kernel<float, 128>), grid, dim3(256), 0, stream, p);
  } else if (max_seqlen <= kTileKeys) {
    // register-only layers: every sequence is a single K/V tile
    if (d == 64) launch_rope_k<__bf16, 64>(k, k_rot, cu_seqlens, positions, batch, total_tokens, p.hkv, p.rope, stream);
    else launch_rope_k<__bf16, 128>(k, k_rot, cu_seqlens, positions, batch, total_tokens, p.hkv, p.rope, stream);
    p.n_qblk = 1;
    const long long pairs8 = ((long long)batch * p.hkv + kXcds - 1) / kXcds * kXcds;
    dim3 grid((unsigned)(pairs8 * (p.hq / p.hkv)), 1, 1);
    if (d == 64) hipLaunchKernelGGL((prefill_mfma_kernel<64, 1, 2, 1>), grid, dim3(128), 0, stream, p);
    else hipLaunchKernelGGL((prefill_mfma_kernel<128, 1, 2, 1>), grid, dim3(128), 0, stream, p);
  } else {
    if (d == 64) launch_rope_k<__bf16, 64>(k, k_rot, cu_seqlens, positions, batch, total_tokens, p.hkv, p.rope, stream);
    else launch_rope_k<__bf16, 128>(k, k_rot, cu_seqlens, positions, batch, total_tokens, p.hkv, p.rope, stream);
    static const int rows_env = getenv("EARN_PREFILL_ROWS") ? atoi(getenv("EARN_PREFILL_ROWS")) : 0;
    const int block_rows = rows_env ? rows_env : (max_seqlen <= 1280 ? 128 : 256);
    p.n_qblk = (max_seqlen + block_rows - 1) / block_rows;
    const long long pairs8 = ((long long)batch * p.hkv + kXcds - 1) / kXcds * kXcds;
    dim3 grid((unsigned)(pairs8 * p.n_qblk * (p.hq / p.hkv)), 1, 1);
    if (block_rows == 128) {
      if (d == 64) hipLaunchKernelGGL((prefill_mfma_kernel<64, 1, 4, EARN_PF_STAGES4>), grid, dim3(256), 0, stream, p);
      else hipLaunchKernelGGL((prefill_mfma_kernel<128, 1, 4, EARN_PF_STAGES4>), grid, dim3(256), 0, stream, p);
    } else {
      if (d == 64) hipLaunchKernelGGL((prefill_mfma_kernel<64, 1, 8, EARN_PF_STAGES8>), grid, dim3(512), 0, stream, p);
      else hipLaunchKernelGGL((prefill_mfma_kernel<128, 1, 8, EARN_PF_STAGES8>), grid, dim3(512), 0, stream, p);
    }
  }
  return hipGetLastError() == hipSuccess ? EARN_OK : EARN_ERR_HIP;
}

}  // namespace earn
