// Pieces shared by the bf16 matrix-core attention kernels (prefill and decode): K/V tiles streamed from global memory
// straight into LDS, their swizzled layout, and the MFMA fragment reads.  gfx950 only.
#pragma once
#include "common.h"

namespace earn {

constexpr int kTileKeys = 64;    // keys per K/V tile in LDS

typedef __attribute__((address_space(3))) s16x4* lds_s16x4_ptr;
typedef __attribute__((address_space(3))) void* lds_void_ptr;

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

// One 16-byte-per-lane buffer load that lands directly in LDS: lane l's chunk goes to lds_addr + 16 l (lds_addr, the
// byte address inside LDS, is wave-uniform and travels in M0); a chunk outside the descriptor's range arrives as zeros.
// Written as an instruction rather than through the compiler's builtin on purpose: the compiler cannot tell which LDS
// reads such a load may alias and drains the whole vector-memory queue before every later LDS read, which would allow
// no more than a fraction of one tile's compute time for a tile to arrive.  Here the kernels keep the order themselves:
// a buffer is read only after a wait for the wave's own loads plus a workgroup barrier.  The kernels use M0 for
// nothing else.  (M0 cannot be named in the clobber list: the compiler treats it as a reserved register and warns that
// such a clobber is not honoured.  It only places values in M0 itself for instructions that read M0, none of which
// these kernels contain: no LDS-direct or GWS operations, no relative register indexing, no s_sendmsg.)  The wait
// state between the M0 write and the load is the one the compiler also leaves.
// The whole byte offset travels in `voff`: the descriptor's range check covers the vector offset, which is what turns
// rows past the end of the range into zeros; the scalar offset operand stays 0.
__device__ __forceinline__ void dma16_to_lds(u32x4 rsrc, unsigned lds_addr, int voff) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds"
               :
               : "s"(lds_addr), "v"(voff), "s"(rsrc)
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
// wait until at most N of this wave's vector-memory loads are in flight (they complete in order)
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
  static_assert(N >= 0 && N < 64);
  __builtin_amdgcn_s_waitcnt(0x0F70 | (N & 15) | ((N >> 4) << 14));
}
// wait until none of this wave's vector-memory loads is in flight, then meet the workgroup
__device__ __forceinline__ void drain_loads_and_barrier() {
  __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0)
  __syncthreads();
}

// Between rescales the exponentials are taken against a stale row maximum, so they can exceed 1; they are allowed to
// grow until a lane's partial row sum of one tile passes this limit.  A reference that is too low by D scales every
// weight, every sum and every output accumulator of the row by the same 2^D, a power of two: exact in fp32 and in the
// bf16 operands alike, and gone again in the final normalisation, so the result is the same function as long as
// nothing overflows.  2^40 per tile leaves fp32 eighty-odd binary orders for the sums over tiles and the products with
// V.  Rescaling touches every accumulator register of a lane and recomputes the tile, so doing it only when it is
// needed takes most vector-ALU work out of the key loop; with keys of very uneven scale (outlier rows) a tight limit
// would send tile after tile down the exact path.
constexpr float kSumLimit = 0x1p40f;

// max / sum of a value with its partner in the other half of the wave (lane ^ 32), without going through LDS
__device__ __forceinline__ float half_max(float x) {
  auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float half_sum(float x) {
  auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

// Row sums over ROUNDED probabilities, two per instruction (exact products with 1, accumulated in fp32): they are the
// weights the second product really applies, and it halves the additions.  acc += w.lo + w.hi.
// Written as instructions: the compiler's own dot builtin came out wrong inside these kernels (half of the words summed
// twice, the other half not at all).  What the compiler would otherwise look after is done by hand: a dot result may
// feed the next dot's accumulator at once, but any other vector instruction has to keep three wait states' distance,
// hence the s_nop in front of the addition that closes the two chains.
__device__ __forceinline__ void add_pair(float& acc, unsigned w) {
  const unsigned ones = 0x3f803f80u;  // (1.0, 1.0) in bf16
  asm("v_dot2c_f32_bf16 %0, %1, %2" : "+v"(acc) : "s"(ones), "v"(w));
}
__device__ __forceinline__ float add_chains(float s0, float s1) {
  float r;
  asm("s_nop 2\n\tv_add_f32 %0, %1, %2" : "=v"(r) : "v"(s0), "v"(s1));
  return r;
}

// ---- tile staging: global -> LDS directly ----
// A tile of ROWS rows is ROWS*UPR 16-byte units = ROWS*UPR/64 wave instructions per tensor (UPR = units per row);
// wave w issues instructions w, w+WAVES, ...  Instruction I fills LDS units [64 I, 64 I + 64): rows RPI*I + lane/UPR, chunk position
// lane%UPR.  Rows past the end of the sequence are outside the buffer descriptor and read as zeros (finite data for
// the masked tail, no clamping).
template <int D, int WAVES, int ROWS = kTileKeys>
struct TileStager {
  static constexpr int UPR = D / 8;
  static constexpr int NI = ROWS * UPR / kWave / WAVES;   // instructions per wave, tile and tensor
  static constexpr int RPI = kWave / UPR;                 // rows per instruction
  static_assert(NI >= 1 && NI * WAVES * kWave == ROWS * UPR);
  u32x4 k_rsrc, v_rsrc;
  int voff[NI];
  int row_bytes, wave;
  // Kg, Vg: row 0 of the range; n: rows in the range (rows beyond it read as zeros)
  __device__ __forceinline__ void init(const __bf16* Kg, const __bf16* Vg, int n, int hkv, int wave_, int lane) {
    row_bytes = hkv * D * 2;
    wave = wave_;
    const int seq_bytes = n > 0 ? (n - 1) * row_bytes + D * 2 : 0;
    k_rsrc = raw_buffer(Kg, seq_bytes);
    v_rsrc = raw_buffer(Vg, seq_bytes);
#pragma unroll
    for (int i = 0; i < NI; ++i) {
      const int row = RPI * (wave + WAVES * i) + lane / UPR;
      voff[i] = row * row_bytes + ((lane % UPR) ^ swz<D>(row)) * 16;
    }
  }
  // this wave's share of tile t of one tensor, into the tile buffer at LDS byte address lds_tile
  __device__ __forceinline__ void issue(const u32x4& rsrc, unsigned lds_tile, int t) const {
    const int toff = t * ROWS * row_bytes;
#pragma unroll
    for (int i = 0; i < NI; ++i) dma16_to_lds(rsrc, lds_tile + (unsigned)((wave + WAVES * i) * 1024), voff[i] + toff);
  }
};

// Per-lane LDS element offsets of the MFMA fragments inside a tile.  The swizzle is an XOR on the chunk index and the
// k-step / d-block enter the chunk index in bits the lane's own part leaves free, so every offset is one base XOR a
// constant: three registers instead of one per fragment.
template <int D>
struct FragOffsets {
  int k_base;     // K fragment of k-step ks: (k_base ^ (ks << 4)) + kb * 32 * D
  int v_base[2];  // V^T fragment of d block db: (v_base[h2] ^ (db << 5)) + kk * 16 * D ; h2 = second group of 4 keys (8 rows further)
  __device__ __forceinline__ void init(int lane) {
    const int r32 = lane & 31, hf = lane >> 5;
    k_base = r32 * D + ((hf ^ swz<D>(r32)) << 3);
#pragma unroll
    for (int h2 = 0; h2 < 2; ++h2) {
      const int row = 4 * hf + 8 * h2 + ((lane & 15) >> 2);
      const int chunk = 2 * ((lane >> 4) & 1) + ((lane & 3) >> 1);
      v_base[h2] = row * D + ((chunk ^ swz<D>(row)) << 3) + 4 * (lane & 1);
    }
  }
  __device__ __forceinline__ int k(int ks) const { return k_base ^ (ks << 4); }
  __device__ __forceinline__ int v(int db, int h2) const { return v_base[h2] ^ (db << 5); }
};
// V^T fragment (d block db, 16-key step kk) of the V tile at smv: two transposing reads, 4 keys each
template <int D>
__device__ __forceinline__ bf16x8 read_v_fragment(const __bf16* smv, const FragOffsets<D>& fo, int db, int kk) {
  typedef short s16x8 __attribute__((ext_vector_type(8)));
  s16x4 v0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(smv + fo.v(db, 0) + kk * 16 * D));
  s16x4 v1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(smv + fo.v(db, 1) + kk * 16 * D));
  return __builtin_bit_cast(bf16x8, (s16x8)__builtin_shufflevector(v0, v1, 0, 1, 2, 3, 4, 5, 6, 7));
}

}  // namespace earn
