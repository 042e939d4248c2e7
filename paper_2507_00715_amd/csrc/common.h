// Shared device/host helpers of libearn (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/earn.h"

namespace earn {

typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

constexpr int kWave = 64;
constexpr int kMaxHalfDim = 64;  // head_dim <= 128

// theta_e / (2 pi) split into a float pair (hi + lo) for every rotary pair e < d/2; filled on the host in fp64.
// With it a position p < 2^24 gives the turn count p*theta/(2 pi) modulo 1 to about 1e-7 without fp64 in the kernel.
struct RopeTable {
  float hi[kMaxHalfDim];
  float lo[kMaxHalfDim];
  int enabled;
};

// Query heads in the order the kernels serve them: slot c * gq + i is the i-th query head (ascending) that reads kv
// head c, gq = Hq / Hkv.  Without an explicit map (enabled == 0) slot and head coincide.
constexpr int kMaxMappedHeads = 128;
struct HeadMap {
  unsigned char q_of_slot[kMaxMappedHeads];
  int enabled;
};
__device__ __forceinline__ int head_of_slot(const HeadMap& m, int slot) { return m.enabled ? (int)m.q_of_slot[slot] : slot; }

void set_error(const char* fmt, ...);
RopeTable make_rope_table(float base, int head_dim);
// Fills `m` from desc->q_to_kv; EARN_OK, or an error (message set) for a map the kernels cannot serve.
int make_head_map(const earn_attn_desc* desc, HeadMap* m, const char* who);

// Several independent layers in one launch: grid row y works on layer y of per-layer-contiguous tensors.  Byte strides
// from one layer to the next; sequence bounds, positions and stream lists are shared by the layers.
struct DecodeLayers { int n_layers; long long q, kv_new, shared, gen, out; };
struct PrefillLayers { int n_layers; long long q, kv, out, k_rot, lse; };

// launch-shape overrides (earn_set_tuning); 0 = default
// Bounds of packed sequence s as the kernels use them: whatever cu holds, rows [b0, b0 + n) lie inside the `total` rows
// of the tensors and n within `max_len` (the length the launch was sized for).  A corrupt or not yet written cu then
// gives wrong values, never an access outside the tensors.
__device__ __forceinline__ void clamped_bounds(const int32_t* cu, int s, int total, int max_len, int& b0, int& n) {
  b0 = min(max(cu[s], 0), total);
  n = min(min(max(cu[s + 1] - b0, 0), total - b0), max_len);
}

constexpr int kXcds = 8;  // accelerator complex dies, each with a private L2; consecutive workgroup ids go to them in turn

enum Tuning { kTunePrefillBlockRows, kTuneDecMfmaMinLen, kTuneDecMfmaShortWgs, kTuneDecMfmaWgs, kTuneDecVecWgs,
              kTuneDecVecWaves, kTuneCompactBlocks, kTuneLinearTile, kTuneLinearSplits, kTuneCount };
int tuning(Tuning t, int dflt);

__device__ __forceinline__ float bf16_bits_to_f32(unsigned short b) { return __uint_as_float(((unsigned int)b) << 16); }
__device__ __forceinline__ float bf16_lo(unsigned int w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(unsigned int w) { return __uint_as_float(w & 0xffff0000u); }
__device__ __forceinline__ unsigned int pack_bf16(float a, float b) {
  f32x2 v = {a, b};
  bf16x2 r = __builtin_convertvector(v, bf16x2);  // v_cvt_pk_bf16_f32, round to nearest even
  return __builtin_bit_cast(unsigned int, r);
}

// Fraction of a turn of p * theta_e, in [0, 1).
// Contraction must stay off here: fusing `h - floor(h)` into fma(p, hi, -floor(h)) would count the residual twice.
__device__ __forceinline__ float rope_turns(float p, float hi, float lo) {
#pragma clang fp contract(off)
  float h = p * hi;
  float err = __builtin_fmaf(p, hi, -h);  // exact residual of the product
  float t = (h - __builtin_floorf(h)) + (err + p * lo);
  return t - __builtin_floorf(t);
}
// cos/sin of 2 pi t, t in [0,1): hardware v_cos/v_sin take turns directly (abs error ~1e-6).
__device__ __forceinline__ void sincos_turns_fast(float t, float* s, float* c) {
  *s = __builtin_amdgcn_sinf(t);
  *c = __builtin_amdgcn_cosf(t);
}
// precise variant for the fp32 path
__device__ __forceinline__ void sincos_turns_precise(float t, float* s, float* c) {
  float a = (t > 0.5f ? t - 1.0f : t) * 6.283185307179586f;
  sincosf(a, s, c);
}

// Sequence containing packed row `row`: largest s with cu[s] <= row (cu non-decreasing, cu[0] = 0).
__device__ __forceinline__ int find_seq(const int32_t* __restrict__ cu, int batch, int row) {
  int lo = 0, hi = batch;  // answer in [lo, hi)
  while (hi - lo > 1) {
    int mid = (lo + hi) >> 1;
    if (cu[mid] <= row) lo = mid; else hi = mid;
  }
  return lo;
}

}  // namespace earn
