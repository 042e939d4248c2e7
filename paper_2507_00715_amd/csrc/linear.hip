// The dense projections around the attention (paper Appendix A.2: per layer, Q/K/V/output projections 8 L d_h d_a FLOPs
// per head and the feed-forward block 4 L d_h d_f) as one bf16 matrix-core GEMM kernel with two epilogues:
//   earn_qkv_rope_project  [rows, d_model] x [d_model, (Hq + 2 Hkv) d]: rotates the Q and K columns at each token's
//                          ORIGINAL position in the epilogue and writes Q, the rotated K (= the layer's key cache) and V
//                          straight into their [rows, heads, d] tensors, so the attention that follows needs no rotation
//                          pass of its own (it is then called with rotation switched off);
//   earn_linear            [rows, k] x [k, n] with an optional SiLU (output projection, feed-forward matrices).
//
// Tiling.  The kernel computes C^T = W^T X^T with v_mfma_f32_32x32x16_bf16, the same shape as the second product of the
// attention kernels (O^T = V^T P^T): the weight tile [64 k][128 n] plays V (kept in its natural layout, read with
// transposing LDS reads as the A operand), the activation tile [256 rows][64 k] supplies the B operand.  The transposing
// reads deliver the inner index of a 16-step in the order {4 hf .. 4 hf + 3, 8 + 4 hf .. 8 + 4 hf + 3} per half wave, so
// the activation fragments are read in the same order: two 8-byte reads instead of one 16-byte read.  A workgroup of 4 waves owns 256 rows x 128 columns; each wave 64 rows x 128 columns (8 accumulator
// tiles), so every weight fragment read feeds two MFMAs.  Tiles stream from global memory straight into a ring of three
// LDS stages (two tiles in flight); rows past the end of the activations read as zeros through the buffer descriptor.
// The accumulator layout gives a lane ONE row and, per 32-column block, columns 8 j + 4 hf + (0..3): the two elements of
// a rotary pair (e, e + d/2) sit in the same lane, two (d = 128) or one (d = 64) column blocks apart, so the rotation
// is lane-private.
#include <string.h>

#include "common.h"
#include "mfma_tiles.h"

namespace earn {

constexpr int kLinRows = 256, kLinCols = 128, kLinK = 64, kLinStages = 3, kLinWaves = 4;

struct LinearParams {
  const __bf16* x; const __bf16* w;
  int rows, k, n;
  // epilogue 0: out[row][col] = act(c);  epilogue 1: Q / K / V split with rotation
  __bf16* out; int activation;
  __bf16* q_out; __bf16* k_out; __bf16* v_out;
  const int32_t* cu; const int32_t* positions; int batch, hq, hkv, head_dim;
  RopeTable rope;
};

template <int EPI, int D>
__global__ __launch_bounds__(64 * kLinWaves, 1) void linear_kernel(LinearParams p) {
  __shared__ __bf16 smx[kLinStages][kLinRows * kLinK];   // 32 KB per stage
  __shared__ __bf16 smw[kLinStages][kLinK * kLinCols];   // 16 KB per stage
  const int lane = threadIdx.x % kWave, wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
  const int r32 = lane & 31, hf = lane >> 5;
  // column tiles vary fastest: the workgroups that run together share the activation rows in L2
  const int n_ct = (p.n + kLinCols - 1) / kLinCols;
  const int ct = blockIdx.x % n_ct, rt = blockIdx.x / n_ct;
  const int m0 = rt * kLinRows, n0 = ct * kLinCols;
  const int n_kt = p.k / kLinK;

  // ---- staging ----
  const int x_pitch = p.k * 2, w_pitch = p.n * 2;  // bytes
  const int rows_here = min(kLinRows, p.rows - m0);
  const u32x4 x_rsrc = raw_buffer(p.x + (long long)m0 * p.k, rows_here * x_pitch);
  // weights: rows kt*64.. of all columns from n0 on; the range ends with the matrix (columns past n are never stored)
  const long long w_bytes = (long long)p.k * w_pitch - (long long)n0 * 2;
  const u32x4 w_rsrc = raw_buffer(p.w + n0, (int)(w_bytes < 0x7fffffffLL ? w_bytes : 0x7fffffffLL));
  constexpr int XI = kLinRows * (kLinK / 8) / kWave / kLinWaves;   // 8 instructions per wave and tile
  constexpr int WI = kLinK * (kLinCols / 8) / kWave / kLinWaves;   // 4
  int x_voff[XI], w_voff[WI];
#pragma unroll
  for (int i = 0; i < XI; ++i) {
    const int row = 8 * (wave + kLinWaves * i) + lane / 8;          // 8 rows of 8 units per instruction
    x_voff[i] = row * x_pitch + ((lane % 8) ^ swz<64>(row)) * 16;
  }
#pragma unroll
  for (int i = 0; i < WI; ++i) {
    const int row = 4 * (wave + kLinWaves * i) + lane / 16;         // 4 rows of 16 units per instruction
    w_voff[i] = row * w_pitch + ((lane % 16) ^ swz<128>(row)) * 16;
  }
  const unsigned lds_x = (unsigned)(size_t)(lds_void_ptr)&smx[0][0], lds_w = (unsigned)(size_t)(lds_void_ptr)&smw[0][0];
  auto issue_tile = [&](int kt) {
    const unsigned sx = lds_x + (unsigned)((kt % kLinStages) * kLinRows * kLinK * 2);
    const unsigned sw = lds_w + (unsigned)((kt % kLinStages) * kLinK * kLinCols * 2);
#pragma unroll
    for (int i = 0; i < XI; ++i) dma16_to_lds(x_rsrc, sx + (unsigned)((wave + kLinWaves * i) * 1024), x_voff[i] + kt * (kLinK * 2));
#pragma unroll
    for (int i = 0; i < WI; ++i) dma16_to_lds(w_rsrc, sw + (unsigned)((wave + kLinWaves * i) * 1024), w_voff[i] + kt * kLinK * w_pitch);
  };
  constexpr int LPT = XI + WI;  // loads per wave and tile
  issue_tile(0);
  if (n_kt > 1) issue_tile(1);

  FragOffsets<128> fw;   // weight fragments: transposing reads on rows of 128 columns
  fw.init(lane);
  // activation fragments: row r32 of a 32-row block, inner indices 16 ks + {4 hf + (0..3), 8 + 4 hf + (0..3)}: the two
  // halves sit in the 16-byte chunks 2 ks and 2 ks + 1 (swizzled), 8 hf bytes in
  const int x_base = r32 * kLinK + 4 * hf, x_chunk = swz<64>(r32) << 3;
  f32x16 acc[2][4];
#pragma unroll
  for (int rb = 0; rb < 2; ++rb)
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[rb][db][i] = 0.f;

  for (int kt = 0; kt < n_kt; ++kt) {
    // tile kt has landed (loads complete in order: at most the next tile's are still in flight); behind the barrier nobody
    // reads tile kt-1 any more, whose stage tile kt+2 now fills
    if (kt + 1 < n_kt) wait_vmcnt<LPT>(); else wait_vmcnt<0>();
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    if (kt + 2 < n_kt) issue_tile(kt + 2);
    const __bf16* sx = smx[kt % kLinStages] + wave * 64 * kLinK;
    const __bf16* sw = smw[kt % kLinStages];
    bf16x8 xf[2][2], wf[2][4];
    auto fetch = [&](int ks, int buf) {
#pragma unroll
      for (int rb = 0; rb < 2; ++rb) {
        const bf16x4 a = *(const bf16x4*)(sx + rb * 32 * kLinK + x_base + (x_chunk ^ (ks << 4)));
        const bf16x4 b = *(const bf16x4*)(sx + rb * 32 * kLinK + x_base + (x_chunk ^ (ks << 4) ^ 8));
        xf[buf][rb] = __builtin_shufflevector(a, b, 0, 1, 2, 3, 4, 5, 6, 7);
      }
#pragma unroll
      for (int db = 0; db < 4; ++db) wf[buf][db] = read_v_fragment<128>(sw, fw, db, ks);
    };
    fetch(0, 0);
#pragma unroll
    for (int ks = 0; ks < kLinK / 16; ++ks) {
      if (ks + 1 < kLinK / 16) fetch(ks + 1, (ks + 1) & 1);   // the next step's fragments arrive behind this step's MFMAs
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int rb = 0; rb < 2; ++rb)
          acc[rb][db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[ks & 1][db], xf[ks & 1][rb], acc[rb][db], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
    }
  }

  // ---- epilogue: lane (r32, hf) holds, of row m0 + 64 wave + 32 rb + r32, columns n0 + 32 db + 8 j + 4 hf + (0..3) ----
#pragma unroll
  for (int rb = 0; rb < 2; ++rb) {
    const int m = m0 + wave * 64 + rb * 32 + r32;
    if (m >= p.rows) continue;
    if constexpr (EPI == 0) {
#pragma unroll
      for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const int col = n0 + 32 * db + 8 * j + 4 * hf;
          if (col >= p.n) continue;  // n is a multiple of 8: a group of 4 columns is inside or outside as a whole
          float c[4];
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            c[e] = acc[rb][db][4 * j + e];
            if (p.activation == 1) c[e] = c[e] / (1.f + __builtin_amdgcn_exp2f(-1.4426950408889634f * c[e]));  // SiLU
          }
          u32x2 w2 = {pack_bf16(c[0], c[1]), pack_bf16(c[2], c[3])};
          *(u32x2*)(p.out + (long long)m * p.n + col) = w2;
        }
    } else {
      constexpr int d = D;
      // (without rotation there is no position to look up, and neither array need exist)
      const float pos = !p.rope.enabled ? 0.f : (float)(p.positions ? p.positions[m] : m - p.cu[find_seq(p.cu, p.batch, m)]);
      // heads of this 128-column tile: one (d = 128) or two (d = 64); a rotary pair is db_step column blocks apart
      constexpr int db_step = d / 64;  // 2 or 1
#pragma unroll
      for (int hb = 0; hb < 2; ++hb) {           // d = 128: hb 0 only covers the tile; d = 64: hb = head within the tile
        if (d == 128 && hb == 1) break;
        const int col0 = n0 + hb * 64;           // first column of the head (d = 64) or of the tile (d = 128)
        if (col0 >= p.n) continue;
        const int head = col0 / d;               // over Q heads, then K heads, then V heads
        __bf16* dst;
        bool rotate;
        if (head < p.hq) { dst = p.q_out + ((long long)m * p.hq + head) * d; rotate = true; }
        else if (head < p.hq + p.hkv) { dst = p.k_out + ((long long)m * p.hkv + (head - p.hq)) * d; rotate = true; }
        else { dst = p.v_out + ((long long)m * p.hkv + (head - p.hq - p.hkv)) * d; rotate = false; }
        rotate = rotate && p.rope.enabled;
#pragma unroll
        for (int dl = 0; dl < 2; ++dl) {         // column blocks of the low half: d = 128: 2 of them; d = 64: 1
          if (d == 64 && dl == 1) break;
          const int db_lo = (d == 64 ? 2 * hb : 0) + dl, db_hi = db_lo + db_step;
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            float lo[4], hi[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              // the four column-block indices are compile-time constants in every unrolled instance
              const float a = db_lo == 0 ? acc[rb][0][4 * j + e] : db_lo == 1 ? acc[rb][1][4 * j + e] : acc[rb][2][4 * j + e];
              const float b = db_hi == 1 ? acc[rb][1][4 * j + e] : db_hi == 2 ? acc[rb][2][4 * j + e] : acc[rb][3][4 * j + e];
              float sn = 0.f, cs = 1.f;
              if (rotate) {
                const int pe = 32 * dl + 8 * j + 4 * hf + e;     // pair index inside the head
                sincos_turns_fast(rope_turns(pos, p.rope.hi[pe], p.rope.lo[pe]), &sn, &cs);
              }
              lo[e] = a * cs - b * sn;
              hi[e] = b * cs + a * sn;
            }
            const int c_lo = 32 * dl + 8 * j + 4 * hf;           // column inside the head
            u32x2 wl = {pack_bf16(lo[0], lo[1]), pack_bf16(lo[2], lo[3])}, wh = {pack_bf16(hi[0], hi[1]), pack_bf16(hi[2], hi[3])};
            *(u32x2*)(dst + c_lo) = wl;
            *(u32x2*)(dst + c_lo + d / 2) = wh;
          }
        }
      }
    }
  }
}

static int check_linear_shape(const char* who, long long rows, int k, int n) {
  if (rows <= 0 || k <= 0 || n <= 0) { set_error("%s: rows, k and n must be positive", who); return EARN_ERR_INVALID_ARG; }
  if (k % kLinK != 0 || n % 8 != 0) {
    set_error("%s: the inner dimension (%d) must be a multiple of 64 and the output width (%d) a multiple of 8", who, k, n);
    return EARN_ERR_UNSUPPORTED;
  }
  if ((long long)kLinRows * k * 2 >= (1ll << 31) || (long long)k * n * 2 >= (1ll << 31)) {
    set_error("%s: a %d x %d weight matrix or a 256-row block of %d columns exceeds the 2 GiB addressing range", who, k, n, k);
    return EARN_ERR_UNSUPPORTED;
  }
  if (rows > 0x7fffffffLL - kLinRows) { set_error("%s: too many rows", who); return EARN_ERR_UNSUPPORTED; }
  return EARN_OK;
}

int launch_linear(const void* x, const void* w, int rows, int k, int n, int activation, void* out, hipStream_t stream) {
  int rc = check_linear_shape("earn_linear", rows, k, n);
  if (rc != EARN_OK) return rc;
  LinearParams p;
  memset(&p, 0, sizeof(p));
  p.x = (const __bf16*)x; p.w = (const __bf16*)w; p.rows = rows; p.k = k; p.n = n; p.out = (__bf16*)out; p.activation = activation;
  const long long grid = (long long)((rows + kLinRows - 1) / kLinRows) * ((n + kLinCols - 1) / kLinCols);
  if (grid > 0x7fffffffLL) { set_error("earn_linear: grid too large"); return EARN_ERR_UNSUPPORTED; }
  hipLaunchKernelGGL((linear_kernel<0, 128>), dim3((unsigned)grid), dim3(64 * kLinWaves), 0, stream, p);
  return hipGetLastError() == hipSuccess ? EARN_OK : EARN_ERR_HIP;
}

int launch_qkv_rope_project(const earn_attn_desc* desc, const void* x, const void* w_qkv, int rows, int d_model,
                            const int32_t* cu_seqlens, const int32_t* positions, int batch, void* q_out, void* k_out,
                            void* v_out, hipStream_t stream) {
  const int n = (desc->n_q_heads + 2 * desc->n_kv_heads) * desc->head_dim;
  int rc = check_linear_shape("earn_qkv_rope_project", rows, d_model, n);
  if (rc != EARN_OK) return rc;
  LinearParams p;
  memset(&p, 0, sizeof(p));
  p.x = (const __bf16*)x; p.w = (const __bf16*)w_qkv; p.rows = rows; p.k = d_model; p.n = n;
  p.q_out = (__bf16*)q_out; p.k_out = (__bf16*)k_out; p.v_out = (__bf16*)v_out;
  p.cu = cu_seqlens; p.positions = positions; p.batch = batch;
  p.hq = desc->n_q_heads; p.hkv = desc->n_kv_heads; p.head_dim = desc->head_dim;
  p.rope = make_rope_table(desc->rope_base, desc->head_dim);
  const long long grid = (long long)((rows + kLinRows - 1) / kLinRows) * ((n + kLinCols - 1) / kLinCols);
  if (grid > 0x7fffffffLL) { set_error("earn_qkv_rope_project: grid too large"); return EARN_ERR_UNSUPPORTED; }
  if (desc->head_dim == 64) hipLaunchKernelGGL((linear_kernel<1, 64>), dim3((unsigned)grid), dim3(64 * kLinWaves), 0, stream, p);
  else hipLaunchKernelGGL((linear_kernel<1, 128>), dim3((unsigned)grid), dim3(64 * kLinWaves), 0, stream, p);
  return hipGetLastError() == hipSuccess ? EARN_OK : EARN_ERR_HIP;
}

}  // namespace earn
