// The dense projections around the attention (paper Appendix A.2: per layer, Q/K/V/output projections 8 L d_h d_a FLOPs
// per head and the feed-forward block 4 L d_h d_f) as one bf16 matrix-core GEMM kernel with two epilogues:
//   earn_qkv_rope_project  [rows, d_model] x [(Hq + 2 Hkv) d, d_model]^T: rotates the Q and K columns at each token's
//                          ORIGINAL position in the epilogue and writes Q, the rotated K (= the layer's key cache) and V
//                          straight into their [rows, heads, d] tensors, so the attention that follows needs no rotation
//                          pass of its own (it is then called with rotation switched off);
//   earn_linear            [rows, k] x [n, k]^T with an optional SiLU (output projection, feed-forward matrices).
// Weights are [outputs][inputs], the inner dimension contiguous (the layout checkpoints store them in): activations and
// weights then both deliver MFMA fragments as plain 16-byte LDS reads, 8 consecutive inner indices per lane.
//
// Tiling.  The kernel computes C^T = W X^T with v_mfma_f32_32x32x16_bf16: the weight tile [128 n][64 k] supplies the A
// operand, the activation tile [256 rows][64 k] the B operand.  A workgroup of 4 waves owns 256 rows x 128 columns; each
// wave 64 rows x 128 columns (8 accumulator tiles), so every weight fragment read feeds two MFMAs.  Tiles stream from
// global memory straight into a ring of three LDS stages (two tiles in flight); rows past the end of the activations
// and weight rows past the last output read as zeros through the buffer descriptors.
// The accumulator layout gives a lane ONE row and, per 32-column block, columns 8 j + 4 hf + (0..3): the two elements of
// a rotary pair (e, e + d/2) sit in the same lane, two (d = 128) or one (d = 64) column blocks apart, so the rotation
// is lane-private.
#include <string.h>

#include <algorithm>

#include "common.h"
#include "mfma_tiles.h"

namespace earn {

constexpr int kLinRows = 256;  // rows of a workgroup's tile
constexpr int kLinKMultiple = 64;  // the inner dimension must be a multiple of this

// chunk swizzle of a tile whose rows hold KT inner indices (KT / 8 chunks of 16 bytes): 64 -> the attention tiles' own
// pattern; 32 -> four rows share 256 bytes of LDS, and rows 4 apart must land on different chunk positions
template <int KT>
__device__ __forceinline__ int lin_swz(int row) {
  if constexpr (KT == 64) return swz<64>(row);
  else return (row >> 2) & 3;
}

struct LinearParams {
  const __bf16* x; const __bf16* w;
  int rows, k, n;
  // epilogue 0: out[row][col] = act(c);  epilogue 1: Q / K / V split with rotation
  __bf16* out; int activation;
  __bf16* q_out; __bf16* k_out; __bf16* v_out;
  const int32_t* cu; const int32_t* positions; int batch, hq, hkv, head_dim;
  // inner dimension split over grid rows (few output rows: too few tiles to fill the GPU otherwise): split z takes
  // K-tiles [z * split_tiles, (z + 1) * split_tiles) and writes its fp32 sums to partial[z][rows][n]; a second kernel
  // adds the splits and applies the epilogue.  n_split == 1: no partials, the kernel finishes the outputs itself.
  float* partial; int n_split, split_tiles;
  int patch_rows, patch_cols;  // tiles an XCD works on together (see the kernel's workgroup -> tile mapping)
  RopeTable rope;
};

// RB: 32-row blocks per wave (the tile's 256 rows are shared by 8 / RB row groups of waves); WC: 128-column groups of
// the tile (waves = 8 / RB x WC); KT: inner indices per LDS stage; STAGES: LDS ring depth (STAGES - 1 tiles in flight)
template <int EPI, int D, int RB, int WC, int KT, int STAGES>
__global__ __launch_bounds__(64 * (8 / RB) * WC, 1) void linear_kernel(LinearParams p) {
  constexpr int WR = 8 / RB;
  constexpr int kLinCols = 128 * WC, kLinWaves = WR * WC, kLinStages = STAGES, kLinK = KT;
  constexpr int CPR = KT / 8, RPI = kWave / CPR;  // chunks per tile row, tile rows per load instruction
  __shared__ __bf16 smx[kLinStages][kLinRows * kLinK];   // 32 KB per stage
  __shared__ __bf16 smw[kLinStages][kLinCols * kLinK];   // 16 KB per stage and column group
  const int lane = threadIdx.x % kWave, wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
  const int wr = wave % WR, wc = wave / WR;              // this wave's 32 RB rows and 128 columns of the tile
  const int r32 = lane & 31, hf = lane >> 5;
  // Workgroup -> tile.  Consecutive workgroup ids go to the 8 XCDs in turn, each with an L2 of its own and 32 CUs: the
  // 32 workgroups an XCD runs side by side are given a patch of patch_rows x patch_cols (4 x 8, host's choice) tiles, so
  // that the XCD fetches 4 activation and 8 weight tile slices per step for 32 workgroups instead of one of each per
  // workgroup.  (Few tiles: smaller patches, down to single tiles, so that every XCD gets some.)
  const int n_ct = (p.n + kLinCols - 1) / kLinCols, n_rt = (p.rows + kLinRows - 1) / kLinRows;
  // The tile rows and columns are dealt to the patches in equal shares (a patch is up to 4 x 8 tiles, not exactly):
  // patches of equal work keep the XCDs, which take them in turn, busy for the same time.
  const int n_pc = (n_ct + p.patch_cols - 1) / p.patch_cols, n_pr = (n_rt + p.patch_rows - 1) / p.patch_rows;
  const int slots = p.patch_rows * p.patch_cols;
  const int xcd = blockIdx.x % kXcds, i_in_xcd = blockIdx.x / kXcds;
  const int patch = (i_in_xcd / slots) * kXcds + xcd, within = i_in_xcd % slots;
  const int pr = patch / n_pc, pc = patch % n_pc;
  if (pr >= n_pr) return;
  const int rt = (int)((long long)pr * n_rt / n_pr) + within % p.patch_rows;
  const int ct = (int)((long long)pc * n_ct / n_pc) + within / p.patch_rows;
  if (rt >= (int)((long long)(pr + 1) * n_rt / n_pr) || ct >= (int)((long long)(pc + 1) * n_ct / n_pc)) return;
  const int m0 = rt * kLinRows, n0_wg = ct * kLinCols, n0 = n0_wg + 128 * wc;
  const int kt0 = blockIdx.y * p.split_tiles;                    // first K-tile of this workgroup's share of the inner dimension
  const int n_kt = min(p.k / kLinK - kt0, p.split_tiles);
  static_assert(STAGES >= 2 && STAGES <= 5);

  // ---- staging ----
  const int x_pitch = p.k * 2;  // bytes, of activation and weight rows alike
  const int rows_here = min(kLinRows, p.rows - m0), cols_here = min(kLinCols, p.n - n0_wg);
  const u32x4 x_rsrc = raw_buffer(p.x + (long long)m0 * p.k, rows_here * x_pitch);
  const u32x4 w_rsrc = raw_buffer(p.w + (long long)n0_wg * p.k, cols_here * x_pitch);
  constexpr int XI = kLinRows * (kLinK / 8) / kWave / kLinWaves;   // instructions per wave and tile
  constexpr int WI = kLinCols * (kLinK / 8) / kWave / kLinWaves;
  static_assert(XI >= 1 && WI >= 1);
  int x_voff[XI], w_voff[WI];
#pragma unroll
  for (int i = 0; i < XI; ++i) {
    const int row = RPI * (wave + kLinWaves * i) + lane / CPR;
    x_voff[i] = row * x_pitch + ((lane % CPR) ^ lin_swz<KT>(row)) * 16;
  }
#pragma unroll
  for (int i = 0; i < WI; ++i) {
    const int row = RPI * (wave + kLinWaves * i) + lane / CPR;
    w_voff[i] = row * x_pitch + ((lane % CPR) ^ lin_swz<KT>(row)) * 16;
  }
  const unsigned lds_x = (unsigned)(size_t)(lds_void_ptr)&smx[0][0], lds_w = (unsigned)(size_t)(lds_void_ptr)&smw[0][0];
  constexpr int LPT = XI + WI;  // loads per wave and tile
  auto k_byte = [&](int kt) { return (kt0 + kt) * (kLinK * 2); };  // byte offset of K-tile kt inside a row
  // load j (0 .. LPT-1) of this wave's share of tile kt
  auto issue_part = [&](int kt, int j) {
    const unsigned sx = lds_x + (unsigned)((kt % kLinStages) * kLinRows * kLinK * 2);
    const unsigned sw = lds_w + (unsigned)((kt % kLinStages) * kLinK * kLinCols * 2);
#pragma unroll
    for (int i = 0; i < XI; ++i)
      if (j == i) dma16_to_lds(x_rsrc, sx + (unsigned)((wave + kLinWaves * i) * 1024), x_voff[i] + k_byte(kt));
#pragma unroll
    for (int i = 0; i < WI; ++i)
      if (j == XI + i) dma16_to_lds(w_rsrc, sw + (unsigned)((wave + kLinWaves * i) * 1024), w_voff[i] + k_byte(kt));
  };
  auto issue_tile = [&](int kt) {
#pragma unroll
    for (int j = 0; j < LPT; ++j) issue_part(kt, j);
  };
#pragma unroll
  for (int t = 0; t < kLinStages - 1; ++t)
    if (t < n_kt) issue_tile(t);

  // fragments of both tiles: row r32 of a 32-row block, inner indices 16 ks + 8 hf + (0..7), i.e. the 16-byte chunk
  // 2 ks + hf of the row (swizzled)
  const int frag_base = r32 * KT + ((hf ^ lin_swz<KT>(r32)) << 3);
  auto frag = [&](int ks) { return frag_base ^ (ks << 4); };
  f32x16 acc[RB][4];
#pragma unroll
  for (int rb = 0; rb < RB; ++rb)
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[rb][db][i] = 0.f;

  // Tile kt has landed when at most the loads of the later tiles already issued are still in flight (they complete in
  // order); behind the barrier nobody reads tile kt-1 any more, whose stage the next tile to be requested fills.
  auto await_tile = [&](int kt) {
    const int later = min(kLinStages - 2, n_kt - 1 - kt);
    if (later >= 3) wait_vmcnt<3 * LPT>(); else if (later == 2) wait_vmcnt<2 * LPT>(); else if (later == 1) wait_vmcnt<LPT>(); else wait_vmcnt<0>();
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_waitcnt(0xC07F);  // lgkmcnt(0): this wave's fragment reads of the tile before are complete
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
  };
  bf16x8 xf[2][RB], wf[2][4];
  // fragment f (0 .. RB + 3: the activation blocks, then the weight blocks) of step ks of tile kt
  auto fetch_one = [&](int kt, int ks, int buf, int f) {
    const __bf16* sx = smx[kt % kLinStages] + wr * (32 * RB) * kLinK;
    const __bf16* sw = smw[kt % kLinStages] + wc * 128 * kLinK;
#pragma unroll
    for (int rb = 0; rb < RB; ++rb)
      if (f == rb) xf[buf][rb] = *(const bf16x8*)(sx + rb * 32 * kLinK + frag(ks));
#pragma unroll
    for (int db = 0; db < 4; ++db)
      if (f == RB + db) wf[buf][db] = *(const bf16x8*)(sw + db * 32 * kLinK + frag(ks));
  };
  auto fetch = [&](int kt, int ks, int buf) {
#pragma unroll
    for (int f = 0; f < RB + 4; ++f) fetch_one(kt, ks, buf, f);
  };
  // One step's products.  The loads of the tile that may be requested since the last barrier (stage_kt; none if past
  // the end) are dealt out between the MFMAs, one behind every second one, `call` counting the steps since that barrier:
  // requesting them takes issue cycles, which are free while the matrix core works off the product just issued.
  // next_ks >= 0: the fragments of step next_ks of tile next_kt are requested into the other buffer on the way, one
  // behind each of the first MFMAs
  auto multiply = [&](int buf, int call, int stage_kt, int next_kt, int next_ks) {
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
      for (int rb = 0; rb < RB; ++rb) {
        acc[rb][db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[buf][db], xf[buf][rb], acc[rb][db], 0, 0, 0);
        const int m = db * RB + rb;
        if (next_ks >= 0 && m < RB + 4) fetch_one(next_kt, next_ks, buf ^ 1, m);
        if ((m & 1) && stage_kt < n_kt) issue_part(stage_kt, call * (2 * RB) + m / 2);
        __builtin_amdgcn_sched_barrier(0);
      }
  };
  // The barrier between two tiles sits in front of the LAST step's products of the tile that ends: its fragments are in
  // registers by then, and its MFMAs run while the first fragments of the next tile make their way out of LDS (right
  // behind a barrier all waves ask for fragments at once).
  constexpr int KS = kLinK / 16;
  static_assert(KS % 2 == 0);  // the fragment buffers alternate: step 0 of every tile uses buffer 0
  static_assert(KS * 2 * RB >= LPT, "a tile's loads are all requested within one tile's steps");
  static_assert(4 * RB >= RB + 4, "a step has at least as many MFMAs as fragments");
  await_tile(0);
#pragma unroll
  for (int j = 0; j < 2 * RB; ++j)
    if (kLinStages - 1 < n_kt) issue_part(kLinStages - 1, j);  // the share of the step that precedes the loop
  fetch(0, 0, 0);
  for (int kt = 0; kt < n_kt; ++kt) {
#pragma unroll
    for (int ks = 0; ks + 1 < KS; ++ks)   // step ks multiplies buffer ks & 1 while the other one takes step ks + 1
      multiply(ks & 1, ks + 1, kt + kLinStages - 1, kt, ks + 1);
    if (kt + 1 < n_kt) {
      await_tile(kt + 1);
      fetch(kt + 1, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
    }
    multiply((KS - 1) & 1, 0, kt + kLinStages, 0, -1);  // (behind the last tile there is no barrier and nothing to request)
  }

  // ---- epilogue: lane (r32, hf) holds, of row m0 + 64 wave + 32 rb + r32, columns n0 + 32 db + 8 j + 4 hf + (0..3) ----
#pragma unroll
  for (int rb = 0; rb < RB; ++rb) {
    const int m = m0 + wr * (32 * RB) + rb * 32 + r32;
    if (m >= p.rows) continue;
    if (p.n_split > 1) {  // this split's sums, as they are
      float* dst = p.partial + ((long long)blockIdx.y * p.rows + m) * p.n;
#pragma unroll
      for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const int col = n0 + 32 * db + 8 * j + 4 * hf;
          if (col < p.n) *(f32x4*)(dst + col) = f32x4{acc[rb][db][4 * j], acc[rb][db][4 * j + 1], acc[rb][db][4 * j + 2], acc[rb][db][4 * j + 3]};
        }
      continue;
    }
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

// Second kernel of a split product: adds the splits' sums and applies the epilogue.  One thread per row and group of 4
// columns (EPI 0) or per row, head and group of 4 rotary pairs (EPI 1: the 4 low-half columns and their partners d/2 on).
template <int EPI>
__global__ __launch_bounds__(256) void linear_reduce_kernel(LinearParams p) {
  const long long t = (long long)blockIdx.x * 256 + threadIdx.x;
  const long long slice = (long long)p.rows * p.n;
  auto sum4 = [&](long long at) {
    f32x4 a = *(const f32x4*)(p.partial + at);
    for (int z = 1; z < p.n_split; ++z) {
      const f32x4 b = *(const f32x4*)(p.partial + z * slice + at);
      a[0] += b[0]; a[1] += b[1]; a[2] += b[2]; a[3] += b[3];
    }
    return a;
  };
  if constexpr (EPI == 0) {
    const int groups = p.n / 4;
    if (t >= (long long)p.rows * groups) return;
    const int m = (int)(t / groups), col = (int)(t % groups) * 4;
    f32x4 c = sum4((long long)m * p.n + col);
    if (p.activation == 1) {
#pragma unroll
      for (int e = 0; e < 4; ++e) c[e] = c[e] / (1.f + __builtin_amdgcn_exp2f(-1.4426950408889634f * c[e]));  // SiLU
    }
    *(u32x2*)(p.out + (long long)m * p.n + col) = u32x2{pack_bf16(c[0], c[1]), pack_bf16(c[2], c[3])};
  } else {
    const int d = p.head_dim, per_head = d / 8, heads = p.hq + 2 * p.hkv;
    if (t >= (long long)p.rows * heads * per_head) return;
    const int g = (int)(t % per_head), head = (int)((t / per_head) % heads), m = (int)(t / ((long long)per_head * heads));
    const long long at = (long long)m * p.n + (long long)head * d + 4 * g;
    const f32x4 a = sum4(at), b = sum4(at + d / 2);
    __bf16* dst;
    bool rotate = p.rope.enabled;
    if (head < p.hq) dst = p.q_out + ((long long)m * p.hq + head) * d;
    else if (head < p.hq + p.hkv) dst = p.k_out + ((long long)m * p.hkv + (head - p.hq)) * d;
    else { dst = p.v_out + ((long long)m * p.hkv + (head - p.hq - p.hkv)) * d; rotate = false; }
    float lo[4], hi[4];
    const float pos = !rotate ? 0.f : (float)(p.positions ? p.positions[m] : m - p.cu[find_seq(p.cu, p.batch, m)]);
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      float sn = 0.f, cs = 1.f;
      if (rotate) sincos_turns_fast(rope_turns(pos, p.rope.hi[4 * g + e], p.rope.lo[4 * g + e]), &sn, &cs);
      lo[e] = a[e] * cs - b[e] * sn;
      hi[e] = b[e] * cs + a[e] * sn;
    }
    *(u32x2*)(dst + 4 * g) = u32x2{pack_bf16(lo[0], lo[1]), pack_bf16(lo[2], lo[3])};
    *(u32x2*)(dst + 4 * g + d / 2) = u32x2{pack_bf16(hi[0], hi[1]), pack_bf16(hi[2], hi[3])};
  }
}

// Splits of the inner dimension for a product with few output rows.  Without a split such a product has one workgroup
// per 128 columns, a fraction of the CUs, each streaming its slice of the weights alone at the rate one workgroup's few
// tiles in flight allow; with z splits there are z times as many, at the price of z * rows * n fp32 partial sums written
// and read again.  The workgroups hold most of a CU's LDS (one per CU at a time), so z is the largest count that still
// fits ONE round of 256 workgroups; at least 4 K-tiles per split, the partial sums no larger than the weights, and
// within the workspace given.  Measured (160 rows, k = 4096): 4096 outputs 56 -> 23 us, 6144 outputs 57 -> 28 us; with
// 86 or more tiles (11008 outputs) the unsplit launch already draws what this access pattern gets from HBM (128-byte
// pieces of rows 8 KB apart: about 1.5 TB/s) and splitting only adds the partial sums.
static int linear_splits(long long rows, int k, int n, size_t workspace_bytes) {
  const long long tiles = ((rows + kLinRows - 1) / kLinRows) * ((n + 127) / 128);
  long long z = tiles <= 64 ? 256 / tiles : (tiles <= 128 && k >= 8192 ? 2 : 1);
  z = std::min<long long>(z, k / 64 / 4);
  z = std::min<long long>(z, k / (2 * rows));
  z = std::min<long long>(z, 16);
  const int forced = tuning(kTuneLinearSplits, 0);
  if (forced > 0) z = std::min<long long>(forced, std::max(1, k / 64));
  while (z > 1 && (size_t)z * rows * n * sizeof(float) > workspace_bytes) --z;
  return (int)std::max<long long>(z, 1);
}
size_t linear_workspace_bytes(long long rows, int k, int n) {
  if (rows <= 0 || k <= 0 || n <= 0 || k % kLinKMultiple != 0) return 0;
  const int z = linear_splits(rows, k, n, ~(size_t)0);
  return z > 1 ? ((size_t)z * rows * n * sizeof(float) + 255) / 256 * 256 : 0;
}

static int check_linear_shape(const char* who, long long rows, int k, int n) {
  if (rows <= 0 || k <= 0 || n <= 0) { set_error("%s: rows, k and n must be positive", who); return EARN_ERR_INVALID_ARG; }
  if (k % kLinKMultiple != 0 || n % 8 != 0) {
    set_error("%s: the inner dimension (%d) must be a multiple of 64 and the output width (%d) a multiple of 8", who, k, n);
    return EARN_ERR_UNSUPPORTED;
  }
  if ((long long)kLinRows * k * 2 >= (1ll << 31)) {
    set_error("%s: a 256-row block of %d columns exceeds the 2 GiB addressing range", who, k);
    return EARN_ERR_UNSUPPORTED;
  }
  if (rows > 0x7fffffffLL - kLinRows) { set_error("%s: too many rows", who); return EARN_ERR_UNSUPPORTED; }
  return EARN_OK;
}

// template arguments and threads of the 256 x 256 form
#define LIN_WIDE 2, 2, 64, 2
#define LIN_WIDE_THREADS 512
// 256 x 256 tiles (8 waves, two per SIMD, two LDS stages) or 256 x 128 tiles (4 waves, three stages), whichever needs
// less time by a simple count: one workgroup per CU at a time, rounds of 256 workgroups, a narrow tile taking about 0.62
// of a wide one's time (measured on large matrices: half the products at a lower rate).  Large matrices take the wide
// tile; a few hundred rows take whichever fills the last round better.
static bool linear_wide_tile(long long rows, int n) {
  const int set = tuning(kTuneLinearTile, 0);
  if (set == 1) return false;
  if (set == 2) return true;
  const long long n_rt = (rows + kLinRows - 1) / kLinRows;
  const long long wide = n_rt * ((n + 255) / 256), narrow = n_rt * ((n + 127) / 128);
  const int cus = 256;
  return (double)((wide + cus - 1) / cus) <= 0.62 * (double)((narrow + cus - 1) / cus);
}

// workgroups: whole patches, a multiple of 8 of them (one per XCD and round); workgroups outside the matrix leave at once
// Patch shape: 4 x 8 tiles when that leaves every XCD at least two patches, else the largest of 2 x 4, 1 x 2 and single
// tiles that does.
static long long linear_grid(long long rows, int n, int cols, int* patch_rows, int* patch_cols) {
  const long long n_rt = (rows + kLinRows - 1) / kLinRows, n_ct = (n + cols - 1) / cols;
  static const int shapes[4][2] = {{4, 8}, {2, 4}, {1, 2}, {1, 1}};
  long long patches = 0;
  for (int i = 0; i < 4; ++i) {
    *patch_rows = shapes[i][0]; *patch_cols = shapes[i][1];
    patches = ((n_rt + *patch_rows - 1) / *patch_rows) * ((n_ct + *patch_cols - 1) / *patch_cols);
    if (patches >= 2 * kXcds) break;
  }
  return (patches + kXcds - 1) / kXcds * kXcds * (*patch_rows * *patch_cols);
}

// tile shape, splits and grid of one product; fills the split fields of p
struct LinearLaunch { bool wide; int splits; dim3 grid; };
static int plan_linear(const char* who, LinearParams& p, void* workspace, size_t workspace_bytes, LinearLaunch* out) {
  const int splits = workspace ? linear_splits(p.rows, p.k, p.n, workspace_bytes) : 1;
  const bool wide = splits == 1 && linear_wide_tile(p.rows, p.n);
  const long long grid = linear_grid(p.rows, p.n, wide ? 256 : 128, &p.patch_rows, &p.patch_cols);
  if (grid > 0x7fffffffLL) { set_error("%s: grid too large", who); return EARN_ERR_UNSUPPORTED; }
  const int k_tiles = p.k / 64;
  p.n_split = splits;
  p.split_tiles = (k_tiles + splits - 1) / splits;
  p.n_split = (k_tiles + p.split_tiles - 1) / p.split_tiles;  // no empty split
  p.partial = p.n_split > 1 ? (float*)workspace : nullptr;
  out->wide = wide; out->splits = p.n_split; out->grid = dim3((unsigned)grid, (unsigned)p.n_split, 1);
  return EARN_OK;
}

int launch_linear(const void* x, const void* w, int rows, int k, int n, int activation, void* out, void* workspace,
                  size_t workspace_bytes, hipStream_t stream) {
  int rc = check_linear_shape("earn_linear", rows, k, n);
  if (rc != EARN_OK) return rc;
  LinearParams p;
  memset(&p, 0, sizeof(p));
  p.x = (const __bf16*)x; p.w = (const __bf16*)w; p.rows = rows; p.k = k; p.n = n; p.out = (__bf16*)out; p.activation = activation;
  LinearLaunch ll;
  if ((rc = plan_linear("earn_linear", p, workspace, workspace_bytes, &ll)) != EARN_OK) return rc;
  if (ll.wide) hipLaunchKernelGGL((linear_kernel<0, 128, LIN_WIDE>), ll.grid, dim3(LIN_WIDE_THREADS), 0, stream, p);
  else hipLaunchKernelGGL((linear_kernel<0, 128, 2, 1, 64, 3>), ll.grid, dim3(256), 0, stream, p);
  if (ll.splits > 1) {
    const long long threads = (long long)rows * (n / 4);
    hipLaunchKernelGGL((linear_reduce_kernel<0>), dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, stream, p);
  }
  return hipGetLastError() == hipSuccess ? EARN_OK : EARN_ERR_HIP;
}

int launch_qkv_rope_project(const earn_attn_desc* desc, const void* x, const void* w_qkv, int rows, int d_model,
                            const int32_t* cu_seqlens, const int32_t* positions, int batch, void* q_out, void* k_out,
                            void* v_out, void* workspace, size_t workspace_bytes, hipStream_t stream) {
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
  LinearLaunch ll;
  if ((rc = plan_linear("earn_qkv_rope_project", p, workspace, workspace_bytes, &ll)) != EARN_OK) return rc;
  if (desc->head_dim == 64) {
    if (ll.wide) hipLaunchKernelGGL((linear_kernel<1, 64, LIN_WIDE>), ll.grid, dim3(LIN_WIDE_THREADS), 0, stream, p);
    else hipLaunchKernelGGL((linear_kernel<1, 64, 2, 1, 64, 3>), ll.grid, dim3(256), 0, stream, p);
  } else {
    if (ll.wide) hipLaunchKernelGGL((linear_kernel<1, 128, LIN_WIDE>), ll.grid, dim3(LIN_WIDE_THREADS), 0, stream, p);
    else hipLaunchKernelGGL((linear_kernel<1, 128, 2, 1, 64, 3>), ll.grid, dim3(256), 0, stream, p);
  }
  if (ll.splits > 1) {
    const long long threads = (long long)rows * (desc->n_q_heads + 2 * desc->n_kv_heads) * (desc->head_dim / 8);
    hipLaunchKernelGGL((linear_reduce_kernel<1>), dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, stream, p);
  }
  return hipGetLastError() == hipSuccess ? EARN_OK : EARN_ERR_HIP;
}

}  // namespace earn
