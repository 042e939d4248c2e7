// Register compaction: X = [X_prefix; X_prompt; X_suffix] -> X' = [X_prefix; X_suffix] at the input of layer k
// (paper Section 3.2, Inference item 2).  A pure byte gather: HBM-bound, so the kernel is organised around the
// OUTPUT, which is contiguous: every lane owns 16-byte units of the compacted tensor, a wave stores 1 KiB of
// consecutive bytes per instruction, and the source of a unit is found with integer arithmetic only.  Source rows
// of one register group (h head rows, t tail rows) are consecutive in memory as well, so loads coalesce too.
#include "common.h"

namespace earn {

struct CompactArgs {
  const u32x4* src[EARN_MAX_COMPACT_TENSORS];
  u32x4* dst[EARN_MAX_COMPACT_TENSORS];
  unsigned int units_per_row[EARN_MAX_COMPACT_TENSORS];  // row_bytes / 16
  // first workgroup of every tensor in the one-dimensional grid (tensors differ in size: a grid row per tensor would
  // launch, for the small ones, mostly workgroups with nothing to do); [n_tensors] = first workgroup of the index part
  unsigned int first_block[EARN_MAX_COMPACT_TENSORS + 1];
};

constexpr int kCompactThreads = 256;
constexpr int kCompactUnroll = 4;  // 16-byte units per lane: 4 loads in flight before the first store
constexpr int kCompactBlocksPerWg = 4;  // blocks (kCompactThreads * kCompactUnroll units) a workgroup copies at most

// source row of compacted row m; a sequence shorter than h + t (a violated precondition) has its rows clamped into the
// sequence, an empty one yields -1 (no row)
__device__ __forceinline__ int source_row(const int32_t* __restrict__ cu, int total, int m, int r, int h, int t, int* pos) {
  int s = m / r, j = m - s * r;
  int b0, n;
  clamped_bounds(cu, s, total, total, b0, n);
  int p = j < h ? j : n - t + (j - h);
  p = max(min(p, n - 1), 0);
  *pos = p;
  return n > 0 ? b0 + p : -1;
}

__global__ __launch_bounds__(kCompactThreads) void compact_kernel(CompactArgs args, const int32_t* __restrict__ cu,
                                                                  int batch, int total, int h, int t, int rows_out,
                                                                  int32_t* __restrict__ idx_out,
                                                                  int32_t* __restrict__ pos_out,
                                                                  int32_t* __restrict__ cu_out, int n_tensors) {
  const int r = h + t;
  // tensor of this workgroup: the last one whose first workgroup is not beyond it (uniform binary search)
  int tensor = 0;
  {
    int lo = 0, hi = n_tensors + 1;  // answer in [lo, hi)
    while (hi - lo > 1) {
      const int mid = (lo + hi) >> 1;
      if (args.first_block[mid] <= blockIdx.x) lo = mid; else hi = mid;
    }
    tensor = lo;
  }
  const unsigned int block_in_tensor = blockIdx.x - args.first_block[tensor];
  if (tensor == n_tensors) {  // the workgroups behind the last tensor write the index outputs
    const unsigned int n_blocks = gridDim.x - args.first_block[n_tensors];
    for (int m = block_in_tensor * kCompactThreads + threadIdx.x; m < rows_out; m += n_blocks * kCompactThreads) {
      int pos;
      int idx = source_row(cu, total, m, r, h, t, &pos);
      if (idx_out) idx_out[m] = idx;
      if (pos_out) pos_out[m] = pos;
    }
    if (cu_out)
      for (int s = block_in_tensor * kCompactThreads + threadIdx.x; s <= batch; s += n_blocks * kCompactThreads)
        cu_out[s] = s * r;
    return;
  }
  const u32x4* __restrict__ src = args.src[tensor];
  u32x4* __restrict__ dst = args.dst[tensor];
  const unsigned int upr = args.units_per_row[tensor];
  const long long total_units = (long long)rows_out * upr;
  const long long stride = (long long)(args.first_block[tensor + 1] - args.first_block[tensor]) * kCompactThreads * kCompactUnroll;
  for (long long base = (long long)block_in_tensor * kCompactThreads * kCompactUnroll; base < total_units; base += stride) {
    u32x4 v[kCompactUnroll];
    long long u[kCompactUnroll];
#pragma unroll
    for (int i = 0; i < kCompactUnroll; ++i) {
      u[i] = base + (long long)i * kCompactThreads + threadIdx.x;
      if (u[i] < total_units) {
        int m = (int)(u[i] / upr);
        unsigned int off = (unsigned int)(u[i] - (long long)m * upr);
        int pos;
        long long row = source_row(cu, total, m, r, h, t, &pos);
        v[i] = row >= 0 ? __builtin_nontemporal_load(src + row * upr + off) : u32x4{0u, 0u, 0u, 0u};
      }
    }
#pragma unroll
    for (int i = 0; i < kCompactUnroll; ++i)
      if (u[i] < total_units) __builtin_nontemporal_store(v[i], dst + u[i]);
  }
}

// q_pos / gen_len of one decode step: a generated token sits at position n_s + step of its sequence
__global__ __launch_bounds__(256) void step_positions_kernel(const int32_t* __restrict__ cu,
                                                             const int32_t* __restrict__ stream_to_seq, int n_streams,
                                                             int batch, int step, int32_t* __restrict__ q_pos,
                                                             int32_t* __restrict__ gen_len) {
  const int u = blockIdx.x * 256 + threadIdx.x;
  if (u >= n_streams) return;
  const int s = stream_to_seq ? max(min(stream_to_seq[u], batch - 1), 0) : u;
  if (q_pos) q_pos[u] = cu[s + 1] - cu[s] + step;
  if (gen_len) gen_len[u] = step;
}

int launch_step_positions(const int32_t* cu, const int32_t* stream_to_seq, int n_streams, int batch, int step,
                          int32_t* q_pos, int32_t* gen_len, hipStream_t stream) {
  hipLaunchKernelGGL(step_positions_kernel, dim3((n_streams + 255) / 256), dim3(256), 0, stream, cu, stream_to_seq,
                     n_streams, batch, step, q_pos, gen_len);
  return hipGetLastError() == hipSuccess ? EARN_OK : EARN_ERR_HIP;
}

int launch_compact(int n_tensors, const void* const* src, void* const* dst, const int64_t* row_bytes,
                   const int32_t* cu_seqlens, int batch, int total_tokens, int h, int t, int32_t* idx_out,
                   int32_t* pos_out, int32_t* cu_out, hipStream_t stream) {
  CompactArgs args;
  const long long rows_out = (long long)batch * (h + t);
  const long long per_block = (long long)kCompactThreads * kCompactUnroll;
  // Blocks a workgroup copies one behind the other (grid stride apart).  More than one pays when few, long rows are
  // gathered (a workgroup's start — finding its tensor, the sequence bounds of its rows — then weighs as much as a
  // block's copy) and costs when many short ones are; the rule is fitted to measurements (1024 rows of 2-8 KB: 4 blocks
  // -14 %; 2048 rows of 8 KB: 2 blocks -2 %; 4096 rows of 0.5-3 KB: 4 blocks +10 %) and never leaves the GPU fewer than
  // a dozen workgroups per CU.
  long long total_blocks = 0;
  for (int i = 0; i < n_tensors; ++i) total_blocks += (rows_out * (row_bytes[i] / 16) + per_block - 1) / per_block;
  const int iters_env = tuning(kTuneCompactBlocks, 0);
  long long iters = iters_env > 0 ? iters_env : 4096 / (rows_out > 0 ? rows_out : 1);
  if (iters_env <= 0 && iters > total_blocks / 4096) iters = total_blocks / 4096;
  if (iters_env <= 0 && iters > kCompactBlocksPerWg) iters = kCompactBlocksPerWg;
  if (iters < 1) iters = 1;
  unsigned int blocks = 0;
  for (int i = 0; i < n_tensors; ++i) {
    args.src[i] = (const u32x4*)src[i];
    args.dst[i] = (u32x4*)dst[i];
    args.units_per_row[i] = (unsigned int)(row_bytes[i] / 16);
    const long long units = rows_out * (row_bytes[i] / 16);
    long long gx = (units + per_block * iters - 1) / (per_block * iters);
    if (gx < 1) gx = 1;
    if (gx > 8192) gx = 8192;  // grid-stride beyond this: 32 workgroups per CU
    args.first_block[i] = blocks;
    blocks += (unsigned int)gx;
  }
  args.first_block[n_tensors] = blocks;
  long long gi = (rows_out + kCompactThreads - 1) / kCompactThreads;  // index outputs
  if (gi < 1) gi = 1;
  if (gi > 256) gi = 256;
  dim3 grid(blocks + (unsigned)gi, 1, 1);
  hipLaunchKernelGGL(compact_kernel, grid, dim3(kCompactThreads), 0, stream, args, cu_seqlens, batch, total_tokens, h, t,
                     (int)rows_out, idx_out, pos_out, cu_out, n_tensors);
  return hipGetLastError() == hipSuccess ? EARN_OK : EARN_ERR_HIP;
}

}  // namespace earn
