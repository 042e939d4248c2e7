// Beam-search bookkeeping around the decode step (paper Appendix, implementation details: inference uses beam search
// with beam size 20).  Three pieces, none of which touches a K/V byte:
//   beam_topk      per sequence, the W best of the W * V candidates  score(beam w) + logprob(w, token t), ordered by
//                  (score descending, candidate index ascending): each winner names its parent beam and its token;
//   beam_reorder   the new beams' ancestor table: which physical stream's cache slot holds each earlier generated row.
//                  The decode kernels read generated rows through this table (DecodeParams::gen_src), so a beam step
//                  moves W * step integers per sequence instead of copying W * step K/V rows in every layer;
// Selection is exact and deterministic: candidates are compared as (score, index) pairs in a total order, and pick i is
// the largest pair strictly below pick i-1.
#include "common.h"

namespace earn {

constexpr int kTopkThreads = 256;
constexpr int kTopkChunk = 8192;   // candidates one workgroup holds in LDS (32 KB of scores)
constexpr int kTopkMaxBeams = 64;

struct Cand { float v; int i; };
// a before b in selection order: larger score first, lower index first among equals
__device__ __forceinline__ bool cand_before(const Cand& a, const Cand& b) { return a.v > b.v || (a.v == b.v && a.i < b.i); }

// The k best of n candidates (scores sc[j], indices ix ? ix[j] : base + j; both arrays in LDS), in selection order, by k
// rounds of "best candidate strictly after the previous pick".  All threads of the workgroup call it; thread 0 writes
// pick r to out_v[r] / out_i[r] (index -1 when fewer than r + 1 candidates exist).
__device__ void select_topk(const float* sc, const int* ix, int base, int n, int k, float* out_v, int* out_i, Cand* red) {
  const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
  Cand prev = {INFINITY, -1};
  for (int r = 0; r < k; ++r) {
    Cand best = {-INFINITY, 0x7fffffff};
    bool any = false;
    for (int j = threadIdx.x; j < n; j += kTopkThreads) {
      const Cand c = {sc[j], ix ? ix[j] : base + j};
      if (c.i >= 0 && cand_before(prev, c) && (!any || cand_before(c, best))) { best = c; any = true; }
    }
    if (!any) best = Cand{-INFINITY, 0x7fffffff};
#pragma unroll
    for (int off = 1; off < kWave; off <<= 1) {
      Cand o = {__shfl_xor(best.v, off, kWave), __shfl_xor(best.i, off, kWave)};
      if (cand_before(o, best)) best = o;
    }
    if (lane == 0) red[wave] = best;
    __syncthreads();
    best = red[0];
#pragma unroll
    for (int w = 1; w < kTopkThreads / kWave; ++w)
      if (cand_before(red[w], best)) best = red[w];
    __syncthreads();
    const bool found = best.i != 0x7fffffff;
    if (threadIdx.x == 0) { out_v[r] = found ? best.v : -INFINITY; out_i[r] = found ? best.i : -1; }
    prev = found ? best : Cand{-INFINITY, 0x7fffffff};  // nothing is after this one: the remaining picks are empty too
  }
}

// Phase 1: workgroup (chunk, sequence) selects the W best of its chunk of candidates.  With one chunk per sequence the
// picks are final (written as parent / token / score); otherwise they go to the workspace for phase 2.
__global__ __launch_bounds__(kTopkThreads) void beam_topk_kernel(const float* __restrict__ beam_scores,
                                                                 const float* __restrict__ logp, int beams, int vocab,
                                                                 int n_chunks, float* __restrict__ ws_v,
                                                                 int* __restrict__ ws_i, int32_t* __restrict__ parent,
                                                                 int32_t* __restrict__ token, float* __restrict__ score) {
  __shared__ float sc[kTopkChunk];
  __shared__ Cand red[kTopkThreads / kWave];
  __shared__ float pick_v[kTopkMaxBeams];
  __shared__ int pick_i[kTopkMaxBeams];
  const int b = blockIdx.y, chunk = blockIdx.x;
  const long long n_cand = (long long)beams * vocab;
  const long long c0 = (long long)chunk * kTopkChunk;
  const int n = (int)min((long long)kTopkChunk, n_cand - c0);
  for (int j = threadIdx.x; j < n; j += kTopkThreads) {
    const long long cand = c0 + j;
    const int w = (int)(cand / vocab);
    float v = logp[(long long)b * n_cand + cand] + (beam_scores ? beam_scores[b * beams + w] : 0.f);
    sc[j] = v == v ? v : -INFINITY;  // a NaN never wins
  }
  __syncthreads();
  select_topk(sc, nullptr, (int)c0, n, beams, pick_v, pick_i, red);
  __syncthreads();
  if (threadIdx.x < beams) {
    const int r = threadIdx.x;
    if (n_chunks == 1) {
      const int i = pick_i[r];
      parent[b * beams + r] = i >= 0 ? b * beams + i / vocab : -1;
      token[b * beams + r] = i >= 0 ? i % vocab : -1;
      score[b * beams + r] = pick_v[r];
    } else {
      ws_v[((long long)b * n_chunks + chunk) * beams + r] = pick_v[r];
      ws_i[((long long)b * n_chunks + chunk) * beams + r] = pick_i[r];
    }
  }
}

// Phase 2: the W best of the chunks' picks of one sequence (the top W of a union lie among the top W of its parts).
__global__ __launch_bounds__(kTopkThreads) void beam_topk_merge_kernel(const float* __restrict__ ws_v,
                                                                       const int* __restrict__ ws_i, int beams,
                                                                       int vocab, int n_chunks,
                                                                       int32_t* __restrict__ parent,
                                                                       int32_t* __restrict__ token,
                                                                       float* __restrict__ score) {
  __shared__ float sc[kTopkChunk];
  __shared__ int ix[kTopkChunk];
  __shared__ Cand red[kTopkThreads / kWave];
  __shared__ float pick_v[kTopkMaxBeams];
  __shared__ int pick_i[kTopkMaxBeams];
  const int b = blockIdx.x, n = n_chunks * beams;
  for (int j = threadIdx.x; j < n; j += kTopkThreads) { sc[j] = ws_v[(long long)b * n + j]; ix[j] = ws_i[(long long)b * n + j]; }
  __syncthreads();
  select_topk(sc, ix, 0, n, beams, pick_v, pick_i, red);
  __syncthreads();
  if (threadIdx.x < beams) {
    const int r = threadIdx.x, i = pick_i[r];
    parent[b * beams + r] = i >= 0 ? b * beams + i / vocab : -1;
    token[b * beams + r] = i >= 0 ? i % vocab : -1;
    score[b * beams + r] = pick_v[r];
  }
}

// gen_src_out[u][g] = g < step ? gen_src_in[parent[u]][g] (parent's own id when gen_src_in is NULL) : parent[u] at g == step;
// slots past `step` are set to u (a stream's future appends go to its own slots).
__global__ __launch_bounds__(256) void beam_reorder_kernel(const int32_t* __restrict__ parent,
                                                           const int32_t* __restrict__ src_in,
                                                           int32_t* __restrict__ src_out, int n_streams, int gen_cap,
                                                           int step) {
  const long long t = (long long)blockIdx.x * 256 + threadIdx.x;
  if (t >= (long long)n_streams * gen_cap) return;
  const int u = (int)(t / gen_cap), g = (int)(t % gen_cap);
  const int par = max(min(parent[u], n_streams - 1), 0);
  int v = u;
  if (g < step) v = src_in ? src_in[(long long)par * gen_cap + g] : par;
  else if (g == step) v = par;
  src_out[t] = v;
}

static int topk_chunks(int beams, int vocab) { return (int)(((long long)beams * vocab + kTopkChunk - 1) / kTopkChunk); }

size_t beam_topk_workspace_bytes(int batch, int beams, int vocab) {
  const int n_chunks = topk_chunks(beams, vocab);
  return n_chunks <= 1 ? 0 : (size_t)batch * n_chunks * beams * 8;
}

int launch_beam_topk(const float* beam_scores, const float* logp, int batch, int beams, int vocab, int32_t* parent,
                     int32_t* token, float* score, void* workspace, hipStream_t stream) {
  const int n_chunks = topk_chunks(beams, vocab);
  float* ws_v = (float*)workspace;
  int* ws_i = (int*)(ws_v + (size_t)batch * n_chunks * beams);
  hipLaunchKernelGGL(beam_topk_kernel, dim3(n_chunks, batch), dim3(kTopkThreads), 0, stream, beam_scores, logp, beams,
                     vocab, n_chunks, ws_v, ws_i, parent, token, score);
  if (n_chunks > 1)
    hipLaunchKernelGGL(beam_topk_merge_kernel, dim3(batch), dim3(kTopkThreads), 0, stream, ws_v, ws_i, beams, vocab,
                       n_chunks, parent, token, score);
  return hipGetLastError() == hipSuccess ? EARN_OK : EARN_ERR_HIP;
}

int launch_beam_reorder(const int32_t* parent, const int32_t* src_in, int32_t* src_out, int n_streams, int gen_cap, int step,
                        hipStream_t stream) {
  const long long n = (long long)n_streams * gen_cap;
  hipLaunchKernelGGL(beam_reorder_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, stream, parent, src_in, src_out,
                     n_streams, gen_cap, step);
  return hipGetLastError() == hipSuccess ? EARN_OK : EARN_ERR_HIP;
}

int beam_topk_limits(int beams, int vocab, const char** why) {
  if (beams > kTopkMaxBeams) { *why = "more than 64 beams"; return 0; }
  if ((long long)topk_chunks(beams, vocab) * beams > kTopkChunk) { *why = "beams * vocab too large for the two-phase selection"; return 0; }
  return 1;
}

}  // namespace earn
