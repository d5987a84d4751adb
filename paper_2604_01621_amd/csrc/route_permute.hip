// Router top-k and permutation-by-expert kernels for gfx950 (64-wide wavefronts).
//
// Route: one wavefront per token.  Scores are staged in LDS, group scores and the kept
// groups are computed by the first n_group lanes, then K rounds of a wave-wide arg-max
// pick the experts in descending score order with ties to the lower index.
//
// Permute: a stable counting sort without atomics on global memory.  A token selects an
// expert at most once, so the rank of (t, e) inside expert e is the number of tokens
// t' < t that selected e.  Each block builds an [E x chunk] bitmask of its token chunk in
// LDS; ranks are popcounts of mask prefixes, chunk bases come from a scan over chunks.
#include "dwdp_kernels.h"

namespace dwdp {

// ----------------------------------------------------------------------------- route

constexpr int kRouteWaves = 4;

__device__ __forceinline__ bool better(float v, int i, float v2, int i2) {
  return v > v2 || (v == v2 && i < i2);
}

__device__ __forceinline__ void route_block(const float* __restrict__ logits, const float* __restrict__ bias, int T,
                                            const RouteParams& p, int32_t* __restrict__ ids,
                                            float* __restrict__ wout, float* smem, int block) {
  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const int t_raw = block * kRouteWaves + wave;
  const bool live = t_raw < T;
  const int t = live ? t_raw : T - 1;  // surplus waves redo the last token and write nothing
  const int E = p.E;
  // per-wave LDS: c[E] selection scores, s[E] un-biased scores, gscore[64], keep[64]
  float* c_s = smem + wave * (2 * E + 128);
  float* s_s = c_s + E;
  float* g_s = s_s + E;
  int* keep_s = (int*)(g_s + 64);

  const float* z = logits + (size_t)t * E;
  for (int e = lane; e < E; e += kWave) {
    float zv = z[e];
    float s, c;
    if (p.score_fn == DWDP_SCORE_SIGMOID) {
      // fp64 evaluation rounded once to fp32: the same value on any IEEE host
      s = (float)(1.0 / (1.0 + exp(-(double)zv)));
      c = bias ? __fadd_rn(s, bias[e]) : s;
    } else {
      s = zv;
      c = zv;
    }
    c_s[e] = c;
    s_s[e] = s;
  }
  __syncthreads();

  if (p.n_group > 1) {
    const int gs = E / p.n_group;
    if (lane < p.n_group) {
      float m1 = -INFINITY, m2 = -INFINITY;
      for (int i = 0; i < gs; i++) {
        float v = c_s[lane * gs + i];
        if (v > m1) {
          m2 = m1;
          m1 = v;
        } else if (v > m2) {
          m2 = v;
        }
      }
      g_s[lane] = __fadd_rn(m1, m2);
    }
    __syncthreads();
    if (lane < p.n_group) {
      float mine = g_s[lane];
      int rank = 0;
      for (int g = 0; g < p.n_group; g++) rank += better(g_s[g], g, mine, lane) ? 1 : 0;
      keep_s[lane] = rank < p.topk_group;
    }
    __syncthreads();
    for (int e = lane; e < E; e += kWave)
      if (!keep_s[e / gs]) c_s[e] = -INFINITY;
    __syncthreads();
  }

  int my_id = 0;  // lane k ends up holding the k-th selected expert
  for (int k = 0; k < p.K; k++) {
    float bv = -INFINITY;
    int bi = 0x7fffffff;
    for (int e = lane; e < E; e += kWave) {
      float v = c_s[e];
      if (better(v, e, bv, bi)) {
        bv = v;
        bi = e;
      }
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
      float ov = __shfl_xor(bv, off);
      int oi = __shfl_xor(bi, off);
      if (better(ov, oi, bv, bi)) {
        bv = ov;
        bi = oi;
      }
    }
    if (lane == k) my_id = bi;
    if (lane == 0) c_s[bi] = -INFINITY;
    __syncthreads();
  }

  const int id0 = __shfl(my_id, 0);  // best expert: its logit is the soft-max shift
  float sv = 0.f;
  if (lane < p.K) {
    sv = s_s[my_id];
    if (p.score_fn != DWDP_SCORE_SIGMOID) sv = expf(sv - s_s[id0]);
  }
  float sum = sv;
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) sum += __shfl_xor(sum, off);
  if (live && lane < p.K) {
    float denom = (p.score_fn == DWDP_SCORE_SIGMOID) ? sum + 1e-20f : sum;
    ids[(size_t)t * p.K + lane] = my_id;
    wout[(size_t)t * p.K + lane] = sv / denom * p.routed_scale;
  }
}

__global__ __launch_bounds__(kRouteWaves* kWave) void route_kernel(const float* __restrict__ logits,
                                                                   const float* __restrict__ bias, int T,
                                                                   RouteParams p, int32_t* __restrict__ ids,
                                                                   float* __restrict__ wout) {
  extern __shared__ float smem[];
  route_block(logits, bias, T, p, ids, wout, smem, blockIdx.x);
}

// Workgroups [0, n_route) route 4 tokens each, the others quantise 16 groups of 128 activations each.
__global__ __launch_bounds__(kRouteWaves* kWave) void route_quant_kernel(
    const float* __restrict__ logits, const float* __restrict__ bias, int T, RouteParams p, int32_t* __restrict__ ids,
    float* __restrict__ wout, int n_route, const uint16_t* __restrict__ x, long n_groups, uint8_t* __restrict__ xq,
    float* __restrict__ xs) {
  extern __shared__ float smem[];
  if ((int)blockIdx.x < n_route)
    route_block(logits, bias, T, p, ids, wout, smem, blockIdx.x);
  else
    quant_act_lane(x, n_groups, xq, xs, (long)(blockIdx.x - n_route) * blockDim.x + threadIdx.x);
}

void launch_route(const float* logits, const float* bias, int T, const RouteParams& p, int32_t* ids, float* w,
                  hipStream_t stream) {
  if (T <= 0) return;
  dim3 grid((T + kRouteWaves - 1) / kRouteWaves);
  size_t lds = (size_t)kRouteWaves * (2 * p.E + 128) * sizeof(float);
  hipLaunchKernelGGL(route_kernel, grid, dim3(kRouteWaves * kWave), lds, stream, logits, bias, T, p, ids, w);
}

void launch_route_quant(const float* logits, const float* bias, int T, const RouteParams& p, int32_t* ids, float* w,
                        const void* x, int H, uint8_t* xq, float* xs, hipStream_t stream) {
  if (T <= 0) return;
  const int n_route = (T + kRouteWaves - 1) / kRouteWaves;
  const long n_groups = (long)T * (H / kBlockScale);
  const long n_quant = (n_groups * 16 + kRouteWaves * kWave - 1) / (kRouteWaves * kWave);
  size_t lds = (size_t)kRouteWaves * (2 * p.E + 128) * sizeof(float);
  hipLaunchKernelGGL(route_quant_kernel, dim3((unsigned)(n_route + n_quant)), dim3(kRouteWaves * kWave), lds, stream,
                     logits, bias, T, p, ids, w, n_route, (const uint16_t*)x, n_groups, xq, xs);
}

// ----------------------------------------------------------------------------- permute

constexpr int kPermThreads = 1024;

int permute_chunk_tokens(int E) {
  int ch = (49152 * 8) / E;  // bits available per expert row in 48 KiB
  ch = (ch / 32) * 32;
  if (ch > 1024) ch = 1024;
  if (ch < 32) ch = 32;
  return ch;
}

// Tokens per workgroup when the permutation runs on several workgroups (T > permute_chunk_tokens):
// small chunks, so that a long token list spreads over many CUs (8192 tokens: 64 workgroups) and
// the rank of a token inside its chunk is a few population counts.
int permute_multi_chunk_tokens(int E) {
  const int ch = permute_chunk_tokens(E);
  return ch < 128 ? ch : 128;
}

// Build the [E x wpe] bitmask of tokens [t0, t0+nt) in LDS.
__device__ __forceinline__ void build_mask(uint32_t* mask, const int32_t* __restrict__ ids, int t0, int nt, int E,
                                           int K, int wpe) {
  for (int i = threadIdx.x; i < E * wpe; i += blockDim.x) mask[i] = 0u;
  __syncthreads();
  for (int i = threadIdx.x; i < nt * K; i += blockDim.x) {
    int tl = i / K;
    int e = ids[(size_t)t0 * K + i];
    if (e >= 0 && e < E) atomicOr(&mask[e * wpe + (tl >> 5)], 1u << (tl & 31));
  }
  __syncthreads();
}

__device__ __forceinline__ int rank_in_chunk(const uint32_t* mask, int e, int tl, int wpe) {
  const uint32_t* row = mask + e * wpe;
  int r = 0;
  for (int w = 0; w < (tl >> 5); w++) r += __popc(row[w]);
  r += __popc(row[tl >> 5] & ((1u << (tl & 31)) - 1u));
  return r;
}

// Exclusive scan of cnt[0..E) by one block (E <= 1024 = blockDim); writes offsets[0..E].
__device__ __forceinline__ void block_scan_offsets(int my_cnt, int E, int32_t* scan_s, int32_t* offsets) {
  int tid = threadIdx.x;
  scan_s[tid] = (tid < E) ? my_cnt : 0;
  __syncthreads();
  for (int d = 1; d < kPermThreads; d <<= 1) {
    int v = (tid >= d) ? scan_s[tid - d] : 0;
    __syncthreads();
    scan_s[tid] += v;
    __syncthreads();
  }
  if (tid < E) offsets[tid + 1] = scan_s[tid];
  if (tid == 0) offsets[0] = 0;
}

// T <= chunk: histogram, scan and scatter in one block.
__global__ __launch_bounds__(kPermThreads) void permute_single_kernel(const int32_t* __restrict__ ids, int T, int E,
                                                                       int K, int has_shared, int wpe,
                                                                       int32_t* __restrict__ offsets,
                                                                       int32_t* __restrict__ perm,
                                                                       int32_t* __restrict__ inv_perm, TileSched list,
                                                                       int stream_max_rows) {
  extern __shared__ uint32_t lds[];
  uint32_t* mask = lds;
  int32_t* scan_s = (int32_t*)(lds + E * wpe);
  int32_t* off_s = scan_s + kPermThreads;  // [E+1]
  build_mask(mask, ids, 0, T, E, K, wpe);
  int cnt = 0;
  if ((int)threadIdx.x < E)
    for (int w = 0; w < wpe; w++) cnt += __popc(mask[threadIdx.x * wpe + w]);
  block_scan_offsets(cnt, E, scan_s, off_s);
  __syncthreads();
  for (int i = threadIdx.x; i <= E; i += blockDim.x) offsets[i] = off_s[i];
  if (has_shared && threadIdx.x == 0) offsets[E + 1] = T * K + T;
  for (int i = threadIdx.x; i < T * K; i += blockDim.x) {
    int e = ids[i];
    if (e < 0 || e >= E) continue;
    int r = off_s[e] + rank_in_chunk(mask, e, i / K, wpe);
    perm[r] = i;
    inv_perm[i] = r;
  }
  if (list.mt_expert || list.mid_expert) {
    __syncthreads();  // offsets[] above were written by other threads of this workgroup
    build_work_lists_block(offsets, E + (has_shared ? 1 : 0), stream_max_rows, list, scan_s);
  }
}

__global__ __launch_bounds__(kPermThreads) void permute_count_kernel(const int32_t* __restrict__ ids, int T, int E,
                                                                      int K, int chunk, int wpe,
                                                                      int32_t* __restrict__ chunk_counts) {
  extern __shared__ uint32_t lds[];
  int t0 = blockIdx.x * chunk;
  int nt = min(chunk, T - t0);
  build_mask(lds, ids, t0, nt, E, K, wpe);
  for (int e = threadIdx.x; e < E; e += blockDim.x) {
    int cnt = 0;
    for (int w = 0; w < wpe; w++) cnt += __popc(lds[e * wpe + w]);
    chunk_counts[(size_t)blockIdx.x * E + e] = cnt;
  }
}

// One block: chunk_counts -> exclusive chunk bases (in place), offsets.
__global__ __launch_bounds__(kPermThreads) void permute_scan_kernel(int32_t* __restrict__ chunk_counts, int n_chunks,
                                                                     int T, int E, int K, int has_shared,
                                                                     int32_t* __restrict__ offsets, TileSched list,
                                                                     int stream_max_rows) {
  __shared__ int32_t scan_s[kPermThreads];
  int e = threadIdx.x;
  int run = 0;
  if (e < E) {
    for (int c = 0; c < n_chunks; c++) {
      int v = chunk_counts[(size_t)c * E + e];
      chunk_counts[(size_t)c * E + e] = run;
      run += v;
    }
  }
  block_scan_offsets(run, E, scan_s, offsets);
  if (has_shared && threadIdx.x == 0) offsets[E + 1] = T * K + T;
  if (list.mt_expert || list.mid_expert) {
    __syncthreads();
    build_work_lists_block(offsets, E + (has_shared ? 1 : 0), stream_max_rows, list, scan_s);
  }
}

__global__ __launch_bounds__(kPermThreads) void permute_scatter_kernel(const int32_t* __restrict__ ids, int T, int E,
                                                                        int K, int chunk, int wpe,
                                                                        const int32_t* __restrict__ chunk_base,
                                                                        const int32_t* __restrict__ offsets,
                                                                        int32_t* __restrict__ perm,
                                                                        int32_t* __restrict__ inv_perm) {
  extern __shared__ uint32_t lds[];
  int t0 = blockIdx.x * chunk;
  int nt = min(chunk, T - t0);
  build_mask(lds, ids, t0, nt, E, K, wpe);
  for (int i = threadIdx.x; i < nt * K; i += blockDim.x) {
    int f = t0 * K + i;
    int e = ids[f];
    if (e < 0 || e >= E) continue;
    int r = offsets[e] + chunk_base[(size_t)blockIdx.x * E + e] + rank_in_chunk(lds, e, i / K, wpe);
    perm[r] = f;
    inv_perm[f] = r;
  }
}

__global__ void permute_empty_kernel(int32_t* offsets, int n) {
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) offsets[i] = 0;
}

void launch_permute(const int32_t* ids, int T, int E, int K, int has_shared, int32_t* chunk_counts, int32_t* offsets,
                    int32_t* perm, int32_t* inv_perm, const TileSched* list_in, int stream_max_rows,
                    hipStream_t stream) {
  const TileSched list = list_in ? *list_in : TileSched{};
  const int n_off = E + 1 + (has_shared ? 1 : 0);
  if (T <= 0) {
    hipLaunchKernelGGL(permute_empty_kernel, dim3((n_off + 255) / 256), dim3(256), 0, stream, offsets, n_off);
    return;
  }
  if (T <= permute_chunk_tokens(E)) {
    const int wpe = permute_chunk_tokens(E) / 32;
    size_t lds = (size_t)E * wpe * sizeof(uint32_t) + (kPermThreads + E + 1) * sizeof(int32_t);
    hipLaunchKernelGGL(permute_single_kernel, dim3(1), dim3(kPermThreads), lds, stream, ids, T, E, K, has_shared, wpe,
                       offsets, perm, inv_perm, list, stream_max_rows);
    return;
  }
  const int chunk = permute_multi_chunk_tokens(E);
  const int wpe = chunk / 32;
  const size_t mask_bytes = (size_t)E * wpe * sizeof(uint32_t);
  const int n_chunks = (T + chunk - 1) / chunk;
  hipLaunchKernelGGL(permute_count_kernel, dim3(n_chunks), dim3(kPermThreads), mask_bytes, stream, ids, T, E, K, chunk,
                     wpe, chunk_counts);
  hipLaunchKernelGGL(permute_scan_kernel, dim3(1), dim3(kPermThreads), 0, stream, chunk_counts, n_chunks, T, E, K,
                     has_shared, offsets, list, stream_max_rows);
  hipLaunchKernelGGL(permute_scatter_kernel, dim3(n_chunks), dim3(kPermThreads), mask_bytes, stream, ids, T, E, K,
                     chunk, wpe, chunk_counts, offsets, perm, inv_perm);
}

}  // namespace dwdp
