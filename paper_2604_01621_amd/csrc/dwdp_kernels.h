// Internal launch interface between the C-ABI host code and the gfx950 kernels.
// Device pointers only; every function enqueues on `stream` and returns.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/dwdp.h"

namespace dwdp {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v8i __attribute__((ext_vector_type(8)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef __bf16 v8bf __attribute__((ext_vector_type(8)));

constexpr int kWave = 64;
constexpr int kBlockScale = 128;  // side of a weight scale block = activation quantisation group
constexpr int kTileBytes = 2048;   // one packed FP8 weight tile: 16 rows x 128 columns

struct RouteParams {
  int E, K, n_group, topk_group, score_fn;
  float routed_scale;
};

// Tokens per permutation chunk for E experts (bitmask of E x chunk bits must fit 48 KiB of LDS).
int permute_chunk_tokens(int E);
// Tokens per workgroup of the multi-workgroup permutation (sizes the chunk_counts scratch).
int permute_multi_chunk_tokens(int E);

void launch_route(const float* logits, const float* bias, int T, const RouteParams& p, int32_t* ids, float* w,
                  hipStream_t stream);
// The same routing plus, in the same launch (extra workgroups), the activation quantisation
// x bf16 [T,H] -> xq fp8 [T,H], xs fp32 [T,H/128]: the two are independent, one launch less.
void launch_route_quant(const float* logits, const float* bias, int T, const RouteParams& p, int32_t* ids, float* w,
                        const void* x, int H, uint8_t* xq, float* xs, hipStream_t stream);

// Device-built list of the M tiles (up to kTileM sorted rows of one expert) the LDS-tiled GEMM works on.
constexpr int kTileM = 288;
struct TileSched {
  int32_t* mt_expert;  // [n_mt_max] expert slot of the tile
  int32_t* mt_row0;    // [n_mt_max] first sorted row
  int32_t* n_mtiles;   // [1] tiles listed
  int32_t* sync;       // [tile_sync_words(capacity)] ticket queues, error word, per-tile counters of the
                       // persistent tiled GEMM; zeroed by the kernel that builds the list
  int n_mt_max;        // host-side upper bound of the tiles listed by this call
  int sync_words;      // words of `sync` to zero
  int wg_limit_full;   // persistent launches: workgroups that take work when (almost) nothing is streamed ...
  int wg_limit_shared; // ... and when at least share_min_experts experts are streamed beside the tiled ones
  int share_min_experts;
  int min_tiles;       // fewer M tiles than this (device-side count): none is listed, and when the row-group
                       // list is built those experts go there instead (see build_work_lists_block)
  // Row groups (up to kMidRows sorted rows of one expert) of the experts with mid_min_rows ..
  // stream_max_rows rows, for the multi-tile weight-streaming kernels; mid_expert == nullptr: not listed.
  int32_t* mid_expert;  // [mid_cap]
  int32_t* mid_row0;    // [mid_cap] first sorted row of the group
  int32_t* n_mid;       // [1]
  int mid_cap;
  int mid_min_rows;
};
constexpr int kMidRows = 64;        // rows of one group of the multi-tile streaming kernels (4 tiles of 16)
// Upper bound of listed row groups for `rows` sorted rows over n_slots experts.
int mid_groups_cap(int rows, int n_slots, int mid_min_rows);
constexpr int kTileSyncError = 16;  // sync[16]: a bounded wait of the tiled GEMM gave up
constexpr int kTileSyncLimit = 17;  // sync[17]: workgroups of a persistent launch that take work (the others exit)
constexpr int kTileSyncDone = 32;   // sync[32 + m]: finished GEMM-1 items of M tile m
// Upper bound of listed tiles when experts with more than stream_max_rows rows are listed.
int tile_mtiles_cap(int rows, int n_slots, int stream_max_rows);
// Words of TileSched::sync for a list of at most mt_cap tiles.
int tile_sync_words(int mt_cap);

// chunk_counts: int32 [n_chunks * E] scratch.  With `list` non-null the single workgroup that
// finishes the offsets also lists the M tiles of all experts with more than stream_max_rows
// rows (list->n_mt_max is the capacity of the arrays).
void launch_permute(const int32_t* ids, int T, int E, int K, int has_shared, int32_t* chunk_counts,
                    int32_t* offsets, int32_t* perm, int32_t* inv_perm, const TileSched* list, int stream_max_rows,
                    hipStream_t stream);

// x bf16 [T,H] -> xq fp8 [T,H], xs fp32 [T,H/128]
void launch_quant_act(const void* x, int T, int H, uint8_t* xq, float* xs, hipStream_t stream);

// One piece of a copy plan (device pointers).
struct CopyUnit {
  void* dst;
  const void* src;
  size_t bytes;
};
// units: device array, plan order; at most n_workgroups workgroups are launched.
void launch_copy_plan(const CopyUnit* units, int n_units, int n_workgroups, hipStream_t stream);

// y[t] = sum_k w[t,k] * yp[inv_perm[t*K+k]] (+ yp[T*K+t]); yp bf16 or fp32 [rows,H]; y bf16 [T,H]
void launch_combine(const void* yp, bool yp_fp32, const int32_t* inv_perm, const float* topk_w, int T, int H, int K,
                    int has_shared, void* y, hipStream_t stream);

struct GemmArgs {
  const dwdp_expert_ptrs* table;  // device, n_slots rows
  const int32_t* offsets;         // device, n_slots + 1
  const int32_t* perm;            // device, T*K
  int n_slots, E, T, H, I, K;
};

// Row-major fp8 [rows, cols] (rows % 16 == 0, cols % 128 == 0) -> tile-major layout of the FP8 GEMMs.
void launch_pack_fp8_tiles(const void* src, void* dst, long rows, int cols, hipStream_t stream);

// FP8 (weights tile-major): h = quant(silu(Xq Wg^T) * (Xq Wu^T)); hq fp8 [rows,I], hs fp32 [rows,I/128]
// Streaming kernels: experts with 1..max_rows rows.  LDS-tiled kernels: the experts in the tile list.
// `ts` carries the row-group list of the experts with 17 .. max_rows rows (ts.mid_expert may be
// nullptr: then experts with more than 16 rows are walked 16 rows at a time, re-reading the weights).
void launch_gemm1_fp8(const GemmArgs& a, int max_rows, const TileSched& ts, const uint8_t* xq, const float* xs,
                      uint8_t* hq, float* hs, hipStream_t stream);
// The LDS-tiled pair for the experts of the tile list.  schedule 0: one workgroup per (M tile,
// panel) item, one launch per GEMM (phase_mask 1, then 2).  schedule 1: persistent launches of at
// most n_cus workgroups that take items by atomic tickets -- phase_mask 3: GEMM-1 then GEMM-2 items
// in one launch with device-side dependency counters; 1 or 2: one GEMM per launch.
// mxfp4: the listed experts' weights are MXFP4 (launch_pack_mxfp4 layouts) instead of FP8.
// Contract on the activation-scale arrays xs [T, H/128] and hs [rows, I/128]: the kernel copies a
// row's scales three K blocks at a time, so when the number of K blocks is not a multiple of three it
// reads up to two floats past the end of a row -- the next row's scales, or, after the last row, past
// the array: both arrays must be followed by at least 8 readable bytes (the library's workspace
// keeps 16 bytes of padding behind each).  What is read there is never used.
void launch_gemm_fp8_tile(const GemmArgs& a, const TileSched& ts, bool mxfp4, int schedule, int phase_mask,
                          const uint8_t* xq, const float* xs, uint8_t* hq, float* hs, void* yp, int n_cus,
                          hipStream_t stream);
// FP8: yp = Hq W2^T, bf16 [rows,H]
void launch_gemm2_fp8(const GemmArgs& a, int max_rows, const TileSched& ts, const uint8_t* hq, const float* hs,
                      void* yp, hipStream_t stream);
// MXFP4 weights (layouts of launch_pack_mxfp4), FP8 activations: same results as the FP8 pair above
void launch_gemm1_mx(const GemmArgs& a, int max_rows, const uint8_t* xq, const float* xs, uint8_t* hq, float* hs,
                     hipStream_t stream);
void launch_gemm2_mx(const GemmArgs& a, int max_rows, const uint8_t* hq, const float* hs, void* yp,
                     hipStream_t stream);
// Row-major packed E2M1 codes [rows, cols/2] and E8M0 scales [rows, cols/32] -> the streaming layouts.
void launch_pack_mxfp4(const void* codes, const void* scales, void* codes_out, void* scales_out, long rows, int cols,
                       hipStream_t stream);
// bf16 weights and activations: h fp32 [rows,I]; yp fp32 [rows,H]
void launch_gemm1_bf16(const GemmArgs& a, const void* x, void* h, hipStream_t stream);
void launch_gemm2_bf16(const GemmArgs& a, const void* h, void* yp, hipStream_t stream);

// ---- small device helpers shared by the kernels ----

__device__ __forceinline__ float bf16_to_f32(uint16_t b) { return __uint_as_float(((uint32_t)b) << 16); }

// Round-to-nearest-even fp32 -> bf16 (inputs are finite here).
__device__ __forceinline__ uint16_t f32_to_bf16(float f) {
  uint32_t u = __float_as_uint(f);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}

// Four fp32 -> four e4m3 bytes (hardware RNE conversion; inputs clamped to +-448 first).
__device__ __forceinline__ uint32_t pack_fp8x4(float a, float b, float c, float d) {
  a = __builtin_fminf(__builtin_fmaxf(a, -448.f), 448.f);
  b = __builtin_fminf(__builtin_fmaxf(b, -448.f), 448.f);
  c = __builtin_fminf(__builtin_fmaxf(c, -448.f), 448.f);
  d = __builtin_fminf(__builtin_fmaxf(d, -448.f), 448.f);
  int v = 0;
  v = __builtin_amdgcn_cvt_pk_fp8_f32(a, b, v, false);
  v = __builtin_amdgcn_cvt_pk_fp8_f32(c, d, v, true);
  return (uint32_t)v;
}

// Quantises 128-element groups of x: 16 lanes own one group (8 bf16 each); `gidx` is this
// thread's global index over n_groups * 16 lanes.
__device__ __forceinline__ void quant_act_lane(const uint16_t* __restrict__ x, long n_groups, uint8_t* __restrict__ xq,
                                               float* __restrict__ xs, long gidx) {
  long g = gidx >> 4;
  const int sub = (int)(gidx & 15);
  const bool live = g < n_groups;
  if (!live) g = n_groups - 1;  // keep the 16-lane reductions convergent
  const v4i raw = *(const v4i*)(x + g * 128 + sub * 8);
  float v[8];
#pragma unroll
  for (int i = 0; i < 4; i++) {
    uint32_t u = (uint32_t)raw[i];
    v[2 * i] = __uint_as_float(u << 16);
    v[2 * i + 1] = __uint_as_float(u & 0xFFFF0000u);
  }
  float amax = 0.f;
#pragma unroll
  for (int i = 0; i < 8; i++) amax = fmaxf(amax, fabsf(v[i]));
#pragma unroll
  for (int off = 8; off >= 1; off >>= 1) amax = fmaxf(amax, __shfl_xor(amax, off));
  const float scale = amax > 0.f ? amax / 448.f : 1.f;
  uint32_t lo = pack_fp8x4(v[0] / scale, v[1] / scale, v[2] / scale, v[3] / scale);
  uint32_t hi = pack_fp8x4(v[4] / scale, v[5] / scale, v[6] / scale, v[7] / scale);
  if (live) {
    uint2 o;
    o.x = lo;
    o.y = hi;
    *(uint2*)(xq + g * 128 + sub * 8) = o;
    if (sub == 0) xs[g] = scale;
  }
}

// Work lists of the grouped GEMMs, built by ONE workgroup of 1024 threads after it has written
// offsets[0..n_slots] (global memory; a __syncthreads separates the writes from this call).
// Thread i owns expert slots 2i and 2i+1; exclusive block scans give every expert its place.
//   * M tiles (kTileM rows each) of all experts with more than stream_max_rows rows, for the LDS-tiled GEMM;
//   * row groups (kMidRows rows each) of all experts with mid_min_rows .. stream_max_rows rows, for
//     the multi-tile streaming kernels (only when s.mid_expert is set).
// Also zeroes the scheduler words of the persistent tiled GEMM.  scan_s: 1024 ints of LDS.
__device__ __forceinline__ void build_work_lists_block(const int32_t* offsets, int n_slots, int stream_max_rows,
                                                       const TileSched& s, int32_t* scan_s) {
  const int tid = threadIdx.x;
  // scheduler words of the persistent tiled GEMM (ticket queues, error word, per-tile counters)
  for (int i = tid; i < s.sync_words; i += 1024) s.sync[i] = 0;
  __syncthreads();
  int m[2], r0[2];
#pragma unroll
  for (int i = 0; i < 2; i++) {
    const int e = 2 * tid + i;
    m[i] = 0;
    r0[i] = 0;
    if (e < n_slots) {
      r0[i] = offsets[e];
      m[i] = offsets[e + 1] - r0[i];
    }
  }
  // exclusive scan of v0 + v1 over the block; returns this thread's prefix, *total = sum over all
  auto scan = [&](int v, int* total) {
    __syncthreads();  // scan_s may still be in use (the caller's own scan, the previous list)
    scan_s[tid] = v;
    __syncthreads();
    for (int d = 1; d < 1024; d <<= 1) {
      const int o = (tid >= d) ? scan_s[tid - d] : 0;
      __syncthreads();
      scan_s[tid] += o;
      __syncthreads();
    }
    *total = scan_s[1023];
    return scan_s[tid] - v;
  };
  // The tiled kernel's workgroups each take a whole compute unit: a handful of M tiles cannot fill
  // the chip and keeps everything else off the units it holds.  Below min_tiles the experts that
  // would be tiled join the row-group list (their weights are then read once per 64 rows).
  bool tiled = false;
  if (s.mt_expert) {
    int cnt[2];
#pragma unroll
    for (int i = 0; i < 2; i++) cnt[i] = m[i] > stream_max_rows ? (m[i] + kTileM - 1) / kTileM : 0;
    int total;
    int pos = scan(cnt[0] + cnt[1], &total);
    tiled = total >= s.min_tiles || !s.mid_expert;
#pragma unroll
    for (int i = 0; i < 2; i++)
      for (int k = 0; k < cnt[i] && tiled; k++, pos++)
        if (pos < s.n_mt_max) {
          s.mt_expert[pos] = 2 * tid + i;
          s.mt_row0[pos] = r0[i] + k * kTileM;
        }
    if (tid == 0) *s.n_mtiles = tiled ? min(total, s.n_mt_max) : 0;
  }
  const int mid_max_rows = tiled ? stream_max_rows : 0x7fffffff;
  if (s.mt_expert) {
    // A persistent tiled launch holds its compute units to the end.  When a substantial number of
    // experts is streamed beside it, it leaves part of the chip to that chain from the start
    // (the streamed chain is bound by HBM and needs few units; the tiled one by unit time).
    int n_str = 0;
#pragma unroll
    for (int i = 0; i < 2; i++) n_str += (m[i] > 0 && m[i] <= mid_max_rows) ? 1 : 0;
    int total;
    scan(n_str, &total);
    if (tid == 0) s.sync[kTileSyncLimit] = total >= s.share_min_experts ? s.wg_limit_shared : s.wg_limit_full;
  }
  if (s.mid_expert) {
    int cnt[2];
#pragma unroll
    for (int i = 0; i < 2; i++)
      cnt[i] = (m[i] >= s.mid_min_rows && m[i] <= mid_max_rows) ? (m[i] + kMidRows - 1) / kMidRows : 0;
    int total;
    int pos = scan(cnt[0] + cnt[1], &total);
#pragma unroll
    for (int i = 0; i < 2; i++)
      for (int k = 0; k < cnt[i]; k++, pos++)
        if (pos < s.mid_cap) {
          s.mid_expert[pos] = 2 * tid + i;
          s.mid_row0[pos] = r0[i] + k * kMidRows;
        }
    if (tid == 0) *s.n_mid = min(total, s.mid_cap);
  }
}

}  // namespace dwdp
