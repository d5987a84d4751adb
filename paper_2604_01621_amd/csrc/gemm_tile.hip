// LDS-tiled FP8 grouped GEMM for gfx950: the large-M (prefill-shaped) path.
//
// A workgroup of 12 waves computes a 256 (weight rows) x 288 (tokens) output tile of one
// expert.  288 tokens cover almost every expert of the prefill workload (256 +- 16 rows), so
// each weight panel is read from HBM once; with 128-token tiles the panels were re-read by
// every M tile and the kernel ran at HBM speed.  Per 128-wide K block -- exactly one
// weight-scale block and one activation-scale group -- the workgroup stages 16 packed
// weight tiles (32 KiB, contiguous 2 KiB pieces located through the expert-pointer table)
// and up to 18 packed token tiles (36 KiB, rows gathered through the permutation) in LDS;
// wave (wn, wm) multiplies weight tiles 4*wn..4*wn+3 with token tiles wm, wm+3, ... on
// v_mfma_f32_16x16x128_f8f6f4 and folds every fp32 partial product into its accumulator
// with s_act[token,kb] * s_w[nblock,kb] on the VALU.  The LDS image of K block kb+1 is
// filled by asynchronous global->LDS copies (global_load_lds_dwordx4, no staging registers,
// no ds_write) while block kb is multiplied; two images of 68 KiB alternate, one barrier
// per K block.
//
// Token tiles of 16 beyond the expert's row count are skipped (not loaded, not
// multiplied).  Workgroups are numbered so that all weight panels of one M tile run on the
// same XCD back to back and share the token rows in its L2: block b runs on XCD b % 8 and
// handles M tile (b/8 / n_panels) * 8 + b % 8, panel (b/8) % n_panels.
//
// GEMM-1 (G1): rows = 128 gate + 128 up rows of W13, epilogue silu(g)*u, per-token amax
// over the block's 128 h columns, e4m3 quantisation of h.  GEMM-2: rows = 256 rows of W2,
// epilogue bf16 store.  Experts with few rows are left to the streaming kernels (they are not listed).
#include "dwdp_kernels.h"

// Timing experiments only (results are wrong when set): 1 = skip the MFMA/VALU work,
// 2 = skip the global->LDS copies after the first K block, 4 = skip the weight copies,
// 8 = skip the token copies.  Never set in a product build.
#ifndef DWDP_TILE_DBG
#define DWDP_TILE_DBG 0
#endif

namespace dwdp {

constexpr int kBM = 288;          // tokens per workgroup tile
constexpr int kTT = kBM / 16;     // token tiles per workgroup (18)
constexpr int kWM = 3;            // waves along the token dimension (x 4 along the weight rows)
constexpr int kTW = (kTT + kWM - 1) / kWM;  // token tiles per wave
constexpr int kTileWaves = 4 * kWM;
constexpr int kTileThreads = 64 * kTileWaves;
constexpr int kLdsA = 16 * kTileBytes;
constexpr int kLdsB = kTT * kTileBytes;
constexpr int kSaLen = 320;
static_assert(kBM <= kSaLen && kTT <= 20, "copy loops cover 40 token half-tiles and 320 scales");

typedef const __attribute__((address_space(1))) v4i* gv4i;
typedef const __attribute__((address_space(1))) float* gf32;
// Read-only data addressed with wave-uniform pointers: the constant address space makes
// these scalar loads (s_load), which do not touch the vector-memory counter the copies use.
typedef const __attribute__((address_space(4))) float* cf32;

__device__ __forceinline__ v8i cat8(v4i lo, v4i hi) { return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7); }

// Lists the M tiles (kBM rows each) of all experts that have more than stream_max_rows rows.
// One block; thread i owns expert slots 2i and 2i+1, an exclusive block scan of the tile
// counts gives every expert its place in the list.
__global__ __launch_bounds__(1024) void build_mtile_list_kernel(const int32_t* __restrict__ offsets, int n_slots,
                                                                int stream_max_rows,
                                                                int32_t* __restrict__ mt_expert,
                                                                int32_t* __restrict__ mt_row0,
                                                                int32_t* __restrict__ n_mtiles, int cap) {
  __shared__ int32_t scan_s[1024];
  const int tid = threadIdx.x;
  int cnt[2], r0[2], r1[2];
#pragma unroll
  for (int i = 0; i < 2; i++) {
    const int e = 2 * tid + i;
    cnt[i] = 0;
    r0[i] = r1[i] = 0;
    if (e < n_slots) {
      r0[i] = offsets[e];
      r1[i] = offsets[e + 1];
      const int m = r1[i] - r0[i];
      if (m > stream_max_rows) cnt[i] = (m + kBM - 1) / kBM;
    }
  }
  scan_s[tid] = cnt[0] + cnt[1];
  __syncthreads();
  for (int d = 1; d < 1024; d <<= 1) {
    const int v = (tid >= d) ? scan_s[tid - d] : 0;
    __syncthreads();
    scan_s[tid] += v;
    __syncthreads();
  }
  int pos = scan_s[tid] - (cnt[0] + cnt[1]);  // exclusive prefix
#pragma unroll
  for (int i = 0; i < 2; i++) {
    for (int k = 0; k < cnt[i]; k++, pos++) {
      if (pos < cap) {
        mt_expert[pos] = 2 * tid + i;
        mt_row0[pos] = r0[i] + k * kBM;
      }
    }
  }
  if (tid == 1023) *n_mtiles = min(scan_s[1023], cap);
}

typedef __attribute__((address_space(1))) const void* gvoid;
typedef __attribute__((address_space(3))) void* lvoid;

// Asynchronous global -> LDS copy of 64 lanes x 16 bytes: lane l's 16 bytes land at dst + l*16.
__device__ __forceinline__ void dma16(const uint8_t* src_lane, uint8_t* dst_wave_uniform) {
  __builtin_amdgcn_global_load_lds((gvoid)src_lane, (lvoid)dst_wave_uniform, 16, 0, 0);
}
__device__ __forceinline__ void dma4(const float* src_lane, float* dst_wave_uniform) {
  __builtin_amdgcn_global_load_lds((gvoid)src_lane, (lvoid)dst_wave_uniform, 4, 0, 0);
}

template <bool G1>
__global__ __launch_bounds__(kTileThreads, 1) void gemm_fp8_tile_kernel(
    const dwdp_expert_ptrs* __restrict__ table, const int32_t* __restrict__ offsets, const int32_t* __restrict__ perm,
    const int32_t* __restrict__ mt_expert, const int32_t* __restrict__ mt_row0, const int32_t* __restrict__ n_mtiles,
    int n_panels, const uint8_t* __restrict__ act, const float* __restrict__ act_s, uint8_t* __restrict__ hq,
    float* __restrict__ hs, uint16_t* __restrict__ yp, int E, int T, int H, int I, int K) {
  // Two LDS images (K block kb and kb+1), each its own array so that the compiler can tell
  // a copy into one from the reads of the other.
  __shared__ __attribute__((aligned(16))) uint8_t lds_a0[kLdsA];
  __shared__ __attribute__((aligned(16))) uint8_t lds_a1[kLdsA];
  __shared__ __attribute__((aligned(16))) uint8_t lds_b0[kLdsB];
  __shared__ __attribute__((aligned(16))) uint8_t lds_b1[kLdsB];
  __shared__ __attribute__((aligned(16))) float lds_sa0[kSaLen];  // 5 waves x 64 activation scales
  __shared__ __attribute__((aligned(16))) float lds_sa1[kSaLen];
  __shared__ float lds_amax[4 * kBM];
  __shared__ int32_t lds_row[kSaLen];

  const int xcd = blockIdx.x & 7;
  const int s = blockIdx.x >> 3;
  const int mq = s / n_panels;
  const int panel = s - mq * n_panels;
  const int m = mq * 8 + xcd;
  if (m >= *n_mtiles) return;
  // wave-uniform values go through readfirstlane so that everything derived from them
  // (weight/scale pointers, tile counts) lives in scalar registers and is loaded with s_load
  const int e = __builtin_amdgcn_readfirstlane(mt_expert[m]);
  const int r0 = __builtin_amdgcn_readfirstlane(mt_row0[m]);
  const int r_end = __builtin_amdgcn_readfirstlane(offsets[e + 1]);
  const int valid = min(kBM, r_end - r0);
  const int ntt = (valid + 15) >> 4;

  const int tid = threadIdx.x;
  const int wave = tid >> 6, lane = tid & 63, lr = lane & 15, lq = lane >> 4;
  const int wn = wave & 3, wm = wave >> 2;  // wm < kWM
  const int Kdim = G1 ? H : I;  // reduction length
  const int nkb = Kdim / 128;
  const int n_tile_rows = (G1 ? 2 * I : H) / 16;
  const uint8_t* wbase = (const uint8_t*)(G1 ? table[e].w13 : table[e].w2);
  const float* sbase = G1 ? table[e].s13 : table[e].s2;

  // ---- copy sources (fixed over the K loop) ----
  // weights: 32 pieces of 1 KiB (16 LDS tiles x 2 halves), kAP per wave; LDS tile a = wn*4 + j
  constexpr int kAP = (32 + kTileWaves - 1) / kTileWaves;
  const uint8_t* a_src[kAP];
#pragma unroll
  for (int i = 0; i < kAP; i++) {
    const int c = min(wave + kTileWaves * i, 31);  // piece: tile c/2, half c&1
    const int a = c >> 1;
    const int w = a >> 2, j = a & 3;
    int tr;
    if (G1)
      tr = (j < 2 ? 0 : I / 16) + panel * 8 + 2 * w + (j & 1);
    else
      tr = min(panel * 16 + a, n_tile_rows - 1);
    a_src[i] = wbase + (size_t)tr * nkb * kTileBytes + (c & 1) * (kTileBytes / 2);  // wave-uniform
  }
  // tokens: wave w copies 1 KiB pieces c = w, w+kTileWaves, ... (piece c = token tile c/2, half c&1)
  // The source row of every token of the tile is kept in LDS (not in registers) and looked
  // up again by each copy: lds_row[i] = row of act / act_s that token i reads.
  constexpr int kBP = (2 * kTT + kTileWaves - 1) / kTileWaves;
  for (int i = tid; i < kSaLen; i += kTileThreads) {
    const int row = min(r0 + i, r_end - 1);
    lds_row[i] = G1 ? ((e < E) ? perm[row] / K : row - T * K) : row;
  }
  __syncthreads();
  // scale rows of this wave's tiles: G1 gate block / up block; GEMM-2 one block per wave pair
  const float* sw0;
  const float* sw1;
  if (G1) {
    sw0 = sbase + (size_t)panel * nkb;
    sw1 = sbase + (size_t)(I / 128 + panel) * nkb;
  } else {
    const int blk = min(panel * 2 + (wn >> 1), H / 128 - 1);
    sw0 = sw1 = sbase + (size_t)blk * nkb;
  }

  v4f acc[4][kTW];
#pragma unroll
  for (int j = 0; j < 4; j++)
#pragma unroll
    for (int t = 0; t < kTW; t++) acc[j][t] = (v4f){0.f, 0.f, 0.f, 0.f};

  auto issue = [&](uint8_t* la, uint8_t* lb, float* lsa, int kb) {
#pragma unroll
    for (int i = 0; i < kAP; i++) {
      const int c = wave + kTileWaves * i;
      if (c < 32 && !(DWDP_TILE_DBG & 4))
        dma16(a_src[i] + (size_t)kb * kTileBytes + lane * 16, la + c * (kTileBytes / 2));
    }
#pragma unroll
    for (int i = 0; i < kBP; i++) {
      const int c = wave + kTileWaves * i;
      if (c < 2 * ntt && !(DWDP_TILE_DBG & 8)) {
        const uint32_t off = (uint32_t)lds_row[(c >> 1) * 16 + lr] * Kdim + lq * 32 + (c & 1) * 16 + kb * 128;
        dma16(act + off, lb + c * (kTileBytes / 2));
      }
    }
    if (wave < 5) dma4(act_s + (size_t)lds_row[wave * 64 + lane] * nkb + kb, lsa + wave * 64);
  };

  auto compute = [&](const uint8_t* la, const uint8_t* lb, const float* lsa, int kb) {
    const float w0 = *(cf32)(sw0 + kb);
    const float w1 = *(cf32)(sw1 + kb);
    // one per-lane base per LDS array; every tile is a compile-time offset from it
    const uint8_t* pa = la + wn * 4 * kTileBytes + lane * 16;
    const uint8_t* pb = lb + wm * kTileBytes + lane * 16;
    const float* ps = lsa + wm * 16 + lr;
    v8i af[4];
#pragma unroll
    for (int j = 0; j < 4; j++)
      af[j] = cat8(*(const v4i*)(pa + j * kTileBytes), *(const v4i*)(pa + j * kTileBytes + kTileBytes / 2));
#pragma unroll
    for (int ti = 0; ti < kTW; ti++) {
      const int t = wm + kWM * ti;
      if (t < ntt) {
        const uint8_t* p = pb + ti * (kWM * kTileBytes);
        const v8i bf = cat8(*(const v4i*)p, *(const v4i*)(p + kTileBytes / 2));
        const float sa = ps[ti * (kWM * 16)];
        const float s0 = sa * w0, s1 = sa * w1;
#pragma unroll
        for (int j = 0; j < 4; j++) {
          const v4f zero = {0.f, 0.f, 0.f, 0.f};
          const v4f pr = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(af[j], bf, zero, 0, 0, 0, 0, 0, 0);
          const float sj = (j < 2) ? s0 : s1;
#pragma unroll
          for (int i = 0; i < 4; i++) acc[j][ti][i] = fmaf(pr[i], sj, acc[j][ti][i]);
        }
      }
    }
  };

  // One barrier per K block: it publishes the image copied during the previous block and
  // retires the reads of the image that the next copy overwrites.
  issue(lds_a0, lds_b0, lds_sa0, 0);
  for (int kb = 0; kb < nkb; kb += 2) {
    __syncthreads();
    if (kb + 1 < nkb && !(DWDP_TILE_DBG & 2)) issue(lds_a1, lds_b1, lds_sa1, kb + 1);
    if (!(DWDP_TILE_DBG & 1)) compute(lds_a0, lds_b0, lds_sa0, kb);
    if (kb + 1 < nkb) {
      __syncthreads();
      if (kb + 2 < nkb && !(DWDP_TILE_DBG & 2)) issue(lds_a0, lds_b0, lds_sa0, kb + 2);
      if (!(DWDP_TILE_DBG & 1)) compute(lds_a1, lds_b1, lds_sa1, kb + 1);
    }
  }

  if (G1) {
    const int njb = I / 128;
    // h = silu(gate) * up, kept in acc[0..1]
#pragma unroll
    for (int ti = 0; ti < kTW; ti++) {
      const int t = wm + kWM * ti;
      float amax = 0.f;
      if (t < ntt) {
#pragma unroll
        for (int j = 0; j < 2; j++)
#pragma unroll
          for (int i = 0; i < 4; i++) {
            const float g = acc[j][ti][i], u = acc[2 + j][ti][i];
            const float v = g / (1.f + __expf(-g)) * u;
            acc[j][ti][i] = v;
            amax = fmaxf(amax, fabsf(v));
          }
      }
      amax = fmaxf(amax, __shfl_xor(amax, 16));
      amax = fmaxf(amax, __shfl_xor(amax, 32));
      if (lq == 0 && t < kTT) lds_amax[wn * kBM + t * 16 + lr] = amax;
    }
    __syncthreads();
#pragma unroll
    for (int ti = 0; ti < kTW; ti++) {
      const int t = wm + kWM * ti;
      if (t < ntt) {
        const int tok = t * 16 + lr;
        const float amax = fmaxf(fmaxf(lds_amax[tok], lds_amax[kBM + tok]),
                                 fmaxf(lds_amax[2 * kBM + tok], lds_amax[3 * kBM + tok]));
        const float scale = amax > 0.f ? amax / 448.f : 1.f;
        const int r = r0 + tok;
        if (r < r_end) {
#pragma unroll
          for (int j = 0; j < 2; j++) {
            const uint32_t q = pack_fp8x4(acc[j][ti][0] / scale, acc[j][ti][1] / scale, acc[j][ti][2] / scale,
                                          acc[j][ti][3] / scale);
            *(uint32_t*)(hq + (size_t)r * I + panel * 128 + wn * 32 + j * 16 + lq * 4) = q;
          }
          if (wn == 0 && lq == 0) hs[(size_t)r * njb + panel] = scale;
        }
      }
    }
  } else {
#pragma unroll
    for (int j = 0; j < 4; j++) {
      const int n0 = panel * 256 + (wn * 4 + j) * 16;
      if (n0 < H) {
#pragma unroll
        for (int ti = 0; ti < kTW; ti++) {
          const int t = wm + kWM * ti;
          const int r = r0 + t * 16 + lr;
          if (t < ntt && r < r_end) {
            uint2 o;
            o.x = (uint32_t)f32_to_bf16(acc[j][ti][0]) | ((uint32_t)f32_to_bf16(acc[j][ti][1]) << 16);
            o.y = (uint32_t)f32_to_bf16(acc[j][ti][2]) | ((uint32_t)f32_to_bf16(acc[j][ti][3]) << 16);
            *(uint2*)(yp + (size_t)r * H + n0 + lq * 4) = o;
          }
        }
      }
    }
  }
}

int tile_mtiles_cap(int rows, int n_slots, int stream_max_rows) {
  // listed experts have more than stream_max_rows rows: at most rows / (stream_max_rows+1) of
  // them, each adding at most one partial tile to the rows / kBM full ones
  long by_rows = (long)rows / ((long)stream_max_rows + 1);
  return rows / kBM + (int)(by_rows < n_slots ? by_rows : n_slots) + 1;
}

void launch_build_mtile_list(const int32_t* offsets, int n_slots, int stream_max_rows, int32_t* mt_expert,
                             int32_t* mt_row0, int32_t* n_mtiles, int cap, hipStream_t stream) {
  hipLaunchKernelGGL(build_mtile_list_kernel, dim3(1), dim3(1024), 0, stream, offsets, n_slots, stream_max_rows,
                     mt_expert, mt_row0, n_mtiles, cap);
}

void launch_gemm1_fp8_tile(const GemmArgs& a, const TileSched& ts, const uint8_t* xq, const float* xs, uint8_t* hq,
                           float* hs, hipStream_t stream) {
  const int n_panels = a.I / 128;
  const int grid = 8 * ((ts.n_mt_max + 7) / 8) * n_panels;
  hipLaunchKernelGGL(gemm_fp8_tile_kernel<true>, dim3(grid), dim3(kTileThreads), 0, stream, a.table,
                     a.offsets, a.perm, ts.mt_expert, ts.mt_row0, ts.n_mtiles, n_panels, xq, xs, hq, hs,
                     (uint16_t*)nullptr, a.E, a.T, a.H, a.I, a.K);
}

void launch_gemm2_fp8_tile(const GemmArgs& a, const TileSched& ts, const uint8_t* hq, const float* hs, void* yp,
                           hipStream_t stream) {
  const int n_panels = (a.H + 255) / 256;
  const int grid = 8 * ((ts.n_mt_max + 7) / 8) * n_panels;
  hipLaunchKernelGGL(gemm_fp8_tile_kernel<false>, dim3(grid), dim3(kTileThreads), 0, stream, a.table,
                     a.offsets, a.perm, ts.mt_expert, ts.mt_row0, ts.n_mtiles, n_panels, hq, hs, (uint8_t*)nullptr,
                     (float*)nullptr, (uint16_t*)yp, a.E, a.T, a.H, a.I, a.K);
}

}  // namespace dwdp
