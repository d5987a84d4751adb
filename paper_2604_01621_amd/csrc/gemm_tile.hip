// LDS-tiled FP8 grouped GEMM for gfx950: the large-M (prefill-shaped) path.
//
// A workgroup (4 waves) computes a 256 (weight rows) x 128 (tokens) output tile of one
// expert.  Per 128-wide K block -- exactly one weight-scale block and one activation-scale
// group -- it stages 16 packed weight tiles (32 KiB, contiguous 2 KiB pieces located
// through the expert-pointer table) and 8 packed token tiles (16 KiB, rows gathered through
// the permutation) in LDS; each wave then runs 4 x 8 v_mfma_f32_16x16x128_f8f6f4 and folds
// every fp32 partial product into its accumulator with s_act[token,kb] * s_w[nblock,kb] on
// the VALU.  Global loads for K block kb+1 are in flight in registers while block kb is
// multiplied (two workgroups per CU hide the barriers of one another).
//
// Token tiles of 16 beyond the expert's row count are skipped, so padding costs LDS
// traffic only.  Workgroups are numbered so that all M tiles of one (expert, weight panel)
// run on the same XCD at about the same time and share its L2: block b runs on XCD b % 8
// and handles panel x + 8*jj, M tile m with b / 8 = jj * n_mt_max + m.
//
// GEMM-1 (G1): rows = 128 gate + 128 up rows of W13, epilogue silu(g)*u, per-token amax
// over the block's 128 h columns, e4m3 quantisation of h.  GEMM-2: rows = 256 rows of W2,
// epilogue bf16 store.  Experts with few rows are left to the streaming kernels (they are not listed).
#include "dwdp_kernels.h"

namespace dwdp {

constexpr int kBM = 128;          // tokens per workgroup tile
constexpr int kTT = kBM / 16;     // token tiles per workgroup
constexpr int kTileThreads = 256;

typedef const __attribute__((address_space(1))) v4i* gv4i;
typedef const __attribute__((address_space(1))) float* gf32;
typedef __attribute__((address_space(3))) v4i* lv4i;

__device__ __forceinline__ v8i cat8(v4i lo, v4i hi) { return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7); }

// One thread lists the M tiles of all experts that have more than stream_max_rows rows.
__global__ __launch_bounds__(1024) void build_mtile_list_kernel(const int32_t* __restrict__ offsets, int n_slots,
                                                                int stream_max_rows,
                                                                int32_t* __restrict__ mt_expert,
                                                                int32_t* __restrict__ mt_row0,
                                                                int32_t* __restrict__ n_mtiles, int cap) {
  __shared__ int32_t off_s[1026];
  for (int i = threadIdx.x; i <= n_slots; i += blockDim.x) off_s[i] = offsets[i];
  __syncthreads();
  if (threadIdx.x == 0) {
    int n = 0;
    for (int e = 0; e < n_slots; e++) {
      const int m = off_s[e + 1] - off_s[e];
      if (m <= stream_max_rows) continue;
      for (int r = off_s[e]; r < off_s[e + 1] && n < cap; r += kBM) {
        mt_expert[n] = e;
        mt_row0[n] = r;
        n++;
      }
    }
    *n_mtiles = n;
  }
}

template <bool G1>
__global__ __launch_bounds__(kTileThreads, 2) void gemm_fp8_tile_kernel(
    const dwdp_expert_ptrs* __restrict__ table, const int32_t* __restrict__ offsets, const int32_t* __restrict__ perm,
    const int32_t* __restrict__ mt_expert, const int32_t* __restrict__ mt_row0, const int32_t* __restrict__ n_mtiles,
    int n_mt_max, int n_panels, const uint8_t* __restrict__ act, const float* __restrict__ act_s,
    uint8_t* __restrict__ hq, float* __restrict__ hs, uint16_t* __restrict__ yp, int E, int T, int H, int I, int K) {
  __shared__ __attribute__((aligned(16))) uint8_t lds_a[16 * kTileBytes];
  __shared__ __attribute__((aligned(16))) uint8_t lds_b[kTT * kTileBytes];
  __shared__ float lds_sa[kBM];
  __shared__ float lds_amax[4][kBM];

  const int xcd = blockIdx.x & 7;
  const int s = blockIdx.x >> 3;
  const int jj = s / n_mt_max;
  const int m = s - jj * n_mt_max;
  const int panel = xcd + 8 * jj;
  if (panel >= n_panels || m >= *n_mtiles) return;
  const int e = mt_expert[m];
  const int r0 = mt_row0[m];
  const int r_end = offsets[e + 1];
  const int valid = min(kBM, r_end - r0);
  const int ntt = (valid + 15) >> 4;

  const int tid = threadIdx.x;
  const int wave = tid >> 6, lane = tid & 63, lr = lane & 15, lq = lane >> 4;
  const int Kdim = G1 ? H : I;           // reduction length
  const int nkb = Kdim / 128;
  const int n_tile_rows = (G1 ? 2 * I : H) / 16;
  const uint8_t* wbase = (const uint8_t*)(G1 ? table[e].w13 : table[e].w2);
  const float* sbase = G1 ? table[e].s13 : table[e].s2;

  // ---- loader addresses (fixed over the K loop) ----
  const int within = tid & 127;
  uint32_t a_src[8];  // byte offsets from wbase / act: 32-bit to keep the loop's address registers few
#pragma unroll
  for (int i = 0; i < 8; i++) {
    const int a = (tid >> 7) + 2 * i;  // LDS tile 0..15 = wave*4 + j
    const int w = a >> 2, j = a & 3;
    int tr;
    if (G1)
      tr = (j < 2 ? 0 : I / 16) + panel * 8 + 2 * w + (j & 1);
    else
      tr = min(panel * 16 + a, n_tile_rows - 1);
    a_src[i] = (uint32_t)tr * nkb * kTileBytes + within * 16;
  }
  uint32_t b_src[4];
#pragma unroll
  for (int i = 0; i < 4; i++) {
    const int tt = (tid >> 7) + 2 * i;
    const int half = within >> 6, l = within & 63;
    const int row = min(r0 + tt * 16 + (l & 15), r_end - 1);
    const int src_row = G1 ? ((e < E) ? perm[row] / K : row - T * K) : row;
    b_src[i] = (uint32_t)src_row * Kdim + (l >> 4) * 32 + half * 16;
  }
  const float* sa_src;
  {
    const int row = min(r0 + (tid & 127), r_end - 1);
    const int src_row = G1 ? ((e < E) ? perm[row] / K : row - T * K) : row;
    sa_src = act_s + (size_t)src_row * nkb;
  }
  // scale rows of this wave's tiles: G1 gate block / up block; GEMM-2 one block per wave pair
  const float* sw0;
  const float* sw1;
  if (G1) {
    sw0 = sbase + (size_t)panel * nkb;
    sw1 = sbase + (size_t)(I / 128 + panel) * nkb;
  } else {
    const int blk = min(panel * 2 + (wave >> 1), H / 128 - 1);
    sw0 = sw1 = sbase + (size_t)blk * nkb;
  }

  v4f acc[4][kTT];
#pragma unroll
  for (int j = 0; j < 4; j++)
#pragma unroll
    for (int t = 0; t < kTT; t++) acc[j][t] = (v4f){0.f, 0.f, 0.f, 0.f};

  v4i ra[8], rb[4];
  float rsa;
#pragma unroll
  for (int i = 0; i < 8; i++) ra[i] = __builtin_nontemporal_load((gv4i)(wbase + a_src[i]));
#pragma unroll
  for (int i = 0; i < 4; i++) rb[i] = *(gv4i)(act + b_src[i]);
  rsa = *(gf32)sa_src;

  for (int kb = 0; kb < nkb; kb++) {
    // registers -> LDS
#pragma unroll
    for (int i = 0; i < 8; i++) *(v4i*)(lds_a + ((tid >> 7) + 2 * i) * kTileBytes + within * 16) = ra[i];
#pragma unroll
    for (int i = 0; i < 4; i++) *(v4i*)(lds_b + ((tid >> 7) + 2 * i) * kTileBytes + within * 16) = rb[i];
    if (tid < kBM) lds_sa[tid] = rsa;
    __syncthreads();
    // next K block's global loads fly during the MFMAs (the last round re-reads block nkb-1)
    {
      const int kn = min(kb + 1, nkb - 1);
#pragma unroll
      for (int i = 0; i < 8; i++) ra[i] = __builtin_nontemporal_load((gv4i)(wbase + (a_src[i] + (uint32_t)kn * kTileBytes)));
#pragma unroll
      for (int i = 0; i < 4; i++) rb[i] = *(gv4i)(act + (b_src[i] + (uint32_t)kn * 128));
      rsa = *(gf32)(sa_src + kn);
    }
    const float w0 = *(gf32)(sw0 + kb);
    const float w1 = *(gf32)(sw1 + kb);
    v8i af[4];
#pragma unroll
    for (int j = 0; j < 4; j++) {
      const uint8_t* p = lds_a + (wave * 4 + j) * kTileBytes + lane * 16;
      af[j] = cat8(*(const v4i*)p, *(const v4i*)(p + kTileBytes / 2));
    }
#pragma unroll
    for (int t = 0; t < kTT; t++) {
      if (t < ntt) {
        const uint8_t* p = lds_b + t * kTileBytes + lane * 16;
        const v8i bf = cat8(*(const v4i*)p, *(const v4i*)(p + kTileBytes / 2));
        const float sa = lds_sa[t * 16 + lr];
        const float s0 = sa * w0, s1 = sa * w1;
#pragma unroll
        for (int j = 0; j < 4; j++) {
          const v4f zero = {0.f, 0.f, 0.f, 0.f};
          const v4f pr = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(af[j], bf, zero, 0, 0, 0, 0, 0, 0);
          const float sj = (j < 2) ? s0 : s1;
#pragma unroll
          for (int i = 0; i < 4; i++) acc[j][t][i] = fmaf(pr[i], sj, acc[j][t][i]);
        }
      }
    }
    __syncthreads();  // everyone is done with this K block's LDS image
  }

  if (G1) {
    const int njb = I / 128;
    // h = silu(gate) * up, kept in acc[0..1]
#pragma unroll
    for (int t = 0; t < kTT; t++) {
      float amax = 0.f;
      if (t < ntt) {
#pragma unroll
        for (int j = 0; j < 2; j++)
#pragma unroll
          for (int i = 0; i < 4; i++) {
            const float g = acc[j][t][i], u = acc[2 + j][t][i];
            const float v = g / (1.f + __expf(-g)) * u;
            acc[j][t][i] = v;
            amax = fmaxf(amax, fabsf(v));
          }
      }
      amax = fmaxf(amax, __shfl_xor(amax, 16));
      amax = fmaxf(amax, __shfl_xor(amax, 32));
      if (lq == 0) lds_amax[wave][t * 16 + lr] = amax;
    }
    __syncthreads();
#pragma unroll
    for (int t = 0; t < kTT; t++) {
      if (t < ntt) {
        const int tok = t * 16 + lr;
        const float amax =
            fmaxf(fmaxf(lds_amax[0][tok], lds_amax[1][tok]), fmaxf(lds_amax[2][tok], lds_amax[3][tok]));
        const float scale = amax > 0.f ? amax / 448.f : 1.f;
        const int r = r0 + tok;
        if (r < r_end) {
#pragma unroll
          for (int j = 0; j < 2; j++) {
            const uint32_t q = pack_fp8x4(acc[j][t][0] / scale, acc[j][t][1] / scale, acc[j][t][2] / scale,
                                          acc[j][t][3] / scale);
            *(uint32_t*)(hq + (size_t)r * I + panel * 128 + wave * 32 + j * 16 + lq * 4) = q;
          }
          if (wave == 0 && lq == 0) hs[(size_t)r * njb + panel] = scale;
        }
      }
    }
  } else {
#pragma unroll
    for (int j = 0; j < 4; j++) {
      const int n0 = panel * 256 + (wave * 4 + j) * 16;
      if (n0 < H) {
#pragma unroll
        for (int t = 0; t < kTT; t++) {
          const int r = r0 + t * 16 + lr;
          if (t < ntt && r < r_end) {
            uint2 o;
            o.x = (uint32_t)f32_to_bf16(acc[j][t][0]) | ((uint32_t)f32_to_bf16(acc[j][t][1]) << 16);
            o.y = (uint32_t)f32_to_bf16(acc[j][t][2]) | ((uint32_t)f32_to_bf16(acc[j][t][3]) << 16);
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
  const int grid = 8 * ((n_panels + 7) / 8) * ts.n_mt_max;
  hipLaunchKernelGGL(gemm_fp8_tile_kernel<true>, dim3(grid), dim3(kTileThreads), 0, stream, a.table, a.offsets, a.perm,
                     ts.mt_expert, ts.mt_row0, ts.n_mtiles, ts.n_mt_max, n_panels, xq, xs, hq, hs, (uint16_t*)nullptr,
                     a.E, a.T, a.H, a.I, a.K);
}

void launch_gemm2_fp8_tile(const GemmArgs& a, const TileSched& ts, const uint8_t* hq, const float* hs, void* yp,
                           hipStream_t stream) {
  const int n_panels = (a.H + 255) / 256;
  const int grid = 8 * ((n_panels + 7) / 8) * ts.n_mt_max;
  hipLaunchKernelGGL(gemm_fp8_tile_kernel<false>, dim3(grid), dim3(kTileThreads), 0, stream, a.table, a.offsets,
                     a.perm, ts.mt_expert, ts.mt_row0, ts.n_mtiles, ts.n_mt_max, n_panels, hq, hs, (uint8_t*)nullptr,
                     (float*)nullptr, (uint16_t*)yp, a.E, a.T, a.H, a.I, a.K);
}

}  // namespace dwdp
