// Weight-streaming grouped GEMM for MXFP4 weights (FP4 E2M1 codes, one E8M0 scale per 32
// elements along K: OCP Microscaling Formats v1.0) -- the gfx950 analogue of the NVFP4 weights
// of the paper's model (its Section 5.1).  Same task decomposition as the FP8 streaming kernels;
// what changes is the matrix-core operand and who applies the weight scale.
//
// v_mfma_scale_f32_16x16x128_f8f6f4 with an FP4 A operand and an FP8 B operand (measured on
// this part with single-element probes):
//   * A (weights): lane (lr = lane % 16, lq = lane / 16) holds row lr, K = 32*lq .. 32*lq+31 as
//     32 nibbles in 4 registers, element k in nibble k (low nibble of a byte first).  That is
//     exactly one MX block, and byte `opsel` of the lane's scale register is its E8M0 scale:
//     the hardware multiplies by 2^(byte-127) inside the instruction.
//   * B (activations, e4m3): lane (n, lq) holds token n; registers 0..3 are K = 16*lq .. +15 and
//     registers 4..7 are K = 64 + 16*lq .. +15 (with two 8-bit operands any consistent order
//     works, with a 4-bit A operand this one is imposed).
//   * D: lane holds rows 4*(lane/16) + i of A, column lane % 16 of B, as for FP8.
// The activation scale (fp32, per token per 128) is still applied on the VALU.
//
// Device layout written by the pack kernels below:
//   codes:  tile (tr, kb) = 16 rows x 128 K = 1 KiB at ((tr * nkb) + kb) * 1024; lane l's 16
//           bytes at l*16 = row tr*16 + l%16, packed bytes [kb*64 + (l/16)*16, +16) of the row.
//   scales: for tile row tr and group g of four K blocks, 256 bytes at (tr * ng + g) * 256:
//           lane l's dword at l*4, byte j = scale of (row tr*16 + l%16, K block 4g+j, sub-block
//           l/16).  ng = ceil(nkb / 4); groups are padded with 127 (= 1.0).
// One dword load per lane and tile therefore brings the scales of four K blocks, and the K loop
// is unrolled by four so that `opsel` is the immediate the instruction needs.
#include "dwdp_kernels.h"

namespace dwdp {

constexpr int kMxTileBytes = 1024;
constexpr int kMxThreads = 256;

typedef const __attribute__((address_space(1))) v4i* gv4i;
typedef const __attribute__((address_space(1))) int* gi32;
typedef const __attribute__((address_space(1))) float* gf32;

__device__ __forceinline__ v8i widen(v4i lo) { return (v8i){lo[0], lo[1], lo[2], lo[3], 0, 0, 0, 0}; }
__device__ __forceinline__ v8i cat_mx(v4i lo, v4i hi) { return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7); }

// One pipeline stage: two K blocks of operands for NT weight tiles and one group of 16 token
// rows, with the scale dwords of the group of four K blocks they belong to.
template <int NT>
struct MxStage {
  v4i w[2][NT];
  v4i x[2][2];
  float sa[2];
  int sc[NT];
};

// wt[j]: this lane's address inside K block 0 of tile row j (tile base + lane*16); xrow: token
// row + (lane/16)*16; stage s = K blocks 2s, 2s+1; blocks past nkb-1 re-read block nkb-1 (they
// are not multiplied).
template <int NT>
__device__ __forceinline__ void mx_load(MxStage<NT>& f, const uint8_t* const (&wt)[NT], const uint8_t* xrow,
                                        const float* xsrow, int s, int nkb) {
#pragma unroll
  for (int u = 0; u < 2; u++) {
    const int kb = min(2 * s + u, nkb - 1);
#pragma unroll
    for (int j = 0; j < NT; j++) f.w[u][j] = __builtin_nontemporal_load((gv4i)(wt[j] + (size_t)kb * kMxTileBytes));
    const uint8_t* px = xrow + (size_t)kb * 128;
    f.x[u][0] = *(gv4i)px;
    f.x[u][1] = *(gv4i)(px + 64);
    f.sa[u] = *(gf32)(xsrow + kb);
  }
}
// st[j]: this lane's dword inside scale group 0 of tile row j
template <int NT>
__device__ __forceinline__ void mx_load_scales(MxStage<NT>& f, const uint8_t* const (&st)[NT], int g) {
#pragma unroll
  for (int j = 0; j < NT; j++) f.sc[j] = *(gi32)(st[j] + (size_t)g * 256);
}

// K block U (0 or 1) of the stage; SEL = that block's byte in the scale dwords (0..3)
template <int NT, int U, int SEL>
__device__ __forceinline__ void mx_mma_block(const MxStage<NT>& f, v4f (&acc)[NT]) {
  const v8i b = cat_mx(f.x[U][0], f.x[U][1]);
#pragma unroll
  for (int j = 0; j < NT; j++) {
    const v4f zero = {0.f, 0.f, 0.f, 0.f};
    // cbsz 4: A is FP4 E2M1; blgp 0: B is FP8 E4M3; A scale = byte SEL of sc[j]; B scale 127 = 1.0
    const v4f p = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(widen(f.w[U][j]), b, zero, 4, 0, SEL, f.sc[j], 0,
                                                                    0x7f7f7f7f);
#pragma unroll
    for (int i = 0; i < 4; i++) acc[j][i] = fmaf(p[i], f.sa[U], acc[j][i]);
  }
}

// HALF = 0: the stage holds blocks 4g, 4g+1 of its group; 1: blocks 4g+2, 4g+3
template <int NT, int HALF>
__device__ __forceinline__ void mx_mma(const MxStage<NT>& f, v4f (&acc)[NT], int s, int nkb) {
  const int left = nkb - 2 * s;  // wave-uniform
  if (left > 0) mx_mma_block<NT, 0, 2 * HALF>(f, acc);
  if (left > 1) mx_mma_block<NT, 1, 2 * HALF + 1>(f, acc);
}

// Two stages alternate: the loads of one are in flight behind the MFMAs of the other.  Even
// stages are the first half of a scale group, odd stages the second half, so each buffer's
// byte selectors are compile-time constants.
template <int NT>
__device__ __forceinline__ void mx_mainloop(const uint8_t* const (&wt)[NT], const uint8_t* const (&st)[NT],
                                            const uint8_t* xrow, const float* xsrow, int nkb, v4f (&acc)[NT]) {
  const int ng = (nkb + 3) >> 2;
  const int nst = 2 * ng;
  MxStage<NT> f0, f1;
  mx_load_scales<NT>(f0, st, 0);
  mx_load<NT>(f0, wt, xrow, xsrow, 0, nkb);
  int s = 0;
  for (; s + 2 < nst; s += 2) {
#pragma unroll
    for (int j = 0; j < NT; j++) f1.sc[j] = f0.sc[j];  // same group
    mx_load<NT>(f1, wt, xrow, xsrow, s + 1, nkb);
    mx_mma<NT, 0>(f0, acc, s, nkb);
    mx_load_scales<NT>(f0, st, s / 2 + 1);
    mx_load<NT>(f0, wt, xrow, xsrow, s + 2, nkb);
    mx_mma<NT, 1>(f1, acc, s + 1, nkb);
  }
  // last group: nothing left to load for f0 (a clamped re-read would still take request slots)
#pragma unroll
  for (int j = 0; j < NT; j++) f1.sc[j] = f0.sc[j];
  mx_load<NT>(f1, wt, xrow, xsrow, s + 1, nkb);
  mx_mma<NT, 0>(f0, acc, s, nkb);
  mx_mma<NT, 1>(f1, acc, s + 1, nkb);
}

// GEMM-1: task = (expert slot e, block jb of 128 h columns); wave w owns gate tiles 2w, 2w+1 and
// the up tiles of the same h columns.  Epilogue as for FP8 weights: h = silu(g) * u, per-token
// amax over the 128 columns, e4m3 quantisation.
__global__ __launch_bounds__(kMxThreads, 2) void gemm1_mx_stream_kernel(
    const dwdp_expert_ptrs* __restrict__ table, const int32_t* __restrict__ offsets, const int32_t* __restrict__ perm,
    const uint8_t* __restrict__ xq, const float* __restrict__ xs, uint8_t* __restrict__ hq, float* __restrict__ hs,
    int E, int T, int H, int I, int K, int max_rows) {
  __shared__ float amax_s[4][16];
  const int njb = I / 128;
  const int e = blockIdx.x / njb;
  const int jb = blockIdx.x - e * njb;
  const int r0 = offsets[e];
  const int r1 = offsets[e + 1];
  if (r1 <= r0 || r1 - r0 > max_rows) return;  // no tokens: weights never touched; many: tiled kernel
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, lr = lane & 15, lq = lane >> 4;
  const int nkb = H / 128;
  const int ng = (nkb + 3) >> 2;
  const uint8_t* w13 = (const uint8_t*)table[e].w13;
  const uint8_t* s13 = (const uint8_t*)table[e].s13;
  const uint8_t* wt[4];
  const uint8_t* st[4];
#pragma unroll
  for (int j = 0; j < 4; j++) {
    const int tile_row = ((j < 2 ? 0 : I) + jb * 128 + wave * 32 + (j & 1) * 16) / 16;
    wt[j] = w13 + (size_t)tile_row * nkb * kMxTileBytes + lane * 16;
    st[j] = s13 + (size_t)tile_row * ng * 256 + lane * 4;
  }
  for (int rt = r0; rt < r1; rt += 16) {
    const int r = rt + lr;
    const int rc = min(r, r1 - 1);  // surplus columns repeat the last row and are not stored
    const int tok = (e < E) ? perm[rc] / K : rc - T * K;
    const uint8_t* xrow = xq + (size_t)tok * H + lq * 16;
    const float* xsrow = xs + (size_t)tok * nkb;
    v4f acc[4];
#pragma unroll
    for (int j = 0; j < 4; j++) acc[j] = (v4f){0.f, 0.f, 0.f, 0.f};
    mx_mainloop<4>(wt, st, xrow, xsrow, nkb, acc);

    float h[2][4];
    float amax = 0.f;
#pragma unroll
    for (int j = 0; j < 2; j++)
#pragma unroll
      for (int i = 0; i < 4; i++) {
        const float g = acc[j][i], u = acc[2 + j][i];
        const float v = g / (1.f + __expf(-g)) * u;
        h[j][i] = v;
        amax = fmaxf(amax, fabsf(v));
      }
    amax = fmaxf(amax, __shfl_xor(amax, 16));
    amax = fmaxf(amax, __shfl_xor(amax, 32));
    if (lq == 0) amax_s[wave][lr] = amax;
    __syncthreads();
    amax = fmaxf(fmaxf(amax_s[0][lr], amax_s[1][lr]), fmaxf(amax_s[2][lr], amax_s[3][lr]));
    const float scale = amax > 0.f ? amax / 448.f : 1.f;
    if (r < r1) {
#pragma unroll
      for (int j = 0; j < 2; j++) {
        const uint32_t q = pack_fp8x4(h[j][0] / scale, h[j][1] / scale, h[j][2] / scale, h[j][3] / scale);
        *(uint32_t*)(hq + (size_t)r * I + jb * 128 + wave * 32 + j * 16 + lq * 4) = q;
      }
      if (wave == 0 && lq == 0) hs[(size_t)r * njb + jb] = scale;
    }
    __syncthreads();  // amax_s is reused by the next token tile
  }
}

// GEMM-2: task = (expert slot e, block nb of 128 output rows); wave w owns two 16-row tiles.
constexpr int kMxG2Tiles = 2;
constexpr int kMxG2Rows = 4 * kMxG2Tiles * 16;
__global__ __launch_bounds__(kMxThreads, 2) void gemm2_mx_stream_kernel(
    const dwdp_expert_ptrs* __restrict__ table, const int32_t* __restrict__ offsets, const uint8_t* __restrict__ hq,
    const float* __restrict__ hs, uint16_t* __restrict__ yp, int H, int I, int max_rows) {
  const int nnb = H / kMxG2Rows;  // H is a multiple of 128
  const int e = blockIdx.x / nnb;
  const int nb = blockIdx.x - e * nnb;
  const int r0 = offsets[e];
  const int r1 = offsets[e + 1];
  if (r1 <= r0 || r1 - r0 > max_rows) return;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, lr = lane & 15, lq = lane >> 4;
  const int nkb = I / 128;
  const int ng = (nkb + 3) >> 2;
  const int row0 = nb * kMxG2Rows + wave * (kMxG2Tiles * 16);
  const uint8_t* w2 = (const uint8_t*)table[e].w2;
  const uint8_t* s2 = (const uint8_t*)table[e].s2;
  const uint8_t* wt[kMxG2Tiles];
  const uint8_t* st[kMxG2Tiles];
#pragma unroll
  for (int j = 0; j < kMxG2Tiles; j++) {
    wt[j] = w2 + (size_t)(row0 / 16 + j) * nkb * kMxTileBytes + lane * 16;
    st[j] = s2 + (size_t)(row0 / 16 + j) * ng * 256 + lane * 4;
  }
  for (int rt = r0; rt < r1; rt += 16) {
    const int r = rt + lr;
    const int rc = min(r, r1 - 1);
    const uint8_t* xrow = hq + (size_t)rc * I + lq * 16;
    const float* xsrow = hs + (size_t)rc * nkb;
    v4f acc[kMxG2Tiles];
#pragma unroll
    for (int j = 0; j < kMxG2Tiles; j++) acc[j] = (v4f){0.f, 0.f, 0.f, 0.f};
    mx_mainloop<kMxG2Tiles>(wt, st, xrow, xsrow, nkb, acc);
    if (r < r1) {
#pragma unroll
      for (int j = 0; j < kMxG2Tiles; j++) {
        uint2 o;
        o.x = (uint32_t)f32_to_bf16(acc[j][0]) | ((uint32_t)f32_to_bf16(acc[j][1]) << 16);
        o.y = (uint32_t)f32_to_bf16(acc[j][2]) | ((uint32_t)f32_to_bf16(acc[j][3]) << 16);
        *(uint2*)(yp + (size_t)r * H + row0 + j * 16 + lq * 4) = o;
      }
    }
  }
}

void launch_gemm1_mx(const GemmArgs& a, int max_rows, const uint8_t* xq, const float* xs, uint8_t* hq, float* hs,
                     hipStream_t stream) {
  if (a.T <= 0) return;
  hipLaunchKernelGGL(gemm1_mx_stream_kernel, dim3(a.n_slots * (a.I / 128)), dim3(kMxThreads), 0, stream, a.table,
                     a.offsets, a.perm, xq, xs, hq, hs, a.E, a.T, a.H, a.I, a.K, max_rows);
}

void launch_gemm2_mx(const GemmArgs& a, int max_rows, const uint8_t* hq, const float* hs, void* yp,
                     hipStream_t stream) {
  if (a.T <= 0) return;
  hipLaunchKernelGGL(gemm2_mx_stream_kernel, dim3(a.n_slots * (a.H / kMxG2Rows)), dim3(kMxThreads), 0, stream,
                     a.table, a.offsets, hq, hs, (uint16_t*)yp, a.H, a.I, max_rows);
}

// Row-major packed codes [rows, cols/2] -> tile-major.  One thread per 16-byte piece of dst.
__global__ __launch_bounds__(256) void pack_mx_codes_kernel(const uint8_t* __restrict__ src, uint8_t* __restrict__ dst,
                                                            long n16, int cols) {
  const long o = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (o >= n16) return;
  const int nkb = cols / 128;
  const long tile = o >> 6;
  const int l = (int)(o & 63), lr = l & 15, lq = l >> 4;
  const long tr = tile / nkb;
  const int kb = (int)(tile - tr * nkb);
  *(v4i*)(dst + o * 16) = *(const v4i*)(src + (size_t)(tr * 16 + lr) * (cols / 2) + kb * 64 + lq * 16);
}

// Row-major scales [rows, cols/32] -> groups of four K blocks per lane.  One thread per dword of dst.
__global__ __launch_bounds__(256) void pack_mx_scales_kernel(const uint8_t* __restrict__ src, uint32_t* __restrict__ dst,
                                                             long n4, int cols) {
  const long o = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (o >= n4) return;
  const int nkb = cols / 128, ng = (nkb + 3) >> 2, nsc = cols / 32;
  const int l = (int)(o & 63), lr = l & 15, lq = l >> 4;
  const long grp = o >> 6;
  const long tr = grp / ng;
  const int g = (int)(grp - tr * ng);
  uint32_t v = 0;
#pragma unroll
  for (int j = 0; j < 4; j++) {
    const int kb = 4 * g + j;
    const uint32_t b = kb < nkb ? src[(size_t)(tr * 16 + lr) * nsc + kb * 4 + lq] : 127u;
    v |= b << (8 * j);
  }
  dst[o] = v;
}

void launch_pack_mxfp4(const void* codes, const void* scales, void* codes_out, void* scales_out, long rows, int cols,
                       hipStream_t stream) {
  const long n16 = rows * (cols / 2) / 16;
  if (n16 <= 0) return;
  hipLaunchKernelGGL(pack_mx_codes_kernel, dim3((unsigned)((n16 + 255) / 256)), dim3(256), 0, stream,
                     (const uint8_t*)codes, (uint8_t*)codes_out, n16, cols);
  const long n4 = (rows / 16) * (((cols / 128) + 3) / 4) * 64;
  hipLaunchKernelGGL(pack_mx_scales_kernel, dim3((unsigned)((n4 + 255) / 256)), dim3(256), 0, stream,
                     (const uint8_t*)scales, (uint32_t*)scales_out, n4, cols);
}

}  // namespace dwdp
