// Weight-streaming grouped GEMM for gfx950: the small-M (decode-shaped) path.
//
// With a handful of tokens per expert the layer is bound by reading each activated
// expert's weights from HBM exactly once.  The kernels below therefore treat the weights
// as a stream: a workgroup owns a panel of 128 weight rows of one expert (located through
// the expert-pointer table, so resident and staged experts look the same), every lane
// loads its 32-byte slice of a 16x128 MFMA operand straight from global memory into
// registers (no LDS: nothing is reused between waves), and 2*kU K-blocks of loads are kept
// in flight per wave while v_mfma_f32_16x16x128_f8f6f4 consumes the previous ones.
//
// FP8 weights are stored tile-major (see pack_fp8_tiles_kernel): the 2 KiB of one
// (16 rows x 128 k) tile are contiguous and ordered so that the two 16-byte loads of a
// wave cover 1 KiB each with lane l at byte l*16.  A row-major matrix read with the MFMA
// lane mapping touches 16 different rows per quarter wave and reached only 5.5 TB/s on
// this part against 7.0 TB/s for contiguous 1 KiB requests.
//
// Operand roles: A = weights (16 rows n x 128 k), B = activations (128 k x 16 tokens), so a
// lane's 4 accumulators are 4 consecutive n for ONE token (lane & 15).  One MFMA covers
// exactly one 128-wide K block, i.e. one weight-scale block and one activation-scale
// group; its fp32 result is multiplied by s_act[token,kb] * s_w[nblock,kb] and added to the
// running accumulator on the VALU.
//
// Experts with more than 16 tokens loop over 16-token tiles and re-stream the panel (served
// by L2 / Infinity Cache); large-M workloads use the LDS-tiled kernel instead.
#include "dwdp_kernels.h"

namespace dwdp {

constexpr int kU = 2;  // K blocks per pipeline half
constexpr int kStreamThreads = 256;

typedef const __attribute__((address_space(1))) v4i* gv4i;
typedef const __attribute__((address_space(1))) float* gf32;

template <int NT, int SG>
struct Frag {
  v4i w[NT][2];
  v4i x[2];
  float sa;
  float sw[SG];
};

__device__ __forceinline__ v8i cat(v4i lo, v4i hi) { return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7); }

// wt[j]: this lane's address inside K-block 0 of packed tile row j (tile base + lane*16);
// consecutive K blocks of a tile row are 2 KiB apart.  Tile j uses scale group j / (NT/SG).
template <int NT, int SG>
__device__ __forceinline__ void load_frag(Frag<NT, SG>& f, const uint8_t* const (&wt)[NT], const float* const (&swp)[SG],
                                          const uint8_t* xrow, const float* xsrow, int kb) {
#pragma unroll
  for (int j = 0; j < NT; j++) {
    const uint8_t* p = wt[j] + (size_t)kb * kTileBytes;
    f.w[j][0] = __builtin_nontemporal_load((gv4i)p);
    f.w[j][1] = __builtin_nontemporal_load((gv4i)(p + kTileBytes / 2));
  }
  const uint8_t* px = xrow + (size_t)kb * 128;
  f.x[0] = *(gv4i)px;
  f.x[1] = *(gv4i)(px + 16);
  f.sa = *(gf32)(xsrow + kb);
#pragma unroll
  for (int g = 0; g < SG; g++) f.sw[g] = *(gf32)(swp[g] + kb);
}

template <int NT, int SG>
__device__ __forceinline__ void mma_frag(const Frag<NT, SG>& f, v4f (&acc)[NT]) {
  const v8i b = cat(f.x[0], f.x[1]);
  float s[SG];
#pragma unroll
  for (int g = 0; g < SG; g++) s[g] = f.sa * f.sw[g];
#pragma unroll
  for (int j = 0; j < NT; j++) {
    const v4f zero = {0.f, 0.f, 0.f, 0.f};
    v4f p = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(cat(f.w[j][0], f.w[j][1]), b, zero, 0, 0, 0, 0, 0, 0);
    const float sj = s[j / (NT / SG)];
#pragma unroll
    for (int i = 0; i < 4; i++) acc[j][i] = fmaf(p[i], sj, acc[j][i]);
  }
}

// Branch-free steady state (so the compiler can count outstanding loads and let the next
// batch stay in flight behind the MFMAs), a last round without loads for the batch after it,
// plain loop for a tail of nkb % (2*kU) blocks.
template <int NT, int SG>
__device__ __forceinline__ void stream_mainloop(const uint8_t* const (&wt)[NT], const float* const (&swp)[SG],
                                                const uint8_t* xrow, const float* xsrow, int nkb, v4f (&acc)[NT]) {
  constexpr int kStep = 2 * kU;
  const int nmain = (nkb / kStep) * kStep;
  if (nmain > 0) {
    Frag<NT, SG> f0[kU], f1[kU];
#pragma unroll
    for (int u = 0; u < kU; u++) load_frag<NT, SG>(f0[u], wt, swp, xrow, xsrow, u);
    int kb0 = 0;
    for (; kb0 + kStep < nmain; kb0 += kStep) {
#pragma unroll
      for (int u = 0; u < kU; u++) load_frag<NT, SG>(f1[u], wt, swp, xrow, xsrow, kb0 + kU + u);
#pragma unroll
      for (int u = 0; u < kU; u++) mma_frag<NT, SG>(f0[u], acc);
#pragma unroll
      for (int u = 0; u < kU; u++) load_frag<NT, SG>(f0[u], wt, swp, xrow, xsrow, kb0 + kStep + u);
#pragma unroll
      for (int u = 0; u < kU; u++) mma_frag<NT, SG>(f1[u], acc);
    }
    // last round: nothing left to load for f0 (a clamped re-read would still take request slots)
#pragma unroll
    for (int u = 0; u < kU; u++) load_frag<NT, SG>(f1[u], wt, swp, xrow, xsrow, kb0 + kU + u);
#pragma unroll
    for (int u = 0; u < kU; u++) mma_frag<NT, SG>(f0[u], acc);
#pragma unroll
    for (int u = 0; u < kU; u++) mma_frag<NT, SG>(f1[u], acc);
  }
  for (int kb = nmain; kb < nkb; kb++) {
    Frag<NT, SG> f;
    load_frag<NT, SG>(f, wt, swp, xrow, xsrow, kb);
    mma_frag<NT, SG>(f, acc);
  }
}

// Task = (expert slot e, block jb of 128 h columns): gate rows jb*128.., up rows I + jb*128..
// Wave w of kG1Waves owns kG1T gate tiles and the kG1T up tiles of the same h columns
// (h columns jb*128 + w*16*kG1T + ..): tiles 0..kG1T-1 gate, kG1T..2*kG1T-1 up.
// (8 waves with one tile pair each, or other pipeline depths, measure the same within 3 %)
constexpr int kG1Waves = 4;
constexpr int kG1T = 8 / kG1Waves;
constexpr int kG1Threads = 64 * kG1Waves;
__device__ __forceinline__ void gemm1_fp8_stream_item(
    int block, float (*amax_s)[16], const dwdp_expert_ptrs* __restrict__ table, const int32_t* __restrict__ offsets,
    const int32_t* __restrict__ perm, const uint8_t* __restrict__ xq, const float* __restrict__ xs,
    uint8_t* __restrict__ hq, float* __restrict__ hs, int E, int T, int H, int I, int K, int max_rows) {
  const int njb = I / 128;
  const int e = block / njb;
  const int jb = block - e * njb;
  const int r0 = offsets[e];
  const int r1 = offsets[e + 1];
  if (r1 <= r0 || r1 - r0 > max_rows) return;  // no tokens: weights never touched; many: tiled kernel
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, lr = lane & 15, lq = lane >> 4;
  const int nkb = H / 128;
  const uint8_t* w13 = (const uint8_t*)table[e].w13;
  const float* s13 = table[e].s13;
  const uint8_t* wt[2 * kG1T];
#pragma unroll
  for (int j = 0; j < 2 * kG1T; j++) {
    const int tile_row = ((j < kG1T ? 0 : I) + jb * 128 + wave * (16 * kG1T) + (j % kG1T) * 16) / 16;
    wt[j] = w13 + (size_t)tile_row * nkb * kTileBytes + lane * 16;
  }
  const float* swp[2] = {s13 + (size_t)jb * nkb, s13 + (size_t)(njb + jb) * nkb};

  for (int rt = r0; rt < r1; rt += 16) {
    const int r = rt + lr;
    const int rc = min(r, r1 - 1);  // surplus columns repeat the last row and are not stored
    const int tok = (e < E) ? perm[rc] / K : rc - T * K;
    const uint8_t* xrow = xq + (size_t)tok * H + lq * 32;
    const float* xsrow = xs + (size_t)tok * nkb;
    v4f acc[2 * kG1T];
#pragma unroll
    for (int j = 0; j < 2 * kG1T; j++) acc[j] = (v4f){0.f, 0.f, 0.f, 0.f};
    stream_mainloop<2 * kG1T, 2>(wt, swp, xrow, xsrow, nkb, acc);

    float h[kG1T][4];
    float amax = 0.f;
#pragma unroll
    for (int j = 0; j < kG1T; j++)
#pragma unroll
      for (int i = 0; i < 4; i++) {
        float g = acc[j][i], u = acc[kG1T + j][i];
        float v = g / (1.f + __expf(-g)) * u;
        h[j][i] = v;
        amax = fmaxf(amax, fabsf(v));
      }
    amax = fmaxf(amax, __shfl_xor(amax, 16));
    amax = fmaxf(amax, __shfl_xor(amax, 32));
    if (lq == 0) amax_s[wave][lr] = amax;
    __syncthreads();
#pragma unroll
    for (int w = 0; w < kG1Waves; w++) amax = fmaxf(amax, amax_s[w][lr]);
    const float scale = amax > 0.f ? amax / 448.f : 1.f;
    if (r < r1) {
#pragma unroll
      for (int j = 0; j < kG1T; j++) {
        uint32_t q = pack_fp8x4(h[j][0] / scale, h[j][1] / scale, h[j][2] / scale, h[j][3] / scale);
        *(uint32_t*)(hq + (size_t)r * I + jb * 128 + wave * (16 * kG1T) + j * 16 + lq * 4) = q;
      }
      if (wave == 0 && lq == 0) hs[(size_t)r * njb + jb] = scale;
    }
    __syncthreads();  // amax_s is reused by the next token tile
  }
}

// Task = (expert slot e, block nb of kG2Rows output rows).  Wave w owns kG2Tiles consecutive
// 16-row tiles, all inside one 128-row scale block.
//
// The B operand (16 token rows of h, the same for all four waves) is staged in LDS once per
// 16-row group instead of being loaded by every wave for every K block: with the MFMA lane
// mapping such a load touches 16 different lines per instruction and costs the address unit
// more time than the 1 KiB weight loads it accompanies.  K is staged in chunks of at most
// kG2ChunkK so that the LDS need does not depend on I.  Layout per K block: 16 rows x 128
// bytes, 16-byte chunks XOR-swizzled (the pattern of the tile kernel's token image) so that
// the 128-bit operand reads are free of bank conflicts.
constexpr int kG2Tiles = 1;
constexpr int kG2Rows = 4 * kG2Tiles * 16;  // rows per workgroup (64)
// K blocks per pipeline half in GEMM-2.  One tile per wave with four blocks per half measured
// best at the decode shape (358 us against 394 us for two tiles and two blocks): the short
// per-expert streams of GEMM-2 (32 KiB per tile row) profit from more, lighter waves.
constexpr int kU2 = 4;
constexpr int kG2ChunkK = 2048;
constexpr int kG2ChunkKb = kG2ChunkK / 128;

typedef const __attribute__((address_space(4))) float* cf32;

__device__ __forceinline__ int g2_swz(int row16) { return (((row16 >> 1) & 3) << 1) ^ (row16 >> 3); }

struct G2Frag {
  v4i w[kG2Tiles][2];
  v4i x[2];
  float sa;
  float sw;
};

// wt[j]: wave-uniform base of packed tile row j; lane16 = lane * 16; xb0/xb1: this lane's two
// chunk addresses inside K block 0 of the LDS image; kb counts from the chunk start, kbg is
// the same block in the weight matrix.
__device__ __forceinline__ void g2_load_w(G2Frag& f, const uint8_t* const (&wt)[kG2Tiles], uint32_t lane16,
                                          const float* swp, int kbg) {
#pragma unroll
  for (int j = 0; j < kG2Tiles; j++) {
    const uint8_t* p = wt[j] + (size_t)kbg * kTileBytes + lane16;
    f.w[j][0] = __builtin_nontemporal_load((gv4i)p);
    f.w[j][1] = __builtin_nontemporal_load((gv4i)(p + kTileBytes / 2));
  }
  f.sw = *(cf32)(swp + kbg);
}

__device__ __forceinline__ void g2_load_x(G2Frag& f, const uint8_t* xb0, const uint8_t* xb1, const float* xsa,
                                          int kb) {
  f.x[0] = *(const v4i*)(xb0 + kb * kTileBytes);
  f.x[1] = *(const v4i*)(xb1 + kb * kTileBytes);
  f.sa = xsa[kb * 16];
}

__device__ __forceinline__ void g2_load(G2Frag& f, const uint8_t* const (&wt)[kG2Tiles], uint32_t lane16,
                                        const float* swp, const uint8_t* xb0, const uint8_t* xb1, const float* xsa,
                                        int kb, int kbg) {
  g2_load_w(f, wt, lane16, swp, kbg);
  g2_load_x(f, xb0, xb1, xsa, kb);
}

__device__ __forceinline__ void g2_mma(const G2Frag& f, v4f (&acc)[kG2Tiles]) {
  const v8i b = cat(f.x[0], f.x[1]);
  const float s = f.sa * f.sw;
#pragma unroll
  for (int j = 0; j < kG2Tiles; j++) {
    const v4f zero = {0.f, 0.f, 0.f, 0.f};
    v4f p = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(cat(f.w[j][0], f.w[j][1]), b, zero, 0, 0, 0, 0, 0, 0);
#pragma unroll
    for (int i = 0; i < 4; i++) acc[j][i] = fmaf(p[i], s, acc[j][i]);
  }
}

__device__ __forceinline__ void gemm2_fp8_stream_item(
    int block, uint8_t* lds_x /* kG2ChunkKb * kTileBytes */, float* lds_sa /* kG2ChunkKb * 16 */,
    const dwdp_expert_ptrs* __restrict__ table, const int32_t* __restrict__ offsets, const uint8_t* __restrict__ hq,
    const float* __restrict__ hs, uint16_t* __restrict__ yp, int H, int I, int max_rows) {
  const int nnb = (H + kG2Rows - 1) / kG2Rows;
  const int e = block / nnb;
  const int nb = block - e * nnb;
  const int r0 = offsets[e];
  const int r1 = offsets[e + 1];
  if (r1 <= r0 || r1 - r0 > max_rows) return;
  const int tid = threadIdx.x;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // scalar: weight and scale addresses stay in SGPRs
  const int lane = tid & 63, lr = lane & 15, lq = lane >> 4;
  const int nkb = I / 128;
  // H is a multiple of 128, not of 256: the last workgroup's upper waves have no rows; they
  // still take part in the staging and its barriers
  const int row0 = nb * kG2Rows + wave * (kG2Tiles * 16);  // first output row of this wave
  const bool has_rows = row0 < H;
  const int tr0 = has_rows ? row0 / 16 : 0;
  const uint8_t* w2 = (const uint8_t*)table[e].w2;
  const float* s2 = table[e].s2;
  const uint8_t* wt[kG2Tiles];
#pragma unroll
  for (int j = 0; j < kG2Tiles; j++) wt[j] = w2 + (size_t)(tr0 + j) * nkb * kTileBytes;
  const float* swp = s2 + (size_t)(tr0 / 8) * nkb;
  const uint32_t lane16 = lane * 16;
  const uint8_t* xb0 = lds_x + lr * 128 + (((2 * lq) ^ g2_swz(lr)) << 4);
  const uint8_t* xb1 = lds_x + lr * 128 + (((2 * lq + 1) ^ g2_swz(lr)) << 4);
  const float* xsa = lds_sa + lr;

  for (int rt = r0; rt < r1; rt += 16) {
    v4f acc[kG2Tiles];
#pragma unroll
    for (int j = 0; j < kG2Tiles; j++) acc[j] = (v4f){0.f, 0.f, 0.f, 0.f};
    for (int kc = 0; kc < nkb; kc += kG2ChunkKb) {
      const int nkc = min(kG2ChunkKb, nkb - kc);
      constexpr int kStep = 2 * kU2;
      const int nmain = (nkc / kStep) * kStep;
      // Stage rows rt..rt+15 (rows past the end repeat the last one), K blocks kc..kc+nkc-1.
      // Order of issue: the chunk's h pieces (cache hits) into registers, then the first
      // weight blocks (HBM); the LDS writes wait for the pieces only, so the weights' latency
      // passes behind the staging and its barriers instead of after them.  The early weight
      // loads are unconditional (block index clamped, a wave without rows reads tile row 0):
      // a branch around them would make the wait before the LDS writes a wait for everything.
      constexpr int kPieces = kG2ChunkKb * 128 / kStreamThreads;
      v4i piece[kPieces];
#pragma unroll
      for (int it = 0; it < kPieces; it++) {
        const int pidx = tid + it * kStreamThreads;
        const int kb = min(pidx >> 7, nkc - 1), row = (pidx >> 3) & 15, c = pidx & 7;
        const int rc = min(rt + row, r1 - 1);
        piece[it] = *(gv4i)(hq + (size_t)rc * I + (size_t)(kc + kb) * 128 + c * 16);
      }
      const float piece_s = hs[(size_t)min(rt + (tid & 15), r1 - 1) * nkb + kc + min(tid >> 4, nkc - 1)];
      G2Frag f0[kU2], f1[kU2];
#pragma unroll
      for (int u = 0; u < kU2; u++) g2_load_w(f0[u], wt, lane16, swp, min(kc + u, nkb - 1));
      __syncthreads();  // the previous chunk's readers are done
#pragma unroll
      for (int it = 0; it < kPieces; it++) {
        const int pidx = tid + it * kStreamThreads;
        const int kb = pidx >> 7, row = (pidx >> 3) & 15, c = pidx & 7;
        if (kb < nkc) *(v4i*)(lds_x + kb * kTileBytes + row * 128 + ((c ^ g2_swz(row)) << 4)) = piece[it];
      }
      if (tid < nkc * 16) lds_sa[tid] = piece_s;
      __syncthreads();
      if (has_rows) {
        // two K blocks of weight loads in flight behind the MFMAs of the previous two
        if (nmain > 0) {
#pragma unroll
          for (int u = 0; u < kU2; u++) g2_load_x(f0[u], xb0, xb1, xsa, u);
          int kb0 = 0;
          for (; kb0 + kStep < nmain; kb0 += kStep) {
#pragma unroll
            for (int u = 0; u < kU2; u++)
              g2_load(f1[u], wt, lane16, swp, xb0, xb1, xsa, kb0 + kU2 + u, kc + kb0 + kU2 + u);
#pragma unroll
            for (int u = 0; u < kU2; u++) g2_mma(f0[u], acc);
#pragma unroll
            for (int u = 0; u < kU2; u++)
              g2_load(f0[u], wt, lane16, swp, xb0, xb1, xsa, kb0 + kStep + u, kc + kb0 + kStep + u);
#pragma unroll
            for (int u = 0; u < kU2; u++) g2_mma(f1[u], acc);
          }
          // last round of the chunk: nothing left to load for f0
#pragma unroll
          for (int u = 0; u < kU2; u++)
            g2_load(f1[u], wt, lane16, swp, xb0, xb1, xsa, kb0 + kU2 + u, kc + kb0 + kU2 + u);
#pragma unroll
          for (int u = 0; u < kU2; u++) g2_mma(f0[u], acc);
#pragma unroll
          for (int u = 0; u < kU2; u++) g2_mma(f1[u], acc);
        }
        for (int kb = nmain; kb < nkc; kb++) {
          G2Frag f;
          g2_load(f, wt, lane16, swp, xb0, xb1, xsa, kb, kc + kb);
          g2_mma(f, acc);
        }
      }
    }
    const int r = rt + lr;
    if (has_rows && r < r1) {
#pragma unroll
      for (int j = 0; j < kG2Tiles; j++) {
        uint2 o;
        o.x = (uint32_t)f32_to_bf16(acc[j][0]) | ((uint32_t)f32_to_bf16(acc[j][1]) << 16);
        o.y = (uint32_t)f32_to_bf16(acc[j][2]) | ((uint32_t)f32_to_bf16(acc[j][3]) << 16);
        *(uint2*)(yp + (size_t)r * H + row0 + j * 16 + lq * 4) = o;
      }
    }
  }
}

// ------------------------------------------------------- experts with 17 .. max_rows rows
// The same weight streams with several 16-token tiles per pass: a workgroup item is (row group
// of up to kMidRows = 64 sorted rows of one expert, panel of 128 h columns or 128 output rows).
// Every weight fragment in registers feeds kMidNB matrix instructions (one per token tile)
// instead of one, so an expert with up to 64 rows is still read from HBM once and an expert
// with more rows once per 64 -- without the whole-compute-unit workgroups of the LDS-tiled
// kernel, which a short list of such experts cannot fill and which cannot share a compute unit
// with anything else.  The token operand (the same for the four waves) is staged in LDS in
// chunks of kMidKC K blocks, in the swizzled 16-row images of the one-tile GEMM-2 above; the
// weight loads of the next K blocks stay in flight across a chunk boundary.
constexpr int kMidNB = kMidRows / 16;                      // token tiles per pass (4)
constexpr int kMidKC = 8;                                  // K blocks per staged chunk
constexpr int kMidImgBytes = kMidKC * kMidNB * kTileBytes;  // 64 KiB
constexpr int kMidLdsBytes = kMidImgBytes + kMidKC * kMidRows * 4 + kMidRows * 4 + 4 * kMidRows * 4;
// K blocks per pipeline half of the multi-tile items: one in GEMM-1 (four weight tiles and 64
// accumulators per wave leave registers for two K blocks of weights, 16 KiB per wave, in flight),
// two in GEMM-2 (two weight tiles per wave)
constexpr int kMidU1 = 1, kMidU2 = 2;
static_assert(kMidKC % (2 * kMidU1) == 0 && kMidKC % (2 * kMidU2) == 0, "a chunk boundary falls on a pipeline round");

template <int NT, int SG>
struct WFrag {
  v4i w[NT][2];
  float sw[SG];
};

// wt[j]: this lane's address inside K block 0 of packed tile row j; tile j uses scale group j / (NT/SG)
template <int NT, int SG>
__device__ __forceinline__ void mid_load(WFrag<NT, SG>& f, const uint8_t* const (&wt)[NT],
                                         const float* const (&swp)[SG], int kb) {
#pragma unroll
  for (int j = 0; j < NT; j++) {
    const uint8_t* p = wt[j] + (size_t)kb * kTileBytes;
    f.w[j][0] = __builtin_nontemporal_load((gv4i)p);
    f.w[j][1] = __builtin_nontemporal_load((gv4i)(p + kTileBytes / 2));
  }
#pragma unroll
  for (int g = 0; g < SG; g++) f.sw[g] = *(gf32)(swp[g] + kb);
}

// img: LDS image of this K block (kMidNB tiles of 16 rows x 128 bytes, swizzled); sa: its 64
// activation scales; xo0/xo1: this lane's two chunk offsets inside a tile image
template <int NT, int SG>
__device__ __forceinline__ void mid_mma(const WFrag<NT, SG>& f, const uint8_t* img, const float* sa, int xo0, int xo1,
                                        int lr, v4f (&acc)[NT][kMidNB]) {
#pragma unroll
  for (int tb = 0; tb < kMidNB; tb++) {
    const v8i b = cat(*(const v4i*)(img + tb * kTileBytes + xo0), *(const v4i*)(img + tb * kTileBytes + xo1));
    const float sat = sa[tb * 16 + lr];
#pragma unroll
    for (int j = 0; j < NT; j++) {
      const v4f zero = {0.f, 0.f, 0.f, 0.f};
      const v4f p = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(cat(f.w[j][0], f.w[j][1]), b, zero, 0, 0, 0, 0, 0, 0);
      const float sj = sat * f.sw[j / (NT / SG)];
#pragma unroll
      for (int i = 0; i < 4; i++) acc[j][tb][i] = fmaf(p[i], sj, acc[j][tb][i]);
    }
  }
}

// G1: act/act_s = quantised x (rows gathered through perm), out = hq/hs; else act/act_s = hq/hs, out = yp.
template <bool G1>
__device__ __forceinline__ void gemm_fp8_mid_item(int block, uint8_t* lds, const dwdp_expert_ptrs* __restrict__ table,
                                                  const int32_t* __restrict__ offsets, const int32_t* __restrict__ perm,
                                                  const int32_t* __restrict__ mid_expert,
                                                  const int32_t* __restrict__ mid_row0, const int32_t* __restrict__ n_mid,
                                                  const uint8_t* __restrict__ act, const float* __restrict__ act_s,
                                                  uint8_t* __restrict__ hq, float* __restrict__ hs,
                                                  uint16_t* __restrict__ yp, int E, int T, int H, int I, int K) {
  constexpr int NT = G1 ? 4 : 2;  // 16-row weight tiles per wave: G1 two gate + two up, GEMM-2 two
  constexpr int SG = G1 ? 2 : 1;
  const int n_panels = (G1 ? I : H) / 128;
  const int g = block / n_panels;
  const int panel = block - g * n_panels;
  if (g >= *n_mid) return;
  const int e = mid_expert[g];
  const int r0 = mid_row0[g];
  const int r1 = min(r0 + kMidRows, offsets[e + 1]);
  uint8_t* img = lds;
  float* lds_sa = (float*)(lds + kMidImgBytes);                  // [kMidKC][kMidRows]
  int32_t* lds_row = (int32_t*)(lds_sa + kMidKC * kMidRows);     // [kMidRows] source row of every slot
  float* amax_s = (float*)(lds_row + kMidRows);                  // [4 waves][kMidRows]
  const int tid = threadIdx.x;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int lane = tid & 63, lr = lane & 15, lq = lane >> 4;
  const int Kdim = G1 ? H : I;
  const int nkb = Kdim / 128;
  if (tid < kMidRows) {
    const int r = min(r0 + tid, r1 - 1);  // slots past the end repeat the last row and are not stored
    lds_row[tid] = G1 ? ((e < E) ? perm[r] / K : r - T * K) : r;
  }
  const uint8_t* wbase = (const uint8_t*)(G1 ? table[e].w13 : table[e].w2);
  const float* sbase = G1 ? table[e].s13 : table[e].s2;
  const uint8_t* wt[NT];
  const float* swp[SG];
#pragma unroll
  for (int j = 0; j < NT; j++) {
    int row;  // first row of weight tile j
    if (G1)
      row = (j < 2 ? 0 : I) + panel * 128 + wave * 32 + (j & 1) * 16;
    else
      row = panel * 128 + wave * 32 + j * 16;
    wt[j] = wbase + (size_t)(row / 16) * nkb * kTileBytes + lane * 16;
  }
  swp[0] = sbase + (size_t)panel * nkb;                                   // GEMM-1: the gate rows' scale block
  if constexpr (G1) swp[1] = sbase + (size_t)(I / 128 + panel) * nkb;     // the up rows' scale block
  const int xo0 = lr * 128 + (((2 * lq) ^ g2_swz(lr)) << 4);
  const int xo1 = lr * 128 + (((2 * lq + 1) ^ g2_swz(lr)) << 4);

  v4f acc[NT][kMidNB];
#pragma unroll
  for (int j = 0; j < NT; j++)
#pragma unroll
    for (int tb = 0; tb < kMidNB; tb++) acc[j][tb] = (v4f){0.f, 0.f, 0.f, 0.f};

  // stage K blocks kc .. kc+nkc-1 of the group's rows (all threads; two barriers)
  auto stage = [&](int kc) {
    const int nkc = min(kMidKC, nkb - kc);
    __syncthreads();  // the previous chunk's readers are done (and lds_row is written)
    for (int p0 = 0; p0 < nkc * (kMidRows * 8); p0 += 8 * kStreamThreads) {
      v4i v[8];
#pragma unroll
      for (int u = 0; u < 8; u++) {
        const int pidx = min(p0 + u * kStreamThreads + tid, nkc * (kMidRows * 8) - 1);
        const int kb = pidx >> 9, slot = (pidx >> 3) & (kMidRows - 1), c = pidx & 7;
        v[u] = *(gv4i)(act + (size_t)lds_row[slot] * Kdim + (size_t)(kc + kb) * 128 + c * 16);
      }
#pragma unroll
      for (int u = 0; u < 8; u++) {
        const int pidx = p0 + u * kStreamThreads + tid;
        const int kb = pidx >> 9, slot = (pidx >> 3) & (kMidRows - 1), c = pidx & 7;
        if (pidx < nkc * (kMidRows * 8))
          *(v4i*)(img + kb * (kMidNB * kTileBytes) + (slot >> 4) * kTileBytes + (slot & 15) * 128 +
                  ((c ^ g2_swz(slot & 15)) << 4)) = v[u];
      }
    }
    for (int i = tid; i < nkc * kMidRows; i += kStreamThreads) {
      const int kb = i / kMidRows, slot = i - kb * kMidRows;
      lds_sa[i] = act_s[(size_t)lds_row[slot] * nkb + kc + kb];
    }
    __syncthreads();
  };
  auto mma = [&](const WFrag<NT, SG>& f, int kb) {
    const int kl = kb & (kMidKC - 1);
    mid_mma<NT, SG>(f, img + kl * (kMidNB * kTileBytes), lds_sa + kl * kMidRows, xo0, xo1, lr, acc);
  };

  __syncthreads();  // lds_row
  constexpr int kUm = G1 ? kMidU1 : kMidU2;
  constexpr int kStep = 2 * kUm;
  const int nmain = (nkb / kStep) * kStep;
  if (nmain > 0) {
    WFrag<NT, SG> f0[kUm], f1[kUm];
#pragma unroll
    for (int u = 0; u < kUm; u++) mid_load<NT, SG>(f0[u], wt, swp, u);
    for (int kb0 = 0; kb0 < nmain; kb0 += kStep) {
      if ((kb0 & (kMidKC - 1)) == 0) stage(kb0);  // f0's loads stay in flight behind the staging
#pragma unroll
      for (int u = 0; u < kUm; u++) mid_load<NT, SG>(f1[u], wt, swp, kb0 + kUm + u);
#pragma unroll
      for (int u = 0; u < kUm; u++) mma(f0[u], kb0 + u);
      if (kb0 + kStep < nmain) {
#pragma unroll
        for (int u = 0; u < kUm; u++) mid_load<NT, SG>(f0[u], wt, swp, kb0 + kStep + u);
      }
#pragma unroll
      for (int u = 0; u < kUm; u++) mma(f1[u], kb0 + kUm + u);
    }
  }
  for (int kb = nmain; kb < nkb; kb++) {
    if ((kb & (kMidKC - 1)) == 0) stage(kb);
    WFrag<NT, SG> f;
    mid_load<NT, SG>(f, wt, swp, kb);
    mma(f, kb);
  }

  if (G1) {
    // tiles 0,1 = gate and 2,3 = up rows of h columns panel*128 + wave*32 + {0,16} + lq*4 + i
    const int njb = I / 128;
    float amax[kMidNB];
#pragma unroll
    for (int tb = 0; tb < kMidNB; tb++) {
      float m = 0.f;
#pragma unroll
      for (int j = 0; j < 2; j++)
#pragma unroll
        for (int i = 0; i < 4; i++) {
          const float gv = acc[j][tb][i], uv = acc[2 + j][tb][i];
          const float v = gv / (1.f + __expf(-gv)) * uv;
          acc[j][tb][i] = v;
          m = fmaxf(m, fabsf(v));
        }
      m = fmaxf(m, __shfl_xor(m, 16));
      m = fmaxf(m, __shfl_xor(m, 32));
      if (lq == 0) amax_s[wave * kMidRows + tb * 16 + lr] = m;
      amax[tb] = m;
    }
    __syncthreads();
#pragma unroll
    for (int tb = 0; tb < kMidNB; tb++) {
      float m = amax[tb];
#pragma unroll
      for (int w = 0; w < 4; w++) m = fmaxf(m, amax_s[w * kMidRows + tb * 16 + lr]);
      const float scale = m > 0.f ? m / 448.f : 1.f;
      const int r = r0 + tb * 16 + lr;
      if (r < r1) {
#pragma unroll
        for (int j = 0; j < 2; j++) {
          const uint32_t q = pack_fp8x4(acc[j][tb][0] / scale, acc[j][tb][1] / scale, acc[j][tb][2] / scale,
                                        acc[j][tb][3] / scale);
          *(uint32_t*)(hq + (size_t)r * I + panel * 128 + wave * 32 + j * 16 + lq * 4) = q;
        }
        if (wave == 0 && lq == 0) hs[(size_t)r * njb + panel] = scale;
      }
    }
  } else {
#pragma unroll
    for (int tb = 0; tb < kMidNB; tb++) {
      const int r = r0 + tb * 16 + lr;
      if (r < r1) {
#pragma unroll
        for (int j = 0; j < NT; j++) {
          uint2 o;
          o.x = (uint32_t)f32_to_bf16(acc[j][tb][0]) | ((uint32_t)f32_to_bf16(acc[j][tb][1]) << 16);
          o.y = (uint32_t)f32_to_bf16(acc[j][tb][2]) | ((uint32_t)f32_to_bf16(acc[j][tb][3]) << 16);
          *(uint2*)(yp + (size_t)r * H + panel * 128 + wave * 32 + j * 16 + lq * 4) = o;
        }
      }
    }
  }
}

// One launch per GEMM serves both streaming families: the first n_mid_blocks workgroups take the
// row groups of the experts with 17 .. max_rows rows (longer items first), the others the
// (expert, panel) items of the experts with 1 .. 16 rows.  With no row-group list
// (n_mid_blocks = 0) the one-tile items also walk larger experts, 16 rows at a time.
__global__ __launch_bounds__(kStreamThreads, 2) void gemm1_fp8_stream_kernel(
    const dwdp_expert_ptrs* __restrict__ table, const int32_t* __restrict__ offsets, const int32_t* __restrict__ perm,
    const int32_t* __restrict__ mid_expert, const int32_t* __restrict__ mid_row0, const int32_t* __restrict__ n_mid,
    int n_mid_blocks, const uint8_t* __restrict__ xq, const float* __restrict__ xs, uint8_t* __restrict__ hq,
    float* __restrict__ hs, int E, int T, int H, int I, int K, int max_rows) {
  __shared__ __attribute__((aligned(16))) uint8_t lds[kMidLdsBytes];
  if ((int)blockIdx.x < n_mid_blocks)
    gemm_fp8_mid_item<true>(blockIdx.x, lds, table, offsets, perm, mid_expert, mid_row0, n_mid, xq, xs, hq, hs, nullptr,
                            E, T, H, I, K);
  else
    gemm1_fp8_stream_item(blockIdx.x - n_mid_blocks, (float(*)[16])lds, table, offsets, perm, xq, xs, hq, hs, E, T, H, I,
                          K, max_rows);
}

__global__ __launch_bounds__(kStreamThreads, 2) void gemm2_fp8_stream_kernel(
    const dwdp_expert_ptrs* __restrict__ table, const int32_t* __restrict__ offsets,
    const int32_t* __restrict__ mid_expert, const int32_t* __restrict__ mid_row0, const int32_t* __restrict__ n_mid,
    int n_mid_blocks, const uint8_t* __restrict__ hq, const float* __restrict__ hs, uint16_t* __restrict__ yp, int E,
    int T, int H, int I, int K, int max_rows) {
  __shared__ __attribute__((aligned(16))) uint8_t lds[kMidLdsBytes];
  static_assert(kMidLdsBytes >= kG2ChunkKb * kTileBytes + kG2ChunkKb * 16 * 4, "the one-tile item's staging fits");
  if ((int)blockIdx.x < n_mid_blocks)
    gemm_fp8_mid_item<false>(blockIdx.x, lds, table, offsets, nullptr, mid_expert, mid_row0, n_mid, hq, hs, nullptr,
                             nullptr, yp, E, T, H, I, K);
  else
    gemm2_fp8_stream_item(blockIdx.x - n_mid_blocks, lds, (float*)(lds + kG2ChunkKb * kTileBytes), table, offsets, hq,
                          hs, yp, H, I, max_rows);
}

int mid_groups_cap(int rows, int n_slots, int mid_min_rows) {
  // listed experts have at least mid_min_rows rows: at most rows / mid_min_rows of them, each
  // adding at most one partial group to the rows / kMidRows full ones
  const long by_rows = (long)rows / (mid_min_rows > 0 ? mid_min_rows : 1);
  return rows / kMidRows + (int)(by_rows < n_slots ? by_rows : n_slots) + 1;
}

void launch_gemm1_fp8(const GemmArgs& a, int max_rows, const TileSched& ts, const uint8_t* xq, const float* xs,
                      uint8_t* hq, float* hs, hipStream_t stream) {
  if (a.T <= 0) return;
  const int n_mid_blocks = ts.mid_expert ? ts.mid_cap * (a.I / 128) : 0;
  dim3 grid(n_mid_blocks + a.n_slots * (a.I / 128));
  hipLaunchKernelGGL(gemm1_fp8_stream_kernel, grid, dim3(kStreamThreads), 0, stream, a.table, a.offsets, a.perm,
                     ts.mid_expert, ts.mid_row0, ts.n_mid, n_mid_blocks, xq, xs, hq, hs, a.E, a.T, a.H, a.I, a.K,
                     ts.mid_expert ? (max_rows < 16 ? max_rows : 16) : max_rows);
}

void launch_gemm2_fp8(const GemmArgs& a, int max_rows, const TileSched& ts, const uint8_t* hq, const float* hs,
                      void* yp, hipStream_t stream) {
  if (a.T <= 0) return;
  const int n_mid_blocks = ts.mid_expert ? ts.mid_cap * (a.H / 128) : 0;
  dim3 grid(n_mid_blocks + a.n_slots * ((a.H + kG2Rows - 1) / kG2Rows));
  hipLaunchKernelGGL(gemm2_fp8_stream_kernel, grid, dim3(kStreamThreads), 0, stream, a.table, a.offsets,
                     ts.mid_expert, ts.mid_row0, ts.n_mid, n_mid_blocks, hq, hs, (uint16_t*)yp, a.E, a.T, a.H, a.I,
                     a.K, ts.mid_expert ? (max_rows < 16 ? max_rows : 16) : max_rows);
}

// Row-major fp8 [rows, cols] -> tile-major.  Tile (tr, kb) = rows tr*16.., columns kb*128..
// lives at ((tr * cols/128) + kb) * 2048; inside it, byte  half*1024 + (lq*16 + lr)*16 + b
// holds element (row lr, column lq*32 + half*16 + b): exactly the two 16-byte pieces lane
// lq*16+lr of a wave feeds to a 16x16x128 MFMA operand.
__global__ __launch_bounds__(256) void pack_fp8_tiles_kernel(const uint8_t* __restrict__ src, uint8_t* __restrict__ dst,
                                                             long n16, int cols) {
  long o = (long)blockIdx.x * blockDim.x + threadIdx.x;  // index of a 16-byte piece of dst
  if (o >= n16) return;
  const int nkb = cols / 128;
  long tile = o >> 7;
  int in = (int)(o & 127);
  int half = in >> 6, l = in & 63, lr = l & 15, lq = l >> 4;
  long tr = tile / nkb;
  int kb = (int)(tile - tr * nkb);
  const uint8_t* s = src + (size_t)(tr * 16 + lr) * cols + kb * 128 + lq * 32 + half * 16;
  *(v4i*)(dst + o * 16) = *(const v4i*)s;
}

void launch_pack_fp8_tiles(const void* src, void* dst, long rows, int cols, hipStream_t stream) {
  long n16 = rows * cols / 16;
  if (n16 <= 0) return;
  hipLaunchKernelGGL(pack_fp8_tiles_kernel, dim3((unsigned)((n16 + 255) / 256)), dim3(256), 0, stream,
                     (const uint8_t*)src, (uint8_t*)dst, n16, cols);
}

// ------------------------------------------------------------------------------ bf16 weights
// Same task decomposition for bf16 weights and activations, no scales.  GEMM-1 multiplies
// exact bf16 operands on v_mfma_f32_16x16x32_bf16; h and the down projection stay fp32
// (v_mfma_f32_16x16x4_f32 with the bf16 weights widened in registers) so that the only
// rounding of the layer is the final one to bf16.  Serves the small bf16 configuration;
// not tuned.

__global__ __launch_bounds__(kStreamThreads) void gemm1_bf16_kernel(const dwdp_expert_ptrs* __restrict__ table,
                                                                    const int32_t* __restrict__ offsets,
                                                                    const int32_t* __restrict__ perm,
                                                                    const uint16_t* __restrict__ x,
                                                                    float* __restrict__ h, int E, int T, int H,
                                                                    int I, int K) {
  const int njb = I / 128;
  const int e = blockIdx.x / njb;
  const int jb = blockIdx.x - e * njb;
  const int r0 = offsets[e];
  const int r1 = offsets[e + 1];
  if (r1 <= r0) return;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, lr = lane & 15, lq = lane >> 4;
  const uint16_t* w13 = (const uint16_t*)table[e].w13;
  const uint16_t* wrow[4];
#pragma unroll
  for (int j = 0; j < 4; j++) {
    int n = (j < 2 ? 0 : I) + jb * 128 + wave * 32 + (j & 1) * 16 + lr;
    wrow[j] = w13 + (size_t)n * H + lq * 8;
  }
  for (int rt = r0; rt < r1; rt += 16) {
    const int r = rt + lr;
    const int rc = min(r, r1 - 1);
    const int tok = (e < E) ? perm[rc] / K : rc - T * K;
    const uint16_t* xrow = x + (size_t)tok * H + lq * 8;
    v4f acc[4];
#pragma unroll
    for (int j = 0; j < 4; j++) acc[j] = (v4f){0.f, 0.f, 0.f, 0.f};
    for (int k = 0; k < H; k += 32) {
      const v8bf b = *(const v8bf*)(xrow + k);
#pragma unroll
      for (int j = 0; j < 4; j++)
        acc[j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(*(const v8bf*)(wrow[j] + k), b, acc[j], 0, 0, 0);
    }
    if (r < r1) {
#pragma unroll
      for (int j = 0; j < 2; j++) {
        v4f v;
#pragma unroll
        for (int i = 0; i < 4; i++) {
          float g = acc[j][i], u = acc[2 + j][i];
          v[i] = g / (1.f + expf(-g)) * u;
        }
        *(v4f*)(h + (size_t)r * I + jb * 128 + wave * 32 + j * 16 + lq * 4) = v;
      }
    }
  }
}

__global__ __launch_bounds__(kStreamThreads) void gemm2_bf16_kernel(const dwdp_expert_ptrs* __restrict__ table,
                                                                    const int32_t* __restrict__ offsets,
                                                                    const float* __restrict__ h,
                                                                    float* __restrict__ yp, int H, int I) {
  const int nnb = H / 128;
  const int e = blockIdx.x / nnb;
  const int nb = blockIdx.x - e * nnb;
  const int r0 = offsets[e];
  const int r1 = offsets[e + 1];
  if (r1 <= r0) return;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, lr = lane & 15, lq = lane >> 4;
  const uint16_t* w2 = (const uint16_t*)table[e].w2;
  const uint16_t* wrow[2];
#pragma unroll
  for (int j = 0; j < 2; j++) wrow[j] = w2 + (size_t)(nb * 128 + wave * 32 + j * 16 + lr) * I + lq * 8;
  for (int rt = r0; rt < r1; rt += 16) {
    const int r = rt + lr;
    const int rc = min(r, r1 - 1);
    const float* hrow = h + (size_t)rc * I + lq * 8;
    v4f acc[2];
    acc[0] = (v4f){0.f, 0.f, 0.f, 0.f};
    acc[1] = (v4f){0.f, 0.f, 0.f, 0.f};
    for (int k = 0; k < I; k += 32) {
      // lane group lq covers k + lq*8 .. +8 of this 32-wide chunk on both operands
      const v4f b0 = *(const v4f*)(hrow + k);
      const v4f b1 = *(const v4f*)(hrow + k + 4);
#pragma unroll
      for (int j = 0; j < 2; j++) {
        const v4i raw = *(const v4i*)(wrow[j] + k);
#pragma unroll
        for (int i = 0; i < 8; i++) {
          uint32_t u = (uint32_t)raw[i >> 1];
          float a = __uint_as_float((i & 1) ? (u & 0xFFFF0000u) : (u << 16));
          float b = i < 4 ? b0[i] : b1[i - 4];
          acc[j] = __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, acc[j], 0, 0, 0);
        }
      }
    }
    if (r < r1) {
#pragma unroll
      for (int j = 0; j < 2; j++) *(v4f*)(yp + (size_t)r * H + nb * 128 + wave * 32 + j * 16 + lq * 4) = acc[j];
    }
  }
}

void launch_gemm1_bf16(const GemmArgs& a, const void* x, void* h, hipStream_t stream) {
  if (a.T <= 0) return;
  dim3 grid(a.n_slots * (a.I / 128));
  hipLaunchKernelGGL(gemm1_bf16_kernel, grid, dim3(kStreamThreads), 0, stream, a.table, a.offsets, a.perm,
                     (const uint16_t*)x, (float*)h, a.E, a.T, a.H, a.I, a.K);
}

void launch_gemm2_bf16(const GemmArgs& a, const void* h, void* yp, hipStream_t stream) {
  if (a.T <= 0) return;
  dim3 grid(a.n_slots * (a.H / 128));
  hipLaunchKernelGGL(gemm2_bf16_kernel, grid, dim3(kStreamThreads), 0, stream, a.table, a.offsets, (const float*)h,
                     (float*)yp, a.H, a.I);
}

}  // namespace dwdp
