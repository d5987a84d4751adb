// LDS-tiled FP8 grouped GEMM for gfx950: the large-M (prefill-shaped) path.
//
// A workgroup of 8 waves computes a 256 (weight rows) x 288 (tokens) output tile of one
// expert; 288 tokens cover almost every expert of the prefill workload (256 +- 16 rows),
// so each weight panel is read from HBM once.  Per 128-wide K block -- exactly one
// weight-scale block and one activation-scale group:
//   * tokens (B operand, shared by all waves): 18 tiles of 16 rows x 128 bytes = 36 KiB,
//     gathered through the permutation by asynchronous global->LDS copies
//     (global_load_lds_dwordx4, 8 whole 128-byte rows per instruction, chunks XOR-swizzled
//     against LDS bank conflicts) into a ring of three LDS images, two K blocks ahead;
//   * weights (A operand): wave w owns two 16-row tiles of the panel that no other wave
//     needs, so they bypass LDS: tile-major weights are loaded straight into MFMA operand
//     registers (contiguous 1 KiB per load) into a ring of three register sets, two K
//     blocks ahead.
// LDS capacity bounds how far ahead a workgroup can fetch; staging only the shared operand
// in LDS halves the bytes per stage, which is what lets both operands run two blocks ahead
// (with both operands in LDS only one block of lookahead fit and every K block paid the
// HBM latency: 2.6 us against 1.8 us of compute).
// Each wave multiplies its 2 weight tiles with all 18 token tiles on
// v_mfma_f32_16x16x128_f8f6f4 and folds every fp32 partial product into its accumulator with
// s_act[token,kb] * s_w[nblock,kb] on the VALU.
//
// Synchronisation is explicit: vector-memory operations complete in order and every wave
// issues the same operations per K block (5 token pieces, 4 weight loads, every third block a scale copy;
// spread between the token tiles of the running multiply, because a wave that issues them in
// one burst sits at the memory pipeline's door instead of feeding the MFMA), so "everything
// of block kb has landed" is s_waitcnt vmcnt(n) with n = the operations of block kb+1 (9, or
// 10 when it carries a scale copy) -- only those may still be in flight -- followed by one
// s_barrier per K block.  Past the end of K the ring
// keeps issuing (clamped to the last block) so the count stays valid.  The product of tile
// t is folded into the accumulators after the MFMAs of tile t+1 have been issued, so the
// VALU never waits for the matrix pipe.
//
// The multiply of a K block is a chain of token-tile pairs, each behind one scalar branch
// (pairs beyond the expert's row count are skipped; with an odd tile count the last pair
// multiplies one tile of repeated rows), and inside a pair the code is straight-line: the
// LDS read of tile t+1's operand, the two MFMAs of tile t each followed by the five VALU
// operations that scale tile t-1's products, the LDS read of tile t+1's activation scale.
// LDS reads return in order, so every use waits for exactly its own read (lgkmcnt(n) with
// the younger reads still in flight).  That only works while no scalar load is pending
// (scalar loads share the counter and return out of order: with one in flight every wait
// becomes a wait for everything), so the weight scales of block kb+1 are loaded at the end
// of block kb's multiply and waited for together with the vector-memory wait.
// Workgroups are numbered so that all weight panels of one M tile run on the same XCD back
// to back and share the token rows in its L2: block b runs on XCD b % 8 and handles M tile
// (b/8 / n_panels) * 8 + b % 8, panel (b/8) % n_panels.
//
// GEMM-1 (G1): wave w owns gate tile w and up tile w of the panel (16 h columns), epilogue
// silu(g)*u, per-token amax over the panel's 128 h columns (LDS, 8 waves), e4m3
// quantisation of h.  GEMM-2: wave w owns rows 32w..32w+31 of the 256-row panel, bf16 store
// through an LDS transpose.  Experts with few rows are left to the streaming kernels.
#include <type_traits>
#include <utility>

#include "dwdp_kernels.h"

// Timing experiments only (results are wrong when set): 1 = skip the MFMA/VALU work,
// 16 = no per-block wait and barrier, 32 = no LDS operand reads, 64 = no VALU scaling,
// 128 = no global loads or copies at all, 4 = no weight loads, 8 = no token copies,
// 512 = every workgroup reads the same (L2-resident) weight panel, 1024 = print the shader
// clock of two workgroups (cycle counter over the 100 MHz counter), 2048 = no scale products.
// Never set in a product build.
#ifndef DWDP_TILE_DBG
#define DWDP_TILE_DBG 0
#endif

namespace dwdp {

constexpr int kBM = kTileM;     // tokens per workgroup tile (288)
constexpr int kTT = kBM / 16;   // token tiles per workgroup (18)
constexpr int kTileWaves = 8;
#ifndef DWDP_TILE_BDEPTH
#define DWDP_TILE_BDEPTH 1
#endif
constexpr int kBDepth = DWDP_TILE_BDEPTH;  // token tiles whose LDS operand reads run ahead of the multiply
constexpr int kTileThreads = 64 * kTileWaves;
constexpr int kLdsB = kTT * kTileBytes;  // one token image: 36 KiB
constexpr int kBPieces = 2 * kTT;        // 1 KiB pieces of a token image
constexpr int kBP = (kBPieces + kTileWaves - 1) / kTileWaves;  // pieces copied per wave (5)
constexpr int kSaLen = 64 * kTileWaves;  // scale slots per image: every wave copies 64
// epilogue scratch: GEMM-1 keeps one amax per (wave, token), GEMM-2 stages 16 tokens x 80 bytes per wave
constexpr int kStagePitch = 80;
constexpr int kEpiBytes =
    kTileWaves * kBM * 4 > kTileWaves * 16 * kStagePitch ? kTileWaves * kBM * 4 : kTileWaves * 16 * kStagePitch;
static_assert(kBM <= kSaLen, "one scale slot per token");
// vector-memory operations per wave and K block, and the wait that proves block kb landed:
// operations issued after its copies = weights(kb) + all of blocks kb+1's issue
// Vector-memory operations per wave that fetch one K block: 5 token pieces, 4 weight loads and,
// for every third block, one copy of the activation scales of three blocks (a token's scales
// of consecutive K blocks are adjacent in memory while 64 tokens' scales of one block lie in 64
// different cache lines, and the memory pipeline's cost is per line touched).
constexpr int kVmemPerStep = kBP + 1 + 4;  // operation slots per block: pieces, (scales), weights
constexpr int kVmemNoScale = kVmemPerStep - 1;
static_assert(kVmemPerStep == 10, "the s_waitcnt immediates below assume 10 and 9");
// s_waitcnt immediate (gfx9 layout): vmcnt[3:0] | expcnt[6:4] | lgkmcnt[11:8] | vmcnt[5:4] << 14
constexpr int wait_vm(int n) { return (n & 15) | (7 << 4) | (15 << 8) | ((n >> 4) << 14); }
// the same with lgkmcnt(0): scalar loads and LDS operations have completed as well
constexpr int wait_vm_lgkm0(int n) { return (n & 15) | (7 << 4) | (0 << 8) | ((n >> 4) << 14); }
constexpr int kWaitVm0 = wait_vm(0);

typedef const __attribute__((address_space(1))) v4i* gv4i;
typedef const __attribute__((address_space(1))) float* gf32;
// Read-only data addressed with wave-uniform pointers: the constant address space makes
// these scalar loads (s_load), which do not touch the vector-memory counter.
typedef const __attribute__((address_space(4))) float* cf32;

__device__ __forceinline__ v8i cat8(v4i lo, v4i hi) { return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7); }

// Asynchronous global -> LDS copy of 64 lanes x 16 (or 4) bytes: lane l's bytes land at
// dst + l*16 (l*4); dst is wave-uniform and goes through M0.  Issued from inline assembly
// for the same reason as the weight loads below: the compiler must not model these
// operations, all waiting on them is done with explicit s_waitcnt.
__device__ __forceinline__ uint32_t lds_offset(const void* p) {
  return (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const void*)p;
}
__device__ __forceinline__ void dma16(const uint8_t* src_lane, uint8_t* dst_wave_uniform) {
  const uint32_t d = __builtin_amdgcn_readfirstlane(lds_offset(dst_wave_uniform));
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(d), "v"(src_lane) : "memory");
}
// 12 bytes per lane; lane l's bytes land at dst + l*16 (measured: the fourth dword of a slot is not written)
__device__ __forceinline__ void dma12(const float* src_lane, float* dst_wave_uniform) {
  const uint32_t d = __builtin_amdgcn_readfirstlane(lds_offset(dst_wave_uniform));
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx3 %1, off" ::"s"(d), "v"(src_lane) : "memory");
}

// f(integral_constant<int, 0>) ... f(integral_constant<int, N-1>), in order
template <int... Is, class F>
__device__ __forceinline__ void static_for_impl(std::integer_sequence<int, Is...>, F&& f) {
  (f(std::integral_constant<int, Is>{}), ...);
}
template <int N, class F>
__device__ __forceinline__ void static_for(F&& f) {
  static_for_impl(std::make_integer_sequence<int, N>{}, f);
}

struct AFrag {  // two 16x128 weight tiles in MFMA operand layout (16 registers)
  v4i t[2][2];
};

template <bool G1>
__global__ __launch_bounds__(kTileThreads, 1) void gemm_fp8_tile_kernel(
    const dwdp_expert_ptrs* __restrict__ table, const int32_t* __restrict__ offsets, const int32_t* __restrict__ perm,
    const int32_t* __restrict__ mt_expert, const int32_t* __restrict__ mt_row0, const int32_t* __restrict__ n_mtiles,
    int n_panels, const uint8_t* __restrict__ act, const float* __restrict__ act_s, uint8_t* __restrict__ hq,
    float* __restrict__ hs, uint16_t* __restrict__ yp, int E, int T, int H, int I, int K) {
  // Three token images, each its own array so that the compiler can tell a copy into one
  // from the reads of another.
  __shared__ __attribute__((aligned(16))) uint8_t lds_b0[kLdsB];
  __shared__ __attribute__((aligned(16))) uint8_t lds_b1[kLdsB];
  __shared__ __attribute__((aligned(16))) uint8_t lds_b2[kLdsB];
  // activation scales of three consecutive K blocks per token slot (16-byte slots, the layout
  // the 12-byte copy writes), double-buffered by block triple
  __shared__ __attribute__((aligned(16))) float lds_sg0[kSaLen * 4];
  __shared__ __attribute__((aligned(16))) float lds_sg1[kSaLen * 4];
  __shared__ int32_t lds_row[kSaLen];
  __shared__ __attribute__((aligned(16))) uint8_t lds_epi[kEpiBytes];  // amax / store staging

  long long dbg_c0 = 0, dbg_w0 = 0;
  if (DWDP_TILE_DBG & 1024) { dbg_c0 = clock64(); dbg_w0 = wall_clock64(); }
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
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // scalar: pointers derived from it stay in SGPRs
  const int lane = tid & 63, lr = lane & 15, lq = lane >> 4;
  const int Kdim = G1 ? H : I;  // reduction length
  const int nkb = Kdim / 128;
  __builtin_assume(nkb >= 1);  // the host rejects reduction lengths that are not positive multiples of 128
  const int n_tile_rows = (G1 ? 2 * I : H) / 16;
  const uint8_t* wbase = (const uint8_t*)(G1 ? table[e].w13 : table[e].w2);
  const float* sbase = G1 ? table[e].s13 : table[e].s2;

  // ---- sources, fixed over the K loop ----
  // weights: this wave's two tiles (G1: gate tile and up tile of 16 h columns; GEMM-2: 32 rows)
  const uint8_t* a_src[2];
  const float* sw[2];
#pragma unroll
  for (int j = 0; j < 2; j++) {
    int tr;
    if (G1)
      tr = (j == 0 ? 0 : I / 16) + panel * 8 + wave;
    else
      tr = min(panel * 16 + wave * 2 + j, n_tile_rows - 1);
    if (DWDP_TILE_DBG & 512) tr = G1 ? (j == 0 ? 0 : I / 16) + wave : wave * 2 + j;  // every workgroup reads panel 0
    a_src[j] = ((DWDP_TILE_DBG & 512) ? (const uint8_t*)(G1 ? table[0].w13 : table[0].w2) : wbase) +
               (size_t)tr * nkb * kTileBytes;  // wave-uniform
    sw[j] = sbase + (size_t)(tr / 8) * nkb;  // 8 tiles of 16 rows per 128-row scale block
  }
  // tokens: the source row of every token slot of the tile (slots past the end repeat the last row)
  for (int i = tid; i < kSaLen; i += kTileThreads) {
    const int row = min(r0 + i, r_end - 1);
    lds_row[i] = G1 ? ((e < E) ? perm[row] / K : row - T * K) : row;
  }
  __syncthreads();
  // this wave's token pieces: piece c = rows 8*(c&1)..+7 of tile c/2, all 128 K bytes of each
  // row, so that 8 consecutive lanes fetch one whole 128-byte line (lanes that fetch from
  // different lines are served one after the other by the address unit).  Lane l's 16 bytes
  // land in slot l of the piece; slot (row, p) holds the row's 16-byte chunk p ^ swz(row):
  // with this XOR the 128-bit operand reads below (lane (lr, lq) reads chunks 2lq, 2lq+1 of
  // row lr) run at the full LDS rate -- measured; a plain row-major image runs at a quarter,
  // XOR with (row>>1)&7 at half.  Slots past the image repeat the last piece.
  auto swz = [](int row16) { return (((row16 >> 1) & 3) << 1) ^ (row16 >> 3); };
  uint32_t b_src[kBP];
#pragma unroll
  for (int i = 0; i < kBP; i++) {
    const int c = min(wave + kTileWaves * i, kBPieces - 1);
    const int row16 = (c & 1) * 8 + (lane >> 3);
    b_src[i] = (uint32_t)lds_row[(c >> 1) * 16 + row16] * Kdim + (((lane & 7) ^ swz(row16)) << 4);
  }
  // operand reads: lane (lr, lq) needs chunks 2lq and 2lq+1 of row lr of every tile
  const int b_rd0 = lr * 128 + (((2 * lq) ^ swz(lr)) << 4);
  const uint32_t sa_src = (uint32_t)lds_row[wave * 64 + lane] * nkb;

  v4f acc[2][kTT];
#pragma unroll
  for (int j = 0; j < 2; j++)
#pragma unroll
    for (int t = 0; t < kTT; t++) acc[j][t] = (v4f){0.f, 0.f, 0.f, 0.f};

  // Issue everything block kb needs: always exactly kVmemPerStep operations, tokens first.
  // One of the kVmemPerStep vector-memory operations that fetch block kb: ops 0..kBP-1 copy
  // token pieces, op kBP the activation scales, the last four load this wave's weights.
  // The weight loads are issued from inline assembly so that the compiler does not model
  // them: it cannot order loads that stay in flight across the loop's back edge and would
  // drain the whole queue before the first MFMA of every block.  Their completion is covered
  // by the explicit s_waitcnt in publish(); the registers are read-write operands so each
  // fragment keeps its registers, and nothing reads them between issue and wait.
  const uint32_t lane16 = lane * 16;
  // the tile of the running multiply after which operation i of the next fetch is issued
  auto op_slot = [](int i) { return i < kVmemPerStep - 1 ? 2 * i + 1 : kTT - 1; };
  // One operation of the fetch of the pos-th block of the walk over K (block min(pos, nkb-1):
  // past the end the ring re-fetches the last block so that the counts the waits rely on stay
  // the same).  Operation kBP, the scale copy, exists only for pos % 3 == 0 and brings the
  // scales of blocks pos..pos+2 (with nkb % 3 != 0 the last copy reads one or two floats past
  // a token's row: the next row's, or the padding the workspace keeps behind the array).
  auto issue_op = [&](int op, int pos, uint8_t* lb, AFrag& a) __attribute__((always_inline)) {
    if (DWDP_TILE_DBG & 128) return;
    const int kb = min(pos, nkb - 1);
    if (op < kBP) {
      const int c = min(wave + kTileWaves * op, kBPieces - 1);
      if (!(DWDP_TILE_DBG & 8)) dma16(act + (b_src[op] + (uint32_t)kb * 128), lb + c * (kTileBytes / 2));
    } else if (op == kBP) {
      float* lsg = ((pos / 3) & 1) ? lds_sg1 : lds_sg0;
      if (!(DWDP_TILE_DBG & 8)) dma12(act_s + (sa_src + (uint32_t)kb), lsg + wave * (64 * 4));
    } else if (!(DWDP_TILE_DBG & 4)) {
      const int j = (op - kBP - 1) >> 1, half = (op - kBP - 1) & 1;
      const uint8_t* base = a_src[j] + (size_t)kb * kTileBytes;  // wave-uniform: scalar registers
      if (half == 0)
        asm volatile("global_load_dwordx4 %0, %1, %2 nt" : "+v"(a.t[j][0]) : "v"(lane16), "s"(base));
      else
        asm volatile("global_load_dwordx4 %0, %1, %2 offset:1024 nt"
                     : "+v"(a.t[j][1])
                     : "v"(lane16), "s"(base));
    }
  };
  // the whole fetch of position pos (prologue); C = pos % 3 decides whether it has a scale copy
  auto issue = [&](int pos, bool has_scales, uint8_t* lb, AFrag& a) {
#pragma unroll
    for (int op = 0; op < kVmemPerStep; op++)
      if (op != kBP || has_scales) issue_op(op, pos, lb, a);
  };

  // Weight scales of the block about to be multiplied: scalar loads issued at the end of the
  // previous block's multiply and waited for in publish(), so that no scalar load is pending
  // while LDS reads are in flight (both count on lgkmcnt, and with a scalar load outstanding
  // every wait on an LDS read has to be a wait for everything).
  float wc0 = *(cf32)(sw[0]), wc1 = *(cf32)(sw[1]);
  // Multiply block kb from (lb, a) and, spread between its token tiles, issue the fetch of
  // position kb + 2 into (lbn, an): issued in one burst the operations keep
  // the wave at the memory pipeline's door for as long as the transfers take, one every
  // other tile they slip in under the MFMAs.
  // Token tiles are processed in pairs with two operand buffers (no register copies): while
  // the MFMAs of tile t run, the LDS reads of tile t+1 are already in flight.
  // C = kb % 3 is a compile-time constant of each unrolled call: it selects this block's scale
  // inside its triple and tells whether the fetch issued here (position kb + 2) has a scale copy.
  auto compute = [&](auto c_const, const uint8_t* lb, const AFrag& a, int kb, uint8_t* lbn, AFrag& an) __attribute__((always_inline)) {
    constexpr int C = decltype(c_const)::value;
    constexpr bool kNextHasScales = (C + 2) % 3 == 0;
    const int pos_n = kb + 2;
    const float w0 = wc0, w1 = wc1;
    const v8i af0 = cat8(a.t[0][0], a.t[0][1]);
    const v8i af1 = cat8(a.t[1][0], a.t[1][1]);
    const uint8_t* pb0 = lb + b_rd0;
    const uint8_t* pb1 = lb + (b_rd0 ^ 16);  // chunk 2lq+1 sits in the neighbouring slot
    const float* ps = (((kb / 3) & 1) ? lds_sg1 : lds_sg0) + lr * 4 + C;
    const v4f zero = {0.f, 0.f, 0.f, 0.f};
    // The scaling of tile t-1's products is issued after the MFMAs of tile t, so the VALU
    // never waits for an MFMA result: two operand buffers (bfx, bfy), two product sets
    // (px, py) and two activation scales alternate.  Tile t's scale is only needed by that
    // later scaling, so it is read from LDS together with tile t+1's operand.
    v8i bf[kBDepth + 1];
    v4f p0[2] = {zero, zero}, p1[2] = {zero, zero};
    float sa[2] = {0.f, 0.f};
    auto read_b = [&](int t) __attribute__((always_inline)) -> v8i {
      if (DWDP_TILE_DBG & 32) return (v8i){1, 2, 3, 4, 5, 6, 7, 8};
      return cat8(*(const v4i*)(pb0 + t * kTileBytes), *(const v4i*)(pb1 + t * kTileBytes));
    };
    auto read_s = [&](int t) __attribute__((always_inline)) { return (DWDP_TILE_DBG & 32) ? 1.f : ps[t * 64]; };
    auto mul = [&](int t, const v8i& bf, v4f& p0, v4f& p1) __attribute__((always_inline)) {
      if (DWDP_TILE_DBG & 1) return;
      if (DWDP_TILE_DBG & 64) {
        acc[0][t] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(af0, bf, acc[0][t], 0, 0, 0, 0, 0, 0);
        acc[1][t] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(af1, bf, acc[1][t], 0, 0, 0, 0, 0, 0);
      } else {
        p0 = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(af0, bf, zero, 0, 0, 0, 0, 0, 0);
        p1 = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(af1, bf, zero, 0, 0, 0, 0, 0, 0);
      }
    };
    auto fold = [&](int t, const v4f& p0, const v4f& p1, float sa) __attribute__((always_inline)) {
      if (DWDP_TILE_DBG & (1 | 64)) return;
      // timing experiment 2048: no scale products (wrong results)
      const float s0 = (DWDP_TILE_DBG & 2048) ? sa : sa * w0;
      const float s1 = (!G1 || (DWDP_TILE_DBG & 2048)) ? s0 : sa * w1;  // GEMM-2: both tiles lie in one scale block
      // whole-vector read and write of the accumulator: element-wise stores into it under
      // nested conditions keep the compiler from holding the array in registers
      v4f a0v = acc[0][t], a1v = acc[1][t];
#pragma unroll
      for (int i = 0; i < 4; i++) a0v[i] = fmaf(p0[i], s0, a0v[i]);
#pragma unroll
      for (int i = 0; i < 4; i++) a1v[i] = fmaf(p1[i], s1, a1v[i]);
      acc[0][t] = a0v;
      acc[1][t] = a1v;
    };
    // operations of the next fetch that follow tile t / that have not been issued before tile t
    auto ops_at = [&](int t) __attribute__((always_inline)) {
#pragma unroll
      for (int op = 0; op < kVmemPerStep; op++)
        if (op_slot(op) == t && (op != kBP || kNextHasScales)) issue_op(op, pos_n, lbn, an);
    };
    // Token tiles in pairs behind one wave-uniform branch per pair (a pair past the expert's
    // last row only settles the scaling still pending); the operations of the next fetch are
    // issued between the pairs, whether or not they were multiplied.  With an odd tile count
    // the last pair multiplies one tile of repeated rows.
    // Per tile t, in program order: issue the LDS read of tile t+1's operand, multiply tile t
    // (its operand was requested one tile ago), scale tile t-1's products, then request tile
    // t+1's activation scale into the register that scaling has just released.  LDS reads
    // return in order, so each use waits exactly until its own read has landed and never for
    // the younger ones.
    // issue order inside a tile: operand reads, then each MFMA followed by the five VALU
    // operations that scale the older products of the same weight tile, then the scale read
    auto tile_order = []() __attribute__((always_inline)) {
      __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);  // LDS reads (operand, kBDepth tiles ahead)
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);  // MFMA
      __builtin_amdgcn_sched_group_barrier(0x002, 5, 0);  // VALU
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
      __builtin_amdgcn_sched_group_barrier(0x002, 5, 0);
      __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
    };
    int ntt_v = ntt;
    asm volatile("" : "+s"(ntt_v));  // compared afresh in every block: the comparisons stay scalar compares
#pragma unroll
    for (int t = 0; t < kBDepth; t++) bf[t] = read_b(t);
    sa[0] = read_s(0);
    auto tile = [&](auto t_const) __attribute__((always_inline)) {
      constexpr int t = decltype(t_const)::value;
      if constexpr (t + kBDepth < kTT) bf[(t + kBDepth) % (kBDepth + 1)] = read_b(t + kBDepth);
      mul(t, bf[t % (kBDepth + 1)], p0[t % 2], p1[t % 2]);
      if constexpr (t > 0) fold(t - 1, p0[(t - 1) % 2], p1[(t - 1) % 2], sa[(t - 1) % 2]);
      if constexpr (t + 1 < kTT) sa[(t + 1) % 2] = read_s(t + 1);
      tile_order();
    };
    static_for<kTT / 2>([&](auto pair_const) __attribute__((always_inline)) {
      constexpr int t = 2 * decltype(pair_const)::value;
      if (t < ntt_v) {
        tile(std::integral_constant<int, t>{});
        __builtin_amdgcn_sched_barrier(0);
        tile(std::integral_constant<int, t + 1>{});
      }
      __builtin_amdgcn_sched_barrier(0);
      ops_at(t);
      ops_at(t + 1);
      __builtin_amdgcn_sched_barrier(0);
    });
    // the scaling still pending after the last pair that was multiplied
    static_for<kTT / 2>([&](auto pair_const) __attribute__((always_inline)) {
      constexpr int t = 2 * decltype(pair_const)::value + 2;
      if (t - 2 < ntt_v && t >= ntt_v) fold(t - 1, p0[1], p1[1], sa[1]);
    });
    const int kn = min(kb + 1, nkb - 1);
    wc0 = *(cf32)(sw[0] + kn);
    wc1 = *(cf32)(sw[1] + kn);
  };
  static_assert(kTT / 2 >= kVmemPerStep - 1 && kTT % 2 == 0, "every operation has a tile to follow");

  // "block kb has landed for everyone, and everyone is done with the image that the next
  // issue overwrites": own copies complete (in-order counter), then one barrier.
  // n_next: operations of the following block's fetch, the only ones that may be outstanding
  auto publish = [&](auto n_next) {
    if (DWDP_TILE_DBG & 16) return;
    // pinned between scheduling barriers: nothing of the following issue (its address
    // arithmetic reuses registers of retired loads) may move above the wait
    __builtin_amdgcn_sched_barrier(0);
    __builtin_amdgcn_s_waitcnt(wait_vm_lgkm0(decltype(n_next)::value));
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_sched_barrier(0);
  };

  auto keep = [](const AFrag& a) {
    asm volatile("" ::"v"(a.t[0][0]), "v"(a.t[0][1]), "v"(a.t[1][0]), "v"(a.t[1][1]));
  };
  AFrag a0 = {}, a1 = {}, a2 = {};
  using std::integral_constant;
  issue(0, true, lds_b0, a0);
  issue(1, false, lds_b1, a1);
  for (int kb = 0; kb < nkb; kb += 3) {
    publish(integral_constant<int, kVmemNoScale>{});  // position kb+1 has no scale copy
    compute(integral_constant<int, 0>{}, lds_b0, a0, kb, lds_b2, a2);
    if (kb + 1 < nkb) {
      publish(integral_constant<int, kVmemNoScale>{});
      compute(integral_constant<int, 1>{}, lds_b1, a1, kb + 1, lds_b0, a0);
    }
    if (kb + 2 < nkb) {
      publish(integral_constant<int, kVmemPerStep>{});  // position kb+3 starts a triple
      compute(integral_constant<int, 2>{}, lds_b2, a2, kb + 2, lds_b1, a1);
    }
  }
  // Drain the ring's surplus copies before LDS is reused.  The fragments are named as
  // operands after the wait so that their registers stay allocated until every load that
  // targets them has landed: a register freed earlier could be handed to another value and
  // then be overwritten by a late load.
  __builtin_amdgcn_sched_barrier(0);
  __builtin_amdgcn_s_waitcnt(kWaitVm0);
  keep(a0);
  keep(a1);
  keep(a2);
  __builtin_amdgcn_sched_barrier(0);
  __syncthreads();
  if ((DWDP_TILE_DBG & 1024) && threadIdx.x == 0 && (blockIdx.x == 0 || blockIdx.x == 1001)) {
    const long long dc = clock64() - dbg_c0, dw = wall_clock64() - dbg_w0;
    printf("tile kernel G1=%d block %d: %lld cycles, %lld ticks of 10 ns -> %.0f MHz, %d K blocks\n", (int)G1, (int)blockIdx.x, dc, dw, (double)dc / (double)dw * 100.0, nkb);
  }

  if (G1) {
    const int njb = I / 128;
    float* lds_amax = (float*)lds_epi;  // [8 waves][kBM]
    // h = silu(gate) * up, kept in acc[0]
#pragma unroll
    for (int t = 0; t < kTT; t++) {
      float amax = 0.f;
      if (t < ntt) {
#pragma unroll
        for (int i = 0; i < 4; i++) {
          const float g = acc[0][t][i], u = acc[1][t][i];
          const float v = g / (1.f + __expf(-g)) * u;
          acc[0][t][i] = v;
          amax = fmaxf(amax, fabsf(v));
        }
      }
      amax = fmaxf(amax, __shfl_xor(amax, 16));
      amax = fmaxf(amax, __shfl_xor(amax, 32));
      if (lq == 0) lds_amax[wave * kBM + t * 16 + lr] = amax;
    }
    __syncthreads();
#pragma unroll
    for (int t = 0; t < kTT; t++) {
      if (t < ntt) {
        const int tok = t * 16 + lr;
        float amax = 0.f;
#pragma unroll
        for (int w = 0; w < kTileWaves; w++) amax = fmaxf(amax, lds_amax[w * kBM + tok]);
        const float scale = amax > 0.f ? amax / 448.f : 1.f;
        const int r = r0 + tok;
        if (r < r_end) {
          const uint32_t q =
              pack_fp8x4(acc[0][t][0] / scale, acc[0][t][1] / scale, acc[0][t][2] / scale, acc[0][t][3] / scale);
          *(uint32_t*)(hq + (size_t)r * I + panel * 128 + wave * 16 + lq * 4) = q;
          if (wave == 0 && lq == 0) hs[(size_t)r * njb + panel] = scale;
        }
      }
    }
  } else {
    // bf16 output through LDS: a lane holds 4 consecutive n of ONE token, so direct stores
    // would be 8-byte pieces scattered over 16 rows; staged per wave as [16 tokens][32 n]
    // (row pitch 80 B against bank conflicts) a lane stores 16 bytes and 4 lanes cover one
    // token's 64 contiguous bytes.
    constexpr int kPitch = kStagePitch;
    uint8_t* stage = lds_epi + wave * (16 * kPitch);
    const int n_wave = panel * 256 + wave * 32;
    if (n_wave < H) {
#pragma unroll
      for (int t = 0; t < kTT; t++) {
        if (t < ntt) {
#pragma unroll
          for (int j = 0; j < 2; j++) {
            uint2 o;
            o.x = (uint32_t)f32_to_bf16(acc[j][t][0]) | ((uint32_t)f32_to_bf16(acc[j][t][1]) << 16);
            o.y = (uint32_t)f32_to_bf16(acc[j][t][2]) | ((uint32_t)f32_to_bf16(acc[j][t][3]) << 16);
            *(uint2*)(stage + lr * kPitch + (j * 16 + lq * 4) * 2) = o;
          }
          const int tok = lane >> 2, chunk = lane & 3;
          const v4i v = *(const v4i*)(stage + tok * kPitch + chunk * 16);
          const int r = r0 + t * 16 + tok;
          if (r < r_end) *(v4i*)(yp + (size_t)r * H + n_wave + chunk * 8) = v;
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
