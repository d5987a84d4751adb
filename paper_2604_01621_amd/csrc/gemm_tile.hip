// LDS-tiled FP8 grouped GEMM for gfx950: the large-M (prefill-shaped) path.
//
// A workgroup of 8 waves computes a 256 (weight rows) x 288 (tokens) output tile of one
// expert; 288 tokens cover almost every expert of the prefill workload (256 +- 16 rows),
// so each weight panel is read from HBM once.  Per 128-wide K block -- exactly one
// weight-scale block and one activation-scale group:
//   * tokens (B operand, shared by all waves): 288 rows x 128 bytes = 36 KiB, gathered
//     through the permutation by asynchronous global->LDS copies (global_load_lds_dwordx4,
//     8 whole 128-byte rows per instruction, 16-byte chunks XOR-swizzled against LDS bank
//     conflicts) into a ring of three LDS images, two K blocks ahead;
//   * weights (A operand): wave w owns 32 rows of the panel that no other wave needs, so they
//     bypass LDS: tile-major weights are loaded straight into MFMA operand registers into a
//     ring of three register sets, two K blocks ahead.
// LDS capacity bounds how far ahead a workgroup can fetch; staging only the shared operand
// in LDS halves the bytes per stage, which is what lets both operands run two blocks ahead.
//
// The multiply runs on v_mfma_f32_32x32x64_f8f6f4: per K block and 32-token tile two
// instructions (the two 64-wide halves of the block, the second accumulating onto the first)
// give the 32 x 32 partial products, which the VALU then folds into the accumulators with
// s_act[token,kb] * s_w[row block,kb].  The instruction shape matters because matrix and
// vector instructions leave through the same issue port: measured on this part, a
// 16x16x128 instruction (32 cycles of matrix pipe) leaves room for 4.4 vector operations and
// the scaling needs 5 per instruction (4 accumulates and a scale product), while a 32x32x64
// instruction (64 cycles) leaves room for 12 and needs 9.
//
// Synchronisation is explicit: vector-memory operations complete in order and every wave
// issues the same operations per K block (5 token pieces, 4 weight loads, every third block a
// scale copy; spread between the token tiles of the running multiply, because a wave that
// issues them in one burst sits at the memory pipeline's door instead of feeding the MFMA),
// so "everything of block kb has landed" is s_waitcnt vmcnt(n) with n = the operations of
// block kb+1 (9, or 10 when it carries a scale copy) -- only those may still be in flight --
// followed by one s_barrier per K block.  Past the end of K the ring keeps issuing (clamped
// to the last block) so the count stays valid.
//
// The multiply of a K block is a chain of 32-token tiles, each behind one scalar branch (tiles
// beyond the expert's row count are skipped), and inside a tile the code is straight-line:
// LDS reads of the next operand half, an MFMA, nine VALU operations that scale the previous
// tile's products, again for the second half, the LDS read of the next tile's activation
// scale.  LDS reads return in order, so every use waits for exactly its own read
// (lgkmcnt(n) with the younger reads still in flight).  That only works while no scalar load
// is pending (scalar loads share the counter and return out of order: with one in flight
// every wait becomes a wait for everything), so the weight scales of block kb+1 are loaded at
// the end of block kb's multiply and waited for together with the vector-memory wait.
//
// Scheduling: ONE persistent launch of at most one workgroup per compute unit computes both
// grouped GEMMs of the listed experts.  Work items are (M tile, weight panel) pairs, first all of
// GEMM-1 (gate/up + SwiGLU, 128 h columns per panel), then all of GEMM-2 (down, 256 output rows per
// panel); a workgroup takes its next item with an atomic ticket.  There is one ticket queue per
// XCD (the eight dies have private L2 caches): M tile m belongs to the queue of XCD m % 8 and its
// panels are consecutive tickets, so the workgroups of one die work on the same M tile at the same
// time and share its token rows in that die's L2; with many M tiles (kPairMinTiles or more) a
// queue takes list neighbours in pairs, panel by panel -- (pair, panel 0, first), (pair, panel 0,
// second), (pair, panel 1, first) ... -- so that the further M tiles of an expert with many rows
// fetch a weight panel while the die's L2 still holds it.  A workgroup whose own queue is empty
// takes tickets of the other dies' queues.  A GEMM-2 item reads the h rows of its M tile, which
// the GEMM-1 items of that tile write: each finished GEMM-1 item adds one (release, device scope)
// to the tile's counter and a GEMM-2 item waits (acquire) until the counter has reached the
// number of GEMM-1 panels.  The wait ends: tickets of a queue are handed out in order, GEMM-1
// items first, so when a workgroup holds a GEMM-2 ticket every GEMM-1 ticket of that queue is
// already held by a workgroup that is running.  As a second line of defence the wait is bounded
// (kSpinLimit polls); a workgroup that gives up raises the error word and goes on, so the grid
// always drains.  Compared with one workgroup per item this launches no workgroup that only
// exits (each needs a whole compute unit to start), has no partial last round, and keeps the
// compute units the tiled chain holds from GEMM-1 through GEMM-2 while other kernels (the
// weight-streaming chain, a prefetch copy) fill the rest of the chip.  `phase_mask` restricts a
// launch to the items of one GEMM (1 or 2; then no waiting takes place: stream order separates
// the launches); 3 is the fused launch.
//
// GEMM-1 (G1): wave w owns gate rows and up rows of 16 h columns of the panel (the 32 rows of
// its A operand), epilogue silu(g)*u, per-token amax over the panel's 128 h columns (LDS, 8
// waves), e4m3 quantisation of h.  GEMM-2: wave w owns rows 32w..32w+31 of the 256-row
// panel, bf16 store through an LDS transpose.  Experts with few rows are left to the
// streaming kernels.
#include <type_traits>
#include <utility>

#include "dwdp_kernels.h"

namespace dwdp {

typedef float v16f __attribute__((ext_vector_type(16)));

constexpr int kBM = kTileM;     // tokens per workgroup tile (288)
constexpr int kTT = kBM / 32;   // 32-token tiles per workgroup (9)
constexpr int kPairMinTiles = 32;  // M tiles from which an XCD takes them in pairs (4 per XCD)
constexpr int kTileWaves = 8;
constexpr int kTileThreads = 64 * kTileWaves;
constexpr int kLdsB = kBM * 128;         // one token image: 36 KiB
constexpr int kBPieces = kBM / 8;        // 1 KiB pieces (8 rows) of a token image
constexpr int kBP = (kBPieces + kTileWaves - 1) / kTileWaves;  // pieces copied per wave (5)
constexpr int kSaLen = 64 * kTileWaves;  // scale slots per image: every wave copies 64
// epilogue scratch: GEMM-1 keeps one amax per (wave, token), GEMM-2 stages 32 tokens x 80 bytes per wave
constexpr int kStagePitch = 80;
constexpr int kEpiBytes =
    kTileWaves * kBM * 4 > kTileWaves * 32 * kStagePitch ? kTileWaves * kBM * 4 : kTileWaves * 32 * kStagePitch;
static_assert(kBM % 32 == 0 && kBM <= kSaLen, "whole 32-token tiles, one scale slot per token");
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

// Read-only data addressed with wave-uniform pointers: the constant address space makes
// these scalar loads (s_load), which do not touch the vector-memory counter.
typedef const __attribute__((address_space(4))) float* cf32;

__device__ __forceinline__ v8i cat8(v4i lo, v4i hi) { return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7); }

// Asynchronous global -> LDS copy of 64 lanes x 16 (or 12) bytes: lane l's bytes land at
// dst + l*16; dst is a wave-uniform LDS byte offset and goes through M0.  Issued from inline
// assembly for the same reason as the weight loads below: the compiler must not model these
// operations, all waiting on them is done with explicit s_waitcnt.
__device__ __forceinline__ uint32_t lds_offset(const void* p) {
  return (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const void*)p;
}
// The source is a wave-uniform base (scalar register pair) plus a 32-bit per-lane byte offset.
__device__ __forceinline__ void dma16(const uint8_t* base_uniform, uint32_t off_lane, uint32_t dst_wave_uniform) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(dst_wave_uniform), "v"(off_lane),
               "s"(base_uniform)
               : "memory");
}
// 12 bytes per lane; lane l's bytes land at dst + l*16 (measured: the fourth dword of a slot is not written)
__device__ __forceinline__ void dma12(const float* base_uniform, uint32_t off_lane, uint32_t dst_wave_uniform) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx3 %1, %2" ::"s"(dst_wave_uniform), "v"(off_lane),
               "s"(base_uniform)
               : "memory");
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

// The 32 weight rows of a wave for one K block in the operand layout of the 32x32x64
// instruction: t[c][h] = this lane's bytes 16h..16h+15 of the 32 it feeds to the instruction
// of the block's 64-wide half c (16 registers in all).
// MXFP4 weights: t[0][c] = the 32 four-bit elements of half c (16 bytes), s[c] = the dword
// whose byte (K block % 4) is their E8M0 scale; t[1][*] unused.
struct AFrag {
  v4i t[2][2];
  int s[2];
};

// LDS of a workgroup, declared once in the kernel and handed to the item functions (a function-local
// __shared__ array in a template would be allocated once per instantiation).
struct TileLds {
  // Three token images, each its own array so that the compiler can tell a copy into one from
  // the reads of another.
  uint8_t* b0;
  uint8_t* b1;
  uint8_t* b2;
  // activation scales of three consecutive K blocks per token slot (16-byte slots, the layout
  // the 12-byte copy writes), double-buffered by block triple
  float* sg0;
  float* sg1;
  int32_t* row;
  uint8_t* epi;  // amax / store staging
};

// One work item: the kBM x (128 h columns | 256 output rows) tile (M tile starting at sorted row r0 of
// expert e, panel `panel`).  G1: act/act_s = quantised x, writes hq/hs; otherwise act/act_s = hq/hs,
// writes yp.  All threads of the workgroup call it with the same arguments; it starts and ends
// with the workgroup's LDS free for reuse (a barrier separates it from what follows).
// MX = false: FP8 e4m3 weights (packed 2 KiB tiles, fp32 scale per 128x128 block, applied by the
// VALU scaling).  MX = true: MXFP4 weights (packed 1 KiB tiles of E2M1 codes, one E8M0 scale per
// 32 along K, applied by the matrix instruction itself), FP8 activations as before.
template <bool G1, bool MX>
__device__ __forceinline__ void tile_item(const TileLds& L, const dwdp_expert_ptrs* __restrict__ table,
                                          const int32_t* __restrict__ perm, int e, int r0, int r_end, int panel,
                                          const uint8_t* __restrict__ act, const float* __restrict__ act_s,
                                          uint8_t* __restrict__ hq, float* __restrict__ hs,
                                          uint16_t* __restrict__ yp, int E, int T, int H, int I, int K) {
  uint8_t* const lds_b0 = L.b0;
  uint8_t* const lds_b1 = L.b1;
  uint8_t* const lds_b2 = L.b2;
  float* const lds_sg0 = L.sg0;
  float* const lds_sg1 = L.sg1;
  int32_t* const lds_row = L.row;
  uint8_t* const lds_epi = L.epi;
  const int valid = min(kBM, r_end - r0);
  const int ntt = (valid + 31) >> 5;  // 32-token tiles that hold rows of the expert

  // Everything below is recomputed per item on purpose.  The thread index and the sizes pass
  // through empty asm statements so that the compiler cannot hoist the (many) lane offsets and
  // addresses derived from them out of the scheduler's loop, where the hoisted values of both
  // GEMMs' item functions would stay live across every item and push the K loops into spilling.
  int tid = threadIdx.x;
  asm volatile("" : "+v"(tid));
  asm volatile("" : "+s"(H), "+s"(I), "+s"(K), "+s"(T), "+s"(E));
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // scalar: pointers derived from it stay in SGPRs
  const int lane = tid & 63;
  const int ln = lane & 31;  // the weight row (A operand) and the token (B operand) this lane feeds
  const int lg = lane >> 5;  // which 32 of the 64 K bytes of an instruction
  const int Kdim = G1 ? H : I;  // reduction length
  const int nkb = Kdim / 128;
  __builtin_assume(nkb >= 1);  // the host rejects reduction lengths that are not positive multiples of 128
  const int n_tile_rows = (G1 ? 2 * I : H) / 16;
  const uint8_t* wbase = (const uint8_t*)(G1 ? table[e].w13 : table[e].w2);
  const float* sbase = G1 ? table[e].s13 : table[e].s2;

  // ---- sources, fixed over the K loop ----
  // weights: this wave's two packed 16-row tiles (G1: gate tile and up tile of 16 h columns;
  // GEMM-2: 32 consecutive rows).  Rows 0..15 of the A operand are tile 0, rows 16..31 tile 1.
  constexpr int kABytes = MX ? 1024 : kTileBytes;  // one packed 16-row tile of one K block
  const uint8_t* a_src[2];
  const float* sw[2];
  const uint8_t* ms_src[2];
#pragma unroll
  for (int j = 0; j < 2; j++) {
    int tr;
    if (G1)
      tr = (j == 0 ? 0 : I / 16) + panel * 8 + wave;
    else
      tr = min(panel * 16 + wave * 2 + j, n_tile_rows - 1);
    a_src[j] = wbase + (size_t)tr * nkb * kABytes;  // wave-uniform
    sw[j] = sbase + (size_t)(tr / 8) * nkb;  // 8 tiles of 16 rows per 128-row scale block (FP8 weights)
    ms_src[j] = (const uint8_t*)sbase + (size_t)tr * ((nkb + 3) >> 2) * 256;  // packed E8M0 scales (MXFP4 weights)
  }
  // Inside a packed tile, byte half*1024 + (q*16 + r)*16 + b is element (row r, column
  // 32q + 16*half + b).  The instruction of half c wants from lane (ln, lg) the 32 columns
  // 64c + 32lg .. +31 of row ln: q = 2c + lg, both 16-byte halves.  One load per (c, half)
  // with a per-lane offset (tile 1 lies a fixed distance behind tile 0) and an immediate.
  // MXFP4: a packed tile holds at (q*16 + r)*16 the 32 elements 32q..32q+31 of row r, and the scale
  // group of four K blocks holds at (q*16 + r)*4 their four scale bytes: the same lane offsets
  // with 16 and 4 bytes per lane, half c at +512 and +128.
  const uint32_t a_voff = (uint32_t)((ln >> 4) ? (a_src[1] - a_src[0]) : 0) + (uint32_t)((lg * 16 + (ln & 15)) * 16);
  const uint32_t ms_voff = (uint32_t)((ln >> 4) ? (ms_src[1] - ms_src[0]) : 0) + (uint32_t)((lg * 16 + (ln & 15)) * 4);
  // tokens: the source row of every token slot of the tile (slots past the end repeat the last row)
  for (int i = tid; i < kSaLen; i += kTileThreads) {
    const int row = min(r0 + i, r_end - 1);
    lds_row[i] = G1 ? ((e < E) ? perm[row] / K : row - T * K) : row;
  }
  __syncthreads();
  // This wave's token pieces: piece c = rows 8c..8c+7 of the image, all 128 K bytes of each
  // row, so that 8 consecutive lanes fetch one whole 128-byte line (lanes that fetch from
  // different lines are served one after the other by the address unit).  Lane l's 16 bytes
  // land in slot l of the piece; the image is row-major (128 bytes per token) and slot
  // (row, p) holds the row's 16-byte chunk p ^ swz(row).  With this XOR the 128-bit operand
  // reads below (lane (ln, lg) reads chunks 4c + 2lg and 4c + 2lg + 1 of row ln) run at the
  // full LDS rate -- measured: 550 bytes/ns per CU against 76 for a plain row-major image and
  // 300 for XORs with the row's low bits.  Slots past the image repeat the last piece.
  auto swz = [](int row) { return (row >> 1) & 7; };
  uint32_t b_src[kBP];
#pragma unroll
  for (int i = 0; i < kBP; i++) {
    const int c = min(wave + kTileWaves * i, kBPieces - 1);
    const int row = c * 8 + (lane >> 3);
    b_src[i] = (uint32_t)lds_row[row] * Kdim + (((lane & 7) ^ swz(row)) << 4);
  }
  // operand reads: byte offset of chunk 2lg of row ln inside a 32-token tile; chunk 2lg+1 is
  // at ^16, the chunks of the second half of the K block at ^64
  // With an FP4 A operand the instruction pairs K elements by position, and the position of an
  // 8-bit operand's bytes is registers 0..3 = bytes 16lg..16lg+15 and registers 4..7 = bytes
  // 32+16lg.. of the 64 (measured with single-element probes); with two 8-bit operands any order
  // both share works, and the contiguous one is used.
  constexpr int kBSecond = MX ? 32 : 16;  // address XOR from a lane's first 16 bytes to its second
  const int b_rd0 = ln * 128 + (((MX ? lg : 2 * lg) ^ swz(ln)) << 4);
  const uint32_t sa_src = (uint32_t)lds_row[wave * 64 + lane] * nkb;
  // LDS byte offsets of the copy targets (wave-uniform, kept in scalar registers)
  auto uniform = [](uint32_t v) { return (uint32_t)__builtin_amdgcn_readfirstlane((int)v); };
  const uint32_t img_off[3] = {uniform(lds_offset(lds_b0)), uniform(lds_offset(lds_b1)), uniform(lds_offset(lds_b2))};
  const uint32_t sg_off[2] = {uniform(lds_offset(lds_sg0) + wave * (64 * 16)),
                              uniform(lds_offset(lds_sg1) + wave * (64 * 16))};

  v16f acc[kTT];
#pragma unroll
  for (int t = 0; t < kTT; t++)
#pragma unroll
    for (int i = 0; i < 16; i++) acc[t][i] = 0.f;

  // One of the kVmemPerStep vector-memory operations that fetch a K block: ops 0..kBP-1 copy
  // token pieces, op kBP the activation scales, the last four load this wave's weights.
  // The weight loads are issued from inline assembly so that the compiler does not model
  // them: it cannot order loads that stay in flight across the loop's back edge and would
  // drain the whole queue before the first MFMA of every block.  Their completion is covered
  // by the explicit s_waitcnt in publish(); the registers are read-write operands so each
  // fragment keeps its registers, and nothing reads them between issue and wait.
  // the tile of the running multiply after which operation i of the next fetch is issued
  auto op_slot = [](int i) { return i < kVmemPerStep - 1 ? i : kTT - 1; };
  // One operation of the fetch of the pos-th block of the walk over K (block min(pos, nkb-1):
  // past the end the ring re-fetches the last block so that the counts the waits rely on stay
  // the same) into image ring slot IMG.  Operation kBP, the scale copy, exists only for
  // pos % 3 == 0 and brings the scales of blocks pos..pos+2 (with nkb % 3 != 0 the last copy
  // reads one or two floats past a token's row: the next row's, or the padding the workspace
  // keeps behind the array).
  auto issue_op = [&](int op, int pos, int img, AFrag& a) __attribute__((always_inline)) {
    const int kb = min(pos, nkb - 1);
    if (op < kBP) {
      const int c = min(wave + kTileWaves * op, kBPieces - 1);
      dma16(act, b_src[op] + (uint32_t)kb * 128, img_off[img] + c * 1024);
    } else if (op == kBP) {
      dma12(act_s, (sa_src + (uint32_t)kb) * 4, sg_off[(pos / 3) & 1]);
    } else {
      const int w = op - kBP - 1;  // FP8: 0..3 = (c, half); MXFP4: codes of half 0, half 1, scales of half 0, half 1
      if (!MX) {
        const uint8_t* base = a_src[0] + (size_t)kb * kABytes;  // wave-uniform: scalar registers
        if (w == 0)
          asm volatile("global_load_dwordx4 %0, %1, %2 nt" : "+v"(a.t[0][0]) : "v"(a_voff), "s"(base));
        else if (w == 1)
          asm volatile("global_load_dwordx4 %0, %1, %2 offset:1024 nt" : "+v"(a.t[0][1]) : "v"(a_voff), "s"(base));
        else if (w == 2)
          asm volatile("global_load_dwordx4 %0, %1, %2 offset:512 nt" : "+v"(a.t[1][0]) : "v"(a_voff), "s"(base));
        else
          asm volatile("global_load_dwordx4 %0, %1, %2 offset:1536 nt" : "+v"(a.t[1][1]) : "v"(a_voff), "s"(base));
      } else {
        const uint8_t* base = a_src[0] + (size_t)kb * kABytes;
        const uint8_t* sbase_kb = ms_src[0] + (size_t)(kb >> 2) * 256;
        if (w == 0)
          asm volatile("global_load_dwordx4 %0, %1, %2 nt" : "+v"(a.t[0][0]) : "v"(a_voff), "s"(base));
        else if (w == 1)
          asm volatile("global_load_dwordx4 %0, %1, %2 offset:512 nt" : "+v"(a.t[0][1]) : "v"(a_voff), "s"(base));
        else if (w == 2)
          asm volatile("global_load_dword %0, %1, %2" : "+v"(a.s[0]) : "v"(ms_voff), "s"(sbase_kb));
        else
          asm volatile("global_load_dword %0, %1, %2 offset:128" : "+v"(a.s[1]) : "v"(ms_voff), "s"(sbase_kb));
      }
    }
  };
  // the whole fetch of position pos (prologue)
  auto issue = [&](int pos, bool has_scales, int img, AFrag& a) {
#pragma unroll
    for (int op = 0; op < kVmemPerStep; op++)
      if (op != kBP || has_scales) issue_op(op, pos, img, a);
  };

  // Weight scales of the block about to be multiplied: scalar loads issued at the end of the
  // previous block's multiply and waited for in publish(), so that no scalar load is pending
  // while LDS reads are in flight.
  float wc0 = MX ? 1.f : *(cf32)(sw[0]), wc1 = MX ? 1.f : *(cf32)(sw[1]);
  // Multiply block kb from (image IMG, a) and, spread between its token tiles, issue the
  // fetch of position kb + 2 into (image IMGN, an): issued in one burst the operations keep
  // the wave at the memory pipeline's door for as long as the transfers take, one per tile
  // they slip in under the MFMAs.
  // C = kb % 3 is a compile-time constant of each unrolled call: it selects this block's scale
  // inside its triple and tells whether the fetch issued here (position kb + 2) has a scale copy.
  auto compute = [&](auto c_const, auto img_const, const AFrag& a, int kb, auto imgn_const, AFrag& an)
                     __attribute__((always_inline)) {
    constexpr int C = decltype(c_const)::value;
    constexpr int IMG = decltype(img_const)::value, IMGN = decltype(imgn_const)::value;
    constexpr bool kNextHasScales = (C + 2) % 3 == 0;
    const int pos_n = kb + 2;
    const float w0 = wc0, w1 = wc1;
    const v4i zero4 = {0, 0, 0, 0};
    const v8i af0 = MX ? cat8(a.t[0][0], zero4) : cat8(a.t[0][0], a.t[0][1]);
    const v8i af1 = MX ? cat8(a.t[0][1], zero4) : cat8(a.t[1][0], a.t[1][1]);
    // MXFP4: this block's scale byte moved to byte 0 of the scale operand
    const int ms0 = MX ? (int)((uint32_t)a.s[0] >> (8 * (kb & 3))) : 0;
    const int ms1 = MX ? (int)((uint32_t)a.s[1] >> (8 * (kb & 3))) : 0;
    // cbsz 4: A is FP4 E2M1; blgp 0: B is FP8 E4M3; A scale = byte 0 of ms; B scale 127 = 1.0
    auto mfma = [&](const v8i& af, const v8i& bf, const v16f& c, int ms) __attribute__((always_inline)) -> v16f {
      if (MX) return __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(af, bf, c, 4, 0, 0, ms, 0, 0x7f7f7f7f);
      return __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(af, bf, c, 0, 0, 0, 0, 0, 0);
    };
    const uint8_t* lb = IMG == 0 ? lds_b0 : (IMG == 1 ? lds_b1 : lds_b2);
    const uint8_t* pb00 = lb + b_rd0;         // half 0 of the block, bytes 0..15 of the lane's 32
    const uint8_t* pb01 = lb + (b_rd0 ^ kBSecond);  //                the lane's second 16 bytes
    const uint32_t ab0 = lds_offset(pb00), ab1 = lds_offset(pb01);
    const float* ps = (((kb / 3) & 1) ? lds_sg1 : lds_sg0) + ln * 4 + C;
    v16f zero;
#pragma unroll
    for (int i = 0; i < 16; i++) zero[i] = 0.f;
    // Two operand buffers alternate between the halves of the K block (the read of the next
    // half is in flight while the MFMA of this one runs).  One set of product registers: the
    // products of a tile are scaled right after its second MFMA, which this wave has to wait
    // for -- the other wave of the SIMD owns the matrix pipe meanwhile (a second product set
    // would hide the wait inside one wave but does not fit the register file).
    v8i bq[2];
    v16f pr = zero;
    float sa[2] = {0.f, 0.f}, sp0 = 0.f, sp1 = 0.f;
    auto read_b = [&](int t, int c) __attribute__((always_inline)) -> v8i {
      // half 1 of the block: chunk index + 4, which the swizzle turns into address ^ 64 (formed
      // when needed: two more resident address registers do not fit)
      typedef __attribute__((address_space(3))) const uint8_t* lp;
      if (c == 0) return cat8(*(const v4i*)(pb00 + t * 4096), *(const v4i*)(pb01 + t * 4096));
      return cat8(*(const __attribute__((address_space(3))) v4i*)((lp)(uintptr_t)(ab0 ^ 64) + t * 4096),
                  *(const __attribute__((address_space(3))) v4i*)((lp)(uintptr_t)(ab1 ^ 64) + t * 4096));
    };
    auto read_s = [&](int t) __attribute__((always_inline)) { return ps[t * 128]; };
    auto scale_products = [&](float sa_t, float& s0, float& s1) __attribute__((always_inline)) {
      if (MX) {
        s0 = s1 = sa_t;  // the weight scales were applied inside the instruction
      } else {
        s0 = sa_t * w0;
        s1 = G1 ? sa_t * w1 : s0;  // GEMM-2: the 32 rows lie in one scale block
      }
    };
    // acc[t] += products * scale: rows 0..15 of the A operand (registers 0..7) with s0, rows
    // 16..31 with s1.  Whole-vector read and write of the accumulator: element-wise stores
    // into it under conditions keep the compiler from holding the array in registers.
    auto fold = [&](int t, const v16f& p, float s0, float s1) __attribute__((always_inline)) {
      v16f av = acc[t];
#pragma unroll
      for (int i = 0; i < 8; i++) av[i] = fmaf(p[i], s0, av[i]);
#pragma unroll
      for (int i = 8; i < 16; i++) av[i] = fmaf(p[i], s1, av[i]);
      acc[t] = av;
    };
    // operations of the next fetch that follow tile t
    auto ops_at = [&](int t) __attribute__((always_inline)) {
#pragma unroll
      for (int op = 0; op < kVmemPerStep; op++)
        if (op_slot(op) == t && (op != kBP || kNextHasScales)) issue_op(op, pos_n, IMGN, an);
    };
    // issue order inside a tile: operand reads of the following half before each MFMA, then
    // the scaling, then the scale read
    auto tile_order = []() __attribute__((always_inline)) {
      __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);  // LDS reads
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);  // MFMA
      __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
      __builtin_amdgcn_sched_group_barrier(0x002, 18, 0);  // VALU
      __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
    };
    int ntt_v = ntt;
    asm volatile("" : "+s"(ntt_v));  // compared afresh in every block: the comparisons stay scalar compares
    bq[0] = read_b(0, 0);
    sa[0] = read_s(0);
    sa[1] = read_s(1);
    auto tile = [&](auto t_const) __attribute__((always_inline)) {
      constexpr int t = decltype(t_const)::value;
      bq[1] = read_b(t, 1);
      pr = mfma(af0, bq[0], zero, ms0);
      if constexpr (t + 1 < kTT) bq[0] = read_b(t + 1, 0);
      pr = mfma(af1, bq[1], pr, ms1);
      scale_products(sa[t % 2], sp0, sp1);
      fold(t, pr, sp0, sp1);
      if constexpr (t + 2 < kTT) sa[t % 2] = read_s(t + 2);
      tile_order();
    };
    static_for<kTT>([&](auto t_const) __attribute__((always_inline)) {
      constexpr int t = decltype(t_const)::value;
      if (t < ntt_v) tile(t_const);
      __builtin_amdgcn_sched_barrier(0);
      ops_at(t);
      __builtin_amdgcn_sched_barrier(0);
    });
    if (!MX) {
      const int kn = min(kb + 1, nkb - 1);
      wc0 = *(cf32)(sw[0] + kn);
      wc1 = *(cf32)(sw[1] + kn);
    }
  };
  static_assert(kTT >= kVmemPerStep - 1, "every operation has a tile to follow");

  // "block kb has landed for everyone, and everyone is done with the image that the next
  // issue overwrites": own copies complete (in-order counter), then one barrier.
  // n_next: operations of the following block's fetch, the only ones that may be outstanding
  auto publish = [&](auto n_next) {
    // pinned between scheduling barriers: nothing of the following issue (its address
    // arithmetic reuses registers of retired loads) may move above the wait
    __builtin_amdgcn_sched_barrier(0);
    __builtin_amdgcn_s_waitcnt(wait_vm_lgkm0(decltype(n_next)::value));
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_sched_barrier(0);
  };

  auto keep = [](const AFrag& a) {
    asm volatile("" ::"v"(a.t[0][0]), "v"(a.t[0][1]), "v"(a.t[1][0]), "v"(a.t[1][1]), "v"(a.s[0]), "v"(a.s[1]));
  };
  AFrag a0 = {}, a1 = {}, a2 = {};
  using std::integral_constant;
  using I0 = integral_constant<int, 0>;
  using I1 = integral_constant<int, 1>;
  using I2 = integral_constant<int, 2>;
  issue(0, true, 0, a0);
  issue(1, false, 1, a1);
  for (int kb = 0; kb < nkb; kb += 3) {
    publish(integral_constant<int, kVmemNoScale>{});  // position kb+1 has no scale copy
    compute(I0{}, I0{}, a0, kb, I2{}, a2);
    if (kb + 1 < nkb) {
      publish(integral_constant<int, kVmemNoScale>{});
      compute(I1{}, I1{}, a1, kb + 1, I0{}, a0);
    }
    if (kb + 2 < nkb) {
      publish(integral_constant<int, kVmemPerStep>{});  // position kb+3 starts a triple
      compute(I2{}, I2{}, a2, kb + 2, I1{}, a1);
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

  // Accumulator layout of the 32x32 result: this lane holds token ln of every tile and, in
  // register 4q + i (q = 0..3, i = 0..3), row 8q + 4lg + i of the wave's 32 rows.
  if (G1) {
    // rows 0..15 are the gate rows and rows 16..31 the up rows of h columns 0..15 of the wave:
    // register 4q + i (q = 0, 1) pairs with register 8 + 4q + i, h column 8q + 4lg + i
    const int njb = I / 128;
    float* lds_amax = (float*)lds_epi;  // [8 waves][kBM]
#pragma unroll
    for (int t = 0; t < kTT; t++) {
      float amax = 0.f;
      if (t < ntt) {
#pragma unroll
        for (int i = 0; i < 8; i++) {
          const float g = acc[t][i], u = acc[t][8 + i];
          const float v = g / (1.f + __expf(-g)) * u;
          acc[t][i] = v;
          amax = fmaxf(amax, fabsf(v));
        }
      }
      amax = fmaxf(amax, __shfl_xor(amax, 32));
      if (lg == 0) lds_amax[wave * kBM + t * 32 + ln] = amax;
    }
    __syncthreads();
#pragma unroll
    for (int t = 0; t < kTT; t++) {
      if (t < ntt) {
        const int tok = t * 32 + ln;
        float amax = 0.f;
#pragma unroll
        for (int w = 0; w < kTileWaves; w++) amax = fmaxf(amax, lds_amax[w * kBM + tok]);
        const float scale = amax > 0.f ? amax / 448.f : 1.f;
        const int r = r0 + tok;
        if (r < r_end) {
#pragma unroll
          for (int q = 0; q < 2; q++) {
            const uint32_t c = pack_fp8x4(acc[t][4 * q] / scale, acc[t][4 * q + 1] / scale, acc[t][4 * q + 2] / scale,
                                          acc[t][4 * q + 3] / scale);
            *(uint32_t*)(hq + (size_t)r * I + panel * 128 + wave * 16 + q * 8 + lg * 4) = c;
          }
          if (wave == 0 && lg == 0) hs[(size_t)r * njb + panel] = scale;
        }
      }
    }
  } else {
    // bf16 output through LDS: a lane holds four groups of 4 consecutive n of ONE token, so
    // direct stores would be 8-byte pieces; staged per wave as [32 tokens][32 n] (row pitch
    // 80 B against bank conflicts) a lane stores 16 bytes and 4 lanes cover one token's 64
    // contiguous bytes, 16 tokens per store instruction.
    constexpr int kPitch = kStagePitch;
    uint8_t* stage = lds_epi + wave * (32 * kPitch);
    const int n_wave = panel * 256 + wave * 32;
    if (n_wave < H) {
#pragma unroll
      for (int t = 0; t < kTT; t++) {
        if (t < ntt) {
#pragma unroll
          for (int q = 0; q < 4; q++) {
            uint2 o;
            o.x = (uint32_t)f32_to_bf16(acc[t][4 * q]) | ((uint32_t)f32_to_bf16(acc[t][4 * q + 1]) << 16);
            o.y = (uint32_t)f32_to_bf16(acc[t][4 * q + 2]) | ((uint32_t)f32_to_bf16(acc[t][4 * q + 3]) << 16);
            *(uint2*)(stage + ln * kPitch + (q * 8 + lg * 4) * 2) = o;
          }
#pragma unroll
          for (int hhalf = 0; hhalf < 2; hhalf++) {
            const int tok = hhalf * 16 + (lane >> 2), chunk = lane & 3;
            const v4i v = *(const v4i*)(stage + tok * kPitch + chunk * 16);
            const int r = r0 + t * 32 + tok;
            if (r < r_end) *(v4i*)(yp + (size_t)r * H + n_wave + chunk * 8) = v;
          }
        }
      }
    }
  }
}

// ---------------------------------------------------------------- persistent scheduler

constexpr int kSpinLimit = 1 << 22;  // polls (of about 640 cycles) a GEMM-2 item waits for its GEMM-1 items

// Layout of the scheduler's words (TileSched::sync), all zeroed by the kernel that builds the list:
//   [0, 8)   ticket queues of the fused or the GEMM-1-only launch, one per XCD
//   [8, 16)  ticket queues of the GEMM-2-only launch
//   [16]     error word: a bounded wait gave up
//   [17]     workgroups of a persistent launch that take work
//   [kSyncDone + m] finished GEMM-1 items of M tile m
static_assert(kTileSyncDone == 32, "layout documented above");

// Ticket t of queue v -> item.  Returns 0 when the queue is exhausted, 1 for an item (phase 1 or
// 2 in *phase), 2 for a ticket that names no M tile (padding of the last group) and is skipped.
__device__ __forceinline__ int decode_ticket(int t, int v, int n_mt, int p1, int p2, int phase_mask, int* phase, int* m,
                                             int* panel) {
  const bool pairs = n_mt >= kPairMinTiles;
  const int tiles = pairs ? 2 * ((n_mt + 15) / 16) : (n_mt + 7) / 8;  // M tile places of one queue
  const int n1 = (phase_mask & 1) ? tiles * p1 : 0;
  const int n2 = (phase_mask & 2) ? tiles * p2 : 0;
  if (t >= n1 + n2) return 0;
  const int ph = t < n1 ? 1 : 2;
  const int i = ph == 1 ? t : t - n1;
  const int np = ph == 1 ? p1 : p2;
  int mm;
  if (pairs) {
    const int pq = i / (2 * np), within = i - pq * (2 * np);
    *panel = within >> 1;
    mm = (pq * 8 + v) * 2 + (within & 1);
  } else {
    const int mq = i / np;
    *panel = i - mq * np;
    mm = mq * 8 + v;
  }
  *phase = ph;
  *m = mm;
  return mm < n_mt ? 1 : 2;
}

template <bool MX>
__global__ __launch_bounds__(kTileThreads, 1) void gemm_tile_persistent_kernel(
    const dwdp_expert_ptrs* __restrict__ table, const int32_t* __restrict__ offsets, const int32_t* __restrict__ perm,
    const int32_t* __restrict__ mt_expert, const int32_t* __restrict__ mt_row0, const int32_t* __restrict__ n_mtiles,
    int32_t* __restrict__ sync, int phase_mask, const uint8_t* __restrict__ xq, const float* __restrict__ xs,
    uint8_t* __restrict__ hq, float* __restrict__ hs, uint16_t* __restrict__ yp, int E, int T, int H, int I, int K) {
  __shared__ __attribute__((aligned(16))) uint8_t lds_b0[kLdsB];
  __shared__ __attribute__((aligned(16))) uint8_t lds_b1[kLdsB];
  __shared__ __attribute__((aligned(16))) uint8_t lds_b2[kLdsB];
  __shared__ __attribute__((aligned(16))) float lds_sg0[kSaLen * 4];
  __shared__ __attribute__((aligned(16))) float lds_sg1[kSaLen * 4];
  __shared__ int32_t lds_row[kSaLen];
  __shared__ __attribute__((aligned(16))) uint8_t lds_epi[kEpiBytes];
  __shared__ int32_t lds_item[4];  // phase (0 = no more work), M tile, panel
  const TileLds L{lds_b0, lds_b1, lds_b2, lds_sg0, lds_sg1, lds_row, lds_epi};

  // the list builder bounds how many workgroups of a persistent launch take work (whole rounds over
  // the dies); the others give their compute unit back at once
  if ((int)blockIdx.x >= sync[kTileSyncLimit]) return;
  const int xcd = blockIdx.x & 7;  // workgroups are dealt to the dies in turn
  const int n_mt = *n_mtiles;
  const int p1 = I / 128, p2 = (H + 255) / 256;
  int32_t* tickets = sync + (phase_mask == 2 ? 8 : 0);
  int32_t* done1 = sync + kTileSyncDone;
  int first_victim = 0;  // queues before this one (counted from the own) are known to be empty

  for (;;) {
    if (threadIdx.x == 0) {
      int phase = 0, m = 0, panel = 0;
      while (first_victim < 8) {
        const int v = (xcd + first_victim) & 7;
        const int t = atomicAdd(&tickets[v], 1);
        const int r = decode_ticket(t, v, n_mt, p1, p2, phase_mask, &phase, &m, &panel);
        if (r == 1) break;
        phase = 0;
        if (r == 0) first_victim++;
      }
      if (phase == 2 && phase_mask == 3) {
        // the h rows of this M tile are complete once all its GEMM-1 items have signalled
        int spins = 0;
        while (__hip_atomic_load(&done1[m], __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_AGENT) < p1) {
          __builtin_amdgcn_s_sleep(10);
          if (++spins > kSpinLimit) {
            atomicExch(&sync[kTileSyncError], 1);
            break;
          }
        }
      }
      lds_item[0] = phase;
      lds_item[1] = m;
      lds_item[2] = panel;
    }
    __syncthreads();
    const int phase = __builtin_amdgcn_readfirstlane(lds_item[0]);
    const int m = __builtin_amdgcn_readfirstlane(lds_item[1]);
    const int panel = __builtin_amdgcn_readfirstlane(lds_item[2]);
    if (phase == 0) return;
    // every wave orders its reads of h behind the counter it (through thread 0) has seen
    if (phase == 2 && phase_mask == 3) __atomic_thread_fence(__ATOMIC_ACQUIRE);
    // wave-uniform values go through readfirstlane so that everything derived from them
    // (weight/scale pointers, tile counts) lives in scalar registers and is loaded with s_load
    const int e = __builtin_amdgcn_readfirstlane(mt_expert[m]);
    const int r0 = __builtin_amdgcn_readfirstlane(mt_row0[m]);
    const int r_end = __builtin_amdgcn_readfirstlane(offsets[e + 1]);
    if (phase == 1) {
      tile_item<true, MX>(L, table, perm, e, r0, r_end, panel, xq, xs, hq, hs, nullptr, E, T, H, I, K);
      // all of this workgroup's h stores are ordered before the signal: barrier (workgroup
      // scope), then one release at device scope
      __syncthreads();
      if (threadIdx.x == 0) __hip_atomic_fetch_add(&done1[m], 1, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
    } else {
      tile_item<false, MX>(L, table, perm, e, r0, r_end, panel, hq, hs, nullptr, nullptr, yp, E, T, H, I, K);
      __syncthreads();  // lds_item and the epilogue staging are rewritten by the next round
    }
  }
}

// One workgroup per (M tile, panel) item of ONE GEMM, numbered so that all weight panels of an M
// tile run on the same XCD back to back and share the token rows in its L2: block b runs on XCD
// b % 8 and handles M tile (b/8 / n_panels) * 8 + b % 8, panel (b/8) % n_panels; with
// kPairMinTiles or more M tiles an XCD takes list neighbours in pairs, panel by panel (the same
// order as the persistent kernel's ticket queues).  The grid is sized from a host-side upper
// bound of the list; surplus workgroups exit.  Unlike the persistent launch, finished
// workgroups give their compute unit back, so a concurrently running kernel (the weight-streaming
// chain) gets compute units whenever this one has fewer items left than the chip has units.
template <bool G1, bool MX>
__global__ __launch_bounds__(kTileThreads, 1) void gemm_tile_item_kernel(
    const dwdp_expert_ptrs* __restrict__ table, const int32_t* __restrict__ offsets, const int32_t* __restrict__ perm,
    const int32_t* __restrict__ mt_expert, const int32_t* __restrict__ mt_row0, const int32_t* __restrict__ n_mtiles,
    int n_panels, const uint8_t* __restrict__ act, const float* __restrict__ act_s, uint8_t* __restrict__ hq,
    float* __restrict__ hs, uint16_t* __restrict__ yp, int E, int T, int H, int I, int K) {
  __shared__ __attribute__((aligned(16))) uint8_t lds_b0[kLdsB];
  __shared__ __attribute__((aligned(16))) uint8_t lds_b1[kLdsB];
  __shared__ __attribute__((aligned(16))) uint8_t lds_b2[kLdsB];
  __shared__ __attribute__((aligned(16))) float lds_sg0[kSaLen * 4];
  __shared__ __attribute__((aligned(16))) float lds_sg1[kSaLen * 4];
  __shared__ int32_t lds_row[kSaLen];
  __shared__ __attribute__((aligned(16))) uint8_t lds_epi[kEpiBytes];
  const TileLds L{lds_b0, lds_b1, lds_b2, lds_sg0, lds_sg1, lds_row, lds_epi};
  int phase, m, panel;
  const int n_mt = *n_mtiles;
  // the numbering of the persistent kernel's queues: this workgroup is ticket blockIdx / 8 of queue blockIdx % 8
  if (decode_ticket(blockIdx.x >> 3, blockIdx.x & 7, n_mt, G1 ? n_panels : 0, G1 ? 0 : n_panels, G1 ? 1 : 2, &phase, &m,
                    &panel) != 1)
    return;
  const int e = __builtin_amdgcn_readfirstlane(mt_expert[m]);
  const int r0 = __builtin_amdgcn_readfirstlane(mt_row0[m]);
  const int r_end = __builtin_amdgcn_readfirstlane(offsets[e + 1]);
  tile_item<G1, MX>(L, table, perm, e, r0, r_end, panel, act, act_s, hq, hs, yp, E, T, H, I, K);
}

int tile_mtiles_cap(int rows, int n_slots, int stream_max_rows) {
  // listed experts have more than stream_max_rows rows: at most rows / (stream_max_rows+1) of
  // them, each adding at most one partial tile to the rows / kBM full ones
  long by_rows = (long)rows / ((long)stream_max_rows + 1);
  return rows / kBM + (int)(by_rows < n_slots ? by_rows : n_slots) + 1;
}

int tile_sync_words(int mt_cap) { return kTileSyncDone + mt_cap; }

// schedule 0: one workgroup per item (phase_mask 1 or 2 only); 1: the persistent kernel.
// phase_mask 3 (persistent only): both GEMMs in one launch; 1 / 2: one of them (two launches in stream order).
void launch_gemm_fp8_tile(const GemmArgs& a, const TileSched& ts, bool mxfp4, int schedule, int phase_mask,
                          const uint8_t* xq, const float* xs, uint8_t* hq, float* hs, void* yp, int n_cus,
                          hipStream_t stream) {
  const int p1 = a.I / 128, p2 = (a.H + 255) / 256;
  if (schedule == 0) {
    const bool g1 = phase_mask == 1;
    const int n_panels = g1 ? p1 : p2;
    // covers both numberings of the kernel: M tiles rounded up to whole pairs on all 8 XCDs
    const int grid = 16 * ((ts.n_mt_max + 15) / 16) * n_panels;
    if (g1) {
      auto kern = mxfp4 ? gemm_tile_item_kernel<true, true> : gemm_tile_item_kernel<true, false>;
      hipLaunchKernelGGL(kern, dim3(grid), dim3(kTileThreads), 0, stream, a.table, a.offsets, a.perm, ts.mt_expert,
                         ts.mt_row0, ts.n_mtiles, n_panels, xq, xs, hq, hs, (uint16_t*)nullptr, a.E, a.T, a.H, a.I, a.K);
    } else {
      auto kern = mxfp4 ? gemm_tile_item_kernel<false, true> : gemm_tile_item_kernel<false, false>;
      hipLaunchKernelGGL(kern, dim3(grid), dim3(kTileThreads), 0, stream, a.table, a.offsets, a.perm, ts.mt_expert,
                         ts.mt_row0, ts.n_mtiles, n_panels, (const uint8_t*)hq, (const float*)hs, (uint8_t*)nullptr,
                         (float*)nullptr, (uint16_t*)yp, a.E, a.T, a.H, a.I, a.K);
    }
    return;
  }
  const long items = (long)ts.n_mt_max * ((phase_mask & 1 ? p1 : 0) + (phase_mask & 2 ? p2 : 0));
  // one workgroup per compute unit at most, in whole rounds over the 8 dies
  long grid = items < n_cus ? items : n_cus;
  grid = (grid + 7) / 8 * 8;
  if (grid < 8) grid = 8;
  auto kern = mxfp4 ? gemm_tile_persistent_kernel<true> : gemm_tile_persistent_kernel<false>;
  hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(kTileThreads), 0, stream, a.table, a.offsets, a.perm,
                     ts.mt_expert, ts.mt_row0, ts.n_mtiles, ts.sync, phase_mask, xq, xs, hq, hs, (uint16_t*)yp, a.E, a.T,
                     a.H, a.I, a.K);
}

}  // namespace dwdp
