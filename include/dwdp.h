/*
 * dwdp.h -- C ABI of the MI355X (gfx950) DWDP MoE-layer hot path.
 *
 * One rank of Distributed Weight Data Parallelism (paper Section 2, "Methodology
 * Overview"): the rank keeps a subset of each MoE layer's experts resident, pulls the
 * rest from peers into a double-buffered staging area one layer ahead, and runs the MoE
 * block as soon as the layer's experts have arrived.  The grouped GEMM reads every
 * expert through a pointer table, so resident and staged weights are consumed in place
 * with no merge copy (paper Section 4.2, "Eliminating Split-Weight Merge Overhead").
 *
 * General conventions
 *   - Every data pointer is DEVICE memory owned by the caller unless marked HOST.  The
 *     library never frees caller memory; it allocates its own workspace in dwdp_create.
 *   - Calls enqueue work on the context's compute stream (or its private copy stream for
 *     dwdp_prefetch_layer) and return without waiting on the device.  Buffers must stay valid
 *     until the stream has passed the call.  Calls that allocate (dwdp_create, and the first
 *     dwdp_prefetch_layer / dwdp_prepare_prefetch with given arguments in copy-kernel mode) say so.  dwdp_moe_forward may run part of its grouped GEMM
 *     on a second private stream; that work is forked from and joined back into the
 *     compute stream with events, so callers only ever order against the compute stream.
 *   - Errors are return codes; argument errors are detected on the host before anything
 *     is enqueued.  dwdp_last_error() gives a message for the last failure on a context.
 *   - Not thread-safe per context; use one context per host thread.
 *   - Row-major everywhere.  "bf16" is the upper half of an IEEE fp32.  "fp8" is OCP
 *     e4m3 (finite-only, max 448).
 */
#ifndef DWDP_H
#define DWDP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct dwdp_ctx dwdp_ctx;

typedef enum {
  DWDP_OK = 0,
  DWDP_EINVAL = 1, /* null pointer, negative size, bad enum                          */
  DWDP_ESHAPE = 2, /* shape the kernels do not support (see dwdp_create)             */
  DWDP_ENOMEM = 3, /* workspace allocation failed                                    */
  DWDP_EHIP = 4,   /* a HIP runtime call failed; message holds the HIP error string  */
  DWDP_ESTATE = 5  /* call order violates the double-buffer protocol                 */
} dwdp_status;

enum { DWDP_SCORE_SOFTMAX = 0, DWDP_SCORE_SIGMOID = 1 };
enum { DWDP_W_BF16 = 0, DWDP_W_FP8 = 1, DWDP_W_MXFP4 = 2 };

/* Shape and routing parameters of one MoE layer; all layers of a context share them. */
typedef struct {
  int32_t T_max;        /* largest token count of any call                                  */
  int32_t H;            /* hidden size                                                       */
  int32_t I;            /* expert intermediate size                                          */
  int32_t E;            /* routed experts                                                    */
  int32_t K;            /* experts per token                                                 */
  int32_t n_group;      /* expert groups for group-limited routing (1 = none)                */
  int32_t topk_group;   /* groups kept per token                                             */
  int32_t has_shared;   /* 1: slot E of the table is an always-on shared expert              */
  int32_t score_fn;     /* DWDP_SCORE_*                                                      */
  float routed_scale;   /* routing weights of a token sum to this                            */
  int32_t w_dtype;      /* DWDP_W_*                                                          */
  int32_t n_layers;     /* layers that will be addressed by dwdp_moe_forward/prefetch (>=1)  */
} dwdp_config;

/*
 * One row of the expert-pointer table (the "TensorList" of paper Section 4.2): where one
 * expert's weights are.  Entries may point into resident memory or into a staging
 * buffer; the kernels do not care.  Slot e < E is routed expert e, slot E the shared one.
 *   w13  [2I, H]  rows 0..I-1 gate projection, rows I..2I-1 up projection
 *   w2   [H, I]   down projection
 *   FP8:  1 byte/element, stored TILE-MAJOR as written by dwdp_pack_fp8_weight (the
 *         kernels stream whole 2 KiB tiles); s13 fp32 [2I/128, H/128], s2 fp32
 *         [H/128, I/128] row-major: one scale per 128x128 block of the logical matrix,
 *         weight = decode(byte) * scale.  Pointers 16-byte aligned.
 *   MXFP4: FP4 E2M1 codes, two per byte, with one E8M0 scale (2^(byte-127)) per 32 elements
 *         along K (OCP Microscaling Formats v1.0; the analogue on this hardware of the NVFP4
 *         weights of the paper's model, Section 5.1).  Codes and scales in the layouts written
 *         by dwdp_pack_mxfp4_weight; s13 / s2 point at the packed scale bytes (the pointer
 *         type is only nominal).  Pointers 16-byte aligned.
 *   bf16: 2 bytes/element, plain row-major; s13 = s2 = NULL.
 */
typedef struct {
  const void* w13;
  const float* s13;
  const void* w2;
  const float* s2;
} dwdp_expert_ptrs;

/*
 * Create a context bound to `compute_stream` (a hipStream_t; NULL = the default stream)
 * on the current device.  Allocates the workspace for T_max tokens and a private copy
 * stream at default priority.
 * Supported shapes: H, I multiples of 128; 1 <= K <= E <= 1024; K <= 32; E % n_group == 0;
 * at least 2 experts per group when n_group > 1; K <= topk_group * E / n_group;
 * T_max * (K + has_shared) * max(H, I) < 2^32 and 2 * I * H < 2^32.  DWDP_ESHAPE otherwise.
 */
dwdp_status dwdp_create(const dwdp_config* cfg, void* compute_stream, dwdp_ctx** out);
void dwdp_destroy(dwdp_ctx* ctx);
/* Message of the last failure on ctx (or of the last failed dwdp_create if ctx is NULL). */
const char* dwdp_last_error(const dwdp_ctx* ctx);

/*
 * Router top-k (the MoE arithmetic is DeepSeek-V3's, which the paper's Section 5.1 names
 * as the evaluated model).  logits fp32 [T,E]; bias fp32 [E] or NULL.
 *   sigmoid: s = fp32(1/(1+exp(-fp64(z)))); selection score c = s + bias (fp32 add);
 *            group score = sum of the two largest c of the group; keep topk_group groups,
 *            then the K largest c among them; w_k = s_k / (sum_j s_j + 1e-20) * routed_scale.
 *   softmax: selection on the raw logits (bias ignored), w = softmax over the K selected
 *            logits * routed_scale.
 * Ties go to the lower index; topk_ids [T,K] int32 are ordered by descending selection
 * score; topk_w [T,K] fp32.  T = 0 is a no-op.
 */
dwdp_status dwdp_route(dwdp_ctx* ctx, const float* logits, const float* bias, int32_t T,
                       int32_t* topk_ids, float* topk_w);

/*
 * Permutation by expert (the paper names no sorting rule; grouped GEMMs over per-expert row
 * ranges, its Section 4.2, need rows grouped by expert, and the stable order makes the
 * result unique): stable counting sort of f = t*K + k by topk_ids[f].
 *   expert_offsets int32 [E+1 (+1 if has_shared)]  exclusive prefix sums; with a shared
 *                  expert the last entry is T*K + T (its rows are T*K + t)
 *   perm     int32 [T*K]  perm[r] = f of sorted row r
 *   inv_perm int32 [T*K]  inv_perm[f] = r
 * Every topk_ids value must be in [0,E) (values outside are ignored by the histogram and
 * leave their perm rows unwritten).  T = 0 writes all-zero offsets.
 */
dwdp_status dwdp_permute(dwdp_ctx* ctx, const int32_t* topk_ids, int32_t T,
                         int32_t* expert_offsets, int32_t* perm, int32_t* inv_perm);

/*
 * dwdp_permute for callers that cannot allocate device memory and hold no context: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same outputs as
 * dwdp_permute for the same topk_ids (bit for bit); E, K, has_shared and the stream (a
 * hipStream_t, NULL = the default stream) are arguments instead of context state.  The only
 * scratch of the permutation -- the per-chunk expert histograms of the multi-workgroup path
 * used when T exceeds one chunk (1024 tokens for E <= 384) -- lives in a static device array of
 * DWDP_STATIC_SCRATCH_BYTES that every GPU the library runs on holds until the process ends;
 * the call allocates and frees nothing.  Limits: K <= E <= 1024, K <= 32 and
 * ceil(T / 128) * E * 4 <= DWDP_STATIC_SCRATCH_BYTES (T <= 131072 at E = 256); DWDP_ESHAPE
 * beyond them, with the message in dwdp_last_error(NULL).  All calls on one GPU share the array:
 * calls that may overlap on a GPU (different streams, different threads) race and must be
 * ordered by the caller.  Nothing in the array has to start at zero (every entry that is read
 * is written by the same call first).
 */
enum { DWDP_STATIC_SCRATCH_BYTES = 1 << 20 };
dwdp_status dwdp_permute_static(const int32_t* topk_ids, int32_t T, int32_t E, int32_t K, int32_t has_shared,
                                void* stream, int32_t* expert_offsets, int32_t* perm, int32_t* inv_perm);

/*
 * One MoE layer forward: route -> permute -> (FP8: quantise x per token per 128) ->
 * grouped GEMM gate/up + SwiGLU (FP8: quantise h per token per 128) -> grouped GEMM down
 * -> y[t] = sum_k w[t,k] * out[t,k] (+ shared expert, weight 1).
 *   x bf16 [T,H]; logits fp32 [T,E]; bias fp32 [E] or NULL; table [E (+1)] rows of
 *   dwdp_expert_ptrs in DEVICE memory; y bf16 [T,H] out.
 * If dwdp_prefetch_layer(layer) was issued and not yet consumed, the compute stream first
 * waits for its copies (paper Section 2: a layer waits until all remote experts have
 * arrived); when the layer is done its staging buffer (layer % 2) is released for the
 * next prefetch.  0 <= layer < n_layers.  Experts with no tokens are never read.
 */
dwdp_status dwdp_moe_forward(dwdp_ctx* ctx, int32_t layer, const void* x, const float* logits,
                             const float* bias, int32_t T, const dwdp_expert_ptrs* table, void* y);

/*
 * Prefetch the non-resident experts of `layer` into staging buffer layer % 2 on the
 * context's copy stream, as the batched copy plan in round-robin slice order of paper
 * Section 4.3.2 (Listing 1): for each parameter p, for each slice offset, for each peer in
 * the given order, one asynchronous device copy of min(slice_bytes, bytes[p] - offset).
 *   src, dst  HOST arrays [n_peers * n_params] of device pointers, index peer*n_params + p:
 *             the peer's region of parameter p and its place in the staging buffer
 *   bytes     HOST array [n_params]: bytes pulled of parameter p from each peer
 * The copies start only after the previous reader of that staging buffer has finished
 * (double buffering, paper Section 2).  DWDP_ESTATE if the buffer still holds a prefetched
 * layer that no dwdp_moe_forward has consumed.  slice_bytes = 0 means unsliced.
 */
dwdp_status dwdp_prefetch_layer(dwdp_ctx* ctx, int32_t layer, const void* const* src, void* const* dst,
                                const size_t* bytes, int32_t n_peers, int32_t n_params, size_t slice_bytes);

/*
 * Kernel selection of the FP8 / MXFP4 grouped GEMM by an expert's number of sorted rows m.
 *   1 <= m <= min(max_rows, 16): weight-streaming kernels, one 16-token tile per pass over the weights;
 *   16 < m <= max_rows (FP8 weights): the same streams with four token tiles per pass, in row
 *     groups of 64 (weights read once per 64 rows; workgroups small enough to share a compute
 *     unit with other kernels); with MXFP4 weights these experts are walked 16 rows at a time;
 *   m > max_rows: LDS-tiled kernels (288-token tiles, weights read once per tile, workgroups
 *     that each fill a compute unit) -- unless fewer than about half a chip's worth of tiles
 *     come together in a call (decided on the device) or the experts of the call average fewer
 *     than 16 rows (decided on the host): such outliers join the row groups (FP8 weights).
 * Default: 64 with FP8 weights, 16 with MXFP4 weights.  0 sends every expert to the tiled
 * kernels; a value >= T_max sends every expert to the streaming kernels.  Results are the same
 * function either way (accumulation order differs).
 */
dwdp_status dwdp_set_stream_max_rows(dwdp_ctx* ctx, int32_t max_rows);

/*
 * How the work items (M tile of up to 288 rows x weight panel) of the LDS-tiled kernels are handed
 * to workgroups.  Same results in every mode, bit for bit.
 *   DWDP_TILE_PER_ITEM (default): one workgroup per item, one launch per GEMM; finished
 *     workgroups return their compute unit, so the weight-streaming chain that runs beside the
 *     tiled one gets units as soon as fewer items are left than the chip has units.
 *   DWDP_TILE_PERSISTENT: per GEMM one launch of at most one workgroup per compute unit; the
 *     workgroups take items by atomic tickets (one queue per XCD, idle dies take others' tickets).
 *   DWDP_TILE_PERSISTENT_FUSED: ONE such launch computes both grouped GEMMs of the tiled experts; a
 *     down-projection item waits on a device-side counter for the gate/up items of its rows
 *     (bounded wait; DWDP_WS_SCHED word 16 reports a wait that gave up).
 */
enum { DWDP_TILE_PER_ITEM = 0, DWDP_TILE_PERSISTENT = 1, DWDP_TILE_PERSISTENT_FUSED = 2 };
dwdp_status dwdp_set_tile_schedule(dwdp_ctx* ctx, int32_t mode);
/*
 * Persistent schedules only: how many workgroups (= compute units; a multiple of 8, one round over
 * the XCDs) a persistent tiled launch uses when at least 16 experts are streamed beside the tiled
 * ones, so that the HBM-bound streaming chain has units of its own from the start.  0 = the
 * default (13/16 of the chip).  With fewer streamed experts the launch uses every unit.
 */
dwdp_status dwdp_set_tile_share(dwdp_ctx* ctx, int32_t n_workgroups);

/*
 * Weight preparation, done once when weights are loaded (on the owner of every expert,
 * so that resident and peer copies are byte-identical and prefetch stays a plain copy):
 * rearrange a row-major FP8 matrix src [rows, cols] into the tile-major layout the FP8
 * grouped GEMM streams.  Tiles are 16 rows x 128 columns = 2 KiB, ordered row-of-tiles
 * first; inside a tile byte half*1024 + (q*16 + r)*16 + b holds element (row r,
 * column q*32 + half*16 + b), r < 16, q < 4, half < 2, b < 16 -- the order in which the
 * 64 lanes of a wavefront feed a 16x16x128 matrix-core operand, so every load
 * instruction of a wave covers 1 KiB of contiguous memory.  rows % 16 == 0,
 * cols % 128 == 0 (DWDP_ESHAPE otherwise); src and dst must not overlap.  Enqueued on the
 * compute stream.
 */
dwdp_status dwdp_pack_fp8_weight(dwdp_ctx* ctx, const void* src, void* dst, int64_t rows, int64_t cols);

/*
 * The same preparation for MXFP4 weights: src_codes [rows, cols/2] (element 2i in the low
 * nibble of byte i) and src_scales uint8 [rows, cols/32], both row-major, are rearranged into
 *   dst_codes  [rows * cols / 2] bytes: 16-row x 128-column tiles of 1 KiB, row-of-tiles first;
 *              inside a tile byte (q*16 + r)*16 + b holds packed byte q*16 + b of row r's 64
 *              bytes of that K block -- lane q*16+r of a wavefront feeds elements
 *              32q..32q+31 of row r to a 16x16x128 matrix-core operand;
 *   dst_scales [rows/16 * ceil(cols/512) * 256] bytes: per row-of-tiles and group of four K
 *              blocks, lane q*16+r's dword holds the scales of (row r, K blocks 4g..4g+3,
 *              32-element sub-block q), padded with 127.
 * rows % 16 == 0, cols % 128 == 0 (DWDP_ESHAPE otherwise).  Enqueued on the compute stream.
 */
dwdp_status dwdp_pack_mxfp4_weight(dwdp_ctx* ctx, const void* src_codes, const void* src_scales, void* dst_codes,
                                   void* dst_scales, int64_t rows, int64_t cols);

/*
 * How dwdp_prefetch_layer moves the bytes of its copy plan.
 *   DWDP_COPY_MEMCPY (default): one hipMemcpyAsync (device to device) per plan entry, the
 *     counterpart of the copy-engine cudaMemcpyAsync pulls of paper Section 2.  Each entry
 *     costs a runtime call, so small slices are launch-bound.
 *   DWDP_COPY_KERNEL: the whole plan is executed by one kernel launch of at most
 *     n_workgroups workgroups that walk the plan in order (entries cut into pieces of at
 *     most 256 KiB).  The slice order of the plan is kept, the slice size costs nothing,
 *     and n_workgroups bounds how many compute units the copy takes from the GEMMs.
 *     With n_workgroups at or above the number of pieces every piece gets a workgroup of
 *     its own, of 1024 threads (the shape with the best HBM rate); a smaller n_workgroups
 *     gives that many 256-thread workgroups that walk the pieces round-robin.
 *     The device copy of a layer's plan is built on the first call with given arguments
 *     (one pinned-host and one device allocation, an asynchronous upload on the copy stream;
 *     no wait on any stream) and reused while the arguments stay the same.
 *     dwdp_prepare_prefetch builds it ahead of time, so that no allocation falls inside the
 *     pipeline.
 */
enum { DWDP_COPY_MEMCPY = 0, DWDP_COPY_KERNEL = 1 };
dwdp_status dwdp_set_copy_engine(dwdp_ctx* ctx, int32_t mode, int32_t n_workgroups);

/*
 * Set-up half of dwdp_prefetch_layer for the copy-kernel engine: builds (or rebuilds, when the
 * arguments differ from the cached ones) the device copy of `layer`'s plan and copies nothing.
 * Same arguments and errors as dwdp_prefetch_layer, without its protocol check.  Calling it
 * once per layer after the buffers exist keeps every later dwdp_prefetch_layer with the same
 * arguments free of allocations.  Valid in either engine mode.
 */
dwdp_status dwdp_prepare_prefetch(dwdp_ctx* ctx, int32_t layer, const void* const* src, void* const* dst,
                                  const size_t* bytes, int32_t n_peers, int32_t n_params, size_t slice_bytes);

/*
 * Host-only: the copy plan dwdp_prefetch_layer would issue, written to HOST arrays of
 * capacity `cap` entries (may be NULL with cap = 0 to query the length).  *n_out receives
 * the plan length.  Same argument meaning as dwdp_prefetch_layer.  Touches no GPU.
 */
dwdp_status dwdp_build_copy_plan(const void* const* src, void* const* dst, const size_t* bytes,
                                 int32_t n_peers, int32_t n_params, size_t slice_bytes,
                                 void** plan_dst, const void** plan_src, size_t* plan_bytes,
                                 size_t cap, size_t* n_out);

/*
 * Naive split-weight baseline of paper Section 4.2: merge the experts named by `table`
 * (DEVICE, n_slots rows) into contiguous caller buffers with device-to-device copies on
 * the compute stream and write the table of the merged copy to merged_table (DEVICE).
 * w13_out/w2_out/s13_out/s2_out hold n_slots experts back to back.
 * table_host is the HOST copy of `table` (the library cannot read device memory on the host).
 * `layer` names the layer the table belongs to: when a dwdp_prefetch_layer of it is pending,
 * the copies wait for the staged experts; the staging buffer still belongs to the layer until
 * its dwdp_moe_forward (called with the merged table) has run.  Experts that already lie
 * back to back in the source are moved with one copy.  bf16 and FP8 weights (DWDP_ESHAPE for
 * MXFP4).
 */
dwdp_status dwdp_merge_experts(dwdp_ctx* ctx, int32_t layer, const dwdp_expert_ptrs* table_host, int32_t n_slots,
                               void* w13_out, float* s13_out, void* w2_out, float* s2_out,
                               dwdp_expert_ptrs* merged_table_host);

/*
 * Per-stage timing with HIP events on the streams the kernels are launched on.  While
 * enabled, every dwdp_moe_forward records an event before each stage.  dwdp_profile_read
 * synchronises, adds up the elapsed milliseconds per stage over the calls since the last
 * read into ms_sum[DWDP_N_STAGES] (HOST), stores the number of calls in *n_calls and
 * resets.  At most DWDP_PROFILE_MAX_CALLS calls are kept between reads.
 * With FP8 weights the grouped GEMMs run as two concurrent chains: GEMM1_TILE/GEMM2_TILE are
 * the LDS-tiled kernels on the compute stream (with DWDP_TILE_PERSISTENT_FUSED, GEMM1_TILE is the
 * one launch that computes both and GEMM2_TILE is zero), GEMM1/GEMM2 the weight-streaming kernels on an
 * internal stream forked from and joined back into it (on the compute stream when no expert
 * can be tiled); QUANT is the time between the permutation's end and the first GEMM (any wait
 * for prefetched experts).
 */
enum {
  DWDP_STAGE_ROUTE = 0,
  DWDP_STAGE_PERMUTE = 1,
  DWDP_STAGE_QUANT = 2,
  DWDP_STAGE_GEMM1 = 3,
  DWDP_STAGE_GEMM2 = 4,
  DWDP_STAGE_COMBINE = 5,
  DWDP_STAGE_GEMM1_TILE = 6,
  DWDP_STAGE_GEMM2_TILE = 7,
  DWDP_N_STAGES = 8
};
enum { DWDP_PROFILE_MAX_CALLS = 512 };
dwdp_status dwdp_profile_enable(dwdp_ctx* ctx, int32_t on);
dwdp_status dwdp_profile_read(dwdp_ctx* ctx, float* ms_sum, int32_t* n_calls);

/*
 * Timeline of the two streams, for measuring how much of the staging-copy time is hidden
 * behind compute (paper Section 2).  While enabled, every dwdp_prefetch_layer records a
 * DWDP_SPAN_COPY span on the copy stream (first copy issued .. last copy done, i.e. after
 * the wait for the buffer's previous reader) and every dwdp_moe_forward a DWDP_SPAN_GEMM
 * span on the compute stream (grouped GEMM-1 start .. GEMM-2 end: the part that reads
 * expert weights).  dwdp_timeline_enable(on) synchronises both streams, drops old spans
 * and, when on, sets time zero.  dwdp_timeline_read synchronises both streams and writes
 * up to cap spans, in issue order, to HOST arrays: kind, layer, start and end in
 * milliseconds since time zero; *n_out is the number recorded (at most
 * DWDP_TIMELINE_MAX are kept).
 */
enum { DWDP_SPAN_COPY = 0, DWDP_SPAN_GEMM = 1 };
enum { DWDP_TIMELINE_MAX = 4096 };
dwdp_status dwdp_timeline_enable(dwdp_ctx* ctx, int32_t on);
dwdp_status dwdp_timeline_read(dwdp_ctx* ctx, int32_t* kind, int32_t* layer, float* start_ms, float* end_ms,
                               int32_t cap, int32_t* n_out);

/*
 * Device pointers of the context's workspace for inspection by tests (valid until
 * dwdp_destroy; contents are those of the last dwdp_moe_forward once the stream is idle).
 */
enum {
  DWDP_WS_TOPK_IDS = 0, /* int32 [T,K]                      */
  DWDP_WS_TOPK_W = 1,   /* fp32  [T,K]                      */
  DWDP_WS_OFFSETS = 2,  /* int32 [E+1(+1)]                  */
  DWDP_WS_PERM = 3,     /* int32 [T*K]                      */
  DWDP_WS_INV_PERM = 4, /* int32 [T*K]                      */
  DWDP_WS_XQ = 5,       /* fp8 [T,H]          (FP8 only)    */
  DWDP_WS_XS = 6,       /* fp32 [T,H/128]     (FP8 only)    */
  DWDP_WS_HQ = 7,       /* fp8 (FP8) or fp32 (bf16) [rows,I] */
  DWDP_WS_HS = 8,       /* fp32 [rows,I/128]  (FP8 only)    */
  DWDP_WS_YP = 9,       /* bf16 (FP8) or fp32 (bf16) [rows,H] */
  DWDP_WS_SCHED = 10,   /* int32 [32 + tiles]: scheduler words of the persistent tiled GEMM; [16] != 0
                           after a call means a bounded device-side wait gave up (results invalid)  */
  DWDP_N_WS = 11
};
void* dwdp_workspace_ptr(dwdp_ctx* ctx, int32_t which);

/* The copy stream (hipStream_t) used by dwdp_prefetch_layer, for tracing and tests. */
void* dwdp_copy_stream(dwdp_ctx* ctx);

#ifdef __cplusplus
}
#endif
#endif /* DWDP_H */
