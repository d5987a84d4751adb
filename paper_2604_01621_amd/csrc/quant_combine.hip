// Activation quantisation (bf16 -> e4m3 with one fp32 scale per token per 128 elements)
// and the weighted combine of the expert outputs.  Both are pure HBM streams: 16-byte
// loads per lane, reductions inside 16-lane groups, no LDS.
#include "dwdp_kernels.h"

namespace dwdp {

__global__ __launch_bounds__(256) void quant_act_kernel(const uint16_t* __restrict__ x, long n_groups,
                                                        uint8_t* __restrict__ xq, float* __restrict__ xs) {
  quant_act_lane(x, n_groups, xq, xs, (long)blockIdx.x * blockDim.x + threadIdx.x);
}

void launch_quant_act(const void* x, int T, int H, uint8_t* xq, float* xs, hipStream_t stream) {
  long n_groups = (long)T * (H / kBlockScale);
  if (n_groups <= 0) return;
  long threads = n_groups * 16;
  dim3 grid((unsigned)((threads + 255) / 256));
  hipLaunchKernelGGL(quant_act_kernel, grid, dim3(256), 0, stream, (const uint16_t*)x, n_groups, xq, xs);
}

// One block per token; each thread owns 8 consecutive columns per step.  The K routed rows
// are added in slot order k = 0..K-1, then the shared expert's row: deterministic.
// YP32 = false: yp is bf16 (FP8-weight path); true: yp is fp32 (bf16-weight path).
constexpr int kCombineThreads = 128;  // H / 8 = 896 column chunks of the R1 shape are 7 whole steps of 128

template <bool YP32>
__global__ __launch_bounds__(kCombineThreads) void combine_kernel(const void* __restrict__ yp_,
                                                      const int32_t* __restrict__ inv_perm,
                                                      const float* __restrict__ topk_w, int T, int H, int K,
                                                      int has_shared, uint16_t* __restrict__ y) {
  __shared__ int32_t row_s[33];
  __shared__ float w_s[33];
  const int t = blockIdx.x;
  if ((int)threadIdx.x < K) {
    row_s[threadIdx.x] = inv_perm[(size_t)t * K + threadIdx.x];
    w_s[threadIdx.x] = topk_w[(size_t)t * K + threadIdx.x];
  }
  if ((int)threadIdx.x == K && has_shared) {
    row_s[K] = T * K + t;
    w_s[K] = 1.f;
  }
  __syncthreads();
  const int n = K + (has_shared ? 1 : 0);
  for (int c = threadIdx.x * 8; c < H; c += blockDim.x * 8) {
    float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    if (YP32) {
      for (int k = 0; k < n; k++) {
        const float wk = w_s[k];
        const float* p = (const float*)yp_ + (size_t)row_s[k] * H + c;
        const v4f a = *(const v4f*)p;
        const v4f b = *(const v4f*)(p + 4);
#pragma unroll
        for (int i = 0; i < 4; i++) {
          acc[i] = fmaf(wk, a[i], acc[i]);
          acc[4 + i] = fmaf(wk, b[i], acc[4 + i]);
        }
      }
    } else {
      // rows in groups of kG (one group for top-8 routing with a shared expert): all loads of a
      // group are issued before the first is used (the rows of a token lie far apart, one load
      // at a time leaves the lane waiting on each); the adds keep the order k = 0..n-1.  Slots
      // past n re-read the last row and are not added.
      constexpr int kG = 9;
      for (int k0 = 0; k0 < n; k0 += kG) {
        v4i raw[kG];
#pragma unroll
        for (int j = 0; j < kG; j++)
          // non-temporal: every yp row is read once (0.26 -> 0.21 ms at 8192 tokens)
          raw[j] = __builtin_nontemporal_load(
              (const v4i*)((const uint16_t*)yp_ + (size_t)row_s[min(k0 + j, n - 1)] * H + c));
#pragma unroll
        for (int j = 0; j < kG; j++) {
          if (k0 + j < n) {
            const float wk = w_s[k0 + j];
#pragma unroll
            for (int i = 0; i < 4; i++) {
              uint32_t u = (uint32_t)raw[j][i];
              acc[2 * i] = fmaf(wk, __uint_as_float(u << 16), acc[2 * i]);
              acc[2 * i + 1] = fmaf(wk, __uint_as_float(u & 0xFFFF0000u), acc[2 * i + 1]);
            }
          }
        }
      }
    }
    v4i o;
#pragma unroll
    for (int i = 0; i < 4; i++)
      o[i] = (int)((uint32_t)f32_to_bf16(acc[2 * i]) | ((uint32_t)f32_to_bf16(acc[2 * i + 1]) << 16));
    *(v4i*)(y + (size_t)t * H + c) = o;
  }
}

// Executes a copy plan in one launch: unit u (dst, src, bytes) is copied by workgroup
// u % gridDim.x, units in plan order, so the slice interleaving of the plan is kept while the
// number of workgroups bounds how much of the chip the copy occupies.
//
// Shape of a workgroup, measured on an 8 GiB copy between two allocations (HBM traffic read +
// written; a read-only kernel reaches 7.1 TB/s, a write-only one 6.1, hipMemcpyAsync 4.4-4.9):
//   one workgroup per 256 KiB unit:  256 threads x 8 loads in flight 5.50 TB/s, 512 x 8 5.71,
//                                    1024 x 4 5.84, 1024 x 8 6.05, 1024 x 16 5.94
//   512 workgroups walking the plan: 256 threads 5.27 TB/s, 1024 threads 5.83
// (plain instead of non-temporal loads or stores: 2-7 % less).  The larger the block a compute
// unit reads before it turns to writing, the better the rate, so a launch that may take the
// whole chip uses 1024 threads (128 KiB read, then written, per step); a launch bounded to fewer
// workgroups than units is meant to run beside the GEMMs and keeps the light 256-thread shape,
// which leaves the registers of a compute unit to them.
template <int kThreads>
__global__ __launch_bounds__(kThreads) void copy_plan_kernel(const CopyUnit* __restrict__ units, int n_units) {
  for (int u = blockIdx.x; u < n_units; u += gridDim.x) {
    const CopyUnit cu = units[u];
    const uint8_t* src = (const uint8_t*)cu.src;
    uint8_t* dst = (uint8_t*)cu.dst;
    size_t done = 0;
    if ((((uintptr_t)src | (uintptr_t)dst) & 15) == 0) {
      const size_t n16 = cu.bytes >> 4;
      const v4i* s16 = (const v4i*)src;
      v4i* d16 = (v4i*)dst;
      size_t i = threadIdx.x;
      constexpr int kUn = 8;  // 16-byte loads in flight per lane
      for (; i + (size_t)(kUn - 1) * kThreads < n16; i += (size_t)kUn * kThreads) {
        v4i v[kUn];
#pragma unroll
        for (int j = 0; j < kUn; j++) v[j] = __builtin_nontemporal_load(s16 + i + j * kThreads);
#pragma unroll
        for (int j = 0; j < kUn; j++) __builtin_nontemporal_store(v[j], d16 + i + j * kThreads);
      }
      for (; i < n16; i += kThreads) d16[i] = s16[i];
      done = n16 << 4;
    }
    for (size_t i = done + threadIdx.x; i < cu.bytes; i += kThreads) dst[i] = src[i];
  }
}

void launch_copy_plan(const CopyUnit* units, int n_units, int n_workgroups, hipStream_t stream) {
  if (n_units <= 0) return;
  if (n_workgroups >= n_units)
    hipLaunchKernelGGL(copy_plan_kernel<1024>, dim3(n_units), dim3(1024), 0, stream, units, n_units);
  else
    hipLaunchKernelGGL(copy_plan_kernel<256>, dim3(n_workgroups), dim3(256), 0, stream, units, n_units);
}

void launch_combine(const void* yp, bool yp_fp32, const int32_t* inv_perm, const float* topk_w, int T, int H, int K,
                    int has_shared, void* y, hipStream_t stream) {
  if (T <= 0) return;
  if (yp_fp32)
    hipLaunchKernelGGL(combine_kernel<true>, dim3(T), dim3(kCombineThreads), 0, stream, yp, inv_perm, topk_w, T, H, K,
                       has_shared, (uint16_t*)y);
  else
    hipLaunchKernelGGL(combine_kernel<false>, dim3(T), dim3(kCombineThreads), 0, stream, yp, inv_perm, topk_w, T, H, K,
                       has_shared, (uint16_t*)y);
}

}  // namespace dwdp
