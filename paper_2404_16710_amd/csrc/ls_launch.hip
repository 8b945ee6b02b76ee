// Launches of the persistent decode kernels (one translation unit per (dtype, head_dim) variant
// holds the kernels themselves) and the plain copy kernel used as a byte-counter reference.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdlib.h>

#include "ls_internal.h"

#define LS_PROF_EVENTS 512

extern "C" void ls_variant_kernels_bf16_hd128(const void** out);
extern "C" void ls_variant_kernels_bf16_hd64(const void** out);
extern "C" void ls_variant_kernels_f32_hd128(const void** out);
extern "C" void ls_variant_kernels_f32_hd64(const void** out);

// Plain copy, 16 bytes per thread per step: the known-size reference for hardware byte counters.
__global__ __launch_bounds__(256) void ls_copy_kernel(const uint4* __restrict__ src, uint4* __restrict__ dst, size_t n16) {
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += (size_t)gridDim.x * blockDim.x)
    dst[i] = src[i];
}

extern "C" int ls_launch_copy(const void* src, void* dst, size_t bytes, hipStream_t stream) {
  ls_copy_kernel<<<dim3(2048), dim3(256), 0, stream>>>(static_cast<const uint4*>(src), static_cast<uint4*>(dst), bytes / 16);
  return hipGetLastError() == hipSuccess ? 0 : 1;
}

// Read-only stream in the launch shape of the decode kernels: every workgroup walks its own contiguous
// share with 16-byte loads, 16 per lane in flight (the 64 KB per compute unit that the decode kernels
// keep in flight for weights), and folds what it read into one 16-byte value per thread so that the
// loads stay.  The rate of this kernel is what a stage's weight stream can reach at best.
__global__ __launch_bounds__(256) void ls_read_kernel(const uint4* __restrict__ src, size_t n16, uint4* __restrict__ sink) {
  constexpr int D = 16;
  const size_t share = n16 / gridDim.x;                 // a multiple of 256 * D (checked by the caller)
  const uint4* p = src + (size_t)blockIdx.x * share + threadIdx.x;
  uint4 v[D];
#pragma unroll
  for (int q = 0; q < D; ++q) v[q] = p[(size_t)q * 256];
  uint4 acc = make_uint4(0, 0, 0, 0);
  const size_t steps = share / (256 * D);
  for (size_t i = 1; i < steps; ++i) {
    const uint4* pn = p + i * (size_t)(256 * D);
#pragma unroll
    for (int q = 0; q < D; ++q) {
      acc.x ^= v[q].x; acc.y ^= v[q].y; acc.z ^= v[q].z; acc.w ^= v[q].w;
      v[q] = pn[(size_t)q * 256];
    }
  }
#pragma unroll
  for (int q = 0; q < D; ++q) { acc.x ^= v[q].x; acc.y ^= v[q].y; acc.z ^= v[q].z; acc.w ^= v[q].w; }
  sink[(size_t)blockIdx.x * 256 + threadIdx.x] = acc;
}

extern "C" int ls_launch_read(const void* src, size_t bytes, void* sink, int workgroups, hipStream_t stream) {
  ls_read_kernel<<<dim3(workgroups), dim3(256), 0, stream>>>(static_cast<const uint4*>(src), bytes / 16, static_cast<uint4*>(sink));
  return hipGetLastError() == hipSuccess ? 0 : 1;
}

// Workspace of ls_generate_static: callers that may not allocate device memory get the KV cache and all
// per-stage scratch from this fixed array instead of a buffer of their own.  Every GPU the library runs
// on holds its own copy at its own address; host code never uses the array's name as an address, only
// the pointer hipGetSymbolAddress returns for the current device, looked up once per device.
static __device__ __align__(256) unsigned char ls_static_scratch[LS_STATIC_SCRATCH_BYTES];

extern "C" int ls_static_scratch_ptr(void** ptr) {
  constexpr int kMaxDev = 64;
  static void* dev_ptr[kMaxDev];   // zero-initialised: not looked up yet
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDev) return 1;
  void* p = __atomic_load_n(&dev_ptr[dev], __ATOMIC_ACQUIRE);
  if (p == nullptr) {
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(ls_static_scratch)) != hipSuccess || p == nullptr) return 1;
    __atomic_store_n(&dev_ptr[dev], p, __ATOMIC_RELEASE);   // every thread finds the same address
  }
  *ptr = p;
  return 0;
}

enum { LS_K_PROMPT = 0, LS_K_DECODE, LS_K_GREEDY, LS_K_STEP, LS_K_AUX, LS_K_COUNT };

static const void* kernel_symbol(int which, int dtype_is_bf16, int hd) {
  const void* k[LS_K_COUNT];
  if (dtype_is_bf16) { if (hd == 128) ls_variant_kernels_bf16_hd128(k); else ls_variant_kernels_bf16_hd64(k); }
  else { if (hd == 128) ls_variant_kernels_f32_hd128(k); else ls_variant_kernels_f32_hd64(k); }
  return k[which];
}

// Which of the five names a launch runs under (they share one body): whole self-speculative jobs,
// whole full-model greedy jobs, single draft / verify launches, and the ablation and early-exit
// jobs are kept apart so that per-name statistics of a kernel trace are of one kind of work each.
static int kernel_index(const LsKParams* p) {
  switch (p->kind) {
    case LS_PROG_PREFILL: case LS_PROG_SCORE: case LS_PROG_PF_FINISH: return LS_K_PROMPT;
    case LS_PROG_DRAFT: case LS_PROG_VERIFY: return LS_K_STEP;
    default: break;
  }
  if (p->d == 0) return p->layers_used == p->L ? LS_K_GREEDY : LS_K_AUX;
  return (p->no_reuse || p->E_low > 0) ? LS_K_AUX : LS_K_DECODE;
}

extern "C" int ls_launch_program(const LsKParams* p, int dtype_is_bf16, int grid, hipStream_t stream) {
  void* args[1] = {const_cast<LsKParams*>(p)};
  // The grid is sized to be co-resident (occupancy x compute units) and the barrier wait is bounded,
  // so an ordinary launch is used; LS_COOPERATIVE_LAUNCH=1 asks the runtime to guarantee residency.
  static const bool coop = []() { const char* v = getenv("LS_COOPERATIVE_LAUNCH"); return v != nullptr && v[0] == '1'; }();
  const size_t smem = LS_SMEM_BYTES + (p->prof != nullptr ? LS_PROF_EVENTS * 8 : 0);
  const void* fn = kernel_symbol(kernel_index(p), dtype_is_bf16, p->hd);
  hipError_t e = coop ? hipLaunchCooperativeKernel(fn, dim3(grid), dim3(LS_THREADS), args, smem, stream)
                      : hipLaunchKernel(fn, dim3(grid), dim3(LS_THREADS), args, smem, stream);
  return e == hipSuccess ? 0 : (int)e;
}

extern "C" int ls_kernel_setup(int dtype_is_bf16, int hd, int* max_blocks_per_cu) {
  int nb_min = 1 << 30;
  for (int v = 0; v < LS_K_COUNT; ++v) {
    const void* fn = kernel_symbol(v, dtype_is_bf16, hd);
    hipError_t e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, LS_SMEM_BYTES + LS_PROF_EVENTS * 8);
    if (e != hipSuccess) return (int)e;
    int nb = 0;
    e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&nb, fn, LS_THREADS, LS_SMEM_BYTES + LS_PROF_EVENTS * 8);
    if (e != hipSuccess) return (int)e;
    if (nb < nb_min) nb_min = nb;
  }
  *max_blocks_per_cu = nb_min;
  return 0;
}
