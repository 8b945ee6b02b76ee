// Persistent decode kernel for gfx950: every pass of greedy self-speculative decoding
// (draft step, tail pass, verify pass, full-model step, prefill chunk) is one walk over
//   [RMSNorm + QKV + RoPE + KV append] -> [attention] -> [O proj + residual]
//   -> [RMSNorm + gate/up + SwiGLU] -> [down proj + residual]   per layer, then
//   [final RMSNorm + LM head + argmax]
// executed by one grid that stays resident, with grid-wide barriers between stages.  The control
// flow of the method (Sections 4.3.1-4.3.3 and Appendix A.4 of the paper: draft d tokens with the
// first E layers, verify 1+d rows with the remaining layers, keep the matching prefix, crop the
// cache) runs on the device: every workgroup keeps an identical copy of the decoding state in LDS,
// so no host round-trip is needed between rounds.
//
// All matrix products use one scheme for every row count m in [1,16]: weights are the MFMA A
// operand (16 output features x K), the m activation rows are the B operand padded to 16 columns.
// A column's result therefore does not depend on how many other rows share the pass.
//
// Memory discipline.  Weights, embeddings and the rotary table are immutable and read with plain
// loads.  Everything a kernel writes for other workgroups (residual rows, q, attention output,
// SwiGLU output, KV cache, partial results) is written and read with agent-scope relaxed atomic
// accesses of 4 or 8 bytes, which go to the coherent level of the memory system directly; the grid
// barrier then needs no cache write-back or invalidate, only "my stores have completed" before the
// arrival and a compiler barrier around it.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <limits.h>
#include <math.h>
#include <stdlib.h>

#include "ls_internal.h"

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint16_t bf16_t;

#define TID ((int)threadIdx.x)
#define WAVE (TID >> 6)
#define LANE (TID & 63)

__device__ __forceinline__ float bf2f(uint32_t b) { return __uint_as_float(b << 16); }
__device__ __forceinline__ uint32_t f2bf(float f) {  // round to nearest even
  uint32_t u = __float_as_uint(f);
  return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
}

// LDS-only barrier: waits for this wave's LDS traffic, not for its global loads, so weight
// fragments that are still in flight stay in flight across it.
__device__ __forceinline__ void lds_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }
// All of this wave's global stores and loads have completed.
__device__ __forceinline__ void drain_vmem() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

// Device memory is addressed as global (address space 1), never through flat instructions: a flat
// access also counts as an LDS access, so the LDS-only barrier would wait for weight loads.
#define LS_GLOBAL __attribute__((address_space(1)))
typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint4 ldg128(const void* p) {
  const u32x4_t v = *(const LS_GLOBAL u32x4_t*)(p);
  return make_uint4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ float ldgf(const float* p) { return *(const LS_GLOBAL float*)(p); }
__device__ __forceinline__ uint32_t ldg16(const void* p) { return *(const LS_GLOBAL uint16_t*)(p); }
__device__ __forceinline__ void stg128(void* p, const float4& v) {
  *(LS_GLOBAL f32x4*)(p) = f32x4{v.x, v.y, v.z, v.w};
}

// Coherent (agent-scope) accesses for data exchanged between workgroups.
__device__ __forceinline__ uint64_t ldc64(const void* p) {
  return __hip_atomic_load((const LS_GLOBAL uint64_t*)(p), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ uint32_t ldc32(const void* p) {
  return __hip_atomic_load((const LS_GLOBAL uint32_t*)(p), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void stc64(void* p, uint64_t v) {
  __hip_atomic_store((LS_GLOBAL uint64_t*)(p), v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void stc32(void* p, uint32_t v) {
  __hip_atomic_store((LS_GLOBAL uint32_t*)(p), v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float ldcf(const float* p) { return __uint_as_float(ldc32(p)); }
__device__ __forceinline__ void stcf(float* p, float v) { stc32(p, __float_as_uint(v)); }
__device__ __forceinline__ float2 ldcf2(const float* p) {
  const uint64_t v = ldc64(p);
  return make_float2(__uint_as_float((uint32_t)v), __uint_as_float((uint32_t)(v >> 32)));
}
__device__ __forceinline__ void stcf2(float* p, float a, float b) {
  stc64(p, (uint64_t)__float_as_uint(a) | ((uint64_t)__float_as_uint(b) << 32));
}
__device__ __forceinline__ uint4 ldc128(const void* p) {
  const uint64_t a = ldc64(p), b = ldc64(static_cast<const char*>(p) + 8);
  return make_uint4((uint32_t)a, (uint32_t)(a >> 32), (uint32_t)b, (uint32_t)(b >> 32));
}

template <typename T> struct TT;
template <> struct TT<float> {
  static constexpr int EPV = 4;  // elements per 16-byte unit
  static __device__ __forceinline__ void unpack(const uint4& v, float* f) {
    f[0] = __uint_as_float(v.x); f[1] = __uint_as_float(v.y); f[2] = __uint_as_float(v.z); f[3] = __uint_as_float(v.w);
  }
  static __device__ __forceinline__ uint4 pack(const float* f) {
    return make_uint4(__float_as_uint(f[0]), __float_as_uint(f[1]), __float_as_uint(f[2]), __float_as_uint(f[3]));
  }
  static __device__ __forceinline__ float ld(const float* p) { return ldgf(p); }
  // 4 consecutive elements, coherent
  static __device__ __forceinline__ void ldc4(const float* p, float* f) {
    const float2 a = ldcf2(p), b = ldcf2(p + 2);
    f[0] = a.x; f[1] = a.y; f[2] = b.x; f[3] = b.y;
  }
  static __device__ __forceinline__ void stc4(float* p, const float* f) { stcf2(p, f[0], f[1]); stcf2(p + 2, f[2], f[3]); }
  static __device__ __forceinline__ void stc2(float* p, float a, float b) { stcf2(p, a, b); }
  static __device__ __forceinline__ void mma(f32x4& acc, const uint4& a, const uint4& b) {
    acc = __builtin_amdgcn_mfma_f32_16x16x4f32(__uint_as_float(a.x), __uint_as_float(b.x), acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_16x16x4f32(__uint_as_float(a.y), __uint_as_float(b.y), acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_16x16x4f32(__uint_as_float(a.z), __uint_as_float(b.z), acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_16x16x4f32(__uint_as_float(a.w), __uint_as_float(b.w), acc, 0, 0, 0);
  }
};
template <> struct TT<bf16_t> {
  static constexpr int EPV = 8;
  static __device__ __forceinline__ void unpack(const uint4& v, float* f) {
    f[0] = bf2f(v.x & 0xFFFFu); f[1] = bf2f(v.x >> 16); f[2] = bf2f(v.y & 0xFFFFu); f[3] = bf2f(v.y >> 16);
    f[4] = bf2f(v.z & 0xFFFFu); f[5] = bf2f(v.z >> 16); f[6] = bf2f(v.w & 0xFFFFu); f[7] = bf2f(v.w >> 16);
  }
  static __device__ __forceinline__ uint4 pack(const float* f) {
    return make_uint4(f2bf(f[0]) | (f2bf(f[1]) << 16), f2bf(f[2]) | (f2bf(f[3]) << 16),
                      f2bf(f[4]) | (f2bf(f[5]) << 16), f2bf(f[6]) | (f2bf(f[7]) << 16));
  }
  static __device__ __forceinline__ float ld(const bf16_t* p) { return bf2f(ldg16(p)); }
  static __device__ __forceinline__ void ldc4(const bf16_t* p, float* f) {
    const uint64_t t = ldc64(p);
    const uint32_t lo = (uint32_t)t, hi = (uint32_t)(t >> 32);
    f[0] = bf2f(lo & 0xFFFFu); f[1] = bf2f(lo >> 16); f[2] = bf2f(hi & 0xFFFFu); f[3] = bf2f(hi >> 16);
  }
  static __device__ __forceinline__ void stc4(bf16_t* p, const float* f) {
    stc64(p, (uint64_t)(f2bf(f[0]) | (f2bf(f[1]) << 16)) | ((uint64_t)(f2bf(f[2]) | (f2bf(f[3]) << 16)) << 32));
  }
  static __device__ __forceinline__ void stc2(bf16_t* p, float a, float b) { stc32(p, f2bf(a) | (f2bf(b) << 16)); }
  static __device__ __forceinline__ void mma(f32x4& acc, const uint4& a, const uint4& b) {
    acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), acc, 0, 0, 0);
  }
};

// ------------------------------------------------------------------------------------------
// LDS bookkeeping
struct Best { float v1; int i1; float v2; };
#define LS_LDS_LAYERS 64   // layer pointer tables of the first 64 layers are mirrored in LDS

struct Misc {
  LsKParams P;                 // kernel parameters (LDS copy: uniform reads without scratch or global trips)
  LsLayerW lw[LS_LDS_LAYERS];
  LsState st;
  int tok[LS_ROWS];
  float rinv[LS_ROWS];
  int r_tok[LS_ROWS];
  float r_margin[LS_ROWS];
  Best wb[LS_WAVES][LS_ROWS];
  unsigned epoch;
  int flag;
  int abort;
  int prof_n;
};
static_assert(sizeof(Misc) <= LS_MISC_BYTES, "Misc must fit its LDS slot");

extern __shared__ __align__(16) char ls_smem[];
__device__ __forceinline__ Misc* MS() { return reinterpret_cast<Misc*>(ls_smem + LS_ACT_BYTES + LS_RED_BYTES); }
// Every stage function starts with this: LDS views that the compiler can see are LDS.
#define LS_CTX                      \
  Misc* const ms = MS();            \
  char* const act = ls_smem;        \
  const LsKParams& P = ms->P;       \
  (void)act

__device__ __forceinline__ LsLayerW layer_w(const LsKParams& P, const Misc* ms, int l) {
  if (l < LS_LDS_LAYERS) return ms->lw[l];
  LsLayerW w;
  const LS_GLOBAL uint64_t* src = (const LS_GLOBAL uint64_t*)(P.layers + l);
  uint64_t* dst = reinterpret_cast<uint64_t*>(&w);
#pragma unroll
  for (int i = 0; i < (int)(sizeof(LsLayerW) / 8); ++i) dst[i] = src[i];
  return w;
}

// Timeline event of the profiled workgroup (debug aid).  Events go to a spare LDS region that
// only profiled launches allocate, and are copied out when the kernel ends, so that recording
// one costs a clock read and an LDS write (a global store here would be waited for by the next
// "all loads done" and distort what it measures).
#define LS_PROF_EVENTS 512
#define LS_PROF(tag)                                                                              \
  do {                                                                                            \
    if (P.prof != nullptr && (int)blockIdx.x == P.prof_wg && TID == 0 && ms->prof_n < LS_PROF_EVENTS) \
      reinterpret_cast<unsigned long long*>(ls_smem + LS_SMEM_BYTES)[ms->prof_n++] =              \
          (wall_clock64() << 8) | (unsigned long long)(tag);                                      \
  } while (0)

struct PassCtx {
  int m, row0, pos0, l0, l1;
  bool embed_src;  // rows come from the embedding table (tokens in Misc::tok) instead of xbuf
  bool head;
  void* qrows;     // q rows of the pass [m][qd] (written by the QKV stage, read by attention)
  void* orows;     // attention output rows [m][qd]
};

__device__ __forceinline__ Best best_merge(const Best& a, const Best& b) {
  const bool aw = (a.v1 > b.v1) || (a.v1 == b.v1 && a.i1 < b.i1);
  Best r;
  r.v1 = aw ? a.v1 : b.v1;
  r.i1 = aw ? a.i1 : b.i1;
  r.v2 = fmaxf(aw ? a.v2 : b.v2, aw ? b.v1 : a.v1);
  return r;
}
__device__ __forceinline__ Best best_shfl_xor(const Best& a, int mask) {
  Best b;
  b.v1 = __shfl_xor(a.v1, mask);
  b.i1 = __shfl_xor(a.i1, mask);
  b.v2 = __shfl_xor(a.v2, mask);
  return b;
}

// ------------------------------------------------------------------------------------------
// Grid barrier, two levels: workgroups are split into 8 groups by (id mod 8); the last arriver of
// a group bumps the grid counter, which everybody polls.  Counters are zero at launch and only
// grow: barrier number e completes when the grid counter reaches e * groups.  The caller must
// have drained its stores (drain_vmem) before; loads issued earlier may still be in flight.
// The wait is bounded: when it expires the error flag is raised and every workgroup leaves.
__device__ __forceinline__ void grid_arrive(const LsKParams& P, Misc* ms) {
  lds_barrier();   // every wave of this workgroup has drained its stores
  if (TID == 0) {
    const unsigned epoch = ++ms->epoch;
    const unsigned nwg = gridDim.x, wg = blockIdx.x;
    const unsigned ngrp = nwg < 8u ? nwg : 8u;
    const unsigned grp = wg % ngrp;
    const unsigned gsize = (nwg - grp + ngrp - 1) / ngrp;
    LS_GLOBAL uint32_t* gcnt = (LS_GLOBAL uint32_t*)(P.bar + 64 * (1 + grp));
    LS_GLOBAL uint32_t* gbar = (LS_GLOBAL uint32_t*)(P.bar);
    const unsigned old = __hip_atomic_fetch_add(gcnt, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (old == epoch * gsize - 1) __hip_atomic_fetch_add(gbar, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
}
__device__ __forceinline__ bool grid_wait(const LsKParams& P, Misc* ms) {
  if (TID == 0) {
    const unsigned nwg = gridDim.x;
    const unsigned ngrp = nwg < 8u ? nwg : 8u;
    LS_GLOBAL uint32_t* gbar = (LS_GLOBAL uint32_t*)(P.bar);
    LS_GLOBAL int32_t* gerr = (LS_GLOBAL int32_t*)(&P.state->error);
    const unsigned target = ms->epoch * ngrp;
    int it = 0;
    while (__hip_atomic_load(gbar, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < target) {
      __builtin_amdgcn_s_sleep(1);
      if (++it > P.spin_limit ||
          ((it & 1023) == 0 && __hip_atomic_load(gerr, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0)) {
        __hip_atomic_store(gerr, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        ms->abort = 1;
        break;
      }
    }
  }
  lds_barrier();
  return ms->abort == 0;
}
// Arrival is signalled first; what the caller does between grid_arrive and grid_wait (issuing the
// next stage's weight loads) overlaps with the other workgroups' arrival.
__device__ __forceinline__ bool grid_barrier(const LsKParams& P, Misc* ms) {
  grid_arrive(P, ms);
  return grid_wait(P, ms);
}

// ------------------------------------------------------------------------------------------
// Matmul input rows (the MFMA B operand)
enum { ACT_PLAIN = 0, ACT_NORM_X = 1, ACT_NORM_EMB = 2 };
struct ActDesc {
  int mode;
  const void* src;   // PLAIN: T[n][ld];  NORM_X: float[n][ld];  NORM_EMB: T embed[vocab][ld]
  int ld;
  const void* gain;  // T[K] RMSNorm gain (NORM modes)
  const float* ssq;  // NORM_X: per-16-column sums of squares of the rows, [n][ssq_nt]; the first chunk
  int ssq_nt;        //         turns them into Misc::rinv while the rows themselves are in flight
};

// Writes rows [0,m) x columns [k0, k0+klen) of the input into LDS as T, 16-byte units swizzled
// by the row index so that the 16 rows of one unit column hit distinct banks.  Columns at or past
// K are written as zeros (their loads read column 0 instead, so that no load sits under a branch).
template <typename T, int MODE>
__device__ __forceinline__ void stage_act(const ActDesc& A, const Misc* ms, int m, int K, int k0, int klen,
                                          int rs_units, char* act, int first = 0) {
  constexpr int EPV = TT<T>::EPV;
  const int upr = klen / EPV;
  for (int idx = first + TID; idx < m * upr; idx += LS_THREADS) {
    const int n = idx / upr, u = idx - n * upr;
    const int k = k0 + u * EPV;
    const bool ok = k < K;
    const int kc = ok ? k : 0;
    uint4 v;
    if (MODE == ACT_PLAIN) {
      v = ldc128(static_cast<const T*>(A.src) + (size_t)n * A.ld + kc);
    } else {
      float f[EPV], gn[EPV];
      if (MODE == ACT_NORM_X) {
        const float* s = static_cast<const float*>(A.src) + (size_t)n * A.ld + kc;
#pragma unroll
        for (int e = 0; e < EPV; e += 2) {
          const float2 t = ldcf2(s + e);
          f[e] = t.x; f[e + 1] = t.y;
        }
      } else {
        TT<T>::unpack(ldg128(static_cast<const T*>(A.src) + (size_t)ms->tok[n] * A.ld + kc), f);
      }
      TT<T>::unpack(ldg128(static_cast<const T*>(A.gain) + kc), gn);
      const float r = ms->rinv[n];
#pragma unroll
      for (int e = 0; e < EPV; ++e) f[e] = (f[e] * r) * gn[e];
      v = TT<T>::pack(f);
    }
    const uint32_t keep = ok ? 0xFFFFFFFFu : 0u;
    v = make_uint4(v.x & keep, v.y & keep, v.z & keep, v.w & keep);
    const int pu = (u & ~15) | ((u ^ n) & 15);
    *reinterpret_cast<uint4*>(act + ((size_t)n * rs_units + pu) * 16) = v;
  }
}

// First chunk of an RMS-normalised input taken from the fp32 residual rows: the per-tile sums of
// squares and the raw rows are requested together (one memory round trip instead of two), then
// 1/rms goes to Misc::rinv and the scaled rows to LDS.
template <typename T>
__device__ __forceinline__ void stage_act_norm_first(const ActDesc& A, const LsKParams& P, Misc* ms, int m, int K,
                                                     int klen, int rs_units, char* act) {
  constexpr int EPV = TT<T>::EPV;
  constexpr int UMAX = 2;
  const int lane = LANE, wave = WAVE;
  const int upr = klen / EPV, total = m * upr;
  // raw rows first: UMAX units per thread
  float f[UMAX][EPV];
  int un[UMAX], uu[UMAX];
#pragma unroll
  for (int q = 0; q < UMAX; ++q) {
    const int idx = TID + q * LS_THREADS;
    un[q] = idx / upr;
    uu[q] = idx - un[q] * upr;
    const bool ok = idx < total && uu[q] * EPV < K;
    const float* src = static_cast<const float*>(A.src) + (ok ? (size_t)un[q] * A.ld + uu[q] * EPV : 0);
#pragma unroll
    for (int e = 0; e < EPV; e += 2) {
      const float2 t = ldcf2(src + e);
      f[q][e] = t.x; f[q][e + 1] = t.y;
    }
  }
  // statistics: wave w owns rows w, w+4, ...; lanes run over the 16-column tiles
  for (int n = wave; n < m; n += LS_WAVES) {
    float sacc = 0.f;
    for (int k0 = 0; k0 < A.ssq_nt; k0 += 256) {
      float v[4];
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int k = k0 + lane + 64 * j;
        const bool ok = k < A.ssq_nt;
        const float t = ldcf(A.ssq + (size_t)n * A.ssq_nt + (ok ? k : 0));
        v[j] = ok ? t : 0.f;
      }
      sacc += (v[0] + v[1]) + (v[2] + v[3]);
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) sacc += __shfl_xor(sacc, o);
    if (lane == 0) ms->rinv[n] = 1.0f / sqrtf(sacc / (float)P.dm + P.eps);
  }
  lds_barrier();
#pragma unroll
  for (int q = 0; q < UMAX; ++q) {
    const int idx = TID + q * LS_THREADS;
    if (idx < total) {
      const int n = un[q], u = uu[q], k = u * EPV;
      const bool ok = k < K;
      float gn[EPV];
      TT<T>::unpack(ldg128(static_cast<const T*>(A.gain) + (ok ? k : 0)), gn);
      const float r = ms->rinv[n];
#pragma unroll
      for (int e = 0; e < EPV; ++e) f[q][e] = (f[q][e] * r) * gn[e];
      uint4 v = TT<T>::pack(f[q]);
      const uint32_t keep = ok ? 0xFFFFFFFFu : 0u;
      v = make_uint4(v.x & keep, v.y & keep, v.z & keep, v.w & keep);
      const int pu = (u & ~15) | ((u ^ n) & 15);
      *reinterpret_cast<uint4*>(act + ((size_t)n * rs_units + pu) * 16) = v;
    }
  }
  if (total > UMAX * LS_THREADS) stage_act<T, ACT_NORM_X>(A, ms, m, K, 0, klen, rs_units, act, UMAX * LS_THREADS);
}

// NT weight tiles (16 rows x K each, row-major with leading dimension K) times the staged input.
// The waves of the workgroup take the 256-byte blocks of K round-robin; DEPTH blocks per wave are
// kept in flight.
// begin() issues the first loads (it may be called before a grid barrier: weights do not depend
// on other workgroups); run() stages the input, multiplies, and leaves the per-wave partial sums
// in LDS (`act` region) as red[wave][tile][lane]; tile_sum() adds them in wave order.
// K is walked in whole rounds of waves*DEPTH blocks: blocks past the end multiply clamped (finite)
// weight loads with zero-filled input, so the loop has no conditional loads.
template <typename T, int NT, int DEPTH>
struct Gemm {
  static constexpr int KB = 256 / (int)sizeof(T);
  static constexpr int EPV = TT<T>::EPV;
  static constexpr int ROUND = LS_WAVES * DEPTH;
  // a chunk of 16 rows must hold at least one round
  static_assert(LS_ACT_BYTES / (LS_ROWS * 256) >= ROUND, "LDS chunk too small for this prefetch depth");
  static_assert(LS_WAVES * NT * 64 * 16 <= LS_RED_BYTES, "reduction scratch too small");
  uint4 slot[DEPTH][NT][4];
  const T* rp[NT];       // row pointers of the current group of tiles
  const T* rp_next[NT];  // ... of the group this workgroup multiplies next (or the same again)
  int K, nkb, nkb_pad;

  // Blocks are numbered along K of the current group and continue into the next group: the loads
  // that run past the end of this group already fetch the first blocks of the next one.
  __device__ __forceinline__ void load_slot(int s, int kb) {
    const int e0 = (LANE >> 4) * EPV;
    const bool nxt = kb >= nkb_pad;
    const int kbb = nxt ? kb - nkb_pad : kb;
#pragma unroll
    for (int t = 0; t < NT; ++t) {
      const T* base = nxt ? rp_next[t] : rp[t];
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int idx = e0 + kbb * KB + j * (KB / 4);
        const int idc = (idx + EPV <= K) ? idx : 0;
        slot[s][t][j] = ldg128(base + idc);
      }
    }
  }

  __device__ __forceinline__ void begin(const T* const (&wt)[NT], int K_) {
    const int r = LANE & 15;
    K = K_;
    nkb = (K + KB - 1) / KB;
    nkb_pad = (nkb + ROUND - 1) / ROUND * ROUND;
#pragma unroll
    for (int t = 0; t < NT; ++t) rp_next[t] = rp[t] = (wt[t] ? wt[t] : wt[0]) + (size_t)r * K;
#pragma unroll
    for (int s = 0; s < DEPTH; ++s) load_slot(s, WAVE + LS_WAVES * s);
  }
  __device__ __forceinline__ void set_next(const T* const (&wt)[NT]) {
    const int r = LANE & 15;
#pragma unroll
    for (int t = 0; t < NT; ++t) rp_next[t] = (wt[t] ? wt[t] : wt[0]) + (size_t)r * K;
  }
  __device__ __forceinline__ void advance() {
#pragma unroll
    for (int t = 0; t < NT; ++t) rp[t] = rp_next[t];
  }

  template <int MODE>
  // `staged` (in/out): the input of this stage is already in LDS from an earlier group; it stays
  // valid when all of K fits one chunk.
  __device__ __forceinline__ void run(const ActDesc& A, const LsKParams& P, Misc* ms, int m, char* act, bool& staged) {
    const int lane = LANE, wave = WAVE;
    const int r = lane & 15, g = lane >> 4;
    int kcb = (LS_ACT_BYTES / (m * 256)) / ROUND * ROUND;
    if (kcb > nkb_pad) kcb = nkb_pad;
    const int rs_units = kcb * 16;
    f32x4 acc[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t) acc[t] = f32x4{0.f, 0.f, 0.f, 0.f};
    const int rr = (r < m) ? r : 0;                  // columns past m read row 0 and are masked to zero
    const uint32_t bmask = (r < m) ? 0xFFFFFFFFu : 0u;
    const char* brow = act + (size_t)rr * rs_units * 16;

    lds_barrier();  // the previous user of the LDS region is done with it
    for (int c0 = 0; c0 < nkb_pad; c0 += kcb) {
      const int clen = (c0 + kcb <= nkb_pad) ? kcb : nkb_pad - c0;
      if (c0) lds_barrier();
      if (!staged) {
        if (MODE == ACT_NORM_X && c0 == 0 && A.ssq != nullptr)
          stage_act_norm_first<T>(A, P, ms, m, K, clen * KB, rs_units, act);
        else
          stage_act<T, MODE>(A, ms, m, K, c0 * KB, clen * KB, rs_units, act);
        lds_barrier();
      }
      for (int kb0 = wave; kb0 < clen; kb0 += ROUND) {
#pragma unroll
        for (int s = 0; s < DEPTH; ++s) {
          const int kbl = kb0 + LS_WAVES * s;   // block within the chunk
          uint4 b[4];
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            const int u = kbl * 16 + j * 4 + g;
            const int pu = (u & ~15) | ((u ^ rr) & 15);
            const uint4 bv = *reinterpret_cast<const uint4*>(brow + (size_t)pu * 16);
            b[j] = make_uint4(bmask & bv.x, bmask & bv.y, bmask & bv.z, bmask & bv.w);
          }
#pragma unroll
          for (int t = 0; t < NT; ++t) {
#pragma unroll
            for (int j = 0; j < 4; ++j) TT<T>::mma(acc[t], slot[s][t][j], b[j]);
          }
          load_slot(s, c0 + kbl + ROUND);
        }
      }
    }
    staged = (kcb == nkb_pad);
    f32x4* red = reinterpret_cast<f32x4*>(ls_smem + LS_ACT_BYTES);
#pragma unroll
    for (int t = 0; t < NT; ++t) red[(wave * NT + t) * 64 + lane] = acc[t];
    lds_barrier();
  }
};

template <int NT>
__device__ __forceinline__ f32x4 tile_sum(const char* act, int t) {
  (void)act;
  const f32x4* red = reinterpret_cast<const f32x4*>(ls_smem + LS_ACT_BYTES);
  f32x4 s = red[(0 * NT + t) * 64 + LANE];
#pragma unroll
  for (int w = 1; w < LS_WAVES; ++w) {
    const f32x4 v = red[(w * NT + t) * 64 + LANE];
    s[0] += v[0]; s[1] += v[1]; s[2] += v[2]; s[3] += v[3];
  }
  return s;
}

// 1/sqrt(mean(x^2) + eps) for the pass rows, into Misc::rinv.
template <typename T>
__device__ __forceinline__ void compute_rinv(const LsKParams& P, const PassCtx& pc, bool from_embed, Misc* ms) {
  const int lane = LANE, wave = WAVE;
  for (int n = wave; n < pc.m; n += LS_WAVES) {
    float s = 0.f;
    if (from_embed) {
      const T* e = static_cast<const T*>(P.embed) + (size_t)ms->tok[n] * P.dm;
      for (int k = lane; k < P.dm; k += 64) { const float v = TT<T>::ld(e + k); s += v * v; }
    } else {
      const int nt = P.dm / 16;
      const float* q = P.ssq + (size_t)(pc.row0 + n) * nt;
      for (int k = lane; k < nt; k += 64) s += ldcf(q + k);
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) s += __shfl_xor(s, o);
    if (lane == 0) ms->rinv[n] = 1.0f / sqrtf(s / (float)P.dm + P.eps);
  }
  lds_barrier();
}

// ------------------------------------------------------------------------------------------
// Stage A: RMSNorm + QKV projection + RoPE + KV append.  A work item is a pair of 16-row tiles:
// for q and k the rows (j, j + hd/2) that one rotation mixes, for v two adjacent tiles.
template <typename T, int NT>
__device__ __forceinline__ bool stage_qkv(const PassCtx pc, int l) {
  LS_CTX;
  constexpr int DEPTH = 4 / NT;
  constexpr int IPG = NT / 2;
  const LsLayerW W = layer_w(P, ms, l);
  const int hd = P.hd, dm = P.dm, half = hd / 2;
  const int pph = hd / 32;
  const int nq_items = P.nq * pph, nk_items = P.nkv * pph, nv_items = P.kvd / 32;
  const int items = nq_items + nk_items + nv_items;
  const int groups = (items + IPG - 1) / IPG;
  const bool emb = pc.embed_src && l == pc.l0;
  ActDesc A;
  A.mode = emb ? ACT_NORM_EMB : ACT_NORM_X;
  A.src = emb ? P.embed : static_cast<const void*>(P.xbuf + (size_t)pc.row0 * dm);
  A.ld = dm;
  A.gain = W.attn_norm;
  A.ssq = emb ? nullptr : P.ssq + (size_t)pc.row0 * (dm / 16);
  A.ssq_nt = dm / 16;
  const int lane = LANE, wave = WAVE, n = lane & 15, g = lane >> 4;
  auto tiles_of = [&](int grp, const T* (&wt)[NT]) {
#pragma unroll
    for (int u = 0; u < IPG; ++u) {
      const int item = grp * IPG + u;
      const T *t0 = nullptr, *t1 = nullptr;
      if (item < nq_items) {
        const int h = item / pph, jb = item - h * pph;
        t0 = static_cast<const T*>(W.wq) + (size_t)(h * hd + jb * 16) * dm;
        t1 = t0 + (size_t)half * dm;
      } else if (item < nq_items + nk_items) {
        const int it = item - nq_items, h = it / pph, jb = it - h * pph;
        t0 = static_cast<const T*>(W.wk) + (size_t)(h * hd + jb * 16) * dm;
        t1 = t0 + (size_t)half * dm;
      } else if (item < items) {
        const int it = item - nq_items - nk_items;
        t0 = static_cast<const T*>(W.wv) + (size_t)(it * 32) * dm;
        t1 = t0 + (size_t)16 * dm;
      }
      wt[2 * u] = t0;
      wt[2 * u + 1] = t1;
    }
  };
  Gemm<T, NT, DEPTH> G;
  const T* wt[NT];
  int grp = blockIdx.x;
  LS_PROF(0x10);
  grid_arrive(P, ms);
  if (grp < groups) { tiles_of(grp, wt); G.begin(wt, dm); }
  LS_PROF(0x11);
  if (!grid_wait(P, ms)) return false;
  LS_PROF(0x12);
  if (emb) compute_rinv<T>(P, pc, true, ms);
  LS_PROF(0x13);
  bool staged = false;
  for (; grp < groups; grp += gridDim.x) {
    {
      const T* wtn[NT];
      const int nx = grp + (int)gridDim.x;
      tiles_of(nx < groups ? nx : grp, wtn);
      G.set_next(wtn);
    }
    if (emb) G.template run<ACT_NORM_EMB>(A, P, ms, pc.m, act, staged);
    else G.template run<ACT_NORM_X>(A, P, ms, pc.m, act, staged);
    LS_PROF(0x14);
    G.advance();
    if (wave < IPG) {
      const int item = grp * IPG + wave;
      if (item < items) {
        const f32x4 a = tile_sum<NT>(act, 2 * wave), b = tile_sum<NT>(act, 2 * wave + 1);
        if (n < pc.m) {
          const int pos = pc.pos0 + n;
          if (item < nq_items + nk_items) {
            const bool isq = item < nq_items;
            const int it = isq ? item : item - nq_items;
            const int h = it / pph, jb = it - h * pph;
            T* dst = isq ? static_cast<T*>(pc.qrows) + (size_t)n * P.qd + h * hd
                         : static_cast<T*>(P.kcache) + (((size_t)l * P.nkv + h) * P.max_seq + pos) * hd;
            float lo[4], hi[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
              const int dj = jb * 16 + 4 * g + j;
              const float c = ldgf(P.rope_cos + (size_t)pos * half + dj), s = ldgf(P.rope_sin + (size_t)pos * half + dj);
              lo[j] = a[j] * c - b[j] * s;
              hi[j] = b[j] * c + a[j] * s;
            }
            TT<T>::stc4(dst + jb * 16 + 4 * g, lo);
            TT<T>::stc4(dst + jb * 16 + 4 * g + half, hi);
          } else {
            const int it = item - nq_items - nk_items;
            const int row = it * 32;  // within kv_dim
            const int h = row / hd, d0 = row - h * hd;
            T* dst = static_cast<T*>(P.vcache) + (((size_t)l * P.nkv + h) * P.max_seq + pos) * hd + d0;
            const float va[4] = {a[0], a[1], a[2], a[3]}, vb[4] = {b[0], b[1], b[2], b[3]};
            TT<T>::stc4(dst + 4 * g, va);
            TT<T>::stc4(dst + 16 + 4 * g, vb);
          }
        }
      }
    }
  }
  LS_PROF(0x15);
  drain_vmem();
  LS_PROF(0x16);
  return true;
}

// ------------------------------------------------------------------------------------------
// Stage B: attention of the m query rows (x G query heads per KV head) over the shared cache.
// A work item is (kv head, super-tile of C consecutive 64-position tiles); C is fixed by the
// cache capacity, so the partition depends on absolute positions only.  Inside an item the tiles
// are walked in order with a running softmax (the next tile's K and V are requested while the
// current one is processed); the last workgroup to finish a kv head merges the per-item partial
// results in item order.
template <typename T, int HD>
__device__ __forceinline__ bool stage_attn(const PassCtx pc, int l) {
  LS_CTX;
  constexpr int TP = LS_ATTN_TILE;
  constexpr int NSEG = LS_THREADS / TP; // threads per key in the q.k product
  constexpr int SEG = HD / NSEG;        // dims per thread in the q.k product
  constexpr int DQ = HD / 4;            // threads across one V row (4 dims each)
  constexpr int PARTS = LS_THREADS / DQ;
  constexpr int KPP = TP / PARTS;       // keys per thread in the p.v product
  constexpr int PSTRIDE = HD + 2;
  const int tid = TID, lane = LANE, wave = WAVE;
  const int G = P.G, nQ = pc.m * G;
  const int tend = pc.pos0 + pc.m;  // positions in the cache after this pass
  const int ntiles = (tend + TP - 1) / TP;
  const int C = P.attn_ctiles;
  const int nsuper = (ntiles + C - 1) / C;
  const int items = P.nkv * nsuper;
  float* qs = reinterpret_cast<float*>(act);   // [64][HD]  queries
  float* orun = qs + 64 * HD;                   // [64][HD]  running output
  float* mrun = orun + 64 * HD;                 // [64] running max, [64] running sum
  float* lrun = mrun + 64;
  float* sc = lrun + 64;                        // [16][TP]
  float* smx = sc + 16 * TP;                    // [16]
  float* ssm = smx + 16;                        // [16]
  float* red = ssm + 16;                        // [waves][16][HD]
  const T* kc = static_cast<const T*>(P.kcache) + (size_t)l * P.nkv * P.max_seq * HD;
  const T* vc = static_cast<const T*>(P.vcache) + (size_t)l * P.nkv * P.max_seq * HD;
  const int u = tid / NSEG, seg = tid % NSEG;   // K: thread (key u, segment seg)
  const int dq = tid % DQ, part = tid / DQ;     // V: thread (dim quad dq, key part)

  LS_PROF(0x20);
  if (!grid_barrier(P, ms)) return false;
  LS_PROF(0x22);
  for (int item = blockIdx.x; item < items; item += gridDim.x) {
    const int c = item / nsuper, si = item - c * nsuper;
    const int t0 = si * C;
    const int t1 = (t0 + C < ntiles) ? t0 + C : ntiles;
    float kreg[SEG], vreg[KPP][4], knext[SEG], vnext[KPP][4];
    auto load_tile = [&](int ti, float (&kr)[SEG], float (&vr)[KPP][4]) {
      const int kp0 = ti * TP;
      const int nvalid = (tend - kp0 < TP) ? tend - kp0 : TP;
      {
        const bool ok = u < nvalid;   // keys past the end read key 0 of the tile and are zeroed
        const T* kp = kc + ((size_t)c * P.max_seq + kp0 + (ok ? u : 0)) * HD + seg * SEG;
#pragma unroll
        for (int e = 0; e < SEG; e += 4) TT<T>::ldc4(kp + e, &kr[e]);
#pragma unroll
        for (int e = 0; e < SEG; ++e) kr[e] = ok ? kr[e] : 0.f;
      }
#pragma unroll
      for (int kk = 0; kk < KPP; ++kk) {
        const int key = part * KPP + kk;
        const bool ok = key < nvalid;
        TT<T>::ldc4(vc + ((size_t)c * P.max_seq + kp0 + (ok ? key : 0)) * HD + dq * 4, vr[kk]);
#pragma unroll
        for (int e = 0; e < 4; ++e) vr[kk][e] = ok ? vr[kk][e] : 0.f;
      }
    };
    load_tile(t0, kreg, vreg);
    lds_barrier();   // previous item (or stage) is done with the LDS region
    for (int idx = tid; idx < nQ * (HD / 4); idx += LS_THREADS) {
      const int qg = idx / (HD / 4), d4 = (idx - qg * (HD / 4)) * 4;
      const int n = qg / G, gq = qg - n * G;
      float f[4];
      TT<T>::ldc4(static_cast<const T*>(pc.qrows) + (size_t)n * P.qd + (c * G + gq) * HD + d4, f);
      *reinterpret_cast<float4*>(qs + qg * HD + d4) = make_float4(f[0], f[1], f[2], f[3]);
      *reinterpret_cast<float4*>(orun + qg * HD + d4) = make_float4(0.f, 0.f, 0.f, 0.f);
    }
    if (tid < nQ) { mrun[tid] = -INFINITY; lrun[tid] = 0.f; }

    for (int ti = t0; ti < t1; ++ti) {
      const int kp0 = ti * TP;
      const int nvalid = (tend - kp0 < TP) ? tend - kp0 : TP;
      if (ti + 1 < t1) load_tile(ti + 1, knext, vnext);
      for (int qb = 0; qb < nQ; qb += 16) {
        const int nqb = (nQ - qb < 16) ? nQ - qb : 16;
        lds_barrier();
        for (int qi = 0; qi < nqb; ++qi) {
          const float* q = qs + (qb + qi) * HD + seg * SEG;
          float dot = 0.f;
#pragma unroll
          for (int e = 0; e < SEG; e += 4) {
            const float4 qv = *reinterpret_cast<const float4*>(q + e);
            dot += kreg[e] * qv.x; dot += kreg[e + 1] * qv.y; dot += kreg[e + 2] * qv.z; dot += kreg[e + 3] * qv.w;
          }
#pragma unroll
          for (int o = 1; o < NSEG; o <<= 1) dot += __shfl_xor(dot, o);
          if (seg == 0) {
            const int qpos = pc.pos0 + (qb + qi) / G;
            sc[qi * TP + u] = (u < nvalid && kp0 + u <= qpos) ? dot * P.attn_scale : -INFINITY;
          }
        }
        lds_barrier();
        for (int qi = wave; qi < nqb; qi += LS_WAVES) {
          const float s = sc[qi * TP + lane];
          float mx = s;
#pragma unroll
          for (int o = 32; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o));
          const float p = (s == -INFINITY) ? 0.f : expf(s - mx);
          float sum = p;
#pragma unroll
          for (int o = 32; o > 0; o >>= 1) sum += __shfl_xor(sum, o);
          sc[qi * TP + lane] = p;
          if (lane == 0) { smx[qi] = mx; ssm[qi] = sum; }
        }
        lds_barrier();
        for (int qi = 0; qi < nqb; ++qi) {
          float o0 = 0.f, o1 = 0.f, o2 = 0.f, o3 = 0.f;
#pragma unroll
          for (int kk = 0; kk < KPP; ++kk) {
            const float p = sc[qi * TP + part * KPP + kk];
            o0 += p * vreg[kk][0]; o1 += p * vreg[kk][1]; o2 += p * vreg[kk][2]; o3 += p * vreg[kk][3];
          }
#pragma unroll
          for (int o = DQ; o < 64; o <<= 1) {
            o0 += __shfl_xor(o0, o); o1 += __shfl_xor(o1, o); o2 += __shfl_xor(o2, o); o3 += __shfl_xor(o3, o);
          }
          if (lane < DQ) *reinterpret_cast<float4*>(red + (wave * 16 + qi) * HD + lane * 4) = make_float4(o0, o1, o2, o3);
        }
        lds_barrier();
        // fold this tile into the running softmax of each query (skipped when the tile is fully masked)
        for (int idx = tid; idx < nqb * (HD / 2); idx += LS_THREADS) {
          const int qi = idx / (HD / 2), dim = (idx - qi * (HD / 2)) * 2;
          const float mx = smx[qi], mo = mrun[qb + qi];
          if (mx != -INFINITY) {
            const float mn = fmaxf(mo, mx);
            const float a = (mo == -INFINITY) ? 0.f : expf(mo - mn), b = expf(mx - mn);
#pragma unroll
            for (int e = 0; e < 2; ++e) {
              float t = red[(0 * 16 + qi) * HD + dim + e];
#pragma unroll
              for (int w = 1; w < LS_WAVES; ++w) t += red[(w * 16 + qi) * HD + dim + e];
              orun[(qb + qi) * HD + dim + e] = orun[(qb + qi) * HD + dim + e] * a + t * b;
            }
          }
        }
        lds_barrier();
        if (tid < nqb) {
          const float mx = smx[tid], mo = mrun[qb + tid];
          if (mx != -INFINITY) {
            const float mn = fmaxf(mo, mx);
            const float a = (mo == -INFINITY) ? 0.f : expf(mo - mn), b = expf(mx - mn);
            lrun[qb + tid] = lrun[qb + tid] * a + ssm[tid] * b;
            mrun[qb + tid] = mn;
          }
        }
      }
      if (ti + 1 < t1) {
#pragma unroll
        for (int e = 0; e < SEG; ++e) kreg[e] = knext[e];
#pragma unroll
        for (int kk = 0; kk < KPP; ++kk)
#pragma unroll
          for (int e = 0; e < 4; ++e) vreg[kk][e] = vnext[kk][e];
      }
    }
    lds_barrier();
    float* pout = P.attn_part + ((size_t)(c * P.max_tiles + si) * 64) * PSTRIDE;
    for (int idx = tid; idx < nQ * (HD / 2); idx += LS_THREADS) {
      const int qg = idx / (HD / 2), dim = (idx - qg * (HD / 2)) * 2;
      float* dst = pout + (size_t)qg * PSTRIDE;
      stcf2(dst + dim, orun[qg * HD + dim], orun[qg * HD + dim + 1]);
      if (dim == 0) stcf2(dst + HD, mrun[qg], lrun[qg]);
    }
    // last arriver of this kv head merges the items (partials are coherent stores: once they have
    // completed, whoever sees the counter reach nsuper sees them)
    drain_vmem();
    lds_barrier();
    if (tid == 0) {
      const unsigned old = __hip_atomic_fetch_add((LS_GLOBAL uint32_t*)(P.attn_cnt + c), 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      ms->flag = (old == (unsigned)(nsuper - 1));
    }
    lds_barrier();
    if (ms->flag) {
      const float* pin = P.attn_part + ((size_t)(c * P.max_tiles) * 64) * PSTRIDE;
      float* wts = reinterpret_cast<float*>(act);   // [16][nsuper] softmax weights of the items
      float* dens = wts + 16 * nsuper;              // [16]
      for (int qb = 0; qb < nQ; qb += 16) {
        const int nqb = (nQ - qb < 16) ? nQ - qb : 16;
        lds_barrier();
        for (int qi = wave; qi < nqb; qi += LS_WAVES) {
          const int qg = qb + qi;
          float M = -INFINITY;
          for (int t = lane; t < nsuper; t += 64) M = fmaxf(M, ldcf(pin + ((size_t)t * 64 + qg) * PSTRIDE + HD));
#pragma unroll
          for (int o = 32; o > 0; o >>= 1) M = fmaxf(M, __shfl_xor(M, o));
          float den = 0.f;
          for (int tb = 0; tb < nsuper; tb += 64) {
            const int t = tb + lane;
            float w = 0.f, lsum = 0.f;
            if (t < nsuper) {
              const float2 stt = ldcf2(pin + ((size_t)t * 64 + qg) * PSTRIDE + HD);
              w = (stt.x == -INFINITY) ? 0.f : expf(stt.x - M);
              lsum = stt.y;
              wts[qi * nsuper + t] = w;
            }
            float part_sum = w * lsum;
#pragma unroll
            for (int o = 32; o > 0; o >>= 1) part_sum += __shfl_xor(part_sum, o);
            den += part_sum;
          }
          if (lane == 0) dens[qi] = den;
        }
        lds_barrier();
        for (int idx = tid; idx < nqb * (HD / 2); idx += LS_THREADS) {
          const int qi = idx / (HD / 2), dim = (idx - qi * (HD / 2)) * 2;
          const int qg = qb + qi;
          float n0 = 0.f, n1 = 0.f;
          for (int tb = 0; tb < nsuper; tb += 8) {
            float2 ov[8];
#pragma unroll
            for (int j = 0; j < 8; ++j)
              ov[j] = ldcf2(pin + ((size_t)((tb + j < nsuper) ? tb + j : 0) * 64 + qg) * PSTRIDE + dim);
#pragma unroll
            for (int j = 0; j < 8; ++j) {
              const float w = (tb + j < nsuper) ? wts[qi * nsuper + tb + j] : 0.f;
              n0 += w * ov[j].x;
              n1 += w * ov[j].y;
            }
          }
          const float den = dens[qi];
          const int n = qg / G, gq = qg - n * G;
          TT<T>::stc2(static_cast<T*>(pc.orows) + (size_t)n * P.qd + (c * G + gq) * HD + dim, n0 / den, n1 / den);
        }
      }
      if (tid == 0) stc32(P.attn_cnt + c, 0u);
    }
  }
  LS_PROF(0x25);
  drain_vmem();
  LS_PROF(0x26);
  return true;
}

// ------------------------------------------------------------------------------------------
// Stages C and E: x += W * in  (O projection of the attention output; down projection of the
// SwiGLU output), plus the per-tile sums of squares the next RMSNorm needs.
template <typename T, int NT>
__device__ __forceinline__ bool stage_resid(const PassCtx pc, int l, bool is_down) {
  LS_CTX;
  constexpr int DEPTH = 4 / NT;
  const LsLayerW W = layer_w(P, ms, l);
  const int dm = P.dm;
  const int K = is_down ? P.ffn : P.qd;
  const T* wmat = static_cast<const T*>(is_down ? W.wd : W.wo);
  const int tiles = dm / 16;
  const int groups = (tiles + NT - 1) / NT;
  ActDesc A;
  A.mode = ACT_PLAIN;
  A.src = is_down ? P.actbuf : pc.orows;
  A.ld = K;
  A.gain = nullptr;
  A.ssq = nullptr;
  A.ssq_nt = 0;
  const bool emb = !is_down && pc.embed_src && l == pc.l0;  // residual comes from the embedding row
  const int lane = LANE, wave = WAVE, n = lane & 15, g = lane >> 4;
  auto tiles_of = [&](int grp, const T* (&wt)[NT]) {
#pragma unroll
    for (int t = 0; t < NT; ++t) {
      const int tile = grp * NT + t;
      wt[t] = tile < tiles ? wmat + (size_t)tile * 16 * K : nullptr;
    }
  };
  Gemm<T, NT, DEPTH> G;
  const T* wt[NT];
  int grp = blockIdx.x;
  LS_PROF(is_down ? 0x50 : 0x30);
  grid_arrive(P, ms);
  if (grp < groups) { tiles_of(grp, wt); G.begin(wt, K); }
  // residual values of this workgroup's first tiles: written at least one barrier ago, so they can
  // be requested ahead of this stage's barrier
  float xres[4] = {0.f, 0.f, 0.f, 0.f};
  if (grp < groups && wave < NT && grp * NT + wave < tiles && n < pc.m) {
    const int row = (grp * NT + wave) * 16 + 4 * g;
    if (emb) {
      const T* e = static_cast<const T*>(P.embed) + (size_t)ms->tok[n] * dm + row;
#pragma unroll
      for (int j = 0; j < 4; ++j) xres[j] = TT<T>::ld(e + j);
    } else {
      const float* xr = P.xbuf + (size_t)(pc.row0 + n) * dm + row;
      const float2 o0 = ldcf2(xr), o1 = ldcf2(xr + 2);
      xres[0] = o0.x; xres[1] = o0.y; xres[2] = o1.x; xres[3] = o1.y;
    }
  }
  LS_PROF(is_down ? 0x51 : 0x31);
  if (!grid_wait(P, ms)) return false;
  LS_PROF(is_down ? 0x52 : 0x32);
  bool staged = false;
  for (; grp < groups; grp += gridDim.x) {
    {
      const T* wtn[NT];
      const int nx = grp + (int)gridDim.x;
      tiles_of(nx < groups ? nx : grp, wtn);
      G.set_next(wtn);
    }
    G.template run<ACT_PLAIN>(A, P, ms, pc.m, act, staged);
    LS_PROF(is_down ? 0x54 : 0x34);
    G.advance();
    for (int t = wave; t < NT; t += LS_WAVES) {
      const int tile = grp * NT + t;
      if (tile >= tiles) continue;
      const f32x4 v = tile_sum<NT>(act, t);
      const int row = tile * 16 + 4 * g;
      float nx[4] = {0.f, 0.f, 0.f, 0.f};
      if (n < pc.m) {
        float* xr = P.xbuf + (size_t)(pc.row0 + n) * dm + row;
        if (grp == (int)blockIdx.x) {
#pragma unroll
          for (int j = 0; j < 4; ++j) nx[j] = xres[j] + v[j];
        } else if (emb) {
          const T* e = static_cast<const T*>(P.embed) + (size_t)ms->tok[n] * dm + row;
#pragma unroll
          for (int j = 0; j < 4; ++j) nx[j] = TT<T>::ld(e + j) + v[j];
        } else {
          const float2 o0 = ldcf2(xr), o1 = ldcf2(xr + 2);
          nx[0] = o0.x + v[0]; nx[1] = o0.y + v[1]; nx[2] = o1.x + v[2]; nx[3] = o1.y + v[3];
        }
        stcf2(xr, nx[0], nx[1]);
        stcf2(xr + 2, nx[2], nx[3]);
        if (is_down && P.capture != nullptr)
          stg128(P.capture + ((size_t)l * P.max_seq + pc.pos0 + n) * dm + row, make_float4(nx[0], nx[1], nx[2], nx[3]));
      }
      float s = nx[0] * nx[0] + nx[1] * nx[1] + nx[2] * nx[2] + nx[3] * nx[3];
      s += __shfl_xor(s, 16);
      s += __shfl_xor(s, 32);
      if (g == 0 && n < pc.m) stcf(P.ssq + (size_t)(pc.row0 + n) * tiles + tile, s);
    }
  }
  LS_PROF(is_down ? 0x55 : 0x35);
  drain_vmem();
  LS_PROF(is_down ? 0x56 : 0x36);
  return true;
}

// ------------------------------------------------------------------------------------------
// Stage D: RMSNorm + gate/up projection + SwiGLU.  A work item pairs the gate tile and the up
// tile of the same 16 features.
template <typename T, int NT>
__device__ __forceinline__ bool stage_gu(const PassCtx pc, int l) {
  LS_CTX;
  constexpr int DEPTH = 4 / NT;
  constexpr int IPG = NT / 2;
  const LsLayerW W = layer_w(P, ms, l);
  const int dm = P.dm;
  const int items = P.ffn / 16;
  const int groups = (items + IPG - 1) / IPG;
  ActDesc A;
  A.mode = ACT_NORM_X;
  A.src = P.xbuf + (size_t)pc.row0 * dm;
  A.ld = dm;
  A.gain = W.ffn_norm;
  A.ssq = P.ssq + (size_t)pc.row0 * (dm / 16);
  A.ssq_nt = dm / 16;
  const int lane = LANE, wave = WAVE, n = lane & 15, g = lane >> 4;
  auto tiles_of = [&](int grp, const T* (&wt)[NT]) {
#pragma unroll
    for (int u = 0; u < IPG; ++u) {
      const int item = grp * IPG + u;
      wt[2 * u] = item < items ? static_cast<const T*>(W.wg) + (size_t)item * 16 * dm : nullptr;
      wt[2 * u + 1] = item < items ? static_cast<const T*>(W.wu) + (size_t)item * 16 * dm : nullptr;
    }
  };
  Gemm<T, NT, DEPTH> G;
  const T* wt[NT];
  int grp = blockIdx.x;
  LS_PROF(0x40);
  grid_arrive(P, ms);
  if (grp < groups) { tiles_of(grp, wt); G.begin(wt, dm); }
  LS_PROF(0x41);
  if (!grid_wait(P, ms)) return false;
  LS_PROF(0x42);
  LS_PROF(0x43);
  bool staged = false;
  for (; grp < groups; grp += gridDim.x) {
    {
      const T* wtn[NT];
      const int nx = grp + (int)gridDim.x;
      tiles_of(nx < groups ? nx : grp, wtn);
      G.set_next(wtn);
    }
    G.template run<ACT_NORM_X>(A, P, ms, pc.m, act, staged);
    LS_PROF(0x44);
    G.advance();
    if (wave < IPG) {
      const int item = grp * IPG + wave;
      if (item < items && n < pc.m) {
        const f32x4 gt = tile_sum<NT>(act, 2 * wave), up = tile_sum<NT>(act, 2 * wave + 1);
        float o[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const float z = gt[j];
          o[j] = (z / (1.0f + expf(-z))) * up[j];
        }
        TT<T>::stc4(static_cast<T*>(P.actbuf) + (size_t)n * P.ffn + item * 16 + 4 * g, o);
      }
    }
  }
  LS_PROF(0x45);
  drain_vmem();
  LS_PROF(0x46);
  return true;
}

// ------------------------------------------------------------------------------------------
// Head: final RMSNorm + LM head + per-row argmax (highest value, lowest index on ties) with the
// runner-up value kept for the margin.  Each workgroup writes one candidate per row.
template <typename T>
__device__ __noinline__ bool stage_head(const PassCtx pc) {
  LS_CTX;
  constexpr int NT = 2, DEPTH = 2;
  const int dm = P.dm;
  const int tiles = P.vocab / 16;
  const int groups = (tiles + NT - 1) / NT;
  ActDesc A;
  A.mode = ACT_NORM_X;
  A.src = P.xbuf + (size_t)pc.row0 * dm;
  A.ld = dm;
  A.gain = P.final_norm;
  A.ssq = P.ssq + (size_t)pc.row0 * (dm / 16);
  A.ssq_nt = dm / 16;
  const int lane = LANE, wave = WAVE, n = lane & 15, g = lane >> 4;
  auto tiles_of = [&](int grp, const T* (&wt)[NT]) {
#pragma unroll
    for (int t = 0; t < NT; ++t) {
      const int tile = grp * NT + t;
      wt[t] = tile < tiles ? static_cast<const T*>(P.lm_head) + (size_t)tile * 16 * dm : nullptr;
    }
  };
  Best best;
  best.v1 = -INFINITY; best.i1 = INT_MAX; best.v2 = -INFINITY;
  Gemm<T, NT, DEPTH> G;
  const T* wt[NT];
  int grp = blockIdx.x;
  LS_PROF(0x60);
  grid_arrive(P, ms);
  if (grp < groups) { tiles_of(grp, wt); G.begin(wt, dm); }
  LS_PROF(0x61);
  if (!grid_wait(P, ms)) return false;
  LS_PROF(0x62);
  LS_PROF(0x63);
  bool staged = false;
  for (; grp < groups; grp += gridDim.x) {
    {
      const T* wtn[NT];
      const int nx = grp + (int)gridDim.x;
      tiles_of(nx < groups ? nx : grp, wtn);
      G.set_next(wtn);
    }
    G.template run<ACT_NORM_X>(A, P, ms, pc.m, act, staged);
    LS_PROF(0x64);
    G.advance();
    const int tile = grp * NT + wave;
    if (wave < NT && tile < tiles) {
      const f32x4 v = tile_sum<NT>(act, wave);
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        Best c;
        c.v1 = v[j]; c.i1 = tile * 16 + 4 * g + j; c.v2 = -INFINITY;
        best = best_merge(best, c);
      }
    }
  }
  best = best_merge(best, best_shfl_xor(best, 16));
  best = best_merge(best, best_shfl_xor(best, 32));
  lds_barrier();
  if (g == 0) ms->wb[wave][n] = best;
  lds_barrier();
  if (TID < LS_ROWS) {
    Best b = ms->wb[0][TID];
#pragma unroll
    for (int w = 1; w < LS_WAVES; ++w) b = best_merge(b, ms->wb[w][TID]);
    float* dst = P.cand + ((size_t)blockIdx.x * LS_ROWS + TID) * 4;
    stcf2(dst, b.v1, __int_as_float(b.i1));
    stcf2(dst + 2, b.v2, 0.f);
  }
  drain_vmem();
  return true;
}

// After the head stage: every workgroup merges all candidates (same result everywhere).
__device__ __noinline__ bool reduce_cands(const PassCtx pc) {
  LS_CTX;
  LS_PROF(0x70);
  if (!grid_barrier(P, ms)) return false;
  LS_PROF(0x72);
  const int lane = LANE, wave = WAVE;
  for (int n = 0; n < pc.m; ++n) {
    Best b;
    b.v1 = -INFINITY; b.i1 = INT_MAX; b.v2 = -INFINITY;
    for (int w = TID; w < (int)gridDim.x; w += LS_THREADS) {
      const float* src = P.cand + ((size_t)w * LS_ROWS + n) * 4;
      const float2 c0 = ldcf2(src), c1 = ldcf2(src + 2);
      Best cb;
      cb.v1 = c0.x; cb.i1 = __float_as_int(c0.y); cb.v2 = c1.x;
      b = best_merge(b, cb);
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) b = best_merge(b, best_shfl_xor(b, o));
    if (lane == 0) ms->wb[wave][n] = b;
  }
  lds_barrier();
  if (TID < pc.m) {
    Best b = ms->wb[0][TID];
#pragma unroll
    for (int w = 1; w < LS_WAVES; ++w) b = best_merge(b, ms->wb[w][TID]);
    ms->r_tok[TID] = b.i1;
    ms->r_margin[TID] = b.v1 - b.v2;
  }
  lds_barrier();
  LS_PROF(0x76);
  return true;
}

// ------------------------------------------------------------------------------------------
// One decoder layer for the rows of a pass.  The five stages are inlined into ONE function per
// (dtype, head_dim, tiles-per-group) so that the call overhead (saving and restoring the callee-
// saved registers of a 250-register function) is paid once per layer, not once per stage.
template <typename T, int HD, int NTO>
__device__ __noinline__ bool layer_pass(const PassCtx pc, int l) {
  if (!stage_qkv<T, 2>(pc, l)) return false;
  if (!stage_attn<T, HD>(pc, l)) return false;
  if (!stage_resid<T, NTO>(pc, l, false)) return false;
  if (!stage_gu<T, 2>(pc, l)) return false;
  return stage_resid<T, NTO>(pc, l, true);
}

// One pass.  Every stage starts with the grid barrier that orders it after the stage before
// (weight loads for its first tiles are issued ahead of that barrier).
template <typename T>
__device__ __forceinline__ bool run_pass(const PassCtx& pc) {
  LS_CTX;
  const int variant = (P.hd == 128 ? 2 : 0) | (P.nt_o == 2 ? 1 : 0);
  for (int l = pc.l0; l < pc.l1; ++l) {
    bool ok;
    switch (variant) {
      case 0: ok = layer_pass<T, 64, 1>(pc, l); break;
      case 1: ok = layer_pass<T, 64, 2>(pc, l); break;
      case 2: ok = layer_pass<T, 128, 1>(pc, l); break;
      default: ok = layer_pass<T, 128, 2>(pc, l); break;
    }
    if (!ok) return false;
  }
  if (pc.head) {
    if (!stage_head<T>(pc)) return false;
    if (!reduce_cands(pc)) return false;
  }
  return true;
}

__device__ __forceinline__ int clamp_tok(int t, int vocab) { return t < 0 ? 0 : (t >= vocab ? vocab - 1 : t); }

// Self-drafting (Section 4.3.1) followed by the early-layer pass for the last draft.
template <typename T>
__device__ __forceinline__ bool do_draft(int E, int d) {
  LS_CTX;
  PassCtx pc;
  pc.qrows = P.qbuf; pc.orows = P.obuf;
  pc.m = 1; pc.l0 = 0; pc.l1 = E; pc.embed_src = true;
  for (int i = 0; i <= d; ++i) {
    if (TID == 0) ms->tok[0] = clamp_tok(i == 0 ? ms->st.last : ms->st.D[i - 1], P.vocab);
    __syncthreads();
    pc.row0 = i; pc.pos0 = ms->st.pos + i; pc.head = i < d;
    if (!run_pass<T>(pc)) return false;
    if (i < d && TID == 0) { ms->st.D[i] = ms->r_tok[0]; ms->st.dmargin[i] = ms->r_margin[0]; }
    __syncthreads();
  }
  if (TID == 0) { ms->st.draft_valid = 1; ms->st.draft_E = E; ms->st.draft_d = d; }
  __syncthreads();
  return true;
}

// Self-verification (Section 4.3.2), acceptance and cache crop (Appendix A.4).
template <typename T>
__device__ __forceinline__ bool do_verify(int E, int d) {
  LS_CTX;
  PassCtx pc;
  pc.qrows = P.qbuf; pc.orows = P.obuf;
  pc.m = d + 1; pc.row0 = 0; pc.pos0 = ms->st.pos; pc.l0 = E; pc.l1 = P.L; pc.embed_src = false; pc.head = true;
  if (!run_pass<T>(pc)) return false;
  if (TID == 0) {
    LsState& st = ms->st;
    for (int i = 0; i <= d; ++i) { st.V[i] = ms->r_tok[i]; st.vmargin[i] = ms->r_margin[i]; }
    int n = 0;
    while (n < d && st.D[n] == st.V[n]) ++n;
    st.n_acc = n;
    st.n_emit = n + 1;
    int used = 0;
    for (int i = 0; i <= n; ++i) {
      const int tok = (i < n) ? st.D[i] : st.V[n];
      if (st.n_gen + i >= P.max_new) break;
      if (P.out_tokens != nullptr && blockIdx.x == 0) P.out_tokens[st.n_gen + i] = tok;
      used = i + 1;
      if (tok == P.eos) { st.done = 1; break; }
    }
    st.pos += n + 1;
    st.last = st.V[n];
    st.n_gen += used;
    st.rounds += 1;
    st.drafted += d;
    st.accepted += n;
    st.draft_valid = 0;
    if (st.n_gen >= P.max_new) st.done = 1;
  }
  __syncthreads();
  return true;
}

template <typename T>
__device__ __forceinline__ void program_body(const LsKParams& Pk) {
  {
    Misc* const m0 = MS();
    if (TID == 0) m0->P = Pk;
    const int nptr = (Pk.L < LS_LDS_LAYERS ? Pk.L : LS_LDS_LAYERS) * (int)(sizeof(LsLayerW) / sizeof(void*));
    for (int i = TID; i < nptr; i += LS_THREADS)
      reinterpret_cast<const void**>(m0->lw)[i] = reinterpret_cast<const void* const*>(Pk.layers)[i];
    __syncthreads();
  }
  LS_CTX;
  if (TID == 0) {
    ms->st = *P.state;
    ms->epoch = 0;
    ms->abort = 0;
    ms->flag = 0;
    ms->prof_n = 0;
  }
  __syncthreads();
  bool ok = true;

  if (P.kind == LS_PROG_PREFILL || P.kind == LS_PROG_SCORE) {
    const int n = P.n_tokens;
    for (int c0 = 0; c0 < n && ok; c0 += LS_ROWS) {
      PassCtx pc;
  pc.qrows = P.qbuf; pc.orows = P.obuf;
      pc.m = (n - c0 < LS_ROWS) ? n - c0 : LS_ROWS;
      pc.row0 = 0; pc.pos0 = c0; pc.l0 = 0; pc.l1 = P.layers_used; pc.embed_src = true;
      pc.head = (P.kind == LS_PROG_SCORE) || (c0 + LS_ROWS >= n);
      if (TID < pc.m) ms->tok[TID] = clamp_tok(P.tokens[c0 + TID], P.vocab);
      __syncthreads();
      ok = run_pass<T>(pc);
      if (!ok) break;
      if (P.kind == LS_PROG_SCORE && blockIdx.x == 0 && TID < pc.m) {
        P.out_tokens[c0 + TID] = ms->r_tok[TID];
        if (P.out_margin != nullptr) P.out_margin[c0 + TID] = ms->r_margin[TID];
      }
      if (c0 + LS_ROWS >= n && TID == 0) {
        LsState& st = ms->st;
        const int keep_err = st.error;
        st = LsState{};
        st.error = keep_err;
        if (P.kind == LS_PROG_PREFILL) {
          st.pos = n; st.last = ms->r_tok[pc.m - 1]; st.n_gen = 1;
          st.vmargin[0] = ms->r_margin[pc.m - 1];
          if (P.out_tokens != nullptr && blockIdx.x == 0) P.out_tokens[0] = st.last;
          if (st.last == P.eos || P.max_new <= 1) st.done = 1;
        }
      }
      __syncthreads();
    }
  } else if (P.kind == LS_PROG_PF_ATTN) {
    // attention of prompt rows in blocks of 64/G query rows over the cache (K, V of all rows are in)
    const int n = P.n_tokens;
    const int rows = 64 / P.G;   // the attention stage takes up to 64 (row, query head) pairs per kv head
    for (int c0 = 0; c0 < n && ok; c0 += rows) {
      PassCtx pc;
      pc.m = (n - c0 < rows) ? n - c0 : rows;
      pc.row0 = 0; pc.pos0 = P.pf_pos0 + c0; pc.l0 = pc.l1 = P.pf_layer; pc.embed_src = false; pc.head = false;
      const size_t esz = sizeof(T);
      pc.qrows = static_cast<char*>(P.q_pf) + (size_t)c0 * P.qd * esz;
      pc.orows = static_cast<char*>(P.o_pf) + (size_t)c0 * P.qd * esz;
      ok = (P.hd == 128) ? stage_attn<T, 128>(pc, P.pf_layer) : stage_attn<T, 64>(pc, P.pf_layer);
    }
  } else if (P.kind == LS_PROG_PF_FINISH) {
    PassCtx pc;
    pc.qrows = P.qbuf; pc.orows = P.obuf;
    pc.m = 1; pc.row0 = 0; pc.pos0 = P.n_tokens - 1; pc.l0 = pc.l1 = 0; pc.embed_src = false; pc.head = true;
    ok = run_pass<T>(pc);
    if (ok && TID == 0) {
      LsState& st = ms->st;
      const int keep_err = st.error;
      st = LsState{};
      st.error = keep_err;
      st.pos = P.n_tokens; st.last = ms->r_tok[0]; st.n_gen = 1;
      st.vmargin[0] = ms->r_margin[0];
      if (P.out_tokens != nullptr && blockIdx.x == 0) P.out_tokens[0] = st.last;
      if (st.last == P.eos || P.max_new <= 1) st.done = 1;
    }
    __syncthreads();
  } else if (P.kind == LS_PROG_DRAFT) {
    if (ms->st.pos + P.d + 1 > P.max_seq) {
      if (TID == 0) ms->st.error = 2;
      __syncthreads();
    } else {
      ok = do_draft<T>(P.E, P.d);
    }
  } else if (P.kind == LS_PROG_VERIFY) {
    if (ms->st.draft_valid && ms->st.draft_E == P.E && ms->st.draft_d == P.d) ok = do_verify<T>(P.E, P.d);
  } else if (P.kind == LS_PROG_GENERATE) {
    while (ok && !ms->st.done && ms->st.n_gen < P.max_new) {
      if (ms->st.pos + P.d + 1 > P.max_seq) {
        if (TID == 0) { ms->st.error = 2; ms->st.done = 1; }
        __syncthreads();
        break;
      }
      if (P.d > 0) {
        ok = do_draft<T>(P.E, P.d);
        if (ok) ok = do_verify<T>(P.E, P.d);
      } else {
        PassCtx pc;
  pc.qrows = P.qbuf; pc.orows = P.obuf;
        pc.m = 1; pc.row0 = 0; pc.pos0 = ms->st.pos; pc.l0 = 0; pc.l1 = P.layers_used; pc.embed_src = true; pc.head = true;
        if (TID == 0) ms->tok[0] = clamp_tok(ms->st.last, P.vocab);
        __syncthreads();
        ok = run_pass<T>(pc);
        if (ok && TID == 0) {
          LsState& st = ms->st;
          const int tok = ms->r_tok[0];
          if (P.out_tokens != nullptr && blockIdx.x == 0) P.out_tokens[st.n_gen] = tok;
          st.vmargin[0] = ms->r_margin[0];
          st.pos += 1; st.last = tok; st.n_gen += 1;
          if (tok == P.eos || st.n_gen >= P.max_new) st.done = 1;
        }
        __syncthreads();
      }
    }
  }
  if (P.prof != nullptr && (int)blockIdx.x == P.prof_wg) {
    __syncthreads();
    const int nev = ms->prof_n < P.prof_cap ? ms->prof_n : P.prof_cap;
    for (int i = TID; i < nev; i += LS_THREADS)
      P.prof[i] = reinterpret_cast<const unsigned long long*>(ls_smem + LS_SMEM_BYTES)[i];
  }
  if (ok && blockIdx.x == 0 && TID == 0) {
    const int dev_err = P.state->error;
    LsState out = ms->st;
    if (dev_err != 0 && out.error == 0) out.error = dev_err;
    *P.state = out;
  }
}

// Three kernel symbols so that profiles separate the prompt passes, the self-speculative rounds
// and plain full-model greedy decoding.
template <typename T>
__global__ __launch_bounds__(LS_THREADS, 1) void ls_prompt_kernel(const LsKParams P) { program_body<T>(P); }
template <typename T>
__global__ __launch_bounds__(LS_THREADS, 1) void ls_decode_kernel(const LsKParams P) { program_body<T>(P); }
template <typename T>
__global__ __launch_bounds__(LS_THREADS, 1) void ls_greedy_kernel(const LsKParams P) { program_body<T>(P); }

// Plain copy, 16 bytes per thread per step: the known-size reference for hardware byte counters.
__global__ __launch_bounds__(256) void ls_copy_kernel(const uint4* __restrict__ src, uint4* __restrict__ dst, size_t n16) {
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += (size_t)gridDim.x * blockDim.x)
    dst[i] = src[i];
}

extern "C" int ls_launch_copy(const void* src, void* dst, size_t bytes, hipStream_t stream) {
  ls_copy_kernel<<<dim3(2048), dim3(256), 0, stream>>>(static_cast<const uint4*>(src), static_cast<uint4*>(dst), bytes / 16);
  return hipGetLastError() == hipSuccess ? 0 : 1;
}

// ------------------------------------------------------------------------------------------
static const void* kernel_for(int kind, int d, int dtype_is_bf16) {
  const bool prompt = kind == LS_PROG_PREFILL || kind == LS_PROG_SCORE || kind == LS_PROG_PF_ATTN || kind == LS_PROG_PF_FINISH;
  const bool greedy = kind == LS_PROG_GENERATE && d == 0;
  if (dtype_is_bf16)
    return prompt ? reinterpret_cast<const void*>(&ls_prompt_kernel<bf16_t>)
         : greedy ? reinterpret_cast<const void*>(&ls_greedy_kernel<bf16_t>)
                  : reinterpret_cast<const void*>(&ls_decode_kernel<bf16_t>);
  return prompt ? reinterpret_cast<const void*>(&ls_prompt_kernel<float>)
       : greedy ? reinterpret_cast<const void*>(&ls_greedy_kernel<float>)
                : reinterpret_cast<const void*>(&ls_decode_kernel<float>);
}

extern "C" int ls_launch_program(const LsKParams* p, int dtype_is_bf16, int grid, hipStream_t stream) {
  void* args[1] = {const_cast<LsKParams*>(p)};
  // The grid is sized to be co-resident (occupancy x compute units) and the barrier wait is bounded,
  // so an ordinary launch is used; LS_COOPERATIVE_LAUNCH=1 asks the runtime to guarantee residency.
  static const bool coop = []() { const char* v = getenv("LS_COOPERATIVE_LAUNCH"); return v != nullptr && v[0] == '1'; }();
  const size_t smem = LS_SMEM_BYTES + (p->prof != nullptr ? LS_PROF_EVENTS * 8 : 0);
  hipError_t e = coop ? hipLaunchCooperativeKernel(kernel_for(p->kind, p->d, dtype_is_bf16), dim3(grid), dim3(LS_THREADS),
                                                   args, smem, stream)
                      : hipLaunchKernel(kernel_for(p->kind, p->d, dtype_is_bf16), dim3(grid), dim3(LS_THREADS), args,
                                        smem, stream);
  return e == hipSuccess ? 0 : (int)e;
}

extern "C" int ls_kernel_setup(int dtype_is_bf16, int* max_blocks_per_cu) {
  int nb_min = 1 << 30;
  for (int v = 0; v < 3; ++v) {
    const void* fn = kernel_for(v == 0 ? (int)LS_PROG_PREFILL : (int)LS_PROG_GENERATE, v == 1 ? 0 : 1, dtype_is_bf16);
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
