// Prompt pass (prefill) for gfx950: all rows of the prompt go through each layer together, so the
// projections are real GEMMs (M = prompt rows) on the MFMA units instead of 16-row passes that
// re-read every weight.  Per layer:
//   RMSNorm -> Q/K/V GEMMs (+RoPE, KV append) -> causal attention over the shared cache (MFMA,
//   running softmax over K/V tiles) -> O GEMM (+residual) -> RMSNorm -> gate/up GEMM (+SwiGLU) ->
//   down GEMM (+residual).
// Rounding points are the ones of the decode path: RMSNorm output, q/k after RoPE, v, the
// attention output and the SwiGLU output are stored in the model dtype; the residual stream and
// all accumulation are fp32.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <math.h>
#include <stdlib.h>

#include "ls_internal.h"

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint16_t bf16_t;

namespace {

__device__ __forceinline__ float bf2f(uint32_t b) { return __uint_as_float(b << 16); }
__device__ __forceinline__ uint32_t f2bf(float f) {
  uint32_t u = __float_as_uint(f);
  return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
}

template <typename T> struct PT;
template <> struct PT<float> {
  static constexpr int EPV = 4;
  static __device__ __forceinline__ float ld(const float* p) { return *p; }
  static __device__ __forceinline__ void st(float* p, float v) { *p = v; }
  static __device__ __forceinline__ void mma(f32x4& acc, const uint4& a, const uint4& b) {
    acc = __builtin_amdgcn_mfma_f32_16x16x4f32(__uint_as_float(a.x), __uint_as_float(b.x), acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_16x16x4f32(__uint_as_float(a.y), __uint_as_float(b.y), acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_16x16x4f32(__uint_as_float(a.z), __uint_as_float(b.z), acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_16x16x4f32(__uint_as_float(a.w), __uint_as_float(b.w), acc, 0, 0, 0);
  }
};
template <> struct PT<bf16_t> {
  static constexpr int EPV = 8;
  static __device__ __forceinline__ float ld(const bf16_t* p) { return bf2f(*p); }
  static __device__ __forceinline__ void st(bf16_t* p, float v) { *p = (bf16_t)f2bf(v); }
  static __device__ __forceinline__ void mma(f32x4& acc, const uint4& a, const uint4& b) {
    acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), acc, 0, 0, 0);
  }
};

// ------------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void pf_embed_kernel(const int32_t* tok, const T* embed, float* x, int dm, int vocab) {
  const int m = blockIdx.x;
  int t = tok[m];
  t = t < 0 ? 0 : (t >= vocab ? vocab - 1 : t);
  const T* e = embed + (size_t)t * dm;
  for (int k = threadIdx.x; k < dm; k += 256) x[(size_t)m * dm + k] = PT<T>::ld(e + k);
}

// a[m][k] = T((x[m][k] * rinv_m) * gain[k]),  rinv_m = 1/sqrt(mean_k x[m][k]^2 + eps)
template <typename T>
__global__ __launch_bounds__(256) void pf_rmsnorm_kernel(const float* x, const T* gain, T* a, int dm, float eps) {
  __shared__ float red[4];
  const int m = blockIdx.x;
  const float* xr = x + (size_t)m * dm;
  float s = 0.f;
  for (int k = threadIdx.x; k < dm; k += 256) { const float v = xr[k]; s += v * v; }
  for (int o = 32; o > 0; o >>= 1) s += __shfl_xor(s, o);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = s;
  __syncthreads();
  const float tot = (red[0] + red[1]) + (red[2] + red[3]);
  const float r = 1.0f / sqrtf(tot / (float)dm + eps);
  for (int k = threadIdx.x; k < dm; k += 256) PT<T>::st(a + (size_t)m * dm + k, (xr[k] * r) * PT<T>::ld(gain + k));
}

// The last prompt row goes to row 0 of the decode residual buffer, with its sum of squares spread
// over the nt slots the decode kernel's RMSNorm adds up (slot t: columns [t*gs, (t+1)*gs), zero past
// the end of the row); the head then runs in the decode kernel.
__global__ __launch_bounds__(256) void pf_finish_kernel(const float* xrow, float* xbuf, float* ssq, int dm, int nt) {
  const int gs = (dm + nt - 1) / nt;
  for (int t = threadIdx.x; t < nt; t += 256) {
    float s = 0.f;
    for (int j = 0; j < gs && t * gs + j < dm; ++j) { const float v = xrow[t * gs + j]; xbuf[t * gs + j] = v; s += v * v; }
    ssq[t] = s;
  }
}

// ------------------------------------------------------------------------------------------
// EPI_QKV: the three projections of the attention input in one launch; a tile's columns decide which
// matrix it multiplies and which of the first three epilogues it takes (q_dim and kv_dim are multiples
// of the tile width there, so a tile never straddles two matrices).  Three launches of 640 tiles each
// (13B shape, 1024 prompt rows) fill the 512 resident workgroups one and a quarter times each; one
// launch of 1920 tiles fills them three and three quarter times.
enum { EPI_ROPE_Q = 0, EPI_ROPE_K = 1, EPI_V = 2, EPI_RESID = 3, EPI_GU = 4, EPI_QKV = 5 };

struct PfGemm {
  const void* A;    // [M][K] activations (model dtype), row stride lda
  int lda;
  const void* W;    // [N][K] weights
  const void* W2;   // second weight matrix (gate/up: W = gate, W2 = up; QKV: W = wq, W2 = wk, W3 = wv)
  const void* W3;
  int M, N, K;      // (QKV: N = q_dim + 2 kv_dim, N_q = q_dim, N_kv = kv_dim)
  int N_q, N_kv;
  void* out;        // q rows [M][ldo] / SwiGLU rows [M][ldo] (model dtype); KV cache base for K, V
  void* out_k;      // QKV: the K and the V cache (out = q rows)
  void* out_v;
  int ldo;
  float* x;         // residual rows [M][N] fp32 (EPI_RESID)
  float* capture;   // optional copy of the new residual rows, [max_seq][N] of this layer
  const float* rope_cos; const float* rope_sin;
  int hd, pos0, max_seq, nkv, layer;
  int tile_rows;    // 0: chosen from the number of tiles; 32, 64, 128: forced (host only)
};

// Which output tile a workgroup computes.  Workgroups are dealt round-robin to the 8 dies, each with
// an L2 of its own, so the ids that are congruent mod 8 are renumbered consecutively and walk the
// tile grid in panels of 4 tile columns, row by row: the workgroups that run together on a die then
// cover a compact block of tiles (for the 7B prompt exactly 12 x 4), and every A and W tile is
// fetched from memory once per die and panel instead of once per workgroup.  (If the dealing were
// different, the map would still be a bijection; only the locality would suffer.)
__device__ __forceinline__ void pf_tile_of(int MT, int NT, int& tm, int& tn) {
  constexpr int NX = 8, PN = 4;
  const int total = MT * NT, id = (int)blockIdx.x;
  const int x = id % NX, local = id / NX;
  int base = 0;
  for (int y = 0; y < x; ++y) base += (total - y + NX - 1) / NX;
  const int lin = base + local;
  const int panel = lin / (MT * PN), n_first = panel * PN;
  const int pw = NT - n_first < PN ? NT - n_first : PN;
  const int r = lin - panel * MT * PN;
  tm = r / pw;
  tn = n_first + (r - tm * pw);
}

constexpr int BM = 128, BN = 128;
constexpr int ROWB = 128;          // bytes of K per tile row
constexpr int ROWP = ROWB + 16;    // padded LDS row

// BMT: rows of the output tile (128, or 64 when there are too few 128-row tiles to keep several
// workgroups resident per compute unit); a wave computes BMT/4 rows x BNT columns.
// BNT: columns of the output tile, 128, or 160 for the products into the residual rows when that makes
// the number of tiles fit the resident workgroups better (see launch_gemm).
template <typename T, int EPI, int BMT, int BNT = BN>
__global__ __launch_bounds__(256, 2) void pf_gemm_kernel(const PfGemm g) {
  static_assert(BNT % 32 == 0 && (BNT == BN || EPI == EPI_RESID), "rotations pair columns inside a 128-column tile");
  constexpr int NF = BNT / 16;          // 16-column fragments per tile
  constexpr int LW = BNT * 8 / 256;     // 16-byte units of a W tile per thread
  constexpr int EPV = PT<T>::EPV;
  constexpr int BK = ROWB / (int)sizeof(T);
  constexpr int NW = (EPI == EPI_GU) ? 2 : 1;
  constexpr int RT = BMT / 64;          // 16-row tiles per wave
  constexpr int LA = BMT * 8 / 256;     // 16-byte units of the A tile per thread
  __shared__ __align__(16) char As[BMT * ROWP];
  __shared__ __align__(16) char Ws[NW][BNT * ROWP];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int r = lane & 15, gq = lane >> 4;
  int tile_m, tile_n;
  pf_tile_of((g.M + BMT - 1) / BMT, (g.N + BNT - 1) / BNT, tile_m, tile_n);
  int n0 = tile_n * BNT;
  const int m0 = tile_m * BMT;
  const T* Ag = static_cast<const T*>(g.A);
  const T* Wg[2] = {static_cast<const T*>(g.W), static_cast<const T*>(g.W2)};
  int epi = EPI, n_cols = g.N;   // this tile's epilogue and the columns of its matrix (uniform; constants unless QKV)
  void* outp = g.out;
  if (EPI == EPI_QKV) {
    if (n0 < g.N_q) { epi = EPI_ROPE_Q; n_cols = g.N_q; }
    else if (n0 < g.N_q + g.N_kv) { epi = EPI_ROPE_K; n0 -= g.N_q; n_cols = g.N_kv; Wg[0] = static_cast<const T*>(g.W2); outp = g.out_k; }
    else { epi = EPI_V; n0 -= g.N_q + g.N_kv; n_cols = g.N_kv; Wg[0] = static_cast<const T*>(g.W3); outp = g.out_v; }
  }

  f32x4 acc[NW][RT][NF];
#pragma unroll
  for (int w = 0; w < NW; ++w)
#pragma unroll
    for (int i = 0; i < RT; ++i)
#pragma unroll
      for (int j = 0; j < NF; ++j) acc[w][i][j] = f32x4{0.f, 0.f, 0.f, 0.f};

  uint4 ra[LA], rw[NW][LW];
  auto gload = [&](int k0) {
#pragma unroll
    for (int i = 0; i < LA; ++i) {
      const int unit = tid + 256 * i, row = unit >> 3, u = unit & 7;
      const int k = k0 + u * EPV, ma = m0 + row;
      const bool aok = k < g.K && ma < g.M;
      const uint4 va = *reinterpret_cast<const uint4*>(Ag + (size_t)(aok ? ma : 0) * g.lda + (aok ? k : 0));
      ra[i] = aok ? va : make_uint4(0, 0, 0, 0);
    }
#pragma unroll
    for (int i = 0; i < LW; ++i) {
      const int unit = tid + 256 * i, row = unit >> 3, u = unit & 7;
      const int k = k0 + u * EPV, na = n0 + row;
      const bool wok = k < g.K && na < n_cols;
#pragma unroll
      for (int w = 0; w < NW; ++w) {
        const uint4 vw = *reinterpret_cast<const uint4*>(Wg[w] + (size_t)(wok ? na : 0) * g.K + (wok ? k : 0));
        rw[w][i] = wok ? vw : make_uint4(0, 0, 0, 0);
      }
    }
  };
  auto lstore = [&]() {
#pragma unroll
    for (int i = 0; i < LA; ++i) {
      const int unit = tid + 256 * i, row = unit >> 3, u = unit & 7;
      *reinterpret_cast<uint4*>(As + row * ROWP + u * 16) = ra[i];
    }
#pragma unroll
    for (int i = 0; i < LW; ++i) {
      const int unit = tid + 256 * i, row = unit >> 3, u = unit & 7;
#pragma unroll
      for (int w = 0; w < NW; ++w) *reinterpret_cast<uint4*>(Ws[w] + row * ROWP + u * 16) = rw[w][i];
    }
  };

  gload(0);
  for (int k0 = 0; k0 < g.K; k0 += BK) {
    __syncthreads();
    lstore();
    __syncthreads();
    if (k0 + BK < g.K) gload(k0 + BK);
#pragma unroll
    for (int s = 0; s < 2; ++s) {
      uint4 fa[RT];
#pragma unroll
      for (int i = 0; i < RT; ++i)
        fa[i] = *reinterpret_cast<const uint4*>(As + (wave * (16 * RT) + i * 16 + r) * ROWP + (s * 4 + gq) * 16);
#pragma unroll
      for (int w = 0; w < NW; ++w) {
#pragma unroll
        for (int j = 0; j < NF; ++j) {
          const uint4 fb = *reinterpret_cast<const uint4*>(Ws[w] + (j * 16 + r) * ROWP + (s * 4 + gq) * 16);
#pragma unroll
          for (int i = 0; i < RT; ++i) PT<T>::mma(acc[w][i][j], fa[i], fb);
        }
      }
    }
  }

  // epilogue: the lane holds rows m = base + 4*gq + jj (jj = 0..3) of column n = n0 + 16*j + r
  const int half = g.hd / 2;
#pragma unroll
  for (int i = 0; i < RT; ++i) {
#pragma unroll
    for (int jj = 0; jj < 4; ++jj) {
      const int m = m0 + wave * (16 * RT) + i * 16 + 4 * gq + jj;
      if (m >= g.M) continue;
      const int pos = g.pos0 + m;
#pragma unroll
      for (int j = 0; j < NF; ++j) {
        const int n = n0 + 16 * j + r;
        if (n >= n_cols) continue;
        const float v = acc[0][i][j][jj];
        if (epi == EPI_RESID) {
          float* xr = g.x + (size_t)m * g.N + n;
          const float nv = *xr + v;
          *xr = nv;
          if (g.capture != nullptr) g.capture[(size_t)pos * g.N + n] = nv;
        } else if (epi == EPI_GU) {
          const float up = acc[NW - 1][i][j][jj];
          PT<T>::st(static_cast<T*>(outp) + (size_t)m * g.ldo + n, (v / (1.0f + expf(-v))) * up);
        } else if (epi == EPI_V) {
          const int h = n / g.hd, d = n - h * g.hd;
          PT<T>::st(static_cast<T*>(outp) + (((size_t)g.layer * g.nkv + h) * g.max_seq + pos) * g.hd + d, v);
        } else {
          // rotation mixes columns d and d + hd/2 of one head; both sit in this lane (tile j and j + half/16)
          const int h = n / g.hd, d = n - h * g.hd;
          if (d < half) {
            // partner tile: 4 tiles on for head_dim 128, 2 tiles on for head_dim 64 (static indices)
            const float b = (g.hd == 128) ? acc[0][i][(j + 4) % NF][jj] : acc[0][i][(j + 2) % NF][jj];
            const float c = g.rope_cos[(size_t)pos * half + d], s = g.rope_sin[(size_t)pos * half + d];
            const float lo = v * c - b * s, hi = b * c + v * s;
            if (epi == EPI_ROPE_Q) {
              T* dst = static_cast<T*>(outp) + (size_t)m * g.ldo + h * g.hd;
              PT<T>::st(dst + d, lo);
              PT<T>::st(dst + d + half, hi);
            } else {
              T* dst = static_cast<T*>(outp) + (((size_t)g.layer * g.nkv + h) * g.max_seq + pos) * g.hd;
              PT<T>::st(dst + d, lo);
              PT<T>::st(dst + d + half, hi);
            }
          }
        }
      }
    }
  }
}

// The same product for few rows: 32 x 128 output tiles, so that a prompt of a few hundred rows
// still gives every compute unit a tile, with the four waves splitting K (each wave takes one
// 64-byte sub-step of a 256-byte step and keeps a partial 32 x 128 tile, i.e. the same operand
// reuse per wave as above); the partial tiles are added through LDS in a fixed order and the
// epilogue then walks the tile row by row, which also makes its stores contiguous.
constexpr int SBM = 32;
constexpr int SROWB = 256;
constexpr int SROWP = SROWB + 16;
constexpr int SREDP = BN + 4;      // padded fp32 row of the reduction buffer

template <int NW>
constexpr int ks_smem_bytes() {
  return (SBM * SROWP + NW * BN * SROWP) > (2 * NW * SBM * SREDP * 4) ? (SBM * SROWP + NW * BN * SROWP)
                                                                     : (2 * NW * SBM * SREDP * 4);
}

template <typename T, int EPI>
__global__ __launch_bounds__(256, 2) void pf_gemm_ks_kernel(const PfGemm g) {
  constexpr int EPV = PT<T>::EPV;
  constexpr int BK = SROWB / (int)sizeof(T);
  constexpr int NW = (EPI == EPI_GU) ? 2 : 1;
  extern __shared__ __align__(16) char ks_smem[];
  char* As = ks_smem;
  char* Ws = ks_smem + SBM * SROWP;   // [NW][BN][SROWP]
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int r = lane & 15, gq = lane >> 4;
  int tile_m, tile_n;
  pf_tile_of((g.M + SBM - 1) / SBM, (g.N + BN - 1) / BN, tile_m, tile_n);
  const int n0 = tile_n * BN, m0 = tile_m * SBM;
  const T* Ag = static_cast<const T*>(g.A);
  const T* Wg[2] = {static_cast<const T*>(g.W), static_cast<const T*>(g.W2)};

  f32x4 acc[NW][2][8];
#pragma unroll
  for (int w = 0; w < NW; ++w)
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int j = 0; j < 8; ++j) acc[w][i][j] = f32x4{0.f, 0.f, 0.f, 0.f};

  uint4 ra[2], rw[NW][8];
  auto gload = [&](int k0) {
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int unit = tid + 256 * i, row = unit >> 4, u = unit & 15;
      const int k = k0 + u * EPV, ma = m0 + row;
      const bool aok = k < g.K && ma < g.M;
      const uint4 va = *reinterpret_cast<const uint4*>(Ag + (size_t)(aok ? ma : 0) * g.lda + (aok ? k : 0));
      ra[i] = aok ? va : make_uint4(0, 0, 0, 0);
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int unit = tid + 256 * i, row = unit >> 4, u = unit & 15;
      const int k = k0 + u * EPV, na = n0 + row;
      const bool wok = k < g.K && na < g.N;
#pragma unroll
      for (int w = 0; w < NW; ++w) {
        const uint4 vw = *reinterpret_cast<const uint4*>(Wg[w] + (size_t)(wok ? na : 0) * g.K + (wok ? k : 0));
        rw[w][i] = wok ? vw : make_uint4(0, 0, 0, 0);
      }
    }
  };
  auto lstore = [&]() {
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int unit = tid + 256 * i, row = unit >> 4, u = unit & 15;
      *reinterpret_cast<uint4*>(As + row * SROWP + u * 16) = ra[i];
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int unit = tid + 256 * i, row = unit >> 4, u = unit & 15;
#pragma unroll
      for (int w = 0; w < NW; ++w) *reinterpret_cast<uint4*>(Ws + (w * BN + row) * SROWP + u * 16) = rw[w][i];
    }
  };

  gload(0);
  for (int k0 = 0; k0 < g.K; k0 += BK) {
    __syncthreads();
    lstore();
    __syncthreads();
    if (k0 + BK < g.K) gload(k0 + BK);
    uint4 fa[2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
      fa[i] = *reinterpret_cast<const uint4*>(As + (i * 16 + r) * SROWP + (wave * 4 + gq) * 16);
#pragma unroll
    for (int w = 0; w < NW; ++w) {
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const uint4 fb = *reinterpret_cast<const uint4*>(Ws + (w * BN + j * 16 + r) * SROWP + (wave * 4 + gq) * 16);
#pragma unroll
        for (int i = 0; i < 2; ++i) PT<T>::mma(acc[w][i][j], fa[i], fb);
      }
    }
  }

  // waves 0 and 1 store their partial tiles, waves 2 and 3 add theirs on top (each lane to the
  // addresses of the same tile elements), the epilogue adds the two buffers: ((w0 + w2) + (w1 + w3))
  float* red = reinterpret_cast<float*>(ks_smem);   // [2][NW][SBM][SREDP]
  __syncthreads();
#pragma unroll
  for (int phase = 0; phase < 2; ++phase) {
    if ((wave >> 1) == phase) {
      float* rb = red + (size_t)(wave & 1) * NW * SBM * SREDP;
#pragma unroll
      for (int w = 0; w < NW; ++w)
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
          for (int j = 0; j < 8; ++j)
#pragma unroll
            for (int jj = 0; jj < 4; ++jj) {
              float* dst = rb + ((size_t)w * SBM + i * 16 + 4 * gq + jj) * SREDP + 16 * j + r;
              if (phase == 0) *dst = acc[w][i][j][jj];
              else *dst += acc[w][i][j][jj];
            }
    }
    __syncthreads();
  }

  const int half = g.hd / 2;
  const float* r0 = red;
  const float* r1 = red + (size_t)NW * SBM * SREDP;
  auto val = [&](int w, int ml, int nl) {
    const size_t o = ((size_t)w * SBM + ml) * SREDP + nl;
    return r0[o] + r1[o];
  };
  for (int e = tid; e < SBM * BN; e += 256) {
    const int ml = e / BN, nl = e - ml * BN;
    const int m = m0 + ml, n = n0 + nl;
    if (m >= g.M || n >= g.N) continue;
    const int pos = g.pos0 + m;
    const float v = val(0, ml, nl);
    if (EPI == EPI_RESID) {
      float* xr = g.x + (size_t)m * g.N + n;
      const float nv = *xr + v;
      *xr = nv;
      if (g.capture != nullptr) g.capture[(size_t)pos * g.N + n] = nv;
    } else if (EPI == EPI_GU) {
      const float up = val(NW - 1, ml, nl);
      PT<T>::st(static_cast<T*>(g.out) + (size_t)m * g.ldo + n, (v / (1.0f + expf(-v))) * up);
    } else if (EPI == EPI_V) {
      const int h = n / g.hd, d = n - h * g.hd;
      PT<T>::st(static_cast<T*>(g.out) + (((size_t)g.layer * g.nkv + h) * g.max_seq + pos) * g.hd + d, v);
    } else {
      // rotation mixes columns d and d + hd/2 of one head; a 128-column tile holds whole heads
      const int h = n / g.hd, d = n - h * g.hd;
      if (d < half) {
        const float b = val(0, ml, nl + half);
        const float c = g.rope_cos[(size_t)pos * half + d], sn = g.rope_sin[(size_t)pos * half + d];
        const float lo = v * c - b * sn, hi = b * c + v * sn;
        T* dst = (EPI == EPI_ROPE_Q) ? static_cast<T*>(g.out) + (size_t)m * g.ldo + h * g.hd
                                     : static_cast<T*>(g.out) + (((size_t)g.layer * g.nkv + h) * g.max_seq + pos) * g.hd;
        PT<T>::st(dst + d, lo);
        PT<T>::st(dst + d + half, hi);
      }
    }
  }
}

// Few 128 x 128 tiles (a short prompt) leave most compute units without work: then 32-row tiles.
// Both kernels are bound by how fast a compute unit takes in its operand tiles (one K step in
// flight per workgroup), so the small tile's lower reuse only pays below about half a tile per
// compute unit (measured on 256 CUs: 64 tiles 1.8x faster, 176 tiles 1.5x slower).
static bool use_small_tiles(const PfGemm& g) {
  if (g.tile_rows) return g.tile_rows == SBM;
  const long tiles = (long)((g.N + BN - 1) / BN) * ((g.M + BM - 1) / BM);
  return tiles < 128;
}

template <typename T, int EPI>
hipError_t launch_gemm(const PfGemm& g, hipStream_t s) {
  if constexpr (EPI != EPI_QKV) {   // (the fused launch exists for the large tiles only; its caller checks)
  if (use_small_tiles(g)) {
    constexpr int NW = (EPI == EPI_GU) ? 2 : 1;
    constexpr int smem = ks_smem_bytes<NW>();
    static bool configured = false;   // (per instantiation; the attribute is per function, not per device state that could go stale)
    if (!configured) {
      const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&pf_gemm_ks_kernel<T, EPI>),
                                               hipFuncAttributeMaxDynamicSharedMemorySize, smem);
      if (e != hipSuccess) return e;
      configured = true;
    }
    dim3 grid(((g.N + BN - 1) / BN) * ((g.M + SBM - 1) / SBM));
    pf_gemm_ks_kernel<T, EPI><<<grid, dim3(256), smem, s>>>(g);
    return hipGetLastError();
  }
  }
  // 64-row tiles while 128-row tiles would leave fewer than about two per compute unit
  const long tiles128 = (long)((g.N + BN - 1) / BN) * ((g.M + BM - 1) / BM);
  const bool rows64 = g.tile_rows == 64 || g.tile_rows == 160 || (g.tile_rows != 128 && tiles128 < 600);
  if constexpr (EPI == EPI_RESID) {
    // Tiles of 160 columns where they divide the width and fill the resident workgroups (two per compute
    // unit, 512 on this chip) in fewer, fuller rounds: 1024 rows x 5120 columns are 640 tiles of 64 x 128,
    // i.e. one full round and a quarter of one, but 512 tiles of 64 x 160, exactly one round.
    if (rows64 && g.N % 160 == 0) {
      const long t128 = (long)(g.N / BN) * ((g.M + 63) / 64), t160 = (long)(g.N / 160) * ((g.M + 63) / 64);
      const long cost128 = ((t128 + 511) / 512) * 128, cost160 = ((t160 + 511) / 512) * 160;
      if (g.tile_rows == 160 || (g.tile_rows == 0 && cost160 < cost128)) {
        pf_gemm_kernel<T, EPI, 64, 160><<<dim3((unsigned)t160), dim3(256), 0, s>>>(g);
        return hipGetLastError();
      }
    }
  }
  if (rows64) {
    dim3 grid(((g.N + BN - 1) / BN) * ((g.M + 63) / 64));
    pf_gemm_kernel<T, EPI, 64><<<grid, dim3(256), 0, s>>>(g);
  } else {
    dim3 grid(((g.N + BN - 1) / BN) * ((g.M + BM - 1) / BM));
    pf_gemm_kernel<T, EPI, 128><<<grid, dim3(256), 0, s>>>(g);
  }
  return hipGetLastError();
}


// ------------------------------------------------------------------------------------------
// Causal attention of the prompt rows on the MFMA units.  One workgroup = 64 query rows of one
// query head (a wave = 16 of them); K/V tiles of TK positions are staged in LDS (V transposed, so
// that both operands of both products are contiguous along the contracted index) and folded in
// with a running softmax.  Everything is computed transposed:
//   S^T = K . Q^T   (rows: keys,  columns: the wave's 16 queries)
//   O^T = V^T . P^T (rows: dims,  columns: the same queries)
// so a lane keeps one query's statistics: lane (c = lane & 15, g = lane >> 4) holds S^T rows
// 4g..4g+3 of column c for each 16-key block, which are exactly the slots 8g..8g+7 of the P^T
// operand when a 32-key half is numbered (block 0: keys 4g..4g+3, block 1: keys 16+4g..16+4g+3);
// the V^T operand is read from LDS in that order.  Probabilities stay fp32 in effect: for bf16
// models P is fed as a bf16 head plus a bf16 remainder (two products), scores, statistics and the
// output accumulate in fp32; the output is rounded to the model dtype on store, like the decode path.
template <typename T> struct AT;
template <> struct AT<bf16_t> {
  struct Op { uint4 v; };
  static __device__ __forceinline__ Op ld8(const bf16_t* p) { Op o; o.v = *reinterpret_cast<const uint4*>(p); return o; }
  static __device__ __forceinline__ Op ld44(const bf16_t* p0, const bf16_t* p1) {
    const uint2 a = *reinterpret_cast<const uint2*>(p0), b = *reinterpret_cast<const uint2*>(p1);
    Op o; o.v = make_uint4(a.x, a.y, b.x, b.y); return o;
  }
  static __device__ __forceinline__ void mma(f32x4& acc, const Op& a, const Op& b) {
    acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a.v), __builtin_bit_cast(bf16x8, b.v), acc, 0, 0, 0);
  }
  static __device__ __forceinline__ void mma_p(f32x4& acc, const Op& a, const float* p) {
    uint32_t hi[8], lo[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) { hi[j] = f2bf(p[j]); lo[j] = f2bf(p[j] - bf2f(hi[j])); }
    Op h, l;
    h.v = make_uint4(hi[0] | (hi[1] << 16), hi[2] | (hi[3] << 16), hi[4] | (hi[5] << 16), hi[6] | (hi[7] << 16));
    l.v = make_uint4(lo[0] | (lo[1] << 16), lo[2] | (lo[3] << 16), lo[4] | (lo[5] << 16), lo[6] | (lo[7] << 16));
    mma(acc, a, h);
    mma(acc, a, l);
  }
  static __device__ __forceinline__ void scatter(bf16_t* vt, int stride, const uint4& v) {  // 8 elements, one per row
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int e = 0; e < 8; ++e) vt[e * stride] = (bf16_t)((w[e >> 1] >> ((e & 1) * 16)) & 0xFFFFu);
  }
};
template <> struct AT<float> {
  struct Op { float f[8]; };
  static __device__ __forceinline__ Op ld8(const float* p) {
    const float4 a = *reinterpret_cast<const float4*>(p), b = *reinterpret_cast<const float4*>(p + 4);
    Op o; o.f[0] = a.x; o.f[1] = a.y; o.f[2] = a.z; o.f[3] = a.w; o.f[4] = b.x; o.f[5] = b.y; o.f[6] = b.z; o.f[7] = b.w; return o;
  }
  static __device__ __forceinline__ Op ld44(const float* p0, const float* p1) {
    const float4 a = *reinterpret_cast<const float4*>(p0), b = *reinterpret_cast<const float4*>(p1);
    Op o; o.f[0] = a.x; o.f[1] = a.y; o.f[2] = a.z; o.f[3] = a.w; o.f[4] = b.x; o.f[5] = b.y; o.f[6] = b.z; o.f[7] = b.w; return o;
  }
  static __device__ __forceinline__ void mma(f32x4& acc, const Op& a, const Op& b) {
#pragma unroll
    for (int j = 0; j < 8; ++j) acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a.f[j], b.f[j], acc, 0, 0, 0);
  }
  static __device__ __forceinline__ void mma_p(f32x4& acc, const Op& a, const float* p) {
#pragma unroll
    for (int j = 0; j < 8; ++j) acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a.f[j], p[j], acc, 0, 0, 0);
  }
  static __device__ __forceinline__ void scatter(float* vt, int stride, const uint4& v) {   // 4 elements
    vt[0] = __uint_as_float(v.x); vt[stride] = __uint_as_float(v.y);
    vt[2 * stride] = __uint_as_float(v.z); vt[3 * stride] = __uint_as_float(v.w);
  }
};

template <typename T, int HD>
__global__ __launch_bounds__(256) void pf_attn_kernel(const T* __restrict__ q, T* __restrict__ o,
                                                      const T* __restrict__ kc, const T* __restrict__ vc, int M,
                                                      int pos0, int qd, int G, int max_seq, float scale) {
  constexpr int EPV = 16 / (int)sizeof(T);          // elements per 16 bytes
  constexpr int TK = sizeof(T) == 2 ? 64 : 32;      // positions per K/V tile
  constexpr int KB16 = TK / 16, HF = TK / 32, KS = HD / 32, DB = HD / 16;
  constexpr int KROW = HD + EPV;                    // padded rows: conflict-free 16-byte reads down a column of rows
  constexpr int VROW = TK + 4;
  constexpr int UPR = HD / EPV;                     // 16-byte units per K/V row
  __shared__ __align__(16) T Ks[TK * KROW];
  __shared__ __align__(16) T VTs[HD * VROW];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, cq = lane & 15, g = lane >> 4;
  const int qb = (int)gridDim.x - 1 - (int)blockIdx.x;   // blocks with the most tiles start first
  const int h = blockIdx.y, c = h / G;
  const int row = qb * 64 + wave * 16 + cq;
  const bool rowok = row < M;
  const int qpos = pos0 + row;
  const T* kbase = kc + (size_t)c * max_seq * HD;
  const T* vbase = vc + (size_t)c * max_seq * HD;
  typename AT<T>::Op qop[KS];
  {
    const T* qp = q + (size_t)(rowok ? row : 0) * qd + h * HD + 8 * g;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) qop[ks] = AT<T>::ld8(qp + 32 * ks);
  }
  f32x4 oacc[DB];
#pragma unroll
  for (int db = 0; db < DB; ++db) oacc[db] = f32x4{0.f, 0.f, 0.f, 0.f};
  float mrun = -INFINITY, lrun = 0.f;
  const int last_row = qb * 64 + 63 < M - 1 ? qb * 64 + 63 : M - 1;
  const int nt = (pos0 + last_row) / TK + 1;
  const int written = pos0 + M;                     // cache positions [0, written) hold this layer's K and V
  const int wave_last = pos0 + qb * 64 + wave * 16 + 15;
  for (int t = 0; t < nt; ++t) {
    const int kp0 = t * TK;
    __syncthreads();
    for (int u = tid; u < TK * UPR; u += 256) {
      const int key = u / UPR, part = u - key * UPR;
      const int kp = kp0 + key;
      uint4 v = make_uint4(0u, 0u, 0u, 0u);
      if (kp < written) v = *reinterpret_cast<const uint4*>(kbase + (size_t)kp * HD + part * EPV);
      *reinterpret_cast<uint4*>(Ks + key * KROW + part * EPV) = v;
    }
    for (int u = tid; u < TK * UPR; u += 256) {
      const int part = u / TK, key = u - part * TK;
      const int kp = kp0 + key;
      uint4 v = make_uint4(0u, 0u, 0u, 0u);            // zeros past the end: 0 * (stale bits) must not give NaN
      if (kp < written) v = *reinterpret_cast<const uint4*>(vbase + (size_t)kp * HD + part * EPV);
      AT<T>::scatter(VTs + (part * EPV) * VROW + key, VROW, v);
    }
    __syncthreads();
    if (kp0 > wave_last) continue;                  // wholly in this wave's future (the barriers above still match)
    f32x4 s[KB16];
#pragma unroll
    for (int kb = 0; kb < KB16; ++kb) {
      s[kb] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int ks = 0; ks < KS; ++ks)
        AT<T>::mma(s[kb], AT<T>::ld8(Ks + (kb * 16 + cq) * KROW + 32 * ks + 8 * g), qop[ks]);
    }
    float sv[KB16][4];
    float mx = -INFINITY;
#pragma unroll
    for (int kb = 0; kb < KB16; ++kb) {
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int kp = kp0 + kb * 16 + 4 * g + j;
        sv[kb][j] = kp <= qpos ? s[kb][j] * scale : -INFINITY;
        mx = fmaxf(mx, sv[kb][j]);
      }
    }
    mx = fmaxf(mx, __shfl_xor(mx, 16));
    mx = fmaxf(mx, __shfl_xor(mx, 32));
    const float mnew = fmaxf(mrun, mx);
    const float alpha = mrun == -INFINITY ? 0.f : expf(mrun - mnew);
    float psum = 0.f;
#pragma unroll
    for (int kb = 0; kb < KB16; ++kb) {
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        sv[kb][j] = sv[kb][j] == -INFINITY ? 0.f : expf(sv[kb][j] - mnew);
        psum += sv[kb][j];
      }
    }
    psum += __shfl_xor(psum, 16);
    psum += __shfl_xor(psum, 32);
    lrun = lrun * alpha + psum;
    mrun = mnew;
#pragma unroll
    for (int db = 0; db < DB; ++db) {
      oacc[db][0] *= alpha; oacc[db][1] *= alpha; oacc[db][2] *= alpha; oacc[db][3] *= alpha;
    }
#pragma unroll
    for (int hf = 0; hf < HF; ++hf) {
      const float pp[8] = {sv[2 * hf][0], sv[2 * hf][1], sv[2 * hf][2], sv[2 * hf][3],
                           sv[2 * hf + 1][0], sv[2 * hf + 1][1], sv[2 * hf + 1][2], sv[2 * hf + 1][3]};
#pragma unroll
      for (int db = 0; db < DB; ++db) {
        const T* vt = VTs + (db * 16 + cq) * VROW + 32 * hf + 4 * g;
        AT<T>::mma_p(oacc[db], AT<T>::ld44(vt, vt + 16), pp);
      }
    }
  }
  if (rowok) {
    const float inv = 1.0f / lrun;
    T* op = o + (size_t)row * qd + h * HD + 4 * g;
#pragma unroll
    for (int db = 0; db < DB; ++db) {
#pragma unroll
      for (int j = 0; j < 4; ++j) PT<T>::st(op + db * 16 + j, oacc[db][j] * inv);
    }
  }
}

template <typename T>
hipError_t launch_attn(const LsPfParams& p, int layer, int pos0, int M, hipStream_t s) {
  const int nq = p.qd / p.hd, G = nq / p.nkv;
  const size_t lofs = (size_t)layer * p.nkv * p.max_seq * p.hd;
  const T* kc = static_cast<const T*>(p.kcache) + lofs;
  const T* vc = static_cast<const T*>(p.vcache) + lofs;
  const float scale = (float)(1.0 / sqrt((double)p.hd));
  dim3 grid((M + 63) / 64, nq);
  if (p.hd == 128)
    pf_attn_kernel<T, 128><<<grid, dim3(256), 0, s>>>(static_cast<const T*>(p.q_pf), static_cast<T*>(p.o_pf), kc, vc, M, pos0, p.qd, G, p.max_seq, scale);
  else
    pf_attn_kernel<T, 64><<<grid, dim3(256), 0, s>>>(static_cast<const T*>(p.q_pf), static_cast<T*>(p.o_pf), kc, vc, M, pos0, p.qd, G, p.max_seq, scale);
  return hipGetLastError();
}

template <typename T>
int run_layers(const LsPfParams& p, const LsLayerW* lw, int pos0, int M, hipStream_t s) {
  const int dm = p.dm, qd = p.qd, kvd = p.kvd, ffn = p.ffn;
  pf_embed_kernel<T><<<dim3(M), dim3(256), 0, s>>>(p.tokens + pos0, static_cast<const T*>(p.embed), p.x_pf, dm, p.vocab);
  for (int l = 0; l < p.layers_used; ++l) {
    const LsLayerW& W = lw[l];
    pf_rmsnorm_kernel<T><<<dim3(M), dim3(256), 0, s>>>(p.x_pf, static_cast<const T*>(W.attn_norm), static_cast<T*>(p.a_pf), dm, p.eps);
    PfGemm g{};
    g.A = p.a_pf; g.lda = dm; g.M = M; g.K = dm; g.hd = p.hd; g.pos0 = pos0; g.max_seq = p.max_seq; g.nkv = p.nkv;
    g.layer = l; g.rope_cos = p.rope_cos; g.rope_sin = p.rope_sin; g.tile_rows = p.tile_rows;
    g.W = W.wq; g.N = qd; g.out = p.q_pf; g.ldo = qd;
    bool fused = false;
    if (qd % BN == 0 && kvd % BN == 0) {
      // one launch for the three projections, when it would run on the large tiles anyway
      PfGemm f = g;
      f.W2 = W.wk; f.W3 = W.wv; f.N = qd + 2 * kvd; f.N_q = qd; f.N_kv = kvd; f.out_k = p.kcache; f.out_v = p.vcache;
      if (!use_small_tiles(f) && !use_small_tiles(g)) {
        if (launch_gemm<T, EPI_QKV>(f, s) != hipSuccess) return 1;
        fused = true;
      }
    }
    if (!fused) {
      if (launch_gemm<T, EPI_ROPE_Q>(g, s) != hipSuccess) return 1;
      g.W = W.wk; g.N = kvd; g.out = p.kcache;
      if (launch_gemm<T, EPI_ROPE_K>(g, s) != hipSuccess) return 1;
      g.W = W.wv; g.N = kvd; g.out = p.vcache;
      if (launch_gemm<T, EPI_V>(g, s) != hipSuccess) return 1;
    }
    if (launch_attn<T>(p, l, pos0, M, s) != hipSuccess) return 1;
    g.A = p.o_pf; g.lda = qd; g.K = qd; g.W = W.wo; g.N = dm; g.x = p.x_pf; g.capture = nullptr;
    if (launch_gemm<T, EPI_RESID>(g, s) != hipSuccess) return 1;
    pf_rmsnorm_kernel<T><<<dim3(M), dim3(256), 0, s>>>(p.x_pf, static_cast<const T*>(W.ffn_norm), static_cast<T*>(p.a_pf), dm, p.eps);
    g.A = p.a_pf; g.lda = dm; g.K = dm; g.W = W.wg; g.W2 = W.wu; g.N = ffn; g.out = p.act_pf; g.ldo = ffn;
    if (launch_gemm<T, EPI_GU>(g, s) != hipSuccess) return 1;
    g.A = p.act_pf; g.lda = ffn; g.K = ffn; g.W = W.wd; g.W2 = nullptr; g.N = dm; g.x = p.x_pf;
    g.capture = p.capture ? p.capture + (size_t)l * p.max_seq * dm : nullptr;
    if (launch_gemm<T, EPI_RESID>(g, s) != hipSuccess) return 1;
  }
  return hipGetLastError() == hipSuccess ? 0 : 1;
}

}  // namespace

// Runs layers 0..layers_used-1 over rows [pos0, pos0+M) of the prompt (M <= pf_rows).
extern "C" int ls_prefill_layers(const LsPfParams* p, const LsLayerW* host_layers, int pos0, int M, hipStream_t s) {
  return p->is_bf16 ? run_layers<bf16_t>(*p, host_layers, pos0, M, s) : run_layers<float>(*p, host_layers, pos0, M, s);
}

extern "C" int ls_prefill_finish(const LsPfParams* p, int last_row, hipStream_t s) {
  pf_finish_kernel<<<dim3(1), dim3(256), 0, s>>>(p->x_pf + (size_t)last_row * p->dm, p->xbuf, p->ssq, p->dm, p->ssq_nt);
  return hipGetLastError() == hipSuccess ? 0 : 1;
}
