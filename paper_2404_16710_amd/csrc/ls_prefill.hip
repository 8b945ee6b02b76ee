// Prompt pass (prefill) for gfx950: all rows of the prompt go through each layer together, so the
// projections are real GEMMs (M = prompt rows) on the MFMA units instead of 16-row passes that
// re-read every weight.  Per layer:
//   RMSNorm -> Q/K/V GEMMs (+RoPE, KV append) -> causal attention (the decode attention stage, in
//   blocks of query rows over the shared cache) -> O GEMM (+residual) -> RMSNorm ->
//   gate/up GEMM (+SwiGLU) -> down GEMM (+residual).
// Rounding points are the ones of the decode path: RMSNorm output, q/k after RoPE, v, the
// attention output and the SwiGLU output are stored in the model dtype; the residual stream and
// all accumulation are fp32.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <math.h>

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

// The last prompt row goes to row 0 of the decode residual buffer, with the sums of squares per
// gs columns its RMSNorm needs; the head then runs in the decode kernel.
__global__ __launch_bounds__(256) void pf_finish_kernel(const float* xrow, float* xbuf, float* ssq, int dm, int gs) {
  for (int t = threadIdx.x; t * gs < dm; t += 256) {
    float s = 0.f;
    for (int j = 0; j < gs && t * gs + j < dm; ++j) { const float v = xrow[t * gs + j]; xbuf[t * gs + j] = v; s += v * v; }
    ssq[t] = s;
  }
}

// ------------------------------------------------------------------------------------------
enum { EPI_ROPE_Q = 0, EPI_ROPE_K = 1, EPI_V = 2, EPI_RESID = 3, EPI_GU = 4 };

struct PfGemm {
  const void* A;    // [M][K] activations (model dtype), row stride lda
  int lda;
  const void* W;    // [N][K] weights
  const void* W2;   // second weight matrix (gate/up: W = gate, W2 = up)
  int M, N, K;
  void* out;        // q rows [M][ldo] / SwiGLU rows [M][ldo] (model dtype); KV cache base for K, V
  int ldo;
  float* x;         // residual rows [M][N] fp32 (EPI_RESID)
  float* capture;   // optional copy of the new residual rows, [max_seq][N] of this layer
  const float* rope_cos; const float* rope_sin;
  int hd, pos0, max_seq, nkv, layer;
};

constexpr int BM = 128, BN = 128;
constexpr int ROWB = 128;          // bytes of K per tile row
constexpr int ROWP = ROWB + 16;    // padded LDS row

template <typename T, int EPI>
__global__ __launch_bounds__(256) void pf_gemm_kernel(const PfGemm g) {
  constexpr int EPV = PT<T>::EPV;
  constexpr int BK = ROWB / (int)sizeof(T);
  constexpr int NW = (EPI == EPI_GU) ? 2 : 1;
  __shared__ __align__(16) char As[BM * ROWP];
  __shared__ __align__(16) char Ws[NW][BN * ROWP];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int r = lane & 15, gq = lane >> 4;
  const int n0 = blockIdx.x * BN, m0 = blockIdx.y * BM;
  const T* Ag = static_cast<const T*>(g.A);
  const T* Wg[2] = {static_cast<const T*>(g.W), static_cast<const T*>(g.W2)};

  f32x4 acc[NW][2][8];
#pragma unroll
  for (int w = 0; w < NW; ++w)
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int j = 0; j < 8; ++j) acc[w][i][j] = f32x4{0.f, 0.f, 0.f, 0.f};

  uint4 ra[4], rw[NW][4];
  auto gload = [&](int k0) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int unit = tid + 256 * i, row = unit >> 3, u = unit & 7;
      const int k = k0 + u * EPV;
      const bool kok = k < g.K;
      const int ma = m0 + row, na = n0 + row;
      const bool aok = kok && ma < g.M, wok = kok && na < g.N;
      const uint4 va = *reinterpret_cast<const uint4*>(Ag + (size_t)(aok ? ma : 0) * g.lda + (aok ? k : 0));
      ra[i] = aok ? va : make_uint4(0, 0, 0, 0);
#pragma unroll
      for (int w = 0; w < NW; ++w) {
        const uint4 vw = *reinterpret_cast<const uint4*>(Wg[w] + (size_t)(wok ? na : 0) * g.K + (wok ? k : 0));
        rw[w][i] = wok ? vw : make_uint4(0, 0, 0, 0);
      }
    }
  };
  auto lstore = [&]() {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int unit = tid + 256 * i, row = unit >> 3, u = unit & 7;
      *reinterpret_cast<uint4*>(As + row * ROWP + u * 16) = ra[i];
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
      uint4 fa[2];
#pragma unroll
      for (int i = 0; i < 2; ++i)
        fa[i] = *reinterpret_cast<const uint4*>(As + (wave * 32 + i * 16 + r) * ROWP + (s * 4 + gq) * 16);
#pragma unroll
      for (int w = 0; w < NW; ++w) {
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          const uint4 fb = *reinterpret_cast<const uint4*>(Ws[w] + (j * 16 + r) * ROWP + (s * 4 + gq) * 16);
#pragma unroll
          for (int i = 0; i < 2; ++i) PT<T>::mma(acc[w][i][j], fa[i], fb);
        }
      }
    }
  }

  // epilogue: the lane holds rows m = base + 4*gq + jj (jj = 0..3) of column n = n0 + 16*j + r
  const int half = g.hd / 2;
#pragma unroll
  for (int i = 0; i < 2; ++i) {
#pragma unroll
    for (int jj = 0; jj < 4; ++jj) {
      const int m = m0 + wave * 32 + i * 16 + 4 * gq + jj;
      if (m >= g.M) continue;
      const int pos = g.pos0 + m;
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const int n = n0 + 16 * j + r;
        if (n >= g.N) continue;
        const float v = acc[0][i][j][jj];
        if (EPI == EPI_RESID) {
          float* xr = g.x + (size_t)m * g.N + n;
          const float nv = *xr + v;
          *xr = nv;
          if (g.capture != nullptr) g.capture[(size_t)pos * g.N + n] = nv;
        } else if (EPI == EPI_GU) {
          const float up = acc[NW - 1][i][j][jj];
          PT<T>::st(static_cast<T*>(g.out) + (size_t)m * g.ldo + n, (v / (1.0f + expf(-v))) * up);
        } else if (EPI == EPI_V) {
          const int h = n / g.hd, d = n - h * g.hd;
          PT<T>::st(static_cast<T*>(g.out) + (((size_t)g.layer * g.nkv + h) * g.max_seq + pos) * g.hd + d, v);
        } else {
          // rotation mixes columns d and d + hd/2 of one head; both sit in this lane (tile j and j + half/16)
          const int h = n / g.hd, d = n - h * g.hd;
          if (d < half) {
            // partner tile: 4 tiles on for head_dim 128, 2 tiles on for head_dim 64 (static indices)
            const float b = (g.hd == 128) ? acc[0][i][(j + 4) & 7][jj] : acc[0][i][(j + 2) & 7][jj];
            const float c = g.rope_cos[(size_t)pos * half + d], s = g.rope_sin[(size_t)pos * half + d];
            const float lo = v * c - b * s, hi = b * c + v * s;
            if (EPI == EPI_ROPE_Q) {
              T* dst = static_cast<T*>(g.out) + (size_t)m * g.ldo + h * g.hd;
              PT<T>::st(dst + d, lo);
              PT<T>::st(dst + d + half, hi);
            } else {
              T* dst = static_cast<T*>(g.out) + (((size_t)g.layer * g.nkv + h) * g.max_seq + pos) * g.hd;
              PT<T>::st(dst + d, lo);
              PT<T>::st(dst + d + half, hi);
            }
          }
        }
      }
    }
  }
}

template <typename T, int EPI>
hipError_t launch_gemm(const PfGemm& g, hipStream_t s) {
  dim3 grid((g.N + BN - 1) / BN, (g.M + BM - 1) / BM);
  pf_gemm_kernel<T, EPI><<<grid, dim3(256), 0, s>>>(g);
  return hipGetLastError();
}

template <typename T>
int run_layers(const LsPfParams& p, const LsLayerW* lw, int pos0, int M, hipStream_t s,
               int (*attn)(void*, int, int, int, hipStream_t), void* attn_ctx) {
  const int dm = p.dm, qd = p.qd, kvd = p.kvd, ffn = p.ffn;
  pf_embed_kernel<T><<<dim3(M), dim3(256), 0, s>>>(p.tokens + pos0, static_cast<const T*>(p.embed), p.x_pf, dm, p.vocab);
  for (int l = 0; l < p.layers_used; ++l) {
    const LsLayerW& W = lw[l];
    pf_rmsnorm_kernel<T><<<dim3(M), dim3(256), 0, s>>>(p.x_pf, static_cast<const T*>(W.attn_norm), static_cast<T*>(p.a_pf), dm, p.eps);
    PfGemm g{};
    g.A = p.a_pf; g.lda = dm; g.M = M; g.K = dm; g.hd = p.hd; g.pos0 = pos0; g.max_seq = p.max_seq; g.nkv = p.nkv;
    g.layer = l; g.rope_cos = p.rope_cos; g.rope_sin = p.rope_sin;
    g.W = W.wq; g.N = qd; g.out = p.q_pf; g.ldo = qd;
    if (launch_gemm<T, EPI_ROPE_Q>(g, s) != hipSuccess) return 1;
    g.W = W.wk; g.N = kvd; g.out = p.kcache;
    if (launch_gemm<T, EPI_ROPE_K>(g, s) != hipSuccess) return 1;
    g.W = W.wv; g.N = kvd; g.out = p.vcache;
    if (launch_gemm<T, EPI_V>(g, s) != hipSuccess) return 1;
    if (attn(attn_ctx, l, pos0, M, s) != 0) return 1;
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

// Runs layers 0..layers_used-1 over rows [pos0, pos0+M) of the prompt (M <= pf_rows).  `attn` is
// called once per layer to enqueue the attention of those rows (q rows in q_pf, output to o_pf).
extern "C" int ls_prefill_layers(const LsPfParams* p, const LsLayerW* host_layers, int pos0, int M, hipStream_t s,
                                 int (*attn)(void*, int, int, int, hipStream_t), void* attn_ctx) {
  return p->is_bf16 ? run_layers<bf16_t>(*p, host_layers, pos0, M, s, attn, attn_ctx)
                    : run_layers<float>(*p, host_layers, pos0, M, s, attn, attn_ctx);
}

extern "C" int ls_prefill_finish(const LsPfParams* p, int last_row, hipStream_t s) {
  pf_finish_kernel<<<dim3(1), dim3(256), 0, s>>>(p->x_pf + (size_t)last_row * p->dm, p->xbuf, p->ssq, p->dm, p->gs_x);
  return hipGetLastError() == hipSuccess ? 0 : 1;
}
