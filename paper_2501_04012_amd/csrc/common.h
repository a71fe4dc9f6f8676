// Shared device/host helpers of the denoising library (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>

namespace fc {

typedef __bf16 bf16_t;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;

constexpr int kWave = 64;

__device__ __forceinline__ float to_f32(float v) { return v; }
__device__ __forceinline__ float to_f32(bf16_t v) { return (float)v; }
template <typename T> __device__ __forceinline__ T from_f32(float v);
template <> __device__ __forceinline__ float from_f32<float>(float v) { return v; }
template <> __device__ __forceinline__ bf16_t from_f32<bf16_t>(float v) { return (bf16_t)v; }

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}

__device__ __forceinline__ float silu_f(float v) { return v / (1.0f + __expf(-v)); }

// GELU, tanh form: 0.5 v (1 + tanh(u)) = v / (1 + exp(-2u)), u = c (v + 0.044715 v^3).
// One exp2 and one reciprocal (hardware approximations, about 1 ulp; the callers round
// to bf16 or compare at 1e-4); finite at both ends: exp2 -> inf gives v * 0.
__device__ __forceinline__ float gelu_tanh_f(float v) {
  const float k1 = -2.0f * 0.7978845608028654f * 1.4426950408889634f;   // -2 c log2(e)
  const float k2 = k1 * 0.044715f;
  const float e = __builtin_amdgcn_exp2f(v * __builtin_fmaf(v * v, k2, k1));
  return v * __builtin_amdgcn_rcpf(1.0f + e);
}

inline int ceil_div(long long a, long long b) { return (int)((a + b - 1) / b); }
inline size_t round_up(size_t a, size_t b) { return (a + b - 1) / b * b; }

// ---------------------------------------------------------------- GEMM epilogues
// Two interfaces, one arithmetic.
//  * Column form (plain kernel, and the MFMA kernel for EPI_UNPATCH): four consecutive
//    rows (m0..m0+3) of one column n; column-only quantities are hoisted into a `Col`.
//  * Row-run form (MFMA kernel, every mode whose output rows are contiguous along n):
//    `apply4` turns four consecutive columns of one row into final values (bias,
//    activation, gate or q scale), `run8` gives the address of eight consecutive outputs
//    of a row, which the kernel writes with one 16-byte store.
// `Mvalid` bounds rows, `Nvalid` bounds columns.

enum EpiMode : int {
  EPI_STORE = 0,     // out[m,n] = acc + bias
  EPI_GELU = 1,      // out[m,n] = gelu(acc + bias)
  EPI_GATE = 2,      // out[m,n] = gate[n] * (acc + bias)    (gate NULL: 1); the residual add is the next LN's
  EPI_HEADS = 3,     // scatter into per-head q / k / v tensors
  EPI_UNPATCH = 4    // scatter token rows back into a latent-shaped fp32 tensor
};

struct EpiParams {
  const float* bias = nullptr;   // [N]
  void* out = nullptr;           // EPI_STORE / EPI_GELU / EPI_GATE: act [M, ldo]
  int ldo = 0;
  const float* gate = nullptr;   // EPI_GATE: [N] or NULL
  // EPI_HEADS: column n -> which = which0 + n / D (0 q, 1 k, 2 v), head = (n % D) / hd.
  // Row m -> (b, tok) = (m / tokens, m % tokens).
  // q, k, v: [b, head, tok, hd].
  // Queries are stored multiplied by qscale (softmax scale * log2 e), in fp32 before rounding.
  void* q = nullptr; void* k = nullptr; void* v = nullptr;
  int which0 = 0, D = 0, heads = 0, hd = 0, tokens = 0;
  float qscale = 1.0f;
  // EPI_UNPATCH: row m -> (b, t, h', w'), column f -> (dh, dw, c); eps [b, T, H, W, C]
  float* eps = nullptr;
  int T = 0, H = 0, W = 0, C = 0, p = 0;
};

// Division of a row index by a runtime constant without an integer divide:
// q = (m * mul) >> 40 with mul = ceil(2^40 / d) is exact while m * d < 2^40.
struct FastDiv {
  unsigned long long mul = 0;
  unsigned d = 1;
  FastDiv() = default;
  explicit FastDiv(unsigned div) : mul(((1ull << 40) + div - 1) / div), d(div) {}
  __device__ __forceinline__ unsigned div(unsigned m) const { return (unsigned)(((unsigned long long)m * mul) >> 40); }
};

template <typename T, int MODE>
struct Epilogue {
  EpiParams P;
  int Mvalid, Nvalid;
  FastDiv rows_per_b;          // EPI_HEADS: tokens;  EPI_UNPATCH: T*S
  FastDiv unp_S, unp_gw;       // EPI_UNPATCH
  FastDiv col_D, col_hd;       // EPI_HEADS, row-run form
  static constexpr bool kRowRuns = MODE != EPI_UNPATCH;
  static constexpr bool kLinearOut = MODE == EPI_STORE || MODE == EPI_GELU || MODE == EPI_GATE;   // out[m * ldo + n]
  static constexpr bool kHasGate = MODE == EPI_GATE;

  // host side: fills the divisors the mode needs
  static Epilogue make(const EpiParams& p, int M, int N) {
    Epilogue e{p, M, N, FastDiv(), FastDiv(), FastDiv(), FastDiv(), FastDiv()};
    if (MODE == EPI_HEADS) {
      e.rows_per_b = FastDiv((unsigned)p.tokens);
      e.col_D = FastDiv((unsigned)p.D);
      e.col_hd = FastDiv((unsigned)p.hd);
    }
    if (MODE == EPI_UNPATCH) {
      const int gw = p.W / p.p, S = gw * (p.H / p.p);
      e.rows_per_b = FastDiv((unsigned)(p.T * S));
      e.unp_S = FastDiv((unsigned)S);
      e.unp_gw = FastDiv((unsigned)gw);
    }
    return e;
  }

  // Everything that depends on the output column only, computed once per column.
  struct Col {
    float bias, mul;           // mul: gate (EPI_GATE) or q scale (EPI_HEADS)
    T* base;                   // column base pointer (EPI_UNPATCH: nullptr, see foff)
    size_t foff;               // EPI_UNPATCH: offset of (dh, dw, c) inside a patch origin
    bool valid;
  };

  __device__ __forceinline__ Col col(int n) const {
    Col c;
    c.valid = n < Nvalid;
    const int nn = c.valid ? n : 0;
    c.bias = P.bias ? P.bias[nn] : 0.0f;
    c.mul = 1.0f;
    c.base = nullptr;
    c.foff = 0;
    if constexpr (MODE == EPI_STORE || MODE == EPI_GELU || MODE == EPI_GATE) {
      c.base = (T*)P.out + nn;
      if constexpr (MODE == EPI_GATE) c.mul = P.gate ? P.gate[nn] : 1.0f;
    } else if constexpr (MODE == EPI_HEADS) {
      const int which = P.which0 + nn / P.D;
      const int cc = nn % P.D;
      const int head = cc / P.hd, dd = cc % P.hd;
      c.base = (T*)(which == 0 ? P.q : which == 1 ? P.k : P.v) + (size_t)head * P.tokens * P.hd + dd;
      c.mul = which == 0 ? P.qscale : 1.0f;
    } else if constexpr (MODE == EPI_UNPATCH) {
      const int dh = nn / (P.p * P.C), dw = (nn / P.C) % P.p, ch = nn % P.C;
      c.foff = ((size_t)dh * P.W + dw) * P.C + ch;
    }
    return c;
  }

  // Row-run form.  Preconditions (checked by the dispatcher): Nvalid, ldo, hd and D are
  // multiples of 8; bias, gate and the output tensors are 16-byte aligned.
  // v: accumulators of columns n0..n0+3 (n0 % 4 == 0) of one row -> final values.
  // lbias / lgate: LDS copies of bias[n0..] and gate[n0..] (the tile's slices; garbage-free
  // for columns past Nvalid, which are never stored).
  // (a kernel without a bias or a gate keeps zeros or ones in the LDS copies: no branch here,
  // so that the reads of a whole pass can be issued together)
  __device__ __forceinline__ void apply4(int n0, float (&v)[4], const float* lbias, const float* lgate) const {
    {
      const f32x4 b = *(const f32x4*)lbias;
#pragma unroll
      for (int e = 0; e < 4; ++e) v[e] += b[e];
    }
    if constexpr (MODE == EPI_GELU) {
#pragma unroll
      for (int e = 0; e < 4; ++e) v[e] = gelu_tanh_f(v[e]);
    } else if constexpr (MODE == EPI_GATE) {
      {
        const f32x4 g = *(const f32x4*)lgate;
#pragma unroll
        for (int e = 0; e < 4; ++e) v[e] *= g[e];
      }
    } else if constexpr (MODE == EPI_HEADS) {
      const float sc = (P.which0 + (int)col_D.div((unsigned)n0) == 0) ? P.qscale : 1.0f;
#pragma unroll
      for (int e = 0; e < 4; ++e) v[e] *= sc;
    }
  }
  // Row-major outputs: address of (m, n) for wave-uniform m and n
  __device__ __forceinline__ T* row_ptr(int m, int n) const { return (T*)P.out + (size_t)m * P.ldo + n; }
  // EPI_HEADS, the two halves of run8: the column's part of the address (tensor, head, offset in
  // the head: fixed for a lane over a whole tile when its column is) and the row's part.
  __device__ __forceinline__ T* head_col_ptr(int n0) const {
    const unsigned w = col_D.div((unsigned)n0), cc = (unsigned)n0 - w * col_D.d;
    const unsigned head = col_hd.div(cc), dd = cc - head * col_hd.d;
    const int which = P.which0 + (int)w;
    T* base = (T*)(which == 0 ? P.q : which == 1 ? P.k : P.v);
    return base + (size_t)head * P.tokens * P.hd + dd;
  }
  __device__ __forceinline__ size_t head_row_off(int m) const {
    const unsigned bb = rows_per_b.div((unsigned)m);
    return ((size_t)m + (size_t)bb * (P.heads - 1) * P.tokens) * P.hd;
  }
  // Address of outputs (m, n0 .. n0+7), n0 % 8 == 0: one 16-byte run in every row-run mode.
  __device__ __forceinline__ T* run8(int m, int n0) const {
    if constexpr (MODE == EPI_HEADS) {
      const unsigned w = col_D.div((unsigned)n0), cc = (unsigned)n0 - w * col_D.d;
      const unsigned head = col_hd.div(cc), dd = cc - head * col_hd.d;
      const int which = P.which0 + (int)w;
      const unsigned bb = rows_per_b.div((unsigned)m);
      T* base = (T*)(which == 0 ? P.q : which == 1 ? P.k : P.v);
      return base + ((size_t)head * P.tokens + (size_t)m + (size_t)bb * (P.heads - 1) * P.tokens) * P.hd + dd;
    } else {
      return (T*)P.out + (size_t)m * P.ldo + n0;
    }
  }

  // Four consecutive rows m0..m0+3 of column c (the unit of the 32x32 MFMA accumulator).
  __device__ __forceinline__ void store4(const Col& c, int m0, const float (&acc)[4]) const {
    if (!c.valid || m0 >= Mvalid) return;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const int m = m0 + e;
      if (m >= Mvalid) break;
      float v = acc[e] + c.bias;
      if constexpr (MODE == EPI_GELU) v = gelu_tanh_f(v);
      if constexpr (MODE == EPI_GATE || MODE == EPI_HEADS) v *= c.mul;
      if constexpr (MODE == EPI_STORE || MODE == EPI_GELU || MODE == EPI_GATE) {
        c.base[(size_t)m * P.ldo] = from_f32<T>(v);
      } else if constexpr (MODE == EPI_HEADS) {
        // row (bb, tok) of [b, head, tok, hd]: offset (m + bb*(heads-1)*tokens) * hd
        const unsigned bb = rows_per_b.div((unsigned)m);
        c.base[((size_t)m + (size_t)bb * (P.heads - 1) * P.tokens) * P.hd] = from_f32<T>(v);
      } else if constexpr (MODE == EPI_UNPATCH) {
        const unsigned bb = rows_per_b.div((unsigned)m);
        const unsigned r = (unsigned)m - bb * rows_per_b.d;
        const unsigned t = unp_S.div(r), sidx = r - t * unp_S.d;
        const unsigned hp = unp_gw.div(sidx), wp = sidx - hp * unp_gw.d;
        const size_t origin = ((((size_t)bb * P.T + t) * P.H + hp * P.p) * P.W + wp * P.p) * P.C;
        P.eps[origin + c.foff] = v;
      }
    }
  }
};

// ---------------------------------------------------------------- attention problem description
// One problem = one (batch row b, head, group g).  Query i of the problem is token
// g*q_gstride + i*q_istride of batch row b; key j likewise with the k_* strides.
//   q  [B, heads, q_tokens, hd]     k, v [KB, heads, k_tokens, hd]
//   out[B, q_tokens, heads*hd]      (token-major, heads concatenated)
// Keys of batch row b come from key batch kb = b < kv_split ? b : kv_split when
// kv_shared_tail is set (guidance rows share one 'null' text), else kb = b.
struct AttnParams {
  const void* q; const void* k; const void* v; void* out;
  int B, heads, hd;
  int groups, nq, nk;
  int q_tokens, q_gstride, q_istride;
  int k_tokens, k_gstride, k_istride;
  int kv_split, kv_shared_tail;
  float scale_log2;   // factor still to be applied to q.k: scale*log2(e), or 1 if q already carries it
  // Optional (bf16 flash kernel, long key sequences): [KB, heads, kKeyNormChunks] partial maxima of
  // the key rows' Euclidean norms, from launch_key_norm_max.  With them a query's scores are
  // bounded by |q| max|k| and the kernel can drop the per-tile maximum (see k_attn_flash).
  const float* key_norm_max;
};
constexpr int kKeyNormChunks = 32;

// ---------------------------------------------------------------- launchers (defined in the .hip files)
hipError_t launch_convert_f32(const float* in, void* out, size_t n, int to_bf16, hipStream_t s);
hipError_t launch_transpose_convert(const float* in, void* out, int rows, int cols, int to_bf16, hipStream_t s);
hipError_t launch_act_to_f32_rows(int bf16, const void* in, float* out, int rows, int D,
                                  int in_rows_per_b, int out_rows_per_b, int out_row_off,
                                  int in_b_split, int in_shared_tail, hipStream_t s);
hipError_t launch_sinusoid(float t, int dim, float* out, hipStream_t s);
hipError_t launch_gemv(int bf16, const float* in, int K, const void* Wt, const float* bias, float* out, int N,
                       int in_silu, int out_silu, int layers, size_t w_layer_stride, size_t b_layer_stride,
                       size_t out_layer_stride, hipStream_t s, const void* Wt2 = nullptr,
                       const float* bias2 = nullptr, float* out2 = nullptr, int N2 = 0);
hipError_t launch_patch_embed(const float* latent, int R, int B, const float* Wp, const float* bp,
                              const float* pos_sp, const float* pos_t, float* x, int T, int H, int W, int C,
                              int p, int D, int rows_per_b, int row_off, int impl, hipStream_t s);
hipError_t launch_ln_modulate(int bf16, float* x, const void* y, const float* gate, const void* y2,
                              const float* gate2, const float* shift, const float* scale, void* out, int rows, int D,
                              float eps, int in_rows_per_b, int out_rows_per_b, int in_row_off, int alt_rows,
                              int alt_off, int write_x, hipStream_t s);
hipError_t launch_cfg_ddim(float* x, const float* eps_c, const float* eps_u, float* eps_out, size_t n,
                           float gscale, float c0, float c1, float c2, float c3, hipStream_t s);
hipError_t launch_cfg_ddim_noise(float* x, const float* eps_c, const float* eps_u, float* eps_out, size_t per_request,
                                 int requests, float gscale, float c0, float c1, float c2, float c3, float sigma,
                                 unsigned long long seed, int step, hipStream_t s);
// scratch (optional, dev, 16-byte aligned): memory the product may use for split-K partial tiles
// (fp32, at most 64 MB); without it every tile is computed whole
hipError_t launch_gemm(int bf16, int mode, const void* A, const void* Wt, int M, int N, int K,
                       const EpiParams& ep, hipStream_t s, void* scratch = nullptr, size_t scratch_bytes = 0);
hipError_t launch_attention(int bf16, const AttnParams& p, int impl, hipStream_t s);
// out [KB * heads * kKeyNormChunks] (f32): per (key batch, head) and chunk of the k_tokens rows of
// k [KB, heads, k_tokens, hd] (bf16), the largest Euclidean row norm (0 for an empty chunk)
hipError_t launch_key_norm_max(const void* k, int KB, int heads, int k_tokens, int hd, float* out, hipStream_t s);
// true where launch_attention would make use of key_norm_max
bool attention_uses_key_norms(int bf16, const AttnParams& p);

// cache restore (cache.hip)
constexpr int kMaxCacheFrames = 256;     // frames of one entry (source codes travel as a kernel argument)
constexpr size_t kCacheReduceWsBytes = 256 * 2 * sizeof(double);
hipError_t launch_stitch(const float* x_obj, const float* x_bg, const uint8_t* m_obj, const uint8_t* m_bg, float* out,
                         long long pixels, int channels, hipStream_t s);
hipError_t launch_decompress(const float* first, const float* diff_base, float alpha, const float* extra,
                             const int* src_host, int T, long long F, float* out, hipStream_t s);
hipError_t launch_alpha(const float* first_s, const float* keys_s, const float* diff_base, int n_base, long long F,
                        float* alpha_out, double* ws, hipStream_t s);
hipError_t launch_frame_similarity(const float* frames, int T, long long F, float* sim, double* ws, hipStream_t s);
hipError_t launch_frame_similarity_static(const float* frames, int T, long long F, float* sim, hipStream_t s);
hipError_t launch_pipe_rates(const void* operands, int iters, int mode_a, int mode_b, int blocks, float* sink,
                             long long* clocks, hipStream_t s);
hipError_t launch_copy_f32(const float* in, float* out, size_t n, hipStream_t s);

}  // namespace fc
