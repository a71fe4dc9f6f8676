// HBM-bound kernels of the denoising step: dtype conversion, timestep sinusoid,
// batched GEMV (timestep MLP and adaLN modulation vectors), patch embedding,
// residual add + LayerNorm + modulate, and the fused guidance + DDIM latent update.
#include "common.h"
#include <type_traits>

namespace fc {

// ---------------------------------------------------------------- conversions
template <typename T>
__global__ void k_convert(const float* __restrict__ in, T* __restrict__ out, size_t n) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  size_t stride = (size_t)gridDim.x * blockDim.x;
  for (; i < n; i += stride) out[i] = from_f32<T>(in[i]);
}

hipError_t launch_convert_f32(const float* in, void* out, size_t n, int to_bf16, hipStream_t s) {
  if (n == 0) return hipSuccess;
  int blocks = (int)((n + 255) / 256);
  if (blocks > 65536) blocks = 65536;
  if (to_bf16) k_convert<bf16_t><<<blocks, 256, 0, s>>>(in, (bf16_t*)out, n);
  else k_convert<float><<<blocks, 256, 0, s>>>(in, (float*)out, n);
  return hipGetLastError();
}

// in [rows, cols] fp32 row-major -> out [cols, rows] (T): linear weights are kept
// [out, in] on the device so that both GEMM operands are contiguous along K.
template <typename T>
__global__ void k_transpose_convert(const float* __restrict__ in, T* __restrict__ out, int rows, int cols) {
  __shared__ float tile[32][33];
  int c0 = blockIdx.x * 32, r0 = blockIdx.y * 32;
  int tx = threadIdx.x, ty = threadIdx.y;   // 32 x 8
  for (int j = ty; j < 32; j += 8) {
    int r = r0 + j, c = c0 + tx;
    tile[j][tx] = (r < rows && c < cols) ? in[(size_t)r * cols + c] : 0.0f;
  }
  __syncthreads();
  for (int j = ty; j < 32; j += 8) {
    int c = c0 + j, r = r0 + tx;
    if (c < cols && r < rows) out[(size_t)c * rows + r] = from_f32<T>(tile[tx][j]);
  }
}

hipError_t launch_transpose_convert(const float* in, void* out, int rows, int cols, int to_bf16, hipStream_t s) {
  dim3 grid(ceil_div(cols, 32), ceil_div(rows, 32)), block(32, 8);
  if (to_bf16) k_transpose_convert<bf16_t><<<grid, block, 0, s>>>(in, (bf16_t*)out, rows, cols);
  else k_transpose_convert<float><<<grid, block, 0, s>>>(in, (float*)out, rows, cols);
  return hipGetLastError();
}

// Copy activation rows into the fp32 residual stream (text rows of the full-3D
// sequence).  Output row (b, out_row_off + r) <- input row (src_b(b), r).
template <typename T>
__global__ void k_act_to_f32_rows(const T* __restrict__ in, float* __restrict__ out, int D, int in_rows_per_b,
                                  int out_rows_per_b, int out_row_off, int in_b_split, int in_shared_tail) {
  int row = blockIdx.x;                 // over B * in_rows_per_b
  int b = row / in_rows_per_b, r = row % in_rows_per_b;
  int sb = (in_shared_tail && b >= in_b_split) ? in_b_split : b;
  const T* src = in + ((size_t)sb * in_rows_per_b + r) * D;
  float* dst = out + ((size_t)b * out_rows_per_b + out_row_off + r) * D;
  for (int c = threadIdx.x; c < D; c += blockDim.x) dst[c] = to_f32(src[c]);
}

hipError_t launch_act_to_f32_rows(int bf16, const void* in, float* out, int rows, int D, int in_rows_per_b,
                                  int out_rows_per_b, int out_row_off, int in_b_split, int in_shared_tail,
                                  hipStream_t s) {
  if (rows == 0) return hipSuccess;
  if (bf16) k_act_to_f32_rows<bf16_t><<<rows, 256, 0, s>>>((const bf16_t*)in, out, D, in_rows_per_b,
                                                           out_rows_per_b, out_row_off, in_b_split, in_shared_tail);
  else k_act_to_f32_rows<float><<<rows, 256, 0, s>>>((const float*)in, out, D, in_rows_per_b, out_rows_per_b,
                                                      out_row_off, in_b_split, in_shared_tail);
  return hipGetLastError();
}

// ---------------------------------------------------------------- timestep sinusoid
// out = [cos(t f_0..f_{h-1}) | sin(t f_0..f_{h-1})], f_i = 10000^(-i/h), h = dim/2.
// Arguments reach ~1e3 rad; the angle is formed in double so that fp32 range
// reduction does not cost accuracy.
__global__ void k_sinusoid(float t, int dim, float* __restrict__ out) {
  int half = dim / 2;
  for (int i = threadIdx.x; i < half; i += blockDim.x) {
    double f = exp(-log(10000.0) * (double)i / (double)half);
    double a = (double)t * f;
    out[i] = (float)cos(a);
    out[half + i] = (float)sin(a);
  }
}

hipError_t launch_sinusoid(float t, int dim, float* out, hipStream_t s) {
  k_sinusoid<<<1, 128, 0, s>>>(t, dim, out);
  return hipGetLastError();
}

// ---------------------------------------------------------------- GEMV
// out[l][n] = f_out( sum_k f_in(in[k]) * Wt[l][n][k] + bias[l][n] ): a wave owns NOUT
// consecutive outputs, lanes stride K with 16-byte loads, the weight loads of all NOUT
// rows of a K slice are in flight together and run one slice ahead of the arithmetic; the
// first slice is requested before the input vector is staged, so that staging (a dependent
// load, SiLU, an LDS write and a barrier) costs no memory time.  The input vector is shared by
// all layers l (the adaLN layers of every block read the same SiLU(c)); a workgroup stages it
// in LDS once, 16-byte chunk q at position q ^ ((q >> 4) & 1) so that the two chunks a lane
// reads per step (2 lane, 2 lane + 1) fall into distinct banks across 16 lanes.
// A second product on the same input (Wt2, bias2, out2, N2: one layer) can ride in the same
// launch: its workgroups follow the first product's in layer 0 of the grid.
template <typename T, int NOUT>
__global__ __launch_bounds__(256) void k_gemv(const float* __restrict__ in, int K, const T* __restrict__ Wt,
                                              const float* __restrict__ bias, float* __restrict__ out, int N, int in_silu,
                                              int out_silu, size_t w_layer_stride, size_t b_layer_stride,
                                              size_t out_layer_stride, const T* __restrict__ Wt2,
                                              const float* __restrict__ bias2, float* __restrict__ out2, int N2) {
  extern __shared__ __attribute__((aligned(16))) float s_in[];
  constexpr int V = 16 / sizeof(T);          // weights per 16-byte load
  typedef typename std::conditional<sizeof(T) == 2, bf16x8, f32x4>::type wvec;
  const bool vec = K % V == 0;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int nb1 = (N + 4 * NOUT - 1) / (4 * NOUT);            // workgroups of the first product
  int bx = blockIdx.x;
  const T* w; const float* bs; float* dst; int n_out;
  if (bx < nb1) {
    w = Wt + blockIdx.y * w_layer_stride; bs = bias + blockIdx.y * b_layer_stride;
    dst = out + blockIdx.y * out_layer_stride; n_out = N;
  } else {
    if (blockIdx.y != 0) return;
    bx -= nb1; w = Wt2; bs = bias2; dst = out2; n_out = N2;
  }
  const int n0 = (bx * 4 + wave) * NOUT;
  const bool active = n0 < n_out;                              // wave-uniform
  w += (size_t)n0 * K;
  auto fetch = [&](int k, wvec (&r)[NOUT]) {
#pragma unroll
    for (int o = 0; o < NOUT; ++o)
      if (n0 + o < n_out && k < K) r[o] = *(const wvec*)(w + (size_t)o * K + k);
  };
  wvec cur[NOUT], nxt[NOUT];
  if (active && vec) fetch(lane * V, cur);

  for (int k = threadIdx.x; k < K; k += blockDim.x) {
    float v = in[k];
    const int q = k >> 2;
    s_in[vec ? ((q ^ ((q >> 4) & 1)) << 2) + (k & 3) : k] = in_silu ? silu_f(v) : v;
  }
  __syncthreads();
  if (!active) return;
  float acc[NOUT];
#pragma unroll
  for (int o = 0; o < NOUT; ++o) acc[o] = 0.0f;
  if (vec) {
    for (int k = lane * V; k < K; k += 64 * V) {
      fetch(k + 64 * V, nxt);
      float x[V];
#pragma unroll
      for (int c = 0; c < V / 4; ++c) {
        const int q = (k >> 2) + c;
        const f32x4 xv = *(const f32x4*)(s_in + ((q ^ ((q >> 4) & 1)) << 2));
#pragma unroll
        for (int e = 0; e < 4; ++e) x[4 * c + e] = xv[e];
      }
#pragma unroll
      for (int o = 0; o < NOUT; ++o) {
        if (n0 + o < n_out) {                  // wave-uniform
#pragma unroll
          for (int e = 0; e < V; ++e) acc[o] += x[e] * (float)cur[o][e];
        }
      }
#pragma unroll
      for (int o = 0; o < NOUT; ++o) cur[o] = nxt[o];
    }
  } else {
    for (int k = lane; k < K; k += 64)
#pragma unroll
      for (int o = 0; o < NOUT; ++o)
        if (n0 + o < n_out) acc[o] += s_in[k] * to_f32(w[(size_t)o * K + k]);
  }
#pragma unroll
  for (int o = 0; o < NOUT; ++o) {
    const float a = wave_sum(acc[o]);
    if (lane == 0 && n0 + o < n_out) {
      float v = a + bs[n0 + o];
      dst[n0 + o] = out_silu ? silu_f(v) : v;
    }
  }
}

template <typename T>
static hipError_t run_gemv(const float* in, int K, const void* Wt, const float* bias, float* out, int N, int in_silu,
                           int out_silu, int layers, size_t w_layer_stride, size_t b_layer_stride,
                           size_t out_layer_stride, const void* Wt2, const float* bias2, float* out2, int N2,
                           hipStream_t s) {
  const size_t sh = ((size_t)K + 3) / 4 * 4 * sizeof(float) + 16;      // the chunk swap may touch one chunk past K
  // 8 outputs per wave where that still leaves several workgroups per CU; else 4, else one each
  const long long outs = (long long)N * layers + N2;
#define FC_GEMV(NOUT)                                                                                               \
  k_gemv<T, NOUT><<<dim3(ceil_div(N, 4 * NOUT) + ceil_div(N2, 4 * NOUT), layers), 256, sh, s>>>(                    \
      in, K, (const T*)Wt, bias, out, N, in_silu, out_silu, w_layer_stride, b_layer_stride, out_layer_stride,       \
      (const T*)Wt2, bias2, out2, N2)
  if (outs >= 8 * 4 * 2048) FC_GEMV(8);
  else if (outs >= 4 * 4 * 1024) FC_GEMV(4);
  else FC_GEMV(1);
#undef FC_GEMV
  return hipGetLastError();
}

hipError_t launch_gemv(int bf16, const float* in, int K, const void* Wt, const float* bias, float* out, int N,
                       int in_silu, int out_silu, int layers, size_t w_layer_stride, size_t b_layer_stride,
                       size_t out_layer_stride, hipStream_t s, const void* Wt2, const float* bias2, float* out2,
                       int N2) {
  if (N == 0 || layers == 0) return hipSuccess;
  if (bf16)
    return run_gemv<bf16_t>(in, K, Wt, bias, out, N, in_silu, out_silu, layers, w_layer_stride, b_layer_stride,
                            out_layer_stride, Wt2, bias2, out2, N2, s);
  return run_gemv<float>(in, K, Wt, bias, out, N, in_silu, out_silu, layers, w_layer_stride, b_layer_stride,
                         out_layer_stride, Wt2, bias2, out2, N2, s);
}

// ---------------------------------------------------------------- patch embedding
// x[b, row_off + n, :] = patch(latent[b % R], n) . Wp + bp + pos_sp[s] + pos_t[t]
// with n = t*S + s, patch feature order (dh, dw, c).  K = p*p*C is tiny, so the
// kernel is bound by the write of x: a block takes TOK tokens so that Wp is read
// from L2 once per TOK rows, and each thread owns 4 consecutive columns.
constexpr int PE_TOK = 16;
__global__ void k_patch_embed(const float* __restrict__ latent, int R, const float* __restrict__ Wp,
                              const float* __restrict__ bp, const float* __restrict__ pos_sp,
                              const float* __restrict__ pos_t, float* __restrict__ x, int T, int H, int W, int C,
                              int p, int D, int rows_per_b, int row_off) {
  extern __shared__ float s_patch[];   // [PE_TOK][pd]
  const int pd = p * p * C;
  const int gw = W / p, S = (H / p) * gw, N = T * S;
  const int b = blockIdx.y;
  const int n0 = blockIdx.x * PE_TOK;
  const float* lat = latent + (size_t)(b % R) * T * H * W * C;
  for (int i = threadIdx.x; i < PE_TOK * pd; i += blockDim.x) {
    int tk = i / pd, f = i % pd;
    int n = n0 + tk;
    float v = 0.0f;
    if (n < N) {
      int t = n / S, s = n % S, hp = s / gw, wp = s % gw;
      int dh = f / (p * C), dw = (f / C) % p, c = f % C;
      v = lat[(((size_t)t * H + hp * p + dh) * W + wp * p + dw) * C + c];
    }
    s_patch[i] = v;
  }
  __syncthreads();
  for (int c0 = threadIdx.x * 4; c0 < D; c0 += blockDim.x * 4) {
    f32x4 acc[PE_TOK];
#pragma unroll
    for (int tk = 0; tk < PE_TOK; ++tk) acc[tk] = f32x4{0, 0, 0, 0};
    for (int f = 0; f < pd; ++f) {
      f32x4 w = *(const f32x4*)(Wp + (size_t)f * D + c0);
#pragma unroll
      for (int tk = 0; tk < PE_TOK; ++tk) acc[tk] += s_patch[tk * pd + f] * w;
    }
    f32x4 bias = *(const f32x4*)(bp + c0);
#pragma unroll
    for (int tk = 0; tk < PE_TOK; ++tk) {
      int n = n0 + tk;
      if (n < N) {
        int t = n / S, s = n % S;
        f32x4 ps = *(const f32x4*)(pos_sp + (size_t)s * D + c0);
        f32x4 pt = *(const f32x4*)(pos_t + (size_t)t * D + c0);
        *(f32x4*)(x + ((size_t)b * rows_per_b + row_off + n) * D + c0) = acc[tk] + bias + (ps + pt);
      }
    }
  }
}

// K = 64 as 2x2 patches of 16 channels: enough arithmetic (2 N D 64 FLOP) to keep the
// vector ALU busy for several times longer than the write of x takes, so this shape goes
// to the matrix cores.  Both fp32 operands are split into bf16 high and low parts and
// the product is taken as hi*hi + hi*lo + lo*hi (v_mfma_f32_32x32x16_bf16, fp32
// accumulation): the dropped lo*lo term is below 2^-16 of a product.
//   A operand: lane (i, h) = token i of a 32-position tile.  Patch feature order is
//   (dh, dw, c), so features 32 dh .. 32 dh + 31 of a token are one contiguous run of the
//   latent (row 2 hp + dh, pixels 2 wp and 2 wp + 1, 16 channels).  The contraction
//   order is free as long as both operands agree: lane half h takes the run dh = h, and
//   step s of 4 uses its elements 8 s .. 8 s + 7 (feature 32 h + 8 s + x); Wp rows are
//   fetched in the same order.
//   D: lane (i, h) holds column i of a 32-column tile, tokens 8 g + 4 h + e.
// A block owns 32 spatial positions and 256 columns (4 waves x 2 column tiles) and walks
// a run of (batch row, frame) pairs with its split weight fragments and bias + pos_sp in
// registers (the latter as the C operand of the first MFMA); pos_t is added at the store.
// The runs are cut so that the grid is several rounds of workgroups: a grid of slightly
// more than one round would cost two.
__device__ __forceinline__ void split_bf16(float v, bf16_t& hi, bf16_t& lo) {
  hi = (bf16_t)v;
  lo = (bf16_t)(v - (float)hi);
}

__global__ __launch_bounds__(256) void k_patch_embed_mfma(const float* __restrict__ latent, int R, int B,
                                                          const float* __restrict__ Wp, const float* __restrict__ bp,
                                                          const float* __restrict__ pos_sp,
                                                          const float* __restrict__ pos_t, float* __restrict__ x, int T,
                                                          int H, int W, int D, int rows_per_b, int row_off, int frames_per_block) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, li = lane & 31, lh = lane >> 5;
  const int gw = W / 2, S = (H / 2) * gw;
  const int s0 = blockIdx.x * 32;
  const int col0 = blockIdx.y * 256 + wave * 64;
  const int bt0 = blockIdx.z * frames_per_block;
  const int bt1 = min(bt0 + frames_per_block, B * T);
  const int s_l = s0 + li < S ? s0 + li : S - 1;          // rows past S are computed from a valid token, never stored
  const size_t a_off = ((size_t)((s_l / gw) * 2 + lh) * W + (size_t)(s_l % gw) * 2) * 16;
  f32x16 base[2];
  bf16x8 w_hi[2][4], w_lo[2][4];
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    const int col = col0 + 32 * j + li;
    const float bias = bp[col];
#pragma unroll
    for (int g = 0; g < 4; ++g)
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const int tok = s0 + 8 * g + 4 * lh + e;
        base[j][4 * g + e] = bias + pos_sp[(size_t)(tok < S ? tok : S - 1) * D + col];
      }
#pragma unroll
    for (int st = 0; st < 4; ++st)
#pragma unroll
      for (int xx = 0; xx < 8; ++xx) {
        bf16_t hi, lo;
        split_bf16(Wp[(size_t)(32 * lh + 8 * st + xx) * D + col], hi, lo);
        w_hi[j][st][xx] = hi;
        w_lo[j][st][xx] = lo;
      }
  }
  // the patch values of frame bt+1 are fetched while frame bt is multiplied and stored
  const size_t frame = (size_t)H * W * 16;
  f32x4 av[8], an[8];
#pragma unroll
  for (int q = 0; q < 8; ++q)
    an[q] = *(const f32x4*)(latent + ((size_t)((bt0 / T) % R) * T + bt0 % T) * frame + a_off + 4 * q);
  for (int bt = bt0; bt < bt1; ++bt) {
    const int b = bt / T, t = bt % T;
#pragma unroll
    for (int q = 0; q < 8; ++q) av[q] = an[q];
    if (bt + 1 < bt1) {
      const int b1 = (bt + 1) / T, t1 = (bt + 1) % T;
      const float* ap = latent + ((size_t)(b1 % R) * T + t1) * frame + a_off;
#pragma unroll
      for (int q = 0; q < 8; ++q) an[q] = *(const f32x4*)(ap + 4 * q);
    }
    f32x16 acc[2] = {base[0], base[1]};
#pragma unroll
    for (int st = 0; st < 4; ++st) {
      bf16x8 a_hi, a_lo;
#pragma unroll
      for (int xx = 0; xx < 8; ++xx) {
        bf16_t hi, lo;
        split_bf16(av[2 * st + (xx >> 2)][xx & 3], hi, lo);
        a_hi[xx] = hi;
        a_lo[xx] = lo;
      }
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a_hi, w_hi[j][st], acc[j], 0, 0, 0);
        acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a_hi, w_lo[j][st], acc[j], 0, 0, 0);
        acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a_lo, w_hi[j][st], acc[j], 0, 0, 0);
      }
    }
    // stores: a wave-uniform row pointer plus one per-lane offset (scalar address arithmetic), and
    // no per-store predicate except in the one ragged tile of a frame
    const unsigned lane_off = (unsigned)(4 * lh) * (unsigned)D + (unsigned)li;
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const float pt = pos_t[(size_t)t * D + col0 + 32 * j + li];
      float* xu = x + ((size_t)b * rows_per_b + row_off + (size_t)t * S + s0) * D + col0 + 32 * j;
      if (s0 + 32 <= S) {
#pragma unroll
        for (int g = 0; g < 4; ++g)
#pragma unroll
          for (int e = 0; e < 4; ++e) xu[(size_t)(8 * g + e) * D + lane_off] = acc[j][4 * g + e] + pt;
      } else {
#pragma unroll
        for (int g = 0; g < 4; ++g)
#pragma unroll
          for (int e = 0; e < 4; ++e)
            if (s0 + 8 * g + 4 * lh + e < S) xu[(size_t)(8 * g + e) * D + lane_off] = acc[j][4 * g + e] + pt;
      }
    }
  }
}

// impl 0: by shape; 1: general kernel; 2: matrix-core kernel (hipErrorInvalidValue if the shape does not fit it)
hipError_t launch_patch_embed(const float* latent, int R, int B, const float* Wp, const float* bp,
                              const float* pos_sp, const float* pos_t, float* x, int T, int H, int W, int C,
                              int p, int D, int rows_per_b, int row_off, int impl, hipStream_t s) {
  const int S = (H / p) * (W / p), N = T * S;
  if (N == 0 || B == 0) return hipSuccess;
  const bool mfma_fits = p == 2 && C == 16 && D % 256 == 0;
  if (impl == 2 && !mfma_fits) return hipErrorInvalidValue;
  // by shape: worth it once its grid fills the chip (every block walks all B*T frames)
  if (impl == 2 || (impl == 0 && mfma_fits && (long long)ceil_div(S, 32) * (D / 256) >= 256)) {
    const int tiles = ceil_div(S, 32) * (D / 256);
    int runs = ceil_div(2048, tiles);
    runs = runs < 1 ? 1 : (runs > B * T ? B * T : runs);
    const int fpb = ceil_div(B * T, runs);
    dim3 grid(ceil_div(S, 32), D / 256, ceil_div(B * T, fpb));
    k_patch_embed_mfma<<<grid, 256, 0, s>>>(latent, R, B, Wp, bp, pos_sp, pos_t, x, T, H, W, D, rows_per_b, row_off,
                                            fpb);
    return hipGetLastError();
  }
  dim3 grid(ceil_div(N, PE_TOK), B);
  size_t sh = (size_t)PE_TOK * p * p * C * sizeof(float);
  k_patch_embed<<<grid, 256, sh, s>>>(latent, R, Wp, bp, pos_sp, pos_t, x, T, H, W, C, p, D, rows_per_b, row_off);
  return hipGetLastError();
}

// ---------------------------------------------------------------- residual add + LayerNorm + modulate
// One wave per row, the row held in registers (NCH 16-byte chunks per lane, all loads
// issued before the first use).  If `y` is given, the pending branch output of the
// previous linear layer is folded in first: x <- x + gate * y (gate NULL = ones), and after
// it a second one, `y2` with `gate2`, if given.  The sum is written back in fp32 only if
// write_x is set: a caller that keeps y pending and passes it again with the next branch's
// output saves one write and one read of x for one more read of y (half the size), with the
// same additions in the same order; the last LayerNorm of a step never writes x.  Then
//   out = (x - mean) * rsqrt(var + eps) * (1 + scale) + shift
// with mean and centred variance as wave reductions (two passes over registers).
// Output row r reads input row (r / out_rows_per_b) * in_rows_per_b + in_row_off +
// r % out_rows_per_b, which lets the output head skip text rows.  Rows whose position in
// their sequence (in_row_off + r % out_rows_per_b) is below alt_rows read shift, scale and
// gate alt_off floats further on: the text rows' own modulation set.
template <typename T, int NCH, bool TWO>
__global__ __launch_bounds__(256) void k_ln_modulate(float* __restrict__ x, const T* __restrict__ y,
                                                     const float* __restrict__ gate, const T* __restrict__ y2,
                                                     const float* __restrict__ gate2, const float* __restrict__ shift,
                                                     const float* __restrict__ scale, T* __restrict__ out, int rows, int D,
                                                     float eps, int in_rows_per_b, int out_rows_per_b, int in_row_off,
                                                     int alt_rows, int alt_off, int write_x) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int r = blockIdx.x * (blockDim.x >> 6) + wave;
  if (r >= rows) return;
  const int pos = in_row_off + r % out_rows_per_b;
  const size_t in_r = (size_t)(r / out_rows_per_b) * in_rows_per_b + pos;
  if (pos < alt_rows) {                 // wave-uniform
    if (gate) gate += alt_off;
    if (gate2) gate2 += alt_off;
    if (scale) { scale += alt_off; shift += alt_off; }
  }
  float* xr = x + in_r * D;
  // every load of the row (x, the pending y and y2, scale, shift) is issued before the
  // first use: the kernel lives on loads in flight, not on arithmetic
  // (for rows of up to 1280 elements; wider rows would need more registers than leave
  // enough waves per SIMD, and read y, gate, scale and shift chunk by chunk instead)
  constexpr bool BATCH = NCH <= 5;
  constexpr int NB = BATCH ? NCH : 1;
  typedef typename std::conditional<sizeof(T) == 2, bf16x4, f32x4>::type yvec;
  f32x4 v[NCH], scv[NB], shv[NB];
  yvec yv[NB], yv2[TWO ? NB : 1];
  const T* yr = y ? y + in_r * D : nullptr;
  const T* yr2 = TWO ? y2 + in_r * D : nullptr;
#pragma unroll
  for (int j = 0; j < NCH; ++j) {
    const int c = lane * 4 + j * 256;
    v[j] = c < D ? *(const f32x4*)(xr + c) : f32x4{0, 0, 0, 0};
  }
  if constexpr (BATCH) {
    if (y) {
#pragma unroll
      for (int j = 0; j < NCH; ++j) {
        const int c = lane * 4 + j * 256;
        if (c < D) yv[j] = *(const yvec*)(yr + c);
      }
    }
    if constexpr (TWO) {
#pragma unroll
      for (int j = 0; j < NCH; ++j) {
        const int c = lane * 4 + j * 256;
        if (c < D) yv2[j] = *(const yvec*)(yr2 + c);
      }
    }
    if (scale) {
#pragma unroll
      for (int j = 0; j < NCH; ++j) {
        const int c = lane * 4 + j * 256;
        if (c < D) { scv[j] = *(const f32x4*)(scale + c); shv[j] = *(const f32x4*)(shift + c); }
      }
    }
  }
  if (y) {
#pragma unroll
    for (int j = 0; j < NCH; ++j) {
      const int c = lane * 4 + j * 256;
      if (c < D) {
        const int jb = BATCH ? j : 0;
        if constexpr (!BATCH) {
          yv[0] = *(const yvec*)(yr + c);
          if constexpr (TWO) yv2[0] = *(const yvec*)(yr2 + c);
        }
        f32x4 yf;
#pragma unroll
        for (int e = 0; e < 4; ++e) yf[e] = (float)yv[jb][e];
        if (gate) yf = yf * *(const f32x4*)(gate + c);       // per-row gates: the rare case, read at use
        v[j] += yf;
        if constexpr (TWO) {                  // only ever given together with y
#pragma unroll
          for (int e = 0; e < 4; ++e) yf[e] = (float)yv2[jb][e];
          if (gate2) yf = yf * *(const f32x4*)(gate2 + c);
          v[j] += yf;
        }
        if (write_x) *(f32x4*)(xr + c) = v[j];
      }
    }
  }
  float sum = 0.0f;
#pragma unroll
  for (int j = 0; j < NCH; ++j) sum += (v[j][0] + v[j][1]) + (v[j][2] + v[j][3]);
  const float mean = wave_sum(sum) / (float)D;
  float sq = 0.0f;
#pragma unroll
  for (int j = 0; j < NCH; ++j) {
    const int c = lane * 4 + j * 256;
    if (c < D) {
      f32x4 d = v[j] - mean;
      sq += (d[0] * d[0] + d[1] * d[1]) + (d[2] * d[2] + d[3] * d[3]);
    }
  }
  const float rstd = 1.0f / sqrtf(wave_sum(sq) / (float)D + eps);
  T* o = out + (size_t)r * D;
#pragma unroll
  for (int j = 0; j < NCH; ++j) {
    const int c = lane * 4 + j * 256;
    if (c < D) {
      f32x4 w = (v[j] - mean) * rstd;
      if (scale) {
        if constexpr (BATCH) w = w * (1.0f + scv[j]) + shv[j];
        else w = w * (1.0f + *(const f32x4*)(scale + c)) + *(const f32x4*)(shift + c);
      }
      if constexpr (sizeof(T) == 2) {
        bf16x4 ov;
#pragma unroll
        for (int e = 0; e < 4; ++e) ov[e] = (bf16_t)w[e];
        *(bf16x4*)(o + c) = ov;
      } else {
        *(f32x4*)(o + c) = w;
      }
    }
  }
}

template <typename T>
static hipError_t run_ln(float* x, const void* y, const float* gate, const void* y2, const float* gate2,
                         const float* shift, const float* scale, void* out,
                         int rows, int D, float eps, int in_rows_per_b, int out_rows_per_b, int in_row_off, int alt_rows,
                         int alt_off, int write_x, hipStream_t s) {
  dim3 grid(ceil_div(rows, 4));
#define FC_LN(N)                                                                                                   \
  do {                                                                                                              \
    if (y2)                                                                                                         \
      k_ln_modulate<T, N, true><<<grid, 256, 0, s>>>(x, (const T*)y, gate, (const T*)y2, gate2, shift, scale, (T*)out, \
                                                     rows, D, eps, in_rows_per_b, out_rows_per_b, in_row_off,       \
                                                     alt_rows, alt_off, write_x);                                   \
    else                                                                                                            \
      k_ln_modulate<T, N, false><<<grid, 256, 0, s>>>(x, (const T*)y, gate, nullptr, nullptr, shift, scale, (T*)out, \
                                                      rows, D, eps, in_rows_per_b, out_rows_per_b, in_row_off,      \
                                                      alt_rows, alt_off, write_x);                                  \
  } while (0)
  if (D <= 256) FC_LN(1);
  else if (D <= 1280) FC_LN(5);
  else if (D <= 3072) FC_LN(12);
  else if (D <= 4096) FC_LN(16);
  else return hipErrorInvalidValue;
#undef FC_LN
  return hipGetLastError();
}

hipError_t launch_ln_modulate(int bf16, float* x, const void* y, const float* gate, const void* y2,
                              const float* gate2, const float* shift, const float* scale, void* out, int rows, int D,
                              float eps, int in_rows_per_b, int out_rows_per_b, int in_row_off, int alt_rows,
                              int alt_off, int write_x, hipStream_t s) {
  if (rows == 0) return hipSuccess;
  if (y2 && !y) return hipErrorInvalidValue;
  if (bf16)
    return run_ln<bf16_t>(x, y, gate, y2, gate2, shift, scale, out, rows, D, eps, in_rows_per_b, out_rows_per_b,
                          in_row_off, alt_rows, alt_off, write_x, s);
  return run_ln<float>(x, y, gate, y2, gate2, shift, scale, out, rows, D, eps, in_rows_per_b, out_rows_per_b, in_row_off,
                       alt_rows, alt_off, write_x, s);
}

// ---------------------------------------------------------------- guidance + DDIM update
// eps = eps_u + s (eps_c - eps_u);  x0 = (x - c1 eps) / c0;  x <- c2 x0 + c3 eps.
// 16 algorithmic bytes per element with guidance (3 reads + 1 write).
template <bool VEC>
__global__ void k_cfg_ddim(float* __restrict__ x, const float* __restrict__ eps_c, const float* __restrict__ eps_u,
                           float* __restrict__ eps_out, size_t n, float gs, float c0, float c1, float c2, float c3) {
  size_t i = ((size_t)blockIdx.x * blockDim.x + threadIdx.x) * 4;
  if (VEC && i + 3 < n) {
    f32x4 e = *(const f32x4*)(eps_c + i);
    if (eps_u) {
      f32x4 u = *(const f32x4*)(eps_u + i);
      e = u + gs * (e - u);
    }
    f32x4 xv = *(const f32x4*)(x + i);
    f32x4 x0 = (xv - c1 * e) / c0;
    *(f32x4*)(x + i) = c2 * x0 + c3 * e;
    if (eps_out) *(f32x4*)(eps_out + i) = e;
  } else {
    for (size_t end = i + 4 < n ? i + 4 : n; i < end; ++i) {
      float e = eps_c[i];
      if (eps_u) e = eps_u[i] + gs * (e - eps_u[i]);
      float x0 = (x[i] - c1 * e) / c0;
      x[i] = c2 * x0 + c3 * e;
      if (eps_out) eps_out[i] = e;
    }
  }
}

// ---------------------------------------------------------------- guidance + stochastic DDIM update (eta > 0)
// As above plus sigma * z, z standard normal, computed (not drawn) from (seed, request,
// step, element) with Philox4x32-10 (Salmon et al., SC'11): element i of request r takes
// lane i % 4 of the block with counter (i/4 low word, i/4 high word, step, r) and key
// (seed low, seed high); a 32-bit output w becomes u = ((w >> 8) + 0.5) 2^-24; lanes
// (0, 1) and (2, 3) are Box-Muller pairs.  One thread produces one block = 4 elements.
__device__ __forceinline__ void philox4x32_10(unsigned (&c)[4], unsigned k0, unsigned k1) {
#pragma unroll
  for (int r = 0; r < 10; ++r) {
    const unsigned long long p0 = 0xD2511F53ull * c[0], p1 = 0xCD9E8D57ull * c[2];
    const unsigned n0 = (unsigned)(p1 >> 32) ^ c[1] ^ k0, n2 = (unsigned)(p0 >> 32) ^ c[3] ^ k1;
    c[1] = (unsigned)p1; c[3] = (unsigned)p0; c[0] = n0; c[2] = n2;
    k0 += 0x9E3779B9u; k1 += 0xBB67AE85u;
  }
}

__global__ void k_cfg_ddim_noise(float* __restrict__ x, const float* __restrict__ eps_c,
                                 const float* __restrict__ eps_u, float* __restrict__ eps_out, size_t per_request,
                                 int requests, float gs, float c0, float c1, float c2, float c3, float sigma,
                                 unsigned long long seed, int step) {
  const size_t blocks_per_req = (per_request + 3) / 4;
  const size_t b = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (b >= blocks_per_req * (size_t)requests) return;
  const size_t r = b / blocks_per_req, blk = b % blocks_per_req;
  unsigned c[4] = {(unsigned)blk, (unsigned)((unsigned long long)blk >> 32), (unsigned)step, (unsigned)r};
  philox4x32_10(c, (unsigned)seed, (unsigned)(seed >> 32));
  float z[4];
#pragma unroll
  for (int pr = 0; pr < 2; ++pr) {
    const float ua = ((float)(c[2 * pr] >> 8) + 0.5f) * 5.9604644775390625e-8f;       // 2^-24: exact in fp32
    const float ub = ((float)(c[2 * pr + 1] >> 8) + 0.5f) * 5.9604644775390625e-8f;
    const float rad = sqrtf(-2.0f * logf(ua));
    float sn, cs;
    sincosf(6.283185307179586f * ub, &sn, &cs);
    z[2 * pr] = rad * cs;
    z[2 * pr + 1] = rad * sn;
  }
  const size_t base = r * per_request + blk * 4;
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    if (blk * 4 + e >= per_request) break;
    const size_t i = base + e;
    float ev = eps_c[i];
    if (eps_u) ev = eps_u[i] + gs * (ev - eps_u[i]);
    const float x0 = (x[i] - c1 * ev) / c0;
    x[i] = c2 * x0 + c3 * ev + sigma * z[e];
    if (eps_out) eps_out[i] = ev;
  }
}

hipError_t launch_cfg_ddim_noise(float* x, const float* eps_c, const float* eps_u, float* eps_out, size_t per_request,
                                 int requests, float gscale, float c0, float c1, float c2, float c3, float sigma,
                                 unsigned long long seed, int step, hipStream_t s) {
  const size_t threads = (per_request + 3) / 4 * (size_t)requests;
  if (threads == 0) return hipSuccess;
  k_cfg_ddim_noise<<<(unsigned)((threads + 255) / 256), 256, 0, s>>>(x, eps_c, eps_u, eps_out, per_request, requests,
                                                                      gscale, c0, c1, c2, c3, sigma, seed, step);
  return hipGetLastError();
}

hipError_t launch_cfg_ddim(float* x, const float* eps_c, const float* eps_u, float* eps_out, size_t n,
                           float gscale, float c0, float c1, float c2, float c3, hipStream_t s) {
  if (n == 0) return hipSuccess;
  size_t threads = (n + 3) / 4;
  unsigned blocks = (unsigned)((threads + 255) / 256);
  // 16-byte vector access needs every pointer aligned; otherwise each thread walks its 4 elements
  uintptr_t al = (uintptr_t)x | (uintptr_t)eps_c | (uintptr_t)eps_u | (uintptr_t)eps_out;
  if ((al & 15) == 0) k_cfg_ddim<true><<<blocks, 256, 0, s>>>(x, eps_c, eps_u, eps_out, n, gscale, c0, c1, c2, c3);
  else k_cfg_ddim<false><<<blocks, 256, 0, s>>>(x, eps_c, eps_u, eps_out, n, gscale, c0, c1, c2, c3);
  return hipGetLastError();
}

}  // namespace fc
