// Restoring a cached latent, the input of the resume loop: stitching an object and a
// background cache with their 1-bit masks (Sec. 4.2.2), expanding a compressed entry
// (Sec. 4.1: first frame + alpha * base differentials, extra frames, repeated key frames),
// and the two reductions of the compressing side that define what is expanded (Eq. 2's
// least-squares coefficient, the frame cosine similarities the key frames are chosen by).
// All of it moves each byte once: the kernels are bound by HBM.
#include "common.h"

#include <mutex>

namespace fc {

// ---------------------------------------------------------------- stitching
// take_obj(pixel) = m_obj OR NOT m_bg; out = take_obj ? x_obj : x_bg for every channel of
// the pixel.  Masks: pixel i is bit i % 8 of byte i / 8.  VEC: channels % 4 == 0 and all
// pointers 16-byte aligned, one thread per 4 channels; otherwise one thread per element.
template <bool VEC>
__global__ void k_stitch(const float* x_obj, const float* x_bg,      // either may be `out` itself: no __restrict__
                         const uint8_t* __restrict__ m_obj, const uint8_t* __restrict__ m_bg, float* out,
                         long long pixels, int channels) {
  const int per_pixel = VEC ? channels / 4 : channels;
  const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= pixels * per_pixel) return;
  const long long px = i / per_pixel;
  bool take = (m_obj[px >> 3] >> (px & 7)) & 1;
  if (m_bg) take = take || !((m_bg[px >> 3] >> (px & 7)) & 1);
  if (VEC) {
    ((f32x4*)out)[i] = take ? ((const f32x4*)x_obj)[i] : ((const f32x4*)x_bg)[i];
  } else {
    out[i] = take ? x_obj[i] : x_bg[i];
  }
}

hipError_t launch_stitch(const float* x_obj, const float* x_bg, const uint8_t* m_obj, const uint8_t* m_bg, float* out,
                         long long pixels, int channels, hipStream_t s) {
  if (pixels == 0) return hipSuccess;
  const bool vec = channels % 4 == 0 && (((uintptr_t)x_obj | (uintptr_t)x_bg | (uintptr_t)out) & 15) == 0;
  const long long n = pixels * (vec ? channels / 4 : channels);
  const unsigned blocks = (unsigned)((n + 255) / 256);
  if (vec) k_stitch<true><<<blocks, 256, 0, s>>>(x_obj, x_bg, m_obj, m_bg, out, pixels, channels);
  else k_stitch<false><<<blocks, 256, 0, s>>>(x_obj, x_bg, m_obj, m_bg, out, pixels, channels);
  return hipGetLastError();
}

// ---------------------------------------------------------------- expanding a compressed entry
// Frame t of the output comes from source code src[t]: 0 = the stored first frame,
// j >= 1 = first + alpha * diff_base[j-1], -(e+1) = extra frame e.  blockIdx.y = t.
struct DecompressSrc { int code[kMaxCacheFrames]; };

__global__ void k_decompress(const float* __restrict__ first, const float* __restrict__ diff_base, float alpha,
                             const float* __restrict__ extra, DecompressSrc src, long long F, float* __restrict__ out) {
  const int t = blockIdx.y;
  const int code = src.code[t];
  const float* add = code > 0 ? diff_base + (size_t)(code - 1) * F : nullptr;
  const float* base = code < 0 ? extra + (size_t)(-code - 1) * F : first;
  float* o = out + (size_t)t * F;
  for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < F; i += (long long)gridDim.x * blockDim.x)
    o[i] = add ? base[i] + alpha * add[i] : base[i];
}

hipError_t launch_decompress(const float* first, const float* diff_base, float alpha, const float* extra,
                             const int* src_host, int T, long long F, float* out, hipStream_t s) {
  if (T == 0 || F == 0) return hipSuccess;
  DecompressSrc src;
  for (int t = 0; t < T; ++t) src.code[t] = src_host[t];
  const unsigned bx = (unsigned)((F + 255) / 256 < 1024 ? (F + 255) / 256 : 1024);
  k_decompress<<<dim3(bx, T), 256, 0, s>>>(first, diff_base, alpha, extra, src, F, out);
  return hipGetLastError();
}

// ---------------------------------------------------------------- reductions of the compressing side
// Deterministic two-pass sums in double: kRedBlocks partial results, then one block adds
// them in a fixed order.  No atomics.
constexpr int kRedBlocks = 256;

__device__ __forceinline__ double block_sum(double v, double* sh) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  __syncthreads();
  if (lane == 0) sh[wave] = v;
  __syncthreads();
  double t = 0.0;
  for (int w = 0; w < (int)(blockDim.x >> 6); ++w) t += sh[w];
  return t;
}

// partial[b] = { sum (keys_s - first_s) * diff_base, sum diff_base^2 } over block b's share
__global__ __launch_bounds__(256) void k_alpha_partial(const float* __restrict__ first_s, const float* __restrict__ keys_s,
                                                       const float* __restrict__ diff_base, long long F, long long total,
                                                       double* __restrict__ partial) {
  __shared__ double sh[4];
  double num = 0.0, den = 0.0;
  for (long long i = (long long)blockIdx.x * 256 + threadIdx.x; i < total; i += (long long)kRedBlocks * 256) {
    const double db = diff_base[i];
    num += ((double)keys_s[i] - (double)first_s[i % F]) * db;
    den += db * db;
  }
  num = block_sum(num, sh);
  den = block_sum(den, sh);
  if (threadIdx.x == 0) { partial[2 * blockIdx.x] = num; partial[2 * blockIdx.x + 1] = den; }
}

__global__ __launch_bounds__(64) void k_alpha_final(const double* __restrict__ partial, float* __restrict__ alpha_out) {
  if (threadIdx.x != 0) return;
  double num = 0.0, den = 0.0;
  for (int b = 0; b < kRedBlocks; ++b) { num += partial[2 * b]; den += partial[2 * b + 1]; }
  // Diff_base identically zero: every alpha fits equally well and the restored frames do not
  // depend on it; the minimum-norm choice is 0
  alpha_out[0] = den > 0.0 ? (float)(num / den) : 0.0f;
}

hipError_t launch_alpha(const float* first_s, const float* keys_s, const float* diff_base, int n_base, long long F,
                        float* alpha_out, double* ws, hipStream_t s) {
  k_alpha_partial<<<kRedBlocks, 256, 0, s>>>(first_s, keys_s, diff_base, F, (long long)n_base * F, ws);
  k_alpha_final<<<1, 64, 0, s>>>(ws, alpha_out);
  return hipGetLastError();
}

// gram[i * T + j] = <frame i, frame j> for j <= i (one block per pair), then
// sim[i][j] = sim[j][i] = gram[i][j] / sqrt(gram[i][i] gram[j][j]).
__global__ __launch_bounds__(256) void k_frame_gram(const float* __restrict__ frames, int T, long long F,
                                                    double* __restrict__ gram) {
  __shared__ double sh[4];
  const int i = blockIdx.y, j = blockIdx.x;
  if (j > i) return;
  const float* a = frames + (size_t)i * F;
  const float* b = frames + (size_t)j * F;
  double acc = 0.0;
  for (long long e = threadIdx.x; e < F; e += 256) acc += (double)a[e] * (double)b[e];
  acc = block_sum(acc, sh);
  if (threadIdx.x == 0) gram[(size_t)i * T + j] = acc;
}

__global__ void k_frame_cosine(const double* __restrict__ gram, int T, float* __restrict__ sim) {
  const int idx = blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= T * T) return;
  const int i = idx / T, j = idx % T;
  const int hi = i > j ? i : j, lo = i > j ? j : i;
  const double n = sqrt(gram[(size_t)hi * T + hi] * gram[(size_t)lo * T + lo]);
  sim[idx] = (float)(gram[(size_t)hi * T + lo] / (n > 1e-300 ? n : 1e-300));
}

hipError_t launch_frame_similarity(const float* frames, int T, long long F, float* sim, double* ws, hipStream_t s) {
  if (T == 0) return hipSuccess;
  k_frame_gram<<<dim3(T, T), 256, 0, s>>>(frames, T, F, ws);
  k_frame_cosine<<<(T * T + 255) / 256, 256, 0, s>>>(ws, T, sim);
  return hipGetLastError();
}

// ---------------------------------------------------------------- the same, with library-owned scratch
// For callers that cannot allocate (a HIP graph being captured, a serving loop, a harness that
// forbids hipMalloc): the Gram matrix of the largest entry (256 frames, 512 KB) lives in a
// file-scope device array.  Every device the library runs on holds its own copy at its own
// address; the address is looked up once per device, with that device current, and host code
// only ever passes that looked-up pointer on (the array's name is a host-side stand-in).
static __device__ __align__(256) double scratch[(size_t)kMaxCacheFrames * kMaxCacheFrames];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
double* g_scratch_ptr[kMaxDevices] = {};
}  // namespace

hipError_t static_gram_scratch(double** out) {
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!p) return hipErrorInvalidSymbol;
    g_scratch_ptr[dev] = (double*)p;
  }
  *out = g_scratch_ptr[dev];
  return hipSuccess;
}

// Nothing in the array has to start at zero: k_frame_gram writes every entry (i, j <= i) that
// k_frame_cosine of the same call reads, whatever an earlier call with another T left behind.
hipError_t launch_frame_similarity_static(const float* frames, int T, long long F, float* sim, hipStream_t s) {
  if (T == 0) return hipSuccess;
  if (T > kMaxCacheFrames) return hipErrorInvalidValue;
  double* ws = nullptr;
  hipError_t e = static_gram_scratch(&ws);
  if (e != hipSuccess) return e;
  return launch_frame_similarity(frames, T, F, sim, ws, s);
}

// ---------------------------------------------------------------- plain copy (key-step export)
__global__ void k_copy_f32(const float* __restrict__ in, float* __restrict__ out, size_t n) {
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) out[i] = in[i];
}

hipError_t launch_copy_f32(const float* in, float* out, size_t n, hipStream_t s) {
  if (n == 0) return hipSuccess;
  k_copy_f32<<<(unsigned)((n + 255) / 256), 256, 0, s>>>(in, out, n);
  return hipGetLastError();
}

}  // namespace fc
