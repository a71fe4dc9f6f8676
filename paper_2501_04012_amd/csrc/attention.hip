// Unmasked softmax(q k^T / sqrt(d)) v.
//   k_attn_plain : one thread per query row, online softmax in fp32.  Any dtype, any
//                  strides; used by the fp32 configuration and as the fallback.
//   k_attn_flash : bf16 MFMA flash kernel.  Scores are computed transposed
//                  (S^T = K Q^T) so that each query column lives in two lanes, the
//                  running max / sum need one cross-lane exchange per tile, and the
//                  probabilities are already in the register layout the P V MFMA
//                  takes as its B operand: P never touches LDS.  V is staged row-major
//                  like K; the V^T fragments come from the LDS transpose read
//                  (ds_read_b64_tr_b16), so no transposed copy of V exists anywhere.
#include "common.h"

#include <type_traits>

namespace fc {

__device__ __forceinline__ int key_batch(const AttnParams& p, int b) {
  return (p.kv_shared_tail && b >= p.kv_split) ? p.kv_split : b;
}

// Workgroup id -> work item, XCD-aware.  Hardware deals consecutive workgroup ids to the 8
// XCDs in turn; work items are ordered (batch, head, group, query tile) with the query tile
// fastest.  Giving each XCD one contiguous range of work items makes the workgroups that
// run together on an XCD share a (batch, head, group), so its K and V tiles are fetched
// into that XCD's L2 once and hit by the other ~31 workgroups walking the same keys.
// Returns -1 for the padding workgroups of a grid rounded up to a multiple of 8.
__device__ __forceinline__ long long xcd_work_item(long long total) {
  const long long per = (total + 7) / 8;
  const long long w = (long long)(blockIdx.x & 7) * per + (blockIdx.x >> 3);
  return ((long long)(blockIdx.x >> 3) < per && w < total) ? w : -1;
}

// ---------------------------------------------------------------- plain kernel
// One thread per query row, online softmax in fp32, rows read with 16-byte loads.
// Thread order follows memory order: for strided sequences (temporal attention: token
// stride S) neighbouring threads take neighbouring groups, so their q/k/v rows are
// adjacent in memory; for contiguous sequences neighbouring threads take neighbouring
// queries of one group and share its key rows.
template <typename T, int HD>
__device__ __forceinline__ void load_row(const T* __restrict__ src, float (&dst)[HD]) {
  constexpr int V = 16 / sizeof(T);
  static_assert(HD % V == 0, "row must be a whole number of 16-byte chunks");
#pragma unroll
  for (int c = 0; c < HD; c += V) {
    if constexpr (sizeof(T) == 2) {
      bf16x8 v = *(const bf16x8*)(src + c);
#pragma unroll
      for (int e = 0; e < 8; ++e) dst[c + e] = (float)v[e];
    } else {
      f32x4 v = *(const f32x4*)(src + c);
#pragma unroll
      for (int e = 0; e < 4; ++e) dst[c + e] = v[e];
    }
  }
}

template <typename T, int HD>
__global__ __launch_bounds__(64) void k_attn_plain(AttnParams p) {
  const long long gid = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  const long long total = (long long)p.B * p.heads * p.groups * p.nq;
  if (gid >= total) return;
  int i, g;
  long long r;
  if (p.q_istride == 1) { i = (int)(gid % p.nq); r = gid / p.nq; g = (int)(r % p.groups); r /= p.groups; }
  else { g = (int)(gid % p.groups); r = gid / p.groups; i = (int)(r % p.nq); r /= p.nq; }
  const int head = (int)(r % p.heads);
  const int b = (int)(r / p.heads);
  const int kb = key_batch(p, b);

  const int qtok = g * p.q_gstride + i * p.q_istride;
  const T* q = (const T*)p.q + (((size_t)b * p.heads + head) * p.q_tokens + qtok) * HD;
  const T* kbase = (const T*)p.k + ((size_t)kb * p.heads + head) * (size_t)p.k_tokens * HD;
  const T* vbase = (const T*)p.v + ((size_t)kb * p.heads + head) * (size_t)p.k_tokens * HD;

  float qv[HD], o[HD], row[HD];
  load_row<T, HD>(q, qv);
#pragma unroll
  for (int c = 0; c < HD; ++c) o[c] = 0.0f;
  float m = -INFINITY, l = 0.0f;
  for (int j = 0; j < p.nk; ++j) {
    const int ktok = g * p.k_gstride + j * p.k_istride;
    load_row<T, HD>(kbase + (size_t)ktok * HD, row);
    float s = 0.0f;
#pragma unroll
    for (int c = 0; c < HD; ++c) s += qv[c] * row[c];
    s *= p.scale_log2;
    const float mn = fmaxf(m, s);
    const float alpha = exp2f(m - mn);     // m = -inf on the first key: exp2(-inf) = 0
    const float pj = exp2f(s - mn);
    l = l * alpha + pj;
    load_row<T, HD>(vbase + (size_t)ktok * HD, row);
#pragma unroll
    for (int c = 0; c < HD; ++c) o[c] = o[c] * alpha + pj * row[c];
    m = mn;
  }
  const float inv = 1.0f / l;
  T* out = (T*)p.out + ((size_t)b * p.q_tokens + qtok) * ((size_t)p.heads * HD) + (size_t)head * HD;
#pragma unroll
  for (int c = 0; c < HD; ++c) out[c] = from_f32<T>(o[c] * inv);
}

template <typename T, int HD>
static hipError_t run_plain(const AttnParams& p, hipStream_t s) {
  long long total = (long long)p.B * p.heads * p.groups * p.nq;
  if (total == 0) return hipSuccess;
  k_attn_plain<T, HD><<<(unsigned)((total + 63) / 64), 64, 0, s>>>(p);
  return hipGetLastError();
}

// ---------------------------------------------------------------- short strided sequences (temporal)
// Temporal attention: S independent sequences of T <= 32 tokens per (batch, head), token
// t of sequence s being row t*S + s.  A workgroup takes SB = 8 neighbouring sequences:
// for each t their rows are one contiguous run of SB*HD elements, fetched with 16-byte
// loads into LDS (q, k, v tiles [T][SB][HD]); thread (t, s) then runs the plain online
// softmax for its query against the T keys of its sequence out of LDS.  The work is a
// few flops per byte: the kernel is bound by reading q, k, v and writing o once.
constexpr int TS_SB = 8;
template <typename T, int HD>
__global__ __launch_bounds__(256) void k_attn_short_strided(AttnParams p) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_ts[];
  T* qs = (T*)smem_ts;
  const int Tn = p.nq;                       // == nk
  const int tile = Tn * TS_SB * HD;          // elements per tensor tile
  T* ks = qs + tile;
  T* vs = ks + tile;
  const int sblocks = (p.groups + TS_SB - 1) / TS_SB;
  int bid = blockIdx.x;
  const int sb = bid % sblocks; bid /= sblocks;
  const int head = bid % p.heads;
  const int b = bid / p.heads;
  const int s0 = sb * TS_SB;
  const size_t bh = ((size_t)b * p.heads + head) * (size_t)p.q_tokens;
  const T* qg = (const T*)p.q + bh * HD;
  const T* kg = (const T*)p.k + bh * HD;
  const T* vg = (const T*)p.v + bh * HD;

  constexpr int V = 16 / sizeof(T);
  constexpr int CPR = HD / V;                // 16-byte chunks per row
  const int chunks = Tn * TS_SB * CPR;
  for (int ch = threadIdx.x; ch < chunks; ch += blockDim.x) {
    const int c = ch % CPR, r = ch / CPR;
    const int s = r % TS_SB, t = r / TS_SB;
    int sg = s0 + s; sg = sg < p.groups ? sg : p.groups - 1;     // clamp: rows past the last sequence are never stored
    const size_t goff = ((size_t)t * p.q_istride + sg) * HD + c * V;
    const int loff = (t * TS_SB + s) * HD + c * V;
    *(f32x4*)(qs + loff) = *(const f32x4*)(qg + goff);
    *(f32x4*)(ks + loff) = *(const f32x4*)(kg + goff);
    *(f32x4*)(vs + loff) = *(const f32x4*)(vg + goff);
  }
  __syncthreads();

  const int s = threadIdx.x % TS_SB, tq = threadIdx.x / TS_SB;
  if (tq >= Tn || s0 + s >= p.groups) return;
  float qv[HD], o[HD], row[HD];
  load_row<T, HD>(qs + (tq * TS_SB + s) * HD, qv);
#pragma unroll
  for (int c = 0; c < HD; ++c) o[c] = 0.0f;
  float m = -INFINITY, l = 0.0f;
  for (int j = 0; j < Tn; ++j) {
    load_row<T, HD>(ks + (j * TS_SB + s) * HD, row);
    float sc = 0.0f;
#pragma unroll
    for (int c = 0; c < HD; ++c) sc += qv[c] * row[c];
    sc *= p.scale_log2;
    const float mn = fmaxf(m, sc);
    const float alpha = exp2f(m - mn);
    const float pj = exp2f(sc - mn);
    l = l * alpha + pj;
    load_row<T, HD>(vs + (j * TS_SB + s) * HD, row);
#pragma unroll
    for (int c = 0; c < HD; ++c) o[c] = o[c] * alpha + pj * row[c];
    m = mn;
  }
  const float inv = 1.0f / l;
  const int tok = tq * p.q_istride + s0 + s;
  T* out = (T*)p.out + ((size_t)b * p.q_tokens + tok) * ((size_t)p.heads * HD) + (size_t)head * HD;
#pragma unroll
  for (int c = 0; c < HD; c += V) {
    if constexpr (sizeof(T) == 2) {
      bf16x8 ov;
#pragma unroll
      for (int e = 0; e < 8; ++e) ov[e] = (bf16_t)(o[c + e] * inv);
      *(bf16x8*)(out + c) = ov;
    } else {
      f32x4 ov;
#pragma unroll
      for (int e = 0; e < 4; ++e) ov[e] = o[c + e] * inv;
      *(f32x4*)(out + c) = ov;
    }
  }
}

static bool short_strided_ok(const AttnParams& p, size_t esz) {
  return p.nq == p.nk && p.nq >= 1 && p.nq * TS_SB <= 256 && p.q_gstride == 1 && p.k_gstride == 1 &&
         p.q_istride == p.k_istride && p.q_istride == p.groups && p.q_tokens == p.k_tokens && !p.kv_shared_tail &&
         (size_t)3 * p.nq * TS_SB * p.hd * esz <= 64 * 1024;
}

template <typename T, int HD>
static hipError_t run_short_strided(const AttnParams& p, hipStream_t s) {
  const long long blocks = (long long)p.B * p.heads * ((p.groups + TS_SB - 1) / TS_SB);
  if (blocks == 0) return hipSuccess;
  const size_t smem = (size_t)3 * p.nq * TS_SB * HD * sizeof(T);
  const int threads = (p.nq * TS_SB + 63) / 64 * 64;
  k_attn_short_strided<T, HD><<<(unsigned)blocks, threads, smem, s>>>(p);
  return hipGetLastError();
}

// ---------------------------------------------------------------- short strided sequences on the matrix cores
// Same problem as above for bf16 and T <= 64: the scalar kernel spends its time in
// bf16->fp32 unpacking and 2 T HD FMAs per query; here the work is a handful of small
// MFMAs per 16 queries and the kernel is bound by reading q, k, v and writing o once.
// The sequence is cut into KB = ceil(T / 16) blocks of 16 tokens (KB = 1, 2 or 4).
//   S^T (16 keys x 16 queries) = K (A operand) x Q^T (B operand), v_mfma_f32_16x16x32_bf16,
//   contraction over the head dim in steps of 32, one such tile per key block.  Operand
//   lane l = (i, h), i = l % 16, h = l / 16: row/column i, k = 8h .. 8h+7.  D: column i,
//   rows 4h + e in register e.  So lane (i, h) holds the scores of query i against keys
//   16 kb + 4h .. + 3: after exp2 and rounding they are, as they stand, the B operand
//   (k = 4h .. 4h+3) of O^T (16 dims x 16 queries) += V^T (A operand) x P^T,
//   v_mfma_f32_16x16x16_bf16, whose A fragments (dim i, keys 4h .. 4h+3) are transpose
//   reads of the row-major V tile.  All keys of a query are seen at once: plain two-pass
//   softmax in registers, no running maximum.
// A workgroup of 4 waves stages SB = ITEMS / KB neighbouring sequences ([SB][16 KB][PITCH]
// per tensor, coalesced: for one t the SB rows are contiguous in memory) and has ITEMS work
// items (sequence, query block), ITEMS / 4 per wave.  ITEMS = 4: at 28 KB of LDS five
// workgroups share a CU and cover each other's load latency; with 8 items (55 KB, two per
// CU) the launch was 9 % slower.  PITCH/8 is odd so that the 16 rows of a fragment read
// fall into distinct bank groups.
typedef __attribute__((ext_vector_type(4))) short i16x4;
typedef __attribute__((address_space(3))) bf16x4 lds_bf16x4;
constexpr int kShortItems = 4;
template <int HD, int KB, int ITEMS>
struct ShortMfmaCfg {
  static constexpr int SB = ITEMS / KB;                                  // sequences per workgroup
  static constexpr int TP = 16 * KB;                                     // padded sequence length
  static constexpr int PITCH = ((HD / 8) % 2 == 1) ? HD : HD + 8;      // elements
  static constexpr int TILE = SB * TP * PITCH;                           // elements per tensor
  static constexpr size_t SMEM = (size_t)3 * TILE * sizeof(bf16_t) + 64; // slack: the last V fragment reads past HD
  static constexpr int KSTEPS = (HD + 31) / 32;
  static constexpr int DT = (HD + 15) / 16;
};

template <int HD, int KB, int ITEMS>
__global__ __launch_bounds__(256) void k_attn_short_mfma(AttnParams p) {
  using C = ShortMfmaCfg<HD, KB, ITEMS>;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_sm[];
  bf16_t* qs = (bf16_t*)smem_sm;
  bf16_t* ks = qs + C::TILE;
  bf16_t* vs = ks + C::TILE;
  const int Tn = p.nq;                       // == nk, <= 16 KB
  const int sblocks = (p.groups + C::SB - 1) / C::SB;
  int bid = blockIdx.x;
  const int sb = bid % sblocks; bid /= sblocks;
  const int head = bid % p.heads;
  const int b = bid / p.heads;
  const int s0 = sb * C::SB;
  const size_t bh = ((size_t)b * p.heads + head) * (size_t)p.q_tokens;
  const bf16_t* qg = (const bf16_t*)p.q + bh * HD;
  const bf16_t* kg = (const bf16_t*)p.k + bh * HD;
  const bf16_t* vg = (const bf16_t*)p.v + bh * HD;

  // ---- stage: rows t >= Tn are zero (V rows of masked keys must not hold NaN patterns)
  //      All loads of a thread are issued before its first LDS store (one exposed latency).
  constexpr int CPR = HD / 8;
  constexpr int NCHK = C::TP * C::SB * CPR, NIT = (NCHK + 255) / 256;
  f32x4 zq[NIT], zk[NIT], zv[NIT];
#pragma unroll
  for (int i = 0; i < NIT; ++i) {
    const int ch = threadIdx.x + i * 256;
    const int c = ch % CPR, r = ch / CPR;
    const int sq = r % C::SB, t = r / C::SB;
    zq[i] = f32x4{0.0f, 0.0f, 0.0f, 0.0f}; zk[i] = zq[i]; zv[i] = zq[i];
    if (ch < NCHK && t < Tn) {
      int sg = s0 + sq; sg = sg < p.groups ? sg : p.groups - 1;   // sequences past the last are never stored
      const size_t goff = ((size_t)t * p.q_istride + sg) * HD + c * 8;
      zq[i] = *(const f32x4*)(qg + goff);
      zk[i] = *(const f32x4*)(kg + goff);
      zv[i] = *(const f32x4*)(vg + goff);
    }
  }
#pragma unroll
  for (int i = 0; i < NIT; ++i) {
    const int ch = threadIdx.x + i * 256;
    if (ch < NCHK) {
      const int c = ch % CPR, r = ch / CPR;
      const int sq = r % C::SB, t = r / C::SB;
      const int loff = (sq * C::TP + t) * C::PITCH + c * 8;
      *(f32x4*)(qs + loff) = zq[i];
      *(f32x4*)(ks + loff) = zk[i];
      *(f32x4*)(vs + loff) = zv[i];
    }
  }
  __syncthreads();

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int li = lane & 15, lh = lane >> 4;
  const int tr_r = li >> 2, tr_a = li & 3;
#pragma unroll
  for (int w = 0; w < ITEMS / 4; ++w) {
    const int item = wave + 4 * w;                       // (sequence, query block)
    const int sq = item / KB, qb = item % KB;
    if (s0 + sq >= p.groups || 16 * qb >= Tn) continue;  // wave-uniform
    const bf16_t* qrow = qs + (sq * C::TP + 16 * qb + li) * C::PITCH;
    f32x4 sacc[KB];
#pragma unroll
    for (int kb = 0; kb < KB; ++kb) sacc[kb] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
    for (int st = 0; st < C::KSTEPS; ++st) {
      const int d0 = 32 * st + 8 * lh;
      const bool in = d0 < HD;                           // HD % 8 == 0: a fragment is all in or all out
      bf16x8 qf;
#pragma unroll
      for (int e = 0; e < 8; ++e) qf[e] = (bf16_t)0.0f;
      if (in) qf = *(const bf16x8*)(qrow + d0);
#pragma unroll
      for (int kb = 0; kb < KB; ++kb) {
        bf16x8 kf;
#pragma unroll
        for (int e = 0; e < 8; ++e) kf[e] = (bf16_t)0.0f;
        if (in) kf = *(const bf16x8*)(ks + (sq * C::TP + 16 * kb + li) * C::PITCH + d0);
        sacc[kb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf, qf, sacc[kb], 0, 0, 0);
      }
    }
    // ---- softmax over the keys of query 16 qb + li: 4 KB of them here, the rest in lanes li + 16 h'
    float sc[KB][4];
    float mx = -INFINITY;
#pragma unroll
    for (int kb = 0; kb < KB; ++kb)
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        sc[kb][e] = (16 * kb + 4 * lh + e < Tn) ? sacc[kb][e] * p.scale_log2 : -INFINITY;
        mx = fmaxf(mx, sc[kb][e]);
      }
    mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64));              // finite: key 0 is valid
    i16x4 pf[KB];
    float sum = 0.0f;
#pragma unroll
    for (int kb = 0; kb < KB; ++kb) {
      bf16x4 pb;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        pb[e] = (bf16_t)__builtin_amdgcn_exp2f(sc[kb][e] - mx);
        sum += (float)pb[e];
      }
      pf[kb] = __builtin_bit_cast(i16x4, pb);
    }
    sum += __shfl_xor(sum, 16, 64);
    sum += __shfl_xor(sum, 32, 64);
    const float inv = 1.0f / sum;

    const int tq = 16 * qb + li;
    const int tok = tq * p.q_istride + s0 + sq;
    bf16_t* orow = (bf16_t*)p.out + ((size_t)b * p.q_tokens + tok) * ((size_t)p.heads * HD) + (size_t)head * HD;
    const bf16_t* vtile = vs + (sq * C::TP + 4 * lh + tr_r) * C::PITCH + 4 * tr_a;
#pragma unroll
    for (int c = 0; c < C::DT; ++c) {
      f32x4 o = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
      for (int kb = 0; kb < KB; ++kb) {
        const bf16x4 vf = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4*)(vtile + 16 * kb * C::PITCH + 16 * c));
        o = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(__builtin_bit_cast(i16x4, vf), pf[kb], o, 0, 0, 0);
      }
      const int dd = 16 * c + 4 * lh;
      if (tq < Tn && dd < HD) {
        bf16x4 ov;
#pragma unroll
        for (int e = 0; e < 4; ++e) ov[e] = (bf16_t)(o[e] * inv);
        *(bf16x4*)(orow + dd) = ov;
      }
    }
  }
}

static bool short_mfma_ok(const AttnParams& p) {
  return (p.hd == 64 || p.hd == 72) && p.nq == p.nk && p.nq >= 1 && p.nq <= 64 && p.q_gstride == 1 &&
         p.k_gstride == 1 && p.q_istride == p.k_istride && p.q_istride == p.groups && p.q_tokens == p.k_tokens &&
         !p.kv_shared_tail;
}

template <int HD, int KB>
static hipError_t run_short_mfma_kb(const AttnParams& p, hipStream_t s) {
  constexpr int ITEMS = kShortItems;
  using C = ShortMfmaCfg<HD, KB, ITEMS>;
  const long long blocks = (long long)p.B * p.heads * ((p.groups + C::SB - 1) / C::SB);
  if (blocks == 0) return hipSuccess;
  auto kern = k_attn_short_mfma<HD, KB, ITEMS>;
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)C::SMEM);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  kern<<<(unsigned)blocks, 256, C::SMEM, s>>>(p);
  return hipGetLastError();
}

template <int HD>
static hipError_t run_short_mfma(const AttnParams& p, hipStream_t s) {
  if (p.nq <= 16) return run_short_mfma_kb<HD, 1>(p, s);
  if (p.nq <= 32) return run_short_mfma_kb<HD, 2>(p, s);
  return run_short_mfma_kb<HD, 4>(p, s);
}

template <typename T, int HD>
static hipError_t run_non_mfma(const AttnParams& p, bool allow_short, hipStream_t s) {
  if (allow_short && short_strided_ok(p, sizeof(T))) return run_short_strided<T, HD>(p, s);
  return run_plain<T, HD>(p, s);
}

template <typename T>
static hipError_t dispatch_plain(const AttnParams& p, bool allow_short, hipStream_t s) {
  switch (p.hd) {
    case 8: return run_non_mfma<T, 8>(p, allow_short, s);
    case 16: return run_non_mfma<T, 16>(p, allow_short, s);
    case 32: return run_non_mfma<T, 32>(p, allow_short, s);
    case 64: return run_non_mfma<T, 64>(p, allow_short, s);
    case 72: return run_non_mfma<T, 72>(p, allow_short, s);
    case 96: return run_non_mfma<T, 96>(p, allow_short, s);
    case 128: return run_non_mfma<T, 128>(p, allow_short, s);
  }
  return hipErrorInvalidValue;
}

// ---------------------------------------------------------------- flash kernel (bf16, MFMA)
// Workgroup = NWV (4 or 8) waves; wave w owns 32 QT query rows of a 32 QT NWV-row query
// tile (QT = 1 or 2 32-column MFMA tiles qt).  Keys are walked in tiles of 64, staged in LDS as
// K [64][HDP] and V [64][HDV] (double-buffered, register-prefetched).
//
// Per key tile and wave:
//   S^T[a][qt] (32 keys x 32 queries) = K_a (A operand) x Q_qt^T (B operand, in
//   registers for the whole kernel), contraction over the head dim in steps of 16.
//   Lane (i, h) of S^T holds query column i and key rows r = 8g + 4h + e.  The K row
//   fed as MFMA row r is key perm(r) = r with bits 2 and 3 swapped, so that the 8
//   values of registers {4(2s), .., 4(2s+1)+3} are the 8 consecutive keys
//   16s + 8h .. + 7, the k-slice lane half h supplies in the P V step.
//   O^T[c][qt] (32 head dims x 32 queries) += V^T_c (A operand) x P^T (B operand).
//   Softmax cost per score is one max3 half, one exp2, half a cvt_pk and half a dot2:
//   the subtraction of the running reference rides in the MFMA accumulator.
//   A-operand lane (i, h) needs V[key 16s + 8h + x][dim 32c + i], x = 0..7: two
//   transpose reads.  In each 16-lane group, source lane 4r + a addresses the 8
//   bytes V[key0 + r][dim0 + 4a .. +3] and destination lane L receives
//   V[key0 + 0..3][dim0 + L].
//
// HD = true head dim; HDP = HD rounded up to 16 (contraction of Q K^T); HDV = HD
// rounded up to 32 (rows of O^T).  Pad lanes are zero-filled when staged.
//
// Bounded form (p.key_norm_max given).  The running reference only has to keep exp2(s - m)
// inside the floating-point range, and a score cannot exceed |q_i| max_j |k_j| in magnitude
// (Cauchy-Schwarz).  A wave whose query columns all satisfy |q_i| max|k| <= kBoundSlack can
// therefore keep the reference m = 0 for the whole key sequence: no maximum, no comparison,
// no reference update on any tile, and the vector work per score drops to exp2, packing and
// the row sum (a quarter of the vector instructions, and the cross-lane exchange with its
// wait, leave the loop).  Waves that do not satisfy it (large logits: peaked rows) run the
// lazy-maximum loop; the choice is wave-uniform.  Same softmax either way, another reference.
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;

template <int HD>
struct FlashCfg {
  static constexpr int HDP = (HD + 15) / 16 * 16;
  static constexpr int HDV = (HD + 31) / 32 * 32;
  static constexpr int KS = HDP / 16;        // k-steps of Q K^T
  static constexpr int CT = HDV / 32;        // O^T row tiles
  static constexpr int LDK = HDP + 8;        // LDS row of K tile (elements)
  // LDS row of the V tile.  A transpose read's 32 lanes cover 4 consecutive key rows x 64
  // bytes: the rows fall into disjoint bank ranges when the pitch is 64 or 192 bytes mod 256.
  static constexpr int LDV = (HDV % 128 == 32 || HDV % 128 == 96) ? HDV : HDV + 32;
  static constexpr int K_ELEMS = 64 * LDK, V_ELEMS = 64 * LDV;
  static constexpr size_t SMEM = (size_t)2 * (K_ELEMS + V_ELEMS) * sizeof(bf16_t);
  static constexpr int CH = HD / 8;          // 16-byte chunks per K row
  static constexpr int CHUNKS = 64 * CH;     // per tile, K and V alike
};

template <int HD, int QT, int NWV>
__global__ __launch_bounds__(64 * NWV, ((HD <= 64 || QT == 1) ? 2 : 1)) void k_attn_flash(AttnParams p) {
  constexpr int NT = 64 * NWV;              // threads
  constexpr int QROWS = 32 * QT * NWV;      // query rows per workgroup
  using C = FlashCfg<HD>;
  static_assert(HD % 8 == 0, "head dim must be a multiple of 8");
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  bf16_t* Ks = (bf16_t*)smem_raw;                 // [2][64][LDK]
  bf16_t* Vs = Ks + 2 * C::K_ELEMS;               // [2][64][LDV]

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int li = lane & 31, lh = lane >> 5;

  // problem and query tile of this workgroup
  const int qtiles = (p.nq + QROWS - 1) / QROWS;
  const long long work = xcd_work_item((long long)p.B * p.heads * p.groups * qtiles);
  if (work < 0) return;
  int bid = (int)work;
  const int qtile = bid % qtiles; bid /= qtiles;
  const int g = bid % p.groups; bid /= p.groups;
  const int head = bid % p.heads;
  const int b = bid / p.heads;
  const int kb = key_batch(p, b);

  const bf16_t* qbase = (const bf16_t*)p.q + ((size_t)b * p.heads + head) * (size_t)p.q_tokens * HD;
  const bf16_t* kbase = (const bf16_t*)p.k + (((size_t)kb * p.heads + head) * (size_t)p.k_tokens +
                                              (size_t)g * p.k_gstride) * HD;
  const bf16_t* vbase = (const bf16_t*)p.v + (((size_t)kb * p.heads + head) * (size_t)p.k_tokens +
                                              (size_t)g * p.k_gstride) * HD;

  // ---- Q fragments: B operand, lane (i, h) holds Q[row i][16s + 8h .. +7]
  bf16x8 qf[QT][C::KS];
  const int q0 = qtile * QROWS + wave * (32 * QT);
#pragma unroll
  for (int qt = 0; qt < QT; ++qt) {
    int qi = q0 + qt * 32 + li;
    qi = qi < p.nq ? qi : p.nq - 1;
    const bf16_t* qr = qbase + (size_t)(g * p.q_gstride + qi) * HD;
#pragma unroll
    for (int s = 0; s < C::KS; ++s) {
      const int c0 = s * 16 + lh * 8;
      bf16x8 v;
      if (c0 + 8 <= HD) v = *(const bf16x8*)(qr + c0);
      else {
#pragma unroll
        for (int e = 0; e < 8; ++e) v[e] = (bf16_t)0.0f;
      }
      if (p.scale_log2 != 1.0f) {            // queries not pre-multiplied by scale*log2(e): do it here
#pragma unroll
        for (int e = 0; e < 8; ++e) v[e] = (bf16_t)((float)v[e] * p.scale_log2);
      }
      qf[qt][s] = v;
    }
  }

  // ---- bounded form: is |q_i| max_j |k_j| (with a margin for the rounding of the norms) within
  //      the slack for every query column of this wave?  2^kBoundSlack times the number of
  //      keys times |v| stays far inside fp32, and so does 2^-kBoundSlack.
  constexpr float kBoundSlack = 40.0f;
  bool fast = false;
  if (p.key_norm_max != nullptr) {
    const float* kn = p.key_norm_max + ((size_t)kb * p.heads + head) * kKeyNormChunks;
    const float kmax = wave_max(kn[lane & (kKeyNormChunks - 1)]);
    float worst = 0.0f;
#pragma unroll
    for (int qt = 0; qt < QT; ++qt) {
      float ss = 0.0f;
#pragma unroll
      for (int s = 0; s < C::KS; ++s)
#pragma unroll
        for (int e = 0; e < 8; ++e) ss = __builtin_fmaf((float)qf[qt][s][e], (float)qf[qt][s][e], ss);
      worst = fmaxf(worst, ss);
    }
    worst += __shfl_xor(worst, 32, 64);        // at least the larger column's squared norm: a safe over-estimate
    fast = !__any(!(__builtin_sqrtf(worst) * kmax * 1.001f + 0.01f <= kBoundSlack));
  }

  f32x16 oacc[C::CT][QT];
#pragma unroll
  for (int c = 0; c < C::CT; ++c)
#pragma unroll
    for (int qt = 0; qt < QT; ++qt)
#pragma unroll
      for (int r = 0; r < 16; ++r) oacc[c][qt][r] = 0.0f;
  float lrow[QT] = {};             // this lane's partial sum (its 32 of the 64 keys per tile)

  // ---- staging: K and V tiles are both [64 keys][HD] row-major, one 16-byte chunk per thread and pass
  constexpr int CPT = (C::CHUNKS + NT - 1) / NT;
  bf16x8 rk[CPT], rv[CPT];
  const int nkt = (p.nk + 63) / 64;

  auto gload = [&](int kt) {
    const int j0 = kt * 64;
#pragma unroll
    for (int c = 0; c < CPT; ++c) {
      int ch = tid + c * NT;
      if (ch < C::CHUNKS) {
        int row = ch / C::CH, kc = ch % C::CH;
        int j = j0 + row; j = j < p.nk ? j : p.nk - 1;          // keys past nk are masked later
        rk[c] = *(const bf16x8*)(kbase + (size_t)j * HD + kc * 8);
        rv[c] = *(const bf16x8*)(vbase + (size_t)j * HD + kc * 8);
      }
    }
  };
  auto sstore = [&](int buf) {
    bf16_t* ks = Ks + buf * C::K_ELEMS;
    bf16_t* vs = Vs + buf * C::V_ELEMS;
#pragma unroll
    for (int c = 0; c < CPT; ++c) {
      int ch = tid + c * NT;
      if (ch < C::CHUNKS) {
        int row = ch / C::CH, kc = ch % C::CH;
        *(bf16x8*)(ks + row * C::LDK + kc * 8) = rk[c];
        *(bf16x8*)(vs + row * C::LDV + kc * 8) = rv[c];
      }
    }
  };

  // zero the pad columns once, both buffers: K head dims HD..HDP feed the contraction;
  // V head dims HD..HDV only produce output rows that are never stored, but keep them finite
  if constexpr (C::HDP != HD) {
    constexpr int PW = C::HDP - HD;
    for (int i = tid; i < 2 * 64 * PW; i += NT) {
      int buf = i / (64 * PW), r = i % (64 * PW);
      Ks[buf * C::K_ELEMS + (r / PW) * C::LDK + HD + r % PW] = (bf16_t)0.0f;
    }
  }
  if constexpr (C::HDV != HD) {
    constexpr int PW = C::HDV - HD;
    for (int i = tid; i < 2 * 64 * PW; i += NT) {
      int buf = i / (64 * PW), r = i % (64 * PW);
      Vs[buf * C::V_ELEMS + (r / PW) * C::LDV + HD + r % PW] = (bf16_t)0.0f;
    }
  }

  gload(0);
  sstore(0);
  __syncthreads();

  const int prow = (li & 0x13) | ((li & 4) << 1) | ((li & 8) >> 1);   // li with bits 2 and 3 swapped
  // transpose-read addressing: lane 4r + a of a 16-lane group reads key row r, dims 4a..4a+3 of the
  // group's 16 dims (lanes 16..31 and 48..63 serve dims 16..31 of the 32-dim tile)
  const int tr_row = (lane & 15) >> 2;
  const int tr_col = ((lane >> 4) & 1) * 16 + (lane & 3) * 4;

  // minus the running reference of each query column, splat over an accumulator: it is the C
  // operand of the first score MFMA of every tile, so no per-tile accumulator initialisation
  f32x16 negm[QT];
#pragma unroll
  for (int qt = 0; qt < QT; ++qt)
#pragma unroll
    for (int r = 0; r < 16; ++r) negm[qt][r] = 0.0f;
  bf16x2 ones;
  ones[0] = (bf16_t)1.0f; ones[1] = (bf16_t)1.0f;
  constexpr float kLazy = 8.0f;

  // One key tile.  MASKED: the tile holds keys past nk (only the last tile can).  NOMAX: the
  // reference is known to bound every score closely enough (bounded form): no maximum.
  auto tile = [&](int kt, auto masked_tag, auto nomax_tag) {
    constexpr bool MASKED = decltype(masked_tag)::value, NOMAX = decltype(nomax_tag)::value;
    const int buf = kt & 1;
    if (kt + 1 < nkt) gload(kt + 1);
    const bf16_t* ks = Ks + buf * C::K_ELEMS;
    const bf16_t* vs = Vs + buf * C::V_ELEMS;

    // ---- S^T = K Q^T - m (Q carries the factor scale*log2(e))
    f32x16 sacc[2][QT];
#pragma unroll
    for (int s = 0; s < C::KS; ++s) {
      bf16x8 kf[2];
#pragma unroll
      for (int a = 0; a < 2; ++a) kf[a] = *(const bf16x8*)(ks + (a * 32 + prow) * C::LDK + s * 16 + lh * 8);
#pragma unroll
      for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int qt = 0; qt < QT; ++qt)
          sacc[a][qt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[a], qf[qt][s], s == 0 ? negm[qt] : sacc[a][qt],
                                                                0, 0, 0);
    }

    // ---- mask keys past nk.  Register 4g+e of tile a is key 32a + 16(g/2) + 8h + 4(g%2) + e.
    if constexpr (MASKED) {
      const int rem = p.nk - kt * 64;
#pragma unroll
      for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int gg = 0; gg < 4; ++gg)
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            int key = 32 * a + 16 * (gg >> 1) + 8 * lh + 4 * (gg & 1) + e;
            if (key >= rem) {
#pragma unroll
              for (int qt = 0; qt < QT; ++qt) sacc[a][qt][4 * gg + e] = -INFINITY;
            }
          }
    }

    // ---- lazy reference update.  mx = (tile max) - m per query column.  Exponents up to
    //      kLazy are let through (p <= 2^kLazy, harmless in fp32/bf16); only when a column
    //      exceeds it, or on the first tile, is m moved and O, l, S rescaled.  The branch is
    //      wave-uniform and rare after the first tiles.
    if constexpr (!NOMAX) {
    float mx[QT];
#pragma unroll
    for (int qt = 0; qt < QT; ++qt) {
      float v = sacc[0][qt][0];
#pragma unroll
      for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int r = 0; r < 16; ++r) v = fmaxf(v, sacc[a][qt][r]);
      mx[qt] = fmaxf(v, __shfl_xor(v, 32, 64));     // finite: every tile has at least one valid key
    }
    const bool first = kt == 0;
    bool move = first;
#pragma unroll
    for (int qt = 0; qt < QT; ++qt) move = move || mx[qt] > kLazy;
    if (__builtin_expect(__any(move), 0)) {
#pragma unroll
      for (int qt = 0; qt < QT; ++qt) {
        const float delta = (first || mx[qt] > kLazy) ? mx[qt] : 0.0f;
        // on the first tile O and l are zero and exp2(-delta) may overflow: scale by 0 instead
        const float alpha = first ? 0.0f : __builtin_amdgcn_exp2f(-delta);
        lrow[qt] *= alpha;
#pragma unroll
        for (int c = 0; c < C::CT; ++c)
#pragma unroll
          for (int r = 0; r < 16; ++r) oacc[c][qt][r] *= alpha;
#pragma unroll
        for (int a = 0; a < 2; ++a)
#pragma unroll
          for (int r = 0; r < 16; ++r) sacc[a][qt][r] -= delta;
#pragma unroll
        for (int r = 0; r < 16; ++r) negm[qt][r] -= delta;
      }
    }
    }

    // ---- P = exp2(S), packed to bf16 in B-operand order; the row sum adds the rounded
    //      values (dot2 with ones), i.e. exactly what multiplies V.
    bf16x8 pf[QT][2][2];      // [qt][a][s2]
#pragma unroll
    for (int qt = 0; qt < QT; ++qt) {
      float sum = lrow[qt];
#pragma unroll
      for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int s2 = 0; s2 < 2; ++s2) {
          u32x4 pw;
#pragma unroll
          for (int x = 0; x < 4; ++x) {
            bf16x2 pp;
            pp[0] = (bf16_t)__builtin_amdgcn_exp2f(sacc[a][qt][8 * s2 + 2 * x]);
            pp[1] = (bf16_t)__builtin_amdgcn_exp2f(sacc[a][qt][8 * s2 + 2 * x + 1]);
            sum = __builtin_amdgcn_fdot2_f32_bf16(pp, ones, sum, false);
            pw[x] = __builtin_bit_cast(unsigned int, pp);
          }
          const bf16x8 pk = __builtin_bit_cast(bf16x8, pw);
          pf[qt][a][s2] = pk;
        }
      lrow[qt] = sum;
    }

    // ---- O^T += V^T P^T
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
      for (int s2 = 0; s2 < 2; ++s2) {
        bf16x8 vf[C::CT];
#pragma unroll
        for (int c = 0; c < C::CT; ++c) {
          const bf16_t* src = vs + (a * 32 + s2 * 16 + lh * 8 + tr_row) * C::LDV + c * 32 + tr_col;
          bf16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4*)src);
          bf16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4*)(src + 4 * C::LDV));
          vf[c] = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
        }
#pragma unroll
        for (int c = 0; c < C::CT; ++c)
#pragma unroll
          for (int qt = 0; qt < QT; ++qt)
            oacc[c][qt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[c], pf[qt][a][s2], oacc[c][qt], 0, 0, 0);
      }

    if (kt + 1 < nkt) sstore(buf ^ 1);
    __syncthreads();
  };

  const int nfull = p.nk / 64;
  using T_ = std::true_type; using F_ = std::false_type;
  if (fast) {
    for (int kt = 0; kt < nfull; ++kt) tile(kt, F_{}, T_{});
    if (nfull < nkt) tile(nfull, T_{}, T_{});
  } else {
    for (int kt = 0; kt < nfull; ++kt) tile(kt, F_{}, F_{});
    if (nfull < nkt) tile(nfull, T_{}, F_{});
  }

  // ---- finish: O / l, write token-major.  Lane (i, h) holds query column i, head
  //      dims 32c + 8g + 4h + e in register 4g + e.
  bf16_t* obase = (bf16_t*)p.out + (size_t)b * p.q_tokens * ((size_t)p.heads * HD) + (size_t)head * HD;
#pragma unroll
  for (int qt = 0; qt < QT; ++qt) {
    const float ltot = lrow[qt] + __shfl_xor(lrow[qt], 32, 64);
    const float inv = 1.0f / ltot;
    const int qi = q0 + qt * 32 + li;
    if (qi < p.nq) {
      bf16_t* orow = obase + (size_t)(g * p.q_gstride + qi) * ((size_t)p.heads * HD);
#pragma unroll
      for (int c = 0; c < C::CT; ++c)
#pragma unroll
        for (int gg = 0; gg < 4; ++gg) {
          const int dd = 32 * c + 8 * gg + 4 * lh;
          if (dd < HD) {
            bf16x4 ov;
#pragma unroll
            for (int e = 0; e < 4; ++e) ov[e] = (bf16_t)(oacc[c][qt][4 * gg + e] * inv);
            *(bf16x4*)(orow + dd) = ov;
          }
        }
    }
  }
}

template <int HD, int QT, int NWV>
static hipError_t run_flash(const AttnParams& p, hipStream_t s) {
  using C = FlashCfg<HD>;
  auto kern = k_attn_flash<HD, QT, NWV>;
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)C::SMEM);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  constexpr int QROWS = 32 * QT * NWV;
  long long blocks = (long long)p.B * p.heads * p.groups * ((p.nq + QROWS - 1) / QROWS);
  if (blocks == 0) return hipSuccess;
  blocks = (blocks + 7) / 8 * 8;                     // whole rounds over the 8 XCDs
  kern<<<(unsigned)blocks, 64 * NWV, C::SMEM, s>>>(p);
  return hipGetLastError();
}

// ---------------------------------------------------------------- few keys, many queries: keys and values resident in LDS
// Text cross-attention: every query of a (batch, head) attends to the same nk <= 128
// keys.  A workgroup stages them once (K [128][LDK], V [128][LDV], rows past nk zero) and
// its 4 waves then walk a range of query rows, 32 per wave and pass, with no further
// barrier: per pass a wave reads its Q fragments from global memory, forms S^T for all
// keys (K fragments as the A operand, in the flash kernel's permuted row order so that P
// is the B operand of the P V step as it stands), takes a plain two-pass softmax in
// registers (all keys are present: no running reference), multiplies by V through
// transpose reads and writes its 32 output rows.  The launch is bound by reading q and
// writing o once; the staged keys are shared by rows_per_chunk queries instead of 128.
template <int HD>
__global__ __launch_bounds__(256, 2) void k_attn_kvres(AttnParams p, int chunks, int rows_per_chunk) {
  using C = FlashCfg<HD>;
  constexpr int NKP = 128;                            // padded key count
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_kv[];
  bf16_t* Ks = (bf16_t*)smem_kv;                      // [128][LDK]
  bf16_t* Vs = Ks + NKP * C::LDK;                     // [128][LDV]

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int li = lane & 31, lh = lane >> 5;
  int bid = blockIdx.x;
  const int chunk = bid % chunks; bid /= chunks;
  const int g = bid % p.groups; bid /= p.groups;
  const int head = bid % p.heads;
  const int b = bid / p.heads;
  const int kb = key_batch(p, b);
  const bf16_t* qbase = (const bf16_t*)p.q + ((size_t)b * p.heads + head) * (size_t)p.q_tokens * HD;
  const bf16_t* kbase = (const bf16_t*)p.k + (((size_t)kb * p.heads + head) * (size_t)p.k_tokens +
                                              (size_t)g * p.k_gstride) * HD;
  const bf16_t* vbase = (const bf16_t*)p.v + (((size_t)kb * p.heads + head) * (size_t)p.k_tokens +
                                              (size_t)g * p.k_gstride) * HD;

  // ---- stage K and V: 16-byte chunks, zero for rows past nk and for the pad columns.  All
  //      loads of a thread are issued before its first LDS store (one exposed latency).
  {
    constexpr int KC = C::HDP / 8, VC = C::HDV / 8;   // chunks per staged row, pads included
    constexpr int KI = NKP * KC / 256, VI = NKP * VC / 256;
    static_assert(NKP * KC % 256 == 0 && NKP * VC % 256 == 0, "whole passes of the workgroup");
    bf16x8 zero;
#pragma unroll
    for (int e = 0; e < 8; ++e) zero[e] = (bf16_t)0.0f;
    bf16x8 rk[KI], rv[VI];
#pragma unroll
    for (int i = 0; i < KI; ++i) {
      const int ch = tid + i * 256, row = ch / KC, kc = ch % KC;
      rk[i] = zero;
      if (row < p.nk && kc * 8 < HD) rk[i] = *(const bf16x8*)(kbase + (size_t)row * HD + kc * 8);
    }
#pragma unroll
    for (int i = 0; i < VI; ++i) {
      const int ch = tid + i * 256, row = ch / VC, kc = ch % VC;
      rv[i] = zero;
      if (row < p.nk && kc * 8 < HD) rv[i] = *(const bf16x8*)(vbase + (size_t)row * HD + kc * 8);
    }
#pragma unroll
    for (int i = 0; i < KI; ++i) {
      const int ch = tid + i * 256, row = ch / KC, kc = ch % KC;
      *(bf16x8*)(Ks + row * C::LDK + kc * 8) = rk[i];
    }
#pragma unroll
    for (int i = 0; i < VI; ++i) {
      const int ch = tid + i * 256, row = ch / VC, kc = ch % VC;
      *(bf16x8*)(Vs + row * C::LDV + kc * 8) = rv[i];
    }
  }
  __syncthreads();

  const int na = (p.nk + 31) / 32;                    // 32-key groups in use (1..4), wave-uniform
  const int rem_last = p.nk - 32 * (na - 1);          // keys in the last of them (1..32)
  // added to the last group's scores: -inf on the registers of keys past nk.  Register 4g+e
  // of a group is its key 16(g/2) + 8h + 4(g%2) + e.
  f32x16 pen, zero16;
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    zero16[r] = 0.0f;
    pen[r] = (16 * (r >> 3) + 8 * lh + 4 * ((r >> 2) & 1) + (r & 3) >= rem_last) ? -INFINITY : 0.0f;
  }
  const int prow = (li & 0x13) | ((li & 4) << 1) | ((li & 8) >> 1);   // li with bits 2 and 3 swapped
  const int tr_row = (lane & 15) >> 2;
  const int tr_col = ((lane >> 4) & 1) * 16 + (lane & 3) * 4;
  bf16x2 ones;
  ones[0] = (bf16_t)1.0f; ones[1] = (bf16_t)1.0f;
  bf16_t* obase = (bf16_t*)p.out + (size_t)b * p.q_tokens * ((size_t)p.heads * HD) + (size_t)head * HD;

  const int r_begin = chunk * rows_per_chunk;
  const int r_end = min(p.nq, r_begin + rows_per_chunk);
  // Q fragments: B operand, lane (i, h) holds Q[row i][16s + 8h .. +7].  The rows of the
  // next pass are requested before the current pass is computed.
  auto load_q = [&](int q0, bf16x8 (&dst)[C::KS]) {
    int qi = q0 + li;
    qi = qi < p.nq ? qi : p.nq - 1;
    const bf16_t* qr = qbase + (size_t)(g * p.q_gstride + qi) * HD;
#pragma unroll
    for (int s = 0; s < C::KS; ++s) {
      const int c0 = s * 16 + lh * 8;
      if (c0 + 8 <= HD) dst[s] = *(const bf16x8*)(qr + c0);
      else {
#pragma unroll
        for (int e = 0; e < 8; ++e) dst[s][e] = (bf16_t)0.0f;
      }
    }
  };
  // The passes of this wave, with the number of key groups a compile-time constant so that
  // the four score chains and their LDS reads are scheduled together (no branch per group).
  auto passes = [&](auto na_tag) {
  constexpr int NA = decltype(na_tag)::value;
  bf16x8 qn[C::KS];
  if (r_begin + wave * 32 < r_end) load_q(r_begin + wave * 32, qn);
  for (int q0 = r_begin + wave * 32; q0 < r_end; q0 += 4 * 32) {
    bf16x8 qf[C::KS];
#pragma unroll
    for (int s = 0; s < C::KS; ++s) {
      qf[s] = qn[s];
      if (p.scale_log2 != 1.0f) {
#pragma unroll
        for (int e = 0; e < 8; ++e) qf[s][e] = (bf16_t)((float)qf[s][e] * p.scale_log2);
      }
    }
    if (q0 + 4 * 32 < r_end) load_q(q0 + 4 * 32, qn);

    // ---- S^T = K Q^T for every key group in use.  Register 4g+e of group a is key
    //      32a + 16(g/2) + 8h + 4(g%2) + e.
    f32x16 sacc[NA];
#pragma unroll
    for (int s = 0; s < C::KS; ++s)
#pragma unroll
      for (int a = 0; a < NA; ++a) {
        const bf16x8 kf = *(const bf16x8*)(Ks + (a * 32 + prow) * C::LDK + s * 16 + lh * 8);
        sacc[a] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[s], s == 0 ? zero16 : sacc[a], 0, 0, 0);
      }
    sacc[NA - 1] += pen;                              // only the last group can hold keys past nk
    float mx = sacc[0][0];
#pragma unroll
    for (int a = 0; a < NA; ++a)
#pragma unroll
      for (int r = 0; r < 16; ++r) mx = fmaxf(mx, sacc[a][r]);
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64));           // finite: key 0 is valid

    // ---- P = exp2(S - max) rounded to bf16 in B-operand order; O^T += V^T P^T
    f32x16 oacc[C::CT];
    float sum = 0.0f;
#pragma unroll
    for (int a = 0; a < NA; ++a) {
#pragma unroll
        for (int s2 = 0; s2 < 2; ++s2) {
          u32x4 pw;
#pragma unroll
          for (int x = 0; x < 4; ++x) {
            bf16x2 pp;
            pp[0] = (bf16_t)__builtin_amdgcn_exp2f(sacc[a][8 * s2 + 2 * x] - mx);
            pp[1] = (bf16_t)__builtin_amdgcn_exp2f(sacc[a][8 * s2 + 2 * x + 1] - mx);
            sum = __builtin_amdgcn_fdot2_f32_bf16(pp, ones, sum, false);
            pw[x] = __builtin_bit_cast(unsigned int, pp);
          }
          const bf16x8 pk = __builtin_bit_cast(bf16x8, pw);
#pragma unroll
          for (int c = 0; c < C::CT; ++c) {
            const bf16_t* src = Vs + (a * 32 + s2 * 16 + lh * 8 + tr_row) * C::LDV + c * 32 + tr_col;
            const bf16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4*)src);
            const bf16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4*)(src + 4 * C::LDV));
            const bf16x8 vf = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
            oacc[c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pk, (a == 0 && s2 == 0) ? zero16 : oacc[c], 0, 0, 0);
          }
        }
      }

    // ---- O / l, token-major.  Lane (i, h) holds query column i, head dims 32c + 8g + 4h + e.
    const float inv = 1.0f / (sum + __shfl_xor(sum, 32, 64));
    const int qi = q0 + li;
    if (qi < p.nq) {
      bf16_t* orow = obase + (size_t)(g * p.q_gstride + qi) * ((size_t)p.heads * HD);
#pragma unroll
      for (int c = 0; c < C::CT; ++c)
#pragma unroll
        for (int gg = 0; gg < 4; ++gg) {
          const int dd = 32 * c + 8 * gg + 4 * lh;
          if (dd < HD) {
            bf16x4 ov;
#pragma unroll
            for (int e = 0; e < 4; ++e) ov[e] = (bf16_t)(oacc[c][4 * gg + e] * inv);
            *(bf16x4*)(orow + dd) = ov;
          }
        }
    }
  }
  };
  switch (na) {
    case 1: passes(std::integral_constant<int, 1>{}); break;
    case 2: passes(std::integral_constant<int, 2>{}); break;
    case 3: passes(std::integral_constant<int, 3>{}); break;
    default: passes(std::integral_constant<int, 4>{}); break;
  }
}

template <int HD>
static hipError_t run_kvres(const AttnParams& p, hipStream_t s) {
  using C = FlashCfg<HD>;
  constexpr size_t smem = (size_t)128 * (C::LDK + C::LDV) * sizeof(bf16_t);
  const long long problems = (long long)p.B * p.heads * p.groups;
  if (problems == 0) return hipSuccess;
  // about 1024 workgroups (two rounds of two per CU; measured best among 256..2048) where the
  // queries allow it; a chunk is a multiple of the 128 rows the four waves cover per pass
  const int t128 = (p.nq + 127) / 128;
  long long want = (1024 + problems - 1) / problems;
  const int chunks = (int)(want < 1 ? 1 : want > t128 ? t128 : want);
  const int rows_per_chunk = (t128 + chunks - 1) / chunks * 128;
  const int used = (p.nq + rows_per_chunk - 1) / rows_per_chunk;
  if (problems * used > 0x7fffffffLL) return hipErrorInvalidValue;
  k_attn_kvres<HD><<<(unsigned)(problems * used), 256, smem, s>>>(p, used, rows_per_chunk);
  return hipGetLastError();
}

// Keys and values resident: few keys shared by many queries (text cross-attention).
static bool kvres_ok(const AttnParams& p) { return p.nk <= 128 && p.nq >= 512; }

// The flash kernel needs unit-stride tokens inside a group, 16-byte aligned rows
// (head dim a multiple of 8 elements) and head dims it is instantiated for.
static bool flash_ok(const AttnParams& p) {
  if (p.hd != 64 && p.hd != 72) return false;
  if (p.q_istride != 1 || p.k_istride != 1) return false;
  if (p.nk < 1 || p.nq < 1) return false;
  if ((((uintptr_t)p.q | (uintptr_t)p.k | (uintptr_t)p.v | (uintptr_t)p.out) & 15) != 0) return false;
  return true;
}

// ---------------------------------------------------------------- largest key norm per (key batch, head)
// Partial maxima over kKeyNormChunks ranges of the key rows; the flash kernel takes their
// maximum.  Eight lanes share a row of 64 elements (one 16-byte load each, coalesced), else
// one thread per row.  A maximum is order-independent: the result is bitwise repeatable.
template <int HD>
__global__ __launch_bounds__(256) void k_key_norm_max(const bf16_t* __restrict__ k, int k_tokens, float* __restrict__ out) {
  __shared__ float sh[4];
  const int chunk = blockIdx.x, bh = blockIdx.y;
  const int per = (k_tokens + kKeyNormChunks - 1) / kKeyNormChunks;
  const int r0 = chunk * per, r1 = min(k_tokens, r0 + per);
  const bf16_t* base = k + (size_t)bh * k_tokens * HD;
  float best = 0.0f;
  if constexpr (HD == 64) {
    const int sub = threadIdx.x & 7;
    for (int r = r0 + (threadIdx.x >> 3); r < r1; r += 32) {
      const bf16x8 v = *(const bf16x8*)(base + (size_t)r * HD + sub * 8);
      float ss = 0.0f;
#pragma unroll
      for (int e = 0; e < 8; ++e) ss = __builtin_fmaf((float)v[e], (float)v[e], ss);
      ss += __shfl_xor(ss, 1, 64);
      ss += __shfl_xor(ss, 2, 64);
      ss += __shfl_xor(ss, 4, 64);
      best = fmaxf(best, ss);
    }
  } else {
    for (int r = r0 + threadIdx.x; r < r1; r += 256) {
      float ss = 0.0f;
#pragma unroll
      for (int c = 0; c < HD / 8; ++c) {
        const bf16x8 v = *(const bf16x8*)(base + (size_t)r * HD + c * 8);
#pragma unroll
        for (int e = 0; e < 8; ++e) ss = __builtin_fmaf((float)v[e], (float)v[e], ss);
      }
      best = fmaxf(best, ss);
    }
  }
  best = wave_max(best);
  if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = best;
  __syncthreads();
  if (threadIdx.x == 0)
    out[(size_t)bh * kKeyNormChunks + chunk] = __builtin_sqrtf(fmaxf(fmaxf(sh[0], sh[1]), fmaxf(sh[2], sh[3])));
}

hipError_t launch_key_norm_max(const void* k, int KB, int heads, int k_tokens, int hd, float* out, hipStream_t s) {
  if ((long long)KB * heads == 0) return hipSuccess;
  if (k_tokens < 1 || (long long)KB * heads > 65535 || (((uintptr_t)k) & 15) != 0) return hipErrorInvalidValue;
  dim3 grid(kKeyNormChunks, (unsigned)(KB * heads));
  if (hd == 64) k_key_norm_max<64><<<grid, 256, 0, s>>>((const bf16_t*)k, k_tokens, out);
  else if (hd == 72) k_key_norm_max<72><<<grid, 256, 0, s>>>((const bf16_t*)k, k_tokens, out);
  else return hipErrorInvalidValue;
  return hipGetLastError();
}

// The bound pays once there are many key tiles per query tile; the few-keys kernel and the
// short-sequence kernels take no reference from it.
bool attention_uses_key_norms(int bf16, const AttnParams& p) {
  return bf16 && flash_ok(p) && !kvres_ok(p) && p.nk >= 2048 && p.groups == 1 && !p.kv_shared_tail;
}

hipError_t launch_attention(int bf16, const AttnParams& p, int impl, hipStream_t s) {
  // every kernel reads rows with 16-byte loads
  if ((((uintptr_t)p.q | (uintptr_t)p.k | (uintptr_t)p.v | (uintptr_t)p.out) & 15) != 0) return hipErrorInvalidValue;
  if (!bf16) return dispatch_plain<float>(p, impl != 1, s);
  if (impl == 0 && flash_ok(p) && kvres_ok(p)) {
    if (p.hd == 64) return run_kvres<64>(p, s);
    if (p.hd == 72) return run_kvres<72>(p, s);
  }
  if (impl == 0 && flash_ok(p)) {
    // One 32-query tile per wave (half the registers, twice the workgroups) when the key
    // sequence is short: the work per workgroup is then a few tiles and the launch lives
    // on how many workgroups a CU can hold, not on operand reuse.
    // Long sequences with head dim 64 take 8 waves per workgroup: 512 query rows share
    // each staged key/value tile, which halves the L2 -> LDS traffic per FLOP (-3 %).
    const bool narrow = p.nk <= 512;
    if (p.hd == 64)
      return narrow ? run_flash<64, 1, 4>(p, s) : p.nq >= 4096 ? run_flash<64, 2, 8>(p, s) : run_flash<64, 2, 4>(p, s);
    if (p.hd == 72) return narrow ? run_flash<72, 1, 4>(p, s) : run_flash<72, 2, 4>(p, s);
  }
  if (impl == 0 && short_mfma_ok(p)) {
    if (p.hd == 64) return run_short_mfma<64>(p, s);
    if (p.hd == 72) return run_short_mfma<72>(p, s);
  }
  return dispatch_plain<bf16_t>(p, impl != 1, s);
}

}  // namespace fc
