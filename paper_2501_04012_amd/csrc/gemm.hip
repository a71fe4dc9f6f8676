// Linear layers: C[M,N] = A[M,K] * Wt[N,K]^T with fused epilogues.
//   bf16: MFMA (v_mfma_f32_32x32x16_bf16) kernel, operands DMA'd into swizzled LDS tiles,
//         fp32 accumulation.
//   fp32: plain LDS-tiled FMA kernel (the fp32 configuration is tiny and
//         launch-bound; it exists for the 1e-4 parity bar, not for speed).
// Both operands are contiguous along K ("TN" form): activations are [tokens, K]
// and weights are stored [out, in].
#include <type_traits>
#include "common.h"

namespace fc {

// ---------------------------------------------------------------- bf16 MFMA kernel, direct-to-LDS
// (k_gemm_dlds_any: the general form, any K that is a multiple of 64 and operands of any size.
// k_gemm_dlds further down is the one the workloads run; what is said here about tiles, layout,
// tile order and units of work holds for both.)
// Block tile BM x BN x BK, NW = WR x WC waves, each wave owns a (BM/WR) x (BN/WC) tile built
// from 32x32 MFMA accumulators.  MFMA operand layout (32x32x16, wave64), lane = i + 32*h:
//   A: row i of the 32-row tile, k = 8h .. 8h+7        (8 bf16 = one 16-byte LDS read)
//   B: column i of the 32-col tile, k = 8h .. 8h+7
//   D: column i, rows 8g + 4h + e for register 4g + e   (g, e in 0..3)
// The operand tiles go from global memory straight into LDS (global_load_lds_dwordx4: lane l's 16 bytes land at
// base + 16 l), S stages deep, with no register staging and no ds_write.
//
// LDS layout of a stage: BM rows of A then BN rows of B, BK*2 bytes each, unpadded.
// A 256-byte LDS line holds RPL = 128/BK rows; chunk kc (16 bytes) of row r sits at
//   line r/RPL, slot (r % RPL) * CPR + (kc ^ ((r/RPL) % CPR)),   CPR = BK/8,
// so that the 16 rows a ds_read_b128 touches at one kc fall into 16 distinct slots
// (no bank conflicts).  Because the DMA fixes the LDS position per lane, the swizzle
// is applied on the global side: each lane fetches the chunk that belongs in its slot.
//
// Pipeline per K tile: wait until this tile's loads have landed (vmcnt), barrier
// (publishes every wave's part and frees the stage read in the previous iteration),
// issue the loads of tile kt+S-1 into that stage, then run the MFMAs of tile kt.
//
// Tile order.  Workgroup ids are dealt round-robin to the 8 XCDs, each with its own L2.
// Id -> tile index is chosen so that 32 workgroups running together on one XCD hold 32
// consecutive tile indices, and consecutive indices walk GM = 8 tile rows before moving to
// the next tile column: an XCD works on an 8 x 4 patch of C and streams 8 + 4 operand
// panels through its L2 instead of 1 + 32.
typedef __attribute__((address_space(3))) void lds_void;
typedef __attribute__((address_space(1))) const void gbl_void;

// s_waitcnt vmcnt(N) only (gfx9 encoding: vmcnt[3:0] | expcnt[6:4] | lgkmcnt[11:8] | vmcnt_hi[15:14])
template <int N> __device__ __forceinline__ void wait_vm() {
  __builtin_amdgcn_s_waitcnt((N & 0xF) | ((N >> 4) << 14) | (0x7 << 4) | (0xF << 8));
}

// Split-K partial tiles: a wave's accumulators in the order (i, j, register quad, lane), 16
// bytes per lane, so that every wave-store covers 1 KB of consecutive addresses.  The
// fix-up kernel reads them back in the same order: no layout knowledge beyond this pair.
template <int TM, int TN>
__device__ __forceinline__ void store_partial(const f32x16 (&acc)[TM][TN], float* tile) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  f32x4* dst = (f32x4*)tile + (size_t)wave * (TM * TN * 4 * 64) + lane;
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        f32x4 v = {acc[i][j][4 * q], acc[i][j][4 * q + 1], acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]};
        dst[((i * TN + j) * 4 + q) * 64] = v;
      }
}
template <int TM, int TN>
__device__ __forceinline__ void add_partial(f32x16 (&acc)[TM][TN], const float* tile, bool first) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const f32x4* src = (const f32x4*)tile + (size_t)wave * (TM * TN * 4 * 64) + lane;
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const f32x4 v = src[((i * TN + j) * 4 + q) * 64];
#pragma unroll
        for (int e = 0; e < 4; ++e) acc[i][j][4 * q + e] = first ? v[e] : acc[i][j][4 * q + e] + v[e];
      }
}

// Epilogue of one BM x BN tile, shared by the product kernel and the split-K fix-up: bias,
// activation / gate / q scale, conversion and stores.  `stage` is an idle operand stage of
// the workgroup (output rows pass through it), sbias / sgate the tile's bias and gate slices.
template <int BM, int BN, int BK, int WR, int WC, typename Epi>
__device__ __forceinline__ void gemm_tile_epilogue(const f32x16 (&acc)[BM / WR / 32][BN / WC / 32], unsigned char* stage,
                                                   const float* sbias, const float* sgate, const Epi& epi, int bm0,
                                                   int bn0, int M, int N) {
  constexpr int NW = WR * WC;
  constexpr int WTM = BM / WR, WTN = BN / WC;
  constexpr int TM = WTM / 32, TN = WTN / 32;
  constexpr int STAGE_BYTES = (BM + BN) * BK * 2;
  // The lane and wave numbers pass through an empty asm: everything derived from them here (LDS
  // staging offsets, output offsets) is then computed inside the epilogue.  Left to itself the
  // compiler computes these per-lane constants once, ahead of the persistent tile loop, finds no
  // registers for them across the K loop and reloads them from scratch in the epilogue, each
  // reload waiting for the stores issued before it.
  int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  asm volatile("" : "+v"(lane), "+v"(wave));
  const int wr = wave / WC, wc = wave % WC;
  const int li = lane & 31, lh = lane >> 5;
  if constexpr (Epi::kRowRuns) {
    // Accumulator lane (li, lh) holds row m = 32 i + li, columns 32 j + 8 g + 4 lh + e.
    // The finished bf16 values go, 32 rows at a time, through this wave's slice of the
    // idle operand stage, swizzled by 16-byte chunk, and leave as 16-byte stores: a
    // wave-store covers whole 2 WTN-byte row segments instead of 2 bytes per lane.
    constexpr int ROWB = WTN * 2;                     // bytes per staged row
    constexpr int CPRW = WTN / 8;                     // 16-byte chunks per row
    constexpr int RPLC = 256 / ROWB > 0 ? 256 / ROWB : 1;   // rows per 256-byte LDS line
    constexpr bool POW2 = (CPRW & (CPRW - 1)) == 0;
    static_assert(NW * 32 * ROWB <= STAGE_BYTES, "staging area");
    static_assert((32 * CPRW) % 64 == 0, "whole wave-stores");
    // chunk position inside a row: XOR with the line index (power-of-two rows), else a rotation
    auto swz = [](int row, int chunk) {
      return POW2 ? (chunk ^ ((row / RPLC) & (CPRW - 1))) : (chunk + row) % CPRW;
    };
    unsigned char* cst = stage + wave * (32 * ROWB);
    const int wave_u = __builtin_amdgcn_readfirstlane(wave), wr_u = wave_u / WC, wc_u = wave_u % WC;   // known to be uniform
#pragma unroll
    for (int i = 0; i < TM; ++i) {
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int gq = 0; gq < 4; ++gq) {
          const int n0 = bn0 + wc * WTN + j * 32 + gq * 8 + lh * 4;
          float v[4] = {acc[i][j][4 * gq], acc[i][j][4 * gq + 1], acc[i][j][4 * gq + 2], acc[i][j][4 * gq + 3]};
          epi.apply4(n0, v, sbias + (n0 - bn0), sgate + (n0 - bn0));
          bf16x4 o;
#pragma unroll
          for (int e = 0; e < 4; ++e) o[e] = (bf16_t)v[e];
          *(bf16x4*)(cst + li * ROWB + (swz(li, 4 * j + gq) << 4) + lh * 8) = o;
        }
      constexpr int NIT = 32 * CPRW / 64;
      if (bm0 + BM <= M && bn0 + BN <= N) {
        // a whole tile (wave-uniform): all reads of the pass in flight together, no predicates,
        // and for the row-major outputs a wave-uniform row pointer plus a 32-bit lane offset
        constexpr int RB = NIT % 4 == 0 ? 4 : NIT % 3 == 0 ? 3 : NIT % 2 == 0 ? 2 : 1;   // reads in flight together
        const int m0 = bm0 + wr_u * WTM + i * 32, nb = bn0 + wc_u * WTN;
        // per-head outputs: with 64 % CPRW == 0 a lane keeps its column over all passes
        constexpr bool kFixedCol = !Epi::kLinearOut && 64 % CPRW == 0;
        bf16_t* colp = nullptr;
        if constexpr (kFixedCol) colp = epi.head_col_ptr(nb + (lane % CPRW) * 8);
#pragma unroll
        for (int it0 = 0; it0 < NIT; it0 += RB) {
          bf16x8 o[RB];
#pragma unroll
          for (int r = 0; r < RB; ++r) {
            const int idx = (it0 + r) * 64 + lane;
            const int row = idx / CPRW, chunk = idx % CPRW;
            o[r] = *(const bf16x8*)(cst + row * ROWB + (swz(row, chunk) << 4));
          }
#pragma unroll
          for (int r = 0; r < RB; ++r) {
            const int idx = (it0 + r) * 64 + lane;
            const int row = idx / CPRW, chunk = idx % CPRW;
            if constexpr (Epi::kLinearOut)
              __builtin_nontemporal_store(o[r], (bf16x8*)(epi.row_ptr(m0, nb) + ((unsigned)row * (unsigned)epi.P.ldo + (unsigned)chunk * 8u)));
            else if constexpr (kFixedCol)
              __builtin_nontemporal_store(o[r], (bf16x8*)(colp + epi.head_row_off(m0 + row)));
            else
              __builtin_nontemporal_store(o[r], (bf16x8*)epi.run8(m0 + row, nb + chunk * 8));
          }
        }
      } else {
#pragma unroll
        for (int it = 0; it < NIT; ++it) {
          const int idx = it * 64 + lane;
          const int row = idx / CPRW, chunk = idx % CPRW;
          const bf16x8 o = *(const bf16x8*)(cst + row * ROWB + (swz(row, chunk) << 4));
          const int m = bm0 + wr * WTM + i * 32 + row, n0 = bn0 + wc * WTN + chunk * 8;
          if (m < M && n0 < N) __builtin_nontemporal_store(o, (bf16x8*)epi.run8(m, n0));
        }
      }
    }
  } else {
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        const auto col = epi.col(bn0 + wc * WTN + j * 32 + li);
#pragma unroll
        for (int gq = 0; gq < 4; ++gq) {
          const int m0 = bm0 + wr * WTM + i * 32 + gq * 8 + lh * 4;
          float v[4] = {acc[i][j][4 * gq], acc[i][j][4 * gq + 1], acc[i][j][4 * gq + 2], acc[i][j][4 * gq + 3]};
          epi.store4(col, m0, v);
        }
      }
  }
}

template <int BM, int BN, int BK, int WR, int WC, int S, typename Epi>
__global__ __launch_bounds__(WR * WC * 64) void k_gemm_dlds_any(const bf16_t* __restrict__ A,
                                                            const bf16_t* __restrict__ Wt, int M, int N, int K,
                                                            int tiles_m, int tiles_n, Epi epi, int splits,
                                                            float* __restrict__ partial) {
  static_assert(S == 2, "two stages: one being multiplied, one in flight");
  constexpr int NW = WR * WC;
  constexpr int WTM = BM / WR, WTN = BN / WC;
  constexpr int TM = WTM / 32, TN = WTN / 32;
  constexpr int CPR = BK / 8;              // 16-byte chunks per row
  constexpr int RPL = 16 / CPR;            // rows per 256-byte LDS line
  constexpr int RW = 4 * RPL;              // rows per wave-load (1 KB)
  constexpr int ROWS = BM + BN;
  constexpr int WL = ROWS / RW;            // wave-loads per stage
  constexpr int LPW = WL / NW;             // per wave
  constexpr int STAGE_BYTES = ROWS * BK * 2;
  static_assert(WL % NW == 0, "loads must divide among waves");
  static_assert(BM % RW == 0, "A/B boundary must fall between wave-loads");

  extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
  // bias and gate of the current tile's BN columns, 1 KB each behind the two operand stages:
  // fetched by DMA with the tile's first operand loads, read by the epilogue from LDS.  With
  // loads from global memory in the epilogue every one of them was waited for in turn, behind
  // the stores issued before it (the counter is shared): 10 000 cycles per 256x192 tile.
  float* const sbias = (float*)(smem + S * STAGE_BYTES);
  float* const sgate = sbias + 256;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wr = wave / WC, wc = wave % WC;
  const int li = lane & 31, lh = lane >> 5;
  // an absent bias reads as zeros, an absent gate as ones (written once: no DMA touches them)
  if constexpr (Epi::kRowRuns) {
    if (tid < 256) {
      if (!epi.P.bias) sbias[tid] = 0.0f;
      if (Epi::kHasGate && !epi.P.gate) sgate[tid] = 1.0f;
    }
  }

  // ---- tiles of this workgroup: virtual ids blockIdx.x, + gridDim.x, ... below `padded`
  // (the grid may be one workgroup per slot of the chip: persistent).  gridDim.x is a
  // multiple of 8, so every id of a workgroup lands on its XCD.
  // Split-K remainder (splits >= 2; the grid is then 256 workgroups): the tiles of the last,
  // partial round of 256 are each cut into `splits` ranges of K and dealt to the workgroups
  // of that round, which store their fp32 accumulators to `partial` (slot = tile-in-round *
  // splits + range) instead of running the epilogue; k_gemm_fixup adds the ranges in a
  // fixed order and finishes the tile.  A round that leaves most of the chip idle for the
  // time of a whole tile thus costs 1 / splits of it.
  const int total = tiles_m * tiles_n;
  const int nkt = K / BK;
  const int full = total / 256 * 256, rem = total - full;
  // virtual ids run over the whole rounds and, behind them, the units of the last one
  const int padded = splits >= 2 ? ((full + rem * splits + 7) & ~7) : (total + 255) / 256 * 256;
  auto tile_of = [&](int vb, int& bm0, int& bn0, int& kt0, int& kt1, int& slot) {
    const int xcd = vb & 7, local = vb >> 3;
    int t = ((local >> 5) * 8 + xcd) * 32 + (local & 31);
    kt0 = 0; kt1 = nkt; slot = -1;
    if (splits >= 2 && vb >= full) {
      const int w = vb - full;
      if (w >= rem * splits) return false;
      const int r = w / rem;
      t = full + w % rem;
      kt0 = r * nkt / splits; kt1 = (r + 1) * nkt / splits;
      slot = (w % rem) * splits + r;
    }
    if (t >= total) return false;
    constexpr int GM = 8;
    const int per_group = GM * tiles_n;
    const int group = t / per_group;
    const int first_m = group * GM;
    const int gsz = min(tiles_m - first_m, GM);
    bm0 = (first_m + (t % per_group) % gsz) * BM;
    bn0 = ((t % per_group) / gsz) * BN;
    return true;
  };
  // advances vb to this workgroup's next unit of work: a tile, or a K range of a split tile
  auto next_tile = [&](int& vb, int& bm0, int& bn0, int& kt0, int& kt1, int& slot) {
    for (vb += gridDim.x; vb < padded; vb += gridDim.x)
      if (tile_of(vb, bm0, bn0, kt0, kt1, slot)) return true;
    return false;
  };

  // ---- global source pointers of this lane for its LPW wave-loads of a tile
  auto sources = [&](int bm0, int bn0, int kt_first, const bf16_t* (&gp)[LPW]) {
#pragma unroll
    for (int j = 0; j < LPW; ++j) {
      const int wl = wave + NW * j;
      const int line_in = lane >> 4, slot = lane & 15;
      const int row = wl * RW + line_in * RPL + slot / CPR;
      const int kc = (slot % CPR) ^ ((wl * 4 + line_in) % CPR);
      if (row < BM) {
        int gm = bm0 + row; gm = gm < M ? gm : M - 1;
        gp[j] = A + (size_t)gm * K + kc * 8 + kt_first * BK;
      } else {
        int gn = bn0 + row - BM; gn = gn < N ? gn : N - 1;
        gp[j] = Wt + (size_t)gn * K + kc * 8 + kt_first * BK;
      }
    }
  };
  auto issue = [&](const bf16_t* const (&gp)[LPW], int kt, int stage) {
#pragma unroll
    for (int j = 0; j < LPW; ++j) {
      const int wl = wave + NW * j;
      __builtin_amdgcn_global_load_lds((gbl_void*)(gp[j] + (size_t)kt * BK),
                                       (lds_void*)(smem + stage * STAGE_BYTES + wl * 1024), 16, 0, 0);
    }
  };

  auto issue_vectors = [&](int bn0) {
    if constexpr (Epi::kRowRuns) {
      int n = bn0 + lane * 4;
      n = n < N ? n : 0;                           // columns past N are never stored
      if (wave == 0 && epi.P.bias)
        __builtin_amdgcn_global_load_lds((gbl_void*)(epi.P.bias + n), (lds_void*)sbias, 16, 0, 0);
      if (Epi::kHasGate && wave == 1 && epi.P.gate)
        __builtin_amdgcn_global_load_lds((gbl_void*)(epi.P.gate + n), (lds_void*)sgate, 16, 0, 0);
    }
  };

  // ---- fragment read offsets (bytes within a stage)
  const int ra = wr * WTM + li, rb = BM + wc * WTN + li;
  const int a_row = (ra / RPL) * 256 + (ra % RPL) * CPR * 16, a_x = (ra / RPL) % CPR;
  const int b_row = (rb / RPL) * 256 + (rb % RPL) * CPR * 16, b_x = (rb / RPL) % CPR;
  constexpr int TILE_STRIDE = (32 / RPL) * 256;   // 32 rows further down

  int vb = (int)blockIdx.x - (int)gridDim.x, bm0 = 0, bn0 = 0, kt0 = 0, kt1 = 0, slot = -1;
  if (!next_tile(vb, bm0, bn0, kt0, kt1, slot)) return;
  const bf16_t* gp[LPW];
  sources(bm0, bn0, kt0, gp);
  int nk = kt1 - kt0;                              // K tiles of the current unit; gp points at its first one
  issue(gp, 0, 0);
  wait_vm<0>();
  __builtin_amdgcn_s_barrier();
  int g = 0;                                       // K tiles consumed so far; the current one sits in stage g & 1

  // One pass per output tile.  The operand pipeline runs across tiles: the first K tile of
  // the workgroup's next output tile is requested while the last K tile of this one is
  // being multiplied, and lands during the epilogue.
  for (;;) {
    int nvb = vb, nbm0 = 0, nbn0 = 0, nkt0 = 0, nkt1 = 0, nslot = -1;
    const bool has_next = next_tile(nvb, nbm0, nbn0, nkt0, nkt1, nslot);
    const bf16_t* gpn[LPW];
    if (has_next) sources(nbm0, nbn0, nkt0, gpn);

    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

    for (int kt = 0; kt < nk; ++kt, ++g) {
      if (kt > 0) {                                // the unit's first K tile was awaited and published before the previous epilogue
        wait_vm<0>();
        __builtin_amdgcn_s_barrier();
      }
      if (kt == 0) issue_vectors(bn0);
      if (kt + 1 < nk) issue(gp, kt + 1, (g + 1) & 1);
      else if (has_next) issue(gpn, 0, (g + 1) & 1);
      const unsigned char* st = smem + (g & 1) * STAGE_BYTES;
      // Fragment reads run one 16-wide k-slice ahead of the MFMAs that consume them, in
      // two register sets.  The scheduling groups below pin the instruction order the
      // compiler would otherwise collapse into read-all / wait / multiply: after the first
      // slice's reads, every read of slice ks+1 is paired with one MFMA of slice ks, so the
      // LDS latency is spent under matrix work of the same wave.
      constexpr int KS = BK / 16;
      bf16x8 fa[2][TM], fb[2][TN];
      auto load = [&](int ks, bf16x8 (&xa)[TM], bf16x8 (&xb)[TN]) {
        const unsigned char* pa = st + a_row + (((2 * ks + lh) ^ a_x) << 4);
        const unsigned char* pb = st + b_row + (((2 * ks + lh) ^ b_x) << 4);
#pragma unroll
        for (int i = 0; i < TM; ++i) xa[i] = *(const bf16x8*)(pa + i * TILE_STRIDE);
#pragma unroll
        for (int j = 0; j < TN; ++j) xb[j] = *(const bf16x8*)(pb + j * TILE_STRIDE);
      };
      load(0, fa[0], fb[0]);
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        if (ks + 1 < KS) load(ks + 1, fa[(ks + 1) & 1], fb[(ks + 1) & 1]);
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
          for (int j = 0; j < TN; ++j)
            // row-run epilogues want a lane to hold consecutive n: D rows come from the A
            // operand, so the weight fragment goes there (the operand layouts are alike)
            acc[i][j] = Epi::kRowRuns
                            ? __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[ks & 1][j], fa[ks & 1][i], acc[i][j], 0, 0, 0)
                            : __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[ks & 1][i], fb[ks & 1][j], acc[i][j], 0, 0, 0);
      }
      constexpr int kDsRead = 0x100, kMfma = 0x008;
      __builtin_amdgcn_sched_group_barrier(kDsRead, TM + TN, 0);
#pragma unroll
      for (int ks = 0; ks + 1 < KS; ++ks) {
#pragma unroll
        for (int r = 0; r < TM + TN; ++r) {
          __builtin_amdgcn_sched_group_barrier(kMfma, 1, 0);
          __builtin_amdgcn_sched_group_barrier(kDsRead, 1, 0);
        }
        if (TM * TN > TM + TN) __builtin_amdgcn_sched_group_barrier(kMfma, TM * TN - (TM + TN), 0);
      }
      __builtin_amdgcn_sched_group_barrier(kMfma, TM * TN, 0);
    }

    // the next output tile's first K tile has landed (stage g & 1); every wave is done
    // reading the stage just multiplied ((g - 1) & 1), which the epilogue may now reuse
    wait_vm<0>();
    __builtin_amdgcn_s_barrier();

    if (slot < 0) {
      gemm_tile_epilogue<BM, BN, BK, WR, WC>(acc, smem + ((g - 1) & 1) * STAGE_BYTES, sbias, sgate, epi, bm0, bn0, M, N);
    } else {
      store_partial<TM, TN>(acc, partial + (size_t)slot * (BM * BN));
    }
    if (!has_next) break;
    // the staging slices are read out: the next tile's second K tile may overwrite that stage
    __builtin_amdgcn_s_barrier();
    vb = nvb; bm0 = nbm0; bn0 = nbn0; nk = nkt1 - nkt0; slot = nslot;
#pragma unroll
    for (int j = 0; j < LPW; ++j) gp[j] = gpn[j];
  }
}

// ---------------------------------------------------------------- the product kernel
// Same tiles, LDS layout, tile order and epilogue as k_gemm_dlds_any above (which stays for the
// shapes this one does not take), with two changes to the K loop.
//
// Addresses are buffer offsets.  A lane's byte offset inside a 256-row operand panel is the
// same for every tile and every K tile: the tile enters through the base of a buffer resource
// rebuilt per tile in scalar registers, the K tile through the scalar offset of the load.  The
// per-lane pointer arrays of k_gemm_dlds_any (32 registers, recomputed per tile, advanced per
// K tile with 64-bit vector adds) are gone, and so are the clamps at the ragged edges: rows
// past the end of an operand are out of the resource's range and load as zero.
//
// The barrier that publishes K tile g + 1 sits before the MFMAs of g's last k-slice, whose
// fragments are in registers by then.  After it a wave requests K tile g + 2 into the stage it
// has just stopped reading, reads the first fragments of g + 1, and only then multiplies g's
// last slice: neither the requests nor the LDS latency of the first fragments find the matrix
// pipe empty, and a DMA still has a whole K tile of matrix work to land.
//
// Measured against k_gemm_dlds_any in one process, bit-identical results: 5-11 % faster on the
// products of the two large configurations (K = 1152 .. 3072), 5 % at K = 12288, level at
// 256x192 with K = 4608, 5-10 % on the 128x128 products of a single block.
//
// Needs an even number of K tiles (the stage of a K tile is a compile-time constant: units
// start at stage 0) and operands below 4 GB (32-bit buffer ranges).
// s_waitcnt vmcnt(N) lgkmcnt(0)
template <int N> __device__ __forceinline__ void wait_vm_lgkm0() {
  __builtin_amdgcn_s_waitcnt((N & 0xF) | ((N >> 4) << 14) | (0x7 << 4));
}
template <int BM, int BN, int BK, int WR, int WC, typename Epi>
__global__ __launch_bounds__(WR * WC * 64) void k_gemm_dlds(const bf16_t* __restrict__ A, const bf16_t* __restrict__ Wt,
                                                           int M, int N, int K, int tiles_m, int tiles_n, Epi epi,
                                                           int splits, float* __restrict__ partial) {
#if defined(__HIP_DEVICE_COMPILE__)   // buffer resources are a device-side type: the host pass sees an empty body
  constexpr int NW = WR * WC;
  constexpr int WTM = BM / WR, WTN = BN / WC;
  constexpr int TM = WTM / 32, TN = WTN / 32;
  static_assert(BK == 64, "128-byte rows");
  constexpr int CPR = BK / 8, RPL = 16 / CPR, RW = 4 * RPL;
  constexpr int LA = BM / RW / NW, LB = BN / RW / NW;      // wave-loads per wave and K tile: rows of A, rows of Wt
  static_assert(BM % (RW * NW) == 0 && BN % (RW * NW) == 0, "loads must divide among waves");
  static_assert(LB <= LA, "B shares A's lane offsets");
  static_assert((NW * 4) % CPR == 0 && (BM / RW * 4) % CPR == 0, "the swizzle must not depend on the load index");
  constexpr int STAGE_BYTES = (BM + BN) * BK * 2;
  constexpr int B_REGION = BM * BK * 2;
  constexpr int KS = BK / 16;

  extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
  float* const sbias = (float*)(smem + 2 * STAGE_BYTES);
  float* const sgate = sbias + 256;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wr = wave / WC, wc = wave % WC;
  const int li = lane & 31, lh = lane >> 5;
  // an absent bias reads as zeros, an absent gate as ones (written once: no DMA touches them)
  if constexpr (Epi::kRowRuns) {
    if (tid < 256) {
      if (!epi.P.bias) sbias[tid] = 0.0f;
      if (Epi::kHasGate && !epi.P.gate) sgate[tid] = 1.0f;
    }
  }

  // ---- units of work (as in k_gemm_dlds_any; split ranges start at even K tiles)
  const int total = tiles_m * tiles_n;
  const int nkt = K / BK;
  const int full = total / 256 * 256, rem = total - full;
  // virtual ids run over the whole rounds and, behind them, the units of the last one
  const int padded = splits >= 2 ? ((full + rem * splits + 7) & ~7) : (total + 255) / 256 * 256;
  auto tile_of = [&](int vb, int& bm0, int& bn0, int& kt0, int& kt1, int& slot) {
    const int xcd = vb & 7, local = vb >> 3;
    int t = ((local >> 5) * 8 + xcd) * 32 + (local & 31);
    kt0 = 0; kt1 = nkt; slot = -1;
    if (splits >= 2 && vb >= full) {
      const int w = vb - full;
      if (w >= rem * splits) return false;
      const int r = w / rem;
      t = full + w % rem;
      kt0 = (r * nkt / splits) & ~1; kt1 = r + 1 == splits ? nkt : ((r + 1) * nkt / splits) & ~1;   // even: see the K loop
      slot = (w % rem) * splits + r;
    }
    if (t >= total) return false;
    constexpr int GM = 8;
    const int per_group = GM * tiles_n;
    const int group = t / per_group;
    const int first_m = group * GM;
    const int gsz = min(tiles_m - first_m, GM);
    bm0 = (first_m + (t % per_group) % gsz) * BM;
    bn0 = ((t % per_group) / gsz) * BN;
    return true;
  };
  auto next_tile = [&](int& vb, int& bm0, int& bn0, int& kt0, int& kt1, int& slot) {
    for (vb += gridDim.x; vb < padded; vb += gridDim.x)
      if (tile_of(vb, bm0, bn0, kt0, kt1, slot)) return true;
    return false;
  };

  // ---- this lane's byte offsets inside an operand panel, one per wave-load (the swizzled
  // 16-byte chunk of row (wave + NW j) RW + ... that lands in its LDS slot)
  unsigned voff[LA];
  {
    const int line_in = lane >> 4, sl = lane & 15;
    const int row0 = wave * RW + line_in * RPL + sl / CPR;
    const int kc = (sl % CPR) ^ ((wave * 4 + line_in) % CPR);
#pragma unroll
    for (int j = 0; j < LA; ++j) voff[j] = (unsigned)(row0 + NW * RW * j) * (unsigned)K * 2u + (unsigned)kc * 16u;
  }
  struct Panels { __amdgpu_buffer_rsrc_t a, b; int kbase; };
  auto panels = [&](int bm0, int bn0, int kt_first) {
    Panels p;
    p.a = __builtin_amdgcn_make_buffer_rsrc((void*)(A + (size_t)bm0 * K), 0, (int)((unsigned)(M - bm0) * (unsigned)K * 2u), 0x00020000);
    p.b = __builtin_amdgcn_make_buffer_rsrc((void*)(Wt + (size_t)bn0 * K), 0, (int)((unsigned)(N - bn0) * (unsigned)K * 2u), 0x00020000);
    p.kbase = kt_first * BK * 2;
    return p;
  };
  auto dma_a = [&](const Panels& p, int kt, int stage) {
#pragma unroll
    for (int j = 0; j < LA; ++j)
      __builtin_amdgcn_raw_ptr_buffer_load_lds(p.a, (lds_void*)(smem + stage * STAGE_BYTES + (wave + NW * j) * 1024), 16, (int)voff[j],
                                               p.kbase + kt * (BK * 2), 0, 0);
  };
  auto dma_b = [&](const Panels& p, int kt, int stage) {
#pragma unroll
    for (int j = 0; j < LB; ++j)
      __builtin_amdgcn_raw_ptr_buffer_load_lds(p.b, (lds_void*)(smem + stage * STAGE_BYTES + B_REGION + (wave + NW * j) * 1024), 16,
                                               (int)voff[j], p.kbase + kt * (BK * 2), 0, 0);
  };
  auto issue_vectors = [&](int bn0) {
    if constexpr (Epi::kRowRuns) {
      int n = bn0 + lane * 4;
      n = n < N ? n : 0;                           // columns past N are never stored
      if (wave == 0 && epi.P.bias)
        __builtin_amdgcn_global_load_lds((gbl_void*)(epi.P.bias + n), (lds_void*)sbias, 16, 0, 0);
      if (Epi::kHasGate && wave == 1 && epi.P.gate)
        __builtin_amdgcn_global_load_lds((gbl_void*)(epi.P.gate + n), (lds_void*)sgate, 16, 0, 0);
    }
  };

  // ---- fragment read offsets (bytes within a stage)
  const int ra = wr * WTM + li, rb = BM + wc * WTN + li;
  const int a_row = (ra / RPL) * 256 + (ra % RPL) * CPR * 16, a_x = (ra / RPL) % CPR;
  const int b_row = (rb / RPL) * 256 + (rb % RPL) * CPR * 16, b_x = (rb / RPL) % CPR;
  constexpr int TILE_STRIDE = (32 / RPL) * 256;   // 32 rows further down

  int vb = (int)blockIdx.x - (int)gridDim.x, bm0 = 0, bn0 = 0, kt0 = 0, kt1 = 0, slot = -1;
  if (!next_tile(vb, bm0, bn0, kt0, kt1, slot)) return;
  Panels cur = panels(bm0, bn0, kt0);
  int nk = kt1 - kt0;                              // K tiles of the current unit, at least 2

  // K tiles are numbered g = 0, 1, ... across this workgroup's units; K tile g is multiplied
  // out of stage g & 1.
  dma_a(cur, 0, 0);
  dma_b(cur, 0, 0);
  wait_vm<0>();
  __builtin_amdgcn_s_barrier();
  int g = 0;

  constexpr int kDsRead = 0x100, kMfma = 0x008, kVmem = 0x010;
  for (;;) {
    int nvb = vb, nbm0 = 0, nbn0 = 0, nkt0 = 0, nkt1 = 0, nslot = -1;
    const bool has_next = next_tile(nvb, nbm0, nbn0, nkt0, nkt1, nslot);
    Panels nxt = cur;
    if (has_next) nxt = panels(nbm0, nbn0, nkt0);
    issue_vectors(bn0);                            // awaited and published with the unit's first K tile

    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

    bf16x8 fa[2][TM], fb[2][TN];
    auto load = [&](int stage, int ks, bf16x8 (&xa)[TM], bf16x8 (&xb)[TN]) {
      const unsigned char* st = smem + stage * STAGE_BYTES;
      const unsigned char* pa = st + a_row + (((2 * ks + lh) ^ a_x) << 4);
      const unsigned char* pb = st + b_row + (((2 * ks + lh) ^ b_x) << 4);
#pragma unroll
      for (int i = 0; i < TM; ++i) xa[i] = *(const bf16x8*)(pa + i * TILE_STRIDE);
#pragma unroll
      for (int j = 0; j < TN; ++j) xb[j] = *(const bf16x8*)(pb + j * TILE_STRIDE);
    };
    auto multiply = [&](int set) {
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
          // row-run epilogues want a lane to hold consecutive n: D rows come from the A
          // operand, so the weight fragment goes there (the operand layouts are alike)
          acc[i][j] = Epi::kRowRuns ? __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[set][j], fa[set][i], acc[i][j], 0, 0, 0)
                                    : __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[set][i], fb[set][j], acc[i][j], 0, 0, 0);
    };
    // requests K tile ka of this unit into `stage`, continuing into the next unit past the end;
    // past the last K tile of the last unit K tile 0 of the current panels is requested again
    // (in range, never read) rather than branching around the loads
    auto request = [&](int ka, int stage) {
      const bool ina = ka < nk;
      const Panels& pa = ina ? cur : nxt;
      const int k = ina ? ka : (has_next ? ka - nk : 0);
      dma_a(pa, k, stage);
      dma_b(pa, k, stage);
    };

    // One K tile.  PAR = g & 1 selects the stage at compile time: every unit has an even number
    // of K tiles (the dispatcher sends other K to k_gemm_dlds_any), so a unit always starts at
    // PAR 0.  FIRST: the unit's first K tile (its successor not requested yet, no fragments in
    // registers: the only reads of a unit with no matrix work in front of them); LAST: its last
    // one (no requests: the stage it frees is where the epilogue stages its output rows).
    auto kstep = [&](auto par, auto first, auto last, int kt) {
      constexpr int PAR = decltype(par)::value;
      constexpr bool FIRST = decltype(first)::value, LAST = decltype(last)::value;
      if constexpr (FIRST) {
        request(kt + 1, PAR ^ 1);
        load(PAR, 0, fa[0], fb[0]);
        __builtin_amdgcn_sched_group_barrier(kVmem, LA + LB, 0);
        __builtin_amdgcn_sched_group_barrier(kDsRead, TM + TN, 0);
      }
      // k-slices 0 .. KS-2; the fragments of slice ks + 1 are read under the MFMAs of slice ks,
      // the order pinned (left alone the compiler emits read-all / wait / multiply per slice)
#pragma unroll
      for (int ks = 0; ks + 1 < KS; ++ks) {
        load(PAR, ks + 1, fa[(ks + 1) & 1], fb[(ks + 1) & 1]);
        multiply(ks & 1);
      }
#pragma unroll
      for (int ks = 0; ks + 1 < KS; ++ks) {
#pragma unroll
        for (int r = 0; r < TM + TN; ++r) {
          __builtin_amdgcn_sched_group_barrier(kMfma, 1, 0);
          __builtin_amdgcn_sched_group_barrier(kDsRead, 1, 0);
        }
        if (TM * TN > TM + TN) __builtin_amdgcn_sched_group_barrier(kMfma, TM * TN - (TM + TN), 0);
      }
      wait_vm_lgkm0<0>();                          // K tile g + 1 has landed; this wave is done reading g
      __builtin_amdgcn_s_barrier();
      __builtin_amdgcn_sched_barrier(0);
      if constexpr (!LAST) {
        request(kt + 2, PAR);
        load(PAR ^ 1, 0, fa[0], fb[0]);
      }
      multiply((KS - 1) & 1);
      if constexpr (!LAST) {
        constexpr int PER = (LA + LB + TM * TN - 1) / (TM * TN);
#pragma unroll
        for (int r = 0; r < TM * TN; ++r) {
          __builtin_amdgcn_sched_group_barrier(kMfma, 1, 0);
          if (r < TM + TN) __builtin_amdgcn_sched_group_barrier(kDsRead, 1, 0);
          if (r * PER < LA + LB) __builtin_amdgcn_sched_group_barrier(kVmem, PER, 0);
        }
      }
      __builtin_amdgcn_sched_barrier(0);
    };

    using P0 = std::integral_constant<int, 0>; using P1 = std::integral_constant<int, 1>;
    using Yes = std::true_type; using No = std::false_type;
    kstep(P0{}, Yes{}, No{}, 0);
    for (int kt = 1; kt + 1 < nk; kt += 2) {
      kstep(P1{}, No{}, No{}, kt);
      kstep(P0{}, No{}, No{}, kt + 1);
    }
    kstep(P1{}, No{}, Yes{}, nk - 1);
    g += nk;

    // every wave is done reading the stage just multiplied ((g - 1) & 1): the epilogue stages
    // its output rows there; the next unit's first K tile is complete in the other stage
    if (slot < 0) {
      gemm_tile_epilogue<BM, BN, BK, WR, WC>(acc, smem + ((g - 1) & 1) * STAGE_BYTES, sbias, sgate, epi, bm0, bn0, M, N);
    } else {
      store_partial<TM, TN>(acc, partial + (size_t)slot * (BM * BN));
    }
    if (!has_next) break;
    // the staging slices are read out: the next unit's second K tile may overwrite that stage
    __builtin_amdgcn_s_barrier();
    vb = nvb; bm0 = nbm0; bn0 = nbn0; nk = nkt1 - nkt0; slot = nslot;
    cur = nxt;
  }
#endif
}

// ---------------------------------------------------------------- split-K fix-up
// One workgroup per tile of the split round: adds the tile's `splits` partial accumulators in
// range order (bitwise repeatable) and runs the product kernel's epilogue on the sum.
template <int BM, int BN, int BK, int WR, int WC, typename Epi>
__global__ __launch_bounds__(WR * WC * 64) void k_gemm_fixup(int M, int N, int tiles_m, int tiles_n, Epi epi, int splits,
                                                             const float* __restrict__ partial) {
  constexpr int TM = BM / WR / 32, TN = BN / WC / 32;
  constexpr int STAGE_BYTES = (BM + BN) * BK * 2;
  extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
  float* const sbias = (float*)(smem + STAGE_BYTES);
  float* const sgate = sbias + 256;
  const int total = tiles_m * tiles_n;
  const int t = total / 256 * 256 + (int)blockIdx.x;
  if (t >= total) return;
  constexpr int GM = 8;                              // the product kernel's tile order
  const int per_group = GM * tiles_n;
  const int group = t / per_group;
  const int first_m = group * GM;
  const int gsz = min(tiles_m - first_m, GM);
  const int bm0 = (first_m + (t % per_group) % gsz) * BM;
  const int bn0 = ((t % per_group) / gsz) * BN;
  if (threadIdx.x < 256) {
    const int n = bn0 + (int)threadIdx.x;
    sbias[threadIdx.x] = (epi.P.bias && n < N) ? epi.P.bias[n] : 0.0f;
    if constexpr (Epi::kHasGate) sgate[threadIdx.x] = (epi.P.gate && n < N) ? epi.P.gate[n] : 1.0f;
  }
  f32x16 acc[TM][TN];
  const float* mine = partial + (size_t)blockIdx.x * splits * (BM * BN);
  for (int r = 0; r < splits; ++r) add_partial<TM, TN>(acc, mine + (size_t)r * (BM * BN), r == 0);
  __syncthreads();
  gemm_tile_epilogue<BM, BN, BK, WR, WC>(acc, smem, sbias, sgate, epi, bm0, bn0, M, N);
}

// ---------------------------------------------------------------- bf16 MFMA kernel for products with few tiles
// A 128x128 grid of C leaves most CUs idle when there are only a few tiles, and each of
// them walks the whole K alone.  Here a workgroup owns one 32x32 tile and
// its 4 waves split K; fragments come straight from global memory (each lane its own
// 16 bytes: row i of A or Wt, k = 8h .. 8h+7 of the wave's current 16-wide step), the four
// partial tiles are added through LDS in a fixed order, and wave 0 runs the column-form
// epilogue.  Needs K % 64 == 0 and 16-byte aligned rows, like the big kernel.
template <typename Epi>
__global__ __launch_bounds__(256) void k_gemm_skinny(const bf16_t* __restrict__ A, const bf16_t* __restrict__ Wt, int M,
                                                     int N, int K, Epi epi) {
  __shared__ float part[3][64][16 + 1];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int li = lane & 31, lh = lane >> 5;
  const int m0 = blockIdx.y * 32, n0 = blockIdx.x * 32;
  const int am = m0 + li < M ? m0 + li : M - 1;          // rows past the edge: computed from a valid row, never stored
  const int bn = n0 + li < N ? n0 + li : N - 1;
  const int kq = K / 4;
  const bf16_t* ap = A + (size_t)am * K + wave * kq + lh * 8;
  const bf16_t* bp = Wt + (size_t)bn * K + wave * kq + lh * 8;
  f32x16 acc;
#pragma unroll
  for (int r = 0; r < 16; ++r) acc[r] = 0.0f;
  for (int k = 0; k < kq; k += 64) {                     // kq % 16 == 0; 4 steps per trip, loads first
    bf16x8 fa[4], fb[4];
#pragma unroll
    for (int u = 0; u < 4; ++u)
      if (k + 16 * u < kq) { fa[u] = *(const bf16x8*)(ap + k + 16 * u); fb[u] = *(const bf16x8*)(bp + k + 16 * u); }
#pragma unroll
    for (int u = 0; u < 4; ++u)
      if (k + 16 * u < kq) acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[u], fb[u], acc, 0, 0, 0);
  }
  if (wave > 0) {
#pragma unroll
    for (int r = 0; r < 16; ++r) part[wave - 1][lane][r] = acc[r];
  }
  __syncthreads();
  if (wave > 0) return;
#pragma unroll
  for (int w = 0; w < 3; ++w)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[r] += part[w][lane][r];
  // D: lane (li, lh) holds column li, rows 8 g + 4 lh + e in register 4 g + e
  const auto col = epi.col(n0 + li);
#pragma unroll
  for (int g = 0; g < 4; ++g) {
    float v[4] = {acc[4 * g], acc[4 * g + 1], acc[4 * g + 2], acc[4 * g + 3]};
    epi.store4(col, m0 + g * 8 + lh * 4, v);
  }
}

template <int MODE>
static hipError_t run_skinny(const void* A, const void* Wt, int M, int N, int K, const EpiParams& ep, hipStream_t s) {
  using Epi = Epilogue<bf16_t, MODE>;
  Epi epi = Epi::make(ep, M, N);
  dim3 grid(ceil_div(N, 32), ceil_div(M, 32));
  k_gemm_skinny<Epi><<<grid, 256, 0, s>>>((const bf16_t*)A, (const bf16_t*)Wt, M, N, K, epi);
  return hipGetLastError();
}

// ---------------------------------------------------------------- plain kernel (any T, any shape)
// 64x64 block tile, BK = 16, 256 threads each owning a 4(row) x 4(col) micro-tile.
template <typename T, typename Epi>
__global__ __launch_bounds__(256) void k_gemm_plain(const T* __restrict__ A, const T* __restrict__ Wt, int M, int N,
                                                    int K, Epi epi) {
  __shared__ float As[16][64 + 4];
  __shared__ float Bs[16][64 + 4];
  const int tid = threadIdx.x;
  const int tr = tid / 16, tc = tid % 16;
  const int bm0 = blockIdx.y * 64, bn0 = blockIdx.x * 64;
  float acc[4][4] = {};
  for (int k0 = 0; k0 < K; k0 += 16) {
    for (int i = tid; i < 64 * 16; i += 256) {
      int row = i / 16, kk = i % 16;
      int gm = bm0 + row, gn = bn0 + row, gk = k0 + kk;
      As[kk][row] = (gm < M && gk < K) ? to_f32(A[(size_t)gm * K + gk]) : 0.0f;
      Bs[kk][row] = (gn < N && gk < K) ? to_f32(Wt[(size_t)gn * K + gk]) : 0.0f;
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < 16; ++kk) {
      float a[4], b[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) a[i] = As[kk][tr * 4 + i];
#pragma unroll
      for (int j = 0; j < 4; ++j) b[j] = Bs[kk][tc * 4 + j];
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] += a[i] * b[j];
    }
    __syncthreads();
  }
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    float v[4] = {acc[0][j], acc[1][j], acc[2][j], acc[3][j]};
    epi.store4(epi.col(bn0 + tc * 4 + j), bm0 + tr * 4, v);
  }
}

// ---------------------------------------------------------------- dispatch
template <int BM, int BN, int BK, int WR, int WC, int S, int MODE>
static hipError_t run_dlds(const void* A, const void* Wt, int M, int N, int K, const EpiParams& ep, void* scratch,
                           size_t scratch_bytes, hipStream_t s) {
  using Epi = Epilogue<bf16_t, MODE>;
  Epi epi = Epi::make(ep, M, N);
  constexpr size_t smem = (size_t)S * (BM + BN) * BK * sizeof(bf16_t) + 2048;   // + bias and gate of a tile
  // k_gemm_dlds needs an even number of K tiles and addresses its operands as 32-bit buffer
  // ranges; anything else goes to k_gemm_dlds_any
  const bool even = K % (2 * BK) == 0 && (unsigned long long)M * K * 2 < (1ull << 32) && (unsigned long long)N * K * 2 < (1ull << 32);
  auto kern = k_gemm_dlds<BM, BN, BK, WR, WC, Epi>;
  auto kern_any = k_gemm_dlds_any<BM, BN, BK, WR, WC, S, Epi>;
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    if (e == hipSuccess) e = hipFuncSetAttribute((const void*)kern_any, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  const int tiles_m = ceil_div(M, BM), tiles_n = ceil_div(N, BN);
  const long long total = (long long)tiles_m * tiles_n;
  // persistent: as many workgroups as the chip holds at once (by LDS: one of the large
  // configurations per CU, two of the 128x128 one), each walking its share of the tiles
  const long long padded = (total + 255) / 256 * 256;
  const long long slots = 256LL * (smem > 80 * 1024 ? 1 : 2);
  const unsigned grid = (unsigned)(padded < slots ? padded : slots);
  // Split-K for a last round that would leave most of the chip idle: at most half the slots
  // taken, few enough rounds that one of them matters (measured: 3.3 rounds become 11 %
  // faster, 13.1 rounds not at all), a K long enough that the saved part of a tile outweighs
  // the fix-up launch, and a caller that lends scratch memory for the partial tiles.
  int splits = 1;
  unsigned launch = grid;
  const long long rem = total % 256, full = total - rem;
  // (A product of fewer tiles than half the slots is all remainder: its tiles are split the
  // same way; with two workgroups per CU there are 512 slots for the units.)
  // (With two workgroups per CU every product of up to 512 tiles runs in one round anyway: only
  // the all-remainder case is split there.)
  if (total / 256 <= 8 && rem > 0 && rem <= slots / 2 && (slots == 256 || full == 0) && scratch &&
      ((uintptr_t)scratch & 15) == 0) {
    long long sp = slots / rem;
    sp = sp > 4 ? 4 : sp;
    sp = sp > K / BK / 2 ? K / BK / 2 : sp;
    if (sp >= 2 && (long long)K * (sp - 1) / sp >= 1536 &&
        (size_t)(rem * sp) * BM * BN * sizeof(float) <= scratch_bytes) {
      splits = (int)sp;
      const long long units = (full + rem * sp + 7) / 8 * 8;
      launch = (unsigned)(units < slots ? units : slots);
      if (launch < grid) launch = grid;
    }
  }
  if (even)
    kern<<<launch, WR * WC * 64, smem, s>>>((const bf16_t*)A, (const bf16_t*)Wt, M, N, K, tiles_m, tiles_n, epi, splits, (float*)scratch);
  else
    kern_any<<<launch, WR * WC * 64, smem, s>>>((const bf16_t*)A, (const bf16_t*)Wt, M, N, K, tiles_m, tiles_n, epi, splits,
                                              (float*)scratch);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess || splits < 2) return e;
  auto fix = k_gemm_fixup<BM, BN, BK, WR, WC, Epi>;
  constexpr size_t fsmem = (size_t)(BM + BN) * BK * sizeof(bf16_t) + 2048;
  static bool fattr_set = false;
  if (!fattr_set) {
    e = hipFuncSetAttribute((const void*)fix, hipFuncAttributeMaxDynamicSharedMemorySize, (int)fsmem);
    if (e != hipSuccess) return e;
    fattr_set = true;
  }
  fix<<<(unsigned)rem, WR * WC * 64, fsmem, s>>>(M, N, tiles_m, tiles_n, epi, splits, (const float*)scratch);
  return hipGetLastError();
}

template <typename T, int MODE>
static hipError_t run_plain(const void* A, const void* Wt, int M, int N, int K, const EpiParams& ep, hipStream_t s) {
  using Epi = Epilogue<T, MODE>;
  Epi epi = Epi::make(ep, M, N);
  dim3 grid(ceil_div(N, 64), ceil_div(M, 64));
  k_gemm_plain<T, Epi><<<grid, 256, 0, s>>>((const T*)A, (const T*)Wt, M, N, K, epi);
  return hipGetLastError();
}

template <int MODE>
static hipError_t dispatch_mode(int bf16, const void* A, const void* Wt, int M, int N, int K, const EpiParams& ep,
                                void* scratch, size_t scratch_bytes, hipStream_t s) {
  if (!bf16) return run_plain<float, MODE>(A, Wt, M, N, K, ep, s);
  bool aligned = (((uintptr_t)A | (uintptr_t)Wt) & 15) == 0;
  // very few tiles (a request's text rows), or an N too narrow for the tile kernel (a 16-wide
  // output head): split K inside a workgroup instead.  Measured against the 128x128
  // configuration it wins below about 32 of its tiles and loses above (its fragment loads
  // are 32-byte pieces of rows).
  if (aligned && K % 64 == 0 && ((long long)ceil_div(M, 128) * ceil_div(N, 128) < 32 || N < 32) &&
      ceil_div(M, 32) <= 65535)
    return run_skinny<MODE>(A, Wt, M, N, K, ep, s);
  if (MODE != EPI_UNPATCH) {
    // the MFMA kernel writes 16-byte runs of a row and reads bias / gate four at a time
    aligned = aligned && N % 8 == 0 && (((uintptr_t)ep.bias | (uintptr_t)ep.gate) & 15) == 0;
    if (MODE == EPI_HEADS)
      aligned = aligned && ep.hd % 8 == 0 && ep.D % 8 == 0 &&
                (((uintptr_t)ep.q | (uintptr_t)ep.k | (uintptr_t)ep.v) & 15) == 0;
    else
      aligned = aligned && ep.ldo % 8 == 0 && ((uintptr_t)ep.out & 15) == 0;
  }
  if (K % 64 != 0 || !aligned || N < 32) return run_plain<bf16_t, MODE>(A, Wt, M, N, K, ep, s);
  // Tile choice.  256x256 (8 waves, one workgroup per CU) has the best operand reuse but
  // needs several rounds of tiles per CU and wastes the ragged part of N; 256x192 takes
  // over where N is a multiple of 192 that 256 would pad by more than 5 % (N = 1152:
  // 11 % padding and 2.5 rounds of tiles become none and 3); 128x128 (4 waves, two
  // workgroups per CU, so one's epilogue overlaps the other's main loop) wins for
  // narrow or short-K products.  Thresholds from timings of the workload shapes.
  const long long tiles256 = (long long)ceil_div(M, 256) * ceil_div(N, 256);
  const double waste = (double)ceil_div(N, 256) * 256.0 / N - 1.0;
  if (N % 192 == 0 && waste > 0.05 && (long long)ceil_div(M, 256) * (N / 192) >= 192)
    return run_dlds<256, 192, 64, 4, 2, 2, MODE>(A, Wt, M, N, K, ep, scratch, scratch_bytes, s);
  // 384x192 (96x96 per wave) is no faster per tile than 256x256, but where its tile count fills
  // whole rounds of 256 and that of 256x256 does not, it saves most of a round (the full-3D
  // out-projection and fc2: 752 tiles = 2.94 rounds against 840 = 3.28; 2-5 % over the split
  // last round)
  if constexpr (MODE != EPI_UNPATCH) if (N % 192 == 0 && K >= 2048 && tiles256 >= 600) {
    const long long t384 = (long long)ceil_div(M, 384) * (N / 192);
    const double fill384 = (double)t384 / (double)((t384 + 255) / 256 * 256);
    const double fill256 = (double)tiles256 / (double)((tiles256 + 255) / 256 * 256);
    if (fill384 >= 0.95 && fill256 < 0.85 && waste <= 0.05)
      return run_dlds<384, 192, 64, 4, 2, 2, MODE>(A, Wt, M, N, K, ep, scratch, scratch_bytes, s);
  }
  if (tiles256 >= 600 && (waste <= 0.05 || K >= 2048)) return run_dlds<256, 256, 64, 4, 2, 2, MODE>(A, Wt, M, N, K, ep, scratch, scratch_bytes, s);
  // Mid-size products (a few thousand rows) that the thresholds above leave to 128x128: the large
  // tiles still win where their tile count fills its rounds of 256 workgroups (measured at
  // M = 4096 and 8192: QKV of the 1152-wide model 8-14 % faster with 256x256, its fc1 at
  // M = 8192 7 % faster with 256x192; where the last round would be mostly empty, 128x128 stays)
  {
    auto fill = [](long long t) { return (double)t / (double)((t + 255) / 256 * 256); };
    if (tiles256 >= 200 && waste <= 0.05 && fill(tiles256) >= 0.85)
      return run_dlds<256, 256, 64, 4, 2, 2, MODE>(A, Wt, M, N, K, ep, scratch, scratch_bytes, s);
    if (N % 192 == 0) {
      const long long t192 = (long long)ceil_div(M, 256) * (N / 192);
      if (t192 >= 200 && fill(t192) >= 0.95) return run_dlds<256, 192, 64, 4, 2, 2, MODE>(A, Wt, M, N, K, ep, scratch, scratch_bytes, s);
    }
  }
  return run_dlds<128, 128, 64, 2, 2, 2, MODE>(A, Wt, M, N, K, ep, scratch, scratch_bytes, s);
}

hipError_t launch_gemm(int bf16, int mode, const void* A, const void* Wt, int M, int N, int K, const EpiParams& ep,
                       hipStream_t s, void* scratch, size_t scratch_bytes) {
  if (M <= 0 || N <= 0 || K <= 0) return hipSuccess;
  switch (mode) {
    case EPI_STORE: return dispatch_mode<EPI_STORE>(bf16, A, Wt, M, N, K, ep, scratch, scratch_bytes, s);
    case EPI_GELU: return dispatch_mode<EPI_GELU>(bf16, A, Wt, M, N, K, ep, scratch, scratch_bytes, s);
    case EPI_GATE: return dispatch_mode<EPI_GATE>(bf16, A, Wt, M, N, K, ep, scratch, scratch_bytes, s);
    case EPI_HEADS: return dispatch_mode<EPI_HEADS>(bf16, A, Wt, M, N, K, ep, scratch, scratch_bytes, s);
    case EPI_UNPATCH: return dispatch_mode<EPI_UNPATCH>(bf16, A, Wt, M, N, K, ep, scratch, scratch_bytes, s);
  }
  return hipErrorInvalidValue;
}

}  // namespace fc
