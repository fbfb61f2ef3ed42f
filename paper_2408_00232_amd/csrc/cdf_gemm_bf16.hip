// Dense transform for bf16-stored activations on the bf16 matrix cores (Sec. 3.1, Z = M W):
// M [n x f] is bf16 and enters the MFMA unchanged; W [f x g] is fp32 and is split, while it is
// staged into LDS, into a bf16 high part and a bf16 low part (w = hi + lo up to 2^-17 |w|), so
// Z = M hi + M lo with fp32 accumulation inside v_mfma_f32_32x32x16_bf16 - two bf16 products at
// sixteen times the fp32 matrix rate in place of one fp32 product.
//
// Tile: 128 x BN outputs (BN = 128 or 64) per block of four wavefronts (2 x 2), reduction in steps of 32. LDS holds the operands k-contiguous per row (As[m][k], Bh[n][k], Bl[n][k]) so
// that a lane reads its eight consecutive k values of a 32x32x16 operand with one 16-byte access. The next
// k-tile is fetched into registers while the current one is multiplied. The column blocks of a row tile
// run on one XCD at the same time (1-D grid, see xcd_tile), so the row tile's operand comes from memory once.
#include <type_traits>

#include "cdf_common.h"

namespace cdf {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kHK = 32;       // reduction elements per LDS tile
constexpr int kHS = kHK + 8;  // LDS row stride in bf16 elements (80 bytes: 16-byte aligned rows)
constexpr int kHThreads = 256;

// fp32 -> (hi, lo) bf16 bit patterns, both rounded to nearest even.
__device__ __forceinline__ void split_bf16(float w, uint16_t& hi, uint16_t& lo) {
  const __bf16 h = static_cast<__bf16>(w);
  const __bf16 l = static_cast<__bf16>(w - static_cast<float>(h));
  hi = __builtin_bit_cast(uint16_t, h);
  lo = __builtin_bit_cast(uint16_t, l);
}

// W [f x g] fp32 -> Wh, Wl [g x f] bf16 (transposed: the reduction index becomes contiguous), done once
// per product when the caller has workspace, so that the blocks of the product only copy.
__global__ __launch_bounds__(256) void split_transpose_kernel(const float* __restrict__ W, int f, int g,
                                                              uint16_t* __restrict__ Wh, uint16_t* __restrict__ Wl) {
  __shared__ float tile[32][33];
  const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;   // 32 x 8
  const int k0 = blockIdx.x * 32, c0 = blockIdx.y * 32;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int k = k0 + ty + 8 * i, c = c0 + tx;
    tile[ty + 8 * i][tx] = (k < f && c < g) ? W[static_cast<int64_t>(k) * g + c] : 0.0f;
  }
  __syncthreads();
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int c = c0 + ty + 8 * i, k = k0 + tx;
    if (c < g && k < f) {
      uint16_t hi, lo;
      split_bf16(tile[tx][ty + 8 * i], hi, lo);
      Wh[static_cast<int64_t>(c) * f + k] = hi;
      Wl[static_cast<int64_t>(c) * f + k] = lo;
    }
  }
}

// PRE: Wh / Wl hold the split, transposed weight (see above) and W is unused; otherwise every block
// splits its own part of W while staging it.
// W [count] fp32 -> Wh, Wl [count] bf16 in the same order (count a multiple of 8): the weight operand of
// dM = dZ W^T, whose reduction index is already contiguous in W.
__global__ __launch_bounds__(256) void split_kernel(const float* __restrict__ W, int64_t count,
                                                    uint16_t* __restrict__ Wh, uint16_t* __restrict__ Wl) {
  const int64_t i = (static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x) * 8;
  if (i >= count) return;
  const float4 a = *reinterpret_cast<const float4*>(W + i), b = *reinterpret_cast<const float4*>(W + i + 4);
  const float v[8] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
  uint16_t hi[8], lo[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) split_bf16(v[j], hi[j], lo[j]);
  u32x4 ph, pl;
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    ph[q] = static_cast<uint32_t>(hi[2 * q]) | (static_cast<uint32_t>(hi[2 * q + 1]) << 16);
    pl[q] = static_cast<uint32_t>(lo[2 * q]) | (static_cast<uint32_t>(lo[2 * q + 1]) << 16);
  }
  *reinterpret_cast<u32x4*>(Wh + i) = ph;
  *reinterpret_cast<u32x4*>(Wl + i) = pl;
}

// Output tile of a workgroup in a 1-D grid of 8 * ceil(row_tiles / 8) * col_blocks workgroups. Workgroups are
// handed to the 8 XCDs in turn, so workgroup b runs on XCD b mod 8; the column blocks of one row tile get
// consecutive slots of ONE XCD, run there at the same time and read the row tile's operand once into that
// XCD's L2 instead of once per column block from memory. False for the padding of the last group of 8.
__device__ __forceinline__ bool xcd_tile(int row_tiles, int col_blocks, int& row_tile, int& col_block) {
  const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
  col_block = slot % col_blocks;
  row_tile = (slot / col_blocks) * 8 + xcd;
  return row_tile < row_tiles;
}
static unsigned xcd_grid(int64_t row_tiles, int64_t col_blocks) {
  return static_cast<unsigned>(ceil_div(row_tiles, 8) * 8 * col_blocks);
}

template <int BN, bool PRE>
__global__ __launch_bounds__(kHThreads, 2) void gemm_bf16_fwd_kernel(const bf16_t* __restrict__ M, int64_t ldm,
                                                                     const float* __restrict__ W,
                                                                     const uint16_t* __restrict__ Wh,
                                                                     const uint16_t* __restrict__ Wl, int n, int f, int g,
                                                                     int relu, float* __restrict__ Z,
                                                                     float* __restrict__ H) {
  constexpr int TM = 2, TN = BN / 64;
  constexpr int HM = 64 * TM;                     // output rows per block (two wavefronts of TM tiles of 32)
  constexpr int BI = BN * (kHK / 8) / kHThreads;  // (column, k-block) items of the W tile per thread
  __shared__ __attribute__((aligned(16))) uint16_t As[HM][kHS];
  __shared__ __attribute__((aligned(16))) uint16_t Bh[BN][kHS];
  __shared__ __attribute__((aligned(16))) uint16_t Bl[BN][kHS];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int l32 = lane & 31, lh = lane >> 5;
  int row_tile, col_block;
  if (!xcd_tile((n + HM - 1) / HM, (g + BN - 1) / BN, row_tile, col_block)) return;
  const int m0 = row_tile * HM, n0 = col_block * BN;

  constexpr int AI = HM * (kHK / 8) / kHThreads;   // 8-element chunks of the M tile per thread
  u32x4 ra[AI];
  float rb[PRE ? 1 : BI][8];    // BI items of 8 consecutive k for one output column (fp32, to be split)
  u32x4 rh[PRE ? BI : 1], rl[PRE ? BI : 1];   // the same items, already split

  // item -> (column, block of 8 k) of the W tile. Split W is stored transposed, a column's k run is contiguous:
  // neighbouring lanes take neighbouring k blocks of one column (whole 64-byte runs). Unsplit W is row-major
  // [k][column]: neighbouring lanes take neighbouring columns.
  auto b_col = [](int item) { return PRE ? item / (kHK / 8) : item % BN; };
  auto b_kb = [](int item) { return PRE ? item % (kHK / 8) : item / BN; };
  // Loads carry no branches and nothing waits for them before the products of the current tile have been
  // issued: addresses are clamped into the operand (rows past n and columns past g feed outputs that are never
  // stored; k blocks past f are zeroed when they are staged, on both operands).
  auto fetch = [&](int k0) {
#pragma unroll
    for (int i = 0; i < AI; ++i) {
      const int c = tid + kHThreads * i;
      const int row = min(m0 + c / (kHK / 8), n - 1), k = min(k0 + (c % (kHK / 8)) * 8, f - 8);
      ra[i] = *reinterpret_cast<const u32x4*>(M + static_cast<int64_t>(row) * ldm + k);
    }
#pragma unroll
    for (int i = 0; i < BI; ++i) {
      const int item = tid + kHThreads * i;
      const int col = min(n0 + b_col(item), g - 1), kb = min(k0 + b_kb(item) * 8, f - 8);
      if (PRE) {
        rh[i] = *reinterpret_cast<const u32x4*>(Wh + static_cast<int64_t>(col) * f + kb);
        rl[i] = *reinterpret_cast<const u32x4*>(Wl + static_cast<int64_t>(col) * f + kb);
      } else {
#pragma unroll
        for (int j = 0; j < 8; ++j) rb[i][j] = W[static_cast<int64_t>(kb + j) * g + col];
      }
    }
  };
  const u32x4 zero4 = {0u, 0u, 0u, 0u};
  auto stage = [&](int k0) {
#pragma unroll
    for (int i = 0; i < AI; ++i) {
      const int c = tid + kHThreads * i;
      const bool kin = k0 + (c % (kHK / 8)) * 8 < f;
      *reinterpret_cast<u32x4*>(&As[c / (kHK / 8)][(c % (kHK / 8)) * 8]) = kin ? ra[i] : zero4;
    }
#pragma unroll
    for (int i = 0; i < BI; ++i) {
      const int item = tid + kHThreads * i;
      const bool kin = k0 + b_kb(item) * 8 < f;
      if (PRE) {
        *reinterpret_cast<u32x4*>(&Bh[b_col(item)][b_kb(item) * 8]) = kin ? rh[i] : zero4;
        *reinterpret_cast<u32x4*>(&Bl[b_col(item)][b_kb(item) * 8]) = kin ? rl[i] : zero4;
        continue;
      }
      uint16_t hi[8], lo[8];
#pragma unroll
      for (int j = 0; j < 8; ++j) split_bf16(kin ? rb[i][j] : 0.0f, hi[j], lo[j]);
      u32x4 ph, pl;
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        ph[q] = static_cast<uint32_t>(hi[2 * q]) | (static_cast<uint32_t>(hi[2 * q + 1]) << 16);
        pl[q] = static_cast<uint32_t>(lo[2 * q]) | (static_cast<uint32_t>(lo[2 * q + 1]) << 16);
      }
      *reinterpret_cast<u32x4*>(&Bh[b_col(item)][b_kb(item) * 8]) = ph;
      *reinterpret_cast<u32x4*>(&Bl[b_col(item)][b_kb(item) * 8]) = pl;
    }
  };

  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.0f;

  fetch(0);
  for (int k0 = 0; k0 < f; k0 += kHK) {
    stage(k0);
    __syncthreads();
    if (k0 + kHK < f) fetch(k0 + kHK);
#pragma unroll
    for (int ks = 0; ks < kHK; ks += 16) {
      // operand of a 32x32x16 product: lane (l32, lh) supplies row / column l32, k = lh*8 .. lh*8+7
      bf16x8 a[TM], bh[TN], bl[TN];
#pragma unroll
      for (int i = 0; i < TM; ++i)
        a[i] = *reinterpret_cast<const bf16x8*>(&As[wm * (HM / 2) + i * 32 + l32][ks + lh * 8]);
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        bh[j] = *reinterpret_cast<const bf16x8*>(&Bh[wn * (BN / 2) + j * 32 + l32][ks + lh * 8]);
        bl[j] = *reinterpret_cast<const bf16x8*>(&Bl[wn * (BN / 2) + j * 32 + l32][ks + lh * 8]);
      }
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) {
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], bl[j], acc[i][j], 0, 0, 0);
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], bh[j], acc[i][j], 0, 0, 0);
        }
    }
    __syncthreads();
  }

  // lane holds column l32 and rows (e/4)*8 + lh*4 + e%4 of each 32x32 tile; a tile that lies inside the
  // output is stored without per-element checks
  auto store_tile = [&](auto checked) {
    constexpr bool CHECK = decltype(checked)::value;
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        const int col = n0 + wn * (BN / 2) + j * 32 + l32;
        if (CHECK && col >= g) continue;
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          const int row = m0 + wm * (HM / 2) + i * 32 + (e >> 2) * 8 + lh * 4 + (e & 3);
          if (CHECK && row >= n) continue;
          const float v = acc[i][j][e];
          const int64_t off = static_cast<int64_t>(row) * g + col;
          if (Z) Z[off] = v;
          if (H) H[off] = relu ? (v > 0.0f ? v : 0.0f) : v;
        }
      }
  };
  if (m0 + HM <= n && n0 + BN <= g) store_tile(std::false_type{});
  else store_tile(std::true_type{});
}

// ---- dM = dZ W^T for bf16-stored activations (Sec. 3.1, gradient w.r.t. the layer input) --------
// dZ = dH * [Zs > 0] and W are both fp32 and both contiguous along the reduction index (the output
// features), so each is split into bf16 high / low parts while it is staged:
//   dM = dZh Wh^T + dZh Wl^T + dZl Wh^T          (the low x low term is below 2^-16 of the result)
// The result is stored as bf16, which is the type the aggregation that follows reads.
template <int BN, bool RELU, bool PRE>
__global__ __launch_bounds__(kHThreads, 2) void gemm_bf16_dm_kernel(const float* __restrict__ dH,
                                                                    const float* __restrict__ Zs,
                                                                    const float* __restrict__ W,
                                                                    const uint16_t* __restrict__ Wh,
                                                                    const uint16_t* __restrict__ Wl, int n, int f, int g,
                                                                    bf16_t* __restrict__ dM, int64_t ldo) {
  constexpr int TM = 2, TN = BN / 64;
  constexpr int HM = 64 * TM;
  constexpr int AI = HM * (kHK / 8) / kHThreads;
  constexpr int BI = BN * (kHK / 8) / kHThreads;
  __shared__ __attribute__((aligned(16))) uint16_t Ah[HM][kHS];
  __shared__ __attribute__((aligned(16))) uint16_t Al[HM][kHS];
  __shared__ __attribute__((aligned(16))) uint16_t Bh[BN][kHS];
  __shared__ __attribute__((aligned(16))) uint16_t Bl[BN][kHS];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int l32 = lane & 31, lh = lane >> 5;
  int row_tile, col_block;
  if (!xcd_tile((n + HM - 1) / HM, (f + BN - 1) / BN, row_tile, col_block)) return;
  const int m0 = row_tile * HM, n0 = col_block * BN;

  float ra[AI][8], rz[RELU ? AI : 1][8], rb[PRE ? 1 : BI][8];
  u32x4 rh[PRE ? BI : 1], rl[PRE ? BI : 1];   // W already split (by split_kernel) when the caller has workspace
  auto load8 = [](const float* p, float (&v)[8]) {
    const float4 a = *reinterpret_cast<const float4*>(p), b = *reinterpret_cast<const float4*>(p + 4);
    v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w; v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
  };
  // Branch-free loads with clamped addresses; the ReLU mask, the zeroing of k blocks past g and the split are
  // applied when the tile is staged, so that nothing waits for a load before the current tile's products.
  // addresses: a tile base that is the same for the whole block plus 32-bit element offsets
  const float* dHt = dH + static_cast<int64_t>(m0) * g;
  const float* Zt = RELU ? Zs + static_cast<int64_t>(m0) * g : nullptr;
  const float* Wt = W + static_cast<int64_t>(n0) * g;
  const uint16_t* Wht = PRE ? Wh + static_cast<int64_t>(n0) * g : nullptr;
  const uint16_t* Wlt = PRE ? Wl + static_cast<int64_t>(n0) * g : nullptr;
  const int kk = (tid % (kHK / 8)) * 8;   // the thread's k block inside a tile, the same for all its items
  uint32_t arow[AI], brow[BI];
#pragma unroll
  for (int i = 0; i < AI; ++i) arow[i] = static_cast<uint32_t>(min((tid + kHThreads * i) / (kHK / 8), n - 1 - m0)) * g;
#pragma unroll
  for (int i = 0; i < BI; ++i) brow[i] = static_cast<uint32_t>(min((tid + kHThreads * i) / (kHK / 8), f - 1 - n0)) * g;
  auto fetch = [&](int k0) {
    const uint32_t k = min(k0 + kk, g - 8);
#pragma unroll
    for (int i = 0; i < AI; ++i) {
      load8(dHt + (arow[i] + k), ra[i]);
      if (RELU) load8(Zt + (arow[i] + k), rz[i]);
    }
#pragma unroll
    for (int i = 0; i < BI; ++i) {
      if (PRE) {
        rh[i] = *reinterpret_cast<const u32x4*>(Wht + (brow[i] + k));
        rl[i] = *reinterpret_cast<const u32x4*>(Wlt + (brow[i] + k));
      } else {
        load8(Wt + (brow[i] + k), rb[i]);
      }
    }
  };
  auto put = [](const float (&v)[8], uint16_t* hi_dst, uint16_t* lo_dst) {
    uint16_t hi[8], lo[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) split_bf16(v[j], hi[j], lo[j]);
    u32x4 ph, pl;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      ph[q] = static_cast<uint32_t>(hi[2 * q]) | (static_cast<uint32_t>(hi[2 * q + 1]) << 16);
      pl[q] = static_cast<uint32_t>(lo[2 * q]) | (static_cast<uint32_t>(lo[2 * q + 1]) << 16);
    }
    *reinterpret_cast<u32x4*>(hi_dst) = ph;
    *reinterpret_cast<u32x4*>(lo_dst) = pl;
  };
  auto stage = [&](int k0) {
#pragma unroll
    for (int i = 0; i < AI; ++i) {
      const int c = tid + kHThreads * i;
      const bool kin = k0 + (c % (kHK / 8)) * 8 < g;
      float v[8];
#pragma unroll
      for (int j = 0; j < 8; ++j) v[j] = (kin && (!RELU || rz[RELU ? i : 0][j] > 0.0f)) ? ra[i][j] : 0.0f;
      put(v, &Ah[c / (kHK / 8)][(c % (kHK / 8)) * 8], &Al[c / (kHK / 8)][(c % (kHK / 8)) * 8]);
    }
#pragma unroll
    for (int i = 0; i < BI; ++i) {
      const int item = tid + kHThreads * i;
      const bool kin = k0 + (item % (kHK / 8)) * 8 < g;
      if (PRE) {
        *reinterpret_cast<u32x4*>(&Bh[item / (kHK / 8)][(item % (kHK / 8)) * 8]) = kin ? rh[i] : u32x4{0u, 0u, 0u, 0u};
        *reinterpret_cast<u32x4*>(&Bl[item / (kHK / 8)][(item % (kHK / 8)) * 8]) = kin ? rl[i] : u32x4{0u, 0u, 0u, 0u};
        continue;
      }
      float v[8];
#pragma unroll
      for (int j = 0; j < 8; ++j) v[j] = kin ? rb[PRE ? 0 : i][j] : 0.0f;
      put(v, &Bh[item / (kHK / 8)][(item % (kHK / 8)) * 8], &Bl[item / (kHK / 8)][(item % (kHK / 8)) * 8]);
    }
  };

  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.0f;

  fetch(0);
  for (int k0 = 0; k0 < g; k0 += kHK) {
    stage(k0);
    __syncthreads();
    if (k0 + kHK < g) fetch(k0 + kHK);
#pragma unroll
    for (int ks = 0; ks < kHK; ks += 16) {
      bf16x8 ah[TM], al[TM], bh[TN], bl[TN];
#pragma unroll
      for (int i = 0; i < TM; ++i) {
        ah[i] = *reinterpret_cast<const bf16x8*>(&Ah[wm * (HM / 2) + i * 32 + l32][ks + lh * 8]);
        al[i] = *reinterpret_cast<const bf16x8*>(&Al[wm * (HM / 2) + i * 32 + l32][ks + lh * 8]);
      }
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        bh[j] = *reinterpret_cast<const bf16x8*>(&Bh[wn * (BN / 2) + j * 32 + l32][ks + lh * 8]);
        bl[j] = *reinterpret_cast<const bf16x8*>(&Bl[wn * (BN / 2) + j * 32 + l32][ks + lh * 8]);
      }
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) {
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(al[i], bh[j], acc[i][j], 0, 0, 0);
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah[i], bl[j], acc[i][j], 0, 0, 0);
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah[i], bh[j], acc[i][j], 0, 0, 0);
        }
    }
    __syncthreads();
  }
  auto store_tile = [&](auto checked) {
    constexpr bool CHECK = decltype(checked)::value;
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        const int col = n0 + wn * (BN / 2) + j * 32 + l32;
        if (CHECK && col >= f) continue;
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          const int row = m0 + wm * (HM / 2) + i * 32 + (e >> 2) * 8 + lh * 4 + (e & 3);
          if (CHECK && row >= n) continue;
          float one[1] = {acc[i][j][e]};
          VecIO<bf16_t, 1>::store(dM + static_cast<int64_t>(row) * ldo + col, one);
        }
      }
  };
  if (m0 + HM <= n && n0 + BN <= f) store_tile(std::false_type{});
  else store_tile(std::true_type{});
}

// ---- dW = M^T dZ for bf16-stored activations (Sec. 3.1, gradient w.r.t. the weights) ----------------
// The reduction runs over the rows, along which neither operand is contiguous in memory, while a lane of
// a 32x32x16 product supplies eight CONSECUTIVE reduction elements of one output row / column. The
// tiles are kept in LDS in the order they have in memory (As[row][feature], Bh / Bl [row][column], a
// tile of 32 rows) and the operands are read with the transposing LDS load of gfx950
// (ds_read_b64_tr_b16): the 16 lanes of a group each name 8 bytes - lane p the four features
// 4 (p % 4) .. + 3 of row p / 4 - and lane j gets back element j % 4 of the blocks of lanes j / 4,
// 4 + j / 4, 8 + j / 4, 12 + j / 4: feature j of four consecutive rows. Two such loads make the eight
// reduction elements of a lane. The row stride (80 words) puts the four rows a load touches on
// disjoint banks. M is bf16 and enters unchanged; dZ = dH * [Zs > 0] is fp32 and is split into a bf16
// high and low part while it is staged: dW = M^T dZh + M^T dZl, fp32 accumulation. Slabs of rows,
// partial tiles and their ordered reduction are those of the fp32 kernel.
constexpr int kWK = 32;            // rows (reduction elements) per LDS tile
constexpr int kWM = 128;           // features (output rows) per block
constexpr int kWS = 128 + 32;      // LDS row stride in bf16 elements: 80 words, so the next row is 16 banks further

typedef short short4v __attribute__((ext_vector_type(4)));

// Eight reduction elements (rows k .. k + 7 of the tile) of column col0 + (lane % 32) for lane (l32, lh):
// `tile` points at row ks of the LDS tile; see the layout of the transposing load above.
__device__ __forceinline__ bf16x8 read_tr8(const uint16_t* tile, int col0, int lane) {
  const int grp = lane >> 4, p = lane & 15;
  const uint16_t* at = tile + ((grp >> 1) * 8 + (p >> 2)) * kWS + col0 + (grp & 1) * 16 + (p & 3) * 4;
  typedef __attribute__((address_space(3))) short4v* lds_ptr;
  const short4v lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(at));
  const short4v hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(at + 4 * kWS));
  typedef short short8v __attribute__((ext_vector_type(8)));
  const short8v v = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
  return __builtin_bit_cast(bf16x8, v);
}

template <int BN, bool RELU>
__global__ __launch_bounds__(kHThreads, 2) void gemm_bf16_dw_kernel(const bf16_t* __restrict__ M, int64_t ldm,
                                                                    const float* __restrict__ dH,
                                                                    const float* __restrict__ Zs, int n, int f, int g,
                                                                    int slab_rows, float* __restrict__ part) {
  constexpr int TM = 2, TN = BN / 64;
  constexpr int AI = kWK * (kWM / 8) / kHThreads;   // 8-feature chunks of the M tile per thread (2)
  constexpr int BI = kWK * (BN / 4) / kHThreads;    // 4-column chunks of the dZ tile per thread (4 or 2)
  __shared__ __attribute__((aligned(16))) uint16_t As[kWK][kWS];
  __shared__ __attribute__((aligned(16))) uint16_t Bh[kWK][kWS];
  __shared__ __attribute__((aligned(16))) uint16_t Bl[kWK][kWS];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int l32 = lane & 31, lh = lane >> 5;

  // workgroup id -> (slab, tile): the tiles of one slab on ids that are equal modulo 8 (one XCD, shared L2)
  const int tiles_m = f / kWM, tiles_n = g / BN, tiles = tiles_m * tiles_n;
  const int group = blockIdx.x / (8 * tiles), within = blockIdx.x % (8 * tiles);
  const int slab = group * 8 + within % 8;
  if (static_cast<int64_t>(slab) * slab_rows >= n) return;
  const int t = within / 8;
  const int m0 = (t % tiles_m) * kWM, n0 = (t / tiles_m) * BN;
  const int kbeg = slab * slab_rows, kend = min(n, kbeg + slab_rows);

  u32x4 ra[AI];
  float4 rb[BI], rz[RELU ? BI : 1];
  // Branch-free loads (rows past the slab's end are clamped to its last row and zeroed when staged); the
  // ReLU mask and the split are applied at staging, after the current tile's products have been issued.
  auto fetch = [&](int k0) {
#pragma unroll
    for (int i = 0; i < AI; ++i) {
      const int c = tid + kHThreads * i;
      const int row = min(k0 + c / (kWM / 8), kend - 1), col = m0 + (c % (kWM / 8)) * 8;
      ra[i] = *reinterpret_cast<const u32x4*>(M + static_cast<int64_t>(row) * ldm + col);
    }
#pragma unroll
    for (int i = 0; i < BI; ++i) {
      const int c = tid + kHThreads * i;
      const int row = min(k0 + c / (BN / 4), kend - 1), col = n0 + (c % (BN / 4)) * 4;
      const int64_t off = static_cast<int64_t>(row) * g + col;
      rb[i] = *reinterpret_cast<const float4*>(dH + off);
      if (RELU) rz[i] = *reinterpret_cast<const float4*>(Zs + off);
    }
  };
  auto stage = [&](int k0) {
#pragma unroll
    for (int i = 0; i < AI; ++i) {
      const int c = tid + kHThreads * i;
      const bool in = k0 + c / (kWM / 8) < kend;
      *reinterpret_cast<u32x4*>(&As[c / (kWM / 8)][(c % (kWM / 8)) * 8]) = in ? ra[i] : u32x4{0u, 0u, 0u, 0u};
    }
#pragma unroll
    for (int i = 0; i < BI; ++i) {
      const int c = tid + kHThreads * i;
      const bool in = k0 + c / (BN / 4) < kend;
      const float4 z = rz[RELU ? i : 0];
      const float v[4] = {(in && (!RELU || z.x > 0.0f)) ? rb[i].x : 0.0f, (in && (!RELU || z.y > 0.0f)) ? rb[i].y : 0.0f,
                          (in && (!RELU || z.z > 0.0f)) ? rb[i].z : 0.0f, (in && (!RELU || z.w > 0.0f)) ? rb[i].w : 0.0f};
      uint16_t hi[4], lo[4];
#pragma unroll
      for (int j = 0; j < 4; ++j) split_bf16(v[j], hi[j], lo[j]);
      const int r = c / (BN / 4), col = (c % (BN / 4)) * 4;
      *reinterpret_cast<uint2*>(&Bh[r][col]) = make_uint2(hi[0] | (static_cast<uint32_t>(hi[1]) << 16),
                                                         hi[2] | (static_cast<uint32_t>(hi[3]) << 16));
      *reinterpret_cast<uint2*>(&Bl[r][col]) = make_uint2(lo[0] | (static_cast<uint32_t>(lo[1]) << 16),
                                                         lo[2] | (static_cast<uint32_t>(lo[3]) << 16));
    }
  };

  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.0f;

  fetch(kbeg);
  for (int k0 = kbeg; k0 < kend; k0 += kWK) {
    stage(k0);
    __syncthreads();
    if (k0 + kWK < kend) fetch(k0 + kWK);
#pragma unroll
    for (int ks = 0; ks < kWK; ks += 16) {
      // lane (l32, lh): output row / column l32 of its 32x32 tile, reduction rows ks + lh*8 .. + 7
      bf16x8 a[TM], bh[TN], bl[TN];
#pragma unroll
      for (int i = 0; i < TM; ++i) a[i] = read_tr8(&As[ks][0], wm * 64 + i * 32, lane);
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        bh[j] = read_tr8(&Bh[ks][0], wn * (BN / 2) + j * 32, lane);
        bl[j] = read_tr8(&Bl[ks][0], wn * (BN / 2) + j * 32, lane);
      }
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) {
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], bl[j], acc[i][j], 0, 0, 0);
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], bh[j], acc[i][j], 0, 0, 0);
        }
    }
    __syncthreads();
  }

  // lane holds column l32 and rows (e/4)*8 + lh*4 + e%4 of each 32x32 tile; every tile is full
  float* out = part + static_cast<int64_t>(slab) * f * g;
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      const int col = n0 + wn * (BN / 2) + j * 32 + l32;
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int row = m0 + wm * 64 + i * 32 + (e >> 2) * 8 + lh * 4 + (e & 3);
        out[static_cast<int64_t>(row) * g + col] = acc[i][j][e];
      }
    }
}

// The bf16 matrix-core dW kernel takes whole tiles only: 128 features x 64 or 128 columns, 16-byte
// aligned rows of M, dH and Zs.
bool dense_dw_bf16_ok(const void* M, int64_t ldm, const float* Zs, const float* dH, int32_t f_in, int32_t f_out) {
  return f_in % kWM == 0 && f_out % 64 == 0 && ldm % 8 == 0 && aligned(M, 16) && aligned(dH, 16) &&
         (!Zs || aligned(Zs, 16));
}

int launch_dense_dw_bf16(const void* M, int64_t ldm, const float* dH, const float* Zs, int32_t n, int32_t f_in,
                         int32_t f_out, int relu, int slab_rows, int slabs, float* part, hipStream_t st) {
  ProfScope ps(K_GEMM_DW, st);
  const bf16_t* m = static_cast<const bf16_t*>(M);
  const int bn = f_out % 128 == 0 ? 128 : 64;
  const int tiles = (f_in / kWM) * (f_out / bn);
  const unsigned grid = static_cast<unsigned>(ceil_div(slabs, 8) * 8 * tiles);
#define CDF_BF16_DW(BNV)                                                                                              \
  if (relu) gemm_bf16_dw_kernel<BNV, true><<<grid, kHThreads, 0, st>>>(m, ldm, dH, Zs, n, f_in, f_out, slab_rows, part); \
  else gemm_bf16_dw_kernel<BNV, false><<<grid, kHThreads, 0, st>>>(m, ldm, dH, Zs, n, f_in, f_out, slab_rows, part)
  if (bn == 128) { CDF_BF16_DW(128); }
  else { CDF_BF16_DW(64); }
#undef CDF_BF16_DW
  return CDF_OK;
}

bool dense_bwd_bf16_ok(const void* M, const float* W, const float* Zs, const float* dH, int32_t f_out) {
  return f_out % 8 == 0 && aligned(W, 16) && aligned(dH, 16) && (!Zs || aligned(Zs, 16)) && aligned(M, 2);
}

int launch_dense_dm_bf16(const float* dH, const float* Zs, const float* W, int32_t n, int32_t f_in, int32_t f_out,
                         int relu, void* dM, int64_t lddm, void* ws, size_t ws_bytes, hipStream_t st) {
  ProfScope ps(K_GEMM_DM, st);
  const int bn = f_in > 64 ? 128 : 64;
  const unsigned grid = xcd_grid(ceil_div(n, 128), ceil_div(f_in, bn));
  bf16_t* o = static_cast<bf16_t*>(dM);
  // with workspace the weight is split once (same layout as W) instead of in every block
  const int64_t count = static_cast<int64_t>(f_in) * f_out;
  const size_t half = align_up(static_cast<size_t>(count) * 2, 256);
  const bool pre = ws && aligned(ws, 256) && ws_bytes >= 2 * half;
  uint16_t* wh = static_cast<uint16_t*>(ws);
  uint16_t* wl = pre ? wh + half / 2 : nullptr;
  if (pre) split_kernel<<<static_cast<unsigned>(ceil_div(count, 8 * 256)), 256, 0, st>>>(W, count, wh, wl);
#define CDF_BF16_DM2(BNV, RELUV)                                                                                   \
  if (pre) gemm_bf16_dm_kernel<BNV, RELUV, true><<<grid, kHThreads, 0, st>>>(dH, Zs, W, wh, wl, n, f_in, f_out, o, lddm); \
  else gemm_bf16_dm_kernel<BNV, RELUV, false><<<grid, kHThreads, 0, st>>>(dH, Zs, W, nullptr, nullptr, n, f_in, f_out, o, lddm)
#define CDF_BF16_DM(BNV)                \
  if (relu) { CDF_BF16_DM2(BNV, true); } \
  else { CDF_BF16_DM2(BNV, false); }
  if (bn == 128) { CDF_BF16_DM(128); }
  else { CDF_BF16_DM(64); }
#undef CDF_BF16_DM
#undef CDF_BF16_DM2
  return CDF_OK;
}

// True when the bf16 matrix-core kernel can take the product (16-byte aligned rows of M).
bool dense_fwd_bf16_ok(const void* M, int64_t ldm, int32_t f_in) {
  return f_in % 8 == 0 && ldm % 8 == 0 && aligned(M, 16);
}

// Bytes of workspace with which the weight is split once instead of in every block.
size_t dense_fwd_bf16_workspace_bytes(int32_t f_in, int32_t f_out) {
  return align_up(static_cast<size_t>(f_in) * f_out * 2, 256) * 2;
}

int launch_dense_fwd_bf16(const void* M, int64_t ldm, const float* W, int32_t n, int32_t f_in, int32_t f_out, int relu,
                          float* Z, float* H, void* ws, size_t ws_bytes, hipStream_t st) {
  const bf16_t* m = static_cast<const bf16_t*>(M);
  // 128 columns per block at most: the wider tile measured slower (three resident blocks per compute
  // unit hide the barrier and LDS latency of this short pipeline better than one wide block)
  const int bn = f_out > 64 ? 128 : 64;
  const unsigned grid = xcd_grid(ceil_div(n, 128), ceil_div(f_out, bn));
  const bool pre = ws && aligned(ws, 256) && ws_bytes >= dense_fwd_bf16_workspace_bytes(f_in, f_out);
  uint16_t* wh = static_cast<uint16_t*>(ws);
  uint16_t* wl = pre ? wh + align_up(static_cast<size_t>(f_in) * f_out * 2, 256) / 2 : nullptr;
  ProfScope ps(K_GEMM_FWD, st);
  if (pre) {
    const dim3 sg(static_cast<unsigned>(ceil_div(f_in, 32)), static_cast<unsigned>(ceil_div(f_out, 32)));
    split_transpose_kernel<<<sg, 256, 0, st>>>(W, f_in, f_out, wh, wl);
  }
#define CDF_BF16_FWD(BNV)                                                                                            \
  if (pre) gemm_bf16_fwd_kernel<BNV, true><<<grid, kHThreads, 0, st>>>(m, ldm, W, wh, wl, n, f_in, f_out, relu, Z, H); \
  else gemm_bf16_fwd_kernel<BNV, false><<<grid, kHThreads, 0, st>>>(m, ldm, W, nullptr, nullptr, n, f_in, f_out, relu, Z, H)
  if (bn == 128) { CDF_BF16_FWD(128); }
  else { CDF_BF16_FWD(64); }
#undef CDF_BF16_FWD
  return CDF_OK;
}

}  // namespace cdf
