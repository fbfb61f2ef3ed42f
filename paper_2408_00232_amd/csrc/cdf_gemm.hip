// Dense transform of the layer and its gradients on the matrix cores (Sec. 3.1):
//   FWD : Z = M W,  H = relu(Z)                 [n x f] [f x g]
//   DM  : dM = dZ W^T,  dZ = dH * [Zs > 0]      [n x g] [g x f]
//   DW  : dW = M^T dZ                           [f x n] [n x g]   (n split into slabs)
// One tiled kernel serves the three products: a 128 x BN tile of the output per block of
// four wavefronts, fp32 MFMA 32x32x2, operands staged through LDS in k-major order
// (As[k][m], Bs[k][n]) so that a wavefront's operand read is two runs of 32
// consecutive floats. The next k-tile is fetched from global memory into registers while
// the current one is multiplied. The ReLU mask is applied while the dZ operand is loaded,
// so dZ never exists in memory. dW partial tiles of each row slab go to the workspace
// and are summed in slab order by a second kernel: no atomics, reproducible.
#include <type_traits>

#include "cdf_common.h"

namespace cdf {

typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int kBM = 128;
constexpr int kBK = 32;
constexpr int kGemmThreads = 256;

enum GemmMode { GEMM_FWD = 0, GEMM_DM = 1, GEMM_DW = 2 };

struct GemmArgs {
  // FWD: A = M (type T, ld lda), B = W           ; out0 = Z, out1 = H
  // DM : A = dH, Amask = Zs (fp32, ld = g)       ; B = W ; outT = dM (type T, ld ldo)
  // DW : A = M (type T), B = dH, Bmask = Zs      ; out0 = partial slabs
  const void* A;
  int64_t lda;
  const float* B;
  const float* mask;  // Zs or null
  float* out0;
  float* out1;
  void* outT;
  int64_t ldo;
  int n, f, g;        // problem: n rows, f_in, f_out
  int relu;
  int slab_rows;      // DW: rows of M / dZ per slab
};

template <typename T>
__device__ __forceinline__ float ld1(const T* p);
template <>
__device__ __forceinline__ float ld1<float>(const float* p) { return *p; }
template <>
__device__ __forceinline__ float ld1<bf16_t>(const bf16_t* p) { return bf2f(*p); }

// four consecutive elements starting at p (element index `at` of a run of `len` valid ones)
template <typename T>
__device__ __forceinline__ void load_quad(const T* p, int at, int len, bool vec_ok, float (&v)[4]) {
  if (vec_ok && at + 4 <= len) {
    VecIO<T, 4>::load(p, v);
  } else {
#pragma unroll
    for (int c = 0; c < 4; ++c) v[c] = at + c < len ? ld1<T>(p + c) : 0.0f;
  }
}

// FAST: every operand row is 16-byte aligned and the row widths are multiples of four (no scalar
// fall-back); decided on the host. Loads then carry no branches: addresses are clamped into the operand
// (rows and columns past the edge feed outputs that are never stored), reduction elements past the end
// are zeroed when the tile is staged, and so is the ReLU mask applied, so that nothing waits for a
// load before the products of the current tile have been issued.
template <typename T>
__device__ __forceinline__ void load_quad_fast(const T* p, float (&v)[4]) { VecIO<T, 4>::load(p, v); }

template <typename T, int MODE, int BN, bool FAST>
__global__ __launch_bounds__(kGemmThreads, 2) void gemm_kernel(GemmArgs a, int a_vec, int b_vec, int m_vec) {
  // LDS row strides. Tiles written with 16-byte vectors need rows that are multiples of 4 floats;
  // tiles written transposed (one float per lane, k = 4 (tid % 8) + c, column = tid / 8 + 32 i) use a
  // stride that is 2 mod 8, which spreads the 64 lanes of a store over all 32 banks (two lanes per
  // bank, the minimum) instead of 16 banks.
  constexpr int kSA = MODE == GEMM_DW ? kBM + 4 : kBM + 2;
  constexpr int SB = MODE == GEMM_DM ? BN + 2 : BN + 4;
  constexpr int TN = BN / 64;   // 32-wide MFMA tiles per wavefront along n (waves are 2 x 2)
  constexpr int TM = 2;
  constexpr int BQ = BN / 32;   // B quads per thread
  __shared__ float As[kBK][kSA];
  __shared__ float Bs[kBK][SB];

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;

  // output tile and reduction range
  int Mdim, Ndim, Kbeg, Kend;
  if (MODE == GEMM_FWD) { Mdim = a.n; Ndim = a.g; Kbeg = 0; Kend = a.f; }
  else if (MODE == GEMM_DM) { Mdim = a.n; Ndim = a.f; Kbeg = 0; Kend = a.g; }
  else { Mdim = a.f; Ndim = a.g; Kbeg = 0; Kend = 0; }
  // FWD / DM: grid (row tiles, column tiles). DW: a 1-D grid decoded so that the tiles of one row slab
  // (which share the slab's M rows and dZ rows) carry workgroup ids that are equal modulo 8 and follow
  // each other closely: workgroups go to the eight XCDs round-robin, so the slab's operands are then
  // fetched into one L2 once instead of into several.
  int tile_m = blockIdx.x, tile_n = blockIdx.y, slab = 0;
  if (MODE == GEMM_DW) {
    const int tiles_m = (a.f + kBM - 1) / kBM, tiles_n = (a.g + BN - 1) / BN, tiles = tiles_m * tiles_n;
    const int group = blockIdx.x / (8 * tiles), within = blockIdx.x % (8 * tiles);
    const int t = within / 8;
    slab = group * 8 + within % 8;
    if (static_cast<int64_t>(slab) * a.slab_rows >= a.n) return;   // padding of the last group (uniform per block)
    tile_m = t % tiles_m;
    tile_n = t / tiles_m;
    Kbeg = slab * a.slab_rows;
    Kend = min(a.n, Kbeg + a.slab_rows);
  }
  const int m0 = tile_m * kBM;
  const int n0 = tile_n * BN;

  const T* Ap = static_cast<const T*>(a.A);
  const float* dHp = static_cast<const float*>(a.A);

  float ra[4][4];
  float rb[BQ][4];
  float rz[FAST && MODE != GEMM_FWD ? (MODE == GEMM_DM ? 4 : BQ) : 1][4];   // Zs beside dH, masked at staging

  auto fetch_fast = [&](int k0) {
    if (MODE == GEMM_FWD || MODE == GEMM_DM) {
      // A[m][k] contiguous along k: quad (row = tid/8 + 32 i, k = (tid%8)*4)
      const int k = min(k0 + (tid & 7) * 4, Kend - 4);
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int m = min(m0 + (tid >> 3) + 32 * i, Mdim - 1);
        if (MODE == GEMM_FWD) {
          load_quad_fast<T>(Ap + static_cast<int64_t>(m) * a.lda + k, ra[i]);
        } else {
          const int64_t off = static_cast<int64_t>(m) * a.g + k;
          load_quad_fast<float>(dHp + off, ra[i]);
          if (a.relu) load_quad_fast<float>(a.mask + off, rz[i]);
        }
      }
    } else {
      // A[m = feature][k = row] = M[row][feature], contiguous along m: quad (k = tid/32 + 8 i, m = (tid%32)*4)
      const int m = min(m0 + (tid & 31) * 4, Mdim - 4);
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int k = min(k0 + (tid >> 5) + 8 * i, Kend - 1);
        load_quad_fast<T>(Ap + static_cast<int64_t>(k) * a.lda + m, ra[i]);
      }
    }
    if (MODE == GEMM_DM) {
      // B[k = out feature][n = in feature] = W[n][k], contiguous along k: quad (n = tid/8 + 32 i, k = (tid%8)*4)
      const int k = min(k0 + (tid & 7) * 4, Kend - 4);
#pragma unroll
      for (int i = 0; i < BQ; ++i) {
        const int n = min(n0 + (tid >> 3) + 32 * i, Ndim - 1);
        load_quad_fast<float>(a.B + static_cast<int64_t>(n) * a.g + k, rb[i]);
      }
    } else {
      // W[k][n] / dZ[k = row][n], contiguous along n: quad (k = tid/(BN/4) + (1024/BN) i, n = (tid % (BN/4)) * 4)
      const int n = min(n0 + (tid % (BN / 4)) * 4, Ndim - 4);
#pragma unroll
      for (int i = 0; i < BQ; ++i) {
        const int k = min(k0 + tid / (BN / 4) + (1024 / BN) * i, Kend - 1);
        const int64_t off = static_cast<int64_t>(k) * a.g + n;
        load_quad_fast<float>(a.B + off, rb[i]);
        if (MODE == GEMM_DW && a.relu) load_quad_fast<float>(a.mask + off, rz[i]);
      }
    }
  };
  // FAST: zero what lies past the end of the reduction and apply the ReLU mask, in registers, before staging
  auto finish_fast = [&](int k0) {
    if (MODE == GEMM_FWD || MODE == GEMM_DM) {
      const bool kin = k0 + (tid & 7) * 4 < Kend;
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int c = 0; c < 4; ++c) {
          const bool keep = kin && (MODE == GEMM_FWD || !a.relu || rz[MODE == GEMM_DM ? i : 0][c] > 0.0f);
          ra[i][c] = keep ? ra[i][c] : 0.0f;
        }
    } else {
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const bool kin = k0 + (tid >> 5) + 8 * i < Kend;
#pragma unroll
        for (int c = 0; c < 4; ++c) ra[i][c] = kin ? ra[i][c] : 0.0f;
      }
    }
    if (MODE == GEMM_DM) {
      const bool kin = k0 + (tid & 7) * 4 < Kend;
#pragma unroll
      for (int i = 0; i < BQ; ++i)
#pragma unroll
        for (int c = 0; c < 4; ++c) rb[i][c] = kin ? rb[i][c] : 0.0f;
    } else {
#pragma unroll
      for (int i = 0; i < BQ; ++i) {
        const bool kin = k0 + tid / (BN / 4) + (1024 / BN) * i < Kend;
#pragma unroll
        for (int c = 0; c < 4; ++c) {
          const bool keep = kin && (MODE != GEMM_DW || !a.relu || rz[MODE == GEMM_DW ? i : 0][c] > 0.0f);
          rb[i][c] = keep ? rb[i][c] : 0.0f;
        }
      }
    }
  };

  // general path: bounds checks and scalar fall-backs, the mask applied as the operand is loaded
  auto fetch = [&](int k0) {
    if (FAST) {
      fetch_fast(k0);
      return;
    }
    // ---- A operand ----
    if (MODE == GEMM_FWD) {
      // M[m][k], contiguous along k: quad (row = tid/8 + 32 i, k = (tid%8)*4)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int m = m0 + (tid >> 3) + 32 * i;
        const int k = k0 + (tid & 7) * 4;
        if (m < Mdim && k < Kend) load_quad<T>(Ap + static_cast<int64_t>(m) * a.lda + k, k, Kend, a_vec, ra[i]);
        else ra[i][0] = ra[i][1] = ra[i][2] = ra[i][3] = 0.0f;
      }
    } else if (MODE == GEMM_DM) {
      // dZ[m][k] = dH[m][k] * [Zs[m][k] > 0], row-major n x g
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int m = m0 + (tid >> 3) + 32 * i;
        const int k = k0 + (tid & 7) * 4;
        if (m < Mdim && k < Kend) {
          const int64_t off = static_cast<int64_t>(m) * a.g + k;
          load_quad<float>(dHp + off, k, Kend, a_vec, ra[i]);
          if (a.relu) {
            float z[4];
            load_quad<float>(a.mask + off, k, Kend, m_vec, z);
#pragma unroll
            for (int c = 0; c < 4; ++c) ra[i][c] = z[c] > 0.0f ? ra[i][c] : 0.0f;
          }
        } else ra[i][0] = ra[i][1] = ra[i][2] = ra[i][3] = 0.0f;
      }
    } else {
      // A[m = feature][k = row] = M[row][feature], contiguous along m: quad (k = tid/32 + 8 i, m = (tid%32)*4)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int k = k0 + (tid >> 5) + 8 * i;
        const int m = m0 + (tid & 31) * 4;
        if (k < Kend && m < Mdim) load_quad<T>(Ap + static_cast<int64_t>(k) * a.lda + m, m, Mdim, a_vec, ra[i]);
        else ra[i][0] = ra[i][1] = ra[i][2] = ra[i][3] = 0.0f;
      }
    }
    // ---- B operand ----
    if (MODE == GEMM_FWD) {
      // W[k][n], contiguous along n: quad (k = tid/(BN/4) + (1024/BN) i, n = (tid % (BN/4)) * 4)
#pragma unroll
      for (int i = 0; i < BQ; ++i) {
        const int k = k0 + tid / (BN / 4) + (1024 / BN) * i;
        const int n = n0 + (tid % (BN / 4)) * 4;
        if (k < Kend && n < Ndim) load_quad<float>(a.B + static_cast<int64_t>(k) * a.g + n, n, Ndim, b_vec, rb[i]);
        else rb[i][0] = rb[i][1] = rb[i][2] = rb[i][3] = 0.0f;
      }
    } else if (MODE == GEMM_DM) {
      // B[k = out feature][n = in feature] = W[n][k], contiguous along k: quad (n = tid/8 + 32 i, k = (tid%8)*4)
#pragma unroll
      for (int i = 0; i < BQ; ++i) {
        const int n = n0 + (tid >> 3) + 32 * i;
        const int k = k0 + (tid & 7) * 4;
        if (n < Ndim && k < Kend) load_quad<float>(a.B + static_cast<int64_t>(n) * a.g + k, k, Kend, b_vec, rb[i]);
        else rb[i][0] = rb[i][1] = rb[i][2] = rb[i][3] = 0.0f;
      }
    } else {
      // dZ[k = row][n], contiguous along n
#pragma unroll
      for (int i = 0; i < BQ; ++i) {
        const int k = k0 + tid / (BN / 4) + (1024 / BN) * i;
        const int n = n0 + (tid % (BN / 4)) * 4;
        if (k < Kend && n < Ndim) {
          const int64_t off = static_cast<int64_t>(k) * a.g + n;
          load_quad<float>(a.B + off, n, Ndim, b_vec, rb[i]);
          if (a.relu) {
            float z[4];
            load_quad<float>(a.mask + off, n, Ndim, m_vec, z);
#pragma unroll
            for (int c = 0; c < 4; ++c) rb[i][c] = z[c] > 0.0f ? rb[i][c] : 0.0f;
          }
        } else rb[i][0] = rb[i][1] = rb[i][2] = rb[i][3] = 0.0f;
      }
    }
  };

  auto stage = [&](int k0) {
    if (FAST) finish_fast(k0);
    if (MODE == GEMM_DW) {
#pragma unroll
      for (int i = 0; i < 4; ++i)
        *reinterpret_cast<float4*>(&As[(tid >> 5) + 8 * i][(tid & 31) * 4]) =
            make_float4(ra[i][0], ra[i][1], ra[i][2], ra[i][3]);
    } else {
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int c = 0; c < 4; ++c) As[(tid & 7) * 4 + c][(tid >> 3) + 32 * i] = ra[i][c];
    }
    if (MODE == GEMM_DM) {
#pragma unroll
      for (int i = 0; i < BQ; ++i)
#pragma unroll
        for (int c = 0; c < 4; ++c) Bs[(tid & 7) * 4 + c][(tid >> 3) + 32 * i] = rb[i][c];
    } else {
#pragma unroll
      for (int i = 0; i < BQ; ++i)
        *reinterpret_cast<float4*>(&Bs[tid / (BN / 4) + (1024 / BN) * i][(tid % (BN / 4)) * 4]) =
            make_float4(rb[i][0], rb[i][1], rb[i][2], rb[i][3]);
    }
  };

  floatx16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.0f;

  const int l32 = lane & 31, lh = lane >> 5;
  if (Kbeg < Kend) fetch(Kbeg);
  for (int k0 = Kbeg; k0 < Kend; k0 += kBK) {
    stage(k0);
    __syncthreads();
    if (k0 + kBK < Kend) fetch(k0 + kBK);
    // operands of step kk + 2 are read from LDS while the products of step kk run
    float fa[2][TM], fb[2][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i) fa[0][i] = As[lh][wm * 64 + i * 32 + l32];
#pragma unroll
    for (int j = 0; j < TN; ++j) fb[0][j] = Bs[lh][wn * (BN / 2) + j * 32 + l32];
#pragma unroll
    for (int kk = 0; kk < kBK; kk += 2) {
      const int cur = (kk >> 1) & 1, nxt = cur ^ 1;
      if (kk + 2 < kBK) {
#pragma unroll
        for (int i = 0; i < TM; ++i) fa[nxt][i] = As[kk + 2 + lh][wm * 64 + i * 32 + l32];
#pragma unroll
        for (int j = 0; j < TN; ++j) fb[nxt][j] = Bs[kk + 2 + lh][wn * (BN / 2) + j * 32 + l32];
      }
      __builtin_amdgcn_sched_barrier(0);   // keep the LDS reads above the products they overlap with
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[cur][i], fb[cur][j], acc[i][j], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
    }
    __syncthreads();
  }

  // ---- epilogue: lane holds column l32 and rows (e/4)*8 + lh*4 + e%4 of each 32x32 tile ----
  // A workgroup whose tile lies inside the output stores without per-element checks (one uniform branch).
  auto store_tile = [&](auto checked) {
    constexpr bool CHECK = decltype(checked)::value;
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        const int col = n0 + wn * (BN / 2) + j * 32 + l32;
        if (CHECK && col >= Ndim) continue;
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          const int row = m0 + wm * 64 + i * 32 + (e >> 2) * 8 + lh * 4 + (e & 3);
          if (CHECK && row >= Mdim) continue;
          const float v = acc[i][j][e];
          if (MODE == GEMM_FWD) {
            const int64_t off = static_cast<int64_t>(row) * a.g + col;
            if (a.out0) a.out0[off] = v;
            if (a.out1) a.out1[off] = a.relu ? (v > 0.0f ? v : 0.0f) : v;
          } else if (MODE == GEMM_DM) {
            T* o = static_cast<T*>(a.outT) + static_cast<int64_t>(row) * a.ldo + col;
            float one[1] = {v};
            VecIO<T, 1>::store(o, one);
          } else {
            a.out0[(static_cast<int64_t>(slab) * a.f + row) * a.g + col] = v;
          }
        }
      }
  };
  if (m0 + kBM <= Mdim && n0 + BN <= Ndim) store_tile(std::false_type{});
  else store_tile(std::true_type{});
}

// dW[i] = sum over slabs in a fixed order: four interleaved running sums (slab k goes to sum
// k mod 4), combined as (s0 + s1) + (s2 + s3). 64 outputs per block of 256 threads.
__global__ __launch_bounds__(256) void reduce_slabs_kernel(const float* __restrict__ part, int slabs, int64_t count,
                                                           float* __restrict__ out) {
  __shared__ float sh[4][64];
  const int e = threadIdx.x & 63, g = threadIdx.x >> 6;
  const int64_t i = static_cast<int64_t>(blockIdx.x) * 64 + e;
  float s = 0.0f;
  if (i < count)
    for (int k = g; k < slabs; k += 4) s = s + part[k * count + i];
  sh[g][e] = s;
  __syncthreads();
  if (g == 0 && i < count) out[i] = (sh[0][e] + sh[1][e]) + (sh[2][e] + sh[3][e]);
}

constexpr size_t kDwPartialCap = size_t(512) << 20;  // bytes of slab partials at most

constexpr int kDwMinSlab = 256;  // rows per slab at least (a multiple of the k-tile)

static void dw_split(int n, int f, int g, int* slab_rows, int* slabs) {
  int64_t rows = kDwMinSlab;
  const size_t per = static_cast<size_t>(f) * g * sizeof(float);
  // enough blocks to fill the chip a few times over (tiles x slabs >= ~1500), not more
  const int64_t tiles = ceil_div(f, kBM) * ceil_div(g, g > 64 ? 128 : 64);
  // (both loops stop at one slab at the latest: rows >= n)
  while (rows < n && ceil_div(n, rows * 2) * tiles >= 1536) rows *= 2;
  while (rows < n && static_cast<size_t>(ceil_div(n, rows)) * per > kDwPartialCap) rows *= 2;
  *slab_rows = static_cast<int>(rows);
  *slabs = static_cast<int>(ceil_div(n > 0 ? n : 1, rows));
}

// Upper bound of the slab partials for any n' <= n, f' <= f, g' <= g (so that a workspace sized
// for the largest layer serves every layer): the split keeps slabs * tiles below about 3072 and
// a tile's partial is at most 128 x 256 floats; never more than one slab per kDwMinSlab rows.
size_t dense_workspace_bytes(int64_t n, int32_t f, int32_t g) {
  const size_t tiles = static_cast<size_t>(ceil_div(f, kBM)) * static_cast<size_t>(ceil_div(g, 64));
  const size_t by_grid = (3072 + tiles) * static_cast<size_t>(kBM) * 256 * sizeof(float);
  const size_t by_rows = static_cast<size_t>(ceil_div(n > 0 ? n : 1, kDwMinSlab)) * f * g * sizeof(float);
  return align_up(by_grid < by_rows ? by_grid : by_rows, 256);
}

template <typename T, int MODE>
static void launch_gemm(const GemmArgs& a, int Mdim, int Ndim, int slabs, int a_vec, int b_vec, int m_vec,
                        hipStream_t st) {
  ProfScope ps(MODE == GEMM_FWD ? K_GEMM_FWD : MODE == GEMM_DW ? K_GEMM_DW : K_GEMM_DM, st);
  // wide outputs: 256 columns per block so that the A operand is read once (the slab-split dW
  // product has enough blocks already and runs better on 128)
  const int bn = Ndim > 128 && MODE != GEMM_DW ? 256 : Ndim > 64 ? 128 : 64;
  // the branch-free loads need 16-byte aligned rows and widths that are multiples of four, not whole tiles
  const bool fast = a.f % 4 == 0 && a.g % 4 == 0 && a_vec && b_vec && (!a.relu || MODE == GEMM_FWD || m_vec);
  dim3 grid(static_cast<unsigned>(ceil_div(Mdim, kBM)), static_cast<unsigned>(ceil_div(Ndim, bn)), 1);
  if (MODE == GEMM_DW)   // 1-D: groups of eight slabs, all tiles of a slab on ids that are equal modulo 8
    grid = dim3(static_cast<unsigned>(ceil_div(slabs, 8) * 8 * grid.x * grid.y), 1, 1);
  if (bn == 256) {
    if (fast) gemm_kernel<T, MODE, 256, true><<<grid, kGemmThreads, 0, st>>>(a, a_vec, b_vec, m_vec);
    else gemm_kernel<T, MODE, 256, false><<<grid, kGemmThreads, 0, st>>>(a, a_vec, b_vec, m_vec);
  } else if (bn == 128) {
    if (fast) gemm_kernel<T, MODE, 128, true><<<grid, kGemmThreads, 0, st>>>(a, a_vec, b_vec, m_vec);
    else gemm_kernel<T, MODE, 128, false><<<grid, kGemmThreads, 0, st>>>(a, a_vec, b_vec, m_vec);
  } else {
    if (fast) gemm_kernel<T, MODE, 64, true><<<grid, kGemmThreads, 0, st>>>(a, a_vec, b_vec, m_vec);
    else gemm_kernel<T, MODE, 64, false><<<grid, kGemmThreads, 0, st>>>(a, a_vec, b_vec, m_vec);
  }
}

static bool vec4(const void* p, int64_t ld, size_t esz) { return aligned(p, 4 * esz) && ld % 4 == 0; }

// bf16 matrix-core kernels for bf16-stored activations
bool dense_fwd_bf16_ok(const void* M, int64_t ldm, int32_t f_in);
int launch_dense_fwd_bf16(const void* M, int64_t ldm, const float* W, int32_t n, int32_t f_in, int32_t f_out, int relu,
                          float* Z, float* H, void* ws, size_t ws_bytes, hipStream_t st);
bool dense_bwd_bf16_ok(const void* M, const float* W, const float* Zs, const float* dH, int32_t f_out);
int launch_dense_dm_bf16(const float* dH, const float* Zs, const float* W, int32_t n, int32_t f_in, int32_t f_out,
                         int relu, void* dM, int64_t lddm, void* ws, size_t ws_bytes, hipStream_t st);
bool dense_dw_bf16_ok(const void* M, int64_t ldm, const float* Zs, const float* dH, int32_t f_in, int32_t f_out);
int launch_dense_dw_bf16(const void* M, int64_t ldm, const float* dH, const float* Zs, int32_t n, int32_t f_in,
                         int32_t f_out, int relu, int slab_rows, int slabs, float* part, hipStream_t st);

}  // namespace cdf

using namespace cdf;

namespace cdf {
// The dense forward product with an optional workspace (the layer steps have one): with it the bf16
// path splits the weight once per call instead of once per block.
int dense_fwd_ws(const void* M, int64_t ldm, cdf_dtype dt, const float* W, int32_t n, int32_t f_in, int32_t f_out,
                 int relu, float* Z, float* H, void* ws, size_t ws_bytes, void* stream) {
  hipStream_t st = static_cast<hipStream_t>(stream);
  CDF_REQUIRE(n >= 0 && f_in > 0 && f_out > 0 && ldm >= f_in, "cdf_dense_fwd: bad shape n=%d f_in=%d f_out=%d ldm=%lld",
              n, f_in, f_out, (long long)ldm);
  if (dt != CDF_F32 && dt != CDF_BF16) CDF_FAIL(CDF_ERR_UNSUPPORTED, "cdf_dense_fwd: dtype %d", (int)dt);
  if (n == 0) return CDF_OK;
  CDF_REQUIRE(M && W && (Z || H), "cdf_dense_fwd: null pointer");
  const size_t esz = elem_bytes(dt);
  CDF_REQUIRE(aligned(M, esz) && aligned(W, 4) && aligned(Z, 4) && aligned(H, 4), "cdf_dense_fwd: misaligned pointer");
  GemmArgs a = {};
  a.A = M; a.lda = ldm; a.B = W; a.out0 = Z; a.out1 = H; a.n = n; a.f = f_in; a.g = f_out; a.relu = relu ? 1 : 0;
  const int av = vec4(M, ldm, esz), bv = vec4(W, f_out, 4);
  if (dt == CDF_F32) launch_gemm<float, GEMM_FWD>(a, n, f_out, 1, av, bv, 0, st);
  else if (dense_fwd_bf16_ok(M, ldm, f_in)) launch_dense_fwd_bf16(M, ldm, W, n, f_in, f_out, relu ? 1 : 0, Z, H, ws, ws_bytes, st);
  else launch_gemm<bf16_t, GEMM_FWD>(a, n, f_out, 1, av, bv, 0, st);
  CDF_LAUNCH_CHECK("cdf_dense_fwd");
  return CDF_OK;
}
}  // namespace cdf

extern "C" int cdf_dense_fwd(const void* M, int64_t ldm, cdf_dtype dt, const float* W, int32_t n, int32_t f_in,
                             int32_t f_out, int relu, float* Z, float* H, void* stream) {
  return dense_fwd_ws(M, ldm, dt, W, n, f_in, f_out, relu, Z, H, nullptr, 0, stream);
}

extern "C" int cdf_dense_bwd(const void* M, int64_t ldm, cdf_dtype dt, const float* W, const float* Zs,
                             const float* dH, int32_t n, int32_t f_in, int32_t f_out, int relu, float* dW, void* dM,
                             int64_t lddm, void* ws, size_t ws_bytes, void* stream) {
  hipStream_t st = static_cast<hipStream_t>(stream);
  CDF_REQUIRE(n >= 0 && f_in > 0 && f_out > 0 && ldm >= f_in && (!dM || lddm >= f_in),
              "cdf_dense_bwd: bad shape n=%d f_in=%d f_out=%d ldm=%lld lddm=%lld", n, f_in, f_out, (long long)ldm,
              (long long)lddm);
  if (dt != CDF_F32 && dt != CDF_BF16) CDF_FAIL(CDF_ERR_UNSUPPORTED, "cdf_dense_bwd: dtype %d", (int)dt);
  CDF_REQUIRE(dW != nullptr, "cdf_dense_bwd: dW is null");
  CDF_REQUIRE(n == 0 || (M && W && dH && (!relu || Zs)), "cdf_dense_bwd: null pointer");
  const size_t esz = elem_bytes(dt);
  CDF_REQUIRE(aligned(M, esz) && aligned(W, 4) && aligned(Zs, 4) && aligned(dH, 4) && aligned(dW, 4) &&
                  aligned(dM, esz),
              "cdf_dense_bwd: misaligned pointer");
  int slab_rows, slabs;
  dw_split(n, f_in, f_out, &slab_rows, &slabs);
  const size_t need = align_up(static_cast<size_t>(slabs) * f_in * f_out * sizeof(float), 256);
  if (!ws || !aligned(ws, 16) || ws_bytes < need)
    CDF_FAIL(CDF_ERR_WORKSPACE, "cdf_dense_bwd: workspace too small (%zu < %zu)", ws_bytes, need);
  float* part = static_cast<float*>(ws);
  const int64_t count = static_cast<int64_t>(f_in) * f_out;
  // bf16-stored activations: dM and (for whole 128 x 64 tiles) dW on the bf16 matrix cores, fp32 operands
  // split into a bf16 high and low part
  const bool bf16_cores = dt == CDF_BF16 && n > 0 && dense_bwd_bf16_ok(M, W, relu ? Zs : nullptr, dH, f_out);
  // dW = M^T dZ
  {
    GemmArgs a = {};
    a.A = M; a.lda = ldm; a.B = dH; a.mask = Zs; a.out0 = part; a.n = n; a.f = f_in; a.g = f_out;
    a.relu = relu ? 1 : 0; a.slab_rows = slab_rows;
    const int av = vec4(M, ldm, esz), bv = vec4(dH, f_out, 4), mv = relu ? vec4(Zs, f_out, 4) : 0;
    if (dt == CDF_F32) launch_gemm<float, GEMM_DW>(a, f_in, f_out, slabs, av, bv, mv, st);
    else if (n > 0 && dense_dw_bf16_ok(M, ldm, relu ? Zs : nullptr, dH, f_in, f_out))
      launch_dense_dw_bf16(M, ldm, dH, relu ? Zs : nullptr, n, f_in, f_out, relu ? 1 : 0, slab_rows, slabs, part, st);
    else launch_gemm<bf16_t, GEMM_DW>(a, f_in, f_out, slabs, av, bv, mv, st);
    CDF_LAUNCH_CHECK("cdf_dense_bwd/dW");
    {
      ProfScope ps(K_GEMM_DW_REDUCE, st);
      reduce_slabs_kernel<<<static_cast<unsigned>(ceil_div(count, 64)), 256, 0, st>>>(part, slabs, count, dW);
    }
    CDF_LAUNCH_CHECK("cdf_dense_bwd/reduce");
  }
  // dM = dZ W^T
  if (dM && n > 0) {
    GemmArgs a = {};
    a.A = dH; a.lda = f_out; a.B = W; a.mask = Zs; a.outT = dM; a.ldo = lddm; a.n = n; a.f = f_in; a.g = f_out;
    a.relu = relu ? 1 : 0;
    const int av = vec4(dH, f_out, 4), bv = vec4(W, f_out, 4), mv = relu ? vec4(Zs, f_out, 4) : 0;
    if (dt == CDF_F32) launch_gemm<float, GEMM_DM>(a, n, f_in, 1, av, bv, mv, st);
    // (the workspace is free again: the slab partials of dW have been reduced on this stream)
    else if (bf16_cores) launch_dense_dm_bf16(dH, Zs, W, n, f_in, f_out, relu ? 1 : 0, dM, lddm, ws, ws_bytes, st);
    else launch_gemm<bf16_t, GEMM_DM>(a, n, f_in, 1, av, bv, mv, st);
    CDF_LAUNCH_CHECK("cdf_dense_bwd/dM");
  }
  return CDF_OK;
}
