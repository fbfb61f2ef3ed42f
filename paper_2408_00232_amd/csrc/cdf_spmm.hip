// CSR aggregation Y = A X over the normalised adjacency (Sec. 3.1) and its transposed
// counterpart for back-propagation (the same kernel on the CSR of A^T).
//
// Work split: the stored entries are cut into chunks of 64 to 1024 consecutive entries and
// each wavefront takes one chunk, whatever rows it covers - a power-law degree
// distribution (rows of 1 to several 10^5 entries) therefore loads every wavefront
// equally. Inside a chunk the wavefront walks the entries in storage order: the 64
// lanes first fetch 64 (column, value) pairs with one coalesced load each, then the
// entries' feature rows are gathered, several gather instructions in flight at a time,
// and accumulated in fp32 registers. Row ends are wave-uniform: at a row end the
// accumulator is stored as one coalesced row of Y.
//
// Two kernels. spmm_kernel gives the whole wavefront to one entry at a time (lane l reads
// elements [l*EPV, l*EPV+EPV) of each 64*EPV-wide pass; column ids and values reach all lanes
// through v_readlane). spmm_sliced_kernel gives LPR lanes to an entry, so one gather
// instruction serves 64 / LPR entries: rows of whole 128-byte lines are processed in vertical
// slices of one line (LPR = 8), rows of at most 32 lane-vectors in one slice whose lane group is
// just wide enough for the row (LPR = 2 ... 32).
//
// Rows that straddle chunk borders: the piece at the start of a chunk that continues an
// earlier row goes to phead[chunk], the piece at the end of a chunk that continues into
// the next goes to ptail[chunk] (both fp32); a second kernel adds a row's pieces in
// chunk order and writes the row once. No atomics: results are bit-reproducible.
#include "cdf_common.h"

namespace cdf {

constexpr int kChunk = 256;        // stored entries per wavefront on matrices of 1 M entries or more (smallest there)
constexpr int kSpmmThreads = 256;  // 4 wavefronts per block
constexpr int kSpmmWaves = kSpmmThreads / 64;

// chunk_row[c] = row that holds stored entry c*chunk (c >= 1; entry 0 is handled as row 0).
__global__ void chunk_rows_kernel(const int64_t* __restrict__ rowptr, int n_rows, int* __restrict__ chunk_row,
                                  int kChunk) {
  const int r = blockIdx.x * blockDim.x + threadIdx.x;
  if (r >= n_rows) return;
  const int64_t a = rowptr[r], b = rowptr[r + 1];
  for (int64_t c = (a + kChunk - 1) / kChunk; c * kChunk < b; ++c) chunk_row[c] = r;
}

// The dense transform of the layer applied to every finished row (Sec. 3.1, first equation as one
// kernel): z = m W for the aggregated row m, W [dim x G] with G <= 64, kept in LDS.
struct XformArgs {
  const float* W;  // dim x G, row-major
  float* Z;        // nullable, rows x G
  float* H;        // nullable, rows x G: relu ? max(z, 0) : z
  int G;
  int relu;
};

// z[lane] = sum_f row[f] * W[f][lane] for lane < G, f ascending, one fused multiply-add each; `row` is
// in LDS (every lane reads the same address: a broadcast), W in LDS or global memory.
__device__ __forceinline__ void transform_row(const float* row, const float* W, int dim, const XformArgs& xf,
                                              int64_t out_row, int lane) {
  if (lane >= xf.G) return;
  float z = 0.0f;
  int f = 0;
  for (; f + 4 <= dim; f += 4) {
    const float4 m = *reinterpret_cast<const float4*>(row + f);
    z = __fmaf_rn(m.x, W[(f + 0) * xf.G + lane], z);
    z = __fmaf_rn(m.y, W[(f + 1) * xf.G + lane], z);
    z = __fmaf_rn(m.z, W[(f + 2) * xf.G + lane], z);
    z = __fmaf_rn(m.w, W[(f + 3) * xf.G + lane], z);
  }
  for (; f < dim; ++f) z = __fmaf_rn(row[f], W[f * xf.G + lane], z);
  const int64_t at = out_row * xf.G + lane;
  if (xf.Z) xf.Z[at] = z;
  if (xf.H) xf.H[at] = xf.relu ? (z > 0.0f ? z : 0.0f) : z;
}

// LDS of the transforming variants: W, then one row buffer per wavefront (rows padded to 4 floats)
__host__ __device__ inline int xf_row_floats(int dim) { return (dim + 3) / 4 * 4; }

template <typename T, int EPV, int NP, bool XF = false>
__global__ __launch_bounds__(kSpmmThreads) void spmm_kernel(
    const int64_t* __restrict__ rowptr, const int* __restrict__ colidx, const float* __restrict__ vals,
    int n_rows, int64_t nnz, const T* __restrict__ X, int64_t ldx, T* __restrict__ Y, T* __restrict__ Y2,
    int64_t ldy, int dim, const int* __restrict__ chunk_row, int64_t nchunks, float* __restrict__ phead, float* __restrict__ ptail,
    int* __restrict__ tail_row, int kChunk, XformArgs xf) {
  constexpr int U = (8 / NP) > 0 ? (8 / NP) : 1;  // feature rows in flight per wavefront
  extern __shared__ __align__(16) float xf_lds[];
  const int lane = threadIdx.x & 63;
  // the wavefront index is the same in all lanes: say so, and everything derived from it
  // (chunk bounds, row cursor, loop counters) lives in scalar registers
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  if constexpr (XF) {
    for (int i = threadIdx.x; i < dim * xf.G; i += kSpmmThreads) xf_lds[i] = xf.W[i];
    __syncthreads();
  }
  const int64_t chunk = static_cast<int64_t>(blockIdx.x) * kSpmmWaves + wave;
  if (chunk >= nchunks) return;
  const int64_t s = chunk * kChunk;
  const int L = static_cast<int>(nnz - s < kChunk ? nnz - s : kChunk);
  int my_col = 0, krel = 0;
  float my_val = 0.0f;

  int r = chunk == 0 ? 0 : chunk_row[chunk];
  bool head = chunk > 0 && rowptr[r] < s;

  // window of 64 row ends, relative to s and clipped, one per lane
  auto load_rel = [&](int rbase) -> int {
    const int rr = rbase + lane;
    if (rr < n_rows) {
      const int64_t d = rowptr[rr + 1] - s;
      return d > kChunk ? kChunk + 1 : static_cast<int>(d);
    }
    return kChunk + 2;  // past the last row: matches nothing
  };
  int r_base = r;
  int rel = load_rel(r_base);
  int cur_end = __builtin_amdgcn_readlane(rel, 0);

  bool col_on[NP];
#pragma unroll
  for (int p = 0; p < NP; ++p) col_on[p] = (p * 64 + lane) * EPV < dim;

  float acc[NP][EPV];
#pragma unroll
  for (int p = 0; p < NP; ++p)
#pragma unroll
    for (int c = 0; c < EPV; ++c) acc[p][c] = 0.0f;

  auto next_row = [&]() {
    ++r;
    if (r - r_base == 64) {
      r_base = r;
      rel = load_rel(r_base);
    }
    cur_end = __builtin_amdgcn_readlane(rel, r - r_base);
  };
  // a finished row: Y gets the sum (if wanted), Y2 its positive part (if wanted)
  auto store_y = [&](int row) {
    if (Y) {
      T* py = Y + static_cast<int64_t>(row) * ldy;
#pragma unroll
      for (int p = 0; p < NP; ++p)
        if (col_on[p]) VecIO<T, EPV>::store(py + (p * 64 + lane) * EPV, acc[p]);
    }
    if (Y2) {
      T* py = Y2 + static_cast<int64_t>(row) * ldy;
#pragma unroll
      for (int p = 0; p < NP; ++p)
        if (col_on[p]) {
          float pos[EPV];
#pragma unroll
          for (int c = 0; c < EPV; ++c) pos[c] = acc[p][c] > 0.0f ? acc[p][c] : 0.0f;
          VecIO<T, EPV>::store(py + (p * 64 + lane) * EPV, pos);
        }
    }
    if constexpr (XF) {
      // the finished row goes to this wavefront's LDS buffer, then every lane < G forms one output
      float* rb = xf_lds + xf_row_floats(dim * xf.G) + wave * xf_row_floats(dim);
#pragma unroll
      for (int p = 0; p < NP; ++p)
        if (col_on[p]) {
#pragma unroll
          for (int c = 0; c < EPV; ++c) rb[(p * 64 + lane) * EPV + c] = acc[p][c];
        }
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
      transform_row(rb, xf_lds, dim, xf, row, lane);
      __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");   // the next row is written only after every lane has read this one
    }
  };
  auto store_partial = [&](float* buf) {
    float* pp = buf + chunk * static_cast<int64_t>(dim);
#pragma unroll
    for (int p = 0; p < NP; ++p)
      if (col_on[p]) {
#pragma unroll
        for (int c = 0; c < EPV; ++c) pp[(p * 64 + lane) * EPV + c] = acc[p][c];
      }
  };
  auto clear_acc = [&]() {
#pragma unroll
    for (int p = 0; p < NP; ++p)
#pragma unroll
      for (int c = 0; c < EPV; ++c) acc[p][c] = 0.0f;
  };
  // the row that just ended inside this chunk
  auto flush_row = [&]() {
    if (head) store_partial(phead);
    else store_y(r);
    head = false;
    clear_acc();
  };

  // one entry: gather is already in x, add it to the open row (closing rows that ended before it)
  auto consume = [&](const float (&xr)[NP][EPV], int j) {
    while (krel == cur_end) {
      flush_row();
      next_row();
    }
    const float v = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(my_val), j));
#pragma unroll
    for (int p = 0; p < NP; ++p)
      if (col_on[p]) {
#pragma unroll
        for (int c = 0; c < EPV; ++c) acc[p][c] = __fmaf_rn(v, xr[p][c], acc[p][c]);
      }
    ++krel;
  };
  auto gather = [&](float (&xr)[NP][EPV], int j) {
    const int c = __builtin_amdgcn_readlane(my_col, j);
    const T* px = X + static_cast<int64_t>(c) * ldx;
#pragma unroll
    for (int p = 0; p < NP; ++p)
      if (col_on[p]) VecIO<T, EPV>::load(px + (p * 64 + lane) * EPV, xr[p]);
  };

  for (int base = 0; base < L; base += 64) {
    const int cnt = L - base < 64 ? L - base : 64;
    my_col = 0;
    my_val = 0.0f;
    if (lane < cnt) {
      my_col = colidx[s + base + lane];
      my_val = vals[s + base + lane];
    }
    int j = 0;
    for (; j + U <= cnt; j += U) {  // U gathers in flight, no guards
      float x[U][NP][EPV];
#pragma unroll
      for (int u = 0; u < U; ++u) gather(x[u], j + u);
#pragma unroll
      for (int u = 0; u < U; ++u) consume(x[u], j + u);
    }
    for (; j < cnt; ++j) {
      float x[NP][EPV];
      gather(x, j);
      consume(x, j);
    }
  }

  // end of the chunk (krel == L): the open row either ends here or runs on
  int tr = -1;
  if (cur_end > L) {
    if (head) {
      store_partial(phead);  // the whole chunk lies inside one row
    } else {
      store_partial(ptail);
      tr = r;
    }
  } else {
    flush_row();
    next_row();
    // empty rows between this chunk's last entry and the next chunk's first
    while (r < n_rows && cur_end == L) {
      store_y(r);  // acc is zero
      next_row();
    }
  }
  if (lane == 0) tail_row[chunk] = tr;
}

// Column-sliced variant for rows that are several cache lines wide. The feature matrix is
// processed in vertical slices of SW = LPR * EPV elements (grid.y = slice); within a slice a
// gather instruction serves 64 / LPR stored entries at once, LPR lanes each. Narrow slices shrink
// the table the gathers hit by dim / SW, so far more of its rows stay in the 4 MB L2 of an XCD
// and in the memory-side cache; the CSR arrays are re-read once per slice (8 bytes per entry
// against SW * 4 of features). Entries of a row are spread round-robin over the lane groups and
// the groups' partial sums are combined when the row ends - a fixed order, no atomics.
template <typename T, int EPV, int LPR, int UREQ>
__global__ __launch_bounds__(kSpmmThreads) void spmm_sliced_kernel(
    const int64_t* __restrict__ rowptr, const int* __restrict__ colidx, const float* __restrict__ vals,
    int n_rows, int64_t nnz, const T* __restrict__ X, int64_t ldx, T* __restrict__ Y, T* __restrict__ Y2,
    int64_t ldy, int dim, const int* __restrict__ chunk_row, int64_t nchunks, float* __restrict__ phead,
    float* __restrict__ ptail, int* __restrict__ tail_row, int kChunk) {
  constexpr int EPI = 64 / LPR;  // stored entries per gather instruction
  constexpr int SW = LPR * EPV;  // slice width in elements
  constexpr int U = UREQ * EPI > 64 ? 64 / EPI : UREQ;  // gather instructions in flight (a window holds 64 entries)
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int64_t chunk = static_cast<int64_t>(blockIdx.x) * kSpmmWaves + wave;
  if (chunk >= nchunks) return;
  const int g = lane / LPR, lg = lane % LPR;
  const int col0 = blockIdx.y * SW + lg * EPV;  // this lane's columns: [col0, col0 + EPV)
  const bool lane_on = col0 < dim;              // false on the lanes past the row end in a partial last slice
  const int64_t s = chunk * kChunk;
  const int L = static_cast<int>(nnz - s < kChunk ? nnz - s : kChunk);
  int my_col = 0, krel = 0;
  float my_val = 0.0f;

  int r = chunk == 0 ? 0 : chunk_row[chunk];
  bool head = chunk > 0 && rowptr[r] < s;
  auto load_rel = [&](int rbase) -> int {
    const int rr = rbase + lane;
    if (rr < n_rows) {
      const int64_t d = rowptr[rr + 1] - s;
      return d > kChunk ? kChunk + 1 : static_cast<int>(d);
    }
    return kChunk + 2;
  };
  int r_base = r;
  int rel = load_rel(r_base);
  int cur_end = __builtin_amdgcn_readlane(rel, 0);
  auto next_row = [&]() {
    ++r;
    if (r - r_base == 64) {
      r_base = r;
      rel = load_rel(r_base);
    }
    cur_end = __builtin_amdgcn_readlane(rel, r - r_base);
  };

  float acc[EPV];
#pragma unroll
  for (int c = 0; c < EPV; ++c) acc[c] = 0.0f;

  // Combine the lane groups' sums with a halving exchange: at stride 32, 16, ..., LPR each lane
  // passes one half of its components to its partner and adds the partner's other half, so the
  // row slice ends up spread over the lanes (FIN components each, starting at component cbase)
  // with a quarter of the shuffles of a full butterfly. Once a lane is down to one component the
  // remaining strides are plain sums and only the lanes with the stride bit clear keep the result.
  constexpr int FIN = EPV / EPI > 0 ? EPV / EPI : 1;
  int cbase = 0;       // first component (within this lane's EPV) that the lane owns after the exchange
  bool owner = true;   // false on lanes that hold a duplicate
  {
    int cnt = EPV;
#pragma unroll
    for (int off = 32; off >= LPR; off >>= 1) {
      const bool up = (lane & off) != 0;
      if (cnt > 1) {
        cnt >>= 1;
        if (up) cbase += cnt;
      } else if (up) {
        owner = false;
      }
    }
  }
  auto reduce_groups = [&](float (&fin)[FIN]) {
    float a[EPV];
#pragma unroll
    for (int c = 0; c < EPV; ++c) a[c] = acc[c];
    int cnt = EPV;
#pragma unroll
    for (int off = 32; off >= LPR; off >>= 1) {
      const bool up = (lane & off) != 0;
      if (cnt > 1) {
        const int half = cnt >> 1;
#pragma unroll
        for (int i = 0; i < EPV / 2; ++i) {
          if (i < half) {
            const float send = up ? a[i] : a[half + i];
            const float keep = up ? a[half + i] : a[i];
            a[i] = keep + __shfl_xor(send, off, kWave);
          }
        }
        cnt = half;
      } else {
        a[0] = a[0] + __shfl_xor(a[0], off, kWave);
      }
    }
#pragma unroll
    for (int c = 0; c < FIN; ++c) fin[c] = a[c];
  };
  auto store_y = [&](int row, const float (&fin)[FIN]) {
    if (!owner || !lane_on) return;
    const int64_t at = static_cast<int64_t>(row) * ldy + col0 + cbase;
    if (Y) VecIO<T, FIN>::store(Y + at, fin);
    if (Y2) {
      float pos[FIN];
#pragma unroll
      for (int c = 0; c < FIN; ++c) pos[c] = fin[c] > 0.0f ? fin[c] : 0.0f;
      VecIO<T, FIN>::store(Y2 + at, pos);
    }
  };
  auto store_partial = [&](float* buf, const float (&fin)[FIN]) {
    if (!owner || !lane_on) return;
    float* pp = buf + chunk * static_cast<int64_t>(dim) + col0 + cbase;
#pragma unroll
    for (int c = 0; c < FIN; ++c) pp[c] = fin[c];
  };
  auto flush_row = [&]() {
    float fin[FIN];
    reduce_groups(fin);
    if (head) store_partial(phead, fin);
    else store_y(r, fin);
    head = false;
#pragma unroll
    for (int c = 0; c < EPV; ++c) acc[c] = 0.0f;
  };

  const T* xs = X + col0;
  for (int base = 0; base < L; base += 64) {
    const int cnt = L - base < 64 ? L - base : 64;
    my_col = 0;
    my_val = 0.0f;
    if (lane < cnt) {
      my_col = colidx[s + base + lane];
      my_val = vals[s + base + lane];
    }
    for (int j = 0; j < cnt; j += EPI * U) {
      float x[U][EPV];
      float v[U];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int e = j + u * EPI + g;  // this group's entry of instruction u
        const int c = __shfl(my_col, e, kWave);
        v[u] = __shfl(my_val, e, kWave);
#pragma unroll
        for (int q = 0; q < EPV; ++q) x[u][q] = 0.0f;
        if (e < cnt && lane_on) VecIO<T, EPV>::load(xs + static_cast<int64_t>(c) * ldx, x[u]);
      }
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int first = j + u * EPI;
        if (first < cnt) {
          const int avail = cnt - first < EPI ? cnt - first : EPI;
          int done = 0;
          while (done < avail) {
            while (krel == cur_end) {
              flush_row();
              next_row();
            }
            const int room = cur_end - krel;
            const int take = avail - done < room ? avail - done : room;
            if (g >= done && g < done + take) {
#pragma unroll
              for (int q = 0; q < EPV; ++q) acc[q] = __fmaf_rn(v[u], x[u][q], acc[q]);
            }
            done += take;
            krel += take;
          }
        }
      }
    }
  }

  int tr = -1;
  if (cur_end > L) {
    float fin[FIN];
    reduce_groups(fin);
    if (head) {
      store_partial(phead, fin);
    } else {
      store_partial(ptail, fin);
      tr = r;
    }
  } else {
    flush_row();
    next_row();
    float zero[FIN];
#pragma unroll
    for (int c = 0; c < FIN; ++c) zero[c] = 0.0f;
    while (r < n_rows && cur_end == L) {
      store_y(r, zero);
      next_row();
    }
  }
  if (lane == 0 && blockIdx.y == 0) tail_row[chunk] = tr;
}

// Adds the pieces of every row that straddles chunk borders, in chunk order.
template <typename T, int EPV>
__global__ __launch_bounds__(kSpmmThreads) void spmm_fixup_kernel(
    const int64_t* __restrict__ rowptr, const int* __restrict__ tail_row, int64_t nchunks,
    const float* __restrict__ phead, const float* __restrict__ ptail, T* __restrict__ Y, T* __restrict__ Y2,
    int64_t ldy, int dim, int n_rows, int kChunk) {
  const int lane = threadIdx.x & 63;
  const int64_t chunk = static_cast<int64_t>(blockIdx.x) * kSpmmWaves + (threadIdx.x >> 6);
  if (chunk >= nchunks) return;
  const int r = tail_row[chunk];
  if (r < 0 || r >= n_rows) return;
  // last chunk that starts inside row r: the one that holds the row's last entry (the row runs past
  // this chunk, so it has one). Computed, not walked: the longest rows span hundreds of chunks.
  const int64_t last = (rowptr[r + 1] - 1) / kChunk;
  for (int col = lane * EPV; col < dim; col += 64 * EPV) {
    float acc[EPV];
#pragma unroll
    for (int c = 0; c < EPV; ++c) acc[c] = ptail[chunk * static_cast<int64_t>(dim) + col + c];
    int64_t c2 = chunk + 1;
    for (; c2 + 3 <= last; c2 += 4) {
      float t[4][EPV];
#pragma unroll
      for (int q = 0; q < 4; ++q)
#pragma unroll
        for (int c = 0; c < EPV; ++c) t[q][c] = phead[(c2 + q) * static_cast<int64_t>(dim) + col + c];
#pragma unroll
      for (int q = 0; q < 4; ++q)
#pragma unroll
        for (int c = 0; c < EPV; ++c) acc[c] = acc[c] + t[q][c];
    }
    for (; c2 <= last; ++c2)
#pragma unroll
      for (int c = 0; c < EPV; ++c) acc[c] = acc[c] + phead[c2 * static_cast<int64_t>(dim) + col + c];
    if (Y) VecIO<T, EPV>::store(Y + static_cast<int64_t>(r) * ldy + col, acc);
    if (Y2) {
#pragma unroll
      for (int c = 0; c < EPV; ++c) acc[c] = acc[c] > 0.0f ? acc[c] : 0.0f;
      VecIO<T, EPV>::store(Y2 + static_cast<int64_t>(r) * ldy + col, acc);
    }
  }
}

// Entries per wavefront: 64 or 128 on small matrices (so that even a few thousand entries spread over
// all compute units and a wavefront's serial walk stays short), 256 from 1 M entries, up to 1024 for
// large ones (fewer straddling-row pieces). Always a multiple of 64; a function of nnz alone.
static int pick_chunk(int64_t nnz) {
  int c = 64;
  while (c < kChunk && nnz / (2 * c) >= 4096) c *= 2;
  while (c >= kChunk && c < 1024 && nnz / (2 * c) >= 65536) c *= 2;
  return c;
}

// The same for the transforming variant (fp32): the summed row is stored and then transformed (W from
// global memory: only rows that straddle chunk borders come here).
template <int EPV>
__global__ __launch_bounds__(kSpmmThreads) void spmm_fixup_transform_kernel(
    const int64_t* __restrict__ rowptr, const int* __restrict__ tail_row, int64_t nchunks,
    const float* __restrict__ phead, const float* __restrict__ ptail, float* __restrict__ Y, int64_t ldy, int dim,
    int n_rows, int kChunk, XformArgs xf) {
  extern __shared__ __align__(16) float xf_lds[];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int64_t chunk = static_cast<int64_t>(blockIdx.x) * kSpmmWaves + wave;
  if (chunk >= nchunks) return;
  const int r = tail_row[chunk];
  if (r < 0 || r >= n_rows) return;
  const int64_t last = (rowptr[r + 1] - 1) / kChunk;
  float* rb = xf_lds + wave * xf_row_floats(dim);
  for (int col = lane * EPV; col < dim; col += 64 * EPV) {
    float acc[EPV];
#pragma unroll
    for (int c = 0; c < EPV; ++c) acc[c] = ptail[chunk * static_cast<int64_t>(dim) + col + c];
    for (int64_t c2 = chunk + 1; c2 <= last; ++c2)
#pragma unroll
      for (int c = 0; c < EPV; ++c) acc[c] = acc[c] + phead[c2 * static_cast<int64_t>(dim) + col + c];
    if (Y) VecIO<float, EPV>::store(Y + static_cast<int64_t>(r) * ldy + col, acc);
#pragma unroll
    for (int c = 0; c < EPV; ++c) rb[col + c] = acc[c];
  }
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
  transform_row(rb, xf.W, dim, xf, r, lane);
}

int64_t spmm_chunks(int64_t nnz) { return nnz <= 0 ? 1 : ceil_div(nnz, pick_chunk(nnz)); }

// Upper bound of spmm_chunks over every matrix of at most nnz entries (the chunk size steps up with nnz,
// so the count itself is not monotone).
static int64_t spmm_chunks_bound(int64_t nnz) {
  if (nnz <= 0) return 1;
  const int64_t small = ceil_div(nnz, 64) < 8192 ? ceil_div(nnz, 64) : 8192;
  const int64_t large = ceil_div(nnz, kChunk);
  return small > large ? small : large;
}

size_t spmm_workspace_bytes(int64_t nnz, int32_t dim) {
  const int64_t nc = spmm_chunks_bound(nnz);
  return align_up(static_cast<size_t>(nc) * 2 * sizeof(int), 256) +
         2 * align_up(static_cast<size_t>(nc) * dim * sizeof(float), 256);
}

template <typename T, int EPV>
static int launch_spmm(const cdf_csr* A, const T* X, int64_t ldx, T* Y, T* Y2, int64_t ldy, int dim, void* ws,
                       hipStream_t st) {
  const int chunk = pick_chunk(A->nnz);
  const int64_t nc = spmm_chunks(A->nnz);
  char* w = static_cast<char*>(ws);
  int* own_chunk_row = reinterpret_cast<int*>(w);
  int* tail_row = own_chunk_row + nc;
  w += align_up(static_cast<size_t>(nc) * 2 * sizeof(int), 256);
  float* phead = reinterpret_cast<float*>(w);
  w += align_up(static_cast<size_t>(nc) * dim * sizeof(float), 256);
  float* ptail = reinterpret_cast<float*>(w);

  // chunk -> row table: the caller's plan (built once per matrix by cdf_spmm_plan), else rebuilt here
  const int* chunk_row = A->plan;
  if (!chunk_row) {
    {
      ProfScope ps(K_SPMM_PLAN, st);
      chunk_rows_kernel<<<static_cast<unsigned>(ceil_div(A->n_rows, 256)), 256, 0, st>>>(A->rowptr, A->n_rows,
                                                                                         own_chunk_row, chunk);
    }
    CDF_LAUNCH_CHECK("cdf_spmm/chunk_rows");
    chunk_row = own_chunk_row;
  }
  const unsigned nblocks = static_cast<unsigned>(ceil_div(nc, kSpmmWaves));
  const int per_pass = 64 * EPV;
  const int np = static_cast<int>(ceil_div(dim, per_pass));
  const int nvec = dim / EPV;
  constexpr bool lane16 = EPV * static_cast<int>(sizeof(T)) == 16;   // 16-byte lane vectors
#define CDF_SPMM_ARGS                                                                                      \
  (A->rowptr, A->colidx, A->vals, A->n_rows, A->nnz, X, ldx, Y, Y2, ldy, dim, chunk_row, nc, phead, ptail, \
   tail_row, chunk)
#define CDF_SPMM_ARGS_X                                                                                    \
  (A->rowptr, A->colidx, A->vals, A->n_rows, A->nnz, X, ldx, Y, Y2, ldy, dim, chunk_row, nc, phead, ptail, \
   tail_row, chunk, XformArgs{})
  // Lanes per entry. Rows of whole 128-byte lines with eight or more entries on average: one line per
  // row and slice (8 lanes of 16 bytes); it pays when the per-row, per-slice reduction and store are
  // amortised. Rows of at most 32 lane-vectors: one slice, the lane group just wide enough for the row.
  // Everything else: the whole wavefront per entry.
  constexpr int min_avg = 8;
  int lpr = 0, slices = 1;
  if (lane16 && dim % (8 * EPV) == 0 && A->nnz >= static_cast<int64_t>(min_avg) * A->n_rows) {
    lpr = 8;
    slices = dim / (8 * EPV);
  } else if (lane16 && nvec <= 32) {
    lpr = 2;
    while (lpr < nvec) lpr <<= 1;
  }
  if (lpr > 0) {
    if constexpr (lane16) {
      const dim3 grid(nblocks, static_cast<unsigned>(slices));
      prof_begin(K_SPMM_SLICED, st);
      // gather instructions in flight per wavefront: long rows (the forward matrix of a power-law
      // partition averages ~70 entries) run 2-3 % faster with eight, short rows (its transpose, ~20)
      // with four - measured both ways
      const bool deep = A->nnz >= static_cast<int64_t>(40) * A->n_rows;
      switch (lpr) {
        case 2: spmm_sliced_kernel<T, EPV, 2, 4><<<grid, kSpmmThreads, 0, st>>> CDF_SPMM_ARGS; break;
        case 4: spmm_sliced_kernel<T, EPV, 4, 4><<<grid, kSpmmThreads, 0, st>>> CDF_SPMM_ARGS; break;
        case 8:
          if (deep) spmm_sliced_kernel<T, EPV, 8, 8><<<grid, kSpmmThreads, 0, st>>> CDF_SPMM_ARGS;
          else spmm_sliced_kernel<T, EPV, 8, 4><<<grid, kSpmmThreads, 0, st>>> CDF_SPMM_ARGS;
          break;
        case 16: spmm_sliced_kernel<T, EPV, 16, 4><<<grid, kSpmmThreads, 0, st>>> CDF_SPMM_ARGS; break;
        default: spmm_sliced_kernel<T, EPV, 32, 4><<<grid, kSpmmThreads, 0, st>>> CDF_SPMM_ARGS; break;
      }
      prof_end(K_SPMM_SLICED, st);
      CDF_LAUNCH_CHECK("cdf_spmm/sliced");
    }
  } else {
    prof_begin(K_SPMM, st);
    if (np <= 1) spmm_kernel<T, EPV, 1><<<nblocks, kSpmmThreads, 0, st>>> CDF_SPMM_ARGS_X;
    else if (np <= 2) spmm_kernel<T, EPV, 2><<<nblocks, kSpmmThreads, 0, st>>> CDF_SPMM_ARGS_X;
    else if (np <= 4) spmm_kernel<T, EPV, 4><<<nblocks, kSpmmThreads, 0, st>>> CDF_SPMM_ARGS_X;
    else spmm_kernel<T, EPV, 8><<<nblocks, kSpmmThreads, 0, st>>> CDF_SPMM_ARGS_X;
    prof_end(K_SPMM, st);
    CDF_LAUNCH_CHECK("cdf_spmm/main");
  }
#undef CDF_SPMM_ARGS
#undef CDF_SPMM_ARGS_X
  {
    ProfScope ps(K_SPMM_FIXUP, st);
    spmm_fixup_kernel<T, EPV><<<nblocks, kSpmmThreads, 0, st>>>(A->rowptr, tail_row, nc, phead, ptail, Y, Y2, ldy, dim,
                                                                 A->n_rows, chunk);
  }
  CDF_LAUNCH_CHECK("cdf_spmm/fixup");
  return CDF_OK;
}

// Y = A X and/or Y2 = max(A X, 0); either output may be null, both share ldy.
int spmm_run(const char* fn, const cdf_csr* A, const void* X, int64_t ldx, void* Y, void* Y2, int64_t ldy,
             int32_t dim, cdf_dtype dt, void* ws, size_t ws_bytes, hipStream_t st) {
  CDF_REQUIRE(A != nullptr, "%s: matrix is null", fn);
  CDF_REQUIRE(A->n_rows >= 0 && A->n_cols >= 0 && A->nnz >= 0 && dim > 0 && ldx >= dim && ldy >= dim,
              "%s: bad shape rows=%d cols=%d nnz=%lld dim=%d ldx=%lld ldy=%lld", fn, A->n_rows, A->n_cols,
              (long long)A->nnz, dim, (long long)ldx, (long long)ldy);
  if (dt != CDF_F32 && dt != CDF_BF16) CDF_FAIL(CDF_ERR_UNSUPPORTED, "%s: dtype %d", fn, (int)dt);
  if (A->n_rows == 0) return CDF_OK;
  CDF_REQUIRE(A->rowptr && (Y || Y2) && (A->nnz == 0 || (A->colidx && A->vals && X)), "%s: null pointer", fn);
  const size_t esz = elem_bytes(dt);
  CDF_REQUIRE(aligned(A->rowptr, 8) && aligned(A->colidx, 4) && aligned(A->vals, 4) && aligned(X, esz) &&
                  aligned(Y, esz) && aligned(Y2, esz),
              "%s: misaligned pointer", fn);
  if (!ws || !aligned(ws, 256) || ws_bytes < spmm_workspace_bytes(A->nnz, dim))
    CDF_FAIL(CDF_ERR_WORKSPACE, "%s: workspace too small or unaligned (%zu < %zu)", fn, ws_bytes,
             spmm_workspace_bytes(A->nnz, dim));
  // widest lane-vector that both operands allow; at most 8 passes of 64 lanes per launch
  int epv = dt == CDF_BF16 ? 8 : 4;
  for (; epv > 1; epv >>= 1) {
    const size_t vb = esz * epv;
    if (dim % epv == 0 && ldx % epv == 0 && ldy % epv == 0 && aligned(X, vb) && aligned(Y, vb) && aligned(Y2, vb)) break;
  }
  const int max_cols = 64 * epv * 8;
  for (int col0 = 0; col0 < dim; col0 += max_cols) {
    const int d = dim - col0 < max_cols ? dim - col0 : max_cols;
    int rc;
    if (dt == CDF_F32) {
      const float* x = static_cast<const float*>(X) + col0;
      float* y = Y ? static_cast<float*>(Y) + col0 : nullptr;
      float* y2 = Y2 ? static_cast<float*>(Y2) + col0 : nullptr;
      rc = epv == 4 ? launch_spmm<float, 4>(A, x, ldx, y, y2, ldy, d, ws, st)
           : epv == 2 ? launch_spmm<float, 2>(A, x, ldx, y, y2, ldy, d, ws, st)
                      : launch_spmm<float, 1>(A, x, ldx, y, y2, ldy, d, ws, st);
    } else {
      const bf16_t* x = static_cast<const bf16_t*>(X) + col0;
      bf16_t* y = Y ? static_cast<bf16_t*>(Y) + col0 : nullptr;
      bf16_t* y2 = Y2 ? static_cast<bf16_t*>(Y2) + col0 : nullptr;
      rc = epv == 8   ? launch_spmm<bf16_t, 8>(A, x, ldx, y, y2, ldy, d, ws, st)
           : epv == 4 ? launch_spmm<bf16_t, 4>(A, x, ldx, y, y2, ldy, d, ws, st)
           : epv == 2 ? launch_spmm<bf16_t, 2>(A, x, ldx, y, y2, ldy, d, ws, st)
                      : launch_spmm<bf16_t, 1>(A, x, ldx, y, y2, ldy, d, ws, st);
    }
    if (rc != CDF_OK) return rc;
  }
  return CDF_OK;
}

int dense_fwd_ws(const void* M, int64_t ldm, cdf_dtype dt, const float* W, int32_t n, int32_t f_in, int32_t f_out,
                 int relu, float* Z, float* H, void* ws, size_t ws_bytes, void* stream);

// Can the aggregation carry the dense transform in its row epilogue? fp32 rows read as 16-byte lane
// vectors, at most 64 output columns, W and four row buffers within 64 KB of LDS.
bool spmm_transform_ok(const void* X, int64_t ldx, const void* M, int64_t ldm, int32_t dim, int32_t g, cdf_dtype dt) {
  if (dt != CDF_F32 || dim % 4 != 0 || ldx % 4 != 0 || ldm % 4 != 0 || !aligned(X, 16) || !aligned(M, 16)) return false;
  if (g < 1 || g > 64 || dim > 1024) return false;
  const size_t lds = (static_cast<size_t>(xf_row_floats(dim * g)) + kSpmmWaves * xf_row_floats(dim)) * sizeof(float);
  return lds <= 65536;
}

// M = A X, Z = M W, H = sigma(Z) in one pass over the matrix (plus the fix-up of straddling rows).
int spmm_transform_run(const char* fn, const cdf_csr* A, const float* X, int64_t ldx, const float* W, int32_t dim,
                       int32_t g, int relu, float* M, int64_t ldm, float* Z, float* H, void* ws, size_t ws_bytes,
                       hipStream_t st) {
  CDF_REQUIRE(A != nullptr && A->n_rows >= 0 && A->nnz >= 0, "%s: bad matrix", fn);
  if (A->n_rows == 0) return CDF_OK;
  CDF_REQUIRE(A->rowptr && M && W && (Z || H) && (A->nnz == 0 || (A->colidx && A->vals && X)), "%s: null pointer", fn);
  CDF_REQUIRE(aligned(A->rowptr, 8) && aligned(W, 4) && aligned(Z, 4) && aligned(H, 4), "%s: misaligned pointer", fn);
  if (!ws || !aligned(ws, 256) || ws_bytes < spmm_workspace_bytes(A->nnz, dim))
    CDF_FAIL(CDF_ERR_WORKSPACE, "%s: workspace too small or unaligned (%zu < %zu)", fn, ws_bytes,
             spmm_workspace_bytes(A->nnz, dim));
  const int chunk = pick_chunk(A->nnz);
  const int64_t nc = spmm_chunks(A->nnz);
  char* w = static_cast<char*>(ws);
  int* own_chunk_row = reinterpret_cast<int*>(w);
  int* tail_row = own_chunk_row + nc;
  w += align_up(static_cast<size_t>(nc) * 2 * sizeof(int), 256);
  float* phead = reinterpret_cast<float*>(w);
  w += align_up(static_cast<size_t>(nc) * dim * sizeof(float), 256);
  float* ptail = reinterpret_cast<float*>(w);
  const int* chunk_row = A->plan;
  if (!chunk_row) {
    {
      ProfScope ps(K_SPMM_PLAN, st);
      chunk_rows_kernel<<<static_cast<unsigned>(ceil_div(A->n_rows, 256)), 256, 0, st>>>(A->rowptr, A->n_rows,
                                                                                         own_chunk_row, chunk);
    }
    CDF_LAUNCH_CHECK("spmm + transform/chunk_rows");
    chunk_row = own_chunk_row;
  }
  const unsigned nblocks = static_cast<unsigned>(ceil_div(nc, kSpmmWaves));
  const XformArgs xf = {W, Z, H, g, relu ? 1 : 0};
  const size_t lds_main = (static_cast<size_t>(xf_row_floats(dim * g)) + kSpmmWaves * xf_row_floats(dim)) * sizeof(float);
  const size_t lds_fix = static_cast<size_t>(kSpmmWaves) * xf_row_floats(dim) * sizeof(float);
  const int np = static_cast<int>(ceil_div(dim, 256));
  float* none = nullptr;
#define CDF_XF_ARGS                                                                                              \
  (A->rowptr, A->colidx, A->vals, A->n_rows, A->nnz, X, ldx, M, none, ldm, dim, chunk_row, nc, phead, ptail, tail_row, \
   chunk, xf)
  prof_begin(K_SPMM_XFORM, st);
  if (np <= 1) spmm_kernel<float, 4, 1, true><<<nblocks, kSpmmThreads, lds_main, st>>> CDF_XF_ARGS;
  else if (np <= 2) spmm_kernel<float, 4, 2, true><<<nblocks, kSpmmThreads, lds_main, st>>> CDF_XF_ARGS;
  else spmm_kernel<float, 4, 4, true><<<nblocks, kSpmmThreads, lds_main, st>>> CDF_XF_ARGS;
  prof_end(K_SPMM_XFORM, st);
#undef CDF_XF_ARGS
  CDF_LAUNCH_CHECK("spmm + transform/main");
  {
    ProfScope ps(K_SPMM_FIXUP, st);
    spmm_fixup_transform_kernel<4><<<nblocks, kSpmmThreads, lds_fix, st>>>(A->rowptr, tail_row, nc, phead, ptail, M, ldm,
                                                                           dim, A->n_rows, chunk, xf);
  }
  CDF_LAUNCH_CHECK("spmm + transform/fixup");
  return CDF_OK;
}

}  // namespace cdf

using namespace cdf;

extern "C" int cdf_spmm_dense_fwd(const cdf_csr* A, const void* X, int64_t ldx, cdf_dtype dt, const float* W,
                                  int32_t f_in, int32_t f_out, int relu, void* M, int64_t ldm, float* Z, float* H,
                                  void* ws, size_t ws_bytes, void* stream) {
  hipStream_t st = static_cast<hipStream_t>(stream);
  CDF_REQUIRE(A != nullptr && f_in > 0 && f_out > 0 && ldx >= f_in && ldm >= f_in,
              "cdf_spmm_dense_fwd: bad shape f_in=%d f_out=%d ldx=%lld ldm=%lld", f_in, f_out, (long long)ldx,
              (long long)ldm);
  if (spmm_transform_ok(X, ldx, M, ldm, f_in, f_out, dt))
    return spmm_transform_run("cdf_spmm_dense_fwd", A, static_cast<const float*>(X), ldx, W, f_in, f_out, relu,
                              static_cast<float*>(M), ldm, Z, H, ws, ws_bytes, st);
  const int rc = spmm_run("cdf_spmm_dense_fwd", A, X, ldx, M, nullptr, ldm, f_in, dt, ws, ws_bytes, st);
  if (rc != CDF_OK) return rc;
  return dense_fwd_ws(M, ldm, dt, W, A->n_rows, f_in, f_out, relu, Z, H, ws, ws_bytes, stream);
}

extern "C" int cdf_spmm_fwd(const cdf_csr* A, const void* X, int64_t ldx, void* Y, int64_t ldy, int32_t dim,
                            cdf_dtype dt, void* ws, size_t ws_bytes, void* stream) {
  return spmm_run("cdf_spmm_fwd", A, X, ldx, Y, nullptr, ldy, dim, dt, ws, ws_bytes, static_cast<hipStream_t>(stream));
}

extern "C" int cdf_spmm_bwd(const cdf_csr* At, const void* dY, int64_t ldy, void* dX, int64_t ldx, int32_t dim,
                            cdf_dtype dt, void* ws, size_t ws_bytes, void* stream) {
  return spmm_run("cdf_spmm_bwd", At, dY, ldy, dX, nullptr, ldx, dim, dt, ws, ws_bytes, static_cast<hipStream_t>(stream));
}

extern "C" size_t cdf_spmm_plan_bytes(int64_t nnz) {
  return nnz < 0 ? 0 : align_up(static_cast<size_t>(spmm_chunks(nnz)) * sizeof(int), 256);
}

extern "C" int cdf_spmm_plan(const cdf_csr* A, int32_t* plan, size_t plan_bytes, void* stream) {
  CDF_REQUIRE(A != nullptr, "cdf_spmm_plan: matrix is null");
  CDF_REQUIRE(A->n_rows >= 0 && A->nnz >= 0, "cdf_spmm_plan: bad shape rows=%d nnz=%lld", A->n_rows, (long long)A->nnz);
  if (!plan || !aligned(plan, 4) || plan_bytes < cdf_spmm_plan_bytes(A->nnz))
    CDF_FAIL(CDF_ERR_WORKSPACE, "cdf_spmm_plan: plan buffer too small (%zu < %zu)", plan_bytes,
             cdf_spmm_plan_bytes(A->nnz));
  if (A->n_rows == 0) return CDF_OK;
  CDF_REQUIRE(A->rowptr && aligned(A->rowptr, 8), "cdf_spmm_plan: row pointers null or misaligned");
  hipStream_t st = static_cast<hipStream_t>(stream);
  {
    ProfScope ps(K_SPMM_PLAN, st);
    chunk_rows_kernel<<<static_cast<unsigned>(ceil_div(A->n_rows, 256)), 256, 0, st>>>(A->rowptr, A->n_rows, plan,
                                                                                       pick_chunk(A->nnz));
  }
  CDF_LAUNCH_CHECK("cdf_spmm_plan");
  return CDF_OK;
}
