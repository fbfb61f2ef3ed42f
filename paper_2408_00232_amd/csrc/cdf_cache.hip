// Adaptive cache test (Alg. 2, condition of the mirror loop) and the ordered
// compaction of the rows that fail it.
//
// Three launches, no atomics:
//   1. filter_kernel  - streams cur and cached once, writes mask[r] and one count per
//                       block of kRowsPerBlock rows                     (HBM bound)
//   2. scan_kernel    - one block: exclusive scan of the block counts, total -> n_sent
//   3. compact_kernel - block b ranks its mask bytes and writes idx ascending
// (2 and 3 are one launch, scan_compact_kernel, for inputs of up to 131 072 rows)
//
// Lane mapping. A row is read as vectors of EPV elements (16 bytes for fp32 when
// alignment allows). Rows with at most 64 vectors are handled by groups of
// G = 2^glog lanes, 64/G rows per wavefront at a time; longer rows take the whole
// wavefront and loop. For the L2 norm the fp32 summation order is fixed (256
// interleaved chains, then a radix-2 butterfly over the chain index): element j of a
// row sits in chain j mod 256, and with this mapping chain = c + EPV*lane + 64*EPV*a,
// where c is the component inside the vector and a = iteration mod (4/EPV) selects
// one of 4/EPV accumulators per lane-component. The butterfly then runs over c, the
// lane bits and a, in that order.
#include <mutex>

#include "cdf_common.h"

namespace cdf {

constexpr int kFilterThreads = 256;

template <typename T, int EPV, int NORM>
__global__ __launch_bounds__(kFilterThreads) void filter_kernel(
    const T* __restrict__ cur, const T* __restrict__ cached, int n_rows, int dim, int64_t ld, float eps,
    int glog, uint8_t* __restrict__ mask, int* __restrict__ block_counts) {
  constexpr int NACC = 4 / EPV;  // accumulators per lane-component (L2 chains)
  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const int G = 1 << glog;
  const int lg = lane & (G - 1);
  const int sub = lane >> glog;       // which row of the step this lane works on
  const int rows_per_step = 64 >> glog;
  const int nvec = dim / EPV;
  constexpr int kRowsPerWave = kRowsPerBlock / (kFilterThreads / 64);
  const int row0 = blockIdx.x * kRowsPerBlock + wave * kRowsPerWave;
  int sent_here = 0;

  for (int s = 0; s < kRowsPerWave; s += rows_per_step) {
    const int row = row0 + s + sub;
    const bool live = row < n_rows && s + sub < kRowsPerWave;  // narrow rows: a step may span more rows than the wave owns
    float accd[NACC][EPV], accc[NACC][EPV];
#pragma unroll
    for (int a = 0; a < NACC; ++a)
#pragma unroll
      for (int c = 0; c < EPV; ++c) accd[a][c] = accc[a][c] = 0.0f;
    if (live) {
      const T* pc = cur + static_cast<int64_t>(row) * ld;
      const T* pz = cached + static_cast<int64_t>(row) * ld;
      for (int v0 = lg; v0 < nvec; v0 += G * NACC) {
#pragma unroll
        for (int a = 0; a < NACC; ++a) {
          const int v = v0 + a * G;
          if (v < nvec) {
            float x[EPV], z[EPV];
            VecIO<T, EPV>::load(pc + static_cast<int64_t>(v) * EPV, x);
            VecIO<T, EPV>::load(pz + static_cast<int64_t>(v) * EPV, z);
#pragma unroll
            for (int c = 0; c < EPV; ++c) {
              const float d = x[c] - z[c];
              if (NORM == CDF_NORM_LINF) {
                accd[a][c] = fmaxf(accd[a][c], fabsf(d));
                accc[a][c] = fmaxf(accc[a][c], fabsf(z[c]));
              } else {
                accd[a][c] = __fmaf_rn(d, d, accd[a][c]);
                accc[a][c] = __fmaf_rn(z[c], z[c], accc[a][c]);
              }
            }
          }
        }
      }
    }
    // butterfly: components, lanes, accumulators (ascending chain-index bits)
    float D[NACC], C[NACC];
#pragma unroll
    for (int a = 0; a < NACC; ++a) {
      float d, c;
      if (NORM == CDF_NORM_LINF) {
        d = accd[a][0];
        c = accc[a][0];
#pragma unroll
        for (int k = 1; k < EPV; ++k) {
          d = fmaxf(d, accd[a][k]);
          c = fmaxf(c, accc[a][k]);
        }
        d = group_max(d, G);
        c = group_max(c, G);
      } else {
        if (EPV == 4) {
          d = (accd[a][0] + accd[a][1]) + (accd[a][2 % EPV] + accd[a][3 % EPV]);
          c = (accc[a][0] + accc[a][1]) + (accc[a][2 % EPV] + accc[a][3 % EPV]);
        } else if (EPV == 2) {
          d = accd[a][0] + accd[a][1 % EPV];
          c = accc[a][0] + accc[a][1 % EPV];
        } else {
          d = accd[a][0];
          c = accc[a][0];
        }
        d = group_sum(d, G);
        c = group_sum(c, G);
      }
      D[a] = d;
      C[a] = c;
    }
    float Dr, Cr;
    if (NORM == CDF_NORM_LINF) {
      Dr = D[0];
      Cr = C[0];
#pragma unroll
      for (int a = 1; a < NACC; ++a) {
        Dr = fmaxf(Dr, D[a]);
        Cr = fmaxf(Cr, C[a]);
      }
    } else if (NACC == 4) {
      Dr = (D[0] + D[1 % NACC]) + (D[2 % NACC] + D[3 % NACC]);
      Cr = (C[0] + C[1 % NACC]) + (C[2 % NACC] + C[3 % NACC]);
    } else if (NACC == 2) {
      Dr = D[0] + D[1 % NACC];
      Cr = C[0] + C[1 % NACC];
    } else {
      Dr = D[0];
      Cr = C[0];
    }
    bool send;
    if (NORM == CDF_NORM_LINF) {
      const float thr = eps * Cr;
      send = Dr > thr;
    } else {
      const float e2 = eps * eps;
      const float thr = e2 * Cr;
      send = Dr > thr;
    }
    const bool head = live && lg == 0;
    if (head) mask[row] = send ? 1 : 0;
    sent_here += __popcll(__ballot(head && send));
  }

  __shared__ int wave_cnt[kFilterThreads / 64];
  if (lane == 0) wave_cnt[wave] = sent_here;
  __syncthreads();
  if (threadIdx.x == 0) {
    int t = 0;
    for (int w = 0; w < kFilterThreads / 64; ++w) t += wave_cnt[w];
    block_counts[blockIdx.x] = t;
  }
}

// Exclusive scan of n counts by one block; offsets[i] = sum of counts[0..i), *total = sum.
// Every thread takes kScanPer consecutive counts per pass, so a pass covers 1024 * kScanPer of them.
// Whole passes read and write 16-byte vectors without guards, and the counts of the next pass are
// requested two passes ahead (straight-line code, so the wait before the sums leaves the later
// requests in flight); the ragged last pass goes element by element.
constexpr int kScanPer = 8;
constexpr int kScanPass = 1024 * kScanPer;

// One pass: v = this thread's counts; returns their exclusive start within the pass and adds the
// pass total to carry. ws alternates between two buffers, so one barrier per pass is enough.
__device__ __forceinline__ int scan_pass(const int (&v)[kScanPer], int (&ws)[16], int& carry) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  int mine = 0;
#pragma unroll
  for (int j = 0; j < kScanPer; ++j) mine += v[j];
  int incl = mine;
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    const int t = __shfl_up(incl, off, kWave);
    if (lane >= off) incl += t;
  }
  if (lane == 63) ws[wave] = incl;
  __syncthreads();
  int wbase = 0, all = 0;
#pragma unroll
  for (int w = 0; w < 16; ++w) {
    const int t = ws[w];
    if (w < wave) wbase += t;
    all += t;
  }
  const int start = carry + wbase + incl - mine;
  carry += all;
  return start;
}

__global__ __launch_bounds__(1024) void scan_kernel(const int* __restrict__ counts, int n,
                                                    int* __restrict__ offsets, int* __restrict__ total) {
  __shared__ int wsum[2][16];
  int carry = 0;  // sum of all earlier passes, the same in every thread
  int pass = 0, base = 0;
  const bool vec = ((reinterpret_cast<uintptr_t>(counts) | reinterpret_cast<uintptr_t>(offsets)) & 15) == 0;
  if (vec && n >= kScanPass) {
    const int4* src = reinterpret_cast<const int4*>(counts) + threadIdx.x * (kScanPer / 4);
    int4* dst = reinterpret_cast<int4*>(offsets) + threadIdx.x * (kScanPer / 4);
    // Three register sets take turns (this pass, the next, the one after); the loop is unrolled by
    // three so that no set is ever copied - a copy would wait for its pending request.
    int4 a0 = src[0], b0 = src[1], a1, b1, a2 = a0, b2 = b0;
    {
      const int q = 2 * kScanPass <= n ? kScanPass / 4 : 0;
      a1 = src[q];
      b1 = src[q + 1];
    }
    auto one_pass = [&](const int4& a, const int4& b, int4& fa, int4& fb) {
      const int v[kScanPer] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
      // request the pass after next into the set that is free - always, so that every path has the
      // same requests pending (past the last whole pass the first one is read again and not used)
      const int q = base + 3 * kScanPass <= n ? (base + 2 * kScanPass) / 4 : 0;
      fa = src[q];
      fb = src[q + 1];
      int run = scan_pass(v, wsum[pass & 1], carry);
      int o[kScanPer];
#pragma unroll
      for (int j = 0; j < kScanPer; ++j) {
        o[j] = run;
        run += v[j];
      }
      dst[base / 4] = make_int4(o[0], o[1], o[2], o[3]);
      dst[base / 4 + 1] = make_int4(o[4], o[5], o[6], o[7]);
      base += kScanPass;
      ++pass;
    };
    while (base + kScanPass <= n) {
      one_pass(a0, b0, a2, b2);
      if (base + kScanPass > n) break;
      one_pass(a1, b1, a0, b0);
      if (base + kScanPass > n) break;
      one_pass(a2, b2, a1, b1);
    }
  }
  for (; base < n; base += kScanPass, ++pass) {
    const int i0 = base + threadIdx.x * kScanPer;
    int v[kScanPer];
#pragma unroll
    for (int j = 0; j < kScanPer; ++j) v[j] = i0 + j < n ? counts[i0 + j] : 0;
    int run = scan_pass(v, wsum[pass & 1], carry);
#pragma unroll
    for (int j = 0; j < kScanPer; ++j) {
      if (i0 + j < n) offsets[i0 + j] = run;
      run += v[j];
    }
  }
  if (threadIdx.x == 0) *total = carry;
}

__global__ __launch_bounds__(kRowsPerBlock) void compact_kernel(const uint8_t* __restrict__ mask, int n_rows,
                                                                const int* __restrict__ offsets,
                                                                int* __restrict__ idx) {
  __shared__ int wcnt[kRowsPerBlock / 64];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int row = blockIdx.x * kRowsPerBlock + threadIdx.x;
  const bool on = row < n_rows && mask[row] != 0;
  const unsigned long long b = __ballot(on);
  if (lane == 0) wcnt[wave] = __popcll(b);
  __syncthreads();
  int base = offsets[blockIdx.x];
  for (int w = 0; w < wave; ++w) base += wcnt[w];
  if (on) idx[base + __popcll(b & ((1ull << lane) - 1ull))] = row;
}

// Scan and compaction in one launch for inputs of at most kFusedBlocks blocks of kRowsPerBlock rows
// (one pass of the scan): the offsets stay in LDS and the 16 wavefronts then rank the mask bytes of
// blocks w, w + 16, ... exactly as compact_kernel does. Same results, one launch less.
constexpr int kFusedBlocks = 2048;
static_assert(kFusedBlocks <= kScanPass, "the fused kernel scans in one pass");

__global__ __launch_bounds__(1024) void scan_compact_kernel(const int* __restrict__ counts, int nblocks,
                                                            const uint8_t* __restrict__ mask, int n_rows,
                                                            int* __restrict__ idx, int* __restrict__ total) {
  static_assert(kRowsPerBlock == 64, "one wavefront ranks one block of rows");
  __shared__ int wsum[16];
  __shared__ int offs[kFusedBlocks];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int i0 = threadIdx.x * kScanPer;
  int v[kScanPer];
#pragma unroll
  for (int j = 0; j < kScanPer; ++j) v[j] = i0 + j < nblocks ? counts[i0 + j] : 0;
  int carry = 0;
  int run = scan_pass(v, wsum, carry);
#pragma unroll
  for (int j = 0; j < kScanPer; ++j) {
    if (i0 + j < nblocks) offs[i0 + j] = run;
    run += v[j];
  }
  if (threadIdx.x == 0) *total = carry;
  __syncthreads();
  // four blocks per trip, their mask bytes requested together (the loads are what a trip waits for)
  for (int b0 = wave; b0 < nblocks; b0 += 64) {
    bool on[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int row = (b0 + 16 * q) * kRowsPerBlock + lane;
      on[q] = b0 + 16 * q < nblocks && row < n_rows && mask[row] != 0;
    }
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const unsigned long long bal = __ballot(on[q]);
      if (on[q]) idx[offs[b0 + 16 * q] + __popcll(bal & ((1ull << lane) - 1ull))] = (b0 + 16 * q) * kRowsPerBlock + lane;
    }
  }
}

// mask[r] = flags[map[r]] != 0 for a block of kRowsPerBlock rows, plus the block's count.
__global__ __launch_bounds__(kRowsPerBlock) void flag_mask_kernel(const uint8_t* __restrict__ flags,
                                                                  const int* __restrict__ map, int n_rows,
                                                                  uint8_t* __restrict__ mask,
                                                                  int* __restrict__ block_counts) {
  __shared__ int wcnt[kRowsPerBlock / 64];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int row = blockIdx.x * kRowsPerBlock + threadIdx.x;
  const bool on = row < n_rows && flags[map[row]] != 0;
  if (row < n_rows) mask[row] = on ? 1 : 0;
  const unsigned long long b = __ballot(on);
  if (lane == 0) wcnt[wave] = __popcll(b);
  __syncthreads();
  if (threadIdx.x == 0) {
    int t = 0;
    for (int w = 0; w < kRowsPerBlock / 64; ++w) t += wcnt[w];
    block_counts[blockIdx.x] = t;
  }
}

template <typename T, int EPV>
static void launch_filter(const void* cur, const void* cached, int n_rows, int dim, int64_t ld, float eps,
                          cdf_norm norm, int glog, uint8_t* mask, int* counts, int nblocks, hipStream_t st) {
  const T* a = static_cast<const T*>(cur);
  const T* b = static_cast<const T*>(cached);
  if (norm == CDF_NORM_LINF)
    filter_kernel<T, EPV, CDF_NORM_LINF><<<nblocks, kFilterThreads, 0, st>>>(a, b, n_rows, dim, ld, eps, glog,
                                                                             mask, counts);
  else
    filter_kernel<T, EPV, CDF_NORM_L2><<<nblocks, kFilterThreads, 0, st>>>(a, b, n_rows, dim, ld, eps, glog,
                                                                           mask, counts);
}

// Exclusive scan of per-block counts (blocks of kRowsPerBlock rows) and ordered compaction of the
// mask into idx / *n_sent; counts holds ceil(n_rows / kRowsPerBlock) ints, offsets = counts + scan_stride.
int scan_and_compact(const uint8_t* mask, int n_rows, int* counts, int* offsets, int32_t* idx, int32_t* n_sent,
                     hipStream_t st) {
  const int nblocks = static_cast<int>(ceil_div(n_rows, kRowsPerBlock));
  if (nblocks > 0 && nblocks <= kFusedBlocks) {
    { ProfScope ps(K_SCAN, st); scan_compact_kernel<<<1, 1024, 0, st>>>(counts, nblocks, mask, n_rows, idx, n_sent); }
    CDF_LAUNCH_CHECK("scan + compact");
    return CDF_OK;
  }
  { ProfScope ps(K_SCAN, st); scan_kernel<<<1, 1024, 0, st>>>(counts, nblocks, offsets, n_sent); }
  CDF_LAUNCH_CHECK("scan");
  if (nblocks > 0) {
    ProfScope ps(K_COMPACT, st);
    compact_kernel<<<nblocks, kRowsPerBlock, 0, st>>>(mask, n_rows, offsets, idx);
  }
  CDF_LAUNCH_CHECK("compact");
  return CDF_OK;
}

size_t filter_workspace_bytes(int64_t n_rows) {
  const int64_t nb = ceil_div(n_rows > 0 ? n_rows : 0, kRowsPerBlock);
  return align_up(static_cast<size_t>(scan_stride(nb) + nb + 1) * sizeof(int), 256);
}

}  // namespace cdf

using namespace cdf;

// Shared body of the two cache-test entry points: argument checks, then the three launches with the
// per-block counts and offsets in `buf` (buf_bytes available; the caller's workspace or the
// library's own static array).
static int cache_filter_run(const char* fn, const void* cur, const void* cached, int32_t n_rows, int32_t dim,
                            int64_t ld, cdf_dtype dt, float eps, cdf_norm norm, uint8_t* mask, int32_t* idx,
                            int32_t* n_sent, void* buf, size_t buf_bytes, hipStream_t st) {
  CDF_REQUIRE(n_rows >= 0 && dim > 0 && ld >= dim, "%s: bad shape n_rows=%d dim=%d ld=%lld", fn, n_rows, dim,
              (long long)ld);
  CDF_REQUIRE(n_sent != nullptr, "%s: n_sent is null", fn);
  CDF_REQUIRE(eps >= 0.0f && eps <= 3.0e38f, "%s: eps must be finite and >= 0", fn);
  if (dt != CDF_F32 && dt != CDF_BF16) CDF_FAIL(CDF_ERR_UNSUPPORTED, "%s: dtype %d", fn, (int)dt);
  if (norm != CDF_NORM_LINF && norm != CDF_NORM_L2) CDF_FAIL(CDF_ERR_UNSUPPORTED, "%s: norm %d", fn, (int)norm);
  if (n_rows == 0) {
    // nothing to test: the count is still defined (written by a kernel, not a memset node,
    // so that the call can be captured into a graph)
    { ProfScope ps(K_SCAN, st); scan_kernel<<<1, 1024, 0, st>>>(nullptr, 0, nullptr, n_sent); }
    CDF_LAUNCH_CHECK("cache filter/scan");
    return CDF_OK;
  }
  CDF_REQUIRE(cur && cached && mask && idx, "%s: null pointer", fn);
  const size_t esz = elem_bytes(dt);
  CDF_REQUIRE(aligned(cur, esz) && aligned(cached, esz) && aligned(idx, 4) && aligned(n_sent, 4),
              "%s: misaligned pointer", fn);
  const int nblocks = static_cast<int>(ceil_div(n_rows, kRowsPerBlock));
  if (!buf || buf_bytes < filter_workspace_bytes(n_rows) || !aligned(buf, 4))
    CDF_FAIL(CDF_ERR_WORKSPACE, "%s: workspace too small (%zu < %zu)", fn, buf_bytes,
             filter_workspace_bytes(n_rows));
  int* counts = static_cast<int*>(buf);
  int* offsets = counts + scan_stride(nblocks);

  const int epv = pick_epv(dim, ld, esz, cur, cached);
  const int nvec = dim / epv;
  const int glog = nvec >= 64 ? 6 : log2_ceil(nvec);
#define CDF_FILTER_CASE(T, E)                                                                       \
  launch_filter<T, E>(cur, cached, n_rows, dim, ld, eps, norm, glog, mask, counts, nblocks, st)
  prof_begin(K_FILTER, st);
  if (dt == CDF_F32) {
    if (epv == 4) CDF_FILTER_CASE(float, 4);
    else if (epv == 2) CDF_FILTER_CASE(float, 2);
    else CDF_FILTER_CASE(float, 1);
  } else {
    if (epv == 4) CDF_FILTER_CASE(bf16_t, 4);
    else if (epv == 2) CDF_FILTER_CASE(bf16_t, 2);
    else CDF_FILTER_CASE(bf16_t, 1);
  }
#undef CDF_FILTER_CASE
  prof_end(K_FILTER, st);
  CDF_LAUNCH_CHECK("cache filter/filter");
  return scan_and_compact(mask, n_rows, counts, offsets, idx, n_sent, st);
}

extern "C" int cdf_cache_filter(const void* cur, const void* cached, int32_t n_rows, int32_t dim, int64_t ld,
                                cdf_dtype dt, float eps, cdf_norm norm, uint8_t* mask, int32_t* idx,
                                int32_t* n_sent, void* ws, size_t ws_bytes, void* stream) {
  return cache_filter_run("cdf_cache_filter", cur, cached, n_rows, dim, ld, dt, eps, norm, mask, idx, n_sent, ws,
                          ws_bytes, static_cast<hipStream_t>(stream));
}

// ---- the cache test for callers that cannot allocate or pass a workspace ----
// The per-block counts and offsets live in a static device array (one copy per GPU, held until the
// process ends). Host code never uses the array's name as an address: it asks the runtime for the
// device address once per device and passes that to the kernels like any other buffer.
constexpr int32_t kStaticMaxRows = 8 << 20;  // 8 Mi rows -> 131 072 blocks -> about 1 MiB of counts + offsets
constexpr size_t kStaticScratchBytes =
    (((static_cast<size_t>(kStaticMaxRows / kRowsPerBlock) + 1 + 3) / 4 * 4 + kStaticMaxRows / kRowsPerBlock + 1) *
         sizeof(int) + 255) / 256 * 256;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

constexpr int kMaxDevices = 64;
static std::mutex g_scratch_mutex;
static void* g_scratch_ptr[kMaxDevices] = {};

// Device address of `scratch` on the current device (looked up on the first call per device).
static int static_scratch(const char* fn, void** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices)
    CDF_FAIL(CDF_ERR_HIP, "%s: cannot identify the current device", fn);
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !p) CDF_FAIL(CDF_ERR_HIP, "%s: hipGetSymbolAddress: %s", fn, hipGetErrorString(e));
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return CDF_OK;
}

extern "C" int cdf_cache_filter_static(const void* cur, const void* cached, int32_t n_rows, int32_t dim, int64_t ld,
                                       cdf_dtype dt, float eps, cdf_norm norm, uint8_t* mask, int32_t* idx,
                                       int32_t* n_sent, void* stream) {
  static_assert(kStaticScratchBytes >= 256, "scratch size");
  if (n_rows > kStaticMaxRows)
    CDF_FAIL(CDF_ERR_UNSUPPORTED, "cdf_cache_filter_static: %d rows exceed the static scratch (at most %d rows)",
             n_rows, kStaticMaxRows);
  void* sp = nullptr;
  const int rc = static_scratch("cdf_cache_filter_static", &sp);
  if (rc != CDF_OK) return rc;
  return cache_filter_run("cdf_cache_filter_static", cur, cached, n_rows, dim, ld, dt, eps, norm, mask, idx, n_sent,
                          sp, kStaticScratchBytes, static_cast<hipStream_t>(stream));
}

extern "C" int cdf_active_rows(const uint8_t* flags, const int32_t* map, int32_t n_rows, uint8_t* mask, int32_t* idx,
                               int32_t* n_sent, void* ws, size_t ws_bytes, void* stream) {
  hipStream_t st = static_cast<hipStream_t>(stream);
  CDF_REQUIRE(n_rows >= 0, "cdf_active_rows: negative row count");
  CDF_REQUIRE(n_sent != nullptr, "cdf_active_rows: n_sent is null");
  if (n_rows == 0) {
    scan_kernel<<<1, 1024, 0, st>>>(nullptr, 0, nullptr, n_sent);
    CDF_LAUNCH_CHECK("cdf_active_rows/scan");
    return CDF_OK;
  }
  CDF_REQUIRE(flags && map && mask && idx, "cdf_active_rows: null pointer");
  const int nblocks = static_cast<int>(ceil_div(n_rows, kRowsPerBlock));
  if (!ws || ws_bytes < filter_workspace_bytes(n_rows) || !aligned(ws, 4))
    CDF_FAIL(CDF_ERR_WORKSPACE, "cdf_active_rows: workspace too small (%zu < %zu)", ws_bytes,
             filter_workspace_bytes(n_rows));
  int* counts = static_cast<int*>(ws);
  int* offsets = counts + scan_stride(nblocks);
  flag_mask_kernel<<<nblocks, kRowsPerBlock, 0, st>>>(flags, map, n_rows, mask, counts);
  CDF_LAUNCH_CHECK("cdf_active_rows/mask");
  return scan_and_compact(mask, n_rows, counts, offsets, idx, n_sent, st);
}
