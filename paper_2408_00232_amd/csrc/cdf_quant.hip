// Message build (difference, linear quantisation, cache commit) and message recovery
// (dequantise, receiver-side cache update) - Sec. 5 and Alg. 2.
//
// Both kernels give one message row to a group of G = 2^glog lanes (a whole wavefront,
// looping, for rows of more than 64 vectors). A row is held in registers between the
// min/max pass and the coding pass, so it is read from HBM exactly once; the commit
// reuses the same registers. The number of rows comes from device memory (*n_sent);
// the grid is sized for max_sent and surplus groups leave at once.
//
// fp32 sequence (must match on every implementation for bit-equal codes):
//   inv = Lv / (hi - lo)            one correctly rounded division per row
//   q   = floor(fma(m - lo, inv, 0.5)) clamped to [0, Lv]
//   back: scale = (hi - lo) / Lv,   m~ = fma(q, scale, lo)
#include <algorithm>

#include "cdf_common.h"

namespace cdf {

constexpr int kQuantThreads = 256;
// The number of message rows is only known on the device, so grids are sized for the capacity -
// but never beyond this many blocks: the kernels walk the rows in strides, so a call that sends
// nothing costs 0.03 ms instead of up to 0.9 ms of empty blocks (5 M rows), while a call that sends
// everything still runs within a few per cent of a grid with one block per group of rows (smaller
// caps measured up to 25 % slower there).
constexpr int64_t kMessageGridCap = 131072;

// Statistics, codes, meta and cache commit of one message row held in registers: x = current row,
// z = cached row, m = what is sent. Every lane of the group must call it (the row statistics use
// cross-lane exchanges); `live` gates all stores. out / meta_row / pz point at this row's codes,
// its two meta floats and its cached row.
template <typename T, int EPV, int NIT, int BITS, int QS>
__device__ __forceinline__ void encode_row(bool live, int lg, int G, int nvec, const float (&x)[NIT][EPV],
                                           const float (&z)[NIT][EPV], const float (&m)[NIT][EPV], int commit,
                                           int delta, uint8_t* out, float* meta_row, T* pz) {
  // row statistics
  float lo = __builtin_inff(), hi = -__builtin_inff(), amax = 0.0f;
#pragma unroll
  for (int i = 0; i < NIT; ++i) {
    if (lg + i * G < nvec) {
#pragma unroll
      for (int c = 0; c < EPV; ++c) {
        lo = fminf(lo, m[i][c]);
        hi = fmaxf(hi, m[i][c]);
        amax = fmaxf(amax, fabsf(m[i][c]));
      }
    }
  }
  float m0 = 0.0f, m1 = 0.0f, inv = 0.0f, scale = 0.0f, sub = 0.0f;
  int qlo = 0, qhi = 0;
  if (QS == CDF_Q_MINMAX) {
    lo = group_min(lo, G);
    hi = group_max(hi, G);
    const float Lv = static_cast<float>((1 << BITS) - 1);
    const float range = hi - lo;
    inv = range > 0.0f ? Lv / range : 0.0f;
    scale = range / Lv;
    sub = lo;
    m0 = lo;
    m1 = hi;
    qlo = 0;
    qhi = (1 << BITS) - 1;
  } else if (QS == CDF_Q_SYMMETRIC) {
    amax = group_max(amax, G);
    const float Qm = static_cast<float>((1 << (BITS - 1)) - 1);
    inv = amax > 0.0f ? Qm / amax : 0.0f;
    scale = amax / Qm;
    sub = 0.0f;
    m0 = scale;
    m1 = 0.0f;
    qhi = (1 << (BITS - 1)) - 1;
    qlo = -qhi;
  }
  if (live && lg == 0) {
    meta_row[0] = m0;
    meta_row[1] = m1;
  }

#pragma unroll
  for (int i = 0; i < NIT; ++i) {
    const int v = lg + i * G;
    const bool on = live && v < nvec;
    float dq[EPV];
    if (QS == CDF_Q_NONE) {
      if (on) VecIO<float, EPV>::store(reinterpret_cast<float*>(out) + static_cast<int64_t>(v) * EPV, m[i]);
#pragma unroll
      for (int c = 0; c < EPV; ++c) dq[c] = m[i][c];
    } else {
      int q[EPV];
#pragma unroll
      for (int c = 0; c < EPV; ++c) {
        float t = floorf(__fmaf_rn(m[i][c] - sub, inv, 0.5f));
        t = fminf(fmaxf(t, static_cast<float>(qlo)), static_cast<float>(qhi));  // clamp, then convert
        const int qi = static_cast<int>(t);
        q[c] = on ? qi : 0;
        dq[c] = QS == CDF_Q_MINMAX ? __fmaf_rn(static_cast<float>(qi), scale, m0) : static_cast<float>(qi) * scale;
      }
      constexpr unsigned CM = (1u << BITS) - 1u;
      if (EPV == 1 && BITS == 4) {
        // two lanes share a byte: the even element's lane stores both nibbles
        const int partner = __shfl_xor(q[0], 1, kWave);
        if (on && (v & 1) == 0)
          out[v >> 1] = static_cast<uint8_t>((q[0] & CM) | ((partner & CM) << 4));
      } else {
        unsigned word = 0;
#pragma unroll
        for (int c = 0; c < EPV; ++c) word |= (static_cast<unsigned>(q[c]) & CM) << (BITS * c);
        if (on) {
          constexpr int NB = EPV * BITS / 8;  // bytes per lane-vector: 4, 2 or 1
          uint8_t* dstp = out + static_cast<int64_t>(v) * NB;
          if (NB == 4) *reinterpret_cast<uint32_t*>(dstp) = word;
          else if (NB == 2) *reinterpret_cast<uint16_t*>(dstp) = static_cast<uint16_t>(word);
          else *dstp = static_cast<uint8_t>(word);
        }
      }
    }
    if (on) {
      if (commit == CDF_COMMIT_CUR) {
        VecIO<T, EPV>::store(pz + static_cast<int64_t>(v) * EPV, x[i]);
      } else if (commit == CDF_COMMIT_DEQ) {
        float nv[EPV];
#pragma unroll
        for (int c = 0; c < EPV; ++c) nv[c] = delta ? z[i][c] + dq[c] : dq[c];
        VecIO<T, EPV>::store(pz + static_cast<int64_t>(v) * EPV, nv);
      }
    }
  }
}

// `NIT` vectors of EPV elements per lane: covers rows of up to 64*NIT vectors.
template <typename T, int EPV, int NIT, int BITS, int QS>
__global__ __launch_bounds__(kQuantThreads) void quantize_kernel(
    const T* __restrict__ cur, T* cached, const int* __restrict__ idx, const int* __restrict__ n_sent_p, int max_sent,
    int dim, int64_t ld, int glog, int commit, int delta, uint8_t* __restrict__ codes,
    float* __restrict__ meta) {
  const int n_sent = min(*n_sent_p, max_sent);   // never past the capacity of idx / codes / meta
  const int lane = threadIdx.x & 63;
  const int G = 1 << glog;
  const int lg = lane & (G - 1);
  const int rows_per_wave = 64 >> glog;
  const int gwave = blockIdx.x * (kQuantThreads / 64) + (threadIdx.x >> 6);
  const int nvec = dim / EPV;
  const int64_t rb = QS == CDF_Q_NONE ? static_cast<int64_t>(dim) * 4 : (static_cast<int64_t>(dim) * BITS + 7) / 8;
  // the grid is capped; a wavefront walks its share of the rows (the bound is the same for all its lanes)
  const int wave_stride = gridDim.x * (kQuantThreads / 64) * rows_per_wave;
  for (int kb = gwave * rows_per_wave; kb < n_sent; kb += wave_stride) {
  const int k = kb + (lane >> glog);
  const bool live = k < n_sent;

  float x[NIT][EPV], z[NIT][EPV], m[NIT][EPV];
  int64_t r = 0;
  if (live) r = idx[k];
  const T* pc = cur + r * ld;
  T* pz = cached + r * ld;
#pragma unroll
  for (int i = 0; i < NIT; ++i) {
    const int v = lg + i * G;
#pragma unroll
    for (int c = 0; c < EPV; ++c) x[i][c] = z[i][c] = 0.0f;
    if (live && v < nvec) {
      VecIO<T, EPV>::load(pc + static_cast<int64_t>(v) * EPV, x[i]);
      if (delta || commit == CDF_COMMIT_DEQ) VecIO<T, EPV>::load(pz + static_cast<int64_t>(v) * EPV, z[i]);
    }
#pragma unroll
    for (int c = 0; c < EPV; ++c) m[i][c] = delta ? x[i][c] - z[i][c] : x[i][c];
  }

  encode_row<T, EPV, NIT, BITS, QS>(live, lg, G, nvec, x, z, m, commit, delta,
                                    codes + static_cast<int64_t>(live ? k : 0) * rb,
                                    meta + 2 * static_cast<int64_t>(live ? k : 0), pz);
  }
}

// Cache test and message build in one pass over the rows (the two steps of Alg. 2's mirror loop
// back to back): every row is read once, tested (either norm), and - if it fails the test -
// coded and committed from the same registers. The position of a row's message in the output is
// only known after the count of sent rows before it, so codes and meta go to a row-indexed
// scratch area first and gather_codes_kernel moves them to their final place (one byte per
// element instead of re-reading the rows at eight). Blocks of kTestRows rows, one count per block,
// as the cache test writes them.
constexpr int kTestRows = kRowsPerBlock;

template <typename T, int EPV, int NIT, int BITS, int QS>
__global__ __launch_bounds__(kQuantThreads) void test_encode_kernel(
    const T* __restrict__ cur, T* cached, int n_rows, int dim, int64_t ld, float eps, int norm, int glog, int commit,
    int delta, uint8_t* __restrict__ mask, int* __restrict__ block_counts, uint8_t* __restrict__ codes_scratch,
    float* __restrict__ meta_scratch) {
  constexpr int NACC = 4 / EPV;  // L2 norm: accumulators per lane-component, as in the cache test
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int G = 1 << glog;
  const int lg = lane & (G - 1), sub = lane >> glog;
  const int rows_per_step = 64 >> glog;
  const int nvec = dim / EPV;
  const int64_t rb = (static_cast<int64_t>(dim) * BITS + 7) / 8;
  constexpr int kRowsPerWave = kTestRows / (kQuantThreads / 64);
  const int row0 = blockIdx.x * kTestRows + wave * kRowsPerWave;
  int sent_here = 0;
  for (int s = 0; s < kRowsPerWave; s += rows_per_step) {
    const int row = row0 + s + sub;
    const bool live = row < n_rows && s + sub < kRowsPerWave;
    const int64_t r = live ? row : 0;
    const T* pc = cur + r * ld;
    T* pz = cached + r * ld;
    float x[NIT][EPV], z[NIT][EPV], m[NIT][EPV];
#pragma unroll
    for (int i = 0; i < NIT; ++i) {
      const int v = lg + i * G;
#pragma unroll
      for (int c = 0; c < EPV; ++c) x[i][c] = z[i][c] = 0.0f;
      if (live && v < nvec) {
        VecIO<T, EPV>::load(pc + static_cast<int64_t>(v) * EPV, x[i]);
        VecIO<T, EPV>::load(pz + static_cast<int64_t>(v) * EPV, z[i]);
      }
#pragma unroll
      for (int c = 0; c < EPV; ++c) m[i][c] = delta ? x[i][c] - z[i][c] : x[i][c];
    }
    // the test, in the cache test's own order of operations (masks must agree bit for bit)
    float D, C, thr;
    if (norm == CDF_NORM_LINF) {
      D = 0.0f;
      C = 0.0f;
#pragma unroll
      for (int i = 0; i < NIT; ++i)
#pragma unroll
        for (int c = 0; c < EPV; ++c) {
          D = fmaxf(D, fabsf(x[i][c] - z[i][c]));
          C = fmaxf(C, fabsf(z[i][c]));
        }
      D = group_max(D, G);
      C = group_max(C, G);
      thr = eps * C;
    } else {
      // vector i of a lane feeds accumulator i mod NACC; lanes past the row end add exact zeros
      float ad[NACC][EPV], ac[NACC][EPV];
#pragma unroll
      for (int a = 0; a < NACC; ++a)
#pragma unroll
        for (int c = 0; c < EPV; ++c) ad[a][c] = ac[a][c] = 0.0f;
#pragma unroll
      for (int i = 0; i < NIT; ++i)
#pragma unroll
        for (int c = 0; c < EPV; ++c) {
          const float d = x[i][c] - z[i][c];
          ad[i % NACC][c] = __fmaf_rn(d, d, ad[i % NACC][c]);
          ac[i % NACC][c] = __fmaf_rn(z[i][c], z[i][c], ac[i % NACC][c]);
        }
      float Da[NACC], Ca[NACC];
#pragma unroll
      for (int a = 0; a < NACC; ++a) {
        float d, c;
        if (EPV == 4) {
          d = (ad[a][0] + ad[a][1 % EPV]) + (ad[a][2 % EPV] + ad[a][3 % EPV]);
          c = (ac[a][0] + ac[a][1 % EPV]) + (ac[a][2 % EPV] + ac[a][3 % EPV]);
        } else if (EPV == 2) {
          d = ad[a][0] + ad[a][1 % EPV];
          c = ac[a][0] + ac[a][1 % EPV];
        } else {
          d = ad[a][0];
          c = ac[a][0];
        }
        Da[a] = group_sum(d, G);
        Ca[a] = group_sum(c, G);
      }
      if (NACC == 4) {
        D = (Da[0] + Da[1 % NACC]) + (Da[2 % NACC] + Da[3 % NACC]);
        C = (Ca[0] + Ca[1 % NACC]) + (Ca[2 % NACC] + Ca[3 % NACC]);
      } else if (NACC == 2) {
        D = Da[0] + Da[1 % NACC];
        C = Ca[0] + Ca[1 % NACC];
      } else {
        D = Da[0];
        C = Ca[0];
      }
      const float e2 = eps * eps;
      thr = e2 * C;
    }
    const bool send = live && D > thr;
    const bool head = live && lg == 0;
    if (head) mask[row] = send ? 1 : 0;
    sent_here += __popcll(__ballot(head && send));
    encode_row<T, EPV, NIT, BITS, QS>(send, lg, G, nvec, x, z, m, commit, delta, codes_scratch + r * rb,
                                      meta_scratch + 2 * r, pz);
  }
  __shared__ int wave_cnt[kQuantThreads / 64];
  if (lane == 0) wave_cnt[wave] = sent_here;
  __syncthreads();
  if (threadIdx.x == 0) {
    int t = 0;
    for (int w = 0; w < kQuantThreads / 64; ++w) t += wave_cnt[w];
    block_counts[blockIdx.x] = t;
  }
}

// ---- cache test and message build in one pass, every message written once, in its place -------------
// The rank of a sent row among all sent rows is its position in idx / codes / meta. Here the wavefronts
// of a workgroup hold their rows in registers, count how many of them fail the test, and the workgroup
// learns the number of sent rows before its first one from the workgroups before it through a chain of
// status words in device memory (a single-pass scan with look-back): workgroup e publishes its own
// count at once, then its first wavefront reads back over the predecessors' words - counts of those
// that do not know their prefix yet, the prefix of the first one that does - and publishes its own
// prefix. The wavefronts then code their sent rows straight into rows k, k+1, ... of the outputs from
// the registers they still hold.
//
// Progress: workgroups are dispatched in the order of their ids and a workgroup publishes its count
// before it waits, so the workgroups it waits for are resident or finished. The wait is bounded all the
// same: after `spin_limit` polls a workgroup gives up, marks its word, and every later workgroup that
// meets the mark does the same; *n_sent is then -1 and the rows from there on are neither coded nor
// committed. Every wavefront reaches its end either way.
constexpr int kChainEmpty = 0, kChainCount = 1, kChainPrefix = 2, kChainGaveUp = 3;

__device__ __forceinline__ unsigned long long chain_word(int state, int value) {
  return (static_cast<unsigned long long>(static_cast<unsigned>(state)) << 32) | static_cast<unsigned>(value);
}

// Steps of rows a wavefront holds at once: about 32 values of x and of z per lane.
__host__ __device__ constexpr int chain_steps(int per_lane) {
  return per_lane >= 32 ? 1 : per_lane >= 16 ? 2 : per_lane >= 8 ? 4 : 8;
}

__global__ __launch_bounds__(256) void chain_clear_kernel(unsigned long long* __restrict__ status, int n) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i < n) status[i] = 0ull;
}

template <typename T, int EPV, int NIT, int BITS, int QS>
__global__ __launch_bounds__(kQuantThreads) void test_encode_chained_kernel(
    const T* __restrict__ cur, T* cached, int n_rows, int dim, int64_t ld, float eps, int norm, int glog, int commit,
    int delta, uint8_t* __restrict__ mask, int* __restrict__ idx, int* __restrict__ n_sent,
    uint8_t* __restrict__ codes, float* __restrict__ meta, unsigned long long* status, int n_elems, int spin_limit) {
  constexpr int NACC = 4 / EPV;
  constexpr int S = chain_steps(NIT * EPV);
  constexpr int kWaves = kQuantThreads / 64;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int e = blockIdx.x;   // this workgroup's place in the chain (its wavefronts take consecutive rows)
  const int G = 1 << glog;
  const int lg = lane & (G - 1), sub = lane >> glog;
  const int rows_per_step = 64 >> glog;
  const int nvec = dim / EPV;
  const int64_t rb = (static_cast<int64_t>(dim) * BITS + 7) / 8;
  const int row0 = (e * kWaves + wave) * (S * rows_per_step);

  float x[S][NIT][EPV], z[S][NIT][EPV];
  bool send[S];
  unsigned long long bits[S];
  int count = 0;
#pragma unroll
  for (int s = 0; s < S; ++s) {
    const int row = row0 + s * rows_per_step + sub;
    const bool live = row < n_rows;
    const int64_t r = live ? row : 0;
    const T* pc = cur + r * ld;
    const T* pz = cached + r * ld;
#pragma unroll
    for (int i = 0; i < NIT; ++i) {
      const int v = lg + i * G;
#pragma unroll
      for (int c = 0; c < EPV; ++c) x[s][i][c] = z[s][i][c] = 0.0f;
      if (live && v < nvec) {
        VecIO<T, EPV>::load(pc + static_cast<int64_t>(v) * EPV, x[s][i]);
        VecIO<T, EPV>::load(pz + static_cast<int64_t>(v) * EPV, z[s][i]);
      }
    }
  }
#pragma unroll
  for (int s = 0; s < S; ++s) {
    const int row = row0 + s * rows_per_step + sub;
    const bool live = row < n_rows;
    // the test, in the cache test's own order of operations (masks must agree bit for bit)
    float D, C, thr;
    if (norm == CDF_NORM_LINF) {
      D = 0.0f;
      C = 0.0f;
#pragma unroll
      for (int i = 0; i < NIT; ++i)
#pragma unroll
        for (int c = 0; c < EPV; ++c) {
          D = fmaxf(D, fabsf(x[s][i][c] - z[s][i][c]));
          C = fmaxf(C, fabsf(z[s][i][c]));
        }
      D = group_max(D, G);
      C = group_max(C, G);
      thr = eps * C;
    } else {
      float ad[NACC][EPV], ac[NACC][EPV];
#pragma unroll
      for (int a = 0; a < NACC; ++a)
#pragma unroll
        for (int c = 0; c < EPV; ++c) ad[a][c] = ac[a][c] = 0.0f;
#pragma unroll
      for (int i = 0; i < NIT; ++i)
#pragma unroll
        for (int c = 0; c < EPV; ++c) {
          const float d = x[s][i][c] - z[s][i][c];
          ad[i % NACC][c] = __fmaf_rn(d, d, ad[i % NACC][c]);
          ac[i % NACC][c] = __fmaf_rn(z[s][i][c], z[s][i][c], ac[i % NACC][c]);
        }
      float Da[NACC], Ca[NACC];
#pragma unroll
      for (int a = 0; a < NACC; ++a) {
        float d, c;
        if (EPV == 4) {
          d = (ad[a][0] + ad[a][1 % EPV]) + (ad[a][2 % EPV] + ad[a][3 % EPV]);
          c = (ac[a][0] + ac[a][1 % EPV]) + (ac[a][2 % EPV] + ac[a][3 % EPV]);
        } else if (EPV == 2) {
          d = ad[a][0] + ad[a][1 % EPV];
          c = ac[a][0] + ac[a][1 % EPV];
        } else {
          d = ad[a][0];
          c = ac[a][0];
        }
        Da[a] = group_sum(d, G);
        Ca[a] = group_sum(c, G);
      }
      if (NACC == 4) {
        D = (Da[0] + Da[1 % NACC]) + (Da[2 % NACC] + Da[3 % NACC]);
        C = (Ca[0] + Ca[1 % NACC]) + (Ca[2 % NACC] + Ca[3 % NACC]);
      } else if (NACC == 2) {
        D = Da[0] + Da[1 % NACC];
        C = Ca[0] + Ca[1 % NACC];
      } else {
        D = Da[0];
        C = Ca[0];
      }
      const float e2 = eps * eps;
      thr = e2 * C;
    }
    send[s] = live && D > thr;
    const bool head = live && lg == 0;
    if (head) mask[row] = send[s] ? 1 : 0;
    bits[s] = __ballot(head && send[s]);
    count += __popcll(bits[s]);
  }

  // ---- the chain: sent rows before this workgroup's first row (looked up by its first wavefront) ----
  __shared__ int wave_count[kWaves];
  __shared__ int block_before;   // -1: gave up
  if (lane == 0) wave_count[wave] = count;
  __syncthreads();
  int block_count = 0, wave_before = 0;
#pragma unroll
  for (int w = 0; w < kWaves; ++w) {
    const int c = wave_count[w];
    if (w < wave) wave_before += c;
    block_count += c;
  }
  if (wave == 0) {
    int before = 0;
    bool gave_up = false;
    if (e == 0) {
      if (lane == 0)
        __hip_atomic_store(status, chain_word(kChainPrefix, block_count), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    } else {
      if (lane == 0)
        __hip_atomic_store(status + e, chain_word(kChainCount, block_count), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      int pos = e - 1, polls = 0;
      while (true) {
        const int i = pos - lane;   // lane l looks at the l-th workgroup back from pos; past the start counts as prefix 0
        const unsigned long long w = i >= 0 ? __hip_atomic_load(status + i, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)
                                            : chain_word(kChainPrefix, 0);
        const int state = static_cast<int>(w >> 32);
        const unsigned long long known = __ballot(state == kChainPrefix);
        const int first = known != 0ull ? __builtin_ctzll(known) : 64;   // nearest workgroup that knows its prefix
        const unsigned long long needed = first >= 63 ? ~0ull : (2ull << first) - 1ull;   // lanes 0 .. first
        if ((__ballot(state == kChainGaveUp) & needed) != 0ull) {
          gave_up = true;
          break;
        }
        if ((__ballot(state == kChainEmpty) & needed) != 0ull) {
          if (++polls > spin_limit) {
            gave_up = true;
            break;
          }
          __builtin_amdgcn_s_sleep(2);
          continue;
        }
        int v = lane <= first ? static_cast<int>(static_cast<unsigned>(w)) : 0;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) v += __shfl_xor(v, off, kWave);
        before += v;
        if (first < 64) break;
        pos -= 64;
      }
      if (lane == 0)
        __hip_atomic_store(status + e, gave_up ? chain_word(kChainGaveUp, 0) : chain_word(kChainPrefix, before + block_count),
                           __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    if (lane == 0) {
      block_before = gave_up ? -1 : before;
      if (e == n_elems - 1) *n_sent = gave_up ? -1 : before + block_count;
    }
  }
  __syncthreads();
  if (block_before < 0) return;
  int before = block_before + wave_before;

  // ---- code and commit the sent rows, in place ----
#pragma unroll
  for (int s = 0; s < S; ++s) {
    const int row = row0 + s * rows_per_step + sub;
    const int64_t r = send[s] ? row : 0;
    const int64_t k = send[s] ? before + __popcll(bits[s] & ((1ull << (sub << glog)) - 1ull)) : 0;
    float m[NIT][EPV];
#pragma unroll
    for (int i = 0; i < NIT; ++i)
#pragma unroll
      for (int c = 0; c < EPV; ++c) m[i][c] = delta ? x[s][i][c] - z[s][i][c] : x[s][i][c];
    if (send[s] && lg == 0) idx[k] = row;
    encode_row<T, EPV, NIT, BITS, QS>(send[s], lg, G, nvec, x[s], z[s], m, commit, delta, codes + k * rb, meta + 2 * k,
                                      cached + r * ld);
    before += __popcll(bits[s]);
  }
}

// codes[k] = scratch[idx[k]], meta[k] = meta_scratch[idx[k]] for k < *n_sent, rows of rb bytes moved
// in units of U bytes by groups of 16 lanes.
template <typename U>
__global__ __launch_bounds__(256) void gather_codes_kernel(const uint8_t* __restrict__ scratch,
                                                           const float* __restrict__ meta_scratch,
                                                           const int* __restrict__ idx, const int* __restrict__ n_sent_p,
                                                           int max_sent, int64_t rb, uint8_t* __restrict__ codes,
                                                           float* __restrict__ meta) {
  const int n_sent = min(*n_sent_p, max_sent);
  const int l = threadIdx.x & 15;
  const int units = static_cast<int>(rb / sizeof(U));
  for (int k = blockIdx.x * 16 + (threadIdx.x >> 4); k < n_sent; k += gridDim.x * 16) {
    const int64_t r = idx[k];
    const U* src = reinterpret_cast<const U*>(scratch + r * rb);
    U* dst = reinterpret_cast<U*>(codes + static_cast<int64_t>(k) * rb);
    for (int i = l; i < units; i += 16) dst[i] = src[i];
    if (l < 2) meta[2 * static_cast<int64_t>(k) + l] = meta_scratch[2 * r + l];
  }
}

template <typename T, int EPV, int NIT, int BITS, int QS>
__global__ __launch_bounds__(kQuantThreads) void dequantize_kernel(
    const uint8_t* __restrict__ codes, const float* __restrict__ meta, const int* __restrict__ idx,
    const int* __restrict__ n_sent_p, int max_sent, int dim, int glog, T* dst, int64_t ld, int accumulate) {
  const int n_sent = min(*n_sent_p, max_sent);
  const int lane = threadIdx.x & 63;
  const int G = 1 << glog;
  const int lg = lane & (G - 1);
  const int rows_per_wave = 64 >> glog;
  const int gwave = blockIdx.x * (kQuantThreads / 64) + (threadIdx.x >> 6);
  const int nvec = dim / EPV;
  const int64_t rb = QS == CDF_Q_NONE ? static_cast<int64_t>(dim) * 4 : (static_cast<int64_t>(dim) * BITS + 7) / 8;
  const int wave_stride = gridDim.x * (kQuantThreads / 64) * rows_per_wave;
  for (int kb = gwave * rows_per_wave; kb < n_sent; kb += wave_stride) {
  const int k = kb + (lane >> glog);
  if (k >= n_sent) continue;
  const int64_t r = idx[k];
  const uint8_t* in = codes + static_cast<int64_t>(k) * rb;
  T* pd = dst + r * ld;
  const float m0 = meta[2 * static_cast<int64_t>(k)], m1 = meta[2 * static_cast<int64_t>(k) + 1];
  float scale = 0.0f;
  if (QS == CDF_Q_MINMAX) scale = (m1 - m0) / static_cast<float>((1 << BITS) - 1);
  if (QS == CDF_Q_SYMMETRIC) scale = m0;
#pragma unroll
  for (int i = 0; i < NIT; ++i) {
    const int v = lg + i * G;
    if (v >= nvec) continue;
    float val[EPV];
    if (QS == CDF_Q_NONE) {
      VecIO<float, EPV>::load(reinterpret_cast<const float*>(in) + static_cast<int64_t>(v) * EPV, val);
    } else {
      unsigned word;
      constexpr unsigned CM = (1u << BITS) - 1u;
      if (EPV == 1 && BITS == 4) {
        word = (in[v >> 1] >> (4 * (v & 1))) & CM;
      } else {
        constexpr int NB = EPV * BITS / 8 > 0 ? EPV * BITS / 8 : 1;
        const uint8_t* sp = in + static_cast<int64_t>(v) * NB;
        if (NB == 4) word = *reinterpret_cast<const uint32_t*>(sp);
        else if (NB == 2) word = *reinterpret_cast<const uint16_t*>(sp);
        else word = *sp;
      }
#pragma unroll
      for (int c = 0; c < EPV; ++c) {
        int q = static_cast<int>((word >> (BITS * c)) & CM);
        if (QS == CDF_Q_MINMAX) {
          val[c] = __fmaf_rn(static_cast<float>(q), scale, m0);
        } else {
          constexpr int SGN = 1 << (BITS - 1);
          q = (q ^ SGN) - SGN;
          val[c] = static_cast<float>(q) * scale;
        }
      }
    }
    if (accumulate) {
      float old[EPV];
      VecIO<T, EPV>::load(pd + static_cast<int64_t>(v) * EPV, old);
#pragma unroll
      for (int c = 0; c < EPV; ++c) val[c] = old[c] + val[c];
    }
    VecIO<T, EPV>::store(pd + static_cast<int64_t>(v) * EPV, val);
  }
  }
}

struct RowShape {
  int epv, nit, glog;
};

// Lane-vector width, vectors per lane and lanes per row for rows of `dim` elements.
static bool row_shape(int32_t dim, int epv, RowShape* s) {
  const int nvec = dim / epv;
  int nit = 1;
  s->epv = epv;
  while (nit * 64 < nvec) nit <<= 1;
  if (nit > 8) return false;
  s->nit = nit;
  s->glog = nvec >= 64 ? 6 : log2_ceil(nvec);
  if (epv == 1 && s->glog == 0) s->glog = 1;  // nibble pairs need two lanes
  return true;
}

#define CDF_DISPATCH_NIT(K, T, E, B, Q, nit, ...)          \
  switch (nit) {                                            \
    case 1: K<T, E, 1, B, Q> __VA_ARGS__; break;            \
    case 2: K<T, E, 2, B, Q> __VA_ARGS__; break;            \
    case 4: K<T, E, 4, B, Q> __VA_ARGS__; break;            \
    default: K<T, E, 8, B, Q> __VA_ARGS__; break;           \
  }
#define CDF_DISPATCH_EPV(K, T, B, Q, epv, nit, ...)                            \
  switch (epv) {                                                                \
    case 4: CDF_DISPATCH_NIT(K, T, 4, B, Q, nit, __VA_ARGS__) break;            \
    case 2: CDF_DISPATCH_NIT(K, T, 2, B, Q, nit, __VA_ARGS__) break;            \
    default: CDF_DISPATCH_NIT(K, T, 1, B, Q, nit, __VA_ARGS__) break;           \
  }
#define CDF_DISPATCH_Q(K, T, bits, qs, epv, nit, ...)                                              \
  if (qs == CDF_Q_NONE) { CDF_DISPATCH_EPV(K, T, 8, CDF_Q_NONE, epv, nit, __VA_ARGS__) }           \
  else if (qs == CDF_Q_MINMAX && bits == 8) { CDF_DISPATCH_EPV(K, T, 8, CDF_Q_MINMAX, epv, nit, __VA_ARGS__) } \
  else if (qs == CDF_Q_MINMAX) { CDF_DISPATCH_EPV(K, T, 4, CDF_Q_MINMAX, epv, nit, __VA_ARGS__) }  \
  else if (bits == 8) { CDF_DISPATCH_EPV(K, T, 8, CDF_Q_SYMMETRIC, epv, nit, __VA_ARGS__) }        \
  else { CDF_DISPATCH_EPV(K, T, 4, CDF_Q_SYMMETRIC, epv, nit, __VA_ARGS__) }

size_t filter_workspace_bytes(int64_t n_rows);
int scan_and_compact(const uint8_t* mask, int n_rows, int* counts, int* offsets, int32_t* idx, int32_t* n_sent,
                     hipStream_t st);

// Workspace of the one-pass test + message build: block counts and offsets, then row-indexed codes
// and meta. Sized for 8-bit codes of `dim` elements (the largest quantised row).
size_t test_encode_workspace_bytes(int64_t n_rows, int32_t dim) {
  const size_t rows = static_cast<size_t>(n_rows > 0 ? n_rows : 0);
  return filter_workspace_bytes(n_rows) + align_up(rows * static_cast<size_t>(dim), 256) + align_up(rows * 8, 256);
}

}  // namespace cdf

using namespace cdf;

extern "C" size_t cdf_code_row_bytes(int32_t dim, int bits, cdf_qscheme qs) {
  if (dim <= 0) return 0;
  if (qs == CDF_Q_NONE) return static_cast<size_t>(dim) * 4;
  return (static_cast<size_t>(dim) * bits + 7) / 8;
}

// Widest row the message kernels take for this width / pitch / type, assuming 16-byte aligned base
// pointers: 512 lane-vectors of the widest vector both allow.
extern "C" int32_t cdf_max_message_dim(int32_t dim, int64_t ld, cdf_dtype dt) {
  if (dim <= 0 || ld < dim || (dt != CDF_F32 && dt != CDF_BF16)) return 0;
  return 512 * pick_epv(dim, ld, elem_bytes(dt), nullptr);
}

static int check_scheme(const char* fn, int bits, cdf_qscheme qs, cdf_dtype dt) {
  if (dt != CDF_F32 && dt != CDF_BF16) CDF_FAIL(CDF_ERR_UNSUPPORTED, "%s: dtype %d", fn, (int)dt);
  if (qs != CDF_Q_MINMAX && qs != CDF_Q_SYMMETRIC && qs != CDF_Q_NONE)
    CDF_FAIL(CDF_ERR_UNSUPPORTED, "%s: scheme %d", fn, (int)qs);
  if (qs != CDF_Q_NONE && bits != 8 && bits != 4) CDF_FAIL(CDF_ERR_UNSUPPORTED, "%s: bits %d", fn, bits);
  return CDF_OK;
}

extern "C" int cdf_quantize(const void* cur, void* cached, const int32_t* idx, const int32_t* n_sent,
                            int32_t max_sent, int32_t dim, int64_t ld, cdf_dtype dt, int bits, cdf_qscheme qs,
                            cdf_commit commit, int delta, uint8_t* codes, float* meta, void* stream) {
  hipStream_t st = static_cast<hipStream_t>(stream);
  CDF_REQUIRE(max_sent >= 0 && dim > 0 && ld >= dim, "cdf_quantize: bad shape max_sent=%d dim=%d ld=%lld",
              max_sent, dim, (long long)ld);
  int rc = check_scheme("cdf_quantize", bits, qs, dt);
  if (rc != CDF_OK) return rc;
  CDF_REQUIRE(commit == CDF_COMMIT_NONE || commit == CDF_COMMIT_CUR || commit == CDF_COMMIT_DEQ,
              "cdf_quantize: commit %d", (int)commit);
  if (max_sent == 0) return CDF_OK;
  CDF_REQUIRE(cur && idx && n_sent && codes && meta, "cdf_quantize: null pointer");
  CDF_REQUIRE(cached || (!delta && commit == CDF_COMMIT_NONE),
              "cdf_quantize: cached is null but delta/commit need it");
  const size_t esz = elem_bytes(dt);
  CDF_REQUIRE(aligned(cur, esz) && (!cached || aligned(cached, esz)) && aligned(idx, 4) && aligned(n_sent, 4) &&
                  aligned(meta, 8) && aligned(codes, 16),
              "cdf_quantize: misaligned pointer (codes needs 16 bytes, meta 8)");
  RowShape s;
  if (!row_shape(dim, pick_epv(dim, ld, esz, cur, cached), &s))
    CDF_FAIL(CDF_ERR_UNSUPPORTED, "cdf_quantize: dim %d too wide for its alignment (max %d)", dim, 512 * s.epv);
  const int rows_per_block = (kQuantThreads / 64) * (64 >> s.glog);
  const int nblocks = static_cast<int>(std::min<int64_t>(ceil_div(max_sent, rows_per_block), kMessageGridCap));
#define ARGS_F32 <<<nblocks, kQuantThreads, 0, st>>>(static_cast<const float*>(cur), static_cast<float*>(cached), \
                 idx, n_sent, max_sent, dim, ld, s.glog, (int)commit, delta ? 1 : 0, codes, meta)
#define ARGS_BF16 <<<nblocks, kQuantThreads, 0, st>>>(static_cast<const bf16_t*>(cur), static_cast<bf16_t*>(cached), \
                 idx, n_sent, max_sent, dim, ld, s.glog, (int)commit, delta ? 1 : 0, codes, meta)
  prof_begin(K_QUANTIZE, st);
  if (dt == CDF_F32) { CDF_DISPATCH_Q(quantize_kernel, float, bits, qs, s.epv, s.nit, ARGS_F32) }
  else { CDF_DISPATCH_Q(quantize_kernel, bf16_t, bits, qs, s.epv, s.nit, ARGS_BF16) }
  prof_end(K_QUANTIZE, st);
#undef ARGS_F32
#undef ARGS_BF16
  CDF_LAUNCH_CHECK("cdf_quantize");
  return CDF_OK;
}

extern "C" int cdf_dequantize(const uint8_t* codes, const float* meta, const int32_t* idx, const int32_t* n_sent,
                              int32_t max_sent, int32_t dim, int bits, cdf_qscheme qs, void* dst, int64_t ld,
                              cdf_dtype dt, int accumulate, void* stream) {
  hipStream_t st = static_cast<hipStream_t>(stream);
  CDF_REQUIRE(max_sent >= 0 && dim > 0 && ld >= dim, "cdf_dequantize: bad shape max_sent=%d dim=%d ld=%lld",
              max_sent, dim, (long long)ld);
  int rc = check_scheme("cdf_dequantize", bits, qs, dt);
  if (rc != CDF_OK) return rc;
  if (max_sent == 0) return CDF_OK;
  CDF_REQUIRE(codes && meta && idx && n_sent && dst, "cdf_dequantize: null pointer");
  const size_t esz = elem_bytes(dt);
  CDF_REQUIRE(aligned(dst, esz) && aligned(idx, 4) && aligned(n_sent, 4) && aligned(meta, 8) && aligned(codes, 16),
              "cdf_dequantize: misaligned pointer (codes needs 16 bytes, meta 8)");
  RowShape s;
  if (!row_shape(dim, pick_epv(dim, ld, esz, dst), &s))
    CDF_FAIL(CDF_ERR_UNSUPPORTED, "cdf_dequantize: dim %d too wide for its alignment (max %d)", dim, 512 * s.epv);
  const int rows_per_block = (kQuantThreads / 64) * (64 >> s.glog);
  const int nblocks = static_cast<int>(std::min<int64_t>(ceil_div(max_sent, rows_per_block), kMessageGridCap));
#define ARGS_F32 <<<nblocks, kQuantThreads, 0, st>>>(codes, meta, idx, n_sent, max_sent, dim, s.glog, static_cast<float*>(dst), \
                 ld, accumulate ? 1 : 0)
#define ARGS_BF16 <<<nblocks, kQuantThreads, 0, st>>>(codes, meta, idx, n_sent, max_sent, dim, s.glog, static_cast<bf16_t*>(dst), \
                 ld, accumulate ? 1 : 0)
  prof_begin(K_DEQUANTIZE, st);
  if (dt == CDF_F32) { CDF_DISPATCH_Q(dequantize_kernel, float, bits, qs, s.epv, s.nit, ARGS_F32) }
  else { CDF_DISPATCH_Q(dequantize_kernel, bf16_t, bits, qs, s.epv, s.nit, ARGS_BF16) }
  prof_end(K_DEQUANTIZE, st);
#undef ARGS_F32
#undef ARGS_BF16
  CDF_LAUNCH_CHECK("cdf_dequantize");
  return CDF_OK;
}

namespace cdf {

// Cache test followed by the message build, as the layer steps need them. One pass over the rows
// when the messages are quantised and the workspace is large
// enough (test_encode_workspace_bytes); otherwise cdf_cache_filter then cdf_quantize. Both routes
// compute every row with the same instruction sequence: mask, idx, codes, meta and the committed
// cache are bit-identical.
static int g_chain_spin_limit = 1 << 20;   // polls of a workgroup's bounded wait for its predecessors
// The chained kernel is taken while all its workgroups are resident together (inputs of up to some ten
// thousand rows): there it saves two launches and the second pass over the messages. On larger inputs
// the wait for the predecessors costs more latency hiding than the second pass costs bandwidth
// (measured 1.2 to 1.6 times slower from 250 000 rows on), so those stage the messages by row.
constexpr int kChainMaxElems = 2048;

int test_and_encode(const void* cur, void* cached, int32_t n_rows, int32_t dim, int64_t ld, cdf_dtype dt, float eps,
                    cdf_norm norm, int bits, cdf_qscheme qs, cdf_commit commit, int delta, uint8_t* mask, int32_t* idx,
                    int32_t* n_sent, uint8_t* codes, float* meta, void* ws, size_t ws_bytes, void* stream) {
  hipStream_t st = static_cast<hipStream_t>(stream);
  RowShape s = {};
  const size_t esz = elem_bytes(dt);
  const bool types_ok = (dt == CDF_F32 || dt == CDF_BF16) && (qs == CDF_Q_MINMAX || qs == CDF_Q_SYMMETRIC) &&
                        (bits == 8 || bits == 4) && (norm == CDF_NORM_LINF || norm == CDF_NORM_L2) && n_rows > 0 && dim > 0 && ld >= dim &&
                        cur && cached && mask && idx && n_sent && codes && meta && eps >= 0.0f && eps <= 3.0e38f &&
                        (commit == CDF_COMMIT_NONE || commit == CDF_COMMIT_CUR || commit == CDF_COMMIT_DEQ);
  const bool one_pass = types_ok && ws && aligned(ws, 256) && ws_bytes >= test_encode_workspace_bytes(n_rows, dim) &&
                        aligned(cur, esz) && aligned(cached, esz) && aligned(meta, 8) && aligned(codes, 16) &&
                        aligned(idx, 4) && aligned(n_sent, 4) && row_shape(dim, pick_epv(dim, ld, esz, cur, cached), &s);
  if (!one_pass) {
    const int rc = cdf_cache_filter(cur, cached, n_rows, dim, ld, dt, eps, norm, mask, idx, n_sent, ws, ws_bytes, stream);
    if (rc != CDF_OK) return rc;
    return cdf_quantize(cur, cached, idx, n_sent, n_rows, dim, ld, dt, bits, qs, commit, delta, codes, meta, stream);
  }
  // every message written once, in its place: the chained kernel (see test_encode_chained_kernel)
  const int chain_rows = (kQuantThreads / 64) * chain_steps(s.nit * s.epv) * (64 >> s.glog);   // rows per workgroup
  const int n_elems = static_cast<int>(ceil_div(n_rows, chain_rows));
  if (n_elems <= kChainMaxElems && ws_bytes >= align_up(static_cast<size_t>(n_elems) * 8, 256)) {
    unsigned long long* status = static_cast<unsigned long long*>(ws);
    {
      ProfScope ps(K_SCAN, st);
      chain_clear_kernel<<<static_cast<unsigned>(ceil_div(n_elems, 256)), 256, 0, st>>>(status, n_elems);
    }
    CDF_LAUNCH_CHECK("test_and_encode/clear");
    const unsigned grid = static_cast<unsigned>(n_elems);
#define ARGS_CH(T) <<<grid, kQuantThreads, 0, st>>>(static_cast<const T*>(cur), static_cast<T*>(cached), n_rows, dim, ld, \
                 eps, (int)norm, s.glog, (int)commit, delta ? 1 : 0, mask, idx, n_sent, codes, meta, status, n_elems, \
                 g_chain_spin_limit)
#define CDF_DISPATCH_CH(K, T, ...)                                                                         \
  if (qs == CDF_Q_MINMAX && bits == 8) { CDF_DISPATCH_EPV(K, T, 8, CDF_Q_MINMAX, s.epv, s.nit, __VA_ARGS__) } \
  else if (qs == CDF_Q_MINMAX) { CDF_DISPATCH_EPV(K, T, 4, CDF_Q_MINMAX, s.epv, s.nit, __VA_ARGS__) }      \
  else if (bits == 8) { CDF_DISPATCH_EPV(K, T, 8, CDF_Q_SYMMETRIC, s.epv, s.nit, __VA_ARGS__) }            \
  else { CDF_DISPATCH_EPV(K, T, 4, CDF_Q_SYMMETRIC, s.epv, s.nit, __VA_ARGS__) }
    prof_begin(K_TEST_ENCODE, st);
    if (dt == CDF_F32) { CDF_DISPATCH_CH(test_encode_chained_kernel, float, ARGS_CH(float)) }
    else { CDF_DISPATCH_CH(test_encode_chained_kernel, bf16_t, ARGS_CH(bf16_t)) }
    prof_end(K_TEST_ENCODE, st);
#undef ARGS_CH
#undef CDF_DISPATCH_CH
    CDF_LAUNCH_CHECK("test_and_encode/chained");
    return CDF_OK;
  }
  const int nblocks = static_cast<int>(ceil_div(n_rows, kTestRows));
  char* w = static_cast<char*>(ws);
  int* counts = reinterpret_cast<int*>(w);
  int* offsets = counts + scan_stride(nblocks);
  uint8_t* cs = reinterpret_cast<uint8_t*>(w + filter_workspace_bytes(n_rows));
  float* ms = reinterpret_cast<float*>(w + filter_workspace_bytes(n_rows) +
                                       align_up(static_cast<size_t>(n_rows) * static_cast<size_t>(dim), 256));
  const int64_t rb = (static_cast<int64_t>(dim) * bits + 7) / 8;
#define ARGS_F32 <<<nblocks, kQuantThreads, 0, st>>>(static_cast<const float*>(cur), static_cast<float*>(cached), n_rows, \
                 dim, ld, eps, (int)norm, s.glog, (int)commit, delta ? 1 : 0, mask, counts, cs, ms)
#define ARGS_BF16 <<<nblocks, kQuantThreads, 0, st>>>(static_cast<const bf16_t*>(cur), static_cast<bf16_t*>(cached), n_rows, \
                 dim, ld, eps, (int)norm, s.glog, (int)commit, delta ? 1 : 0, mask, counts, cs, ms)
#define CDF_DISPATCH_QQ(K, T, ...)                                                                         \
  if (qs == CDF_Q_MINMAX && bits == 8) { CDF_DISPATCH_EPV(K, T, 8, CDF_Q_MINMAX, s.epv, s.nit, __VA_ARGS__) } \
  else if (qs == CDF_Q_MINMAX) { CDF_DISPATCH_EPV(K, T, 4, CDF_Q_MINMAX, s.epv, s.nit, __VA_ARGS__) }      \
  else if (bits == 8) { CDF_DISPATCH_EPV(K, T, 8, CDF_Q_SYMMETRIC, s.epv, s.nit, __VA_ARGS__) }            \
  else { CDF_DISPATCH_EPV(K, T, 4, CDF_Q_SYMMETRIC, s.epv, s.nit, __VA_ARGS__) }
  prof_begin(K_TEST_ENCODE, st);
  if (dt == CDF_F32) { CDF_DISPATCH_QQ(test_encode_kernel, float, ARGS_F32) }
  else { CDF_DISPATCH_QQ(test_encode_kernel, bf16_t, ARGS_BF16) }
  prof_end(K_TEST_ENCODE, st);
#undef ARGS_F32
#undef ARGS_BF16
#undef CDF_DISPATCH_QQ
  CDF_LAUNCH_CHECK("test_and_encode/encode");
  const int rc = scan_and_compact(mask, n_rows, counts, offsets, idx, n_sent, st);
  if (rc != CDF_OK) return rc;
  {
    ProfScope ps(K_GATHER_CODES, st);
    const unsigned grid = static_cast<unsigned>(std::min<int64_t>(ceil_div(n_rows, 16), kMessageGridCap));
    if (rb % 16 == 0) gather_codes_kernel<uint4><<<grid, 256, 0, st>>>(cs, ms, idx, n_sent, n_rows, rb, codes, meta);
    else if (rb % 4 == 0) gather_codes_kernel<uint32_t><<<grid, 256, 0, st>>>(cs, ms, idx, n_sent, n_rows, rb, codes, meta);
    else gather_codes_kernel<uint8_t><<<grid, 256, 0, st>>>(cs, ms, idx, n_sent, n_rows, rb, codes, meta);
  }
  CDF_LAUNCH_CHECK("test_and_encode/gather");
  return CDF_OK;
}

}  // namespace cdf

extern "C" int cdf_set_message_wait_limit(int polls) {
  cdf::g_chain_spin_limit = polls > 0 ? polls : 1 << 20;
  return CDF_OK;
}

extern "C" int cdf_cache_filter_quantize(const void* cur, void* cached, int32_t n_rows, int32_t dim, int64_t ld,
                                         cdf_dtype dt, float eps, cdf_norm norm, int bits, cdf_qscheme qs,
                                         cdf_commit commit, int delta, uint8_t* mask, int32_t* idx, int32_t* n_sent,
                                         uint8_t* codes, float* meta, void* ws, size_t ws_bytes, void* stream) {
  return cdf::test_and_encode(cur, cached, n_rows, dim, ld, dt, eps, norm, bits, qs, commit, delta, mask, idx, n_sent,
                              codes, meta, ws, ws_bytes, stream);
}
