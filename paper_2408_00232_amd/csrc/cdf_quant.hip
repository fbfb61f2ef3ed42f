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
#include "cdf_common.h"

namespace cdf {

constexpr int kQuantThreads = 256;

// `NIT` vectors of EPV elements per lane: covers rows of up to 64*NIT vectors.
template <typename T, int EPV, int NIT, int BITS, int QS>
__global__ __launch_bounds__(kQuantThreads) void quantize_kernel(
    const T* __restrict__ cur, T* cached, const int* __restrict__ idx, const int* __restrict__ n_sent_p,
    int dim, int64_t ld, int glog, int commit, int delta, uint8_t* __restrict__ codes,
    float* __restrict__ meta) {
  const int n_sent = *n_sent_p;
  const int lane = threadIdx.x & 63;
  const int G = 1 << glog;
  const int lg = lane & (G - 1);
  const int rows_per_wave = 64 >> glog;
  const int gwave = blockIdx.x * (kQuantThreads / 64) + (threadIdx.x >> 6);
  const int k = gwave * rows_per_wave + (lane >> glog);
  const bool live = k < n_sent;
  const int nvec = dim / EPV;
  const int64_t rb = QS == CDF_Q_NONE ? static_cast<int64_t>(dim) * 4 : (static_cast<int64_t>(dim) * BITS + 7) / 8;

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
    meta[2 * static_cast<int64_t>(k)] = m0;
    meta[2 * static_cast<int64_t>(k) + 1] = m1;
  }

  uint8_t* out = codes + static_cast<int64_t>(live ? k : 0) * rb;
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

template <typename T, int EPV, int NIT, int BITS, int QS>
__global__ __launch_bounds__(kQuantThreads) void dequantize_kernel(
    const uint8_t* __restrict__ codes, const float* __restrict__ meta, const int* __restrict__ idx,
    const int* __restrict__ n_sent_p, int dim, int glog, T* dst, int64_t ld, int accumulate) {
  const int n_sent = *n_sent_p;
  const int lane = threadIdx.x & 63;
  const int G = 1 << glog;
  const int lg = lane & (G - 1);
  const int rows_per_wave = 64 >> glog;
  const int gwave = blockIdx.x * (kQuantThreads / 64) + (threadIdx.x >> 6);
  const int k = gwave * rows_per_wave + (lane >> glog);
  if (k >= n_sent) return;
  const int nvec = dim / EPV;
  const int64_t rb = QS == CDF_Q_NONE ? static_cast<int64_t>(dim) * 4 : (static_cast<int64_t>(dim) * BITS + 7) / 8;
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

}  // namespace cdf

using namespace cdf;

extern "C" size_t cdf_code_row_bytes(int32_t dim, int bits, cdf_qscheme qs) {
  if (dim <= 0) return 0;
  if (qs == CDF_Q_NONE) return static_cast<size_t>(dim) * 4;
  return (static_cast<size_t>(dim) * bits + 7) / 8;
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
  const int nblocks = static_cast<int>(ceil_div(max_sent, rows_per_block));
#define ARGS_F32 <<<nblocks, kQuantThreads, 0, st>>>(static_cast<const float*>(cur), static_cast<float*>(cached), \
                 idx, n_sent, dim, ld, s.glog, (int)commit, delta ? 1 : 0, codes, meta)
#define ARGS_BF16 <<<nblocks, kQuantThreads, 0, st>>>(static_cast<const bf16_t*>(cur), static_cast<bf16_t*>(cached), \
                 idx, n_sent, dim, ld, s.glog, (int)commit, delta ? 1 : 0, codes, meta)
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
  const int nblocks = static_cast<int>(ceil_div(max_sent, rows_per_block));
#define ARGS_F32 <<<nblocks, kQuantThreads, 0, st>>>(codes, meta, idx, n_sent, dim, s.glog, static_cast<float*>(dst), \
                 ld, accumulate ? 1 : 0)
#define ARGS_BF16 <<<nblocks, kQuantThreads, 0, st>>>(codes, meta, idx, n_sent, dim, s.glog, static_cast<bf16_t*>(dst), \
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
