// Pieces of the training loop around the layer step: softmax cross-entropy on labelled rows
// (Sec. 7.1; Sec. 3.1: the loss is taken on owned vertices only), the Adam update (Sec. 7.1),
// an in-place accumulate, and the threshold controller of Sec. 4.1 (host arithmetic).
#include <math.h>

#include "cdf_common.h"

namespace cdf {

constexpr int kXentThreads = 256;
constexpr int kXentRowsPerBlock = 64;  // 16 rows per wavefront

// One row per group of G = 2^glog lanes (lane j takes classes j, j+G, ...). Three passes over the
// row (max + argmax, sum of exponentials, gradient); the row stays in L1 between them.
__global__ __launch_bounds__(kXentThreads) void xent_kernel(const float* __restrict__ logits,
                                                            const int* __restrict__ labels, int n, int classes,
                                                            float scale, int glog, float* __restrict__ dlogits,
                                                            float* __restrict__ block_loss,
                                                            int* __restrict__ block_counts) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int G = 1 << glog, lg = lane & (G - 1), sub = lane >> glog;
  const int rows_per_step = 64 >> glog;
  constexpr int kRowsPerWave = kXentRowsPerBlock / (kXentThreads / 64);
  const int row0 = blockIdx.x * kXentRowsPerBlock + wave * kRowsPerWave;
  float loss = 0.0f;
  int correct = 0, labelled = 0;
  for (int s = 0; s < kRowsPerWave; s += rows_per_step) {
    const int row = row0 + s + sub;
    const bool live = row < n && s + sub < kRowsPerWave;
    const int y = live ? labels[row] : -1;
    const bool on = live && y >= 0 && y < classes;
    const float* z = logits + static_cast<int64_t>(live ? row : 0) * classes;
    float* g = dlogits + static_cast<int64_t>(live ? row : 0) * classes;
    // largest logit and its lowest index
    float mx = -__builtin_inff();
    int arg = 0x7fffffff;
    if (on)
      for (int c = lg; c < classes; c += G) {
        const float v = z[c];
        if (v > mx) { mx = v; arg = c; }
      }
    for (int off = 1; off < G; off <<= 1) {
      const float om = __shfl_xor(mx, off, kWave);
      const int oa = __shfl_xor(arg, off, kWave);
      if (om > mx || (om == mx && oa < arg)) { mx = om; arg = oa; }
    }
    float sum = 0.0f;
    if (on)
      for (int c = lg; c < classes; c += G) sum += expf(z[c] - mx);
    sum = group_sum(sum, G);
    if (on) {
      const float inv = 1.0f / sum;
      for (int c = lg; c < classes; c += G) {
        const float p = expf(z[c] - mx) * inv;
        g[c] = scale * (p - (c == y ? 1.0f : 0.0f));
      }
      if (lg == 0) {
        loss += logf(sum) - (z[y] - mx);
        correct += arg == y;
        ++labelled;
      }
    } else if (live) {
      for (int c = lg; c < classes; c += G) g[c] = 0.0f;
    }
  }
  // block totals in a fixed order: lanes of a wavefront by butterfly, wavefronts in index order
  loss = group_sum(loss, 64);
  for (int off = 1; off < 64; off <<= 1) {
    correct += __shfl_xor(correct, off, kWave);
    labelled += __shfl_xor(labelled, off, kWave);
  }
  __shared__ float sl[kXentThreads / 64];
  __shared__ int sc[kXentThreads / 64], sn[kXentThreads / 64];
  if (lane == 0) { sl[wave] = loss; sc[wave] = correct; sn[wave] = labelled; }
  __syncthreads();
  if (threadIdx.x == 0) {
    float tl = 0.0f;
    int tc = 0, tn = 0;
    for (int w = 0; w < kXentThreads / 64; ++w) { tl += sl[w]; tc += sc[w]; tn += sn[w]; }
    block_loss[blockIdx.x] = tl;
    block_counts[2 * blockIdx.x] = tc;
    block_counts[2 * blockIdx.x + 1] = tn;
  }
}

// One block adds the block totals in index order (double for the loss).
__global__ __launch_bounds__(1024) void xent_final_kernel(const float* __restrict__ block_loss,
                                                          const int* __restrict__ block_counts, int nblocks,
                                                          float* __restrict__ loss_sum, int* __restrict__ counts) {
  __shared__ double dl[1024];
  __shared__ int dc[1024], dn[1024];
  double l = 0.0;
  int c = 0, m = 0;
  for (int i = threadIdx.x; i < nblocks; i += 1024) {
    l += static_cast<double>(block_loss[i]);
    c += block_counts[2 * i];
    m += block_counts[2 * i + 1];
  }
  dl[threadIdx.x] = l; dc[threadIdx.x] = c; dn[threadIdx.x] = m;
  __syncthreads();
  for (int off = 512; off > 0; off >>= 1) {
    if (threadIdx.x < off) {
      dl[threadIdx.x] += dl[threadIdx.x + off];
      dc[threadIdx.x] += dc[threadIdx.x + off];
      dn[threadIdx.x] += dn[threadIdx.x + off];
    }
    __syncthreads();
  }
  if (threadIdx.x == 0) {
    *loss_sum = static_cast<float>(dl[0]);
    counts[0] = dc[0];
    counts[1] = dn[0];
  }
}

__global__ __launch_bounds__(256) void adam_kernel(float* __restrict__ W, const float* __restrict__ dW,
                                                   float* __restrict__ m, float* __restrict__ v, int64_t count,
                                                   float lr, float b1, float b2, float eps, float inv_c1,
                                                   float inv_c2) {
  for (int64_t i = blockIdx.x * static_cast<int64_t>(blockDim.x) + threadIdx.x; i < count;
       i += static_cast<int64_t>(gridDim.x) * blockDim.x) {
    const float g = dW[i];
    const float mi = b1 * m[i] + (1.0f - b1) * g;
    const float vi = b2 * v[i] + (1.0f - b2) * g * g;
    m[i] = mi;
    v[i] = vi;
    W[i] = W[i] - lr * (mi * inv_c1) / (sqrtf(vi * inv_c2) + eps);
  }
}

__global__ __launch_bounds__(256) void accumulate_kernel(float* __restrict__ dst, const float* __restrict__ src,
                                                         int64_t count) {
  for (int64_t i = blockIdx.x * static_cast<int64_t>(blockDim.x) + threadIdx.x; i < count;
       i += static_cast<int64_t>(gridDim.x) * blockDim.x)
    dst[i] = dst[i] + src[i];
}

// dst row r = src row idx[r], moved in units of U bytes (the widest that divides the row and both
// leading dimensions). Stands in for the network between partitions stepped on one device.
template <typename U>
__global__ __launch_bounds__(256) void gather_rows_kernel(const U* __restrict__ src, int64_t ld_src,
                                                          const int* __restrict__ idx, int n, int units,
                                                          U* __restrict__ dst, int64_t ld_dst) {
  const int64_t total = static_cast<int64_t>(n) * units;
  for (int64_t i = blockIdx.x * static_cast<int64_t>(blockDim.x) + threadIdx.x; i < total;
       i += static_cast<int64_t>(gridDim.x) * blockDim.x) {
    const int r = static_cast<int>(i / units), c = static_cast<int>(i - static_cast<int64_t>(r) * units);
    dst[r * ld_dst + c] = src[idx[r] * ld_src + c];
  }
}

__global__ __launch_bounds__(256) void map_index_kernel(const int* __restrict__ idx, const int* __restrict__ n_sent,
                                                        int max_sent, const int* __restrict__ map,
                                                        int* __restrict__ out) {
  int n = *n_sent;
  n = n < max_sent ? n : max_sent;
  for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < n; i += gridDim.x * blockDim.x) out[i] = map[idx[i]];
}

__global__ __launch_bounds__(256) void mark_rows_kernel(const int* __restrict__ idx, const int* __restrict__ n_sent,
                                                        int max_sent, const int* __restrict__ map, int offset,
                                                        uint8_t* __restrict__ flags) {
  int n = *n_sent;
  n = n < max_sent ? n : max_sent;
  for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < n; i += gridDim.x * blockDim.x)
    flags[(map ? map[idx[i]] : idx[i]) + offset] = 1;
}

__global__ __launch_bounds__(256) void relu_kernel(const float* __restrict__ z, float* __restrict__ h, int64_t count) {
  for (int64_t i = blockIdx.x * static_cast<int64_t>(blockDim.x) + threadIdx.x; i < count;
       i += static_cast<int64_t>(gridDim.x) * blockDim.x)
    h[i] = fmaxf(z[i], 0.0f);
}

static unsigned grid_for(int64_t count) {
  const int64_t b = ceil_div(count, 256);
  return static_cast<unsigned>(b < 1 ? 1 : (b > 65536 ? 65536 : b));
}

}  // namespace cdf

using namespace cdf;

extern "C" int cdf_softmax_xent(const float* logits, const int32_t* labels, int32_t n, int32_t classes, float scale,
                                float* dlogits, float* loss_sum, int32_t* counts, void* ws, size_t ws_bytes,
                                void* stream) {
  hipStream_t st = static_cast<hipStream_t>(stream);
  CDF_REQUIRE(n >= 0 && classes > 0, "cdf_softmax_xent: bad shape n=%d classes=%d", n, classes);
  CDF_REQUIRE(loss_sum && counts, "cdf_softmax_xent: null result pointer");
  CDF_REQUIRE(n == 0 || (logits && labels && dlogits), "cdf_softmax_xent: null pointer");
  const int nblocks = static_cast<int>(ceil_div(n, kXentRowsPerBlock));
  const size_t need = align_up(static_cast<size_t>(nblocks > 0 ? nblocks : 1) * 12, 256);
  if (!ws || !aligned(ws, 8) || ws_bytes < need)
    CDF_FAIL(CDF_ERR_WORKSPACE, "cdf_softmax_xent: workspace too small (%zu < %zu)", ws_bytes, need);
  float* bl = static_cast<float*>(ws);
  int* bc = reinterpret_cast<int*>(bl + (nblocks > 0 ? nblocks : 1));
  if (n > 0) {
    const int glog = classes >= 64 ? 6 : log2_ceil(classes);
    xent_kernel<<<nblocks, kXentThreads, 0, st>>>(logits, labels, n, classes, scale, glog, dlogits, bl, bc);
    CDF_LAUNCH_CHECK("cdf_softmax_xent");
  }
  xent_final_kernel<<<1, 1024, 0, st>>>(bl, bc, nblocks, loss_sum, counts);
  CDF_LAUNCH_CHECK("cdf_softmax_xent/final");
  return CDF_OK;
}

extern "C" int cdf_adam_step(float* W, const float* dW, float* m, float* v, int64_t count, float lr, float beta1,
                             float beta2, float eps, int32_t t, void* stream) {
  CDF_REQUIRE(count >= 0 && t >= 1, "cdf_adam_step: bad count or step");
  CDF_REQUIRE(beta1 >= 0.0f && beta1 < 1.0f && beta2 >= 0.0f && beta2 < 1.0f, "cdf_adam_step: betas must be in [0, 1)");
  if (count == 0) return CDF_OK;
  CDF_REQUIRE(W && dW && m && v, "cdf_adam_step: null pointer");
  const double c1 = 1.0 - pow(static_cast<double>(beta1), static_cast<double>(t));
  const double c2 = 1.0 - pow(static_cast<double>(beta2), static_cast<double>(t));
  adam_kernel<<<grid_for(count), 256, 0, static_cast<hipStream_t>(stream)>>>(
      W, dW, m, v, count, lr, beta1, beta2, eps, static_cast<float>(1.0 / c1), static_cast<float>(1.0 / c2));
  CDF_LAUNCH_CHECK("cdf_adam_step");
  return CDF_OK;
}

extern "C" int cdf_accumulate(float* dst, const float* src, int64_t count, void* stream) {
  CDF_REQUIRE(count >= 0, "cdf_accumulate: negative count");
  if (count == 0) return CDF_OK;
  CDF_REQUIRE(dst && src, "cdf_accumulate: null pointer");
  accumulate_kernel<<<grid_for(count), 256, 0, static_cast<hipStream_t>(stream)>>>(dst, src, count);
  CDF_LAUNCH_CHECK("cdf_accumulate");
  return CDF_OK;
}

extern "C" int cdf_gather_rows(const void* src, int64_t ld_src, const int32_t* idx, int32_t n, int32_t dim,
                               cdf_dtype dt, void* dst, int64_t ld_dst, void* stream) {
  CDF_REQUIRE(n >= 0 && dim > 0, "cdf_gather_rows: bad shape n=%d dim=%d", n, dim);
  CDF_REQUIRE(dt == CDF_F32 || dt == CDF_BF16, "cdf_gather_rows: unknown element type %d", static_cast<int>(dt));
  CDF_REQUIRE(ld_src >= dim && ld_dst >= dim, "cdf_gather_rows: leading dimension below the row width");
  if (n == 0) return CDF_OK;
  CDF_REQUIRE(src && idx && dst, "cdf_gather_rows: null pointer");
  const size_t es = dt == CDF_F32 ? 4 : 2;
  const size_t rb = dim * es, lsb = static_cast<size_t>(ld_src) * es, ldb = static_cast<size_t>(ld_dst) * es;
  const uintptr_t bits = reinterpret_cast<uintptr_t>(src) | reinterpret_cast<uintptr_t>(dst) | rb | lsb | ldb;
  hipStream_t st = static_cast<hipStream_t>(stream);
#define CDF_GATHER(U)                                                                                      \
  gather_rows_kernel<U><<<grid_for(static_cast<int64_t>(n) * (rb / sizeof(U))), 256, 0, st>>>(             \
      static_cast<const U*>(src), static_cast<int64_t>(lsb / sizeof(U)), idx, n, static_cast<int>(rb / sizeof(U)), \
      static_cast<U*>(dst), static_cast<int64_t>(ldb / sizeof(U)))
  if (bits % 16 == 0) CDF_GATHER(uint4);
  else if (bits % 8 == 0) CDF_GATHER(uint2);
  else if (bits % 4 == 0) CDF_GATHER(uint32_t);
  else CDF_GATHER(uint16_t);
#undef CDF_GATHER
  CDF_LAUNCH_CHECK("cdf_gather_rows");
  return CDF_OK;
}

extern "C" int cdf_map_index(const int32_t* idx, const int32_t* n_sent, int32_t max_sent, const int32_t* map,
                             int32_t* out, void* stream) {
  CDF_REQUIRE(max_sent >= 0, "cdf_map_index: negative capacity");
  if (max_sent == 0) return CDF_OK;
  CDF_REQUIRE(idx && n_sent && map && out, "cdf_map_index: null pointer");
  map_index_kernel<<<grid_for(max_sent), 256, 0, static_cast<hipStream_t>(stream)>>>(idx, n_sent, max_sent, map, out);
  CDF_LAUNCH_CHECK("cdf_map_index");
  return CDF_OK;
}

extern "C" int cdf_mark_rows(const int32_t* idx, const int32_t* n_sent, int32_t max_sent, const int32_t* map,
                             int32_t offset, uint8_t* flags, void* stream) {
  CDF_REQUIRE(max_sent >= 0, "cdf_mark_rows: negative capacity");
  if (max_sent == 0) return CDF_OK;
  CDF_REQUIRE(idx && n_sent && flags, "cdf_mark_rows: null pointer");
  mark_rows_kernel<<<grid_for(max_sent), 256, 0, static_cast<hipStream_t>(stream)>>>(idx, n_sent, max_sent, map, offset,
                                                                                     flags);
  CDF_LAUNCH_CHECK("cdf_mark_rows");
  return CDF_OK;
}

extern "C" int cdf_relu_fwd(const float* z, float* h, int64_t count, void* stream) {
  CDF_REQUIRE(count >= 0, "cdf_relu_fwd: negative count");
  if (count == 0) return CDF_OK;
  CDF_REQUIRE(z && h, "cdf_relu_fwd: null pointer");
  relu_kernel<<<grid_for(count), 256, 0, static_cast<hipStream_t>(stream)>>>(z, h, count);
  CDF_LAUNCH_CHECK("cdf_relu_fwd");
  return CDF_OK;
}

extern "C" float cdf_eps_update(float eps, float acc, float* mean_acc, const cdf_eps_params* p) {
  static const cdf_eps_params dflt = {0.001f, 0.02f, 0.3f, 0.001f, 0.01f, 1.05f, 0.9f, 0};
  if (!p) p = &dflt;
  const float mean = mean_acc ? *mean_acc : acc;
  const bool below = acc < mean - p->mu1, above = acc > mean + p->mu2;
  const bool grow = p->swap_conditions ? above : below, shrink = p->swap_conditions ? below : above;
  float out = eps;
  if (grow && eps < p->nu1) {
    const float a = p->lambda1 * eps, b = eps + p->xi;
    out = a < b ? a : b;
  } else if (shrink && eps > p->nu2) {
    const float a = p->lambda2 * eps, b = eps - p->xi;
    out = a > b ? a : b;
  }
  if (mean_acc) *mean_acc = 0.8f * mean + 0.2f * acc;
  return out;
}
