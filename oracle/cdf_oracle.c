/*
 * CPU oracle for the per-partition GCN layer step of cache-based distributed
 * full-batch training (adaptive vertex cache + linear message quantisation +
 * normalised-adjacency aggregation + dense transform).
 *
 * TEST INFRASTRUCTURE ONLY. This file is the slow, plain statement of what the
 * method computes. It shares no code with the GPU library and is never called
 * by it; only the tests, the smoke check and the benchmark's CPU-baseline leg
 * load it.
 *
 * Every function follows the paper's steps in the paper's order. Where the
 * paper leaves a detail open, the reading taken is stated beside the code.
 *
 * Build: gcc -O2 -ffp-contract=off -fno-fast-math -fopenmp -shared -fPIC
 * (row loops are the only parallel loops; results do not depend on the thread
 * count because each row is computed by one thread in a fixed order).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORC_F32 = 0, ORC_BF16 = 1 };
enum { ORC_NORM_LINF = 0, ORC_NORM_L2 = 1 };
enum { ORC_Q_MINMAX = 0, ORC_Q_SYMMETRIC = 1, ORC_Q_NONE = 2 };
enum { ORC_COMMIT_NONE = 0, ORC_COMMIT_CUR = 1, ORC_COMMIT_DEQ = 2 };

void orc_set_threads(int n) {
#ifdef _OPENMP
  omp_set_num_threads(n > 0 ? n : 1);
#else
  (void)n;
#endif
}

int orc_get_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

/* ---- element access: fp32, or bf16 stored as the upper half of an fp32 ---- */

static float bf16_to_f32(uint16_t b) {
  uint32_t u = (uint32_t)b << 16;
  float f;
  memcpy(&f, &u, 4);
  return f;
}

/* round to nearest, ties to even */
static uint16_t f32_to_bf16(float f) {
  uint32_t u;
  memcpy(&u, &f, 4);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x0040u); /* quiet NaN */
  u += 0x7fffu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}

static float ld(const void* p, int64_t i, int dt) {
  return dt == ORC_BF16 ? bf16_to_f32(((const uint16_t*)p)[i]) : ((const float*)p)[i];
}

static void st(void* p, int64_t i, int dt, float v) {
  if (dt == ORC_BF16) ((uint16_t*)p)[i] = f32_to_bf16(v);
  else ((float*)p)[i] = v;
}

/* ---------------------------------------------------------------------------
 * Adaptive cache test (Alg. 2, the "if" of the mirror loop; Sec. 4.1).
 *
 * For each row r:  send_r = ( ||cur_r - cached_r|| > eps * ||cached_r|| ), strict.
 * The product form of Alg. 2 is used (not the ratio of Sec. 4.1's error measure),
 * so a zero cached row sends on any non-zero difference.
 *
 * Norms:
 *   LINF - the paper's: largest absolute element. Order-independent.
 *   L2   - squared form  sum d^2 > eps^2 * sum c^2  in fp32, whose summation order
 *          is part of the definition: 256 interleaved chains, chain c taking the
 *          elements j = c, c+256, ... in ascending j with one fused multiply-add
 *          each, then a radix-2 butterfly over the chain index with strides
 *          1, 2, 4, ..., 128 (p[c] + p[c ^ stride]).
 *
 * Outputs: mask[r] in {0,1}; idx = ascending rows with mask 1; *n_sent = count.
 * The caches are not modified here.
 * ------------------------------------------------------------------------- */

static float l2_pinned(const float* v, int n) {
  float p[256];
  for (int c = 0; c < 256; ++c) p[c] = 0.0f;
  for (int j = 0; j < n; ++j) p[j & 255] = fmaf(v[j], v[j], p[j & 255]);
  for (int s = 1; s < 256; s <<= 1) {
    float q[256];
    for (int c = 0; c < 256; ++c) q[c] = p[c] + p[c ^ s];
    memcpy(p, q, sizeof p);
  }
  return p[0];
}

int orc_cache_filter(const void* cur, const void* cached, int32_t n_rows, int32_t dim, int64_t ldm,
                     int dt, float eps, int norm, uint8_t* mask, int32_t* idx, int32_t* n_sent) {
  if (n_rows < 0 || dim <= 0 || ldm < dim) return -1;
#pragma omp parallel
  {
    float* d = (float*)malloc(sizeof(float) * (size_t)dim);
    float* c = (float*)malloc(sizeof(float) * (size_t)dim);
#pragma omp for schedule(static)
    for (int32_t r = 0; r < n_rows; ++r) {
      for (int j = 0; j < dim; ++j) {
        float z = ld(cur, r * ldm + j, dt);
        float zc = ld(cached, r * ldm + j, dt);
        d[j] = z - zc;
        c[j] = zc;
      }
      int send;
      if (norm == ORC_NORM_LINF) {
        float D = 0.0f, C = 0.0f;
        for (int j = 0; j < dim; ++j) {
          D = fmaxf(D, fabsf(d[j]));
          C = fmaxf(C, fabsf(c[j]));
        }
        float thr = eps * C;
        send = D > thr;
      } else {
        float D2 = l2_pinned(d, dim);
        float C2 = l2_pinned(c, dim);
        float e2 = eps * eps;
        float thr = e2 * C2;
        send = D2 > thr;
      }
      mask[r] = (uint8_t)send;
    }
    free(d);
    free(c);
  }
  int32_t k = 0;
  for (int32_t r = 0; r < n_rows; ++r)
    if (mask[r]) idx[k++] = r;
  *n_sent = k;
  return 0;
}

/* ---------------------------------------------------------------------------
 * Difference, linear quantisation (Sec. 5, first equation) and cache commit
 * (Alg. 2: "send the difference", then cached <- current).
 *
 * For the k-th listed row r = idx[k]:
 *   m_j = cur[r][j] - cached[r][j]          (delta != 0: the paper's difference message)
 *   m_j = cur[r][j]                         (delta == 0: the row itself; the receiver
 *                                            then replaces instead of adding)
 * MINMAX (the paper's scheme): lo = min m, hi = max m, levels Lv = 2^B - 1
 *   (the printed 2^B would map the maximum to a code that does not fit B bits),
 *   inv = Lv / (hi - lo) by one fp32 division (0 when hi == lo),
 *   q_j = floor( (m_j - lo) * inv + 0.5 ) with the multiply-add fused, clamped to [0, Lv];
 *   meta = (lo, hi).
 * SYMMETRIC: a = max |m|, Qm = 2^(B-1) - 1, inv = Qm / a (0 when a == 0),
 *   q_j = floor( m_j * inv + 0.5 ) clamped to [-Qm, Qm], stored two's complement in B bits;
 *   meta = (a / Qm, 0).
 * NONE: the row's fp32 values are copied as the message (no loss); meta = (0, 0).
 * Packing: row k occupies row_bytes = ceil(dim*B/8) bytes; B = 8 one code per byte;
 *   B = 4 even element in the low nibble, odd element in the high nibble.
 * Commit: CUR: cached[r] <- cur[r] (the paper's rule). DEQ: cached[r] += dequantised
 *   message (= dequantised message when delta == 0), so sender and receiver hold the
 *   same value. NONE: cache untouched.
 * ------------------------------------------------------------------------- */

static int64_t row_bytes_of(int dim, int bits, int qs) {
  if (qs == ORC_Q_NONE) return (int64_t)dim * 4;
  return ((int64_t)dim * bits + 7) / 8;
}

static float deq_minmax(int q, float lo, float scale) { return fmaf((float)q, scale, lo); }

int orc_quantize(const void* cur, void* cached, const int32_t* idx, int32_t n_sent, int32_t dim,
                 int64_t ldm, int dt, int bits, int qs, int commit, int delta, uint8_t* codes,
                 float* meta) {
  if (n_sent < 0 || dim <= 0 || ldm < dim) return -1;
  if (delta && cached == NULL) return -1;
  if (qs != ORC_Q_NONE && bits != 8 && bits != 4) return -2;
  if (commit != ORC_COMMIT_NONE && cached == NULL) return -1;
  const int64_t rb = row_bytes_of(dim, bits, qs);
#pragma omp parallel
  {
    float* m = (float*)malloc(sizeof(float) * (size_t)dim);
    int* q = (int*)malloc(sizeof(int) * (size_t)dim);
#pragma omp for schedule(static)
    for (int32_t k = 0; k < n_sent; ++k) {
      const int64_t r = idx[k];
      uint8_t* out = codes + (int64_t)k * rb;
      for (int j = 0; j < dim; ++j) {
        float z = ld(cur, r * ldm + j, dt);
        m[j] = delta ? z - ld(cached, r * ldm + j, dt) : z;
      }
      float m0 = 0.0f, m1 = 0.0f, scale = 0.0f;
      if (qs == ORC_Q_NONE) {
        memcpy(out, m, (size_t)dim * 4);
      } else if (qs == ORC_Q_MINMAX) {
        const int Lv = (1 << bits) - 1;
        float lo = m[0], hi = m[0];
        for (int j = 1; j < dim; ++j) {
          lo = fminf(lo, m[j]);
          hi = fmaxf(hi, m[j]);
        }
        float range = hi - lo;
        float inv = range > 0.0f ? (float)Lv / range : 0.0f;
        for (int j = 0; j < dim; ++j) {
          float t = floorf(fmaf(m[j] - lo, inv, 0.5f));
          t = fminf(fmaxf(t, 0.0f), (float)Lv); /* clamp before the integer conversion */
          q[j] = (int)t;
        }
        m0 = lo;
        m1 = hi;
        scale = range / (float)Lv;
      } else {
        const int Qm = (1 << (bits - 1)) - 1;
        float a = 0.0f;
        for (int j = 0; j < dim; ++j) a = fmaxf(a, fabsf(m[j]));
        float inv = a > 0.0f ? (float)Qm / a : 0.0f;
        for (int j = 0; j < dim; ++j) {
          float t = floorf(fmaf(m[j], inv, 0.5f));
          t = fminf(fmaxf(t, (float)-Qm), (float)Qm);
          q[j] = (int)t;
        }
        scale = a / (float)Qm;
        m0 = scale;
        m1 = 0.0f;
      }
      if (qs != ORC_Q_NONE) {
        if (bits == 8) {
          for (int j = 0; j < dim; ++j) out[j] = (uint8_t)(q[j] & 0xff);
        } else {
          memset(out, 0, (size_t)rb);
          for (int j = 0; j < dim; ++j) out[j >> 1] |= (uint8_t)((q[j] & 0xf) << (4 * (j & 1)));
        }
      }
      meta[2 * (int64_t)k] = m0;
      meta[2 * (int64_t)k + 1] = m1;
      if (commit == ORC_COMMIT_CUR) {
        for (int j = 0; j < dim; ++j) st(cached, r * ldm + j, dt, ld(cur, r * ldm + j, dt));
      } else if (commit == ORC_COMMIT_DEQ) {
        for (int j = 0; j < dim; ++j) {
          float dq = qs == ORC_Q_NONE ? m[j]
                     : qs == ORC_Q_MINMAX ? deq_minmax(q[j], m0, scale)
                                          : (float)q[j] * scale;
          float old = delta ? ld(cached, r * ldm + j, dt) : 0.0f;
          st(cached, r * ldm + j, dt, delta ? old + dq : dq);
        }
      }
    }
    free(m);
    free(q);
  }
  return 0;
}

/* ---------------------------------------------------------------------------
 * Recovery (Sec. 5, second equation) and the receiver's update of the value it
 * aggregates with (Alg. 2, message loop: cached_total <- cached_total + delta).
 *
 * MINMAX: scale = (hi - lo) / Lv (one fp32 division), m~_j = q_j * scale + lo (fused).
 * SYMMETRIC: m~_j = q_j * scale with scale = meta[0], q_j sign-extended from B bits.
 * NONE: m~_j is the stored fp32 value.
 * accumulate != 0: dst[idx[k]][j] += m~_j (fp32 add, then rounded to the storage type);
 * accumulate == 0: dst[idx[k]][j]  = m~_j.
 * ------------------------------------------------------------------------- */
int orc_dequantize(const uint8_t* codes, const float* meta, const int32_t* idx, int32_t n_sent,
                   int32_t dim, int bits, int qs, void* dst, int64_t ldm, int dt, int accumulate) {
  if (n_sent < 0 || dim <= 0 || ldm < dim) return -1;
  if (qs != ORC_Q_NONE && bits != 8 && bits != 4) return -2;
  const int64_t rb = row_bytes_of(dim, bits, qs);
#pragma omp parallel for schedule(static)
  for (int32_t k = 0; k < n_sent; ++k) {
    const int64_t r = idx[k];
    const uint8_t* in = codes + (int64_t)k * rb;
    const float m0 = meta[2 * (int64_t)k], m1 = meta[2 * (int64_t)k + 1];
    float scale = 0.0f;
    if (qs == ORC_Q_MINMAX) scale = (m1 - m0) / (float)((1 << bits) - 1);
    if (qs == ORC_Q_SYMMETRIC) scale = m0;
    for (int j = 0; j < dim; ++j) {
      float v;
      if (qs == ORC_Q_NONE) {
        memcpy(&v, in + 4 * (int64_t)j, 4);
      } else {
        int q = bits == 8 ? in[j] : (in[j >> 1] >> (4 * (j & 1))) & 0xf;
        if (qs == ORC_Q_MINMAX) {
          v = deq_minmax(q, m0, scale);
        } else {
          int sign = 1 << (bits - 1);
          q = (q ^ sign) - sign; /* sign-extend */
          v = (float)q * scale;
        }
      }
      if (accumulate) v = ld(dst, r * ldm + j, dt) + v;
      st(dst, r * ldm + j, dt, v);
    }
  }
  return 0;
}

/* ---------------------------------------------------------------------------
 * Aggregation over the normalised adjacency (Sec. 3.1, first equation, the
 * product A^_i H):  Y[i][j] = sum over stored entries k of row i of
 * vals[k] * X[colidx[k]][j], accumulated in double in storage order and rounded
 * once to the output type. The transposed product used by back-propagation is
 * the same routine on the transposed CSR.
 * ------------------------------------------------------------------------- */
int orc_spmm(int32_t n_rows, int32_t n_cols, const int64_t* rowptr, const int32_t* colidx,
             const float* vals, const void* X, int64_t ldx, void* Y, int64_t ldy, int32_t dim, int dt) {
  if (n_rows < 0 || dim <= 0 || ldx < dim || ldy < dim) return -1;
#pragma omp parallel
  {
    double* acc = (double*)malloc(sizeof(double) * (size_t)dim);
#pragma omp for schedule(dynamic, 64)
    for (int32_t i = 0; i < n_rows; ++i) {
      for (int j = 0; j < dim; ++j) acc[j] = 0.0;
      for (int64_t k = rowptr[i]; k < rowptr[i + 1]; ++k) {
        const int64_t c = colidx[k];
        if (c < 0 || c >= n_cols) continue; /* malformed input: ignored, never read */
        const double a = (double)vals[k];
        for (int j = 0; j < dim; ++j) acc[j] += a * (double)ld(X, c * ldx + j, dt);
      }
      for (int j = 0; j < dim; ++j) st(Y, (int64_t)i * ldy + j, dt, (float)acc[j]);
    }
    free(acc);
  }
  return 0;
}

/* ---------------------------------------------------------------------------
 * Dense transform and its gradients (Sec. 3.1: Z = (A^ H) W, H' = sigma(Z);
 * back-propagation by the chain rule with sigma = ReLU, sigma'(0) = 0).
 * All sums in double in index order; one rounding to fp32 at the end.
 *   fwd : Z = M W,  H = relu ? max(Z, 0) : Z
 *   bwd : dZ = relu ? dH * [Z > 0] : dH ;  dW = M^T dZ ;  dM = dZ W^T
 * M is n x f (type dt), W is f x g fp32, Z/H/dH are n x g fp32, dM is n x f (type dt).
 * ------------------------------------------------------------------------- */
int orc_dense_fwd(const void* M, int64_t ldm, int dt, const float* W, int32_t n, int32_t f, int32_t g,
                  int relu, float* Z, float* H) {
#pragma omp parallel
  {
    double* acc = (double*)malloc(sizeof(double) * (size_t)g);
#pragma omp for schedule(static)
    for (int32_t i = 0; i < n; ++i) {
      for (int c = 0; c < g; ++c) acc[c] = 0.0;
      for (int k = 0; k < f; ++k) {
        const double a = (double)ld(M, (int64_t)i * ldm + k, dt);
        for (int c = 0; c < g; ++c) acc[c] += a * (double)W[(int64_t)k * g + c];
      }
      for (int c = 0; c < g; ++c) {
        float z = (float)acc[c];
        if (Z) Z[(int64_t)i * g + c] = z;
        if (H) H[(int64_t)i * g + c] = relu ? (z > 0.0f ? z : 0.0f) : z;
      }
    }
    free(acc);
  }
  return 0;
}

int orc_dense_bwd(const void* M, int64_t ldm, int dt, const float* W, const float* Z, const float* dH,
                  int32_t n, int32_t f, int32_t g, int relu, float* dW, void* dM, int64_t lddm) {
  /* dW[k][c] = sum_i M[i][k] * dZ[i][c] : one (k) row per iteration, rows of M/dZ in ascending i */
#pragma omp parallel
  {
    double* acc = (double*)malloc(sizeof(double) * (size_t)g);
#pragma omp for schedule(static)
    for (int32_t k = 0; k < f; ++k) {
      for (int c = 0; c < g; ++c) acc[c] = 0.0;
      for (int32_t i = 0; i < n; ++i) {
        const double a = (double)ld(M, (int64_t)i * ldm + k, dt);
        for (int c = 0; c < g; ++c) {
          float dz = dH[(int64_t)i * g + c];
          if (relu && !(Z[(int64_t)i * g + c] > 0.0f)) dz = 0.0f;
          acc[c] += a * (double)dz;
        }
      }
      for (int c = 0; c < g; ++c) dW[(int64_t)k * g + c] = (float)acc[c];
    }
    free(acc);
  }
  if (dM) {
#pragma omp parallel for schedule(static)
    for (int32_t i = 0; i < n; ++i) {
      for (int k = 0; k < f; ++k) {
        double s = 0.0;
        for (int c = 0; c < g; ++c) {
          float dz = dH[(int64_t)i * g + c];
          if (relu && !(Z[(int64_t)i * g + c] > 0.0f)) dz = 0.0f;
          s += (double)dz * (double)W[(int64_t)k * g + c];
        }
        st(dM, (int64_t)i * lddm + k, dt, (float)s);
      }
    }
  }
  return 0;
}

/* ---------------------------------------------------------------------------
 * Pieces of the training loop around the layer step (Sec. 7.1: cross-entropy loss, Adam
 * with learning rate 0.01; Sec. 3.1: the loss is taken on owned (master) vertices only;
 * Sec. 4.1, last two equations: the threshold controller).
 * ------------------------------------------------------------------------- */

/* Softmax cross-entropy over the rows with label >= 0 (rows with a negative label are not
 * in the loss: not owned, or not in the training set).
 *   loss_sum  = sum_r -log softmax(z_r)[y_r]
 *   dlogits_r = scale * (softmax(z_r) - onehot(y_r)), zero on skipped rows
 *   n_correct = rows whose largest logit (lowest index on ties) is the label
 * All in double, rounded once. */
int orc_softmax_xent(const float* logits, const int32_t* labels, int32_t n, int32_t classes, float scale,
                     float* dlogits, double* loss_sum, int64_t* n_correct, int64_t* n_labelled) {
  double loss = 0.0;
  int64_t correct = 0, labelled = 0;
  for (int32_t r = 0; r < n; ++r) {
    const float* z = logits + (int64_t)r * classes;
    float* g = dlogits + (int64_t)r * classes;
    const int y = labels[r];
    if (y < 0 || y >= classes) {
      for (int c = 0; c < classes; ++c) g[c] = 0.0f;
      continue;
    }
    int arg = 0;
    for (int c = 1; c < classes; ++c)
      if (z[c] > z[arg]) arg = c;
    double mx = (double)z[arg], s = 0.0;
    for (int c = 0; c < classes; ++c) s += exp((double)z[c] - mx);
    loss += log(s) - ((double)z[y] - mx);
    for (int c = 0; c < classes; ++c) {
      double p = exp((double)z[c] - mx) / s;
      g[c] = (float)((double)scale * (p - (c == y ? 1.0 : 0.0)));
    }
    correct += arg == y;
    ++labelled;
  }
  *loss_sum = loss;
  *n_correct = correct;
  *n_labelled = labelled;
  return 0;
}

/* One Adam step (Kingma & Ba): m <- b1 m + (1-b1) g ; v <- b2 v + (1-b2) g^2 ;
 * W <- W - lr * (m / (1 - b1^t)) / (sqrt(v / (1 - b2^t)) + eps),  t = 1, 2, ...  */
int orc_adam_step(float* W, const float* dW, float* m, float* v, int64_t count, float lr, float b1, float b2,
                  float eps, int32_t t) {
  const double c1 = 1.0 - pow((double)b1, (double)t), c2 = 1.0 - pow((double)b2, (double)t);
  for (int64_t i = 0; i < count; ++i) {
    const double g = (double)dW[i];
    const double mi = (double)b1 * (double)m[i] + (1.0 - (double)b1) * g;
    const double vi = (double)b2 * (double)v[i] + (1.0 - (double)b2) * g * g;
    m[i] = (float)mi;
    v[i] = (float)vi;
    W[i] = (float)((double)W[i] - (double)lr * (mi / c1) / (sqrt(vi / c2) + (double)eps));
  }
  return 0;
}

/* Threshold controller (Sec. 4.1, the case equation and the moving average), fp32.
 * params = { mu1, mu2, nu1, nu2, xi, lambda1, lambda2 }.
 *   acc < mean - mu1 and eps < nu1 :  eps <- min(lambda1 * eps, eps + xi)
 *   acc > mean + mu2 and eps > nu2 :  eps <- max(lambda2 * eps, eps - xi)
 *   otherwise unchanged;  then  mean <- 0.8 * mean + 0.2 * acc.
 * The accuracy is compared with the average of the epochs before it (the paper does not
 * say whether the average is updated first). swap != 0 exchanges the two conditions
 * (the prose of Sec. 4.1 describes relaxing on a large gain and tightening on a small
 * loss, the opposite of the printed cases). */
float orc_eps_update(float eps, float acc, float* mean_acc, const float* params, int swap) {
  const float mu1 = params[0], mu2 = params[1], nu1 = params[2], nu2 = params[3], xi = params[4];
  const float l1 = params[5], l2 = params[6];
  const float mean = *mean_acc;
  const int below = acc < mean - mu1, above = acc > mean + mu2;
  const int grow = swap ? above : below, shrink = swap ? below : above;
  float out = eps;
  if (grow && eps < nu1) {
    const float a = l1 * eps, b = eps + xi;
    out = a < b ? a : b;
  } else if (shrink && eps > nu2) {
    const float a = l2 * eps, b = eps - xi;
    out = a > b ? a : b;
  }
  *mean_acc = 0.8f * mean + 0.2f * acc;
  return out;
}
