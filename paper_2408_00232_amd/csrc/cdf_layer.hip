// The per-partition layer step (Alg. 1 with Alg. 2 and Sec. 5 on the rows that cross the
// partition boundary): host-side sequencing of the kernels on one stream, workspace
// partitioning, and the error text.
#include <stdarg.h>

#include "cdf_common.h"

namespace cdf {

size_t filter_workspace_bytes(int64_t n_rows);
size_t spmm_workspace_bytes(int64_t nnz, int32_t dim);
size_t dense_workspace_bytes(int64_t n, int32_t f, int32_t g);
size_t test_encode_workspace_bytes(int64_t n_rows, int32_t dim);
int dense_fwd_ws(const void* M, int64_t ldm, cdf_dtype dt, const float* W, int32_t n, int32_t f_in, int32_t f_out,
                 int relu, float* Z, float* H, void* ws, size_t ws_bytes, void* stream);
int test_and_encode(const void* cur, void* cached, int32_t n_rows, int32_t dim, int64_t ld, cdf_dtype dt, float eps,
                    cdf_norm norm, int bits, cdf_qscheme qs, cdf_commit commit, int delta, uint8_t* mask, int32_t* idx,
                    int32_t* n_sent, uint8_t* codes, float* meta, void* ws, size_t ws_bytes, void* stream);
int spmm_run(const char* fn, const cdf_csr* A, const void* X, int64_t ldx, void* Y, void* Y2, int64_t ldy,
             int32_t dim, cdf_dtype dt, void* ws, size_t ws_bytes, hipStream_t st);

// dZ = dH where Zs > 0, else 0 (16 bytes per lane; count is a multiple of 4 or the tail is scalar)
__global__ __launch_bounds__(256) void relu_mask_kernel(const float* __restrict__ dH, const float* __restrict__ Zs,
                                                        float* __restrict__ dZ, int64_t count) {
  const int64_t stride = static_cast<int64_t>(gridDim.x) * blockDim.x;
  const int64_t quads = count / 4;
  for (int64_t i = blockIdx.x * static_cast<int64_t>(blockDim.x) + threadIdx.x; i < quads; i += stride) {
    const float4 g = reinterpret_cast<const float4*>(dH)[i];
    const float4 z = reinterpret_cast<const float4*>(Zs)[i];
    reinterpret_cast<float4*>(dZ)[i] =
        make_float4(z.x > 0.0f ? g.x : 0.0f, z.y > 0.0f ? g.y : 0.0f, z.z > 0.0f ? g.z : 0.0f, z.w > 0.0f ? g.w : 0.0f);
  }
  for (int64_t i = quads * 4 + blockIdx.x * static_cast<int64_t>(blockDim.x) + threadIdx.x; i < count; i += stride)
    dZ[i] = Zs[i] > 0.0f ? dH[i] : 0.0f;
}

static thread_local char g_err[512] = "";

void set_error(const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof g_err, fmt, ap);
  va_end(ap);
}

static size_t max_sz(size_t a, size_t b) { return a > b ? a : b; }

// ---- per-kernel timing: one (start, stop) event pair per launch, kept in launch order ----
static const char* const kKernelNames[K_COUNT] = {
    "filter_kernel", "scan_kernel", "compact_kernel", "quantize_kernel", "dequantize_kernel",
    "chunk_rows_kernel", "spmm_kernel", "spmm_fixup_kernel", "gemm_kernel<FWD>", "gemm_kernel<DW>",
    "reduce_slabs_kernel", "gemm_kernel<DM>", "spmm_sliced_kernel", "relu_mask_kernel", "test_encode_kernel",
    "gather_codes_kernel", "spmm_kernel<transform>"};
constexpr int kProfCap = 8192;
struct ProfRec {
  int id;
  hipEvent_t a, b;
};
static bool g_prof_on = false;
static ProfRec g_prof[kProfCap];
static int g_prof_n = 0;      // records in use
static int g_prof_made = 0;   // records whose events exist (reused across sessions)

void prof_begin(int id, hipStream_t st) {
  if (!g_prof_on || g_prof_n >= kProfCap) return;
  ProfRec& r = g_prof[g_prof_n];
  if (g_prof_n >= g_prof_made) {
    if (hipEventCreate(&r.a) != hipSuccess || hipEventCreate(&r.b) != hipSuccess) {
      g_prof_on = false;
      return;
    }
    g_prof_made = g_prof_n + 1;
  }
  r.id = id;
  (void)hipEventRecord(r.a, st);
}

void prof_end(int id, hipStream_t st) {
  if (!g_prof_on || g_prof_n >= kProfCap) return;
  ProfRec& r = g_prof[g_prof_n];
  if (r.id != id) return;
  (void)hipEventRecord(r.b, st);
  ++g_prof_n;
}

}  // namespace cdf

using namespace cdf;

extern "C" const char* cdf_last_error(void) { return g_err; }

extern "C" int cdf_profile_enable(int on) {
  g_prof_on = on != 0;
  if (on) g_prof_n = 0;
  return CDF_OK;
}

__global__ __launch_bounds__(256) void copy_kernel(uint4* __restrict__ dst, const uint4* __restrict__ src, size_t n) {
  for (size_t i = blockIdx.x * static_cast<size_t>(blockDim.x) + threadIdx.x; i < n;
       i += static_cast<size_t>(gridDim.x) * blockDim.x)
    dst[i] = src[i];
}

extern "C" int cdf_profile_copy(void* dst, const void* src, size_t bytes, void* stream) {
  CDF_REQUIRE(dst && src && bytes % 16 == 0 && aligned(dst, 16) && aligned(src, 16),
              "cdf_profile_copy: pointers and size must be multiples of 16 bytes");
  if (bytes == 0) return CDF_OK;
  const size_t n = bytes / 16;
  const size_t blocks = (n + 255) / 256;
  copy_kernel<<<static_cast<unsigned>(blocks < 16384 ? blocks : 16384), 256, 0, static_cast<hipStream_t>(stream)>>>(
      static_cast<uint4*>(dst), static_cast<const uint4*>(src), n);
  CDF_LAUNCH_CHECK("cdf_profile_copy");
  return CDF_OK;
}

extern "C" int cdf_profile_kernels(void) { return K_COUNT; }

extern "C" const char* cdf_profile_kernel_name(int kernel) {
  return kernel >= 0 && kernel < K_COUNT ? kKernelNames[kernel] : "";
}

extern "C" int cdf_profile_read(int kernel, float* ms, int cap) {
  int n = 0;
  for (int i = 0; i < g_prof_n; ++i) {
    if (g_prof[i].id != kernel) continue;
    if (n < cap && ms) {
      if (hipEventSynchronize(g_prof[i].b) != hipSuccess) CDF_FAIL(CDF_ERR_HIP, "cdf_profile_read: event sync failed");
      float t = 0.0f;
      if (hipEventElapsedTime(&t, g_prof[i].a, g_prof[i].b) != hipSuccess)
        CDF_FAIL(CDF_ERR_HIP, "cdf_profile_read: elapsed time failed");
      ms[n] = t;
    }
    ++n;
  }
  return n;
}

extern "C" int cdf_profile_read_all(int32_t* kernel, float* ms, int cap) {
  for (int i = 0; i < g_prof_n && i < cap; ++i) {
    if (hipEventSynchronize(g_prof[i].b) != hipSuccess) CDF_FAIL(CDF_ERR_HIP, "cdf_profile_read_all: event sync failed");
    float t = 0.0f;
    if (hipEventElapsedTime(&t, g_prof[i].a, g_prof[i].b) != hipSuccess)
      CDF_FAIL(CDF_ERR_HIP, "cdf_profile_read_all: elapsed time failed");
    if (kernel) kernel[i] = g_prof[i].id;
    if (ms) ms[i] = t;
  }
  return g_prof_n;
}

extern "C" size_t cdf_workspace_bytes(int64_t max_rows, int32_t max_dim, int64_t max_nnz) {
  if (max_rows < 0 || max_dim <= 0 || max_nnz < 0) return 0;
  const size_t steps = filter_workspace_bytes(max_rows) +
                       max_sz(spmm_workspace_bytes(max_nnz, max_dim), dense_workspace_bytes(max_rows, max_dim, max_dim));
  return max_sz(steps, test_encode_workspace_bytes(max_rows, max_dim));
}

extern "C" int cdf_gcn_layer_fwd(const cdf_layer_fwd_args* p, void* ws, size_t ws_bytes, void* stream) {
  CDF_REQUIRE(p != nullptr && p->A != nullptr, "cdf_gcn_layer_fwd: null argument block");
  CDF_REQUIRE(p->n_loc >= 0 && p->n_halo >= 0 && p->f_in > 0 && p->f_out > 0, "cdf_gcn_layer_fwd: bad sizes");
  CDF_REQUIRE(p->A->n_rows == p->n_loc && p->A->n_cols == p->n_loc + p->n_halo,
              "cdf_gcn_layer_fwd: adjacency is %d x %d, expected %d x %d", p->A->n_rows, p->A->n_cols, p->n_loc,
              p->n_loc + p->n_halo);
  CDF_REQUIRE(p->xfull && p->W && p->M && p->H, "cdf_gcn_layer_fwd: null matrix");
  if (p->dt != CDF_F32 && p->dt != CDF_BF16) CDF_FAIL(CDF_ERR_UNSUPPORTED, "cdf_gcn_layer_fwd: dtype %d", (int)p->dt);
  if (p->n_halo > 0 && p->f_in > cdf_max_message_dim(p->f_in, p->f_in, p->dt))
    CDF_FAIL(CDF_ERR_UNSUPPORTED, "cdf_gcn_layer_fwd: halo rows of %d elements are wider than the message kernels take (%d)",
             p->f_in, cdf_max_message_dim(p->f_in, p->f_in, p->dt));
  const size_t fw = filter_workspace_bytes(p->n_halo);
  const size_t need = fw + spmm_workspace_bytes(p->A->nnz, p->f_in);
  if (!ws || !aligned(ws, 256) || ws_bytes < need)
    CDF_FAIL(CDF_ERR_WORKSPACE, "cdf_gcn_layer_fwd: workspace too small or unaligned (%zu < %zu)", ws_bytes, need);
  char* w = static_cast<char*>(ws);
  const size_t esz = elem_bytes(p->dt);
  int rc;
  if (p->n_halo > 0) {
    CDF_REQUIRE(p->halo_fresh && p->cache_sent && p->mask && p->idx && p->n_sent && p->codes && p->meta,
                "cdf_gcn_layer_fwd: null halo buffer");
    rc = test_and_encode(p->halo_fresh, p->cache_sent, p->n_halo, p->f_in, p->f_in, p->dt, p->eps, p->norm, p->bits,
                         p->qs, p->commit, p->delta, p->mask, p->idx, p->n_sent, p->codes, p->meta, w, ws_bytes, stream);
    if (rc != CDF_OK) return rc;
    void* halo_rows = static_cast<char*>(p->xfull) + static_cast<size_t>(p->n_loc) * p->f_in * esz;
    rc = cdf_dequantize(p->codes, p->meta, p->idx, p->n_sent, p->n_halo, p->f_in, p->bits, p->qs, halo_rows, p->f_in,
                        p->dt, p->delta ? 1 : 0, stream);
    if (rc != CDF_OK) return rc;
  }
  rc = cdf_spmm_fwd(p->A, p->xfull, p->f_in, p->M, p->f_in, p->f_in, p->dt, w + fw, ws_bytes - fw, stream);
  if (rc != CDF_OK) return rc;
  return dense_fwd_ws(p->M, p->f_in, p->dt, p->W, p->n_loc, p->f_in, p->f_out, p->relu, p->Z, p->H, w, ws_bytes, stream);
}

extern "C" int cdf_gcn_layer_bwd(const cdf_layer_bwd_args* p, void* ws, size_t ws_bytes, void* stream) {
  CDF_REQUIRE(p != nullptr, "cdf_gcn_layer_bwd: null argument block");
  CDF_REQUIRE(p->n_loc >= 0 && p->n_halo >= 0 && p->f_in > 0 && p->f_out > 0, "cdf_gcn_layer_bwd: bad sizes");
  CDF_REQUIRE(p->dH && p->M && p->W && p->dW && (!p->relu || p->Zs), "cdf_gcn_layer_bwd: null matrix");
  if (p->dt != CDF_F32 && p->dt != CDF_BF16) CDF_FAIL(CDF_ERR_UNSUPPORTED, "cdf_gcn_layer_bwd: dtype %d", (int)p->dt);
  if (p->need_dx) {
    CDF_REQUIRE(p->At != nullptr && p->dM && p->dxfull, "cdf_gcn_layer_bwd: need_dx without At / dM / dxfull");
    CDF_REQUIRE(p->At->n_rows == p->n_loc + p->n_halo && p->At->n_cols == p->n_loc,
                "cdf_gcn_layer_bwd: transposed adjacency is %d x %d, expected %d x %d", p->At->n_rows, p->At->n_cols,
                p->n_loc + p->n_halo, p->n_loc);
  }
  if (p->need_dx && p->n_halo > 0 && p->f_in > cdf_max_message_dim(p->f_in, p->f_in, p->dt))
    CDF_FAIL(CDF_ERR_UNSUPPORTED, "cdf_gcn_layer_bwd: halo rows of %d elements are wider than the message kernels take (%d)",
             p->f_in, cdf_max_message_dim(p->f_in, p->f_in, p->dt));
  const size_t fw = filter_workspace_bytes(p->n_halo);
  size_t need = fw + dense_workspace_bytes(p->n_loc, p->f_in, p->f_out);
  if (p->need_dx) need = max_sz(need, fw + spmm_workspace_bytes(p->At->nnz, p->f_in));
  if (!ws || !aligned(ws, 256) || ws_bytes < need)
    CDF_FAIL(CDF_ERR_WORKSPACE, "cdf_gcn_layer_bwd: workspace too small or unaligned (%zu < %zu)", ws_bytes, need);
  char* w = static_cast<char*>(ws);
  const size_t esz = elem_bytes(p->dt);
  int rc = cdf_dense_bwd(p->M, p->f_in, p->dt, p->W, p->Zs, p->dH, p->n_loc, p->f_in, p->f_out, p->relu, p->dW,
                         p->need_dx ? p->dM : nullptr, p->f_in, w + fw, ws_bytes - fw, stream);
  if (rc != CDF_OK || !p->need_dx) return rc;
  rc = cdf_spmm_bwd(p->At, p->dM, p->f_in, p->dxfull, p->f_in, p->f_in, p->dt, w + fw, ws_bytes - fw, stream);
  if (rc != CDF_OK) return rc;
  if (p->n_halo > 0) {
    CDF_REQUIRE(p->gcache_sent && p->mask && p->idx && p->n_sent && p->codes && p->meta,
                "cdf_gcn_layer_bwd: null halo buffer");
    const void* halo_rows = static_cast<const char*>(p->dxfull) + static_cast<size_t>(p->n_loc) * p->f_in * esz;
    rc = test_and_encode(halo_rows, p->gcache_sent, p->n_halo, p->f_in, p->f_in, p->dt, p->eps, p->norm, p->bits,
                         p->qs, p->commit, p->delta, p->mask, p->idx, p->n_sent, p->codes, p->meta, w, ws_bytes, stream);
  }
  return rc;
}

extern "C" int cdf_gcn_layer_tf_fwd(const cdf_layer_tf_fwd_args* p, void* ws, size_t ws_bytes, void* stream) {
  hipStream_t st = static_cast<hipStream_t>(stream);
  CDF_REQUIRE(p != nullptr && p->A != nullptr, "cdf_gcn_layer_tf_fwd: null argument block");
  CDF_REQUIRE(p->n_loc >= 0 && p->n_halo >= 0 && p->f_in > 0 && p->f_out > 0, "cdf_gcn_layer_tf_fwd: bad sizes");
  CDF_REQUIRE(p->A->n_rows == p->n_loc && p->A->n_cols == p->n_loc + p->n_halo,
              "cdf_gcn_layer_tf_fwd: adjacency is %d x %d, expected %d x %d", p->A->n_rows, p->A->n_cols, p->n_loc,
              p->n_loc + p->n_halo);
  CDF_REQUIRE(p->x_local && p->W && p->tfull && p->H, "cdf_gcn_layer_tf_fwd: null matrix");
  if (p->n_halo > 0 && p->f_out > cdf_max_message_dim(p->f_out, p->f_out, CDF_F32))
    CDF_FAIL(CDF_ERR_UNSUPPORTED, "cdf_gcn_layer_tf_fwd: halo rows of %d elements are wider than the message kernels take (%d)",
             p->f_out, cdf_max_message_dim(p->f_out, p->f_out, CDF_F32));
  const size_t fw = filter_workspace_bytes(p->n_halo);
  const size_t need = fw + spmm_workspace_bytes(p->A->nnz, p->f_out);
  if (!ws || !aligned(ws, 256) || ws_bytes < need)
    CDF_FAIL(CDF_ERR_WORKSPACE, "cdf_gcn_layer_tf_fwd: workspace too small or unaligned (%zu < %zu)", ws_bytes, need);
  char* w = static_cast<char*>(ws);
  int rc = cdf_dense_fwd(p->x_local, p->f_in, CDF_F32, p->W, p->n_loc, p->f_in, p->f_out, 0, nullptr, p->tfull, stream);
  if (rc != CDF_OK) return rc;
  if (p->n_halo > 0) {
    CDF_REQUIRE(p->halo_fresh && p->cache_sent && p->mask && p->idx && p->n_sent && p->codes && p->meta,
                "cdf_gcn_layer_tf_fwd: null halo buffer");
    rc = test_and_encode(p->halo_fresh, p->cache_sent, p->n_halo, p->f_out, p->f_out, CDF_F32, p->eps, p->norm, p->bits,
                         p->qs, p->commit, p->delta, p->mask, p->idx, p->n_sent, p->codes, p->meta, w, ws_bytes, stream);
    if (rc != CDF_OK) return rc;
    rc = cdf_dequantize(p->codes, p->meta, p->idx, p->n_sent, p->n_halo, p->f_out, p->bits, p->qs,
                        p->tfull + static_cast<size_t>(p->n_loc) * p->f_out, p->f_out, CDF_F32, p->delta ? 1 : 0, stream);
    if (rc != CDF_OK) return rc;
  }
  // aggregation with the activation fused into the row store
  if (p->relu)
    return spmm_run("cdf_gcn_layer_tf_fwd", p->A, p->tfull, p->f_out, p->Z, p->H, p->f_out, p->f_out, CDF_F32, w + fw,
                    ws_bytes - fw, st);
  rc = spmm_run("cdf_gcn_layer_tf_fwd", p->A, p->tfull, p->f_out, p->H, nullptr, p->f_out, p->f_out, CDF_F32, w + fw,
                ws_bytes - fw, st);
  if (rc == CDF_OK && p->Z && p->n_loc > 0) {
    if (hipMemcpyAsync(p->Z, p->H, static_cast<size_t>(p->n_loc) * p->f_out * sizeof(float), hipMemcpyDeviceToDevice,
                       st) != hipSuccess)
      CDF_FAIL(CDF_ERR_HIP, "cdf_gcn_layer_tf_fwd: copy of Z failed");
  }
  return rc;
}

extern "C" int cdf_gcn_layer_tf_bwd(const cdf_layer_tf_bwd_args* p, void* ws, size_t ws_bytes, void* stream) {
  hipStream_t st = static_cast<hipStream_t>(stream);
  CDF_REQUIRE(p != nullptr && p->At != nullptr, "cdf_gcn_layer_tf_bwd: null argument block");
  CDF_REQUIRE(p->n_loc >= 0 && p->n_halo >= 0 && p->f_in > 0 && p->f_out > 0, "cdf_gcn_layer_tf_bwd: bad sizes");
  CDF_REQUIRE(p->At->n_rows == p->n_loc + p->n_halo && p->At->n_cols == p->n_loc,
              "cdf_gcn_layer_tf_bwd: transposed adjacency is %d x %d, expected %d x %d", p->At->n_rows, p->At->n_cols,
              p->n_loc + p->n_halo, p->n_loc);
  CDF_REQUIRE(p->dH && p->x_local && p->W && p->dtfull && p->dW && (!p->relu || (p->Zs && p->dZ)),
              "cdf_gcn_layer_tf_bwd: null matrix");
  if (p->n_halo > 0 && p->f_out > cdf_max_message_dim(p->f_out, p->f_out, CDF_F32))
    CDF_FAIL(CDF_ERR_UNSUPPORTED, "cdf_gcn_layer_tf_bwd: halo rows of %d elements are wider than the message kernels take (%d)",
             p->f_out, cdf_max_message_dim(p->f_out, p->f_out, CDF_F32));
  const size_t fw = filter_workspace_bytes(p->n_halo);
  size_t need = fw + spmm_workspace_bytes(p->At->nnz, p->f_out);
  need = max_sz(need, fw + dense_workspace_bytes(p->n_loc, p->f_in, p->f_out));
  if (!ws || !aligned(ws, 256) || ws_bytes < need)
    CDF_FAIL(CDF_ERR_WORKSPACE, "cdf_gcn_layer_tf_bwd: workspace too small or unaligned (%zu < %zu)", ws_bytes, need);
  char* w = static_cast<char*>(ws);
  const float* dz = p->dH;
  const int64_t count = static_cast<int64_t>(p->n_loc) * p->f_out;
  if (p->relu && count > 0) {
    CDF_REQUIRE(aligned(p->dH, 16) && aligned(p->Zs, 16) && aligned(p->dZ, 16), "cdf_gcn_layer_tf_bwd: misaligned matrix");
    const int64_t blocks = ceil_div(ceil_div(count, 4), 256);
    {
      ProfScope ps(K_RELU_MASK, st);
      relu_mask_kernel<<<static_cast<unsigned>(blocks < 65536 ? (blocks > 0 ? blocks : 1) : 65536), 256, 0, st>>>(
          p->dH, p->Zs, p->dZ, count);
    }
    CDF_LAUNCH_CHECK("cdf_gcn_layer_tf_bwd/mask");
    dz = p->dZ;
  }
  int rc = cdf_spmm_bwd(p->At, dz, p->f_out, p->dtfull, p->f_out, p->f_out, CDF_F32, w + fw, ws_bytes - fw, stream);
  if (rc != CDF_OK) return rc;
  if (p->n_halo > 0) {
    CDF_REQUIRE(p->gcache_sent && p->mask && p->idx && p->n_sent && p->codes && p->meta,
                "cdf_gcn_layer_tf_bwd: null halo buffer");
    const float* halo_rows = p->dtfull + static_cast<size_t>(p->n_loc) * p->f_out;
    rc = test_and_encode(halo_rows, p->gcache_sent, p->n_halo, p->f_out, p->f_out, CDF_F32, p->eps, p->norm, p->bits,
                         p->qs, p->commit, p->delta, p->mask, p->idx, p->n_sent, p->codes, p->meta, w, ws_bytes, stream);
    if (rc != CDF_OK) return rc;
  }
  return cdf_dense_bwd(p->x_local, p->f_in, CDF_F32, p->W, nullptr, p->dtfull, p->n_loc, p->f_in, p->f_out, 0, p->dW,
                       p->dx_local, p->f_in, w + fw, ws_bytes - fw, stream);
}
