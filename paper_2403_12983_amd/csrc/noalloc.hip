// osscar_gram_static: the quadratic form of one small layer, H = X^T X + lambda I and G = H W (Section 3, dense-layer
// paragraph), in one call that allocates nothing.  It is osscar_gram (one chunk plus finalize) for callers that cannot
// allocate device memory: there is no context and no workspace argument; what osscar_gram keeps in the caller's workspace
// during the Gram phase -- the float64 accumulator of H, the float32 copy of W, the transposed float32 staging of X and a
// few scalars -- lives in a fixed device array of this file instead.
#include "../../include/osscar.h"
#include "internal.h"

#include <algorithm>
#include <mutex>

using namespace osscar;

namespace {

constexpr int64_t ST_MAX = OSSCAR_STATIC_MAX_DIM;      // largest d1 and m
constexpr int64_t ST_XT_ROWS = 2048;                   // calibration rows per sub-step
constexpr size_t ST_H64 = (size_t)ST_MAX * ST_MAX * 8, ST_WF = (size_t)ST_MAX * ST_MAX * 4, ST_XT = (size_t)ST_MAX * ST_XT_ROWS * 4;
constexpr size_t ST_SMALL = 64 * 1024;                 // scalars and the partial sums of the reductions
constexpr size_t ST_BYTES = ST_H64 + ST_WF + ST_XT + ST_SMALL;
static_assert(ST_BYTES == OSSCAR_STATIC_SCRATCH_BYTES, "the header states the size of the array");

// One copy per GPU, at its own address on each, for as long as the process lives.  In host code this name is only a
// handle for hipGetSymbolAddress: the device address is looked up once per device below and everything else uses that.
static __device__ __align__(256) unsigned char scratch[ST_BYTES];

constexpr int MAX_DEVICES = 64;
std::mutex g_mu;
void* g_scratch_ptr[MAX_DEVICES] = {};

hipError_t scratch_of_current_device(unsigned char** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= MAX_DEVICES) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(g_mu);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!p) return hipErrorInvalidSymbol;
    g_scratch_ptr[dev] = p;
  }
  *out = reinterpret_cast<unsigned char*>(g_scratch_ptr[dev]);
  return hipSuccess;
}

__global__ void st_fill_f64_kernel(double* p, int64_t n, double v) {
  for (int64_t i = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x) p[i] = v;
}
// scal[1] = lambda = lambda_abs + lambda_rel * trace / d1 (scal[0] = trace of X^T X)
__global__ void st_lambda_kernel(double* scal, double lambda_abs, double lambda_rel, int d1) {
  if (threadIdx.x == 0 && blockIdx.x == 0) scal[1] = lambda_abs + lambda_rel * scal[0] / (double)d1;
}
__global__ void st_emit_kernel(const double* scal, double* out) {
  if (threadIdx.x == 0 && blockIdx.x == 0) { out[0] = scal[1]; out[1] = scal[2]; }
}

osscar_status refuse(osscar_status st, const char* msg) { set_contextless_error(msg); return st; }

}  // namespace

extern "C" osscar_status osscar_gram_static(const void* X_dev, int64_t n, int64_t ldx, int32_t x_dtype, const void* W_dev, int64_t ldw,
                                            int32_t w_dtype, int64_t d1, int64_t m, double lambda_abs, double lambda_rel, float* H_dev,
                                            float* G_dev, double* scalars_dev, void* hip_stream) {
  if (d1 < 1 || m < 1 || n < 0) return refuse(OSSCAR_EINVAL, "osscar_gram_static: d1 and m must be positive and n >= 0");
  if (d1 > ST_MAX || m > ST_MAX)
    return refuse(OSSCAR_ENOMEM, "osscar_gram_static: d1 and m may not exceed OSSCAR_STATIC_MAX_DIM (1024): the fixed scratch array "
                                 "is sized for that; larger layers go through osscar_gram with a caller-provided workspace");
  if ((x_dtype != OSSCAR_F32 && x_dtype != OSSCAR_BF16) || (w_dtype != OSSCAR_F32 && w_dtype != OSSCAR_BF16))
    return refuse(OSSCAR_EINVAL, "osscar_gram_static: unknown dtype");
  if (!W_dev || !H_dev || !G_dev || !scalars_dev || (n > 0 && !X_dev) || ldx < d1 || ldw < m)
    return refuse(OSSCAR_EINVAL, "osscar_gram_static: NULL pointer or leading dimension below the row length");
  unsigned char* base = nullptr;
  if (scratch_of_current_device(&base) != hipSuccess) return refuse(OSSCAR_EHIP, "osscar_gram_static: hipGetSymbolAddress failed");
  hipStream_t s = reinterpret_cast<hipStream_t>(hip_stream);
  double* H64 = reinterpret_cast<double*>(base);
  float* Wf = reinterpret_cast<float*>(base + ST_H64);
  float* Xt = reinterpret_cast<float*>(base + ST_H64 + ST_WF);
  double* scal = reinterpret_cast<double*>(base + ST_H64 + ST_WF + ST_XT);      // 64 scalars, then 2048 partial sums
  double* partial = scal + 64;
  const int D = (int)d1, M = (int)m;
  const bool xbf = x_dtype == OSSCAR_BF16;
  // the array keeps the last call's contents: the accumulator starts at zero, everything else is written before it is read
  hipLaunchKernelGGL(st_fill_f64_kernel, dim3((unsigned)std::min<int64_t>((d1 * d1 + 1023) / 1024, 4096)), dim3(256), 0, s, H64, d1 * d1, 0.0);
  const size_t esz = xbf ? 2 : 4;
  hipError_t e = hipSuccess;
  for (int64_t r0 = 0; r0 < n && e == hipSuccess; r0 += ST_XT_ROWS) {
    const int64_t nr = std::min<int64_t>(ST_XT_ROWS, n - r0);
    const char* src = reinterpret_cast<const char*>(X_dev) + (size_t)r0 * ldx * esz;
    e = launch_transpose_to_f32(src, xbf, nr, d1, ldx, Xt, ST_XT_ROWS, s);
    if (e != hipSuccess) break;
    GemmArgs g{};      // H64 += Xt Xt^T on the lower triangle, float64 accumulation on the matrix cores
    g.M = D; g.N = D; g.K = (int)nr; g.A = Xt; g.lda = ST_XT_ROWS; g.B = Xt; g.ldb = ST_XT_ROWS; g.trans_b = 1;
    g.Cin = reinterpret_cast<const float*>(H64); g.ldcin = D; g.C = H64; g.ldc = D; g.alpha = 1.0; g.beta = 1.0;
    g.c_is_f64 = 1; g.lower_only = 1;
    e = launch_gemm_f64acc(g, s);
  }
  if (e == hipSuccess) e = launch_trace64(H64, D, scal, s);
  if (e == hipSuccess) {
    hipLaunchKernelGGL(st_lambda_kernel, dim3(1), dim3(64), 0, s, scal, lambda_abs, lambda_rel, D);
    e = launch_finalize_H(H64, H_dev, D, scal + 1, s);
  }
  if (e == hipSuccess) e = launch_convert_to_f32(W_dev, w_dtype == OSSCAR_BF16, d1, m, ldw, Wf, s);
  if (e == hipSuccess) {
    GemmArgs g{};      // G = H W
    g.M = D; g.N = M; g.K = D; g.A = H_dev; g.lda = D; g.B = Wf; g.ldb = M; g.C = G_dev; g.ldc = M; g.alpha = 1.0; g.beta = 0.0;
    e = launch_gemm_f64acc(g, s);
  }
  if (e == hipSuccess) e = launch_dot64(Wf, G_dev, d1 * m, scal + 2, partial, s);      // c0 = Tr(W^T G)
  if (e == hipSuccess) {
    hipLaunchKernelGGL(st_emit_kernel, dim3(1), dim3(64), 0, s, scal, scalars_dev);
    e = hipGetLastError();
  }
  if (e != hipSuccess) return refuse(OSSCAR_EHIP, hipGetErrorString(e));
  return OSSCAR_OK;
}
