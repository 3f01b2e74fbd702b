// The swept tableau and the kernels of the local search (Section 4.2; Proposition 4.1, Cases 1-3).
//
// State.  For the kept set K the library holds the symmetric d1 x d1 matrix
//        N = [ -P   V ]      P = (H_KK)^-1,  V = P H_{K,Kc},  S = H_cc - H_cK P H_Kc
//            [ V^T  S ]
// in the ORIGINAL row order (row i belongs to group i / q, kept or not), lower triangle only, and
//        Z = [ B ; R ]       B = P G_K (optimal kept weights),  R = G_Kc - H_cK B
// as d1 x m.  N is H with the "sweep operator" applied to the pivots in K, and Z is G carried along.
// In this form Proposition 4.1's Case 2 (a group enters) is a forward sweep on that group's q x q
// pivot block and Case 1 (a group leaves) is the reverse sweep; both are the same rank-q update
//        N_il -= N_it D N_tl,   Z_i -= N_it D Z_t        (D = N_tt^-1, i, l outside the pivot)
// and differ only in the sign given to the pivot rows (+D N_tl entering, -D N_tl leaving; N_tt' = -D).
// The change of the objective is -Tr(Z_t^T D Z_t) in both cases, and the impact score of eq. (impact)
// of ANY group h is Tr(Z_h^T |N_hh|^-1 Z_h): removal cost if h is kept, addition gain otherwise.
// A swap (Case 3) is the reverse sweep on g followed by the forward sweep on j; the two are fused into
// one rank-2q pass over N and Z, with the second pivot's panel corrected for the first sweep beforehand.
#include "internal.h"

namespace osscar {

// ------------------------------------------------------------------------------------------------
// small dense helpers (float64, one workgroup, matrices in global or shared memory)
// ------------------------------------------------------------------------------------------------
// In-place inverse of the n x n matrix A (leading dimension n, n <= 16 T, shared or global memory) by Gauss-Jordan without
// pivoting; valid for definite matrices of either sign.  want_sign = +1 / -1: every pivot must have that sign, else
// *bad = 1.  Called by all 256 threads of a workgroup: thread (ti, tj) of a 16 x 16 grid keeps the T x T block with rows
// ti*T.. and columns tj*T.. in registers (rows and columns past n behave as an identity block); every step broadcasts the
// pivot row and column through buf (64 T doubles of shared memory, two halves used in turn: one barrier per step).
template <int T>
__device__ void small_inverse(double* A, int n, int want_sign, int32_t* bad, double* buf) {
  const int tid = threadIdx.x, ti = tid >> 4, tj = tid & 15;
  double r[T][T];
  __syncthreads();
#pragma unroll
  for (int a = 0; a < T; a++)
#pragma unroll
    for (int b = 0; b < T; b++) {
      const int i = ti * T + a, j = tj * T + b;
      r[a][b] = (i < n && j < n) ? A[i * n + j] : (i == j ? 1.0 : 0.0);
    }
  bool flag = false;
  for (int k0 = 0; k0 < n; k0 += T) {
#pragma unroll
    for (int kk = 0; kk < T; kk++) {
      const int k = k0 + kk;
      if (k < n) {                                   // uniform over the workgroup
        double* rowb = buf + (k & 1) * (32 * T);
        double* colb = rowb + 16 * T;
        if (ti == k0 / T) {
#pragma unroll
          for (int b = 0; b < T; b++) rowb[tj * T + b] = r[kk][b];
        }
        if (tj == k0 / T) {
#pragma unroll
          for (int a = 0; a < T; a++) colb[ti * T + a] = r[a][kk];
        }
        __syncthreads();
        double piv = rowb[k];
        if (!(piv * want_sign > 0.0)) { flag = true; piv = want_sign; }
        const double d = 1.0 / piv;
        double rs[T], cs[T];
#pragma unroll
        for (int b = 0; b < T; b++) rs[b] = rowb[tj * T + b] * d;
#pragma unroll
        for (int a = 0; a < T; a++) cs[a] = colb[ti * T + a];
        // rank-one step on the whole block; the pivot row and column (meaningless after it) are rewritten by their owners
#pragma unroll
        for (int a = 0; a < T; a++)
#pragma unroll
          for (int b = 0; b < T; b++) r[a][b] -= cs[a] * rs[b];
        if (tj == k0 / T) {
#pragma unroll
          for (int a = 0; a < T; a++) r[a][kk] = -cs[a] * d;
        }
        if (ti == k0 / T) {
#pragma unroll
          for (int b = 0; b < T; b++) r[kk][b] = rs[b];
          if (tj == k0 / T) r[kk][kk] = d;
        }
      }
    }
  }
  if (flag && tid == 0) *bad = 1;
#pragma unroll
  for (int a = 0; a < T; a++)
#pragma unroll
    for (int b = 0; b < T; b++) {
      const int i = ti * T + a, j = tj * T + b;
      if (i < n && j < n) A[i * n + j] = r[a][b];
    }
  __syncthreads();
}

__device__ __forceinline__ double wave_sum(double v) {
  for (int o = 32; o > 0; o >>= 1) v += __shfl_down(v, o, 64);
  return v;
}

__device__ __forceinline__ float nsym(const float* __restrict__ N, int64_t ld, int i, int t) {
  return (i >= t) ? N[(int64_t)i * ld + t] : N[(int64_t)t * ld + i];
}

// ------------------------------------------------------------------------------------------------
// gather / scatter / mirror / absmax
// ------------------------------------------------------------------------------------------------
__global__ void gather_kernel(const float* __restrict__ src, int64_t lds_, const int32_t* __restrict__ rows, int nrows,
                              const int32_t* __restrict__ cols, int ncols, float* __restrict__ dst, int64_t ldd) {
  int64_t n = (int64_t)nrows * ncols;
  for (int64_t idx = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; idx < n; idx += (int64_t)gridDim.x * blockDim.x) {
    int i = (int)(idx / ncols), j = (int)(idx % ncols);
    int64_t r = rows ? rows[i] : i, c = cols ? cols[j] : j;
    dst[(int64_t)i * ldd + j] = src[r * lds_ + c];
  }
}
hipError_t launch_gather(const float* src, int64_t lds_, const int32_t* rows, int nrows, const int32_t* cols, int ncols,
                         float* dst, int64_t ldd, hipStream_t s) {
  int64_t n = (int64_t)nrows * ncols;
  if (n <= 0) return hipSuccess;
  int blocks = (int)((n + 1023) / 1024); if (blocks > 131072) blocks = 131072;
  hipLaunchKernelGGL(gather_kernel, dim3(blocks), dim3(256), 0, s, src, lds_, rows, nrows, cols, ncols, dst, ldd);
  return hipGetLastError();
}

// dst[max(r,c)][min(r,c)] = sign * src[i][j], r = rows[i], c = cols[j]; if tri: only i >= j
__global__ void scatter_kernel(const float* __restrict__ src, int64_t lds_, const int32_t* __restrict__ rows, int nrows,
                               const int32_t* __restrict__ cols, int ncols, float* __restrict__ dst, int64_t ldd,
                               float sign, int tri) {
  int64_t n = (int64_t)nrows * ncols;
  for (int64_t idx = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; idx < n; idx += (int64_t)gridDim.x * blockDim.x) {
    int i = (int)(idx / ncols), j = (int)(idx % ncols);
    if (tri && i < j) continue;
    int64_t r = rows[i], c = cols[j];
    int64_t hi = r > c ? r : c, lo = r > c ? c : r;
    dst[hi * ldd + lo] = sign * src[(int64_t)i * lds_ + j];
  }
}
hipError_t launch_scatter(const float* src, int64_t lds_, const int32_t* rows, int nrows, const int32_t* cols, int ncols,
                          float* dst, int64_t ldd, float sign, int tri, hipStream_t s) {
  int64_t n = (int64_t)nrows * ncols;
  if (n <= 0) return hipSuccess;
  int blocks = (int)((n + 1023) / 1024); if (blocks > 131072) blocks = 131072;
  hipLaunchKernelGGL(scatter_kernel, dim3(blocks), dim3(256), 0, s, src, lds_, rows, nrows, cols, ncols, dst, ldd, sign, tri);
  return hipGetLastError();
}

// rows of a dense matrix into rows[] of dst (float or bf16 destination)
__device__ __forceinline__ uint16_t float_to_bf16_rne(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (uint16_t)((u >> 16) | 0x40);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}
__global__ void scatter_rows_kernel(const float* __restrict__ src, int64_t lds_, const int32_t* __restrict__ rows,
                                    int nrows, int ncols, void* __restrict__ dst, int64_t ldd, int dst_is_bf16) {
  int64_t n = (int64_t)nrows * ncols;
  for (int64_t idx = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; idx < n; idx += (int64_t)gridDim.x * blockDim.x) {
    int i = (int)(idx / ncols), j = (int)(idx % ncols);
    float v = src[(int64_t)i * lds_ + j];
    int64_t o = (int64_t)rows[i] * ldd + j;
    if (dst_is_bf16) reinterpret_cast<uint16_t*>(dst)[o] = float_to_bf16_rne(v);
    else reinterpret_cast<float*>(dst)[o] = v;
  }
}
hipError_t launch_scatter_rows(const float* src, int64_t lds_, const int32_t* rows, int nrows, int ncols, void* dst,
                               int64_t ldd, int dst_is_bf16, hipStream_t s) {
  int64_t n = (int64_t)nrows * ncols;
  if (n <= 0) return hipSuccess;
  int blocks = (int)((n + 1023) / 1024); if (blocks > 131072) blocks = 131072;
  hipLaunchKernelGGL(scatter_rows_kernel, dim3(blocks), dim3(256), 0, s, src, lds_, rows, nrows, ncols, dst, ldd, dst_is_bf16);
  return hipGetLastError();
}
__global__ void fill_zero_kernel(void* __restrict__ dst, int64_t ldd, int nrows, int ncols, int dst_is_bf16) {
  int64_t n = (int64_t)nrows * ncols;
  for (int64_t idx = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; idx < n; idx += (int64_t)gridDim.x * blockDim.x) {
    int i = (int)(idx / ncols), j = (int)(idx % ncols);
    int64_t o = (int64_t)i * ldd + j;
    if (dst_is_bf16) reinterpret_cast<uint16_t*>(dst)[o] = 0;
    else reinterpret_cast<float*>(dst)[o] = 0.f;
  }
}
hipError_t launch_fill_rows_zero(void* dst, int64_t ldd, int nrows, int ncols, int dst_is_bf16, hipStream_t s) {
  int64_t n = (int64_t)nrows * ncols;
  if (n <= 0) return hipSuccess;
  int blocks = (int)((n + 1023) / 1024); if (blocks > 131072) blocks = 131072;
  hipLaunchKernelGGL(fill_zero_kernel, dim3(blocks), dim3(256), 0, s, dst, ldd, nrows, ncols, dst_is_bf16);
  return hipGetLastError();
}

// A[i][j] (j > i) = A[j][i]
__global__ void mirror_lower_kernel(float* __restrict__ A, int n, int64_t lda) {
  int64_t tot = (int64_t)n * n;
  for (int64_t idx = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; idx < tot; idx += (int64_t)gridDim.x * blockDim.x) {
    int i = (int)(idx / n), j = (int)(idx % n);
    if (j > i) A[(int64_t)i * lda + j] = A[(int64_t)j * lda + i];
  }
}
hipError_t launch_mirror_lower(float* A, int n, int64_t lda, hipStream_t s) {
  int64_t tot = (int64_t)n * n;
  if (tot <= 0) return hipSuccess;
  int blocks = (int)((tot + 1023) / 1024); if (blocks > 131072) blocks = 131072;
  hipLaunchKernelGGL(mirror_lower_kernel, dim3(blocks), dim3(256), 0, s, A, n, lda);
  return hipGetLastError();
}

// out[b] for 256 blocks, then the caller reduces on the host (256 doubles).  A bandwidth-bound pass: 1024 threads per
// block, four 16-byte loads in flight per thread (scalar loads for an unaligned start and for the tail).
__device__ __forceinline__ float absmax_take(float v, float x) { x = fabsf(x); return (x > v || x != x) ? x : v; }
__global__ __launch_bounds__(1024) void absmax_partial_kernel(const float* __restrict__ A, int64_t n, double* out) {
  __shared__ float sh[16];
  // a NaN is taken (x != x) and then stays (nothing compares greater than it), so a NaN anywhere reaches the result
  float v[4] = {0.f, 0.f, 0.f, 0.f};
  const int64_t head = ((reinterpret_cast<uintptr_t>(A) & 15) == 0) ? 0 : n;      // unaligned: everything in the scalar loop
  const int64_t n4 = (n - head) / 4;
  const float4* A4 = reinterpret_cast<const float4*>(A);
  const int64_t tid = blockIdx.x * 1024 + threadIdx.x, nth = (int64_t)gridDim.x * 1024;
  for (int64_t i = tid; i < n4; i += 4 * nth) {
    float4 q[4];
#pragma unroll
    for (int u = 0; u < 4; u++) { const int64_t k = i + u * nth; q[u] = A4[k < n4 ? k : i]; }
#pragma unroll
    for (int u = 0; u < 4; u++) {
      v[u] = absmax_take(v[u], q[u].x); v[u] = absmax_take(v[u], q[u].y); v[u] = absmax_take(v[u], q[u].z); v[u] = absmax_take(v[u], q[u].w);
    }
  }
  for (int64_t i = head == 0 ? 4 * n4 + tid : tid; i < n; i += nth) v[0] = absmax_take(v[0], A[i]);
  float t = v[0];
#pragma unroll
  for (int u = 1; u < 4; u++) t = (v[u] > t || v[u] != v[u]) ? v[u] : t;
  for (int o = 32; o > 0; o >>= 1) { const float w = __shfl_down(t, o, 64); t = (w > t || w != w) ? w : t; }
  if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = t;
  __syncthreads();
  if (threadIdx.x == 0) { float r = 0.f; for (int i = 0; i < 16; i++) r = (sh[i] > r || sh[i] != sh[i]) ? sh[i] : r; out[blockIdx.x] = (double)r; }
}
hipError_t launch_absmax(const float* A, int64_t n, double* out, hipStream_t s) {  // out: 256 doubles
  hipLaunchKernelGGL(absmax_partial_kernel, dim3(256), dim3(1024), 0, s, A, n, out);
  return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// pivot panels
// ------------------------------------------------------------------------------------------------
// C[i][c] = Nsym(i, t0 + c), c < w <= 128, for all rows i < n.  One workgroup per 64 rows: below the pivot rows the panel
// is a column block of N (read along c); above them it lies transposed in the rows t0 + c of N (read along i and turned
// in shared memory); the few blocks that meet the pivot rows take either side element by element.
constexpr int PANEL_ROWS = 64;
__global__ __launch_bounds__(256) void extract_panel_kernel(const float* __restrict__ N, int64_t ld, int n, int t0,
                                                             int w, float* __restrict__ C) {
  __shared__ float T[PANEL_ROWS][129];
  const int i0 = blockIdx.x * PANEL_ROWS, tid = threadIdx.x;
  if (i0 >= t0 + w) {
    for (int idx = tid; idx < PANEL_ROWS * w; idx += 256) {
      const int r = idx / w, c = idx % w;
      if (i0 + r < n) C[(int64_t)(i0 + r) * w + c] = N[(int64_t)(i0 + r) * ld + t0 + c];
    }
    return;
  }
  if (i0 + PANEL_ROWS <= t0) {
    for (int idx = tid; idx < PANEL_ROWS * w; idx += 256) {
      const int c = idx / PANEL_ROWS, r = idx % PANEL_ROWS;
      T[r][c] = N[(int64_t)(t0 + c) * ld + i0 + r];
    }
  } else {
    for (int idx = tid; idx < PANEL_ROWS * w; idx += 256) {
      const int r = idx / w, c = idx % w;
      T[r][c] = (i0 + r < n) ? nsym(N, ld, i0 + r, t0 + c) : 0.f;
    }
  }
  __syncthreads();
  for (int idx = tid; idx < PANEL_ROWS * w; idx += 256) {
    const int r = idx / w, c = idx % w;
    if (i0 + r < n) C[(int64_t)(i0 + r) * w + c] = T[r][c];
  }
}

// out[i][c] = sum_k C[i][k] * D[k][c]  (D: w x w float64, w <= 128), rows in [t0, t0+w) are written as zero if zero_pivot.
// Optionally also writes Cb = C with the pivot rows zeroed.  16 rows per workgroup: their C values are broadcast from
// LDS, thread (h, c) sums 8 rows of column c in float64, k ascending.
__global__ __launch_bounds__(256) void panel_times_small_kernel(const float* __restrict__ C, const double* __restrict__ D,
                                                                 int n, int w, int t0, int zero_pivot,
                                                                 float* __restrict__ out, float* __restrict__ Cb) {
  __shared__ float Csh[16][128];
  const int r0 = blockIdx.x * 16, tid = threadIdx.x;
  for (int idx = tid; idx < 16 * w; idx += 256) {
    const int r = idx / w, k = idx % w;
    Csh[r][k] = (r0 + r < n) ? C[(int64_t)(r0 + r) * w + k] : 0.f;
  }
  __syncthreads();
  const int c = tid & 127, h = tid >> 7;
  if (c >= w) return;
  double acc[8];
#pragma unroll
  for (int r = 0; r < 8; r++) acc[r] = 0.0;
  for (int k = 0; k < w; k++) {
    const double dv = D[k * w + c];
#pragma unroll
    for (int r = 0; r < 8; r++) acc[r] += (double)Csh[h * 8 + r][k] * dv;
  }
#pragma unroll
  for (int r = 0; r < 8; r++) {
    const int i = r0 + h * 8 + r;
    if (i >= n) continue;
    const bool piv = zero_pivot && i >= t0 && i < t0 + w;
    out[(int64_t)i * w + c] = piv ? 0.f : (float)acc[r];
    if (Cb) Cb[(int64_t)i * w + c] = piv ? 0.f : Csh[h * 8 + r][c];
  }
}

// ------------------------------------------------------------------------------------------------
// blocked in-place inverse of an SPD matrix by sweeping nb columns at a time (lower triangle storage)
// ------------------------------------------------------------------------------------------------
// D = inverse of the w x w pivot block (rows t0.. of the extracted panel), float64
__global__ __launch_bounds__(256) void inv_block_kernel(const float* __restrict__ C, int w, int t0, double* __restrict__ D,
                                                         int32_t* notpd) {
  __shared__ double buf[64 * (INV_NB / 16)];
  for (int idx = threadIdx.x; idx < w * w; idx += 256) {
    int r = idx / w, c = idx % w;
    D[idx] = (double)C[(int64_t)(t0 + r) * w + c];
  }
  small_inverse<INV_NB / 16>(D, w, +1, notpd, buf);
}

// pivot rows after a forward sweep: N(t0+r, l) = CD[l][r] for l outside the pivot, N(tt) = -D
__global__ __launch_bounds__(256) void inv_fix_kernel(float* __restrict__ N, int64_t ld, int n, int t0, int w,
                                                       const float* __restrict__ CD, const double* __restrict__ D) {
  __shared__ float T[PANEL_ROWS][129];
  const int i0 = blockIdx.x * PANEL_ROWS, tid = threadIdx.x;
  if (i0 >= t0 + w) {                         // below the pivot rows: a column block of N
    for (int idx = tid; idx < PANEL_ROWS * w; idx += 256) {
      const int r = idx / w, c = idx % w;
      if (i0 + r < n) N[(int64_t)(i0 + r) * ld + t0 + c] = CD[(int64_t)(i0 + r) * w + c];
    }
    return;
  }
  for (int idx = tid; idx < PANEL_ROWS * w; idx += 256) {
    const int r = idx / w, c = idx % w;
    T[r][c] = (i0 + r < n) ? CD[(int64_t)(i0 + r) * w + c] : 0.f;
  }
  __syncthreads();
  if (i0 + PANEL_ROWS <= t0) {                // above: the rows t0 + c of N, written along i
    for (int idx = tid; idx < PANEL_ROWS * w; idx += 256) {
      const int c = idx / PANEL_ROWS, r = idx % PANEL_ROWS;
      N[(int64_t)(t0 + c) * ld + i0 + r] = T[r][c];
    }
    return;
  }
  for (int idx = tid; idx < PANEL_ROWS * w; idx += 256) {     // a block that meets the pivot rows
    const int r = idx / w, c = idx % w, l = i0 + r;
    if (l >= n) continue;
    if (l < t0) N[(int64_t)(t0 + c) * ld + l] = T[r][c];
    else if (l >= t0 + w) N[(int64_t)l * ld + t0 + c] = T[r][c];
    else if (c <= l - t0) N[(int64_t)l * ld + t0 + c] = (float)(-D[(l - t0) * w + c]);
  }
}

// A[i][j] = -A[max][min] for all i, j (turns the swept lower triangle -A^-1 into the full inverse)
__global__ void negate_mirror_kernel(float* __restrict__ A, int n) {
  int64_t tot = (int64_t)n * n;
  for (int64_t idx = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; idx < tot; idx += (int64_t)gridDim.x * blockDim.x) {
    int i = (int)(idx / n), j = (int)(idx % n);
    if (j <= i) continue;
    float v = -A[(int64_t)j * n + i];
    A[(int64_t)i * n + j] = v;     // upper gets the final value
  }
}
__global__ void negate_lower_kernel(float* __restrict__ A, int n) {
  int64_t tot = (int64_t)n * n;
  for (int64_t idx = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; idx < tot; idx += (int64_t)gridDim.x * blockDim.x) {
    int i = (int)(idx / n), j = (int)(idx % n);
    if (j <= i) A[idx] = -A[idx];
  }
}

hipError_t spd_inverse_inplace(float* A, int n, float* panel, float* panelD, double* small, int32_t* notpd_flag,
                               hipStream_t s) {
  float* panelB = panelD + (int64_t)n * INV_NB;   // caller provides 2*n*nb floats behind panelD
  for (int t0 = 0; t0 < n; t0 += INV_NB) {
    int w = (n - t0 < INV_NB) ? n - t0 : INV_NB;
    int rb = (n + PANEL_ROWS - 1) / PANEL_ROWS;
    hipLaunchKernelGGL(extract_panel_kernel, dim3(rb), dim3(256), 0, s, A, (int64_t)n, n, t0, w, panel);
    hipLaunchKernelGGL(inv_block_kernel, dim3(1), dim3(256), 0, s, panel, w, t0, small, notpd_flag);
    // true C*D for the pivot-row fix, and zeroed copies for the bulk update
    hipLaunchKernelGGL(panel_times_small_kernel, dim3((n + 15) / 16), dim3(256), 0, s, panel, small, n, w, t0, 1, panelD,
                       panelB);
    GemmArgs g{};
    g.M = n; g.N = n; g.K = w; g.A = panelD; g.lda = w; g.B = panelB; g.ldb = w; g.trans_b = 1;
    g.Cin = A; g.ldcin = n; g.C = A; g.ldc = n; g.alpha = -1.0; g.beta = 1.0; g.diag_add = 0.0; g.c_is_f64 = 0;
    g.lower_only = 1; g.acc_f32 = 1;
    hipError_t e = launch_gemm_f64acc(g, s);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(inv_fix_kernel, dim3(rb), dim3(256), 0, s, A, (int64_t)n, n, t0, w, panelD, small);
  }
  int64_t tot = (int64_t)n * n;
  int blocks = (int)((tot + 1023) / 1024); if (blocks > 131072) blocks = 131072;
  hipLaunchKernelGGL(negate_mirror_kernel, dim3(blocks), dim3(256), 0, s, A, n);
  hipLaunchKernelGGL(negate_lower_kernel, dim3(blocks), dim3(256), 0, s, A, n);
  return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// The same blocked sweep with the working matrix held in float64.  In float32 storage every one of the n / 128 panel
// updates rounds every entry again, and the inverse comes out with |I - H P| of 1e-5: it then needs a Newton-Schulz step
// whose residual I - H P is a full n^3 product with float64 sums (93 ms for n = 14336, a third of the state build).  Held
// in float64 the swept matrix is exact to 1e-12 and is rounded to float32 once: the same accuracy as after that step, for a
// rank-128 update that moves 16 bytes per entry instead of 8 (0.5 ms instead of 0.33 ms per panel).
// ------------------------------------------------------------------------------------------------
constexpr int PANEL_ROWS64 = 32;
__device__ __forceinline__ double nsym64(const double* __restrict__ N, int64_t ld, int i, int t) {
  return (i >= t) ? N[(int64_t)i * ld + t] : N[(int64_t)t * ld + i];
}
// A[i][j] = H[i][j] for j <= i (only the lower triangle is ever read)
__global__ void widen_lower_kernel(const float* __restrict__ H, int64_t ldh, int n, double* __restrict__ A) {
  const int64_t tot = (int64_t)n * n;
  for (int64_t idx = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; idx < tot; idx += (int64_t)gridDim.x * blockDim.x) {
    const int i = (int)(idx / n), j = (int)(idx % n);
    if (j <= i) A[idx] = (double)H[(int64_t)i * ldh + j];
  }
}
// P[i][j] = P[j][i] = float(-A[i][j]), j <= i: the swept lower triangle -H^-1 as the full float32 inverse.  One workgroup per
// 32 x 32 tile on or below the diagonal; the mirrored tile is written from shared memory so that both writes run along rows.
__global__ __launch_bounds__(256) void narrow_negate_mirror_kernel(const double* __restrict__ A, int n, float* __restrict__ P) {
  __shared__ float T[32][33];
  int bi = (int)((sqrtf(8.f * (float)blockIdx.x + 1.f) - 1.f) * 0.5f);
  while ((int64_t)(bi + 1) * (bi + 2) / 2 <= (int64_t)blockIdx.x) bi++;
  while ((int64_t)bi * (bi + 1) / 2 > (int64_t)blockIdx.x) bi--;
  const int bj = (int)(blockIdx.x - (int64_t)bi * (bi + 1) / 2);
  const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
#pragma unroll
  for (int k = 0; k < 4; k++) {
    const int r = ty + 8 * k, i = bi * 32 + r, j = bj * 32 + tx;
    T[r][tx] = (i < n && j <= i) ? (float)(-A[(int64_t)i * n + j]) : 0.f;
  }
  __syncthreads();
#pragma unroll
  for (int k = 0; k < 4; k++) {
    const int r = ty + 8 * k;
    const int i = bi * 32 + r, j = bj * 32 + tx;
    if (i < n && j < n) {
      if (j <= i) P[(int64_t)i * n + j] = T[r][tx];
      else if (bi == bj) P[(int64_t)i * n + j] = T[tx][r];       // upper part of a diagonal tile
    }
    if (bi != bj) {
      const int mi = bj * 32 + r, mj = bi * 32 + tx;             // the mirrored tile, row r of it = column r of this one
      if (mi < n && mj < n) P[(int64_t)mi * n + mj] = T[tx][r];
    }
  }
}
__global__ __launch_bounds__(256) void extract_panel64_kernel(const double* __restrict__ N, int64_t ld, int n, int t0, int w,
                                                               double* __restrict__ C) {
  __shared__ double T[PANEL_ROWS64][129];
  const int i0 = blockIdx.x * PANEL_ROWS64, tid = threadIdx.x;
  if (i0 >= t0 + w) {
    for (int idx = tid; idx < PANEL_ROWS64 * w; idx += 256) {
      const int r = idx / w, c = idx % w;
      if (i0 + r < n) C[(int64_t)(i0 + r) * w + c] = N[(int64_t)(i0 + r) * ld + t0 + c];
    }
    return;
  }
  if (i0 + PANEL_ROWS64 <= t0) {
    for (int idx = tid; idx < PANEL_ROWS64 * w; idx += 256) {
      const int c = idx / PANEL_ROWS64, r = idx % PANEL_ROWS64;
      T[r][c] = N[(int64_t)(t0 + c) * ld + i0 + r];
    }
  } else {
    for (int idx = tid; idx < PANEL_ROWS64 * w; idx += 256) {
      const int r = idx / w, c = idx % w;
      T[r][c] = (i0 + r < n) ? nsym64(N, ld, i0 + r, t0 + c) : 0.0;
    }
  }
  __syncthreads();
  for (int idx = tid; idx < PANEL_ROWS64 * w; idx += 256) {
    const int r = idx / w, c = idx % w;
    if (i0 + r < n) C[(int64_t)(i0 + r) * w + c] = T[r][c];
  }
}
__global__ __launch_bounds__(256) void inv_block64_kernel(const double* __restrict__ C, int w, int t0, double* __restrict__ D,
                                                           int32_t* notpd) {
  __shared__ double buf[64 * (INV_NB / 16)];
  for (int idx = threadIdx.x; idx < w * w; idx += 256) {
    const int r = idx / w, c = idx % w;
    D[idx] = C[(int64_t)(t0 + r) * w + c];
  }
  small_inverse<INV_NB / 16>(D, w, +1, notpd, buf);
}
// outz = C D and Cz = C, both with the pivot rows zeroed: the operands of the bulk update; the pivot-row fix reads outz
// outside the pivot rows only.  8 rows per workgroup, thread (h, c) sums 4 rows of column c, k ascending.
__global__ __launch_bounds__(256) void panel_times_small64_kernel(const double* __restrict__ C, const double* __restrict__ D, int n, int w,
                                                                   int t0, double* __restrict__ outz, double* __restrict__ Cz) {
  __shared__ double Csh[8][128];
  const int r0 = blockIdx.x * 8, tid = threadIdx.x;
  for (int idx = tid; idx < 8 * w; idx += 256) {
    const int r = idx / w, k = idx % w;
    Csh[r][k] = (r0 + r < n) ? C[(int64_t)(r0 + r) * w + k] : 0.0;
  }
  __syncthreads();
  const int c = tid & 127, h = tid >> 7;
  if (c >= w) return;
  double acc[4] = {0.0, 0.0, 0.0, 0.0};
  for (int k = 0; k < w; k++) {
    const double dv = D[k * w + c];
#pragma unroll
    for (int r = 0; r < 4; r++) acc[r] += Csh[h * 4 + r][k] * dv;
  }
#pragma unroll
  for (int r = 0; r < 4; r++) {
    const int i = r0 + h * 4 + r;
    if (i >= n) continue;
    const bool piv = i >= t0 && i < t0 + w;
    outz[(int64_t)i * w + c] = piv ? 0.0 : acc[r];
    Cz[(int64_t)i * w + c] = piv ? 0.0 : Csh[h * 4 + r][c];
  }
}
__global__ __launch_bounds__(256) void inv_fix64_kernel(double* __restrict__ N, int64_t ld, int n, int t0, int w,
                                                         const double* __restrict__ CD, const double* __restrict__ D) {
  __shared__ double T[PANEL_ROWS64][129];
  const int i0 = blockIdx.x * PANEL_ROWS64, tid = threadIdx.x;
  if (i0 >= t0 + w) {
    for (int idx = tid; idx < PANEL_ROWS64 * w; idx += 256) {
      const int r = idx / w, c = idx % w;
      if (i0 + r < n) N[(int64_t)(i0 + r) * ld + t0 + c] = CD[(int64_t)(i0 + r) * w + c];
    }
    return;
  }
  for (int idx = tid; idx < PANEL_ROWS64 * w; idx += 256) {
    const int r = idx / w, c = idx % w;
    T[r][c] = (i0 + r < n) ? CD[(int64_t)(i0 + r) * w + c] : 0.0;
  }
  __syncthreads();
  if (i0 + PANEL_ROWS64 <= t0) {
    for (int idx = tid; idx < PANEL_ROWS64 * w; idx += 256) {
      const int c = idx / PANEL_ROWS64, r = idx % PANEL_ROWS64;
      N[(int64_t)(t0 + c) * ld + i0 + r] = T[r][c];
    }
    return;
  }
  for (int idx = tid; idx < PANEL_ROWS64 * w; idx += 256) {
    const int r = idx / w, c = idx % w, l = i0 + r;
    if (l >= n) continue;
    if (l < t0) N[(int64_t)(t0 + c) * ld + l] = T[r][c];
    else if (l >= t0 + w) N[(int64_t)l * ld + t0 + c] = T[r][c];
    else if (c <= l - t0) N[(int64_t)l * ld + t0 + c] = -D[(l - t0) * w + c];
  }
}

// N[i][j] -= sum_k A[i][k] B[j][k] on the tiles of the lower block triangle; A, B: n x w float64 (w <= 128), N: n x n float64.
// One workgroup per half (128 rows x 64 columns) of a 128 x 128 tile, 8 waves x (2 x 2) v_mfma_f64_16x16x4_f64, the
// contraction in steps of 16 through LDS (rows of 144 and 80 doubles: the four k of a quarter-wave's operand read fall in
// different bank groups).  The workgroup's part of N (16 values per thread) is requested while the first products run and is
// there when the last one ends: with a whole tile per workgroup the registers held a quarter of it at a time, and four
// round trips to memory followed the products.  Tiles in 8 x 8 super-blocks per XCD, the two halves of a tile on one XCD.
typedef double swd4 __attribute__((ext_vector_type(4)));
constexpr int SW_LD = 144, SW_LDB = 80;
constexpr size_t SW_LDS_BYTES = (size_t)2 * 16 * (SW_LD + SW_LDB) * sizeof(double);
// part = 0: every tile of the triangle.  The pivot rows of A and B are zero, so the tiles of tile row / column pk (the
// pivot panel's) receive nothing and are always left alone (the pivot-row fix rewrites them, possibly meanwhile).
// part = 1: only tile row and tile column pk + 1, what the next panel is made of (two workgroups per tile, blockIdx / 2 =
// the other tile index); part = 2: everything but those.
__global__ __launch_bounds__(512, 2) void sweep_update64_kernel(const double* __restrict__ A, const double* __restrict__ B, int n, int w,
                                                                 double* __restrict__ N, int part, int pk) {
  extern __shared__ double sw_lds[];           // 56 KB: above the static limit, so taken dynamically
  double (*As)[16][SW_LD] = reinterpret_cast<double (*)[16][SW_LD]>(sw_lds);
  double (*Bs)[16][SW_LDB] = reinterpret_cast<double (*)[16][SW_LDB]>(sw_lds + 2 * 16 * SW_LD);
  int tm, tn, half;
  if (part == 1) {
    const int tiles = (n + 127) / 128, b = blockIdx.x >> 1, nx = pk + 1;
    half = blockIdx.x & 1;
    if (b >= tiles || nx >= tiles || b == pk) return;
    tm = (b <= nx) ? nx : b;
    tn = (b <= nx) ? b : nx;
  } else {
    const int tiles = (n + 127) / 128, nr = (tiles + 7) / 8;
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 4;
    half = (blockIdx.x >> 3) & 1;
    const int sb = (slot / 64) * 8 + xcd, within = slot % 64;
    if (sb >= nr * (nr + 1) / 2) return;
    int r = (int)((sqrtf(8.f * (float)sb + 1.f) - 1.f) * 0.5f);
    while ((r + 1) * (r + 2) / 2 <= sb) r++;
    while (r * (r + 1) / 2 > sb) r--;
    tm = r * 8 + within / 8;
    tn = (sb - r * (r + 1) / 2) * 8 + within % 8;
    if (tm >= tiles || tn > tm) return;
    if (tm == pk || tn == pk) return;
    if (part == 2 && (tm == pk + 1 || tn == pk + 1)) return;
  }
  const int m0 = tm * 128, n0 = tn * 128 + half * 64;
  if (n0 >= n) return;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, wm = wave >> 1, wn = wave & 1;   // wave tile: 32 rows x 32 columns
  const int lrow = tid >> 2, lk = (tid & 3) * 4;        // staging: thread = (row of the tile, quarter of the 16 k)
  const bool stage_b = lrow < 64;                       // B has 64 rows here
  const double* ap = (m0 + lrow < n) ? A + (int64_t)(m0 + lrow) * w : nullptr;
  const double* bp = (stage_b && n0 + lrow < n) ? B + (int64_t)(n0 + lrow) * w : nullptr;
  swd4 acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; i++)
#pragma unroll
    for (int j = 0; j < 2; j++) acc[i][j] = swd4{0.0, 0.0, 0.0, 0.0};
  double ra[4], rb[4];
  const int ktiles = (w + 15) / 16;
  const bool vec = (w & 3) == 0;       // then a thread's four k are inside or outside as a whole, and 32-byte aligned
  auto gload = [&](int kt) {
    const int k0 = kt * 16 + lk;
    if (vec) {
      if (ap && k0 < w) {
        const double2* p = reinterpret_cast<const double2*>(ap + k0);
        const double2 q0 = p[0], q1 = p[1];
        ra[0] = q0.x; ra[1] = q0.y; ra[2] = q1.x; ra[3] = q1.y;
      } else { ra[0] = ra[1] = ra[2] = ra[3] = 0.0; }
      if (bp && k0 < w) {
        const double2* p = reinterpret_cast<const double2*>(bp + k0);
        const double2 q0 = p[0], q1 = p[1];
        rb[0] = q0.x; rb[1] = q0.y; rb[2] = q1.x; rb[3] = q1.y;
      } else { rb[0] = rb[1] = rb[2] = rb[3] = 0.0; }
      return;
    }
#pragma unroll
    for (int e = 0; e < 4; e++) {
      const int k = k0 + e;
      ra[e] = (ap && k < w) ? ap[k] : 0.0;
      rb[e] = (bp && k < w) ? bp[k] : 0.0;
    }
  };
  auto sstore = [&](int buf) {
#pragma unroll
    for (int e = 0; e < 4; e++) As[buf][lk + e][lrow] = ra[e];
    if (stage_b) {
#pragma unroll
      for (int e = 0; e < 4; e++) Bs[buf][lk + e][lrow] = rb[e];
    }
  };
  // lane holds D[4 r + lane/16][lane%16] of each 16 x 16 tile
  const int rbase = m0 + wm * 32 + (lane >> 4), cbase = n0 + wn * 32 + (lane & 15);
  const bool whole = (m0 + 128 <= n && n0 + 64 <= n);
  double* nbase = N + (int64_t)rbase * n + cbase;       // dereferenced only where the row and column exist
  double cv[2][2][4];
#pragma unroll
  for (int i = 0; i < 2; i++)
#pragma unroll
    for (int j = 0; j < 2; j++)
#pragma unroll
      for (int r = 0; r < 4; r++) cv[i][j][r] = 0.0;
  if (ktiles > 0) { gload(0); sstore(0); }
  __syncthreads();
  if (whole && w == 128) {
    // The usual case.  The 16 values of N are requested two per stage, each pair behind the next stage's operands: the wait
    // for those operands at the end of a stage then covers the pair requested a stage earlier, and the requests to memory
    // run through the whole contraction instead of piling up at its start.
#pragma unroll
    for (int kt = 0; kt < 8; kt++) {
      const int buf = kt & 1;
      if (kt + 1 < 8) gload(kt + 1);
#pragma unroll
      for (int e = kt * 2; e < kt * 2 + 2; e++)
        cv[e >> 3][(e >> 2) & 1][e & 3] = nbase[(int64_t)((e >> 3) * 16 + 4 * (e & 3)) * n + ((e >> 2) & 1) * 16];
#pragma unroll
      for (int kk = 0; kk < 4; kk++) {
        const int k = kk * 4 + (lane >> 4);
        double a[2], b[2];
#pragma unroll
        for (int i = 0; i < 2; i++) a[i] = As[buf][k][wm * 32 + i * 16 + (lane & 15)];
#pragma unroll
        for (int j = 0; j < 2; j++) b[j] = Bs[buf][k][wn * 32 + j * 16 + (lane & 15)];
#pragma unroll
        for (int i = 0; i < 2; i++)
#pragma unroll
          for (int j = 0; j < 2; j++) acc[i][j] = __builtin_amdgcn_mfma_f64_16x16x4f64(a[i], b[j], acc[i][j], 0, 0, 0);
      }
      if (kt + 1 < 8) sstore(buf ^ 1);
      __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < 2; i++)
#pragma unroll
      for (int j = 0; j < 2; j++)
#pragma unroll
        for (int r = 0; r < 4; r++) nbase[(int64_t)(i * 16 + 4 * r) * n + j * 16] = cv[i][j][r] - acc[i][j][r];
    return;
  }
  for (int kt = 0; kt < ktiles; kt++) {
    const int buf = kt & 1;
    if (kt + 1 < ktiles) gload(kt + 1);
    if (kt == 0) {
      // requested behind the second stage's operands, so that no operand load queues up behind them before they are back
      if (whole) {
#pragma unroll
        for (int i = 0; i < 2; i++)
#pragma unroll
          for (int j = 0; j < 2; j++)
#pragma unroll
            for (int r = 0; r < 4; r++) cv[i][j][r] = nbase[(int64_t)(i * 16 + 4 * r) * n + j * 16];
      } else {
#pragma unroll
        for (int i = 0; i < 2; i++)
#pragma unroll
          for (int j = 0; j < 2; j++)
#pragma unroll
            for (int r = 0; r < 4; r++) {
              const int row = rbase + i * 16 + 4 * r, col = cbase + j * 16;
              cv[i][j][r] = (row < n && col < n) ? N[(int64_t)row * n + col] : 0.0;
            }
      }
    }
#pragma unroll
    for (int kk = 0; kk < 4; kk++) {
      const int k = kk * 4 + (lane >> 4);
      double a[2], b[2];
#pragma unroll
      for (int i = 0; i < 2; i++) a[i] = As[buf][k][wm * 32 + i * 16 + (lane & 15)];
#pragma unroll
      for (int j = 0; j < 2; j++) b[j] = Bs[buf][k][wn * 32 + j * 16 + (lane & 15)];
#pragma unroll
      for (int i = 0; i < 2; i++)
#pragma unroll
        for (int j = 0; j < 2; j++) acc[i][j] = __builtin_amdgcn_mfma_f64_16x16x4f64(a[i], b[j], acc[i][j], 0, 0, 0);
    }
    if (kt + 1 < ktiles) sstore(buf ^ 1);
    __syncthreads();
  }
  if (ktiles == 0) return;
  if (whole) {
#pragma unroll
    for (int i = 0; i < 2; i++)
#pragma unroll
      for (int j = 0; j < 2; j++)
#pragma unroll
        for (int r = 0; r < 4; r++) nbase[(int64_t)(i * 16 + 4 * r) * n + j * 16] = cv[i][j][r] - acc[i][j][r];
    return;
  }
#pragma unroll
  for (int i = 0; i < 2; i++)
#pragma unroll
    for (int j = 0; j < 2; j++)
#pragma unroll
      for (int r = 0; r < 4; r++) {
        const int row = rbase + i * 16 + 4 * r, col = cbase + j * 16;
        if (row < n && col < n) N[(int64_t)row * n + col] = cv[i][j][r] - acc[i][j][r];
      }
}

// P (n x n float32, full) = H^-1 for the SPD H (n x n float32, leading dimension ldh; only its lower triangle is read).
// A64: n x n float64 work matrix; panels: 5 n INV_NB float64; small: INV_NB^2 float64; notpd_flag as for spd_inverse_inplace.
// With a side stream the panel work of step k + 1 (extract, 128 x 128 inverse, panel x block: 0.2 ms during which one
// workgroup, then a few, have the chip to themselves) runs beside the bulk update of step k: the tiles the next panel is made
// of (tile row and column k + 1) are updated first by a launch of their own, the pivot rows of step k are fixed, and the
// rest of the update goes to the side stream.  Each tile sees the same operations in the same order either way.
hipError_t spd_inverse_f64(const float* H, int64_t ldh, int n, float* P, double* A64, double* panels, double* small,
                           int32_t* notpd_flag, hipStream_t s, const SideStream* side) {
  if (n <= 0) return hipSuccess;
  const int64_t tot = (int64_t)n * n;
  int blocks = (int)((tot + 1023) / 1024); if (blocks > 131072) blocks = 131072;
  hipLaunchKernelGGL(widen_lower_kernel, dim3(blocks), dim3(256), 0, s, H, ldh, n, A64);
  double* panel = panels;
  const size_t shmem = SW_LDS_BYTES;
  {
    const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(sweep_update64_kernel), hipFuncAttributeMaxDynamicSharedMemorySize, (int)shmem);
    if (e != hipSuccess) return e;
  }
  const int tiles = (n + 127) / 128, nr = (tiles + 7) / 8;
  const unsigned upd_grid = (unsigned)((nr * (nr + 1) / 2 + 7) / 8 * 8 * 64) * 2;      // two workgroups per tile
  const int rb = (n + PANEL_ROWS64 - 1) / PANEL_ROWS64;
  const bool two = side && side->stream && tiles > 2;
  hipError_t err;
  bool pending = false;              // a bulk update is running on the side stream
  for (int t0 = 0, k = 0; t0 < n; t0 += INV_NB, k++) {
    const int w = (n - t0 < INV_NB) ? n - t0 : INV_NB;
    // operand panels alternate: the bulk update of step k - 1 may still be reading the other pair
    double* panelDz = panels + (int64_t)(1 + 2 * (k & 1)) * n * INV_NB;
    double* panelCz = panelDz + (int64_t)n * INV_NB;
    hipLaunchKernelGGL(extract_panel64_kernel, dim3(rb), dim3(256), 0, s, A64, (int64_t)n, n, t0, w, panel);
    hipLaunchKernelGGL(inv_block64_kernel, dim3(1), dim3(256), 0, s, panel, w, t0, small, notpd_flag);
    hipLaunchKernelGGL(panel_times_small64_kernel, dim3((n + 7) / 8), dim3(256), 0, s, panel, small, n, w, t0, panelDz, panelCz);
    if (!two) {
      hipLaunchKernelGGL(sweep_update64_kernel, dim3(upd_grid), dim3(512), shmem, s, panelDz, panelCz, n, w, A64, 0, k);
      hipLaunchKernelGGL(inv_fix64_kernel, dim3(rb), dim3(256), 0, s, A64, (int64_t)n, n, t0, w, panelDz, small);
      continue;
    }
    // The bulk updates follow one another on the side stream without a gap: step k's needs its operands (ready here) and
    // step k - 1 on every tile it touches (the stream's order), nothing from this stream's later work.
    if ((err = hipEventRecord(side->fork, s)) != hipSuccess) return err;
    if ((err = hipStreamWaitEvent(side->stream, side->fork, 0)) != hipSuccess) return err;
    // This stream's next launch changes the next panel's tiles, which the bulk update of step k - 1 also does: it waits for
    // that one (the event's latest record), not for step k's, whose launch leaves those tiles out.
    if (pending && (err = hipStreamWaitEvent(s, side->join, 0)) != hipSuccess) return err;
    hipLaunchKernelGGL(sweep_update64_kernel, dim3(upd_grid), dim3(512), shmem, side->stream, panelDz, panelCz, n, w, A64, 2, k);
    if ((err = hipEventRecord(side->join, side->stream)) != hipSuccess) return err;
    pending = true;
    if (k + 1 < tiles) hipLaunchKernelGGL(sweep_update64_kernel, dim3(2 * tiles), dim3(512), shmem, s, panelDz, panelCz, n, w, A64, 1, k);
    // tile row and column k only: no launch of this step's update touches them, the next step's bulk update does (it is
    // enqueued behind an event that this stream records after the fix)
    hipLaunchKernelGGL(inv_fix64_kernel, dim3(rb), dim3(256), 0, s, A64, (int64_t)n, n, t0, w, panelDz, small);
  }
  if (pending && (err = hipStreamWaitEvent(s, side->join, 0)) != hipSuccess) return err;
  const int64_t t32 = (n + 31) / 32;
  hipLaunchKernelGGL(narrow_negate_mirror_kernel, dim3((unsigned)(t32 * (t32 + 1) / 2)), dim3(256), 0, s, A64, n, P);
  return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// scores: gram[h] = Z_h Z_h^T, dblk[h] = N_hh (float64), score[h] = Tr(gram_h |N_hh|^-1)
// ------------------------------------------------------------------------------------------------
// one workgroup per group; wave w takes the pairs (r, c), c <= r, in a fixed order, lanes over columns
__device__ void group_gram(const float* __restrict__ Zg, int q, int m, double* __restrict__ gram_h) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nw = blockDim.x >> 6;
  const int npairs = q * (q + 1) / 2;
  for (int pr = wave; pr < npairs; pr += nw) {
    int r = (int)((sqrtf(8.f * (float)pr + 1.f) - 1.f) * 0.5f);
    while ((r + 1) * (r + 2) / 2 <= pr) r++;
    while (r * (r + 1) / 2 > pr) r--;
    int c = pr - r * (r + 1) / 2;
    const float* zr = Zg + (int64_t)r * m;
    const float* zc = Zg + (int64_t)c * m;
    double v = 0;
    for (int col = lane; col < m; col += 64) v += (double)zr[col] * (double)zc[col];
    v = wave_sum(v);
    if (lane == 0) { gram_h[r * q + c] = v; gram_h[c * q + r] = v; }
  }
}

// groups of one row: gram[h] = |Z_h|^2 and dblk[h] = N_hh, one wave per row (four rows per workgroup), 16-byte loads
__global__ __launch_bounds__(256) void gram_dblk_q1_kernel(int d1, int m, const float* __restrict__ N, const float* __restrict__ Z,
                                                            double* __restrict__ gram, double* __restrict__ dblk) {
  const int h = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
  if (h >= d1) return;
  const float* z = Z + (int64_t)h * m;
  double v = 0;
  if ((m & 3) == 0) {
    const float4* z4 = reinterpret_cast<const float4*>(z);
    for (int c = lane; c < (m >> 2); c += 64) {
      const float4 x = z4[c];
      v += (double)x.x * (double)x.x + (double)x.y * (double)x.y + (double)x.z * (double)x.z + (double)x.w * (double)x.w;
    }
  } else {
    for (int c = lane; c < m; c += 64) v += (double)z[c] * (double)z[c];
  }
  v = wave_sum(v);
  if (lane == 0) { gram[h] = v; dblk[h] = (double)N[(int64_t)h * d1 + h]; }
}

// gram[h] = Z_h Z_h^T for every group: 16 x 16 outputs per workgroup (lower blocks only, mirrored), Z tiles of 64 columns in LDS
__global__ __launch_bounds__(256) void group_gram_kernel(TabDims d, const float* __restrict__ Z, double* __restrict__ gram,
                                                          const SearchCtrl* __restrict__ ctrl) {
  __shared__ float zr[16][65], zc[16][65];
  if (ctrl && ctrl->done) return;
  const int q = d.q, m = d.m, h = blockIdx.x, nb = (q + 15) / 16;
  int br = 0, bc = blockIdx.y;                      // linear index over the lower block triangle
  while (bc > br) { bc -= br + 1; br++; }
  if (br >= nb) return;
  const int tr = threadIdx.x >> 4, tc = threadIdx.x & 15;
  const int r = br * 16 + tr, c = bc * 16 + tc;
  const float* Zh = Z + (int64_t)h * q * m;
  double acc = 0;
  for (int c0 = 0; c0 < m; c0 += 64) {
    __syncthreads();
    for (int idx = threadIdx.x; idx < 16 * 64; idx += 256) {
      const int rr = idx >> 6, cc = idx & 63;
      const bool okc = c0 + cc < m;
      zr[rr][cc] = (okc && br * 16 + rr < q) ? Zh[(int64_t)(br * 16 + rr) * m + c0 + cc] : 0.f;
      zc[rr][cc] = (okc && bc * 16 + rr < q) ? Zh[(int64_t)(bc * 16 + rr) * m + c0 + cc] : 0.f;
    }
    __syncthreads();
#pragma unroll 16
    for (int k = 0; k < 64; k++) acc += (double)zr[tr][k] * (double)zc[tc][k];
  }
  if (r < q && c < q) {
    gram[(int64_t)h * q * q + r * q + c] = acc;
    gram[(int64_t)h * q * q + c * q + r] = acc;
  }
}

__global__ __launch_bounds__(256) void dblk_copy_kernel(TabDims d, const float* __restrict__ N, double* __restrict__ dblk) {
  const int h = blockIdx.x, q = d.q;
  for (int idx = threadIdx.x; idx < q * q; idx += 256) {
    int r = idx / q, c = idx % q;
    dblk[(int64_t)h * q * q + idx] = (double)nsym(N, d.d1, h * q + r, h * q + c);
  }
}

// score[h] = Tr(gram_h * (sigma * dblk_h)^-1), sigma = -1 for kept groups (N_hh = -P_hh), +1 otherwise.
// One workgroup of 64 threads per group; Cholesky in shared memory, then one column solve per thread.
__global__ __launch_bounds__(256) void score_kernel(TabDims d, const int32_t* __restrict__ kept,
                                                     const double* __restrict__ gram, const double* __restrict__ dblk,
                                                     double* __restrict__ score, SearchCtrl* ctrl, int skip_if_done) {
  extern __shared__ double sh[];   // A: q*q, then 256 doubles for the inverse
  __shared__ int32_t bad;
  __shared__ double red[4];
  if (skip_if_done && ctrl->done) return;          // a search iteration that changed nothing
  const int h = blockIdx.x, q = d.q, tid = threadIdx.x;
  const double sigma = kept[h] ? -1.0 : 1.0;
  if (q == 1) {
    if (tid == 0) {
      double a = sigma * dblk[h];
      if (!(a > 0.0)) { ctrl->notpd = 1; a = 1.0; }
      score[h] = gram[h] / a;
    }
    return;
  }
  // Tr(|N_hh|^-1 Z_h Z_h^T): inverse of the q x q block by Gauss-Jordan in registers, then the sum of the products with
  // the Gram block (both symmetric)
  double* A = sh;
  double* buf = sh + q * q;
  if (tid == 0) bad = 0;
  for (int idx = tid; idx < q * q; idx += 256) A[idx] = sigma * dblk[(int64_t)h * q * q + idx];
  small_inverse<4>(A, q, +1, &bad, buf);
  double contrib = 0;
  for (int idx = tid; idx < q * q; idx += 256) contrib += A[idx] * gram[(int64_t)h * q * q + idx];
  contrib = wave_sum(contrib);
  if ((tid & 63) == 0) red[tid >> 6] = contrib;
  __syncthreads();
  if (tid == 0) {
    score[h] = red[0] + red[1] + red[2] + red[3];
    if (bad) ctrl->notpd = 1;
  }
}
// groups of one row: one thread per group
__global__ __launch_bounds__(256) void score_q1_kernel(int p, const int32_t* __restrict__ kept, const double* __restrict__ gram,
                                                        const double* __restrict__ dblk, double* __restrict__ score,
                                                        SearchCtrl* ctrl, int skip_if_done) {
  if (skip_if_done && ctrl->done) return;
  const int h = blockIdx.x * 256 + threadIdx.x;
  if (h >= p) return;
  double a = (kept[h] ? -1.0 : 1.0) * dblk[h];
  if (!(a > 0.0)) { ctrl->notpd = 1; a = 1.0; }
  score[h] = gram[h] / a;
}
static void launch_score(const TabDims& d, const int32_t* kept, const double* gram, const double* dblk, double* score,
                         SearchCtrl* ctrl, int skip_if_done, hipStream_t s) {
  if (d.q == 1)
    hipLaunchKernelGGL(score_q1_kernel, dim3((d.p + 255) / 256), dim3(256), 0, s, d.p, kept, gram, dblk, score, ctrl, skip_if_done);
  else
    hipLaunchKernelGGL(score_kernel, dim3(d.p), dim3(256), (size_t)(d.q * d.q + 256) * 8, s, d, kept, gram, dblk, score, ctrl,
                       skip_if_done);
}

// the two halves of the refresh: the per-group Gram blocks and diagonal blocks (one pass over Z and the diagonal of N),
// then the scores from them; a caller may run the first half on another stream
hipError_t launch_refresh_blocks(const TabDims& d, const TabPtrs& t, hipStream_t s) {
  if (d.q == 1) {
    hipLaunchKernelGGL(gram_dblk_q1_kernel, dim3((d.d1 + 3) / 4), dim3(256), 0, s, d.d1, d.m, t.N, t.Z, t.gram, t.dblk);
  } else {
    const int nb = (d.q + 15) / 16;
    hipLaunchKernelGGL(group_gram_kernel, dim3(d.p, nb * (nb + 1) / 2), dim3(256), 0, s, d, t.Z, t.gram, (const SearchCtrl*)nullptr);
    hipLaunchKernelGGL(dblk_copy_kernel, dim3(d.p), dim3(256), 0, s, d, t.N, t.dblk);
  }
  return hipGetLastError();
}
hipError_t launch_refresh_from_blocks(const TabDims& d, const TabPtrs& t, hipStream_t s) {
  launch_score(d, t.kept, t.gram, t.dblk, t.score, t.ctrl, 0, s);
  return hipGetLastError();
}
hipError_t launch_refresh_scores(const TabDims& d, const TabPtrs& t, hipStream_t s) {
  const hipError_t e = launch_refresh_blocks(d, t, s);
  return e != hipSuccess ? e : launch_refresh_from_blocks(d, t, s);
}

// ------------------------------------------------------------------------------------------------
// one search iteration
// ------------------------------------------------------------------------------------------------
// argmin of the removal costs over kept groups, argmax of the addition gains over the others (lowest
// index on ties), and the relative gap to the second best of each.
__global__ __launch_bounds__(1024) void select_kernel(TabDims d, const int32_t* __restrict__ kept,
                                                       const double* __restrict__ score, SearchCtrl* ctrl, int forced_out,
                                                       int forced_in) {
  __shared__ double s_min1[1024], s_min2[1024], s_max1[1024], s_max2[1024];
  __shared__ int s_imin[1024], s_imax[1024];
  if (ctrl->done || ctrl->pause) return;
  const int tid = threadIdx.x;
  double mn1 = INFINITY, mn2 = INFINITY, mx1 = -INFINITY, mx2 = -INFINITY;
  int imn = -1, imx = -1;
  for (int h = tid; h < d.p; h += 1024) {     // ascending h per thread: strict comparisons keep the lowest index
    double v = score[h];
    if (kept[h]) {
      if (v < mn1) { mn2 = mn1; mn1 = v; imn = h; } else if (v < mn2) mn2 = v;
    } else {
      if (v > mx1) { mx2 = mx1; mx1 = v; imx = h; } else if (v > mx2) mx2 = v;
    }
  }
  s_min1[tid] = mn1; s_min2[tid] = mn2; s_imin[tid] = imn;
  s_max1[tid] = mx1; s_max2[tid] = mx2; s_imax[tid] = imx;
  __syncthreads();
  for (int o = 512; o > 0; o >>= 1) {
    if (tid < o) {
      {  // min side
        double a1 = s_min1[tid], a2 = s_min2[tid], b1 = s_min1[tid + o], b2 = s_min2[tid + o];
        int ia = s_imin[tid], ib = s_imin[tid + o];
        bool takeb = (ib >= 0) && (ia < 0 || b1 < a1 || (b1 == a1 && ib < ia));
        double n1 = takeb ? b1 : a1; int in_ = takeb ? ib : ia;
        double other1 = takeb ? a1 : b1;
        double n2 = fmin(fmin(a2, b2), other1);
        s_min1[tid] = n1; s_min2[tid] = n2; s_imin[tid] = in_;
      }
      {  // max side
        double a1 = s_max1[tid], a2 = s_max2[tid], b1 = s_max1[tid + o], b2 = s_max2[tid + o];
        int ia = s_imax[tid], ib = s_imax[tid + o];
        bool takeb = (ib >= 0) && (ia < 0 || b1 > a1 || (b1 == a1 && ib < ia));
        double n1 = takeb ? b1 : a1; int in_ = takeb ? ib : ia;
        double other1 = takeb ? a1 : b1;
        double n2 = fmax(fmax(a2, b2), other1);
        s_max1[tid] = n1; s_max2[tid] = n2; s_imax[tid] = in_;
      }
    }
    __syncthreads();
  }
  if (tid == 0) {
    int g = s_imin[0], j = s_imax[0];
    if (forced_out >= 0) { g = forced_out; j = forced_in; }
    if (g < 0 || j < 0 || (forced_out >= 0 && (!kept[g] || kept[j]))) { ctrl->done = 1; ctrl->g_out = -1; ctrl->g_in = -1; return; }
    ctrl->g_out = g; ctrl->g_in = j;
    double m1 = s_min1[0], m2 = s_min2[0], x1 = s_max1[0], x2 = s_max2[0];
    ctrl->gap_rem = isfinite(m2) ? fabs(m2 - m1) / fmax(fabs(m1), 1e-300) : INFINITY;
    ctrl->gap_add = isfinite(x2) ? fabs(x1 - x2) / fmax(fabs(x1), 1e-300) : INFINITY;
  }
}

// ------------------------------------------------------------------------------------------------
// Exact entering rule: with the leaving group g fixed, every candidate j is scored at the state WITHOUT g (Case 1 of
// Proposition 4.1 applied to the blocks the score needs, then eq. (impact) there), i.e. by the exact gain of the pair.
// Sweeping g out changes   N_jj -> N_jj - Y N_gj,   Z_j -> Z_j - Y Z_g,   Y = N_jg N_gg^-1,
// so with C_j = Z_j Z_g^T (exact_cross_kernel) the Gram of the new rows is
//   M_j = Z_j Z_j^T - Y C_j^T - C_j Y^T + Y (Z_g Z_g^T) Y^T          and the score is Tr(S'_j^-1 M_j).
// ------------------------------------------------------------------------------------------------
// cross[i][c] = <Z_i, Z_{g, c}> for every row i; one wave per row, Zg = the copy of the rows of g (q x m)
__global__ __launch_bounds__(256) void exact_cross_kernel(TabDims d, const float* __restrict__ Z, const float* __restrict__ Zg,
                                                           const SearchCtrl* __restrict__ ctrl, double* __restrict__ cross) {
  if (ctrl->done) return;
  const int lane = threadIdx.x & 63, row = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= d.d1) return;
  const float* zi = Z + (int64_t)row * d.m;
  for (int c = 0; c < d.q; c++) {
    const float* zg = Zg + (int64_t)c * d.m;
    double v = 0;
    for (int col = lane; col < d.m; col += 64) v += (double)zi[col] * (double)zg[col];
    v = wave_sum(v);
    if (lane == 0) cross[(int64_t)row * d.q + c] = v;
  }
}

// groups of one row: the score itself, one thread per group
__global__ __launch_bounds__(256) void exact_q1_kernel(TabDims d, const float* __restrict__ C1, const double* __restrict__ cross,
                                                        const double* __restrict__ gram, const double* __restrict__ dblk,
                                                        const int32_t* __restrict__ kept, SearchCtrl* ctrl,
                                                        double* __restrict__ xscore) {
  if (ctrl->done) return;
  const int h = blockIdx.x * 256 + threadIdx.x;
  if (h >= d.p) return;
  if (kept[h]) { xscore[h] = 0.0; return; }
  const int g = ctrl->g_out;
  const double x = (double)C1[h], y = x / dblk[g];
  double sp = dblk[h] - y * x;
  const double mj = gram[h] - 2.0 * y * cross[h] + y * y * gram[g];
  if (!(sp > 0.0)) { ctrl->notpd = 1; sp = 1.0; }
  xscore[h] = mj / sp;
}

// groups of q rows: the blocks S'_j -> xdblk[j], M_j -> xgram[j] (kept groups: -I and 0, which score_kernel turns into 0)
__global__ __launch_bounds__(256) void exact_blocks_kernel(TabDims d, const float* __restrict__ C1, const double* __restrict__ cross,
                                                            const double* __restrict__ gram, const double* __restrict__ dblk,
                                                            const int32_t* __restrict__ kept, SearchCtrl* ctrl,
                                                            double* __restrict__ xgram, double* __restrict__ xdblk) {
  extern __shared__ double xsh[];      // Dg (later T = Y Gg), X, Y: q*q each; then 256 doubles for the inverse
  __shared__ int32_t bad;
  if (ctrl->done) return;
  const int q = d.q, qq = q * q, tid = threadIdx.x, j = blockIdx.x, g = ctrl->g_out, j0 = j * q;
  double* outS = xdblk + (int64_t)j * qq;
  double* outM = xgram + (int64_t)j * qq;
  if (kept[j]) {
    for (int idx = tid; idx < qq; idx += 256) { outS[idx] = (idx / q == idx % q) ? -1.0 : 0.0; outM[idx] = 0.0; }
    return;
  }
  double* Dg = xsh; double* X = xsh + qq; double* Y = xsh + 2 * qq; double* buf = xsh + 3 * qq;
  if (tid == 0) bad = 0;
  for (int idx = tid; idx < qq; idx += 256) {
    Dg[idx] = dblk[(int64_t)g * qq + idx];                                   // N_gg, negative definite
    X[idx] = (double)C1[(int64_t)(j0 + idx / q) * q + idx % q];              // N(j_r, g_c)
  }
  small_inverse<4>(Dg, q, -1, &bad, buf);
  for (int idx = tid; idx < qq; idx += 256) {                                // Y = X Dg
    const int r = idx / q, c = idx % q;
    double v = 0;
    for (int k = 0; k < q; k++) v += X[r * q + k] * Dg[k * q + c];
    Y[idx] = v;
  }
  __syncthreads();
  const double* Gg = gram + (int64_t)g * qq;
  const double* Gj = gram + (int64_t)j * qq;
  const double* Sj = dblk + (int64_t)j * qq;
  const double* Cj = cross + (int64_t)j0 * q;                               // C_j[r][c] = <Z_{j,r}, Z_{g,c}>
  double* Tm = Dg;                                                           // T = Y Gg overwrites Dg
  for (int idx = tid; idx < qq; idx += 256) {
    const int r = idx / q, c = idx % q;
    double sv = 0;
    for (int k = 0; k < q; k++) sv += Y[r * q + k] * X[c * q + k];
    outS[idx] = Sj[idx] - sv;                                                // S' = N_jj - Y N_gj
  }
  __syncthreads();
  for (int idx = tid; idx < qq; idx += 256) {
    const int r = idx / q, c = idx % q;
    double v = 0;
    for (int k = 0; k < q; k++) v += Y[r * q + k] * Gg[k * q + c];
    Tm[idx] = v;
  }
  __syncthreads();
  for (int idx = tid; idx < qq; idx += 256) {
    const int r = idx / q, c = idx % q;
    double v = Gj[idx];
    for (int k = 0; k < q; k++) v += -Y[r * q + k] * Cj[c * q + k] - Cj[r * q + k] * Y[c * q + k] + Tm[r * q + k] * Y[c * q + k];
    outM[idx] = v;
  }
  if (tid == 0 && bad) ctrl->notpd = 1;
}

// entering group = argmax of the exact scores over the groups outside the kept set (lowest index on ties)
__global__ __launch_bounds__(1024) void select_in_kernel(TabDims d, const int32_t* __restrict__ kept,
                                                          const double* __restrict__ xscore, SearchCtrl* ctrl) {
  __shared__ double s1[1024], s2[1024];
  __shared__ int si[1024];
  if (ctrl->done) return;
  const int tid = threadIdx.x;
  double mx1 = -INFINITY, mx2 = -INFINITY;
  int imx = -1;
  for (int h = tid; h < d.p; h += 1024) {
    if (kept[h]) continue;
    const double v = xscore[h];
    if (v > mx1) { mx2 = mx1; mx1 = v; imx = h; } else if (v > mx2) mx2 = v;
  }
  s1[tid] = mx1; s2[tid] = mx2; si[tid] = imx;
  __syncthreads();
  for (int o = 512; o > 0; o >>= 1) {
    if (tid < o) {
      const double a1 = s1[tid], a2 = s2[tid], b1 = s1[tid + o], b2 = s2[tid + o];
      const int ia = si[tid], ib = si[tid + o];
      const bool takeb = (ib >= 0) && (ia < 0 || b1 > a1 || (b1 == a1 && ib < ia));
      s1[tid] = takeb ? b1 : a1; si[tid] = takeb ? ib : ia;
      s2[tid] = fmax(fmax(a2, b2), takeb ? a1 : b1);
    }
    __syncthreads();
  }
  if (tid == 0) {
    if (si[0] < 0) { ctrl->done = 1; ctrl->g_out = -1; ctrl->g_in = -1; return; }
    ctrl->g_in = si[0];
    ctrl->gap_add = isfinite(s2[0]) ? fabs(s1[0] - s2[0]) / fmax(fabs(s1[0]), 1e-300) : INFINITY;
  }
}

// panels of both pivots and copies of their Z rows
__global__ __launch_bounds__(256) void extract_pair_kernel(TabDims d, const float* __restrict__ N, const float* __restrict__ Z,
                                                            const SearchCtrl* __restrict__ ctrl, float* __restrict__ C1,
                                                            float* __restrict__ C2, float* __restrict__ Zg,
                                                            float* __restrict__ Zj, const int32_t* __restrict__ single) {
  if (ctrl->done) return;
  // single != nullptr: removal of the one group *single (no group enters); the second pivot then aliases the first
  const int q = d.q, g0 = (single ? *single : ctrl->g_out) * q, j0 = (single ? *single : ctrl->g_in) * q;
  int i = blockIdx.x * 256 + threadIdx.x;
  if (i < d.d1) {
    for (int c = 0; c < q; c++) {
      C1[(int64_t)i * q + c] = nsym(N, d.d1, i, g0 + c);
      C2[(int64_t)i * q + c] = nsym(N, d.d1, i, j0 + c);
    }
  }
  int64_t tot = (int64_t)q * d.m;
  for (int64_t idx = blockIdx.x * 256 + threadIdx.x; idx < tot; idx += (int64_t)gridDim.x * 256) {
    Zg[idx] = Z[(int64_t)g0 * d.m + idx];
    Zj[idx] = Z[(int64_t)j0 * d.m + idx];
  }
}

// q x q algebra of the pair (the exact change of the objective and the acceptance test follow in pair_cols_kernel and
// pair_accept_kernel).
// small layout (doubles, each q*q): [0] Dg, [1] Njg, [2] M1 = Dg Ngj, [3] Dj' , [4] W2Dj = -M1 Dj', [5] scratch
__global__ __launch_bounds__(256) void pair_small_kernel(TabDims d, const float* __restrict__ C1, const float* __restrict__ C2,
                                                          double* __restrict__ small, SearchCtrl* ctrl,
                                                          const int32_t* __restrict__ single) {
  extern __shared__ double psm[];      // three q x q matrices, then 256 doubles for the inverses
  __shared__ int32_t bad;
  if (ctrl->done) return;
  const int q = d.q, qq = q * q, tid = threadIdx.x;
  const int g0 = (single ? *single : ctrl->g_out) * q, j0 = (single ? *single : ctrl->g_in) * q;
  double* Dg = small; double* Njg = small + qq; double* M1 = small + 2 * qq; double* Dj = small + 3 * qq;
  double* W2Dj = small + 4 * qq;
  double* X0 = psm; double* X1 = psm + qq; double* X2 = psm + 2 * qq; double* buf = psm + 3 * qq;
  if (tid == 0) bad = 0;
  for (int idx = tid; idx < qq; idx += 256) {
    const int r = idx / q, c = idx % q;
    X0[idx] = (double)C1[(int64_t)(g0 + r) * q + c];          // N_gg
    const double njg = (double)C1[(int64_t)(j0 + r) * q + c]; // N(j_r, g_c)
    Njg[idx] = njg;
    X1[c * q + r] = njg;                                      // N_gj = Njg^T
  }
  small_inverse<4>(X0, q, -1, &bad, buf);                    // kept pivot: N_gg = -P_gg is negative definite
  for (int idx = tid; idx < qq; idx += 256) Dg[idx] = X0[idx];
  if (single) {
    // Case 1 alone: with M1 = 0 and Dj' = 0 every term of the second sweep below vanishes
    for (int idx = tid; idx < qq; idx += 256) { M1[idx] = 0.0; Dj[idx] = 0.0; W2Dj[idx] = 0.0; Njg[idx] = 0.0; }
  } else {
    for (int idx = tid; idx < qq; idx += 256) {              // M1 = Dg N_gj
      const int r = idx / q, c = idx % q;
      double v = 0;
      for (int k = 0; k < q; k++) v += X0[r * q + k] * X1[k * q + c];
      X2[idx] = v; M1[idx] = v;
    }
    __syncthreads();
    for (int idx = tid; idx < qq; idx += 256) {              // X0 = N_jg
      const int r = idx / q, c = idx % q;
      X0[idx] = X1[c * q + r];
    }
    __syncthreads();
    for (int idx = tid; idx < qq; idx += 256) {              // N'_jj = N_jj - N_jg M1  (into X1, N_gj being spent)
      const int r = idx / q, c = idx % q;
      double v = 0;
      for (int k = 0; k < q; k++) v += X0[r * q + k] * X2[k * q + c];
      Dj[idx] = (double)C2[(int64_t)(j0 + r) * q + c] - v;
    }
    __syncthreads();
    for (int idx = tid; idx < qq; idx += 256) X1[idx] = Dj[idx];
    small_inverse<4>(X1, q, +1, &bad, buf);                  // entering pivot: Schur complement, positive definite
    for (int idx = tid; idx < qq; idx += 256) {              // W2Dj = W2 Dj', W2 = N'_gj = -M1
      const int r = idx / q, c = idx % q;
      double v = 0;
      for (int k = 0; k < q; k++) v -= X2[r * q + k] * X1[k * q + c];
      W2Dj[idx] = v; Dj[idx] = X1[idx];
    }
  }
  __syncthreads();
  if (tid == 0) { ctrl->delta = 0.0; if (bad) ctrl->notpd = 1; }
}

// Column phase of the pair: rZ1 = Dg Zg ; Z'j = Zj - Njg rZ1 ; rZ2 = Dj' Z'j (both written in place of Zg, Zj) and
// delta = -<Zg, rZ1> - <Z'j, rZ2>, one partial sum per workgroup in dpart (added up in a fixed order by the acceptance
// kernel, so that the result does not depend on scheduling).  16 columns x 16 row slots per workgroup; the three q x q
// matrices and the column tiles live in LDS.
constexpr int PC_COLS = 16;
__global__ __launch_bounds__(256) void pair_cols_kernel(TabDims d, float* __restrict__ Zg, float* __restrict__ Zj,
                                                         const double* __restrict__ small, SearchCtrl* ctrl, double* __restrict__ dpart) {
  extern __shared__ double pcs[];   // Dg, Njg, Dj (q*q each), ta, tb (q*16 each)
  __shared__ double red[4];
  if (ctrl->done) return;
  const int q = d.q, qq = q * q, m = d.m, tid = threadIdx.x;
  double* Dg = pcs; double* Njg = pcs + qq; double* Dj = pcs + 2 * qq; double* ta = pcs + 3 * qq; double* tb = ta + q * PC_COLS;
  for (int idx = tid; idx < qq; idx += 256) { Dg[idx] = small[idx]; Njg[idx] = small[qq + idx]; Dj[idx] = small[3 * qq + idx]; }
  const int c = tid & 15, slot = tid >> 4, col = blockIdx.x * PC_COLS + c;
  const bool live = col < m;
  for (int r = slot; r < q; r += 16) ta[r * PC_COLS + c] = live ? (double)Zg[(int64_t)r * m + col] : 0.0;
  __syncthreads();
  double part = 0;
  for (int r = slot; r < q; r += 16) {                       // tb = Dg zg
    double v = 0;
    for (int k = 0; k < q; k++) v += Dg[r * q + k] * ta[k * PC_COLS + c];
    tb[r * PC_COLS + c] = v;
    part -= ta[r * PC_COLS + c] * v;
  }
  __syncthreads();
  for (int r = slot; r < q; r += 16) {                       // ta = z'j = zj - Njg tb ; rZ1 out
    double v = live ? (double)Zj[(int64_t)r * m + col] : 0.0;
    for (int k = 0; k < q; k++) v -= Njg[r * q + k] * tb[k * PC_COLS + c];
    ta[r * PC_COLS + c] = v;
    if (live) Zg[(int64_t)r * m + col] = (float)tb[r * PC_COLS + c];
  }
  __syncthreads();
  for (int r = slot; r < q; r += 16) {                       // rZ2 = Dj' z'j
    double v = 0;
    for (int k = 0; k < q; k++) v += Dj[r * q + k] * ta[k * PC_COLS + c];
    part -= ta[r * PC_COLS + c] * v;
    if (live) Zj[(int64_t)r * m + col] = (float)v;
  }
  part = wave_sum(part);
  if ((tid & 63) == 0) red[tid >> 6] = part;
  __syncthreads();
  if (tid == 0) dpart[blockIdx.x] = red[0] + red[1] + red[2] + red[3];
}

// the acceptance test and the trace
__global__ __launch_bounds__(64) void pair_accept_kernel(SearchCtrl* ctrl, int always_accept, int32_t* trace_out, int32_t* trace_in,
                                                         float* trace_gap, double* trace_obj, const int32_t* __restrict__ single,
                                                         const double* __restrict__ dpart, int nparts) {
  if (ctrl->done) return;
  // lane l adds the partial sums l, l + 64, ... in that order; then the fixed tree of the wave sum
  double dsum = 0;
  for (int b = threadIdx.x; b < nparts; b += 64) dsum += dpart[b];
  dsum = wave_sum(dsum);
  if (threadIdx.x != 0) return;
  const double delta = dsum;
  ctrl->delta = delta;
  const int it = ctrl->iters;
  const bool bad = ctrl->notpd != 0;
  const bool ok = !bad && (always_accept || delta < -ctrl->rel_tol * ctrl->obj);
  ctrl->iters = it + 1;
  if (single) { ctrl->g_out = *single; ctrl->g_in = -1; }
  if (ok) { ctrl->obj += delta; ctrl->accepted += 1; } else { ctrl->done = 1; }
  if (trace_out) trace_out[it] = ctrl->g_out;
  if (trace_in) trace_in[it] = ctrl->g_in;
  if (trace_gap) { trace_gap[2 * it] = (float)ctrl->gap_rem; trace_gap[2 * it + 1] = (float)ctrl->gap_add; }
  if (trace_obj) trace_obj[it] = ctrl->obj;
}

// bulk panels: P1 = C1, P2 = C2 - C1 M1, P1D = P1 Dg, P2D = P2 Dj', with the rows of both pivots zeroed;
// and the new pivot rows of N and Z, the diagonal blocks (float64) and the membership flags.
// T1 (d1 x q) = true C1 Dg, T2 (d1 x q) = true (C2 - C1 M1) Dj' for rows outside the pivots.
__global__ __launch_bounds__(256) void pair_panels_kernel(TabDims d, const float* __restrict__ C1, const float* __restrict__ C2,
                                                           const double* __restrict__ small, const SearchCtrl* __restrict__ ctrl,
                                                           float* __restrict__ P1, float* __restrict__ P2,
                                                           float* __restrict__ P1D, float* __restrict__ P2D,
                                                           const int32_t* __restrict__ single) {
  // one thread per (row, column): 4 rows x 64 columns per workgroup; the q x q matrices are read from global memory
  // (consecutive threads, consecutive columns), the row's own coefficients go through LDS
  __shared__ double sc1[4][64], sc2[4][64];
  if (ctrl->done) return;
  const int q = d.q, qq = q * q;
  const int g0 = (single ? *single : ctrl->g_out) * q, j0 = (single ? *single : ctrl->g_in) * q;
  const double* Dg = small; const double* M1 = small + 2 * qq; const double* Dj = small + 3 * qq;
  const int lr = threadIdx.x >> 6, c = threadIdx.x & 63;
  const int i = blockIdx.x * 4 + lr;
  const bool live = (i < d.d1) && (c < q);
  const bool piv = (i >= g0 && i < g0 + q) || (i >= j0 && i < j0 + q);
  sc1[lr][c] = live ? (double)C1[(int64_t)i * q + c] : 0.0;
  __syncthreads();
  double v = 0;
  if (live) {
    v = (double)C2[(int64_t)i * q + c];
    for (int k = 0; k < q; k++) v -= sc1[lr][k] * M1[k * q + c];
  }
  sc2[lr][c] = v;
  __syncthreads();
  if (!live) return;
  const int64_t o = (int64_t)i * q + c;
  if (piv) { P1[o] = 0.f; P2[o] = 0.f; P1D[o] = 0.f; P2D[o] = 0.f; return; }
  double v1 = 0, v2 = 0;
  for (int k = 0; k < q; k++) { v1 += sc1[lr][k] * Dg[k * q + c]; v2 += sc2[lr][k] * Dj[k * q + c]; }
  P1[o] = (float)sc1[lr][c];
  P2[o] = (float)sc2[lr][c];
  P1D[o] = (float)v1;
  P2D[o] = (float)v2;
}

// New pivot rows (after both sweeps), for every l outside the pivots:
//   N''(g_r, l) = -P1D[l][r] - sum_c W2[r][c] P2D[l][c],  W2 = -M1     (= -P1D[l][r] + sum_c M1[r][c] P2D[l][c])
//   N''(j_r, l) =  P2D[l][r]
// pivot-pivot blocks: N''_gg = -Dg - W2 Dj' W2^T, N''_jj = -Dj', N''(g, j) = W2 Dj'.
// Z''_g = -rZ1 + M1 rZ2, Z''_j = rZ2.  Diagonal blocks of the other groups are updated in float64.
__global__ __launch_bounds__(256) void pair_fix_kernel(TabDims d, float* __restrict__ N, float* __restrict__ Z,
                                                        const float* __restrict__ P1, const float* __restrict__ P2,
                                                        const float* __restrict__ P1D, const float* __restrict__ P2D,
                                                        const float* __restrict__ rZ1, const float* __restrict__ rZ2,
                                                        const double* __restrict__ small, const SearchCtrl* __restrict__ ctrl,
                                                        double* __restrict__ dblk, int32_t* __restrict__ kept,
                                                        const int32_t* __restrict__ single) {
  if (ctrl->done) return;
  const int q = d.q, qq = q * q, m = d.m;
  const int g = single ? *single : ctrl->g_out, j = single ? g : ctrl->g_in, g0 = g * q, j0 = j * q;
  const double* Dg = small; const double* M1 = small + 2 * qq; const double* Dj = small + 3 * qq; const double* W2Dj = small + 4 * qq;
  const int64_t ld = d.d1;
  {
    // one thread per (row l, pivot row r): 4 rows x 64 pivot rows per workgroup
    const int l = blockIdx.x * 4 + (threadIdx.x >> 6), r = threadIdx.x & 63;
    if (l < d.d1 && r < q) {
      const bool in_g = (l >= g0 && l < g0 + q), in_j = (l >= j0 && l < j0 + q);
      if (!in_g && !in_j) {
        double vg = -(double)P1D[(int64_t)l * q + r];
        for (int c = 0; c < q; c++) vg += M1[r * q + c] * (double)P2D[(int64_t)l * q + c];
        const float vj = P2D[(int64_t)l * q + r];
        const int gr = g0 + r, jr = j0 + r;
        if (l < gr) N[(int64_t)gr * ld + l] = (float)vg; else N[(int64_t)l * ld + gr] = (float)vg;
        if (!single) { if (l < jr) N[(int64_t)jr * ld + l] = vj; else N[(int64_t)l * ld + jr] = vj; }
      }
    }
  }
  // pivot-pivot blocks and flags: first workgroup
  if (blockIdx.x == 0) {
    for (int idx = threadIdx.x; idx < qq; idx += 256) {
      int r = idx / q, c = idx % q;
      double ngg = -Dg[idx];
      for (int k = 0; k < q; k++) ngg += W2Dj[r * q + k] * M1[c * q + k];     // - W2 Dj' W2^T = + (W2 Dj') M1^T
      double njj = -Dj[idx];
      double ngj = W2Dj[idx];                                                  // N''(g_r, j_c)
      dblk[(int64_t)g * qq + idx] = ngg;
      if (c <= r) N[(int64_t)(g0 + r) * ld + g0 + c] = (float)ngg;
      if (single) continue;
      dblk[(int64_t)j * qq + idx] = njj;
      if (c <= r) N[(int64_t)(j0 + r) * ld + j0 + c] = (float)njj;
      if (g0 > j0) N[(int64_t)(g0 + r) * ld + j0 + c] = (float)ngj;
      else N[(int64_t)(j0 + c) * ld + g0 + r] = (float)ngj;
    }
    if (threadIdx.x == 0) { kept[g] = 0; if (!single) kept[j] = 1; }
  }
  // Z rows of the pivots
  int64_t tot = (int64_t)q * m;
  for (int64_t idx = blockIdx.x * 256 + threadIdx.x; idx < tot; idx += (int64_t)gridDim.x * 256) {
    int r = (int)(idx / m), col = (int)(idx % m);
    double vg = -(double)rZ1[idx];
    for (int c = 0; c < q; c++) vg += M1[r * q + c] * (double)rZ2[(int64_t)c * m + col];
    Z[(int64_t)(g0 + r) * m + col] = (float)vg;
    if (!single) Z[(int64_t)(j0 + r) * m + col] = rZ2[idx];
  }
}

// float64 diagonal blocks of the groups outside the pivots: dblk[h] -= P1D_h P1_h^T + P2D_h P2_h^T.  One workgroup per group.
__global__ __launch_bounds__(256) void pair_dblk_kernel(TabDims d, const float* __restrict__ P1, const float* __restrict__ P2,
                                                         const float* __restrict__ P1D, const float* __restrict__ P2D,
                                                         const SearchCtrl* __restrict__ ctrl, double* __restrict__ dblk,
                                                         const int32_t* __restrict__ single) {
  extern __shared__ float pds[];   // the four q x q panels of this group
  if (ctrl->done) return;
  const int q = d.q, qq = q * q, h = blockIdx.x;
  const int g = single ? *single : ctrl->g_out, j = single ? g : ctrl->g_in;
  if (h == g || h == j) return;    // pivot groups get their blocks in pair_fix_kernel
  // rows of b1, b2 are read by neighbouring threads: stride q + 1 keeps them in different LDS banks
  const int qs = q + 1;
  float* a1 = pds; float* a2 = pds + qq; float* b1 = pds + 2 * qq; float* b2 = b1 + q * qs;
  const int64_t base = (int64_t)h * qq;
  for (int idx = threadIdx.x; idx < qq; idx += 256) {
    const int r = idx / q, c = idx % q;
    a1[idx] = P1D[base + idx]; a2[idx] = P2D[base + idx]; b1[r * qs + c] = P1[base + idx]; b2[r * qs + c] = P2[base + idx];
  }
  __syncthreads();
  for (int idx = threadIdx.x; idx < qq; idx += 256) {
    const int r = idx / q, c = idx % q;
    double v = 0;
    for (int k = 0; k < q; k++) v += (double)a1[r * q + k] * (double)b1[c * qs + k] + (double)a2[r * q + k] * (double)b2[c * qs + k];
    dblk[base + idx] -= v;
  }
}

// bulk update of the lower triangle: N[i][l] -= sum_c P1D[i][c] P1[l][c] + P2D[i][c] P2[l][c]
// generic in q; 64 x 64 tiles, 16 x 16 threads, 4 x 4 elements per thread, panels staged in LDS 16 columns at a time.
__global__ __launch_bounds__(256) void update_N_kernel(TabDims d, float* __restrict__ N, const float* __restrict__ P1,
                                                        const float* __restrict__ P2, const float* __restrict__ P1D,
                                                        const float* __restrict__ P2D, const SearchCtrl* __restrict__ ctrl) {
  if (ctrl->done) return;
  const int tr = blockIdx.y, tc = blockIdx.x;
  if (tc > tr) return;
  __shared__ float sRD[2][64][17];   // P1D / P2D rows of this tile
  __shared__ float sC[2][64][17];    // P1 / P2 rows of the column range
  const int q = d.q, n = d.d1;
  const int ty = threadIdx.x >> 4, tx = threadIdx.x & 15;
  const int i0 = tr * 64, l0 = tc * 64;
  float acc[4][4] = {};
  for (int c0 = 0; c0 < q; c0 += 16) {
    int cw = (q - c0 < 16) ? q - c0 : 16;
    __syncthreads();
    for (int idx = threadIdx.x; idx < 64 * 16; idx += 256) {
      int r = idx >> 4, c = idx & 15;
      bool okc = c < cw;
      int ri = i0 + r, rl = l0 + r;
      sRD[0][r][c] = (okc && ri < n) ? P1D[(int64_t)ri * q + c0 + c] : 0.f;
      sRD[1][r][c] = (okc && ri < n) ? P2D[(int64_t)ri * q + c0 + c] : 0.f;
      sC[0][r][c] = (okc && rl < n) ? P1[(int64_t)rl * q + c0 + c] : 0.f;
      sC[1][r][c] = (okc && rl < n) ? P2[(int64_t)rl * q + c0 + c] : 0.f;
    }
    __syncthreads();
    for (int c = 0; c < cw; c++) {
      float a1[4], a2[4], b1[4], b2[4];
#pragma unroll
      for (int u = 0; u < 4; u++) { a1[u] = sRD[0][ty * 4 + u][c]; a2[u] = sRD[1][ty * 4 + u][c]; b1[u] = sC[0][tx * 4 + u][c]; b2[u] = sC[1][tx * 4 + u][c]; }
#pragma unroll
      for (int u = 0; u < 4; u++)
#pragma unroll
        for (int v = 0; v < 4; v++) acc[u][v] += a1[u] * b1[v] + a2[u] * b2[v];
    }
  }
#pragma unroll
  for (int u = 0; u < 4; u++) {
    int i = i0 + ty * 4 + u;
    if (i >= n) continue;
#pragma unroll
    for (int v = 0; v < 4; v++) {
      int l = l0 + tx * 4 + v;
      if (l <= i) N[(int64_t)i * n + l] -= acc[u][v];
    }
  }
}

// q = 1 fast path of the bulk update: N[i][l] -= a1[i]*b1[l] + a2[i]*b2[l] on the lower triangle.
// One workgroup streams a 32-row x 1024-column slab: each thread owns 4 consecutive columns and keeps their
// coefficients in registers while it walks down the rows.
__global__ __launch_bounds__(256) void update_N_q1_kernel(int n, float* __restrict__ N, const float* __restrict__ P1,
                                                           const float* __restrict__ P2, const float* __restrict__ P1D,
                                                           const float* __restrict__ P2D, const SearchCtrl* __restrict__ ctrl) {
  if (ctrl->done) return;
  const int r0 = blockIdx.y * 32, c0 = blockIdx.x * 1024;
  if (c0 > r0 + 31) return;
  const int c = c0 + threadIdx.x * 4;
  if (c >= n) return;
  const int rend = (r0 + 32 < n) ? r0 + 32 : n;
  if (c + 3 < n && (n & 3) == 0) {
    const float4 b1 = *reinterpret_cast<const float4*>(P1 + c);
    const float4 b2 = *reinterpret_cast<const float4*>(P2 + c);
#pragma unroll 4
    for (int i = r0; i < rend; i++) {
      if (c > i) continue;
      const float a1 = P1D[i], a2 = P2D[i];
      float4* p = reinterpret_cast<float4*>(N + (int64_t)i * n + c);
      float4 v = *p;
      v.x -= a1 * b1.x + a2 * b2.x;
      v.y -= a1 * b1.y + a2 * b2.y;
      v.z -= a1 * b1.z + a2 * b2.z;
      v.w -= a1 * b1.w + a2 * b2.w;
      *p = v;
    }
  } else {
    for (int i = r0; i < rend; i++)
      for (int u = 0; u < 4; u++) {
        int l = c + u;
        if (l < n && l <= i) N[(int64_t)i * n + l] -= P1D[i] * P1[l] + P2D[i] * P2[l];
      }
  }
}

// Z rows of one group: Z[i][:] -= sum_c P1[i][c] rZ1[c][:] + P2[i][c] rZ2[c][:], then gram[h] = Z_h Z_h^T.
__global__ __launch_bounds__(256) void update_Z_kernel(TabDims d, float* __restrict__ Z, const float* __restrict__ P1,
                                                        const float* __restrict__ P2, const float* __restrict__ rZ1,
                                                        const float* __restrict__ rZ2, double* __restrict__ gram,
                                                        const SearchCtrl* __restrict__ ctrl) {
  if (ctrl->done) return;
  const int h = blockIdx.x, q = d.q, m = d.m;
  float* Zh = Z + (int64_t)h * q * m;
  if (q == 1) {
    const float a1 = P1[h], a2 = P2[h];
    double v = 0;
    if ((m & 3) == 0) {                        // rows are 16-byte aligned: four columns per load
      float4* Z4 = reinterpret_cast<float4*>(Zh);
      const float4* r1 = reinterpret_cast<const float4*>(rZ1);
      const float4* r2 = reinterpret_cast<const float4*>(rZ2);
      for (int c4 = threadIdx.x; c4 < (m >> 2); c4 += 256) {
        float4 z = Z4[c4];
        const float4 x = r1[c4], y = r2[c4];
        z.x -= a1 * x.x + a2 * y.x; z.y -= a1 * x.y + a2 * y.y; z.z -= a1 * x.z + a2 * y.z; z.w -= a1 * x.w + a2 * y.w;
        Z4[c4] = z;
        v += (double)z.x * (double)z.x + (double)z.y * (double)z.y + (double)z.z * (double)z.z + (double)z.w * (double)z.w;
      }
    } else {
      for (int col = threadIdx.x; col < m; col += 256) {
        float z = Zh[col] - (a1 * rZ1[col] + a2 * rZ2[col]);
        Zh[col] = z;
        v += (double)z * (double)z;
      }
    }
    __shared__ double red[4];
    v = wave_sum(v);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
    __syncthreads();
    if (threadIdx.x == 0) gram[h] = red[0] + red[1] + red[2] + red[3];
    return;
  }
  for (int64_t idx = threadIdx.x; idx < (int64_t)q * m; idx += 256) {
    int r = (int)(idx / m), col = (int)(idx % m);
    const float* p1 = P1 + (int64_t)(h * q + r) * q;
    const float* p2 = P2 + (int64_t)(h * q + r) * q;
    float acc = 0.f;
    for (int c = 0; c < q; c++) acc += p1[c] * rZ1[(int64_t)c * m + col] + p2[c] * rZ2[(int64_t)c * m + col];
    Zh[idx] -= acc;
  }
  __syncthreads();
  group_gram(Zh, q, m, gram + (int64_t)h * q * q);
}

// The `take` kept groups with the smallest removal cost (ascending cost, lowest index on ties) -> pick[0..take), and
// the relative gap between the costliest of them and the cheapest kept group left out -> *gap (inf if none is left).
// One workgroup; take <= 64.
// side 1: the same for the groups outside the kept set with the LARGEST addition gain (descending gain).
__global__ __launch_bounds__(1024) void greedy_pick_kernel(TabDims d, const int32_t* __restrict__ kept,
                                                            const double* __restrict__ score, int take,
                                                            int32_t* __restrict__ pick, float* __restrict__ gap,
                                                            const SearchCtrl* __restrict__ ctrl, int side) {
  __shared__ double s_v[1024];
  __shared__ int s_i[1024];
  __shared__ int chosen[65];
  __shared__ double chosen_v[65];
  if (ctrl->done || ctrl->pause) return;
  const int tid = threadIdx.x;
  for (int round = 0; round <= take; round++) {
    double best = INFINITY;
    int ib = -1;
    for (int h = tid; h < d.p; h += 1024) {
      if ((kept[h] != 0) != (side == 0)) continue;
      bool used = false;
      for (int c = 0; c < round; c++) used |= (chosen[c] == h);
      if (used) continue;
      const double v = side ? -score[h] : score[h];
      if (ib < 0 || v < best) { best = v; ib = h; }        // ascending h per thread: strict comparison keeps the lowest index
    }
    s_v[tid] = best; s_i[tid] = ib;
    __syncthreads();
    for (int o = 512; o > 0; o >>= 1) {
      if (tid < o) {
        const double b1 = s_v[tid + o]; const int ib2 = s_i[tid + o];
        const double a1 = s_v[tid]; const int ia = s_i[tid];
        if (ib2 >= 0 && (ia < 0 || b1 < a1 || (b1 == a1 && ib2 < ia))) { s_v[tid] = b1; s_i[tid] = ib2; }
      }
      __syncthreads();
    }
    if (tid == 0) { chosen[round] = s_i[0]; chosen_v[round] = s_v[0]; }
    __syncthreads();
  }
  if (tid < take) pick[tid] = chosen[tid];
  if (tid == 0) {
    const double edge = chosen_v[take - 1];
    *gap = (chosen[take] >= 0) ? (float)(fabs(chosen_v[take] - edge) / fmax(fabs(edge), 1e-300)) : INFINITY;
  }
}

// The same selection for p <= 1024 * KMAX groups with the eligible scores held in registers: every round is a local scan, a
// shuffle reduction per wave and one more over the 16 wave records, instead of another pass over memory.
template <int KMAX>
__global__ __launch_bounds__(1024) void greedy_pick_reg_kernel(TabDims d, const int32_t* __restrict__ kept,
                                                                const double* __restrict__ score, int take,
                                                                int32_t* __restrict__ pick, float* __restrict__ gap,
                                                                const SearchCtrl* __restrict__ ctrl, int side) {
  __shared__ double w_v[16];
  __shared__ int w_i[16];
  __shared__ int chosen[65];
  __shared__ double chosen_v[65];
  if (ctrl->done || ctrl->pause) return;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  double v[KMAX];
#pragma unroll
  for (int k = 0; k < KMAX; k++) {
    const int h = tid + 1024 * k;
    v[k] = INFINITY;
    if (h < d.p && ((kept[h] != 0) == (side == 0))) v[k] = side ? -score[h] : score[h];
  }
  for (int round = 0; round <= take; round++) {
    double best = INFINITY;
    int ib = -1;
#pragma unroll
    for (int k = 0; k < KMAX; k++)
      if (v[k] < best) { best = v[k]; ib = tid + 1024 * k; }      // ascending index per thread: strict comparison keeps the lowest
    for (int o = 32; o > 0; o >>= 1) {
      const double b1 = __shfl_down(best, o, 64);
      const int i2 = __shfl_down(ib, o, 64);
      if (i2 >= 0 && (ib < 0 || b1 < best || (b1 == best && i2 < ib))) { best = b1; ib = i2; }
    }
    if (lane == 0) { w_v[wave] = best; w_i[wave] = ib; }
    __syncthreads();
    if (wave == 0) {
      best = lane < 16 ? w_v[lane] : INFINITY;
      ib = lane < 16 ? w_i[lane] : -1;
      for (int o = 8; o > 0; o >>= 1) {
        const double b1 = __shfl_down(best, o, 64);
        const int i2 = __shfl_down(ib, o, 64);
        if (i2 >= 0 && (ib < 0 || b1 < best || (b1 == best && i2 < ib))) { best = b1; ib = i2; }
      }
      if (lane == 0) { chosen[round] = ib; chosen_v[round] = best; }
    }
    __syncthreads();
    const int c = chosen[round];
    if (c >= 0 && (c & 1023) == tid) {
#pragma unroll
      for (int k = 0; k < KMAX; k++) if (k == (c >> 10)) v[k] = INFINITY;
    }
  }
  if (tid < take) pick[tid] = chosen[tid];
  if (tid == 0) {
    const double edge = chosen_v[take - 1];
    *gap = (chosen[take] >= 0) ? (float)(fabs(chosen_v[take] - edge) / fmax(fabs(edge), 1e-300)) : INFINITY;
  }
}

hipError_t launch_greedy_pick(const TabDims& d, const TabPtrs& t, int take, int32_t* pick, float* gap, hipStream_t s, int side) {
  if (take < 1 || take > 64) return hipErrorInvalidValue;
  if (d.p <= 1024 * 32)
    hipLaunchKernelGGL(greedy_pick_reg_kernel<32>, dim3(1), dim3(1024), 0, s, d, t.kept, t.score, take, pick, gap, t.ctrl, side);
  else
    hipLaunchKernelGGL(greedy_pick_kernel, dim3(1), dim3(1024), 0, s, d, t.kept, t.score, take, pick, gap, t.ctrl, side);
  return hipGetLastError();
}

// Z[i][:] -= sum_c P1[i][c] rZ1[c][:] + P2[i][c] rZ2[c][:] for groups of more than one row: one row x 256 columns per
// workgroup (the row's 2q coefficients are uniform loads); the group Grams follow in group_gram_kernel.
__global__ __launch_bounds__(256) void update_Z_rows_kernel(TabDims d, float* __restrict__ Z, const float* __restrict__ P1,
                                                             const float* __restrict__ P2, const float* __restrict__ rZ1,
                                                             const float* __restrict__ rZ2, const SearchCtrl* __restrict__ ctrl) {
  if (ctrl->done) return;
  const int q = d.q, m = d.m, i = blockIdx.x, col = blockIdx.y * 256 + threadIdx.x;
  if (col >= m) return;
  const float* p1 = P1 + (int64_t)i * q;
  const float* p2 = P2 + (int64_t)i * q;
  float acc = 0.f;
  for (int c = 0; c < q; c++) acc += p1[c] * rZ1[(int64_t)c * m + col] + p2[c] * rZ2[(int64_t)c * m + col];
  Z[(int64_t)i * m + col] -= acc;
}

hipError_t launch_select(const TabDims& d, const TabPtrs& t, int forced_out, int forced_in, hipStream_t s) {
  hipLaunchKernelGGL(select_kernel, dim3(1), dim3(1024), 0, s, d, t.kept, t.score, t.ctrl, forced_out, forced_in);
  return hipGetLastError();
}

hipError_t launch_search_iteration(const TabDims& d, const TabPtrs& t, int forced_out, int forced_in, int always_accept,
                                   hipStream_t s, hipEvent_t* ev, const int32_t* single, int exact_in) {
  const int q = d.q;
  const int rb = (d.d1 + 255) / 256;
  const size_t pc_lds = (size_t)(3 * q * q + 2 * q * PC_COLS) * 8;
  if (pc_lds > 65536) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(pair_cols_kernel), hipFuncAttributeMaxDynamicSharedMemorySize, (int)pc_lds);
    if (e != hipSuccess) return e;
  }
  if (!single) hipLaunchKernelGGL(select_kernel, dim3(1), dim3(1024), 0, s, d, t.kept, t.score, t.ctrl, forced_out, forced_in);
  hipLaunchKernelGGL(extract_pair_kernel, dim3(rb), dim3(256), 0, s, d, t.N, t.Z, t.ctrl, t.C1, t.C2, t.rZ1, t.rZ2, single);
  if (exact_in && !single && forced_out < 0) {
    // the leaving group stands; choose the entering one by the exact gain of the pair and extract its panel again
    hipLaunchKernelGGL(exact_cross_kernel, dim3((d.d1 + 3) / 4), dim3(256), 0, s, d, t.Z, t.rZ1, t.ctrl, t.cross);
    if (q == 1) {
      hipLaunchKernelGGL(exact_q1_kernel, dim3((d.p + 255) / 256), dim3(256), 0, s, d, t.C1, t.cross, t.gram, t.dblk, t.kept, t.ctrl,
                         t.xscore);
    } else {
      const size_t xb_lds = (size_t)(3 * q * q + 256) * 8;
      if (xb_lds > 65536) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(exact_blocks_kernel), hipFuncAttributeMaxDynamicSharedMemorySize, (int)xb_lds);
        if (e != hipSuccess) return e;
      }
      hipLaunchKernelGGL(exact_blocks_kernel, dim3(d.p), dim3(256), xb_lds, s, d, t.C1, t.cross, t.gram, t.dblk, t.kept, t.ctrl,
                         t.xgram, t.xdblk);
      launch_score(d, t.kept, t.xgram, t.xdblk, t.xscore, t.ctrl, 1, s);
    }
    hipLaunchKernelGGL(select_in_kernel, dim3(1), dim3(1024), 0, s, d, t.kept, t.xscore, t.ctrl);
    hipLaunchKernelGGL(extract_pair_kernel, dim3(rb), dim3(256), 0, s, d, t.N, t.Z, t.ctrl, t.C1, t.C2, t.rZ1, t.rZ2, single);
  }
  const size_t ps_lds = (size_t)(3 * q * q + 256) * 8;
  if (ps_lds > 65536) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(pair_small_kernel), hipFuncAttributeMaxDynamicSharedMemorySize, (int)ps_lds);
    if (e != hipSuccess) return e;
  }
  hipLaunchKernelGGL(pair_small_kernel, dim3(1), dim3(256), ps_lds, s, d, t.C1, t.C2, t.small, t.ctrl, single);
  const int ncb = (d.m + PC_COLS - 1) / PC_COLS;
  hipLaunchKernelGGL(pair_cols_kernel, dim3(ncb), dim3(256), pc_lds, s, d, t.rZ1, t.rZ2, t.small, t.ctrl, t.dpart);
  hipLaunchKernelGGL(pair_accept_kernel, dim3(1), dim3(64), 0, s, t.ctrl, always_accept, t.trace_out, t.trace_in, t.trace_gap,
                     t.trace_obj, single, t.dpart, ncb);
  // bulk panels go to C1D/C2D (times D) and to two further panels stored behind them
  float* P1 = t.C1D + (int64_t)2 * d.d1 * q;
  float* P2 = P1 + (int64_t)d.d1 * q;
  float* P1D = t.C1D;
  float* P2D = t.C2D;
  hipLaunchKernelGGL(pair_panels_kernel, dim3((d.d1 + 3) / 4), dim3(256), 0, s, d, t.C1, t.C2, t.small, t.ctrl, P1, P2, P1D, P2D,
                     single);
  hipLaunchKernelGGL(pair_fix_kernel, dim3((d.d1 + 3) / 4), dim3(256), 0, s, d, t.N, t.Z, P1, P2, P1D, P2D, t.rZ1, t.rZ2, t.small,
                     t.ctrl, t.dblk, t.kept, single);
  hipLaunchKernelGGL(pair_dblk_kernel, dim3(d.p), dim3(256), (size_t)(4 * q * q + 2 * q) * 4, s, d, P1, P2, P1D, P2D, t.ctrl, t.dblk, single);
  if (ev) hipEventRecord(ev[0], s);
  if (q == 1) {
    dim3 grid((d.d1 + 1023) / 1024, (d.d1 + 31) / 32);
    hipLaunchKernelGGL(update_N_q1_kernel, grid, dim3(256), 0, s, d.d1, t.N, P1, P2, P1D, P2D, t.ctrl);
  } else {
    int tiles = (d.d1 + 63) / 64;
    hipLaunchKernelGGL(update_N_kernel, dim3(tiles, tiles), dim3(256), 0, s, d, t.N, P1, P2, P1D, P2D, t.ctrl);
  }
  if (ev) hipEventRecord(ev[1], s);
  if (q == 1) {
    hipLaunchKernelGGL(update_Z_kernel, dim3(d.p), dim3(256), 0, s, d, t.Z, P1, P2, t.rZ1, t.rZ2, t.gram, t.ctrl);
  } else {
    const int nb = (q + 15) / 16;
    hipLaunchKernelGGL(update_Z_rows_kernel, dim3(d.d1, (d.m + 255) / 256), dim3(256), 0, s, d, t.Z, P1, P2, t.rZ1, t.rZ2, t.ctrl);
    hipLaunchKernelGGL(group_gram_kernel, dim3(d.p, nb * (nb + 1) / 2), dim3(256), 0, s, d, t.Z, t.gram, t.ctrl);
  }
  if (ev) hipEventRecord(ev[2], s);
  launch_score(d, t.kept, t.gram, t.dblk, t.score, t.ctrl, 1, s);
  return hipGetLastError();
}

}  // namespace osscar
