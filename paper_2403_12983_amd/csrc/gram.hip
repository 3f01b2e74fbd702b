// Quadratic-form construction (Section 3, dense-layer paragraph): H = X^T X accumulated over chunks of
// calibration rows, then the ridge, G = H W and c0.
//
// gram_bf16_kernel: SYRK-style product on the lower-triangle tiles of H with v_mfma_f32_32x32x16_bf16.
//   Both MFMA operands are column panels of the same row-major chunk Xc (rows = tokens), so every lane
//   needs 8 consecutive TOKENS of one column in a register quad.  Threads load 8 x 8 blocks (8 tokens x 8
//   columns, 16-byte row segments), transpose them in registers and store one 16-byte packet per column
//   into LDS in [token-group][column][8 tokens] order; MFMA operands are then single ds_read_b128.
//   The float32 MFMA accumulators are folded into float64 accumulators every FLUSH_ROWS tokens and the
//   tile is added to the float64 H once per chunk, so the result is accurate to float32 rounding.
#include "internal.h"

namespace osscar {

typedef float f16v __attribute__((ext_vector_type(16)));
typedef __bf16 bf8 __attribute__((ext_vector_type(8)));

constexpr int GBK = 64;            // tokens per LDS stage
constexpr int FLUSH_ROWS = 1024;   // tokens between folds of the float32 accumulators into float64

template <int WT>  // WT x WT MFMA tiles per wave; workgroup tile = 64*WT
__global__ __launch_bounds__(256) void gram_bf16_kernel(const uint16_t* __restrict__ X, int64_t n_c, int64_t ldx,
                                                         int d1, double* __restrict__ H64, int splits) {
  constexpr int TS = 64 * WT;
  constexpr int CG = TS / 8;                 // column groups of 8 per panel
  constexpr int BLOCKS_PER_PANEL = 8 * CG;   // 8 x 8 blocks per stage per panel
  constexpr int PER_THREAD = (2 * BLOCKS_PER_PANEL + 255) / 256;
  extern __shared__ uint4 lds[];             // [2 buffers][2 panels][8 kgroups][TS] packets of 16 bytes

  // tile index over the lower triangle
  int t = blockIdx.x;
  int tm = (int)((sqrtf(8.f * (float)t + 1.f) - 1.f) * 0.5f);
  while ((tm + 1) * (tm + 2) / 2 <= t) tm++;
  while (tm * (tm + 1) / 2 > t) tm--;
  const int tn = t - tm * (tm + 1) / 2;
  const bool diag = (tm == tn);
  const int i0 = tm * TS, j0 = tn * TS;

  // token range of this split
  const int64_t rows_per = ((n_c + splits - 1) / splits + GBK - 1) / GBK * GBK;
  const int64_t r_begin = (int64_t)blockIdx.y * rows_per;
  const int64_t r_end = (r_begin + rows_per < n_c) ? r_begin + rows_per : n_c;
  if (r_begin >= r_end) return;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;

  f16v acc[WT][WT];
  double acc64[WT][WT][16];
#pragma unroll
  for (int a = 0; a < WT; a++)
#pragma unroll
    for (int b = 0; b < WT; b++) {
#pragma unroll
      for (int r = 0; r < 16; r++) { acc[a][b][r] = 0.f; acc64[a][b][r] = 0.0; }
    }

  uint4 stage[PER_THREAD][8];   // raw rows of this thread's 8 x 8 blocks

  auto gload = [&](int64_t r0) {
#pragma unroll
    for (int u = 0; u < PER_THREAD; u++) {
      int blk = tid + u * 256;              // 0 .. 2*BLOCKS_PER_PANEL
      int panel = blk / BLOCKS_PER_PANEL;
      int rem = blk % BLOCKS_PER_PANEL;
      int kg = rem / CG, cg = rem % CG;
      int col = (panel == 0 ? i0 : j0) + cg * 8;
      bool live = (blk < 2 * BLOCKS_PER_PANEL) && (col < d1) && !(panel == 1 && diag);
#pragma unroll
      for (int r = 0; r < 8; r++) {
        int64_t row = r0 + kg * 8 + r;
        if (live && row < r_end)
          stage[u][r] = *reinterpret_cast<const uint4*>(X + row * ldx + col);
        else
          stage[u][r] = uint4{0, 0, 0, 0};
      }
    }
  };
  auto sstore = [&](int buf) {
#pragma unroll
    for (int u = 0; u < PER_THREAD; u++) {
      int blk = tid + u * 256;
      if (blk >= 2 * BLOCKS_PER_PANEL) continue;
      int panel = blk / BLOCKS_PER_PANEL;
      int rem = blk % BLOCKS_PER_PANEL;
      int kg = rem / CG, cg = rem % CG;
      if (panel == 1 && diag) continue;
      uint4* base = lds + ((buf * 2 + panel) * 8 + kg) * TS + cg * 8;
      const uint32_t* in[8];
#pragma unroll
      for (int r = 0; r < 8; r++) in[r] = reinterpret_cast<const uint32_t*>(&stage[u][r]);
#pragma unroll
      for (int d = 0; d < 4; d++) {      // dword d of a row holds columns 2d (low half) and 2d+1 (high half)
        uint4 lo, hi;                    // packets of columns 2d and 2d+1: tokens 0..7
        lo.x = (in[0][d] & 0xFFFFu) | (in[1][d] << 16);
        lo.y = (in[2][d] & 0xFFFFu) | (in[3][d] << 16);
        lo.z = (in[4][d] & 0xFFFFu) | (in[5][d] << 16);
        lo.w = (in[6][d] & 0xFFFFu) | (in[7][d] << 16);
        hi.x = (in[0][d] >> 16) | (in[1][d] & 0xFFFF0000u);
        hi.y = (in[2][d] >> 16) | (in[3][d] & 0xFFFF0000u);
        hi.z = (in[4][d] >> 16) | (in[5][d] & 0xFFFF0000u);
        hi.w = (in[6][d] >> 16) | (in[7][d] & 0xFFFF0000u);
        base[2 * d] = lo;
        base[2 * d + 1] = hi;
      }
    }
  };
  auto fold = [&]() {
#pragma unroll
    for (int a = 0; a < WT; a++)
#pragma unroll
      for (int b = 0; b < WT; b++)
#pragma unroll
        for (int r = 0; r < 16; r++) { acc64[a][b][r] += (double)acc[a][b][r]; acc[a][b][r] = 0.f; }
  };

  gload(r_begin);
  sstore(0);
  __syncthreads();
  int since_flush = 0;
  int buf = 0;
  for (int64_t r0 = r_begin; r0 < r_end; r0 += GBK) {
    const bool more = (r0 + GBK < r_end);
    if (more) gload(r0 + GBK);
    const uint4* pa = lds + (buf * 2 + 0) * 8 * TS;
    const uint4* pb = diag ? pa : lds + (buf * 2 + 1) * 8 * TS;
#pragma unroll
    for (int ks = 0; ks < GBK / 16; ks++) {
      const int kg = ks * 2 + (lane >> 5);
      bf8 fa[WT], fb[WT];
#pragma unroll
      for (int a = 0; a < WT; a++) {
        uint4 v = pa[kg * TS + wm * (32 * WT) + a * 32 + (lane & 31)];
        fa[a] = *reinterpret_cast<bf8*>(&v);
      }
#pragma unroll
      for (int b = 0; b < WT; b++) {
        uint4 v = pb[kg * TS + wn * (32 * WT) + b * 32 + (lane & 31)];
        fb[b] = *reinterpret_cast<bf8*>(&v);
      }
#pragma unroll
      for (int a = 0; a < WT; a++)
#pragma unroll
        for (int b = 0; b < WT; b++)
          acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[a], fb[b], acc[a][b], 0, 0, 0);
    }
    since_flush += GBK;
    if (since_flush >= FLUSH_ROWS) { fold(); since_flush = 0; }
    if (more) sstore(buf ^ 1);
    __syncthreads();
    buf ^= 1;
  }
  fold();

  // H64 tile += acc64.  C layout of the 32 x 32 MFMA: lane holds rows (r/4)*8 + (lane/32)*4 + r%4, column lane%32.
#pragma unroll
  for (int a = 0; a < WT; a++)
#pragma unroll
    for (int b = 0; b < WT; b++)
#pragma unroll
      for (int r = 0; r < 16; r++) {
        int row = i0 + wm * (32 * WT) + a * 32 + (r >> 2) * 8 + (lane >> 5) * 4 + (r & 3);
        int col = j0 + wn * (32 * WT) + b * 32 + (lane & 31);
        if (row < d1 && col < d1) {
          double* dst = H64 + (int64_t)row * d1 + col;
          if (splits > 1) unsafeAtomicAdd(dst, acc64[a][b][r]);
          else *dst += acc64[a][b][r];
        }
      }
}

hipError_t launch_gram_bf16(const void* Xc, int64_t n_c, int64_t ldx, int d1, double* H64, hipStream_t s) {
  if (n_c <= 0) return hipSuccess;
  constexpr int WT = 2, TS = 64 * WT;
  int tm = (d1 + TS - 1) / TS;
  int tiles = tm * (tm + 1) / 2;
  int splits = 1;
  if (tiles < 1024) {
    splits = (2048 + tiles - 1) / tiles;
    int64_t maxs = (n_c + 511) / 512;
    if (splits > maxs) splits = (int)maxs;
    if (splits < 1) splits = 1;
  }
  size_t shmem = (size_t)2 * 2 * 8 * TS * 16;
  hipLaunchKernelGGL(gram_bf16_kernel<WT>, dim3(tiles, splits), dim3(256), shmem, s,
                     reinterpret_cast<const uint16_t*>(Xc), n_c, ldx, d1, H64, splits);
  return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// Helpers of the generic (any shape, float32 or bfloat16 input) path and of finalize.
// ------------------------------------------------------------------------------------------------
__device__ __forceinline__ float bf16_bits_to_float(uint16_t b) { return __uint_as_float(((uint32_t)b) << 16); }

// Xt[c][r] = X[r][c] as float32 (32 x 32 tiles through LDS)
__global__ __launch_bounds__(256) void transpose_to_f32_kernel(const void* __restrict__ X, int is_bf16, int64_t rows,
                                                                int64_t cols, int64_t ldx, float* __restrict__ Xt,
                                                                int64_t ldxt) {
  __shared__ float tile[32][33];
  int64_t c0 = (int64_t)blockIdx.x * 32, r0 = (int64_t)blockIdx.y * 32;
  int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
  for (int i = ty; i < 32; i += 8) {
    int64_t r = r0 + i, c = c0 + tx;
    float v = 0.f;
    if (r < rows && c < cols)
      v = is_bf16 ? bf16_bits_to_float(reinterpret_cast<const uint16_t*>(X)[r * ldx + c])
                  : reinterpret_cast<const float*>(X)[r * ldx + c];
    tile[i][tx] = v;
  }
  __syncthreads();
  for (int i = ty; i < 32; i += 8) {
    int64_t c = c0 + i, r = r0 + tx;
    if (c < cols && r < rows) Xt[c * ldxt + r] = tile[tx][i];
  }
}

hipError_t launch_transpose_to_f32(const void* X, int is_bf16, int64_t rows, int64_t cols, int64_t ldx, float* Xt,
                                   int64_t ldxt, hipStream_t s) {
  if (rows <= 0 || cols <= 0) return hipSuccess;
  dim3 grid((unsigned)((cols + 31) / 32), (unsigned)((rows + 31) / 32));
  hipLaunchKernelGGL(transpose_to_f32_kernel, grid, dim3(256), 0, s, X, is_bf16, rows, cols, ldx, Xt, ldxt);
  return hipGetLastError();
}

__global__ void convert_to_f32_kernel(const void* __restrict__ src, int is_bf16, int64_t rows, int64_t cols, int64_t lds_,
                                      float* __restrict__ dst) {
  int64_t n = rows * cols;
  for (int64_t i = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x) {
    int64_t r = i / cols, c = i % cols;
    dst[i] = is_bf16 ? bf16_bits_to_float(reinterpret_cast<const uint16_t*>(src)[r * lds_ + c])
                     : reinterpret_cast<const float*>(src)[r * lds_ + c];
  }
}

hipError_t launch_convert_to_f32(const void* src, int is_bf16, int64_t rows, int64_t cols, int64_t lds_, float* dst,
                                 hipStream_t s) {
  if (rows * cols <= 0) return hipSuccess;
  int blocks = (int)((rows * cols + 1023) / 1024);
  if (blocks > 65536) blocks = 65536;
  hipLaunchKernelGGL(convert_to_f32_kernel, dim3(blocks), dim3(256), 0, s, src, is_bf16, rows, cols, lds_, dst);
  return hipGetLastError();
}

// H[i][j] = float(H64[max(i,j)][min(i,j)] + (i == j ? lam : 0))
__global__ void finalize_H_kernel(const double* __restrict__ H64, float* __restrict__ H, int d1,
                                  const double* __restrict__ lam_dev) {
  const double lam = lam_dev ? lam_dev[0] : 0.0;
  int64_t n = (int64_t)d1 * d1;
  for (int64_t idx = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; idx < n; idx += (int64_t)gridDim.x * blockDim.x) {
    int i = (int)(idx / d1), j = (int)(idx % d1);
    double v = (i >= j) ? H64[idx] : H64[(int64_t)j * d1 + i];
    if (i == j) v += lam;
    H[idx] = (float)v;
  }
}

hipError_t launch_finalize_H(const double* H64, float* H, int d1, const double* lam_dev, hipStream_t s) {
  int64_t n = (int64_t)d1 * d1;
  int blocks = (int)((n + 1023) / 1024);
  if (blocks > 131072) blocks = 131072;
  hipLaunchKernelGGL(finalize_H_kernel, dim3(blocks), dim3(256), 0, s, H64, H, d1, lam_dev);
  return hipGetLastError();
}

__device__ __forceinline__ double block_sum(double v, double* sh) {
  for (int o = 32; o > 0; o >>= 1) v += __shfl_down(v, o, 64);
  int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  __syncthreads();
  if (lane == 0) sh[w] = v;
  __syncthreads();
  double t = 0;
  if (threadIdx.x == 0)
    for (int i = 0; i < (int)(blockDim.x >> 6); i++) t += sh[i];
  return t;   // valid in thread 0
}

__global__ __launch_bounds__(1024) void trace64_kernel(const double* __restrict__ H64, int d1, double* out) {
  __shared__ double sh[16];
  double v = 0;
  for (int i = threadIdx.x; i < d1; i += blockDim.x) v += H64[(int64_t)i * d1 + i];
  double t = block_sum(v, sh);
  if (threadIdx.x == 0) out[0] = t;
}

hipError_t launch_trace64(const double* H64, int d1, double* out, hipStream_t s) {
  hipLaunchKernelGGL(trace64_kernel, dim3(1), dim3(1024), 0, s, H64, d1, out);
  return hipGetLastError();
}

// norms2[j] = sum of squares of the q rows of group j (one workgroup per group, fixed order)
__global__ __launch_bounds__(256) void group_norms_kernel(const float* __restrict__ Wf, int q, int m,
                                                           double* __restrict__ norms2) {
  __shared__ double sh[4];
  int g = blockIdx.x;
  const float* base = Wf + (int64_t)g * q * m;
  double v = 0;
  for (int64_t i = threadIdx.x; i < (int64_t)q * m; i += 256) { double x = base[i]; v += x * x; }
  double t = block_sum(v, sh);
  if (threadIdx.x == 0) norms2[g] = t;
}

hipError_t launch_group_norms(const float* Wf, int p, int q, int m, double* norms2, hipStream_t s) {
  hipLaunchKernelGGL(group_norms_kernel, dim3(p), dim3(256), 0, s, Wf, q, m, norms2);
  return hipGetLastError();
}

// out = sum a[i]*b[i] in float64, two fixed-order stages (partial must hold 1024 doubles)
__global__ __launch_bounds__(256) void dot64_stage1(const float* __restrict__ a, const float* __restrict__ b, int64_t n,
                                                     double* __restrict__ partial) {
  __shared__ double sh[4];
  double v = 0;
  for (int64_t i = blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256) v += (double)a[i] * (double)b[i];
  double t = block_sum(v, sh);
  if (threadIdx.x == 0) partial[blockIdx.x] = t;
}
__global__ __launch_bounds__(1024) void dot64_stage2(const double* __restrict__ partial, int n, double* out) {
  __shared__ double sh[16];
  double v = (threadIdx.x < (unsigned)n) ? partial[threadIdx.x] : 0.0;
  double t = block_sum(v, sh);
  if (threadIdx.x == 0) out[0] = t;
}

hipError_t launch_dot64(const float* a, const float* b, int64_t n, double* out, double* partial, hipStream_t s) {
  hipLaunchKernelGGL(dot64_stage1, dim3(1024), dim3(256), 0, s, a, b, n, partial);
  hipLaunchKernelGGL(dot64_stage2, dim3(1), dim3(1024), 0, s, partial, 1024, out);
  return hipGetLastError();
}

}  // namespace osscar
