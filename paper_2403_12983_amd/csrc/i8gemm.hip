// C = alpha A B + beta Cin for float32 operands, to the accuracy of float64 accumulation, on the int8 matrix cores.
//
// The large products of the state build (B = P G_K, V = P H_{K,Kc}, S, R of Proposition 4.1's closed forms and the
// residuals that refine them) need sums that are exact to far below float32 rounding; the float64 matrix-core
// instruction delivers that at 78.6 TFLOP/s, the int8 one runs 64 times as many multiply-adds per second.  Each row of A
// and each column of B is scaled by a power of two to (-1, 1) and cut into I8_S digits of 7 bits (signed, round to
// nearest: the first digit has 6 bits), x 2^-e = sum_t d_t 2^-(6 + 7 t), |d_t| <= 64, exactly while t < I8_S.  Products of
// digits are summed exactly in int32 (K 64^2 (t+1) < 2^31 for K < 100000), one accumulator set per digit weight
// g = t + u < I8_S: I8_S (I8_S + 1) / 2 = 15 integer products instead of one float64 product, and
//     C[i][j] = 2^(e_i + f_j) * sum_g acc_g[i][j] * 2^-(12 + 7 g)
// in float64.  What is dropped is below 2^-34 of (row maximum) x (column maximum) per term; on the 14336^3 products of the
// benchmark layer the result differs from the float64-accumulated one by 2e-9 of sum |a b|, the size of the float32
// rounding of the result itself.
// The digits are fixed-point relative to the largest entry of the row (column), so an entry 2^-b of that maximum keeps
// 34 - b bits.  The inverse P of a Gram matrix has a diagonal 10^3 - 10^4 times its off-diagonal entries, which would leave
// those with about 21 bits and, through the cancellation in P H_{K,Kc}, a 5e-5 error in V.  So a square operand can have its
// diagonal taken out (diag_a, diag_b): the diagonal is left out of the scaling and the digits, and its term A_ii B_ij
// (A_ij B_jj) is added in float64 in the epilogue.  Likewise along the contraction: the rows and columns of a Gram matrix
// scale with s_k = sqrt(H_kk), those of its inverse with 1 / s_k, so an outlier channel (s_k 20 times the rest) would cost the
// other entries of every row that crosses it 4 - 9 bits.  With kexp[k] = round(log2 s_k) the product is computed as
// (A 2^(+-kexp)) (2^(-+kexp) B), exact scalings that level both operands along k (ksign = +1: A inverse-like, B Gram-like).
//
// Layout of a packed operand: packet (16 consecutive k of one row, one digit) at
//     ((panel * nstages + stage) * I8_S + t) * 256 + kh * 128 + r,   panel = row / 128, stage = k / 32, kh = (k % 32) / 16, r = row % 128,
// so a (stage, panel) block of I8_S * 4 KB is the A- or B-side input of one v_mfma_i32_32x32x32_i8 step of a 128-row tile.
// The kernel: one workgroup of 8 waves (two per SIMD) per 128 x 128 tile, wave tile 64 x 32 = 2 matrix-core tiles x I8_S
// accumulator sets (160 registers); operand blocks go from global memory straight into LDS (global_load_lds_dwordx4), three
// stage buffers, loads three stages ahead; one barrier per stage that waits for LDS traffic only, placed before the last
// two products of the stage so that the next stage's row-side operands are on their way while those run.  (With 4 waves of
// 64 x 64, one per SIMD, the 14336^3 product took 51 ms instead of 41 ms: nothing to run while a wave waits.)
#include "internal.h"

namespace osscar {
namespace {
typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));
constexpr int S = I8_S;
constexpr int BLK = S * 256;                       // packets of one (stage, panel) block

__device__ __forceinline__ int expo_of(unsigned bits) {      // smallest e with v < 2^e (0 for v = 0)
  const float v = __uint_as_float(bits);
  if (!(v > 0.f)) return 0;
  int e;
  frexpf(v, &e);
  return e;
}

// mx[r] = bit pattern of max |X[r, :]| (non-negative floats order like their bit patterns)
__global__ __launch_bounds__(256) void i8_absmax_rows_kernel(const float* __restrict__ X, int R, int K, int64_t ld, int skip_diag,
                                                              const int* __restrict__ kexp, int ks, unsigned* __restrict__ mx) {
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
  if (row >= R) return;
  float v = 0.f;
  for (int k = lane; k < K; k += 64)
    if (!(skip_diag && k == row)) v = fmaxf(v, fabsf(ldexpf(X[(int64_t)row * ld + k], kexp ? ks * kexp[k] : 0)));
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  if (lane == 0) mx[row] = __float_as_uint(v);
}
// mx[c] = max over the rows [256 y, 256 y + 256) of |X[:, c]|, joined by an atomic maximum (order-independent); mx zeroed before
__global__ __launch_bounds__(256) void i8_absmax_cols_kernel(const float* __restrict__ X, int K, int N, int64_t ld, int skip_diag,
                                                              const int* __restrict__ kexp, int ks, unsigned* __restrict__ mx) {
  const int col = blockIdx.x * 256 + threadIdx.x;
  if (col >= N) return;
  const int k0 = blockIdx.y * 256, k1 = min(K, k0 + 256);
  float v = 0.f;
  for (int k = k0; k < k1; k++)
    if (!(skip_diag && k == col)) v = fmaxf(v, fabsf(ldexpf(X[(int64_t)k * ld + col], kexp ? ks * kexp[k] : 0)));
  atomicMax(&mx[col], __float_as_uint(v));
}
__global__ void i8_zero_kernel(unsigned* p, int n) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i < n) p[i] = 0u;
}

// 16 scaled values -> S packets of 16 digits each (every step is exact in float32)
__device__ __forceinline__ void slice16(const float* v, uint4* out) {
  unsigned w[S][4];
#pragma unroll
  for (int t = 0; t < S; t++) { w[t][0] = w[t][1] = w[t][2] = w[t][3] = 0u; }
#pragma unroll
  for (int j = 0; j < 16; j++) {
    float r = v[j] * 64.f;
#pragma unroll
    for (int t = 0; t < S; t++) {
      const float d = rintf(r);
      w[t][j >> 2] |= ((unsigned)((int)d & 0xff)) << (8 * (j & 3));
      r = (r - d) * 128.f;
    }
  }
#pragma unroll
  for (int t = 0; t < S; t++) out[t] = uint4{w[t][0], w[t][1], w[t][2], w[t][3]};
}

// A-side: X is R x K, the contraction runs along a row.  Thread = (packet of 16 k, row), rows fastest.
__global__ __launch_bounds__(256) void i8_pack_rows_kernel(const float* __restrict__ X, int R, int K, int64_t ld, int vec, int skip_diag,
                                                            const int* __restrict__ kexp, int ks, const unsigned* __restrict__ mx, uint4* __restrict__ out, int npanels,
                                                            int nstages) {
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int rpad = npanels * 128;
  const int kp = (int)(idx / rpad), row = (int)(idx % rpad);
  if (kp >= nstages * 2) return;
  float v[16];
#pragma unroll
  for (int j = 0; j < 16; j++) v[j] = 0.f;
  if (row < R) {
    const float sc = ldexpf(1.f, -expo_of(mx[row]));
    const float* p = X + (int64_t)row * ld + kp * 16;
    if (vec) {            // K % 4 == 0, ld % 4 == 0, X 16-byte aligned: a group of four is inside or outside as a whole
#pragma unroll
      for (int j = 0; j < 4; j++)
        if (kp * 16 + 4 * j < K) {
          const float4 q = reinterpret_cast<const float4*>(p)[j];
          v[4 * j] = q.x * sc; v[4 * j + 1] = q.y * sc; v[4 * j + 2] = q.z * sc; v[4 * j + 3] = q.w * sc;
        }
    } else {
#pragma unroll
      for (int j = 0; j < 16; j++)
        if (kp * 16 + j < K) v[j] = p[j] * sc;
    }
    if (kexp) {
#pragma unroll
      for (int j = 0; j < 16; j++)
        if (kp * 16 + j < K) v[j] = ldexpf(v[j], ks * kexp[kp * 16 + j]);
    }
    if (skip_diag && (row >> 4) == kp) {
#pragma unroll
      for (int j = 0; j < 16; j++)
        if (j == (row & 15)) v[j] = 0.f;
    }
  }
  uint4 pk[S];
  slice16(v, pk);
  const int stage = kp >> 1, kh = kp & 1, panel = row >> 7, r = row & 127;
#pragma unroll
  for (int t = 0; t < S; t++) out[(((int64_t)panel * nstages + stage) * S + t) * 256 + kh * 128 + r] = pk[t];
}
// B-side: X is K x N, the contraction runs down a column.  Thread = (packet of 16 k, column), columns fastest.
__global__ __launch_bounds__(256) void i8_pack_cols_kernel(const float* __restrict__ X, int K, int N, int64_t ld, int skip_diag,
                                                            const int* __restrict__ kexp, int ks, const unsigned* __restrict__ mx, uint4* __restrict__ out, int npanels,
                                                            int nstages) {
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int cpad = npanels * 128;
  const int kp = (int)(idx / cpad), col = (int)(idx % cpad);
  if (kp >= nstages * 2) return;
  float v[16];
#pragma unroll
  for (int j = 0; j < 16; j++) v[j] = 0.f;
  if (col < N) {
    const float sc = ldexpf(1.f, -expo_of(mx[col]));
#pragma unroll
    for (int j = 0; j < 16; j++)
      if (kp * 16 + j < K && !(skip_diag && kp * 16 + j == col))
        v[j] = ldexpf(X[(int64_t)(kp * 16 + j) * ld + col], kexp ? ks * kexp[kp * 16 + j] : 0) * sc;
  }
  uint4 pk[S];
  slice16(v, pk);
  const int stage = kp >> 1, kh = kp & 1, panel = col >> 7, r = col & 127;
#pragma unroll
  for (int t = 0; t < S; t++) out[(((int64_t)panel * nstages + stage) * S + t) * 256 + kh * 128 + r] = pk[t];
}

}  // namespace
// kexp[k] = round(log2 sqrt(D[k][k])) for a positive diagonal, 0 otherwise (clamped to +-60)
__global__ void i8_kexp_kernel(const float* __restrict__ D, int n, int64_t ld, int* __restrict__ kexp) {
  const int k = blockIdx.x * 256 + threadIdx.x;
  if (k >= n) return;
  const float d = D[(int64_t)k * ld + k];
  int e = 0;
  if (d > 0.f && d < 3e38f) e = (int)rintf(0.5f * log2f(d));
  kexp[k] = max(-60, min(60, e));
}
hipError_t launch_i8_kexp(const float* D, int n, int64_t ld, int* kexp, hipStream_t s) {
  if (n <= 0) return hipSuccess;
  hipLaunchKernelGGL(i8_kexp_kernel, dim3((n + 255) / 256), dim3(256), 0, s, D, n, ld, kexp);
  return hipGetLastError();
}
namespace {
struct I8Args {
  const uint4* Ap; const uint4* Bp; int nstages;
  const unsigned* mxa; const unsigned* mxb;
  const float* Cin; int64_t ldcin; float* C; int64_t ldc;
  int M, N, tiles_m, tiles_n, lower_only;
  double alpha, beta, diag_add;
  const float* A; int64_t lda; const float* B; int64_t ldb; int diag_a, diag_b;      // the operands themselves, for the diagonal terms
};

__device__ __forceinline__ void lds_only_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

__global__ __launch_bounds__(512, 1) void i8_gemm_kernel(I8Args g) {
  extern __shared__ uint4 lds[];                 // [3 stage buffers][A block | B block]
  // 8 x 8 super-blocks of tiles, dealt to the XCDs in turn (workgroup index modulo 8): the tiles an XCD works on together
  // share row and column panels in its L2.  lower_only: the super-blocks on or below the diagonal.
  int tm, tn;
  {
    const int b = blockIdx.x, xcd = b & 7, slot = b >> 3;
    const int sbi = (slot / 64) * 8 + xcd, within = slot % 64;
    if (g.lower_only) {
      const int nr = (g.tiles_m + 7) / 8;
      if (sbi >= nr * (nr + 1) / 2) return;
      int r = (int)((sqrtf(8.f * (float)sbi + 1.f) - 1.f) * 0.5f);
      while ((r + 1) * (r + 2) / 2 <= sbi) r++;
      while (r * (r + 1) / 2 > sbi) r--;
      tm = r * 8 + within / 8;
      tn = (sbi - r * (r + 1) / 2) * 8 + within % 8;
      if (tm >= g.tiles_m || tn > tm) return;
    } else {
      const int nsb_c = (g.tiles_n + 7) / 8, nsb = ((g.tiles_m + 7) / 8) * nsb_c;
      if (sbi >= nsb) return;
      tm = (sbi / nsb_c) * 8 + within / 8;
      tn = (sbi % nsb_c) * 8 + within % 8;
      if (tm >= g.tiles_m || tn >= g.tiles_n) return;
    }
  }
  const int nstages = g.nstages;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, wm = wave >> 2, wn = wave & 3;      // wave tile: 64 rows x 32 columns
  v16i acc[S][2];
#pragma unroll
  for (int q = 0; q < S; q++)
#pragma unroll
    for (int a = 0; a < 2; a++)
#pragma unroll
      for (int r = 0; r < 16; r++) acc[q][a][r] = 0;
  const uint4* ga = g.Ap + (int64_t)tm * nstages * BLK;
  const uint4* gb = g.Bp + (int64_t)tn * nstages * BLK;
  // A stage is the A block followed by the B block, 2 BLK = 2560 packets; instruction i of a wave moves packets
  // [512 i + 64 wave, + 64) (the boundary 1280 is a multiple of 64: a wave's 64 lie in one block); lane l's 16 bytes
  // land at the LDS base + 16 l.
  constexpr int NI = (2 * BLK) / 512;
  static_assert((2 * BLK) % 512 == 0 && BLK % 64 == 0, "every wave issues the same number of loads per stage");
#define OSSCAR_I8_ISSUE(st_, buf_)                                                                                               \
  {                                                                                                                              \
    _Pragma("unroll") for (int i = 0; i < NI; i++) {                                                                             \
      const int p0 = i * 512 + wave * 64;                                                                                        \
      const uint4* src = (p0 < BLK) ? ga + (int64_t)(st_) * BLK + p0 + lane : gb + (int64_t)(st_) * BLK + (p0 - BLK) + lane;     \
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)src,                                       \
                                       (__attribute__((address_space(3))) void*)(lds + (buf_) * 2 * BLK + p0), 16, 0, 0);        \
    }                                                                                                                            \
  }
  OSSCAR_I8_ISSUE(0, 0);
  if (nstages > 1) OSSCAR_I8_ISSUE(1, 1);
  if (nstages > 2) OSSCAR_I8_ISSUE(2, 2);
  const int oa = (lane >> 5) * 128 + wm * 64 + (lane & 31), ob = (lane >> 5) * 128 + wn * 32 + (lane & 31);
  // stage 0 has landed (each wave waits for its own loads of that stage, then the barrier)
  if (nstages > 2) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(2 * NI) : "memory");
  else if (nstages == 2) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(NI) : "memory");
  else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  lds_only_barrier();
  v4i fa[2][S];
#pragma unroll
  for (int t = 0; t < S; t++)
#pragma unroll
    for (int a = 0; a < 2; a++) { uint4 q = lds[t * 256 + oa + a * 32]; fa[a][t] = *reinterpret_cast<v4i*>(&q); }
  int buf = 0;
  for (int st = 0; st < nstages; st++) {
    __builtin_amdgcn_iglp_opt(0);
    const uint4* pb = lds + buf * 2 * BLK + BLK;
    // column-side digits 0 .. S-2 against every row-side digit they meet: 28 of the stage's 30 products
#pragma unroll
    for (int u = 0; u < S - 1; u++) {
      v4i fb;
      { uint4 q = pb[u * 256 + ob]; fb = *reinterpret_cast<v4i*>(&q); }
#pragma unroll
      for (int t = 0; t + u < S; t++)
#pragma unroll
        for (int a = 0; a < 2; a++)
          acc[t + u][a] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[a][t], fb, acc[t + u][a], 0, 0, 0);
    }
    // The last column-side digit goes to a register; then every wave has taken all it needs from this stage's buffer,
    // which the barrier establishes, and the buffer is refilled with the stage three ahead.  The next stage's row-side
    // operands are requested before the last two products of this one.
    v4i fl;
    { uint4 q = pb[(S - 1) * 256 + ob]; fl = *reinterpret_cast<v4i*>(&q); }
    v4i a0[2];
    a0[0] = fa[0][0]; a0[1] = fa[1][0];
    if (st + 1 < nstages) {
      if (st + 2 < nstages) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(NI) : "memory");      // stage st + 1 has landed, st + 2 may be in flight
      else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
      lds_only_barrier();
      if (st + 3 < nstages) { const int nb = buf; OSSCAR_I8_ISSUE(st + 3, nb); }
      const uint4* qa = lds + ((buf + 1) % 3) * 2 * BLK;
#pragma unroll
      for (int t = 0; t < S; t++)
#pragma unroll
        for (int a = 0; a < 2; a++) { uint4 q = qa[t * 256 + oa + a * 32]; fa[a][t] = *reinterpret_cast<v4i*>(&q); }
    }
#pragma unroll
    for (int a = 0; a < 2; a++) acc[S - 1][a] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a0[a], fl, acc[S - 1][a], 0, 0, 0);
    buf = (buf + 1) % 3;
  }
#undef OSSCAR_I8_ISSUE
  // C layout of a 32 x 32 tile: register r = rr*4 + r3 holds row rr*8 + (lane/32)*4 + r3, column lane%32
  const int col = tn * 128 + wn * 32 + (lane & 31);
  const int eb = expo_of(g.mxb[col < g.N ? col : 0]);
#pragma unroll
  for (int a = 0; a < 2; a++)
#pragma unroll
    for (int r = 0; r < 16; r++) {
      const int row = tm * 128 + wm * 64 + a * 32 + (r >> 2) * 8 + (lane >> 5) * 4 + (r & 3);
      if (row < g.M && col < g.N) {
        double v = 0.0;
#pragma unroll
        for (int q = S - 1; q >= 0; q--) v = v * (1.0 / 128.0) + (double)acc[q][a][r];
        v = ldexp(v, expo_of(g.mxa[row]) + eb - 12);
        // the diagonal terms that were left out of the digits: k = row of A (A square), k = col of B (B square)
        if (g.diag_a) v += (double)g.A[(int64_t)row * g.lda + row] * (double)g.B[(int64_t)row * g.ldb + col];
        if (g.diag_b && !(g.diag_a && row == col)) v += (double)g.A[(int64_t)row * g.lda + col] * (double)g.B[(int64_t)col * g.ldb + col];
        v *= g.alpha;
        if (g.beta != 0.0) v += g.beta * (double)g.Cin[(int64_t)row * g.ldcin + col];
        if (row == col) v += g.diag_add;
        g.C[(int64_t)row * g.ldc + col] = (float)v;
      }
    }
}
}  // namespace

size_t i8_pack_bytes(int64_t rows, int64_t K) {
  return (size_t)S * 16 * (size_t)((rows + 127) / 128 * 128) * (size_t)((K + 31) / 32 * 2);
}

bool i8_gemm_fits(const GemmArgs& g) {
  // int32 sums: K * 64^2 * S must stay below 2^31; float32 in and out, plain A B
  return g.M > 0 && g.N > 0 && g.K > 0 && g.K <= 100000 && !g.c_is_f64 && !g.trans_b && !g.acc_f32 && (g.beta == 0.0 || g.Cin != nullptr);
}

hipError_t launch_i8_gemm(const GemmArgs& g, void* packA, size_t capA, void* packB, size_t capB, unsigned* mx, size_t mx_entries,
                          hipStream_t s) {
  if (!i8_gemm_fits(g) || (g.lower_only && g.M != g.N)) return hipErrorInvalidValue;
  if ((g.i8_diag_a && g.M != g.K) || (g.i8_diag_b && g.N != g.K)) return hipErrorInvalidValue;
  if (g.i8_kexp && g.i8_ksign != 1 && g.i8_ksign != -1) return hipErrorInvalidValue;
  if (i8_pack_bytes(g.M, g.K) > capA || i8_pack_bytes(g.N, g.K) > capB || (size_t)g.M + (size_t)g.N > mx_entries) return hipErrorInvalidValue;
  if ((reinterpret_cast<uintptr_t>(packA) & 15) || (reinterpret_cast<uintptr_t>(packB) & 15)) return hipErrorInvalidValue;
  const int npa = (g.M + 127) / 128, npb = (g.N + 127) / 128, nst = (g.K + 31) / 32;
  unsigned* mxa = mx; unsigned* mxb = mx + g.M;
  int log_slot = -1;
  gemm_log_open(g.M, g.N, g.K, 16 | (g.lower_only ? 4 : 0), s, &log_slot);
  hipLaunchKernelGGL(i8_zero_kernel, dim3((g.N + 255) / 256), dim3(256), 0, s, mxb, g.N);
  hipLaunchKernelGGL(i8_absmax_rows_kernel, dim3((g.M + 3) / 4), dim3(256), 0, s, g.A, g.M, g.K, g.lda, g.i8_diag_a, g.i8_kexp, g.i8_ksign, mxa);
  hipLaunchKernelGGL(i8_absmax_cols_kernel, dim3((g.N + 255) / 256, (g.K + 255) / 256), dim3(256), 0, s, g.B, g.K, g.N, g.ldb, g.i8_diag_b, g.i8_kexp, -g.i8_ksign, mxb);
  const int vec = (g.K % 4 == 0) && (g.lda % 4 == 0) && ((reinterpret_cast<uintptr_t>(g.A) & 15) == 0);
  hipLaunchKernelGGL(i8_pack_rows_kernel, dim3((unsigned)(((int64_t)nst * 2 * npa * 128 + 255) / 256)), dim3(256), 0, s, g.A, g.M, g.K, g.lda, vec,
                     g.i8_diag_a, g.i8_kexp, g.i8_ksign, mxa, reinterpret_cast<uint4*>(packA), npa, nst);
  hipLaunchKernelGGL(i8_pack_cols_kernel, dim3((unsigned)(((int64_t)nst * 2 * npb * 128 + 255) / 256)), dim3(256), 0, s, g.B, g.K, g.N, g.ldb,
                     g.i8_diag_b, g.i8_kexp, -g.i8_ksign, mxb, reinterpret_cast<uint4*>(packB), npb, nst);
  I8Args a{};
  a.Ap = reinterpret_cast<const uint4*>(packA); a.Bp = reinterpret_cast<const uint4*>(packB); a.nstages = nst;
  a.mxa = mxa; a.mxb = mxb; a.Cin = g.Cin; a.ldcin = g.ldcin; a.C = reinterpret_cast<float*>(g.C); a.ldc = g.ldc;
  a.M = g.M; a.N = g.N; a.tiles_m = npa; a.tiles_n = npb; a.lower_only = g.lower_only;
  a.alpha = g.alpha; a.beta = g.beta; a.diag_add = g.diag_add;
  a.A = g.A; a.lda = g.lda; a.B = g.B; a.ldb = g.ldb; a.diag_a = g.i8_diag_a; a.diag_b = g.i8_diag_b;
  int nsb;
  if (g.lower_only) { const int nr = (npa + 7) / 8; nsb = nr * (nr + 1) / 2; }
  else nsb = ((npa + 7) / 8) * ((npb + 7) / 8);
  const size_t shmem = (size_t)3 * 2 * BLK * 16;
  {   // 120 KB of dynamic shared memory needs the opt-in (per device; the call is host-side only)
    const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(i8_gemm_kernel), hipFuncAttributeMaxDynamicSharedMemorySize, (int)shmem);
    if (e != hipSuccess) return e;
  }
  hipLaunchKernelGGL(i8_gemm_kernel, dim3((unsigned)((nsb + 7) / 8 * 8 * 64)), dim3(512), shmem, s, a);
  gemm_log_close(log_slot, s);
  return hipGetLastError();
}

}  // namespace osscar
