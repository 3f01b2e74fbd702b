// Delayed-update form of the local search for groups of one row (q = 1).
//
// The eager search applies every swap as a rank-2 pass over the whole tableau (N, Z): O(d1 (d1 + m)) bytes
// per swap.  Here the tableau in HBM is left at a BASE state (N0, Z0) and the swaps since then are kept as
// the set T of indices swept so far.  By the block form of the sweep operator, with C0 = N0[:, T],
// M = N0[T, T] and J = diag(-1 on the pivots that LEFT the kept set, +1 elsewhere),
//     N_cur[i, l] = N0[i, l] - C0[i, :] M^-1 C0[l, :]^T                (i, l outside T)
//     N_cur[T, l] = J M^-1 C0[l, :]^T,    N_cur[T, T] = -J M^-1 J
//     Z_cur[i, :] = Z0[i, :] - C0[i, :] ZT,   Z_cur[T, :] = J ZT,       ZT = M^-1 Z0[T, :]
// so one iteration needs only two columns of N_cur and two rows of Z_cur (O(tau (d1 + m))), the diagonal
// and the squared row norms of Z_cur for the scores of eq. (impact) -- both updated incrementally, the
// norms through one read-only pass over Z0 (w = Z0 [y1 y2]) -- and a bordering update of M^-1.  Every
// FLUSH iterations the pending rank-tau correction is applied to N0 and Z0 as two matrix products on the
// matrix cores.  The sequence of swaps is exactly that of the eager search (Proposition 4.1, Cases 1-3).
#include "internal.h"

namespace osscar {

__device__ __forceinline__ float nsym1(const float* __restrict__ N, int64_t ld, int i, int t) {
  return (i >= t) ? N[(int64_t)i * ld + t] : N[(int64_t)t * ld + i];
}
__device__ __forceinline__ double wsum(double v) {
  for (int o = 32; o > 0; o >>= 1) v += __shfl_down(v, o, 64);
  return v;
}
__device__ __forceinline__ bool idle(const SearchCtrl* c) { return c->done || c->pause; }

// x_g = M^-1 N0[T, g], x_j = M^-1 N0[T, j]; pauses the search if g or j is already in T.
__global__ __launch_bounds__(256) void lazy_prep_kernel(LazyPtrs L, const float* __restrict__ N0, int d1, SearchCtrl* ctrl) {
  __shared__ double bg[LAZY_TM], bj[LAZY_TM];
  if (idle(ctrl)) return;
  const int g = ctrl->g_out, j = ctrl->g_in, tau = ctrl->tau, tid = threadIdx.x;
  if (L.pos[g] >= 0 || L.pos[j] >= 0 || tau + 2 > LAZY_TM) {
    if (tid == 0) ctrl->pause = 1;
    return;
  }
  for (int s = tid; s < tau; s += 256) {
    int t = L.Tidx[s];
    bg[s] = (double)nsym1(N0, d1, t, g);
    bj[s] = (double)nsym1(N0, d1, t, j);
  }
  __syncthreads();
  for (int r = tid; r < tau; r += 256) {
    double a = 0, b = 0;
    for (int s = 0; s < tau; s++) { double mv = L.Minv[r * LAZY_TM + s]; a += mv * bg[s]; b += mv * bj[s]; }
    L.xg[r] = a; L.xj[r] = b;
  }
}

// current columns g and j of N
__global__ __launch_bounds__(256) void lazy_columns_kernel(LazyPtrs L, const float* __restrict__ N0, int d1,
                                                            const SearchCtrl* __restrict__ ctrl) {
  if (idle(ctrl)) return;
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i >= d1) return;
  const int g = ctrl->g_out, j = ctrl->g_in, tau = ctrl->tau;
  const int ps = L.pos[i];
  if (ps >= 0) {
    double sg = (double)L.Jsg[ps];
    L.cg[i] = sg * L.xg[ps];
    L.cj[i] = sg * L.xj[ps];
    return;
  }
  double a = 0, b = 0;
  for (int s = 0; s < tau; s++) {
    double c = (double)L.C0T[(int64_t)s * d1 + i];
    a += c * L.xg[s]; b += c * L.xj[s];
  }
  L.cg[i] = (double)nsym1(N0, d1, i, g) - a;
  L.cj[i] = (double)nsym1(N0, d1, i, j) - b;
}

// current rows g and j of Z, the scaled rows y1 = Dg z_g, y2 = Dj' (z_j - n_jg y1), and partial sums
__global__ __launch_bounds__(256) void lazy_zrows_kernel(LazyPtrs L, const float* __restrict__ Z0, int d1, int m,
                                                          SearchCtrl* ctrl) {
  __shared__ double red[5][4];
  if (idle(ctrl)) return;
  const int g = ctrl->g_out, j = ctrl->g_in, tau = ctrl->tau;
  const double ngg = L.cg[g], njg = L.cg[j];
  const bool bad1 = !(ngg < 0.0);
  const double Dg = 1.0 / (bad1 ? -1.0 : ngg);
  const double M1 = Dg * njg;
  const double njjp = L.cj[j] - njg * M1;
  const bool bad2 = !(njjp > 0.0);
  const double Dj = 1.0 / (bad2 ? 1.0 : njjp);
  const int col = blockIdx.x * 256 + threadIdx.x;
  double v[5] = {0, 0, 0, 0, 0};
  if (col < m) {
    double zg = (double)Z0[(int64_t)g * m + col], zj = (double)Z0[(int64_t)j * m + col];
    for (int s = 0; s < tau; s++) {
      double zt = L.ZT[(int64_t)s * m + col];
      zg -= (double)L.C0T[(int64_t)s * d1 + g] * zt;
      zj -= (double)L.C0T[(int64_t)s * d1 + j] * zt;
    }
    double y1 = Dg * zg, zjp = zj - njg * y1, y2 = Dj * zjp;
    L.y1[col] = y1; L.y2[col] = y2; L.y1f[col] = (float)y1; L.y2f[col] = (float)y2;
    v[0] = zg * y1; v[1] = zjp * y2; v[2] = y1 * y1; v[3] = y2 * y2; v[4] = y1 * y2;
  }
#pragma unroll
  for (int k = 0; k < 5; k++) {
    double t = wsum(v[k]);
    if ((threadIdx.x & 63) == 0) red[k][threadIdx.x >> 6] = t;
  }
  __syncthreads();
  if (threadIdx.x < 5) L.part[blockIdx.x * 5 + threadIdx.x] = red[threadIdx.x][0] + red[threadIdx.x][1] + red[threadIdx.x][2] + red[threadIdx.x][3];
  if (blockIdx.x == 0 && threadIdx.x == 0) {
    L.ls[0] = Dg; L.ls[1] = njg; L.ls[2] = M1; L.ls[3] = Dj;
    if (bad1 || bad2) ctrl->notpd = 1;
  }
}

// exact change of the objective for the pair (Case 3), acceptance, trace
__global__ __launch_bounds__(64) void lazy_accept_kernel(LazyPtrs L, int nblocks, SearchCtrl* ctrl, int always_accept,
                                                          int32_t* trace_out, int32_t* trace_in, float* trace_gap,
                                                          double* trace_obj) {
  if (idle(ctrl)) return;
  if (threadIdx.x != 0) return;
  double s[5] = {0, 0, 0, 0, 0};
  for (int b = 0; b < nblocks; b++)
    for (int k = 0; k < 5; k++) s[k] += L.part[b * 5 + k];
  L.ls[4] = s[2]; L.ls[5] = s[3]; L.ls[6] = s[4];
  const double delta = -s[0] - s[1];
  ctrl->delta = delta;
  const int it = ctrl->iters;
  const bool ok = !ctrl->notpd && (always_accept || delta < -ctrl->rel_tol * ctrl->obj);
  ctrl->iters = it + 1;
  if (ok) { ctrl->obj += delta; ctrl->accepted += 1; } else { ctrl->done = 1; }
  if (trace_out) {
    trace_out[it] = ctrl->g_out; trace_in[it] = ctrl->g_in;
    trace_gap[2 * it] = (float)ctrl->gap_rem; trace_gap[2 * it + 1] = (float)ctrl->gap_add;
    trace_obj[it] = ctrl->obj;
  }
}

// w1 = Z0 y1, w2 = Z0 y2 (read-only pass over Z0), and u1 = ZT y1, u2 = ZT y2 in the trailing workgroups.
// Each wave owns 8 rows; y1, y2 are staged through LDS in chunks of LAZY_CH columns.
constexpr int LAZY_CH = 4096;
constexpr int GEMV_ROWS = 32;

__global__ __launch_bounds__(256) void lazy_gemv_kernel(LazyPtrs L, const float* __restrict__ Z0, int d1, int m,
                                                         const SearchCtrl* __restrict__ ctrl) {
  __shared__ float sy1[LAZY_CH], sy2[LAZY_CH];
  if (idle(ctrl)) return;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  constexpr int ZTB = LAZY_TM / 4;                    // leading workgroups: one pending row of ZT per wave
  if ((int)blockIdx.x < ZTB) {
    const int row = blockIdx.x * 4 + wave;
    if (row >= ctrl->tau) return;
    const double* zt = L.ZT + (int64_t)row * m;
    double a = 0, b = 0;
#pragma unroll 4
    for (int c = lane; c < m; c += 64) { const double z = zt[c]; a += z * L.y1[c]; b += z * L.y2[c]; }
    a = wsum(a); b = wsum(b);
    if (lane == 0) { L.u1[row] = a; L.u2[row] = b; }
    return;
  }
  const int row0 = ((int)blockIdx.x - ZTB) * GEMV_ROWS + wave * 8;
  double a1[8], a2[8];
#pragma unroll
  for (int r = 0; r < 8; r++) { a1[r] = 0; a2[r] = 0; }
  const bool vec = (m % 4 == 0);
  for (int c0 = 0; c0 < m; c0 += LAZY_CH) {
    const int cw = (m - c0 < LAZY_CH) ? m - c0 : LAZY_CH;
    __syncthreads();
    for (int c = tid; c < cw; c += 256) { sy1[c] = L.y1f[c0 + c]; sy2[c] = L.y2f[c0 + c]; }
    __syncthreads();
    if (vec) {
      // rows beyond the end are clamped (their sums are discarded) so that the 8 loads of a step are issued together
      for (int c = lane * 4; c < cw; c += 256) {
        float4 z[8];
#pragma unroll
        for (int r = 0; r < 8; r++) {
          int row = row0 + r;
          if (row > d1 - 1) row = d1 - 1;
          z[r] = *reinterpret_cast<const float4*>(Z0 + (int64_t)row * m + c0 + c);
        }
        const float4 p1 = *reinterpret_cast<const float4*>(&sy1[c]);
        const float4 p2 = *reinterpret_cast<const float4*>(&sy2[c]);
#pragma unroll
        for (int r = 0; r < 8; r++) {
          a1[r] += (double)z[r].x * p1.x + (double)z[r].y * p1.y + (double)z[r].z * p1.z + (double)z[r].w * p1.w;
          a2[r] += (double)z[r].x * p2.x + (double)z[r].y * p2.y + (double)z[r].z * p2.z + (double)z[r].w * p2.w;
        }
      }
    } else {
      for (int c = lane; c < cw; c += 64) {
        const double p1 = sy1[c], p2 = sy2[c];
#pragma unroll
        for (int r = 0; r < 8; r++) {
          int row = row0 + r;
          if (row > d1 - 1) row = d1 - 1;
          const double z = (double)Z0[(int64_t)row * m + c0 + c];
          a1[r] += z * p1; a2[r] += z * p2;
        }
      }
    }
  }
#pragma unroll
  for (int r = 0; r < 8; r++) {
    double t1 = wsum(a1[r]), t2 = wsum(a2[r]);
    const int row = row0 + r;
    if (lane == 0 && row < d1) { L.w1[row] = t1; L.w2[row] = t2; }
  }
}

// squared row norms, diagonal and scores after the swap; new base columns appended to C0
__global__ __launch_bounds__(256) void lazy_update_kernel(LazyPtrs L, const float* __restrict__ N0, int d1,
                                                           const SearchCtrl* __restrict__ ctrl, int32_t* __restrict__ kept,
                                                           double* __restrict__ rho, double* __restrict__ diag,
                                                           double* __restrict__ score) {
  if (idle(ctrl)) return;
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i >= d1) return;
  const int g = ctrl->g_out, j = ctrl->g_in, tau = ctrl->tau;
  const double Dg = L.ls[0], M1 = L.ls[2], Dj = L.ls[3], y11 = L.ls[4], y22 = L.ls[5], y12 = L.ls[6];
  // append the base columns of g and j (rows tau, tau + 1 of C0T)
  L.C0T[(int64_t)tau * d1 + i] = nsym1(N0, d1, i, g);
  L.C0T[(int64_t)(tau + 1) * d1 + i] = nsym1(N0, d1, i, j);
  if (i == g) {
    rho[i] = y11 - 2.0 * M1 * y12 + M1 * M1 * y22;      // || -y1 + M1 y2 ||^2
    diag[i] = -Dg - M1 * M1 * Dj;
    kept[i] = 0;
    L.pos[i] = tau; L.Tidx[tau] = i; L.Jsg[tau] = -1.f;
    score[i] = rho[i] / fabs(diag[i]);
    return;
  }
  if (i == j) {
    rho[i] = y22;
    diag[i] = -Dj;
    kept[i] = 1;
    L.pos[i] = tau + 1; L.Tidx[tau + 1] = i; L.Jsg[tau + 1] = 1.f;
    score[i] = rho[i] / fabs(diag[i]);
    return;
  }
  double zy1, zy2;
  const int ps = L.pos[i];
  if (ps >= 0) {
    const double sg = (double)L.Jsg[ps];
    zy1 = sg * L.u1[ps]; zy2 = sg * L.u2[ps];
  } else {
    double a = 0, b = 0;
    for (int s = 0; s < tau; s++) {
      const double c = (double)L.C0T[(int64_t)s * d1 + i];
      a += c * L.u1[s]; b += c * L.u2[s];
    }
    zy1 = L.w1[i] - a; zy2 = L.w2[i] - b;
  }
  const double c1 = L.cg[i];
  const double c2 = L.cj[i] - c1 * M1;
  double r = rho[i];
  r += -2.0 * c1 * zy1 + c1 * c1 * y11;                   // after the reverse sweep on g
  const double zy2p = zy2 - c1 * y12;                     // (Z_i - c1 y1) . y2
  r += -2.0 * c2 * zy2p + c2 * c2 * y22;                  // after the forward sweep on j
  if (r < 0.0) r = 0.0;
  const double dnew = diag[i] - c1 * c1 * Dg - c2 * c2 * Dj;
  rho[i] = r; diag[i] = dnew;
  score[i] = r / fabs(dnew);
}

// ZT <- M'^-1 Z0[T', :] for T' = T + {g, j}
__global__ __launch_bounds__(256) void lazy_zt_kernel(LazyPtrs L, int m, const SearchCtrl* __restrict__ ctrl) {
  if (idle(ctrl)) return;
  const int col = blockIdx.x * 256 + threadIdx.x;
  if (col >= m) return;
  const int tau = ctrl->tau;
  const double M1 = L.ls[2];
  const double y1 = L.y1[col], y2 = L.y2[col];
  for (int s = 0; s < tau; s++) {
    const double xg = L.xg[s], xjp = L.xj[s] - xg * M1;
    L.ZT[(int64_t)s * m + col] -= xg * y1 + xjp * y2;
  }
  L.ZT[(int64_t)tau * m + col] = y1 - M1 * y2;
  L.ZT[(int64_t)(tau + 1) * m + col] = y2;
}

// bordering of M^-1 by g then j; tau += 2
__global__ __launch_bounds__(256) void lazy_minv_kernel(LazyPtrs L, SearchCtrl* ctrl) {
  if (idle(ctrl)) return;
  const int tau = ctrl->tau, tid = threadIdx.x;
  const double Dg = L.ls[0], M1 = L.ls[2], Dj = L.ls[3];
  double* Mi = L.Minv;
  // x'_s = x_j[s] - x_g[s] M1 (s < tau), x'_tau = M1
  for (int idx = tid; idx < tau * tau; idx += 256) {
    int r = idx / tau, s = idx % tau;
    double xr = L.xg[r], xs = L.xg[s];
    double pr = L.xj[r] - xr * M1, ps = L.xj[s] - xs * M1;
    Mi[r * LAZY_TM + s] += xr * xs * Dg + pr * ps * Dj;
  }
  for (int r = tid; r < tau; r += 256) {
    double xr = L.xg[r], pr = L.xj[r] - xr * M1;
    double v = -xr * Dg + pr * M1 * Dj;              // bordered by g, then corrected by the sweep on j
    Mi[r * LAZY_TM + tau] = v; Mi[tau * LAZY_TM + r] = v;
    double w = -pr * Dj;
    Mi[r * LAZY_TM + tau + 1] = w; Mi[(tau + 1) * LAZY_TM + r] = w;
  }
  if (tid == 0) {
    Mi[tau * LAZY_TM + tau] = Dg + M1 * M1 * Dj;
    Mi[tau * LAZY_TM + tau + 1] = -M1 * Dj; Mi[(tau + 1) * LAZY_TM + tau] = -M1 * Dj;
    Mi[(tau + 1) * LAZY_TM + tau + 1] = Dj;
  }
  __syncthreads();
  if (tid == 0) ctrl->tau = tau + 2;
}

hipError_t launch_lazy_iteration(const TabDims& d, const TabPtrs& t, const LazyPtrs& L, int always_accept, hipStream_t s,
                                 hipEvent_t* ev) {
  const int rb = (d.d1 + 255) / 256, mb = (d.m + 255) / 256;
  launch_select(d, t, -1, -1, s);
  hipLaunchKernelGGL(lazy_prep_kernel, dim3(1), dim3(256), 0, s, L, t.N, d.d1, t.ctrl);
  hipLaunchKernelGGL(lazy_columns_kernel, dim3(rb), dim3(256), 0, s, L, t.N, d.d1, t.ctrl);
  hipLaunchKernelGGL(lazy_zrows_kernel, dim3(mb), dim3(256), 0, s, L, t.Z, d.d1, d.m, t.ctrl);
  hipLaunchKernelGGL(lazy_accept_kernel, dim3(1), dim3(64), 0, s, L, mb, t.ctrl, always_accept, t.trace_out, t.trace_in,
                     t.trace_gap, t.trace_obj);
  const int gb = (d.d1 + GEMV_ROWS - 1) / GEMV_ROWS + LAZY_TM / 4;
  if (ev) hipEventRecord(ev[0], s);
  hipLaunchKernelGGL(lazy_gemv_kernel, dim3(gb), dim3(256), 0, s, L, t.Z, d.d1, d.m, t.ctrl);
  if (ev) hipEventRecord(ev[1], s);
  hipLaunchKernelGGL(lazy_update_kernel, dim3(rb), dim3(256), 0, s, L, t.N, d.d1, t.ctrl, t.kept, t.gram, t.dblk, t.score);
  hipLaunchKernelGGL(lazy_zt_kernel, dim3(mb), dim3(256), 0, s, L, d.m, t.ctrl);
  hipLaunchKernelGGL(lazy_minv_kernel, dim3(1), dim3(256), 0, s, L, t.ctrl);
  if (ev) hipEventRecord(ev[2], s);
  return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// flush: apply the pending correction to N0, Z0 and empty T
// ------------------------------------------------------------------------------------------------
// E = C0 M^-1 and Cb = C0 as d1 x LAZY_TM row-major panels (rows in T and columns >= tau are zero); Et keeps the
// unzeroed E rows (they are the same rows: rows in T are never needed from E).
__global__ __launch_bounds__(256) void lazy_panels_kernel(LazyPtrs L, int d1, const SearchCtrl* __restrict__ ctrl) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i >= d1) return;
  const int tau = ctrl->tau;
  float* Ei = L.E + (int64_t)i * LAZY_TM;
  float* Ci = L.Cb + (int64_t)i * LAZY_TM;
  if (L.pos[i] >= 0) {
    for (int s = 0; s < LAZY_TM; s++) { Ei[s] = 0.f; Ci[s] = 0.f; }
    return;
  }
  for (int s0 = 0; s0 < LAZY_TM; s0 += 16) {
    double acc[16];
#pragma unroll
    for (int u = 0; u < 16; u++) acc[u] = 0;
    if (s0 < tau) {
      for (int r = 0; r < tau; r++) {
        const double c = (double)L.C0T[(int64_t)r * d1 + i];
        const double* mr = L.Minv + r * LAZY_TM + s0;
#pragma unroll
        for (int u = 0; u < 16; u++) acc[u] += c * mr[u];
      }
    }
#pragma unroll
    for (int u = 0; u < 16; u++) {
      const int s = s0 + u;
      Ei[s] = (s < tau) ? (float)acc[u] : 0.f;
      Ci[s] = (s < tau) ? L.C0T[(int64_t)s * d1 + i] : 0.f;
    }
  }
}

__global__ __launch_bounds__(256) void lazy_zt32_kernel(LazyPtrs L, int m, const SearchCtrl* __restrict__ ctrl) {
  const int col = blockIdx.x * 256 + threadIdx.x;
  if (col >= m) return;
  const int tau = ctrl->tau;
  for (int s = 0; s < LAZY_TM; s++) L.ZT32[(int64_t)s * m + col] = (s < tau) ? (float)L.ZT[(int64_t)s * m + col] : 0.f;
}

// pivot rows / columns of N0 and pivot rows of Z0
__global__ __launch_bounds__(256) void lazy_fix_kernel(LazyPtrs L, float* __restrict__ N0, int d1,
                                                        const SearchCtrl* __restrict__ ctrl) {
  const int l = blockIdx.x * 256 + threadIdx.x;
  if (l >= d1) return;
  const int tau = ctrl->tau;
  const int pr = L.pos[l];
  if (pr < 0) {
    const float* El = L.E + (int64_t)l * LAZY_TM;
    for (int s = 0; s < tau; s++) {
      const int t = L.Tidx[s];
      const float v = L.Jsg[s] * El[s];
      if (l < t) N0[(int64_t)t * d1 + l] = v; else N0[(int64_t)l * d1 + t] = v;
    }
  } else {
    for (int s = 0; s < tau; s++) {
      const int t = L.Tidx[s];
      if (l >= t) N0[(int64_t)l * d1 + t] = (float)(-(double)L.Jsg[pr] * (double)L.Jsg[s] * L.Minv[pr * LAZY_TM + s]);
    }
  }
}
__global__ __launch_bounds__(256) void lazy_fix_z_kernel(LazyPtrs L, float* __restrict__ Z0, int m,
                                                          const SearchCtrl* __restrict__ ctrl) {
  const int col = blockIdx.x * 256 + threadIdx.x;
  if (col >= m) return;
  const int tau = ctrl->tau;
  for (int s = 0; s < tau; s++) Z0[(int64_t)L.Tidx[s] * m + col] = (float)((double)L.Jsg[s] * L.ZT[(int64_t)s * m + col]);
}
__global__ __launch_bounds__(256) void lazy_reset_kernel(LazyPtrs L, SearchCtrl* ctrl) {
  const int tau = ctrl->tau;
  for (int s = threadIdx.x; s < tau; s += 256) L.pos[L.Tidx[s]] = -1;
  __syncthreads();
  if (threadIdx.x == 0) { ctrl->tau = 0; ctrl->pause = 0; }
}

hipError_t launch_lazy_flush(const TabDims& d, const TabPtrs& t, const LazyPtrs& L, hipStream_t s) {
  const int rb = (d.d1 + 255) / 256, mb = (d.m + 255) / 256;
  hipLaunchKernelGGL(lazy_panels_kernel, dim3(rb), dim3(256), 0, s, L, d.d1, t.ctrl);
  hipLaunchKernelGGL(lazy_zt32_kernel, dim3(mb), dim3(256), 0, s, L, d.m, t.ctrl);
  GemmArgs g{};
  g.M = d.d1; g.N = d.d1; g.K = LAZY_TM; g.A = L.E; g.lda = LAZY_TM; g.B = L.Cb; g.ldb = LAZY_TM; g.trans_b = 1;
  g.Cin = t.N; g.ldcin = d.d1; g.C = t.N; g.ldc = d.d1; g.alpha = -1.0; g.beta = 1.0; g.lower_only = 1;
  hipError_t e = launch_gemm_f64acc(g, s);
  if (e != hipSuccess) return e;
  GemmArgs z{};
  z.M = d.d1; z.N = d.m; z.K = LAZY_TM; z.A = L.Cb; z.lda = LAZY_TM; z.B = L.ZT32; z.ldb = d.m;
  z.Cin = t.Z; z.ldcin = d.m; z.C = t.Z; z.ldc = d.m; z.alpha = -1.0; z.beta = 1.0;
  e = launch_gemm_f64acc(z, s);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(lazy_fix_kernel, dim3(rb), dim3(256), 0, s, L, t.N, d.d1, t.ctrl);
  hipLaunchKernelGGL(lazy_fix_z_kernel, dim3(mb), dim3(256), 0, s, L, t.Z, d.m, t.ctrl);
  hipLaunchKernelGGL(lazy_reset_kernel, dim3(1), dim3(256), 0, s, L, t.ctrl);
  return launch_refresh_scores(d, t, s);
}

hipError_t launch_lazy_init(const TabDims& d, const LazyPtrs& L, SearchCtrl* ctrl, hipStream_t s) {
  hipError_t e = hipMemsetAsync(L.pos, 0xFF, (size_t)d.d1 * 4, s);
  if (e != hipSuccess) return e;
  return hipMemsetAsync(L.Minv, 0, (size_t)LAZY_TM * LAZY_TM * 8, s);
}

}  // namespace osscar
