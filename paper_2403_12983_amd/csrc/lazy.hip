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
// norms through w = Z0 [y1 y2] -- and a bordering update of M^-1.
// w without a pass over Z0: y1, y2 are combinations of the current rows g, j of Z, and these of base rows:
//     Z0 z_g^T = Z0 Z0[g, :]^T - sum_r x_g[r] Z0 Z0[T_r, :]^T,     x_g = M^-1 C0[g, :]^T,
// so it is enough to know the products of Z0 with the base rows of g, j and of the pending pivots.  Which rows
// will be pivots before the next flush is predictable (the LAZY_NPICK_OUT cheapest removals and LAZY_NPICK_IN largest
// gains at flush time cover all but a few per thousand of them), so right after each flush one matrix product Zc Z0^T
// computes those products for these candidate rows (GbT); a pivot outside the candidates costs one read-only pass over
// Z0 for its column (kept in one of LAZY_NS spare slots).  Every
// LAZY_TM/2 iterations the pending rank-tau correction is applied to N0 and Z0 by matrix products on the
// matrix cores.  The sequence of swaps is exactly that of the eager search (Proposition 4.1, Cases 1-3).
//
// Four launches per iteration:
//   prep    (1 workgroup)  : argmin / argmax from per-block partial records; x = M^-1 N0[T, {g, j}]; pivots
//   vectors (rows | cols | rows) : current columns g, j of N; current rows g, j of Z scaled to y1, y2; partial sums;
//                            and, independent of these, w = Z0 [y1 y2] from the cached products
//   gemv    (rows)         : exact change of the objective and the acceptance test; u = ZT [y1 y2]; for a pivot that is
//                            not among the candidates, its column Z0 Z0[g, :]^T by a pass over Z0
//   update  (rows|cols|M)  : norms, diagonal, scores and their partial records; C0 append; ZT and M^-1 update
//                            (after a miss also w, whose missing column exists only since gemv)
#include "internal.h"
#include <algorithm>

namespace osscar {

__device__ __forceinline__ float nsym1(const float* __restrict__ N, int64_t ld, int i, int t) {
  return (i >= t) ? N[(int64_t)i * ld + t] : N[(int64_t)t * ld + i];
}
// Sum over the 64 lanes of a wave by data-parallel-primitive moves (no trip through the LDS crossbar, which costs a
// shuffle about 40 ns here and made the reductions the longest part of the small kernels): pairs and quads by quad
// permutations, the four quads of a row of 16 by row rotations, then row 0 -> 1 and 2 -> 3 (row_bcast:15) and
// rows 0-1 -> 3 (row_bcast:31); lane 63 holds the total, which every lane receives.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ double dpp_get(double v) {
  int lo = __double2loint(v), hi = __double2hiint(v);
  lo = __builtin_amdgcn_update_dpp(0, lo, CTRL, ROW_MASK, 0xf, false);
  hi = __builtin_amdgcn_update_dpp(0, hi, CTRL, ROW_MASK, 0xf, false);
  return __hiloint2double(hi, lo);
}
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ double dpp_get_or(double v, double dflt) {
  int lo = __double2loint(v), hi = __double2hiint(v);
  lo = __builtin_amdgcn_update_dpp(__double2loint(dflt), lo, CTRL, ROW_MASK, 0xf, false);
  hi = __builtin_amdgcn_update_dpp(__double2hiint(dflt), hi, CTRL, ROW_MASK, 0xf, false);
  return __hiloint2double(hi, lo);
}
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ int dpp_get_or(int v, int dflt) { return __builtin_amdgcn_update_dpp(dflt, v, CTRL, ROW_MASK, 0xf, false); }
__device__ __forceinline__ double wsum(double v) {
  v += dpp_get<0xb1, 0xf>(v);        // quad_perm [1, 0, 3, 2]
  v += dpp_get<0x4e, 0xf>(v);        // quad_perm [2, 3, 0, 1]
  v += dpp_get<0x124, 0xf>(v);       // row_ror:4
  v += dpp_get<0x128, 0xf>(v);       // row_ror:8
  v += dpp_get<0x142, 0xa>(v);       // row_bcast:15 into rows 1 and 3 (other rows add zero)
  v += dpp_get<0x143, 0xc>(v);       // row_bcast:31 into rows 2 and 3
  const int lo = __builtin_amdgcn_readlane(__double2loint(v), 63), hi = __builtin_amdgcn_readlane(__double2hiint(v), 63);
  return __hiloint2double(hi, lo);
}
__device__ __forceinline__ bool idle(const SearchCtrl* c) { return c->done || c->pause; }
// pending pivots including those of the iteration that ran last (for kernels outside an iteration)
__device__ __forceinline__ int tau_all(const SearchCtrl* c) { return c->tau + c->tau_inc; }

constexpr int ROWS_PER_BLOCK = 32;   // row kernels: 8 lanes per row, 256 threads
constexpr int COLS_PER_BLOCK = 64;   // column kernels: 64 columns x 4 slices of the pending set

// ls[] slots
enum { LS_DG = 0, LS_NJG = 1, LS_M1 = 2, LS_DJ = 3, LS_Y11 = 4, LS_Y22 = 5, LS_Y12 = 6, LS_OBJ = 8 };
// misc[] slots
enum { MI_SPARE = 0, MI_MISS = 1, MI_SG = 2, MI_SJ = 3 };

// merge of two (best, second, index) records; lowest index wins ties
__device__ __forceinline__ void merge_min(double& a1, double& a2, int& ia, double b1, double b2, int ib) {
  const bool takeb = (ib >= 0) && (ia < 0 || b1 < a1 || (b1 == a1 && ib < ia));
  const double n1 = takeb ? b1 : a1, other = takeb ? a1 : b1;
  a2 = fmin(fmin(a2, b2), other); a1 = n1; ia = takeb ? ib : ia;
}
__device__ __forceinline__ void merge_max(double& a1, double& a2, int& ia, double b1, double b2, int ib) {
  const bool takeb = (ib >= 0) && (ia < 0 || b1 > a1 || (b1 == a1 && ib < ia));
  const double n1 = takeb ? b1 : a1, other = takeb ? a1 : b1;
  a2 = fmax(fmax(a2, b2), other); a1 = n1; ia = takeb ? ib : ia;
}

// Sum over each group of eight consecutive lanes (every lane of the group receives it): pairs and quads by quad
// permutations, the two quads of a half row by row_half_mirror (lane i of the half row reads lane 7 - i, which by then
// holds the other quad's sum).
__device__ __forceinline__ double sum8(double v) {
  v += dpp_get<0xb1, 0xf>(v);
  v += dpp_get<0x4e, 0xf>(v);
  v += dpp_get<0x141, 0xf>(v);
  return v;
}

// The (best, second, index) records of the 64 lanes of a wave merged into lane 63, by the same data-parallel moves as
// wsum (each step joins disjoint sets of lanes, so no record meets itself; lanes that a row mask leaves out see the
// neutral record).  Lanes without a candidate hold the neutral record (+-inf, index -1).
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ void dpp_merge_step(double& mn1, double& mn2, int& imn, double& mx1, double& mx2, int& imx) {
  const double b1 = dpp_get_or<CTRL, ROW_MASK>(mn1, INFINITY), b2 = dpp_get_or<CTRL, ROW_MASK>(mn2, INFINITY);
  const int ib = dpp_get_or<CTRL, ROW_MASK>(imn, -1);
  const double c1 = dpp_get_or<CTRL, ROW_MASK>(mx1, -INFINITY), c2 = dpp_get_or<CTRL, ROW_MASK>(mx2, -INFINITY);
  const int ic = dpp_get_or<CTRL, ROW_MASK>(imx, -1);
  merge_min(mn1, mn2, imn, b1, b2, ib);
  merge_max(mx1, mx2, imx, c1, c2, ic);
}
__device__ __forceinline__ void wave_merge(double& mn1, double& mn2, int& imn, double& mx1, double& mx2, int& imx) {
  dpp_merge_step<0xb1, 0xf>(mn1, mn2, imn, mx1, mx2, imx);
  dpp_merge_step<0x4e, 0xf>(mn1, mn2, imn, mx1, mx2, imx);
  dpp_merge_step<0x124, 0xf>(mn1, mn2, imn, mx1, mx2, imx);
  dpp_merge_step<0x128, 0xf>(mn1, mn2, imn, mx1, mx2, imx);
  dpp_merge_step<0x142, 0xa>(mn1, mn2, imn, mx1, mx2, imx);
  dpp_merge_step<0x143, 0xc>(mn1, mn2, imn, mx1, mx2, imx);
}

// The same moves on (value, index) alone: lane 63 ends with the smallest value (lowest index on ties) and the largest.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ void dpp_best_step(double& mn, int& imn, double& mx, int& imx) {
  const double b = dpp_get_or<CTRL, ROW_MASK>(mn, INFINITY), c = dpp_get_or<CTRL, ROW_MASK>(mx, -INFINITY);
  const int ib = dpp_get_or<CTRL, ROW_MASK>(imn, -1), ic = dpp_get_or<CTRL, ROW_MASK>(imx, -1);
  const bool tb = (ib >= 0) && (imn < 0 || b < mn || (b == mn && ib < imn));
  const bool tc = (ic >= 0) && (imx < 0 || c > mx || (c == mx && ic < imx));
  mn = tb ? b : mn; imn = tb ? ib : imn; mx = tc ? c : mx; imx = tc ? ic : imx;
}
// ... and on plain values: lane 63 ends with the minimum of lo and the maximum of hi over the wave
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ void dpp_minmax_step(double& lo, double& hi) {
  lo = fmin(lo, dpp_get_or<CTRL, ROW_MASK>(lo, INFINITY)); hi = fmax(hi, dpp_get_or<CTRL, ROW_MASK>(hi, -INFINITY));
}

// per-block record of the scores of rows [32 b, 32 b + 32): used after a flush; the update kernel writes the same records
__global__ __launch_bounds__(64) void lazy_partials_kernel(LazyPtrs L, int p, const int32_t* __restrict__ kept,
                                                            const double* __restrict__ score) {
  const int h = blockIdx.x * ROWS_PER_BLOCK + threadIdx.x;
  double mn1 = INFINITY, mn2 = INFINITY, mx1 = -INFINITY, mx2 = -INFINITY;
  int imn = -1, imx = -1;
  if (threadIdx.x < ROWS_PER_BLOCK && h < p) {
    if (kept[h]) { mn1 = score[h]; imn = h; } else { mx1 = score[h]; imx = h; }
  }
  for (int o = 16; o > 0; o >>= 1) {
    double b1 = __shfl_down(mn1, o, 64), b2 = __shfl_down(mn2, o, 64); int ib = __shfl_down(imn, o, 64);
    merge_min(mn1, mn2, imn, b1, b2, ib);
    b1 = __shfl_down(mx1, o, 64); b2 = __shfl_down(mx2, o, 64); ib = __shfl_down(imx, o, 64);
    merge_max(mx1, mx2, imx, b1, b2, ib);
  }
  if (threadIdx.x == 0) {
    SelRec r; r.mn1 = mn1; r.mn2 = mn2; r.mx1 = mx1; r.mx2 = mx2; r.imn = imn; r.imx = imx;
    L.sel[blockIdx.x] = r;
  }
}

// ---------------------------------------------------------------------------------------------- prep
// single != nullptr: removal of the one row *single (Case 1 alone, nothing enters): the second pivot's quantities are zero.
__global__ __launch_bounds__(256) void lazy_prep_kernel(LazyPtrs L, const float* __restrict__ N0, int d1, int nrec,
                                                         const int32_t* __restrict__ kept, SearchCtrl* ctrl, const int32_t* __restrict__ single, int forced_g,
                                                         int forced_j) {
  __shared__ double s_mn1[4], s_mn2[4], s_mx1[4], s_mx2[4];
  __shared__ int s_imn[4], s_imx[4];
  __shared__ double bg[LAZY_TM], bj[LAZY_TM], red[3][4], s_n0[3];
  if (idle(ctrl)) return;
  const int tid = threadIdx.x;
  const int tau = tau_all(ctrl);           // every thread reads before thread 0 folds the increment in (after the barrier)
  // argmin of the removal costs / argmax of the addition gains from the per-block records: each thread merges its
  // records, the waves reduce by data-parallel moves, every thread merges the four wave results (lowest index wins
  // ties, so the result does not depend on the order)
  double mn1 = INFINITY, mn2 = INFINITY, mx1 = -INFINITY, mx2 = -INFINITY;
  int imn = -1, imx = -1;
  for (int r0 = tid; r0 < nrec; r0 += 1024) {          // four records in flight per thread
    SelRec c[4];
#pragma unroll
    for (int k = 0; k < 4; k++) { const int r = r0 + 256 * k; c[k] = L.sel[r < nrec ? r : r0]; }
#pragma unroll
    for (int k = 0; k < 4; k++)
      if (r0 + 256 * k < nrec) {
        merge_min(mn1, mn2, imn, c[k].mn1, c[k].mn2, c[k].imn);
        merge_max(mx1, mx2, imx, c[k].mx1, c[k].mx2, c[k].imx);
      }
  }
  wave_merge(mn1, mn2, imn, mx1, mx2, imx);
  if ((tid & 63) == 63) { const int w = tid >> 6; s_mn1[w] = mn1; s_mn2[w] = mn2; s_imn[w] = imn; s_mx1[w] = mx1; s_mx2[w] = mx2; s_imx[w] = imx; }
  __syncthreads();
  if (tid == 0) { ctrl->tau = tau; ctrl->tau_inc = 0; }
  mn1 = s_mn1[0]; mn2 = s_mn2[0]; imn = s_imn[0]; mx1 = s_mx1[0]; mx2 = s_mx2[0]; imx = s_imx[0];
  for (int w = 1; w < 4; w++) { merge_min(mn1, mn2, imn, s_mn1[w], s_mn2[w], s_imn[w]); merge_max(mx1, mx2, imx, s_mx1[w], s_mx2[w], s_imx[w]); }
  const int g = single ? *single : (forced_g >= 0 ? forced_g : imn);
  const int j = single ? g : (forced_g >= 0 ? forced_j : imx);
  if (g < 0 || j < 0 || (forced_g >= 0 && (!kept[g] || kept[j]))) {
    if (tid == 0) { ctrl->done = 1; ctrl->g_out = -1; ctrl->g_in = -1; }
    return;
  }
  // the three base entries of the pivot block: requested now by otherwise idle threads, used by thread 0 at the end
  if (tid == 192) s_n0[0] = (double)nsym1(N0, d1, g, g);
  if (tid == 193) s_n0[1] = (double)nsym1(N0, d1, j, g);
  if (tid == 194) s_n0[2] = (double)nsym1(N0, d1, j, j);
  const int sg0 = L.cslot[g], sj0 = L.cslot[j];
  const int need = (sg0 < 0 ? 1 : 0) + ((!single && sj0 < 0) ? 1 : 0);
  if (L.pos[g] >= 0 || L.pos[j] >= 0 || tau + (single ? 1 : 2) > LAZY_TM || L.misc[MI_SPARE] + need > LAZY_NS) {
    if (tid == 0) ctrl->pause = 1;
    return;
  }
  // b = N0[T, {g, j}] (these are rows g, j of C0), x = M^-1 b, zero beyond tau
  for (int s = tid; s < LAZY_TM; s += 256) {
    bg[s] = (s < tau) ? (double)L.C0R[(int64_t)g * LAZY_TM + s] : 0.0;
    bj[s] = (s < tau && !single) ? (double)L.C0R[(int64_t)j * LAZY_TM + s] : 0.0;
  }
  __syncthreads();
  // two threads per row of M^-1, one half of the columns each
  double pgg = 0, pjg = 0, pjj = 0;
  {
    const int r = tid >> 1, half = tid & 1;
    double a = 0, b = 0;
    if (r < tau) {
      // the whole half row is requested at once (bg, bj are zero beyond tau, M^-1 is finite there)
      const double* mrow = L.Minv + r * LAZY_TM + half * (LAZY_TM / 2);
      const double* pg = bg + half * (LAZY_TM / 2);
      const double* pj = bj + half * (LAZY_TM / 2);
      const int cnt = min(tau - half * (LAZY_TM / 2), LAZY_TM / 2);      // columns of this half below tau (may be <= 0)
      for (int s0 = 0; s0 < cnt; s0 += 32) {
        double mv[32];
#pragma unroll
        for (int u = 0; u < 32; u++) mv[u] = mrow[s0 + u];
#pragma unroll
        for (int u = 0; u < 32; u++) { a += mv[u] * pg[s0 + u]; b += mv[u] * pj[s0 + u]; }
      }
    }
    a += __shfl_xor(a, 1, 64); b += __shfl_xor(b, 1, 64);
    if (half == 0) {
      L.xg[r] = a; L.xj[r] = b;
      pgg = bg[r] * a; pjg = bj[r] * a; pjj = bj[r] * b;
    }
  }
  pgg = wsum(pgg); pjg = wsum(pjg); pjj = wsum(pjj);
  if ((tid & 63) == 0) { red[0][tid >> 6] = pgg; red[1][tid >> 6] = pjg; red[2][tid >> 6] = pjj; }
  __syncthreads();
  if (tid == 0) {
    const double ngg = s_n0[0] - (red[0][0] + red[0][1] + red[0][2] + red[0][3]);
    const double njg = s_n0[1] - (red[1][0] + red[1][1] + red[1][2] + red[1][3]);
    const double njj = s_n0[2] - (red[2][0] + red[2][1] + red[2][2] + red[2][3]);
    const bool bad1 = !(ngg < 0.0);                         // kept pivot: N_gg = -P_gg
    const double Dg = 1.0 / (bad1 ? -1.0 : ngg);
    double M1 = Dg * njg;
    const double njjp = njj - njg * M1;                     // entering pivot after the first sweep: a Schur complement
    bool bad2 = !(njjp > 0.0);
    double Dj = 1.0 / (bad2 ? 1.0 : njjp);
    if (single) { M1 = 0.0; Dj = 0.0; bad2 = false; }
    L.ls[LS_DG] = Dg; L.ls[LS_NJG] = single ? 0.0 : njg; L.ls[LS_M1] = M1; L.ls[LS_DJ] = Dj; L.ls[LS_OBJ] = ctrl->obj;
    if (bad1 || bad2) ctrl->notpd = 1;
    ctrl->g_out = g; ctrl->g_in = j;
    // slots of the two base columns; a pivot that is not among the candidates takes a spare slot, filled by the next kernel
    int ns = L.misc[MI_SPARE], miss = 0, sg = sg0, sj = sj0;
    if (sg < 0) { sg = LAZY_NC + ns++; L.cslot[g] = sg; L.cand[sg] = g; miss |= 1; }
    if (single) sj = sg;
    else if (sj < 0) { sj = LAZY_NC + ns++; L.cslot[j] = sj; L.cand[sj] = j; miss |= 2; }
    L.misc[MI_SPARE] = ns; L.misc[MI_MISS] = miss; L.misc[MI_SG] = sg; L.misc[MI_SJ] = sj;
    ctrl->misses += (miss & 1) + (miss >> 1);
    const double m1 = mn1, m2 = mn2, x1 = mx1, x2 = mx2;
    ctrl->gap_rem = isfinite(m2) ? fabs(m2 - m1) / fmax(fabs(m1), 1e-300) : INFINITY;
    ctrl->gap_add = isfinite(x2) ? fabs(x1 - x2) / fmax(fabs(x1), 1e-300) : INFINITY;
  }
}

// ---------------------------------------------------------------------------------------------- vectors
__device__ __forceinline__ void wcache_block(const LazyPtrs& L, int d1, const SearchCtrl* __restrict__ ctrl, int block);
// 8 lanes of a row: sum_s C0R[row][s] * (xa[s], xb[s]) over the LAZY_TM columns (x is zero beyond tau)
__device__ __forceinline__ void row_dots(const float* __restrict__ crow, const double* __restrict__ xa,
                                         const double* __restrict__ xb, int l8, double& a, double& b) {
  a = 0; b = 0;
#pragma unroll
  for (int t = 0; t < LAZY_TM / 32; t++) {
    const int s = (l8 + 8 * t) * 4;
    const float4 c = *reinterpret_cast<const float4*>(crow + s);
    a += (double)c.x * xa[s] + (double)c.y * xa[s + 1] + (double)c.z * xa[s + 2] + (double)c.w * xa[s + 3];
    b += (double)c.x * xb[s] + (double)c.y * xb[s + 1] + (double)c.z * xb[s + 2] + (double)c.w * xb[s + 3];
  }
  a = sum8(a); b = sum8(b);
}

__global__ __launch_bounds__(256) void lazy_vectors_kernel(LazyPtrs L, const float* __restrict__ N0, const float* __restrict__ Z0,
                                                            int d1, int m, int row_blocks, int col_blocks,
                                                            const SearchCtrl* __restrict__ ctrl) {
  __shared__ double sa[LAZY_TM], sb[LAZY_TM];
  __shared__ double zred[2][4][COLS_PER_BLOCK];
  if (idle(ctrl)) return;
  if ((int)blockIdx.x >= row_blocks + col_blocks) {   // w from the cached products (see wcache_block)
    if (L.misc[MI_MISS] == 0) wcache_block(L, d1, ctrl, blockIdx.x - row_blocks - col_blocks);
    return;
  }
  const int tid = threadIdx.x, g = ctrl->g_out, j = ctrl->g_in, tau = ctrl->tau;
  if ((int)blockIdx.x < row_blocks) {
    // current columns g and j of N
    for (int s = tid; s < LAZY_TM; s += 256) { sa[s] = L.xg[s]; sb[s] = L.xj[s]; }
    __syncthreads();
    const int row = blockIdx.x * ROWS_PER_BLOCK + (tid >> 3), l8 = tid & 7;
    if (row >= d1) return;
    const int ps = L.pos[row];
    double a, b;
    row_dots(L.C0R + (int64_t)row * LAZY_TM, sa, sb, l8, a, b);
    if (l8 == 0) {
      if (ps >= 0) {
        const double sg = (double)L.Jsg[ps];
        L.cg[row] = sg * sa[ps]; L.cj[row] = sg * sb[ps];
      } else {
        L.cg[row] = (double)nsym1(N0, d1, row, g) - a;
        L.cj[row] = (double)nsym1(N0, d1, row, j) - b;
      }
    }
    return;
  }
  // current rows g and j of Z, scaled: y1 = Dg z_g, y2 = Dj (z_j - n_jg y1)
  const int cb = blockIdx.x - row_blocks;
  const int slice = tid >> 6, lc = tid & 63, col = cb * COLS_PER_BLOCK + lc;
  // the base rows g, j of Z are requested first: their latency passes while ZT is read
  float z0g = 0.f, z0j = 0.f;
  if (slice == 0 && col < m) { z0g = Z0[(int64_t)g * m + col]; z0j = Z0[(int64_t)j * m + col]; }
  for (int s = tid; s < LAZY_TM; s += 256) {
    sa[s] = (s < tau) ? (double)L.C0R[(int64_t)g * LAZY_TM + s] : 0.0;
    sb[s] = (s < tau) ? (double)L.C0R[(int64_t)j * LAZY_TM + s] : 0.0;
  }
  __syncthreads();
  double pg = 0, pj = 0;
  if (col < m)
    for (int s = slice; s < tau; s += 64) {               // sixteen loads in flight
      double zt[16];
#pragma unroll
      for (int u = 0; u < 16; u++) { const int ss = s + 4 * u; zt[u] = L.ZT[(int64_t)(ss < tau ? ss : s) * m + col]; }
#pragma unroll
      for (int u = 0; u < 16; u++) { const int ss = s + 4 * u; if (ss < tau) { pg += sa[ss] * zt[u]; pj += sb[ss] * zt[u]; } }
    }
  zred[0][slice][lc] = pg; zred[1][slice][lc] = pj;
  __syncthreads();
  if (slice != 0) return;
  double v[5] = {0, 0, 0, 0, 0};
  if (col < m) {
    const double Dg = L.ls[LS_DG], njg = L.ls[LS_NJG], Dj = L.ls[LS_DJ];
    const double zg = (double)z0g - (zred[0][0][lc] + zred[0][1][lc] + zred[0][2][lc] + zred[0][3][lc]);
    const double zj = (double)z0j - (zred[1][0][lc] + zred[1][1][lc] + zred[1][2][lc] + zred[1][3][lc]);
    const double y1 = Dg * zg, zjp = zj - njg * y1, y2 = Dj * zjp;
    L.y1[col] = y1; L.y2[col] = y2; L.y1f[col] = (float)y1; L.y2f[col] = (float)y2;
    v[0] = zg * y1; v[1] = zjp * y2; v[2] = y1 * y1; v[3] = y2 * y2; v[4] = y1 * y2;
  }
#pragma unroll
  for (int k = 0; k < 5; k++) { const double t = wsum(v[k]); if (lc == 0) L.part[cb * 5 + k] = t; }
}

// ---------------------------------------------------------------------------------------------- gemv + accept
// Every workgroup sums the partial records to the exact change of the objective (Case 3) and takes the same
// accept / reject decision; workgroup 0 records it.  Then w1 = Z0 y1, w2 = Z0 y2 (read-only pass over Z0) and
// u = ZT [y1 y2] in the leading workgroups.  Each wave owns 8 rows; y1, y2 are staged through LDS.
constexpr int LAZY_CH = 4096;
constexpr int GEMV_RPW = 4;        // rows per wave
constexpr int GEMV_UNR = 4;        // float4 loads in flight per row and lane
constexpr int GEMV_ROWS = 4 * GEMV_RPW;
constexpr int GEMV_SPLIT = 4;      // leading workgroups per pending row of ZT (u1, u2 hold one partial sum per workgroup)

__global__ __launch_bounds__(256) void lazy_gemv_kernel(LazyPtrs L, const float* __restrict__ Z0, int d1, int m, int col_blocks,
                                                         SearchCtrl* ctrl, int always_accept, int32_t* trace_out,
                                                         int32_t* trace_in, float* trace_gap, double* trace_obj, int npiv) {
  __shared__ float sy1[LAZY_CH], sy2[LAZY_CH];
  __shared__ int s_ok;
  if (idle(ctrl)) return;
  constexpr int ZTB = LAZY_TM * GEMV_SPLIT;           // leading workgroups: a GEMV_SPLIT-th of one pending row of ZT each
  // the row workgroups have work only when a pivot's products were not computed ahead (workgroup 0 records the decision)
  if ((int)blockIdx.x >= ZTB && L.misc[MI_MISS] == 0) return;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  // The partial records of the acceptance sums are requested first (wave 0; lane l takes the records l, l + 64, ...), then
  // the workgroup's part of u: both are in flight together and neither waits for the other's round trip.
  double pr[2][5];
#pragma unroll
  for (int h = 0; h < 2; h++)
#pragma unroll
    for (int k = 0; k < 5; k++) { const int b = lane + 64 * h; pr[h][k] = (wave == 0 && b < col_blocks) ? L.part[b * 5 + k] : 0.0; }
  // u = ZT [y1 y2]: started before the acceptance sums (it does not depend on them; a rejected swap, which ends the search,
  // just discards it).  Each leading workgroup takes one stretch of columns of one pending row, so that a thread has all its
  // loads in flight at once; the stretches' sums are added in a fixed order by the kernel that uses u.
  double ua = 0, ub = 0;
  const int urow = (int)blockIdx.x / GEMV_SPLIT, upart = (int)blockIdx.x % GEMV_SPLIT;
  if ((int)blockIdx.x < ZTB && urow < ctrl->tau) {
    const double* zt = L.ZT + (int64_t)urow * m;
    const int chunk = (m + GEMV_SPLIT * 256 - 1) / (GEMV_SPLIT * 256) * 256;
    const int c_begin = upart * chunk, c_end = min(m, c_begin + chunk);
    for (int c0 = c_begin + tid; c0 < c_end; c0 += 2048) {             // eight columns in flight per thread
      double z[8], p1[8], p2[8];
#pragma unroll
      for (int u = 0; u < 8; u++) { const int c = c0 + 256 * u, cc = c < c_end ? c : c0; z[u] = zt[cc]; p1[u] = L.y1[cc]; p2[u] = L.y2[cc]; }
#pragma unroll
      for (int u = 0; u < 8; u++) if (c0 + 256 * u < c_end) { ua += z[u] * p1[u]; ub += z[u] * p2[u]; }
    }
  }
  if (wave == 0) {
    // partial sums in a fixed order: lane l adds the records l, l + 64, ...; then a wave reduction
    double sk[5];
#pragma unroll
    for (int k = 0; k < 5; k++) sk[k] = pr[0][k] + pr[1][k];
    for (int b = lane + 128; b < col_blocks; b += 64)
#pragma unroll
      for (int k = 0; k < 5; k++) sk[k] += L.part[b * 5 + k];
#pragma unroll
    for (int k = 0; k < 5; k++) { sk[k] = wsum(sk[k]); }
    if (lane == 0) {
      const double delta = -sk[0] - sk[1];
      const double obj = L.ls[LS_OBJ];
      const bool ok = !ctrl->notpd && (always_accept || delta < -ctrl->rel_tol * obj);
      s_ok = ok ? 1 : 0;
      if (blockIdx.x == 0) {
        L.ls[LS_Y11] = sk[2]; L.ls[LS_Y22] = sk[3]; L.ls[LS_Y12] = sk[4];
        ctrl->delta = delta;
        const int it = ctrl->iters;
        ctrl->iters = it + 1;
        if (ok) { ctrl->obj = obj + delta; ctrl->accepted += 1; ctrl->tau_inc = npiv; } else { ctrl->done = 1; }
        if (trace_out) trace_out[it] = ctrl->g_out;
        if (trace_in) trace_in[it] = ctrl->g_in;
        if (trace_gap) { trace_gap[2 * it] = (float)ctrl->gap_rem; trace_gap[2 * it + 1] = (float)ctrl->gap_add; }
        if (trace_obj) trace_obj[it] = ok ? obj + delta : obj;
      }
    }
  }
  __syncthreads();
  if (!s_ok) return;
  if ((int)blockIdx.x < ZTB) {
    __shared__ double ured[2][4];
    const double a = wsum(ua), b = wsum(ub);
    if (lane == 0) { ured[0][wave] = a; ured[1][wave] = b; }
    __syncthreads();
    if (tid == 0) {                                      // zero beyond tau
      L.u1[upart * LAZY_TM + urow] = ured[0][0] + ured[0][1] + ured[0][2] + ured[0][3];
      L.u2[upart * LAZY_TM + urow] = ured[1][0] + ured[1][1] + ured[1][2] + ured[1][3];
    }
    return;
  }
  // Pivots outside the candidate set: their columns Z0 Z0[g, :]^T, Z0 Z0[j, :]^T by one pass over Z0.  Each wave owns
  // GEMV_RPW rows.  Products are summed four at a time in float32 (one float4 of Z0 against one of the pivot row) and the
  // partial sums are accumulated in float64: the rounding this adds is below that of Z0's own float32 storage.
  const int miss = L.misc[MI_MISS];
  if (miss == 0) return;
  const float* yg = Z0 + (int64_t)ctrl->g_out * m;
  const float* yj = Z0 + (int64_t)ctrl->g_in * m;
  const int row0 = ((int)blockIdx.x - ZTB) * GEMV_ROWS + wave * GEMV_RPW;
  double a1[GEMV_RPW], a2[GEMV_RPW];
  const float* rp[GEMV_RPW];
#pragma unroll
  for (int r = 0; r < GEMV_RPW; r++) {
    a1[r] = 0; a2[r] = 0;
    int row = row0 + r;
    if (row > d1 - 1) row = d1 - 1;                 // clamped rows: their sums are discarded
    rp[r] = Z0 + (int64_t)row * m;
  }
  const bool vec = (m % 4 == 0);
  for (int c0 = 0; c0 < m; c0 += LAZY_CH) {
    const int cw = (m - c0 < LAZY_CH) ? m - c0 : LAZY_CH;
    __syncthreads();
    for (int c = tid; c < cw; c += 256) { sy1[c] = yg[c0 + c]; sy2[c] = yj[c0 + c]; }
    __syncthreads();
    if (vec) {
      for (int c = lane * 4; c < cw; c += 256 * GEMV_UNR) {
        float4 z[GEMV_UNR][GEMV_RPW];
#pragma unroll
        for (int u = 0; u < GEMV_UNR; u++)
#pragma unroll
          for (int r = 0; r < GEMV_RPW; r++) {
            const int cc = c + u * 256;
            z[u][r] = (cc < cw) ? *reinterpret_cast<const float4*>(rp[r] + c0 + cc) : float4{0.f, 0.f, 0.f, 0.f};
          }
#pragma unroll
        for (int u = 0; u < GEMV_UNR; u++) {
          int cc = c + u * 256;
          if (cc >= cw) cc = 0;
          const float4 p1 = *reinterpret_cast<const float4*>(&sy1[cc]);
          const float4 p2 = *reinterpret_cast<const float4*>(&sy2[cc]);
#pragma unroll
          for (int r = 0; r < GEMV_RPW; r++) {
            const float4 v = z[u][r];
            const float s1 = v.x * p1.x + v.y * p1.y + v.z * p1.z + v.w * p1.w;
            const float s2 = v.x * p2.x + v.y * p2.y + v.z * p2.z + v.w * p2.w;
            a1[r] += (double)s1; a2[r] += (double)s2;
          }
        }
      }
    } else {
      for (int c = lane; c < cw; c += 64) {
        const double p1 = sy1[c], p2 = sy2[c];
#pragma unroll
        for (int r = 0; r < GEMV_RPW; r++) {
          const double z = (double)rp[r][c0 + c];
          a1[r] += z * p1; a2[r] += z * p2;
        }
      }
    }
  }
  double* colg = L.GbT + (int64_t)L.misc[MI_SG] * d1;
  double* colj = L.GbT + (int64_t)L.misc[MI_SJ] * d1;
#pragma unroll
  for (int r = 0; r < GEMV_RPW; r++) {
    double t1 = wsum(a1[r]), t2 = wsum(a2[r]);
    const int row = row0 + r;
    if (lane == 0 && row < d1) {
      if (miss & 1) colg[row] = t1;
      if (miss & 2) colj[row] = t2;
    }
  }
}

// ---------------------------------------------------------------------------------------------- wcache
// w1 = Z0 y1, w2 = Z0 y2 from the cached base products: with a_g = col(g) - sum_r x_g[r] col(T_r) (= Z0 z_g^T) and a_j
// likewise, w1 = Dg a_g and w2 = Dj (a_j - n_jg w1).  64 rows x 4 slices of the pending set per workgroup.
__device__ __forceinline__ void wcache_block(const LazyPtrs& L, int d1, const SearchCtrl* __restrict__ ctrl, int block) {
  __shared__ double sxg[LAZY_TM], sxj[LAZY_TM];
  __shared__ int sts[LAZY_TM];
  __shared__ double red[2][4][64];
  const int tid = threadIdx.x, tau = ctrl->tau;
  const int slice = tid >> 6, lr = tid & 63, row = block * 64 + lr;
  const int rc = row < d1 ? row : d1 - 1;
  // the pivots' own products are requested first: their latency passes while the pending pivots' are summed
  double bgv = 0, bjv = 0;
  if (slice == 0) { bgv = L.GbT[(int64_t)L.misc[MI_SG] * d1 + rc]; bjv = L.GbT[(int64_t)L.misc[MI_SJ] * d1 + rc]; }
  for (int s = tid; s < LAZY_TM; s += 256) { sxg[s] = L.xg[s]; sxj[s] = L.xj[s]; sts[s] = (s < tau) ? L.tslot[s] : 0; }
  __syncthreads();
  double ag = 0, aj = 0;
  for (int r = slice; r < tau; r += 64) {                 // sixteen loads in flight
    double bv[16];
#pragma unroll
    for (int u = 0; u < 16; u++) { const int rr = r + 4 * u; bv[u] = L.GbT[(int64_t)sts[rr < tau ? rr : r] * d1 + rc]; }
#pragma unroll
    for (int u = 0; u < 16; u++) { const int rr = r + 4 * u; if (rr < tau) { ag += sxg[rr] * bv[u]; aj += sxj[rr] * bv[u]; } }
  }
  red[0][slice][lr] = ag; red[1][slice][lr] = aj;
  __syncthreads();
  if (slice != 0 || row >= d1) return;
  const double Dg = L.ls[LS_DG], njg = L.ls[LS_NJG], Dj = L.ls[LS_DJ];
  const double tg = bgv - (red[0][0][lr] + red[0][1][lr] + red[0][2][lr] + red[0][3][lr]);
  const double tj = bjv - (red[1][0][lr] + red[1][1][lr] + red[1][2][lr] + red[1][3][lr]);
  const double w1 = Dg * tg;
  L.w1[row] = w1;
  L.w2[row] = Dj * (tj - njg * w1);
}
// w = Z0 [y1 y2] from the cached products runs inside lazy_vectors_kernel's launch, beside the work it does not depend on, when
// both pivots' products were computed ahead (the usual case); after a miss the update kernel forms the sums itself.

// ---------------------------------------------------------------------------------------------- update
// rows    : squared row norms, diagonal, scores (and their per-block records), the two new columns of C0
// columns : ZT <- M'^-1 Z0[T', :] for T' = T + {g, j}
// M       : bordering of M^-1 by g then j
// tau itself is not touched here: the acceptance step has recorded the increment and the next iteration's prep folds it in.
__global__ __launch_bounds__(256) void lazy_update_kernel(LazyPtrs L, const float* __restrict__ N0, int d1, int m, int row_blocks,
                                                           int col_blocks, SearchCtrl* ctrl, int32_t* __restrict__ kept,
                                                           double* __restrict__ rho, double* __restrict__ diag,
                                                           double* __restrict__ score, int single) {
  __shared__ double sa[LAZY_TM], sb[LAZY_TM];
  __shared__ double s_mn[ROWS_PER_BLOCK], s_mx[ROWS_PER_BLOCK];
  __shared__ int s_imn[ROWS_PER_BLOCK], s_imx[ROWS_PER_BLOCK];
  if (idle(ctrl)) return;
  const int tid = threadIdx.x, g = ctrl->g_out, j = ctrl->g_in, tau = ctrl->tau;
  const double Dg = L.ls[LS_DG], M1 = L.ls[LS_M1], Dj = L.ls[LS_DJ];
  const int b = blockIdx.x;
  if (b < row_blocks) {
    for (int s = tid; s < LAZY_TM; s += 256) {            // u = the partial sums of the acceptance kernel's workgroups, in order
      double a = 0, c = 0;
#pragma unroll
      for (int h = 0; h < GEMV_SPLIT; h++) { a += L.u1[h * LAZY_TM + s]; c += L.u2[h * LAZY_TM + s]; }
      sa[s] = a; sb[s] = c;
    }
    __syncthreads();
    const double y11 = L.ls[LS_Y11], y22 = L.ls[LS_Y22], y12 = L.ls[LS_Y12];
    const bool miss = L.misc[MI_MISS] != 0;
    const int row = b * ROWS_PER_BLOCK + (tid >> 3), l8 = tid & 7;
    double mn1 = INFINITY, mx1 = -INFINITY;
    int imn = -1, imx = -1;
    if (row < d1) {
      // what the row's leader needs from memory is requested before the dot products, not after them
      float n0g = 0.f, n0j = 0.f;
      double c1 = 0, cjv = 0, rho0 = 0, diag0 = 0, w1c = 0, w2c = 0;
      int ps = -1, kp0 = 0;
      if (l8 == 0) {
        n0g = nsym1(N0, d1, row, g);
        if (!single) n0j = nsym1(N0, d1, row, j);
        ps = L.pos[row]; c1 = L.cg[row]; cjv = L.cj[row]; rho0 = rho[row]; diag0 = diag[row]; kp0 = kept[row];
        if (!miss) { w1c = L.w1[row]; w2c = L.w2[row]; }
      }
      double da, db;
      row_dots(L.C0R + (int64_t)row * LAZY_TM, sa, sb, l8, da, db);
      // w = Z0 [y1 y2] of this row: computed ahead in lazy_vectors_kernel's launch, unless a pivot's products with Z0 were
      // not among the candidates; its column has existed only since lazy_gemv_kernel's pass, so the sum is formed here
      double w1r, w2r;
      if (miss) {
        double ag = 0, aj = 0;
        for (int r = l8; r < tau; r += 8) {
          const double b = L.GbT[(int64_t)L.tslot[r] * d1 + row];
          ag += L.xg[r] * b; aj += L.xj[r] * b;
        }
        ag = sum8(ag); aj = sum8(aj);
        const double tg = L.GbT[(int64_t)L.misc[MI_SG] * d1 + row] - ag;
        const double tj = L.GbT[(int64_t)L.misc[MI_SJ] * d1 + row] - aj;
        w1r = Dg * tg;
        w2r = Dj * (tj - L.ls[LS_NJG] * w1r);
      } else { w1r = w1c; w2r = w2c; }
      if (l8 == 0) {
        // the base columns of g and j become columns tau, tau + 1 of C0
        L.C0R[(int64_t)row * LAZY_TM + tau] = n0g;
        if (!single) L.C0R[(int64_t)row * LAZY_TM + tau + 1] = n0j;
        double r, dn;
        int kp;
        if (row == g) {
          r = y11 - 2.0 * M1 * y12 + M1 * M1 * y22;          // || -y1 + M1 y2 ||^2
          dn = -Dg - M1 * M1 * Dj;
          kp = 0;
          L.pos[row] = tau; L.Tidx[tau] = row; L.Jsg[tau] = -1.f; L.tslot[tau] = L.misc[MI_SG];
        } else if (row == j) {
          r = y22; dn = -Dj; kp = 1;
          L.pos[row] = tau + 1; L.Tidx[tau + 1] = row; L.Jsg[tau + 1] = 1.f; L.tslot[tau + 1] = L.misc[MI_SJ];
        } else {
          double zy1, zy2;
          if (ps >= 0) { const double sg = (double)L.Jsg[ps]; zy1 = sg * sa[ps]; zy2 = sg * sb[ps]; }
          else { zy1 = w1r - da; zy2 = w2r - db; }
          const double c2 = cjv - c1 * M1;
          r = rho0 - 2.0 * c1 * zy1 + c1 * c1 * y11;           // after the reverse sweep on g
          const double zy2p = zy2 - c1 * y12;                  // (Z_i - c1 y1) . y2
          r += -2.0 * c2 * zy2p + c2 * c2 * y22;               // after the forward sweep on j
          if (r < 0.0) r = 0.0;
          dn = diag0 - c1 * c1 * Dg - c2 * c2 * Dj;
          kp = kp0;
        }
        rho[row] = r; diag[row] = dn; kept[row] = kp;
        const double sc = r / fabs(dn);
        score[row] = sc;
        if (kp) { mn1 = sc; imn = row; } else { mx1 = sc; imx = row; }
      }
    }
    // Per-block record.  The 32 row leaders (lanes 0, 8, 16, ... of each wave) hand their (cost, index) and (gain, index) to
    // the first wave through shared memory; it picks the best of each side by data-parallel moves on (value, index) alone,
    // then the second best as a plain minimum / maximum over the rows that did not win: half the instructions of merging
    // full (best, second, index) records at every step, on what is the longest path through this kernel.
    if ((tid & 7) == 0) { const int e = tid >> 3; s_mn[e] = mn1; s_imn[e] = imn; s_mx[e] = mx1; s_imx[e] = imx; }
    __syncthreads();
    if (tid < 64) {
      const bool have = tid < ROWS_PER_BLOCK;
      double vmn = have ? s_mn[tid & 31] : INFINITY, vmx = have ? s_mx[tid & 31] : -INFINITY;
      int vin = have ? s_imn[tid & 31] : -1, vix = have ? s_imx[tid & 31] : -1;
      const double own_mn = vmn, own_mx = vmx;
      const int own_in = vin, own_ix = vix;
      dpp_best_step<0xb1, 0xf>(vmn, vin, vmx, vix);
      dpp_best_step<0x4e, 0xf>(vmn, vin, vmx, vix);
      dpp_best_step<0x124, 0xf>(vmn, vin, vmx, vix);
      dpp_best_step<0x128, 0xf>(vmn, vin, vmx, vix);
      dpp_best_step<0x142, 0xa>(vmn, vin, vmx, vix);
      dpp_best_step<0x143, 0xc>(vmn, vin, vmx, vix);
      const int win_n = __builtin_amdgcn_readlane(vin, 63), win_x = __builtin_amdgcn_readlane(vix, 63);
      double lo = (own_in >= 0 && own_in != win_n) ? own_mn : INFINITY, hi = (own_ix >= 0 && own_ix != win_x) ? own_mx : -INFINITY;
      dpp_minmax_step<0xb1, 0xf>(lo, hi);
      dpp_minmax_step<0x4e, 0xf>(lo, hi);
      dpp_minmax_step<0x124, 0xf>(lo, hi);
      dpp_minmax_step<0x128, 0xf>(lo, hi);
      dpp_minmax_step<0x142, 0xa>(lo, hi);
      dpp_minmax_step<0x143, 0xc>(lo, hi);
      if (tid == 63) {
        SelRec rec; rec.mn1 = vmn; rec.mn2 = lo; rec.mx1 = vmx; rec.mx2 = hi; rec.imn = vin; rec.imx = vix;
        L.sel[b] = rec;
      }
    }
  } else if (b < row_blocks + col_blocks) {
    const int cb = b - row_blocks, slice = tid >> 6, col = cb * COLS_PER_BLOCK + (tid & 63);
    for (int s = tid; s < LAZY_TM; s += 256) { const double xg = L.xg[s]; sa[s] = xg; sb[s] = L.xj[s] - xg * M1; }
    __syncthreads();
    if (col < m) {
      const double y1 = L.y1[col], y2 = L.y2[col];
      // independent read-modify-writes: issue several before waiting
      int s = slice;
      for (; s + 28 < tau; s += 32) {
        double z[8];
#pragma unroll
        for (int u = 0; u < 8; u++) z[u] = L.ZT[(int64_t)(s + 4 * u) * m + col];
#pragma unroll
        for (int u = 0; u < 8; u++) L.ZT[(int64_t)(s + 4 * u) * m + col] = z[u] - (sa[s + 4 * u] * y1 + sb[s + 4 * u] * y2);
      }
      for (; s < tau; s += 4) L.ZT[(int64_t)s * m + col] -= sa[s] * y1 + sb[s] * y2;
      if (slice == 0) {
        L.ZT[(int64_t)tau * m + col] = y1 - M1 * y2;
        if (!single) L.ZT[(int64_t)(tau + 1) * m + col] = y2;
      }
    }
  } else {
    const int mb = b - row_blocks - col_blocks, nmb = gridDim.x - row_blocks - col_blocks;
    double* Mi = L.Minv;
    for (int idx = mb * 256 + tid; idx < tau * tau; idx += nmb * 256) {
      const int r = idx / tau, s = idx % tau;
      const double xr = L.xg[r], xs = L.xg[s];
      const double pr = L.xj[r] - xr * M1, ps = L.xj[s] - xs * M1;
      Mi[r * LAZY_TM + s] += xr * xs * Dg + pr * ps * Dj;
    }
    if (mb == 0) {
      for (int r = tid; r < tau; r += 256) {
        const double xr = L.xg[r], pr = L.xj[r] - xr * M1;
        const double v = -xr * Dg + pr * M1 * Dj;          // bordered by g, then corrected by the sweep on j
        Mi[r * LAZY_TM + tau] = v; Mi[tau * LAZY_TM + r] = v;
        if (single) continue;
        const double w = -pr * Dj;
        Mi[r * LAZY_TM + tau + 1] = w; Mi[(tau + 1) * LAZY_TM + r] = w;
      }
      if (tid == 0) {
        Mi[tau * LAZY_TM + tau] = Dg + M1 * M1 * Dj;
        if (!single) {
          Mi[tau * LAZY_TM + tau + 1] = -M1 * Dj; Mi[(tau + 1) * LAZY_TM + tau] = -M1 * Dj;
          Mi[(tau + 1) * LAZY_TM + tau + 1] = Dj;
        }
      }
    }
  }
}

hipError_t launch_lazy_iteration(const TabDims& d, const TabPtrs& t, const LazyPtrs& L, int always_accept, hipStream_t s,
                                 hipEvent_t* ev, const int32_t* single, int forced_out, int forced_in) {
  const int rb = (d.d1 + ROWS_PER_BLOCK - 1) / ROWS_PER_BLOCK, cb = (d.m + COLS_PER_BLOCK - 1) / COLS_PER_BLOCK;
  hipLaunchKernelGGL(lazy_prep_kernel, dim3(1), dim3(256), 0, s, L, t.N, d.d1, rb, t.kept, t.ctrl, single, forced_out, forced_in);
  hipLaunchKernelGGL(lazy_vectors_kernel, dim3(rb + cb + (d.d1 + 63) / 64), dim3(256), 0, s, L, t.N, t.Z, d.d1, d.m, rb, cb, t.ctrl);
  const int gb = (d.d1 + GEMV_ROWS - 1) / GEMV_ROWS + LAZY_TM * GEMV_SPLIT;
  if (ev) hipEventRecord(ev[0], s);
  hipLaunchKernelGGL(lazy_gemv_kernel, dim3(gb), dim3(256), 0, s, L, t.Z, d.d1, d.m, cb, t.ctrl, always_accept, t.trace_out,
                     t.trace_in, t.trace_gap, t.trace_obj, single ? 1 : 2);
  if (ev) hipEventRecord(ev[1], s);
  hipLaunchKernelGGL(lazy_update_kernel, dim3(rb + cb + 16), dim3(256), 0, s, L, t.N, d.d1, d.m, rb, cb, t.ctrl, t.kept, t.gram,
                     t.dblk, t.score, single ? 1 : 0);
  if (ev) hipEventRecord(ev[2], s);
  return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// flush: apply the pending correction to N0, Z0 and empty T
// ------------------------------------------------------------------------------------------------
// float32 copies of M^-1 and ZT, zero beyond tau (so that stale columns of C0 drop out of the products)
__global__ __launch_bounds__(256) void lazy_convert_kernel(LazyPtrs L, int m, const SearchCtrl* __restrict__ ctrl) {
  const int tau = tau_all(ctrl);
  const int64_t nz = (int64_t)LAZY_TM * m, nm = (int64_t)LAZY_TM * LAZY_TM;
  for (int64_t idx = blockIdx.x * 256 + threadIdx.x; idx < nz + nm; idx += (int64_t)gridDim.x * 256) {
    if (idx < nz) {
      const int s = (int)(idx / m);
      L.ZT32[idx] = (s < tau) ? (float)L.ZT[idx] : 0.f;
    } else {
      const int64_t k = idx - nz;
      const int r = (int)(k / LAZY_TM), s = (int)(k % LAZY_TM);
      L.Minv32[k] = (r < tau && s < tau) ? (float)L.Minv[k] : 0.f;
    }
  }
}

// pivot rows / columns of N0 and pivot rows of Z0.  Every entry is written by exactly one thread (the pending pivots are
// distinct), so the pivots are spread over blockIdx.y: FIX_SPB of them per thread.
constexpr int FIX_SPB = 8;
__global__ __launch_bounds__(256) void lazy_fix_kernel(LazyPtrs L, float* __restrict__ N0, int d1,
                                                        const SearchCtrl* __restrict__ ctrl) {
  const int l = blockIdx.x * 256 + threadIdx.x;
  if (l >= d1) return;
  const int tau = tau_all(ctrl);
  const int s0 = blockIdx.y * FIX_SPB, s1 = min(tau, s0 + FIX_SPB);
  if (s0 >= s1) return;
  const int pr = L.pos[l];
  if (pr < 0) {
    const float* El = L.E + (int64_t)l * LAZY_TM;
    for (int s = s0; s < s1; s++) {
      const int t = L.Tidx[s];
      const float v = L.Jsg[s] * El[s];
      if (l < t) N0[(int64_t)t * d1 + l] = v; else N0[(int64_t)l * d1 + t] = v;
    }
  } else {
    for (int s = s0; s < s1; s++) {
      const int t = L.Tidx[s];
      if (l >= t) N0[(int64_t)l * d1 + t] = (float)(-(double)L.Jsg[pr] * (double)L.Jsg[s] * L.Minv[pr * LAZY_TM + s]);
    }
  }
}
__global__ __launch_bounds__(256) void lazy_fix_z_kernel(LazyPtrs L, float* __restrict__ Z0, int m,
                                                          const SearchCtrl* __restrict__ ctrl) {
  const int col = blockIdx.x * 256 + threadIdx.x;
  if (col >= m) return;
  const int tau = tau_all(ctrl);
  const int s0 = blockIdx.y * FIX_SPB, s1 = min(tau, s0 + FIX_SPB);
  for (int s = s0; s < s1; s++) Z0[(int64_t)L.Tidx[s] * m + col] = (float)((double)L.Jsg[s] * L.ZT[(int64_t)s * m + col]);
}
__global__ __launch_bounds__(256) void lazy_reset_kernel(LazyPtrs L, SearchCtrl* ctrl) {
  const int tau = tau_all(ctrl);
  for (int s = threadIdx.x; s < tau; s += 256) L.pos[L.Tidx[s]] = -1;
  __syncthreads();
  if (threadIdx.x == 0) { ctrl->tau = 0; ctrl->tau_inc = 0; ctrl->pause = 0; }
}

// ------------------------------------------------------------------------------------------------
// candidate rows and their products with Z0 (after every flush)
// ------------------------------------------------------------------------------------------------
// ascending bitonic sort of 1024 (key, index) pairs in LDS; equal keys: lower index first
__device__ __forceinline__ void bitonic1024(double* key, int* idx, int tid) {
  for (int k = 2; k <= 1024; k <<= 1)
    for (int j = k >> 1; j > 0; j >>= 1) {
      const int other = tid ^ j;
      if (other > tid) {
        const bool up = ((tid & k) == 0);
        const double a = key[tid], b = key[other];
        const int ia = idx[tid], ib = idx[other];
        const bool a_after_b = (a > b) || (a == b && ia > ib);
        if (a_after_b == up) { key[tid] = b; key[other] = a; idx[tid] = ib; idx[other] = ia; }
      }
      __syncthreads();
    }
}

// per block of 1024 groups: the `per_block` cheapest removals among kept rows and the `per_block` largest gains among the others
__global__ __launch_bounds__(1024) void cand_local_kernel(LazyPtrs L, int p, const int32_t* __restrict__ kept,
                                                           const double* __restrict__ score, int per_block) {
  __shared__ double key[1024];
  __shared__ int idx[1024];
  const int tid = threadIdx.x, h = blockIdx.x * 1024 + tid, nblk = gridDim.x;
  for (int side = 0; side < 2; side++) {
    const bool valid = (h < p) && ((kept[h] != 0) == (side == 0));
    key[tid] = valid ? (side == 0 ? score[h] : -score[h]) : INFINITY;
    idx[tid] = valid ? h : 0x7fffffff;
    __syncthreads();
    bitonic1024(key, idx, tid);
    if (tid < per_block) {
      L.lkey[(side * nblk + blockIdx.x) * 32 + tid] = key[tid];
      L.lidx[(side * nblk + blockIdx.x) * 32 + tid] = idx[tid];
    }
    __syncthreads();
  }
}

// merge of the per-block winners: n_k kept rows into slots [0, n_k), n_c others into [n_k, n_k + n_c); unused slots hold -1
__global__ __launch_bounds__(1024) void cand_merge_kernel(LazyPtrs L, int nblk, int per_block, int n_k, int n_c) {
  __shared__ double key[1024];
  __shared__ int idx[1024];
  const int tid = threadIdx.x, total = nblk * per_block;
  for (int s = tid; s < LAZY_NC + LAZY_NS; s += 1024) L.cand[s] = -1;
  if (tid < 8) L.misc[tid] = 0;
  __syncthreads();
  for (int side = 0; side < 2; side++) {
    const int cnt = side == 0 ? n_k : n_c, base = side == 0 ? 0 : n_k;
    if (tid < total) {
      key[tid] = L.lkey[(side * nblk + tid / per_block) * 32 + tid % per_block];
      idx[tid] = L.lidx[(side * nblk + tid / per_block) * 32 + tid % per_block];
    } else { key[tid] = INFINITY; idx[tid] = 0x7fffffff; }
    __syncthreads();
    bitonic1024(key, idx, tid);
    if (tid < cnt && key[tid] < INFINITY) { L.cand[base + tid] = idx[tid]; L.cslot[idx[tid]] = base + tid; }
    __syncthreads();
  }
}

// Zc[s, :] = Z0[cand[s], :] (zero for unused slots)
__global__ __launch_bounds__(256) void cand_gather_kernel(LazyPtrs L, const float* __restrict__ Z0, int m) {
  const int s = blockIdx.x, r = L.cand[s];
  float* dst = L.Zc + (int64_t)s * m;
  for (int c = threadIdx.x; c < m; c += 256) dst[c] = (r >= 0) ? Z0[(int64_t)r * m + c] : 0.f;
}

// ------------------------------------------------------------------------------------------------
// The look-ahead product GbT[s, i] = <Z0[cand[s], :], Z0[i, :]> on the bf16 matrix cores, bound by one read of Z0.
// Every float32 number is cut into three bf16 pieces (each the round-to-nearest bf16 of what the pieces before it leave;
// together 24 significand bits) and the six products of weight >= 2^-16 run as v_mfma_f32_32x32x16_bf16: products of bf16
// numbers are exact in float32, the sums inside the matrix cores restart every 1024 columns (added, round to nearest,
// to a second float32 set), and every element of GbT is written once by the one wave that owns it (no atomics: the
// result does not depend on scheduling).  The candidate rows are cut and laid out in operand order once per flush
// (la_pack_kernel, a few MB that stay in L2); the rows of Z0 are cut in registers, each lane taking 8 consecutive
// columns of one row from the tile in shared memory, which is the operand layout as it stands.
//   one workgroup = 128 rows of Z0 x 128 candidates; wave w owns rows 32 w .. 32 w + 31 as four 32 x 32 tiles.
// ------------------------------------------------------------------------------------------------
typedef float la_f16v __attribute__((ext_vector_type(16)));
typedef __bf16 la_bf8 __attribute__((ext_vector_type(8)));
constexpr int LA_STG = 32;                   // columns of Z per stage (two 16-deep matrix-core steps)
// A workgroup multiplies its rows of Z0 with one block of NC = 32 NT candidates (NT = 4, 5 or 6 tiles of 32 per wave);
// packets per stage and block: 3 pieces x 4 groups of 8 columns x NC candidates.

__device__ __forceinline__ uint32_t la_rne(float x) {
  const uint32_t u = __float_as_uint(x);
  return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
}
// v[0..8) -> three packets of 8 bf16 each
__device__ __forceinline__ void la_split3(const float* v, uint4& p1, uint4& p2, uint4& p3) {
  uint32_t h1[8], h2[8], h3[8];
#pragma unroll
  for (int j = 0; j < 8; j++) {
    const uint32_t b1 = la_rne(v[j]);
    const float r1 = v[j] - __uint_as_float(b1 << 16);
    const uint32_t b2 = la_rne(r1);
    const float r2 = r1 - __uint_as_float(b2 << 16);
    h1[j] = b1; h2[j] = b2; h3[j] = la_rne(r2);
  }
  p1 = uint4{h1[0] | (h1[1] << 16), h1[2] | (h1[3] << 16), h1[4] | (h1[5] << 16), h1[6] | (h1[7] << 16)};
  p2 = uint4{h2[0] | (h2[1] << 16), h2[2] | (h2[3] << 16), h2[4] | (h2[5] << 16), h2[6] | (h2[7] << 16)};
  p3 = uint4{h3[0] | (h3[1] << 16), h3[2] | (h3[3] << 16), h3[4] | (h3[5] << 16), h3[6] | (h3[7] << 16)};
}

// ZcP[(sb * nstg + stage) * 12 nc + piece * 4 nc + kg * nc + s] = columns stage*32 + kg*8 .. +8 of candidate sb*nc + s, piece
// `piece` (zero for unused slots and beyond column m).  grid (nstg, number of blocks of nc candidates), 256 threads.
__global__ __launch_bounds__(256) void la_pack_kernel(LazyPtrs L, const float* __restrict__ Z0, int m, int nstg, int nc, uint4* __restrict__ ZcP) {
  const int stage = blockIdx.x, sb = blockIdx.y, tid = threadIdx.x;
  uint4* out = ZcP + ((int64_t)sb * nstg + stage) * 12 * nc;
  for (int pk = tid; pk < 4 * nc; pk += 256) {
    const int kg = pk / nc, sl = pk % nc;
    const int r = L.cand[sb * nc + sl], c0 = stage * LA_STG + kg * 8;
    float v[8];
#pragma unroll
    for (int j = 0; j < 8; j++) v[j] = 0.f;
    if (r >= 0 && c0 + 8 <= m) {
      const float4 a = *reinterpret_cast<const float4*>(Z0 + (int64_t)r * m + c0);
      const float4 b = *reinterpret_cast<const float4*>(Z0 + (int64_t)r * m + c0 + 4);
      v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w; v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
    }
    uint4 p1, p2, p3;
    la_split3(v, p1, p2, p3);
    out[pk] = p1; out[4 * nc + pk] = p2; out[8 * nc + pk] = p3;
  }
}

// GbT[(sb * NC + s) * d1 + i] for i in [128 blockIdx.x, +128), s in [0, NC), sb = blockIdx.y, NC = 32 NT.  m % 8 == 0.
// Per stage of 32 columns the workgroup copies its 128 x 32 tile of Z0 (each row's 128 bytes by eight neighbouring lanes)
// and the candidates' packed pieces into shared memory; the next stage's loads are in flight while this one is
// multiplied.  Two workgroups share a compute unit.
constexpr int LA_ZLD = LA_STG + 4;           // row stride of the Z0 tile in shared memory (floats)
template <int NT>
__global__ __launch_bounds__(256, 2) void la_product_kernel(const uint4* __restrict__ ZcP, const float* __restrict__ Z0, int d1, int m,
                                                             int nstg, double* __restrict__ GbT) {
  constexpr int NC = 32 * NT, PK = 12 * NC, NLD = (PK + 255) / 256;      // candidates, packets per stage, loads per thread
  __shared__ uint4 lzc[PK];                                    // 6 KB per 32 candidates
  __shared__ __attribute__((aligned(16))) float lz0[128 * LA_ZLD];   // 18 KB
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, sb = blockIdx.y;
  const int i0 = blockIdx.x * 128;
  // blockIdx.z: which part of the contraction (gridDim.z = 1, or 2 with the sums joined by atomic additions to a zeroed GbT:
  // two terms added to zero give the same bits in either order)
  const int st_begin = (int)blockIdx.z * ((nstg + (int)gridDim.z - 1) / (int)gridDim.z);
  const int st_end = min(nstg, st_begin + (nstg + (int)gridDim.z - 1) / (int)gridDim.z);
  const uint4* src = ZcP + (int64_t)sb * nstg * PK + tid;
  // global -> shared assignment of the Z0 tile: thread t takes 4 columns (t % 8) * 4 of rows t / 8 + 32 j, j < 4
  const int lr = tid >> 3, lk = (tid & 7) * 4;
  auto rowp = [&](int j) { const int row = i0 + lr + 32 * j; return Z0 + (int64_t)(row < d1 ? row : d1 - 1) * m + lk; };
  const float *zsrc0 = rowp(0), *zsrc1 = rowp(1), *zsrc2 = rowp(2), *zsrc3 = rowp(3);      // rows past the end: clamped, never stored
  la_f16v acc[NT], acc2[NT];
#pragma unroll
  for (int t = 0; t < NT; t++)
#pragma unroll
    for (int r = 0; r < 16; r++) { acc[t][r] = 0.f; acc2[t][r] = 0.f; }
  uint4 zc[NLD];
  float4 zt0, zt1, zt2, zt3;
  auto gload = [&](int stage_) {
    const uint4* p_ = src + (int64_t)stage_ * PK;
#pragma unroll
    for (int i = 0; i < NLD; i++) zc[i] = (tid + 256 * i < PK) ? p_[256 * i] : uint4{0u, 0u, 0u, 0u};
    const bool in_ = stage_ * LA_STG + lk < m;              /* m % 4 == 0: a float4 is inside or outside as a whole */
    const float4 z_ = float4{0.f, 0.f, 0.f, 0.f};
    zt0 = in_ ? *reinterpret_cast<const float4*>(zsrc0 + stage_ * LA_STG) : z_;
    zt1 = in_ ? *reinterpret_cast<const float4*>(zsrc1 + stage_ * LA_STG) : z_;
    zt2 = in_ ? *reinterpret_cast<const float4*>(zsrc2 + stage_ * LA_STG) : z_;
    zt3 = in_ ? *reinterpret_cast<const float4*>(zsrc3 + stage_ * LA_STG) : z_;
  };
  if (st_begin >= st_end) return;
  gload(st_begin);
  int since = 0;
  const float* myrow = lz0 + (wave * 32 + (lane & 31)) * LA_ZLD + (lane >> 5) * 8;
  for (int stage = st_begin; stage < st_end; stage++) {
    __syncthreads();                                           // the previous stage has been read by every wave
#pragma unroll
    for (int i = 0; i < NLD; i++)
      if (tid + 256 * i < PK) lzc[tid + 256 * i] = zc[i];
    *reinterpret_cast<float4*>(lz0 + lr * LA_ZLD + lk) = zt0;
    *reinterpret_cast<float4*>(lz0 + (lr + 32) * LA_ZLD + lk) = zt1;
    *reinterpret_cast<float4*>(lz0 + (lr + 64) * LA_ZLD + lk) = zt2;
    *reinterpret_cast<float4*>(lz0 + (lr + 96) * LA_ZLD + lk) = zt3;
    __syncthreads();
    if (stage + 1 < st_end) gload(stage + 1);
#pragma unroll
    for (int ks = 0; ks < LA_STG / 16; ks++) {
      const float4 v0 = *reinterpret_cast<const float4*>(myrow + ks * 16), v1 = *reinterpret_cast<const float4*>(myrow + ks * 16 + 4);
      const float v[8] = {v0.x, v0.y, v0.z, v0.w, v1.x, v1.y, v1.z, v1.w};
      uint4 b1, b2, b3;
      la_split3(v, b1, b2, b3);
      const la_bf8 f1 = *reinterpret_cast<const la_bf8*>(&b1), f2 = *reinterpret_cast<const la_bf8*>(&b2), f3 = *reinterpret_cast<const la_bf8*>(&b3);
      const int off = (ks * 2 + (lane >> 5)) * NC + (lane & 31);
#pragma unroll
      for (int t = 0; t < NT; t++) {
        uint4 q1 = lzc[off + t * 32], q2 = lzc[4 * NC + off + t * 32], q3 = lzc[8 * NC + off + t * 32];
        const la_bf8 a1 = *reinterpret_cast<la_bf8*>(&q1), a2 = *reinterpret_cast<la_bf8*>(&q2), a3 = *reinterpret_cast<la_bf8*>(&q3);
        // smallest terms first
        acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a3, f1, acc[t], 0, 0, 0);
        acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a2, f2, acc[t], 0, 0, 0);
        acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1, f3, acc[t], 0, 0, 0);
        acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a2, f1, acc[t], 0, 0, 0);
        acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1, f2, acc[t], 0, 0, 0);
        acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1, f1, acc[t], 0, 0, 0);
      }
    }
    if (++since == 1024 / LA_STG && stage + 1 < st_end) {     // the sums inside the matrix cores never span more than 1024 columns
      since = 0;
#pragma unroll
      for (int t = 0; t < NT; t++)
#pragma unroll
        for (int r = 0; r < 16; r++) { acc2[t][r] += acc[t][r]; acc[t][r] = 0.f; }
    }
  }
  // C layout of the 32 x 32 tile: register r = rr*4 + r3 holds row rr*8 + (lane/32)*4 + r3 (a candidate), column lane%32 (a row of Z0)
  const int i_lane = i0 + wave * 32 + (lane & 31);
  if (i_lane < d1) {
#pragma unroll
    for (int t = 0; t < NT; t++)
#pragma unroll
      for (int r = 0; r < 16; r++) {
        const int sl = t * 32 + (r >> 2) * 8 + (lane >> 5) * 4 + (r & 3);
        double* dst = GbT + (int64_t)(sb * NC + sl) * d1 + i_lane;
        const double v = (double)acc[t][r] + (double)acc2[t][r];
        if (gridDim.z == 1) *dst = v; else unsafeAtomicAdd(dst, v);
      }
  }
}

// mode 0: half of the slots for kept rows, half for the others; 1: all for kept rows (removal-only loops); 2: none
struct CandCounts { int n_k, n_c; };
static CandCounts cand_counts(int mode) {
  // Swap search: a cycle of 64 swaps takes 64 pivots from each side, and which rows they will be is known at flush time only
  // up to the changes the swaps themselves make to the scores.  With exactly 64 + 64 rows picked, 8 % of the leaving and 2 %
  // of the entering pivots of the 28672 x 7168 layer were not among them, and each such swap pays a pass over Z0 for the
  // missing products (0.155 ms: 70 ms over 5000 swaps).  With 88 + 72 it is 0.4 % and 0.2 % (80 + 80: 1.3 % and none;
  // 96 + 64: 0.2 % and 2 %), for a product that is a quarter longer.  256 picked rows (two blocks of the product) cost more
  // than they save.  The removal-only loops take all LAZY_NC rows: their block pivots cannot fetch a missing product.
  static_assert((LAZY_NPICK_OUT + LAZY_NPICK_IN) % 32 == 0 && LAZY_NPICK_OUT + LAZY_NPICK_IN <= LAZY_NC, "blocks of 32 candidates");
  return CandCounts{mode == 2 ? 0 : (mode == 1 ? LAZY_NC : LAZY_NPICK_OUT), mode == 0 ? LAZY_NPICK_IN : 0};
}
// the pick: reads the scores and the kept flags only (two sorts in one workgroup each: latency, no bandwidth)
static hipError_t launch_candidate_pick(const TabDims& d, const TabPtrs& t, const LazyPtrs& L, hipStream_t s, int mode) {
  const int nblk = (d.p + 1023) / 1024;               // <= 64 (d1 <= 65536)
  const int per_block = std::min(32, 1024 / nblk);
  hipError_t e = hipMemsetAsync(L.cslot, 0xFF, (size_t)d.d1 * 4, s);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(cand_local_kernel, dim3(nblk), dim3(1024), 0, s, L, d.p, t.kept, t.score, per_block);
  const CandCounts cc = cand_counts(mode);
  hipLaunchKernelGGL(cand_merge_kernel, dim3(1), dim3(1024), 0, s, L, nblk, per_block, cc.n_k, cc.n_c);
  return hipGetLastError();
}
// the products of the picked rows with the (flushed) Z0
static hipError_t launch_candidate_products(const TabDims& d, const TabPtrs& t, const LazyPtrs& L, hipStream_t s, int mode) {
  const CandCounts cc = cand_counts(mode);
  const int n_k = cc.n_k, n_c = cc.n_c;
  if (mode == 2) return hipSuccess;
  // one block of 32 NT candidates per workgroup: 128 (and multiples of it, block by block), 160 or 192
  const int ncand = n_k + n_c;
  const int nt = (ncand % 128 == 0) ? 4 : ((ncand == 160) ? 5 : ((ncand == 192) ? 6 : 0));
  if (d.m % 8 == 0 && nt > 0) {
    const int nstg = (d.m + LA_STG - 1) / LA_STG, nc = 32 * nt, nsb = ncand / nc;
    hipLaunchKernelGGL(la_pack_kernel, dim3(nstg, nsb), dim3(256), 0, s, L, t.Z, d.m, nstg, nc, reinterpret_cast<uint4*>(L.ZcP));
    // one block of candidates: 224 workgroups for 28672 rows would leave compute units empty and each of them with one
    // latency chain over all of m; the contraction is then cut in two
    const int ksplit = (((d.d1 + 127) / 128) * nsb < 400 && nstg >= 64) ? 2 : 1;
    if (ksplit > 1) {
      const hipError_t ez = hipMemsetAsync(L.GbT, 0, (size_t)ncand * d.d1 * sizeof(double), s);
      if (ez != hipSuccess) return ez;
    }
    const dim3 grid((d.d1 + 127) / 128, nsb, ksplit);
    const uint4* zcp = reinterpret_cast<const uint4*>(L.ZcP);
    if (nt == 4) hipLaunchKernelGGL(la_product_kernel<4>, grid, dim3(256), 0, s, zcp, t.Z, d.d1, d.m, nstg, L.GbT);
    else if (nt == 5) hipLaunchKernelGGL(la_product_kernel<5>, grid, dim3(256), 0, s, zcp, t.Z, d.d1, d.m, nstg, L.GbT);
    else hipLaunchKernelGGL(la_product_kernel<6>, grid, dim3(256), 0, s, zcp, t.Z, d.d1, d.m, nstg, L.GbT);
    return hipGetLastError();
  }
  // other shapes: the general matrix-product kernel on the gathered rows
  hipLaunchKernelGGL(cand_gather_kernel, dim3(n_k + n_c), dim3(256), 0, s, L, t.Z, d.m);
  GemmArgs g{};                         // GbT[0 .. LAZY_NC) = Zc Z0^T, float64 accumulation and output
  g.M = n_k + n_c; g.N = d.d1; g.K = d.m; g.A = L.Zc; g.lda = d.m; g.B = t.Z; g.ldb = d.m; g.trans_b = 1;
  g.C = L.GbT; g.ldc = d.d1; g.alpha = 1.0; g.beta = 0.0; g.c_is_f64 = 1;
  return launch_gemm_f64acc(g, s);
}
static hipError_t launch_candidates(const TabDims& d, const TabPtrs& t, const LazyPtrs& L, hipStream_t s, int mode) {
  const hipError_t e = launch_candidate_pick(d, t, L, s, mode);
  return e != hipSuccess ? e : launch_candidate_products(d, t, L, s, mode);
}

static hipError_t launch_partials(const TabDims& d, const TabPtrs& t, const LazyPtrs& L, hipStream_t s) {
  const int rb = (d.d1 + ROWS_PER_BLOCK - 1) / ROWS_PER_BLOCK;
  hipLaunchKernelGGL(lazy_partials_kernel, dim3(rb), dim3(64), 0, s, L, d.p, t.kept, t.score);
  return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// The two rank-LAZY_TM updates of a flush, C -= A B^T with A (M x 128) and B (N x 128): N0 -= E C0^T on the lower block
// triangle and Z0 -= C0 ZT.  Both are bound by the read and write of C once the product itself is cheap, so the three
// thin operands (E, C0, ZT: a few MB) are cut into three bf16 pieces once per flush and laid out in matrix-core operand
// order (rk_pack_*), and the six products of weight >= 2^-16 run as v_mfma_f32_32x32x16_bf16 (exact products, float32
// sums over the 128 terms): a sixth of the matrix-core time of the float32 instruction for the same accuracy.
// Layout of a packed operand: packet (piece, kg, row) = columns 8 kg .. 8 kg + 7 of `row`, at (piece * 16 + kg) * rpad + row.
// One workgroup per 128 x 128 tile of C (the Gram kernel's tile schedules), four quarters of the contraction through
// 48 KB of shared memory, two workgroups per compute unit so that one's read-modify-write of C overlaps the other's products.
// ------------------------------------------------------------------------------------------------
// X: rows x 128 row-major (ld = 128): thread = one packet
__global__ __launch_bounds__(256) void rk_pack_rows_kernel(const float* __restrict__ X, int rows, int rpad, uint4* __restrict__ out) {
  const int idx = blockIdx.x * 256 + threadIdx.x;          // (kg, row), row fastest
  if (idx >= 16 * rpad) return;
  const int kg = idx / rpad, row = idx % rpad;
  float v[8];
#pragma unroll
  for (int j = 0; j < 8; j++) v[j] = 0.f;
  if (row < rows) {
    const float4 a = *reinterpret_cast<const float4*>(X + (int64_t)row * LAZY_TM + kg * 8);
    const float4 b = *reinterpret_cast<const float4*>(X + (int64_t)row * LAZY_TM + kg * 8 + 4);
    v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w; v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
  }
  uint4 p1, p2, p3;
  la_split3(v, p1, p2, p3);
  out[(int64_t)kg * rpad + row] = p1;
  out[(int64_t)(16 + kg) * rpad + row] = p2;
  out[(int64_t)(32 + kg) * rpad + row] = p3;
}
// X: 128 x cols row-major (the contraction runs along the rows): packet (kg, c) = X[8 kg .. 8 kg + 7][c]
__global__ __launch_bounds__(256) void rk_pack_cols_kernel(const float* __restrict__ X, int cols, int cpad, uint4* __restrict__ out) {
  const int idx = blockIdx.x * 256 + threadIdx.x;
  if (idx >= 16 * cpad) return;
  const int kg = idx / cpad, c = idx % cpad;
  float v[8];
#pragma unroll
  for (int j = 0; j < 8; j++) v[j] = (c < cols) ? X[(int64_t)(kg * 8 + j) * cols + c] : 0.f;
  uint4 p1, p2, p3;
  la_split3(v, p1, p2, p3);
  out[(int64_t)kg * cpad + c] = p1;
  out[(int64_t)(16 + kg) * cpad + c] = p2;
  out[(int64_t)(32 + kg) * cpad + c] = p3;
}

// Sums of squares of the new values of a wave's 32 rows x 64 columns, one number per row, into out[row] (rows_left of them
// exist).  v0, v1: the two 32 x 32 tiles side by side in the matrix cores' result layout (register r = rr*4 + r3 holds row
// rr*8 + (lane/32)*4 + r3, column lane%32).  Squares and sums in float64; the 32 lanes of a half wave are added by
// data-parallel moves in a fixed order, and lanes 31 and 63 write.
__device__ __forceinline__ void rk_row_squares(const float* v0, const float* v1, double* __restrict__ out, int lane, int rows_left) {
#pragma unroll
  for (int r = 0; r < 16; r++) {
    double q = (double)v0[r] * (double)v0[r] + (double)v1[r] * (double)v1[r];
    q += dpp_get<0xb1, 0xf>(q);        // quad_perm [1, 0, 3, 2]
    q += dpp_get<0x4e, 0xf>(q);        // quad_perm [2, 3, 0, 1]
    q += dpp_get<0x124, 0xf>(q);       // row_ror:4
    q += dpp_get<0x128, 0xf>(q);       // row_ror:8
    q += dpp_get<0x142, 0xa>(q);       // row_bcast:15 into rows 1 and 3: lanes 16-31 and 48-63 hold their half wave's sum
    const int row = (r >> 2) * 8 + (lane >> 5) * 4 + (r & 3);
    if ((lane & 31) == 31 && row < rows_left) out[row] = q;
  }
}

__global__ __launch_bounds__(256, 2) void rk_update_kernel(const uint4* __restrict__ Apk, int apad, const uint4* __restrict__ Bpk, int bpad,
                                                            float* __restrict__ C, int64_t ldc, int M, int N,
                                                            const int2* __restrict__ tiles, double* __restrict__ rowsq) {
  __shared__ uint4 la[3 * 4 * 128], lb[3 * 4 * 128];          // 24 KB each: [piece][kg of this quarter][row]
  const int2 tile = tiles[blockIdx.x];
  if (tile.x < 0) return;
  const int i0 = tile.x * 128, j0 = tile.y * 128;
  if (i0 >= M || j0 >= N) return;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, wm = wave >> 1, wn = wave & 1;
  la_f16v acc[2][2];
#pragma unroll
  for (int a = 0; a < 2; a++)
#pragma unroll
    for (int b = 0; b < 2; b++)
#pragma unroll
      for (int r = 0; r < 16; r++) acc[a][b][r] = 0.f;
  // packet tid + 256 u of a quarter's 1536: piece = idx / 512, kg = (idx / 128) % 4, row = idx % 128
  uint4 ra0, ra1, ra2, ra3, ra4, ra5, rb0, rb1, rb2, rb3, rb4, rb5;
#define OSSCAR_RK_ADDR(P_, pad_, base_, u_, kq_) \
  ((P_) + (int64_t)((((tid + 256 * (u_)) >> 9) * 16 + (kq_) * 4 + (((tid + 256 * (u_)) >> 7) & 3))) * (pad_) + (base_) + ((tid + 256 * (u_)) & 127))
#define OSSCAR_RK_GLOAD(kq_)                                                                                       \
  {                                                                                                                \
    ra0 = *OSSCAR_RK_ADDR(Apk, apad, i0, 0, kq_); ra1 = *OSSCAR_RK_ADDR(Apk, apad, i0, 1, kq_);                    \
    ra2 = *OSSCAR_RK_ADDR(Apk, apad, i0, 2, kq_); ra3 = *OSSCAR_RK_ADDR(Apk, apad, i0, 3, kq_);                    \
    ra4 = *OSSCAR_RK_ADDR(Apk, apad, i0, 4, kq_); ra5 = *OSSCAR_RK_ADDR(Apk, apad, i0, 5, kq_);                    \
    rb0 = *OSSCAR_RK_ADDR(Bpk, bpad, j0, 0, kq_); rb1 = *OSSCAR_RK_ADDR(Bpk, bpad, j0, 1, kq_);                    \
    rb2 = *OSSCAR_RK_ADDR(Bpk, bpad, j0, 2, kq_); rb3 = *OSSCAR_RK_ADDR(Bpk, bpad, j0, 3, kq_);                    \
    rb4 = *OSSCAR_RK_ADDR(Bpk, bpad, j0, 4, kq_); rb5 = *OSSCAR_RK_ADDR(Bpk, bpad, j0, 5, kq_);                    \
  }
#define OSSCAR_RK_STAGE()                                                                                          \
  {                                                                                                                \
    __syncthreads();                                                                                               \
    la[tid] = ra0; la[tid + 256] = ra1; la[tid + 512] = ra2; la[tid + 768] = ra3; la[tid + 1024] = ra4; la[tid + 1280] = ra5; \
    lb[tid] = rb0; lb[tid + 256] = rb1; lb[tid + 512] = rb2; lb[tid + 768] = rb3; lb[tid + 1024] = rb4; lb[tid + 1280] = rb5; \
    __syncthreads();                                                                                               \
  }
// the six piece products of a quarter, smallest terms first
#define OSSCAR_RK_PRODUCTS()                                                                                       \
  _Pragma("unroll") for (int ks = 0; ks < 2; ks++) {                                                               \
    const int off = (ks * 2 + (lane >> 5)) * 128 + (lane & 31);                                                    \
    la_bf8 fa[2][3], fb[2][3];                                                                                     \
    _Pragma("unroll") for (int a = 0; a < 2; a++)                                                                  \
      _Pragma("unroll") for (int p = 0; p < 3; p++) { uint4 q = la[p * 512 + off + wm * 64 + a * 32]; fa[a][p] = *reinterpret_cast<la_bf8*>(&q); } \
    _Pragma("unroll") for (int b = 0; b < 2; b++)                                                                  \
      _Pragma("unroll") for (int p = 0; p < 3; p++) { uint4 q = lb[p * 512 + off + wn * 64 + b * 32]; fb[b][p] = *reinterpret_cast<la_bf8*>(&q); } \
    _Pragma("unroll") for (int a = 0; a < 2; a++)                                                                  \
      _Pragma("unroll") for (int b = 0; b < 2; b++) {                                                              \
        acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[a][2], fb[b][0], acc[a][b], 0, 0, 0);               \
        acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[a][0], fb[b][2], acc[a][b], 0, 0, 0);               \
        acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[a][1], fb[b][1], acc[a][b], 0, 0, 0);               \
        acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[a][1], fb[b][0], acc[a][b], 0, 0, 0);               \
        acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[a][0], fb[b][1], acc[a][b], 0, 0, 0);               \
        acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[a][0], fb[b][0], acc[a][b], 0, 0, 0);               \
      }                                                                                                            \
  }
  OSSCAR_RK_GLOAD(0);
#pragma unroll 1
  for (int kq = 0; kq < 3; kq++) {
    OSSCAR_RK_STAGE();
    OSSCAR_RK_GLOAD(kq + 1);
    OSSCAR_RK_PRODUCTS();
  }
  OSSCAR_RK_STAGE();
  // C layout of a 32 x 32 tile: register r = rr*4 + r3 holds row rr*8 + (lane/32)*4 + r3, column lane%32.
  // A whole tile's values of C are requested before the last quarter's products, in the registers the operand loads have
  // left free, so that their way from memory runs beside the matrix-core work instead of after it (requesting half of them
  // a quarter earlier changed nothing).
  float* cbase = C + (int64_t)(i0 + wm * 64 + (lane >> 5) * 4) * ldc + j0 + wn * 64 + (lane & 31);
  const bool whole = (i0 + 128 <= M && j0 + 128 <= N);
  float cv[2][2][16];
  if (whole) {
#pragma unroll
    for (int a = 0; a < 2; a++)
#pragma unroll
      for (int r = 0; r < 16; r++) {
        const float* pr = cbase + (int64_t)(a * 32 + (r >> 2) * 8 + (r & 3)) * ldc;
        cv[a][0][r] = pr[0]; cv[a][1][r] = pr[32];
      }
  }
  OSSCAR_RK_PRODUCTS();
#undef OSSCAR_RK_PRODUCTS
#undef OSSCAR_RK_STAGE
#undef OSSCAR_RK_GLOAD
#undef OSSCAR_RK_ADDR
  if (whole) {
#pragma unroll
    for (int a = 0; a < 2; a++) {
      float* ca = cbase + (int64_t)(a * 32) * ldc;
#pragma unroll
      for (int r = 0; r < 16; r++) {
        float* pr = ca + (int64_t)((r >> 2) * 8 + (r & 3)) * ldc;
        cv[a][0][r] -= acc[a][0][r]; cv[a][1][r] -= acc[a][1][r];
        pr[0] = cv[a][0][r]; pr[32] = cv[a][1][r];
      }
      if (rowsq) rk_row_squares(cv[a][0], cv[a][1], rowsq + (int64_t)(tile.y * 2 + wn) * M + i0 + wm * 64 + a * 32, lane, M - (i0 + wm * 64 + a * 32));
    }
  } else {
#pragma unroll
    for (int a = 0; a < 2; a++) {
      float nv[2][16];
#pragma unroll
      for (int b = 0; b < 2; b++) {
        const int col = j0 + wn * 64 + b * 32 + (lane & 31);
        float cv[16];
#pragma unroll
        for (int r = 0; r < 16; r++) {
          const int row = i0 + wm * 64 + a * 32 + (r >> 2) * 8 + (lane >> 5) * 4 + (r & 3);
          cv[r] = (row < M && col < N) ? C[(int64_t)row * ldc + col] : 0.f;
        }
#pragma unroll
        for (int r = 0; r < 16; r++) {
          const int row = i0 + wm * 64 + a * 32 + (r >> 2) * 8 + (lane >> 5) * 4 + (r & 3);
          const bool in = row < M && col < N;
          nv[b][r] = in ? cv[r] - acc[a][b][r] : 0.f;
          if (in) C[(int64_t)row * ldc + col] = nv[b][r];
        }
      }
      if (rowsq) rk_row_squares(nv[0], nv[1], rowsq + (int64_t)(tile.y * 2 + wn) * M + i0 + wm * 64 + a * 32, lane, M - (i0 + wm * 64 + a * 32));
    }
  }
}

// E = C0 M^-1 of the flush (d1 x 128 times 128 x 128, float32 operands, float64 sums on v_mfma_f64_16x16x4_f64, float32
// result).  It stands at the head of the flush's longest chain, so what counts is its latency: the general matrix-product
// kernel runs it as 224 workgroups of one 128 x 128 tile each (0.085 ms); here a workgroup takes 64 rows with all of M^-1
// and its rows of C0 in shared memory (448 workgroups, no barrier inside the contraction).  M^-1 is symmetric bit for bit,
// so its rows serve as the columns the product needs.  Wave w: rows 16 w .. 16 w + 15, eight 16 x 16 tiles.
typedef double te_d4 __attribute__((ext_vector_type(4)));
constexpr int TE_LD = LAZY_TM + 4;       // row stride in shared memory (floats): a quarter wave's 16 rows x 4 k fall on 32 banks twice
__global__ __launch_bounds__(256) void thin_e_kernel(const float* __restrict__ C0R, const float* __restrict__ M32, float* __restrict__ E,
                                                      int d1) {
  static_assert(LAZY_TM == 128, "eight column tiles, thirty-two steps of four");
  extern __shared__ float te_lds[];      // [128 rows of M^-1 | 64 rows of C0][TE_LD]
  float* Ms = te_lds;
  float* As = te_lds + LAZY_TM * TE_LD;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, i0 = blockIdx.x * 64;
  for (int idx = tid; idx < LAZY_TM * (LAZY_TM / 4); idx += 256) {
    const int r = idx >> 5, c4 = (idx & 31) * 4;
    *reinterpret_cast<float4*>(Ms + r * TE_LD + c4) = *reinterpret_cast<const float4*>(M32 + r * LAZY_TM + c4);
  }
  for (int idx = tid; idx < 64 * (LAZY_TM / 4); idx += 256) {
    const int r = idx >> 5, c4 = (idx & 31) * 4;
    const float4 v = (i0 + r < d1) ? *reinterpret_cast<const float4*>(C0R + (int64_t)(i0 + r) * LAZY_TM + c4) : float4{0.f, 0.f, 0.f, 0.f};
    *reinterpret_cast<float4*>(As + r * TE_LD + c4) = v;
  }
  __syncthreads();
  te_d4 acc[8];
#pragma unroll
  for (int ct = 0; ct < 8; ct++) acc[ct] = te_d4{0.0, 0.0, 0.0, 0.0};
  const float* arow = As + (wave * 16 + (lane & 15)) * TE_LD + (lane >> 4);
  const float* mrow = Ms + (lane & 15) * TE_LD + (lane >> 4);
#pragma unroll 4
  for (int k0 = 0; k0 < LAZY_TM; k0 += 4) {
    const double a = (double)arow[k0];
#pragma unroll
    for (int ct = 0; ct < 8; ct++) acc[ct] = __builtin_amdgcn_mfma_f64_16x16x4f64(a, (double)mrow[ct * 16 * TE_LD + k0], acc[ct], 0, 0, 0);
  }
  // lane holds D[4 r + lane/16][lane%16] of each 16 x 16 tile
#pragma unroll
  for (int r = 0; r < 4; r++) {
    const int row = i0 + wave * 16 + 4 * r + (lane >> 4);
    if (row < d1) {
#pragma unroll
      for (int ct = 0; ct < 8; ct++) E[(int64_t)row * LAZY_TM + ct * 16 + (lane & 15)] = (float)acc[ct][r];
    }
  }
}

// First half of the score refresh after a flush: gram[h] = |Z0[h, :]|^2 from the stretch sums that Z0's update left (added in
// a fixed order), dblk[h] = N0[h][h].  The pending pivots' rows were rewritten after the update (the fix): the trailing
// LAZY_TM workgroups take one of them each and sum its squares from Z0 itself (wave sums, then the four waves in order).
__global__ __launch_bounds__(256) void norms_from_stretches_kernel(LazyPtrs L, int d1, int m, int nstretch, int row_blocks,
                                                                    const float* __restrict__ N0, const float* __restrict__ Z0,
                                                                    double* __restrict__ gram, double* __restrict__ dblk,
                                                                    const SearchCtrl* __restrict__ ctrl) {
  if ((int)blockIdx.x < row_blocks) {
    const int h = blockIdx.x * 256 + threadIdx.x;
    if (h >= d1) return;
    dblk[h] = (double)N0[(int64_t)h * d1 + h];
    if (L.pos[h] >= 0) return;                     // a pending pivot: its row is summed below
    double v = 0;
    for (int p0 = 0; p0 < nstretch; p0 += 8) {     // eight loads in flight
      double q[8];
#pragma unroll
      for (int u = 0; u < 8; u++) q[u] = (p0 + u < nstretch) ? L.rowsq[(int64_t)(p0 + u) * d1 + h] : 0.0;
#pragma unroll
      for (int u = 0; u < 8; u++) v += q[u];
    }
    gram[h] = v;
    return;
  }
  __shared__ double red[4];
  const int sidx = blockIdx.x - row_blocks;
  if (sidx >= tau_all(ctrl)) return;
  const int h = L.Tidx[sidx];
  const float* z = Z0 + (int64_t)h * m;
  double v = 0;
  for (int c = threadIdx.x; c < m; c += 256) v += (double)z[c] * (double)z[c];
  v = wsum(v);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
  __syncthreads();
  if (threadIdx.x == 0) gram[h] = red[0] + red[1] + red[2] + red[3];
}

hipError_t launch_lazy_flush(const TabDims& d, const TabPtrs& t, const LazyPtrs& L, hipStream_t s, int mode,
                             const SideStream* side) {
  const int rb = (d.d1 + 255) / 256, mb = (d.m + 255) / 256;
  const bool two = side && side->stream;
  hipStream_t sn = two ? side->stream : s;          // stream of the N0 update
  hipError_t err;
  hipLaunchKernelGGL(lazy_convert_kernel, dim3(512), dim3(256), 0, s, L, d.m, t.ctrl);
  {                                     // E = C0 M^-1 (entered in the log of matrix products like the general kernel's launches)
    const size_t shmem = (size_t)(LAZY_TM + 64) * TE_LD * sizeof(float);
    if ((err = hipFuncSetAttribute(reinterpret_cast<const void*>(thin_e_kernel), hipFuncAttributeMaxDynamicSharedMemorySize, (int)shmem)) != hipSuccess)
      return err;
    int log_slot = -1;
    gemm_log_open(d.d1, LAZY_TM, LAZY_TM, 0, s, &log_slot);
    hipLaunchKernelGGL(thin_e_kernel, dim3((d.d1 + 63) / 64), dim3(256), shmem, s, L.C0R, L.Minv32, L.E, d.d1);
    gemm_log_close(log_slot, s);
  }
  // the three thin operands in matrix-core order (C0's pieces serve both updates)
  const int dpad = (d.d1 + 127) / 128 * 128, mpad = (d.m + 127) / 128 * 128;
  uint4* Epk = reinterpret_cast<uint4*>(L.Epk); uint4* Cpk = reinterpret_cast<uint4*>(L.Cpk); uint4* Zpk = reinterpret_cast<uint4*>(L.Zpk);
  hipLaunchKernelGGL(rk_pack_rows_kernel, dim3((16 * dpad + 255) / 256), dim3(256), 0, s, L.C0R, d.d1, dpad, Cpk);
  hipLaunchKernelGGL(rk_pack_rows_kernel, dim3((16 * dpad + 255) / 256), dim3(256), 0, s, L.E, d.d1, dpad, Epk);
  hipLaunchKernelGGL(rk_pack_cols_kernel, dim3((16 * mpad + 255) / 256), dim3(256), 0, s, L.ZT32, d.m, mpad, Zpk);
  if (two) {
    if ((err = hipEventRecord(side->fork, s)) != hipSuccess) return err;
    if ((err = hipStreamWaitEvent(sn, side->fork, 0)) != hipSuccess) return err;
  }
  // N0 -= E C0^T on the lower block triangle (pivot rows and columns are rewritten below)
  hipLaunchKernelGGL(rk_update_kernel, dim3((unsigned)L.n_tiles_sym), dim3(256), 0, sn, Epk, dpad, Cpk, dpad, t.N, (int64_t)d.d1, d.d1, d.d1,
                     L.tiles_sym, (double*)nullptr);
  hipLaunchKernelGGL(lazy_fix_kernel, dim3(rb, LAZY_TM / FIX_SPB), dim3(256), 0, sn, L, t.N, d.d1, t.ctrl);
  // Z0 -= C0 ZT
  // (with two streams the kernel also leaves the sums of squares of every row's 64-column stretches: the row norms of the
  // score refresh then come from these 25 MB instead of another pass over Z0)
  hipLaunchKernelGGL(rk_update_kernel, dim3((unsigned)L.n_tiles_rect), dim3(256), 0, s, Cpk, dpad, Zpk, mpad, t.Z, (int64_t)d.m, d.d1, d.m,
                     L.tiles_rect, two ? L.rowsq : (double*)nullptr);
  hipLaunchKernelGGL(lazy_fix_z_kernel, dim3(mb, LAZY_TM / FIX_SPB), dim3(256), 0, s, L, t.Z, d.m, t.ctrl);
  if (two) {
    // The second stream goes on, once both matrices are final, with the first half of the score refresh (row norms from the
    // stretch sums, diagonal of N0); this one with the products of the picked rows with the new Z0.
    if ((err = hipEventRecord(side->fork, s)) != hipSuccess) return err;
    if ((err = hipStreamWaitEvent(sn, side->fork, 0)) != hipSuccess) return err;
    hipLaunchKernelGGL(norms_from_stretches_kernel, dim3((d.d1 + 255) / 256 + LAZY_TM), dim3(256), 0, sn, L, d.d1, d.m, 2 * ((d.m + 127) / 128),
                       (d.d1 + 255) / 256, t.N, t.Z, t.gram, t.dblk, t.ctrl);
    if ((err = hipEventRecord(side->join, sn)) != hipSuccess) return err;
    // The candidates of the next cycle, from the scores as the swaps left them (the refresh below changes them in the last
    // digits only, and the choice of candidates decides what is computed ahead, not any result): two sorts of one
    // workgroup each; this stream has the time, the second one's chain is the longer.
    err = launch_candidates(d, t, L, s, mode);
    if (err != hipSuccess) return err;
    if ((err = hipStreamWaitEvent(s, side->join, 0)) != hipSuccess) return err;
  }
  hipLaunchKernelGGL(lazy_reset_kernel, dim3(1), dim3(256), 0, s, L, t.ctrl);
  err = two ? launch_refresh_from_blocks(d, t, s) : launch_refresh_scores(d, t, s);
  if (err != hipSuccess) return err;
  err = launch_partials(d, t, L, s);
  if (err != hipSuccess) return err;
  return two ? hipGetLastError() : launch_candidates(d, t, L, s, mode);
}

// ------------------------------------------------------------------------------------------------
// Block removal: the t <= LAZY_BT rows that one iteration of the nested schedule prunes (Algorithm 1 with p-hat = t-hat:
// all of them scored at the state the iteration starts from) leave as ONE block pivot instead of t pivots in a row.
// With G the picks, b = N0[T, G] (tau x t), X = M^-1 b, the current block N_GG = N0[G, G] - b^T X and D = N_GG^-1:
//   Y = D Z_G (t x m), Z_G = Z0[G, :] - b^T ZT the current rows;       obj rises by -sum_a <Z_G[a], Y[a]>
//   every other row i: c_i = N[i, G] = N0[i, G] - C0[i, :] X,  Z_i -= c_i Y,  N_ii -= c_i D c_i^T
//   |Z_i|^2 changes by -2 c_i (Y Z_i^T) + c_i (Y Y^T) c_i^T,  Y Z_i^T = W_i - (ZT Y^T)^T C0[i, :]^T,
//   W_i = Z0_i Y^T = D (GbT[G, i] - X^T GbT[T, i])  from the products computed ahead
//   M^-1 grows by the block [[X D X^T, -X D], [-D X^T, D]],  ZT <- [ZT - X Y; Y].
// Four launches per iteration of t removals (prep, cols, gemv, update) instead of four per removal.
// ------------------------------------------------------------------------------------------------
constexpr int BT = LAZY_BT;

// n x n inverse (n <= BT) in shared memory by Gauss-Jordan without pivoting; every pivot must be negative (the block is
// minus a principal block of a positive definite inverse), else *bad is set.  All threads of the workgroup call it.
__device__ void blk_inverse(double* A, int n, int* bad) {
  __shared__ double col[BT], rowk[BT];
  const int tid = threadIdx.x;
  for (int k = 0; k < n; k++) {
    __syncthreads();
    double piv = A[k * n + k];
    if (!(piv < 0.0)) { if (tid == 0) *bad = 1; piv = -1.0; }
    const double dinv = 1.0 / piv;
    if (tid < n) { col[tid] = A[tid * n + k]; rowk[tid] = A[k * n + tid] * dinv; }
    __syncthreads();
    for (int idx = tid; idx < n * n; idx += blockDim.x) {
      const int i = idx / n, j = idx % n;
      double v;
      if (i == k) v = (j == k) ? dinv : rowk[j];
      else if (j == k) v = -col[i] * dinv;
      else v = A[idx] - col[i] * rowk[j];
      A[idx] = v;
    }
  }
  __syncthreads();
}

__global__ __launch_bounds__(256) void blk_prep_kernel(LazyPtrs L, const float* __restrict__ N0, int d1, int t,
                                                        const int32_t* __restrict__ pick, const int32_t* __restrict__ kept,
                                                        SearchCtrl* ctrl) {
  __shared__ double sb[LAZY_TM * BT], sX[LAZY_TM * BT], sD[BT * BT];
  __shared__ int sG[BT], s_bad, s_notpd;
  if (idle(ctrl)) return;
  const int tid = threadIdx.x, tau = tau_all(ctrl);      // every thread reads before thread 0 folds the increment in
  if (tid == 0) { s_bad = 0; s_notpd = 0; }
  __syncthreads();
  if (tid == 0) { ctrl->tau = tau; ctrl->tau_inc = 0; }
  if (tid < t) {
    const int g = pick[tid];
    sG[tid] = g;
    if (g < 0 || g >= d1 || !kept[g] || L.pos[g] >= 0 || L.cslot[g] < 0) s_bad = 1;
  }
  if (tid == 0 && tau + t > LAZY_TM) s_bad = 1;
  __syncthreads();
  if (s_bad) { if (tid == 0) ctrl->pause = 1; return; }
  for (int idx = tid; idx < tau * t; idx += 256) { const int r = idx / t, a = idx % t; sb[r * BT + a] = (double)L.C0R[(int64_t)sG[a] * LAZY_TM + r]; }
  __syncthreads();
  for (int idx = tid; idx < tau * t; idx += 256) {
    const int r = idx / t, a = idx % t;
    double v = 0;
    for (int q = 0; q < tau; q++) v += L.Minv[r * LAZY_TM + q] * sb[q * BT + a];
    sX[r * BT + a] = v;
  }
  __syncthreads();
  for (int idx = tid; idx < t * t; idx += 256) {
    const int a = idx / t, b = idx % t;
    double v = (double)nsym1(N0, d1, sG[a], sG[b]);
    for (int r = 0; r < tau; r++) v -= sb[r * BT + a] * sX[r * BT + b];
    sD[idx] = v;
  }
  blk_inverse(sD, t, &s_notpd);
  for (int idx = tid; idx < LAZY_TM * BT; idx += 256) {
    const int r = idx / BT, a = idx % BT;
    const bool in = (r < tau && a < t);
    L.bB[idx] = in ? sb[idx] : 0.0; L.bX[idx] = in ? sX[idx] : 0.0;
  }
  for (int idx = tid; idx < BT * BT; idx += 256) { const int a = idx / BT, b = idx % BT; L.bD[idx] = (a < t && b < t) ? sD[a * t + b] : 0.0; }
  if (tid < BT) L.bG[tid] = tid < t ? sG[tid] : -1;
  if (tid == 0 && s_notpd) ctrl->notpd = 1;
}

// current rows of the picks, Y = D Z_G, and per column block the partial sums of Y Y^T and <Z_G[a], Y[a]>
__global__ __launch_bounds__(256) void blk_cols_kernel(LazyPtrs L, const float* __restrict__ Z0, int m, int t,
                                                        const SearchCtrl* __restrict__ ctrl) {
  __shared__ double sb[LAZY_TM * BT], sD[BT * BT];
  __shared__ double zred[3][COLS_PER_BLOCK][BT];
  if (idle(ctrl)) return;
  const int tid = threadIdx.x, tau = ctrl->tau, cb = blockIdx.x;
  const int slice = tid >> 6, lc = tid & 63, col = cb * COLS_PER_BLOCK + lc;
  for (int idx = tid; idx < LAZY_TM * BT; idx += 256) sb[idx] = L.bB[idx];
  for (int idx = tid; idx < BT * BT; idx += 256) sD[idx] = L.bD[idx];
  __syncthreads();
  double acc[BT];
#pragma unroll
  for (int a = 0; a < BT; a++) acc[a] = 0.0;
  if (col < m)
    for (int r = slice; r < tau; r += 4) {
      const double zt = L.ZT[(int64_t)r * m + col];
#pragma unroll
      for (int a = 0; a < BT; a++) acc[a] += sb[r * BT + a] * zt;
    }
  if (slice > 0) {
#pragma unroll
    for (int a = 0; a < BT; a++) zred[slice - 1][lc][a] = acc[a];
  }
  __syncthreads();
  if (slice != 0) return;
  double zg[BT], y[BT];
#pragma unroll
  for (int a = 0; a < BT; a++) {
    zg[a] = 0.0;
    if (a < t && col < m) zg[a] = (double)Z0[(int64_t)L.bG[a] * m + col] - (acc[a] + zred[0][lc][a] + zred[1][lc][a] + zred[2][lc][a]);
  }
#pragma unroll
  for (int a = 0; a < BT; a++) {
    double v = 0;
#pragma unroll
    for (int b = 0; b < BT; b++) v += sD[a * BT + b] * zg[b];
    y[a] = v;
    if (a < t && col < m) L.bY[(int64_t)a * m + col] = v;
  }
  double* part = L.bpart + (int64_t)cb * (BT * BT + BT);
  for (int a = 0; a < t; a++) {
    for (int b = 0; b <= a; b++) { const double v = wsum(y[a] * y[b]); if (lc == 0) part[a * BT + b] = v; }
    const double v = wsum(zg[a] * y[a]);
    if (lc == 0) part[BT * BT + a] = v;
  }
}

// U = ZT Y^T: workgroup (rg, slab) takes four pending pivots and a quarter of the columns and leaves its part in
// bU[slab] (the reader adds the four up); the last workgroup adds up the column blocks' sums and books the move
constexpr int BU_SLABS = 4;
__global__ __launch_bounds__(256) void blk_gemv_kernel(LazyPtrs L, int m, int t, int col_blocks, SearchCtrl* ctrl,
                                                        int32_t* __restrict__ trace_out) {
  __shared__ double red[4][4 * BT];
  if (idle(ctrl)) return;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, tau = ctrl->tau;
  if ((int)blockIdx.x < LAZY_TM) {
    const int r0 = ((int)blockIdx.x / BU_SLABS) * 4, slab = (int)blockIdx.x % BU_SLABS;
    const int cs = (m + BU_SLABS - 1) / BU_SLABS, c0 = slab * cs, c1 = min(m, c0 + cs);
    double acc[4][BT];
#pragma unroll
    for (int e = 0; e < 4; e++)
#pragma unroll
      for (int a = 0; a < BT; a++) acc[e][a] = 0.0;
    if (r0 < tau) {
      for (int c = c0 + tid; c < c1; c += 256) {
        double z[4], y[BT];
#pragma unroll
        for (int e = 0; e < 4; e++) z[e] = (r0 + e < tau) ? L.ZT[(int64_t)(r0 + e) * m + c] : 0.0;
#pragma unroll
        for (int a = 0; a < BT; a++) y[a] = (a < t) ? L.bY[(int64_t)a * m + c] : 0.0;
#pragma unroll
        for (int e = 0; e < 4; e++)
#pragma unroll
          for (int a = 0; a < BT; a++) acc[e][a] += z[e] * y[a];
      }
    }
#pragma unroll
    for (int e = 0; e < 4; e++)
#pragma unroll
      for (int a = 0; a < BT; a++) { const double v = wsum(acc[e][a]); if (lane == 0) red[wave][e * BT + a] = v; }
    __syncthreads();
    if (tid < 4 * BT) L.bU[(int64_t)slab * LAZY_TM * BT + r0 * BT + tid] = red[0][tid] + red[1][tid] + red[2][tid] + red[3][tid];
    return;
  }
  // sums in a fixed order: thread (a, b) walks the column blocks
  for (int idx = tid; idx < BT * BT + BT; idx += 256) {
    double v = 0;
    int cb = 0;
    for (; cb + 8 <= col_blocks; cb += 8) {     // eight loads in flight; the order of the sum stays fixed
      double pv[8];
#pragma unroll
      for (int u = 0; u < 8; u++) pv[u] = L.bpart[(int64_t)(cb + u) * (BT * BT + BT) + idx];
#pragma unroll
      for (int u = 0; u < 8; u++) v += pv[u];
    }
    for (; cb < col_blocks; cb++) v += L.bpart[(int64_t)cb * (BT * BT + BT) + idx];
    if (idx < BT * BT) { const int a = idx / BT, b = idx % BT; if (b <= a && a < t) { L.bYY[a * BT + b] = v; L.bYY[b * BT + a] = v; } }
    else if (idx - BT * BT < t) L.bdl[idx - BT * BT] = v;
  }
  __syncthreads();
  if (tid == 0) {
    double dsum = 0;
    for (int a = 0; a < t; a++) dsum += L.bdl[a];
    const int it = ctrl->iters;
    ctrl->obj = ctrl->obj - dsum;            // D is negative definite: -sum <Z_G[a], Y[a]> >= 0
    ctrl->iters = it + t; ctrl->accepted += t; ctrl->tau_inc = t;
    if (trace_out) for (int a = 0; a < t; a++) trace_out[it + a] = L.bG[a];
  }
}

__global__ __launch_bounds__(256) void blk_update_kernel(LazyPtrs L, const float* __restrict__ N0, int d1, int m, int t, int row_blocks,
                                                          int row_wgs, int col_blocks, SearchCtrl* ctrl, int32_t* __restrict__ kept,
                                                          double* __restrict__ rho, double* __restrict__ diag,
                                                          double* __restrict__ score) {
  __shared__ double sX[LAZY_TM * BT], sU[LAZY_TM * BT], sD[BT * BT], sYY[BT * BT];
  __shared__ int sts[LAZY_TM], sG[BT], sSlot[BT];
  __shared__ double w_mn1[4], w_mn2[4], w_mx1[4], w_mx2[4];
  __shared__ int w_imn[4], w_imx[4];
  if (idle(ctrl)) return;
  const int tid = threadIdx.x, tau = ctrl->tau, b = blockIdx.x;
  if (b < row_wgs) {
    // sX, sU transposed to [a][r]: the eight lanes of a row read eight consecutive r
    for (int idx = tid; idx < LAZY_TM * BT; idx += 256) {
      const int r = idx / BT, a = idx % BT;
      double u = 0;
#pragma unroll
      for (int sl = 0; sl < BU_SLABS; sl++) u += L.bU[(int64_t)sl * LAZY_TM * BT + idx];
      sX[a * LAZY_TM + r] = L.bX[idx]; sU[a * LAZY_TM + r] = u;
    }
    for (int idx = tid; idx < BT * BT; idx += 256) { sD[idx] = L.bD[idx]; sYY[idx] = L.bYY[idx]; }
    for (int s = tid; s < LAZY_TM; s += 256) sts[s] = (s < tau) ? L.tslot[s] : 0;
    if (tid < BT) { const int g = L.bG[tid]; sG[tid] = g; sSlot[tid] = (tid < t) ? L.cslot[g] : 0; }
    __syncthreads();
    // a workgroup walks blocks of 32 rows (one selection record each), so the tables above are loaded once for several
    for (int rbk = b; rbk < row_blocks; rbk += row_wgs) {
    const int row = rbk * ROWS_PER_BLOCK + (tid >> 3), l8 = tid & 7;
    double mn1 = INFINITY, mx1 = -INFINITY;
    int imn = -1, imx = -1;
    if (row < d1) {
      double dx[BT], du[BT], dw[BT];
#pragma unroll
      for (int a = 0; a < BT; a++) { dx[a] = 0.0; du[a] = 0.0; dw[a] = 0.0; }
      const float* crow = L.C0R + (int64_t)row * LAZY_TM;
      for (int r = l8; r < tau; r += 8) {
        const double c = (double)crow[r];
        const double gb = L.GbT[(int64_t)sts[r] * d1 + row];
#pragma unroll
        for (int a = 0; a < BT; a++) {
          const double x = sX[a * LAZY_TM + r];
          dx[a] += c * x; du[a] += c * sU[a * LAZY_TM + r]; dw[a] += gb * x;
        }
      }
#pragma unroll
      for (int a = 0; a < BT; a++) {
        dx[a] = sum8(dx[a]); du[a] = sum8(du[a]); dw[a] = sum8(dw[a]);
      }
      // the base entries N0[row, G] (new columns of C0) and the products GbT[G, row]: lane l8 fetches a = l8 and l8 + 8
      static_assert(BT == 16, "two picks per lane");
      float n_lo = 0.f, n_hi = 0.f;
      double g_lo = 0.0, g_hi = 0.0;
      if (l8 < t) { n_lo = nsym1(N0, d1, row, sG[l8]); g_lo = L.GbT[(int64_t)sSlot[l8] * d1 + row]; L.C0R[(int64_t)row * LAZY_TM + tau + l8] = n_lo; }
      if (l8 + 8 < t) { n_hi = nsym1(N0, d1, row, sG[l8 + 8]); g_hi = L.GbT[(int64_t)sSlot[l8 + 8] * d1 + row]; L.C0R[(int64_t)row * LAZY_TM + tau + l8 + 8] = n_hi; }
      double nrow[BT], grow[BT];
      const int lane0 = (tid & 63) & ~7;
#pragma unroll
      for (int a = 0; a < BT; a++) {
        nrow[a] = (double)__shfl(a < 8 ? n_lo : n_hi, lane0 + (a & 7), 64);
        grow[a] = __shfl(a < 8 ? g_lo : g_hi, lane0 + (a & 7), 64);
      }
      if (l8 == 0) {
        int mine = -1;
        for (int a = 0; a < t; a++) if (sG[a] == row) mine = a;
        const int ps = L.pos[row];
        double r, dn;
        int kp;
        if (mine >= 0) {
          r = sYY[mine * BT + mine]; dn = -sD[mine * BT + mine]; kp = 0;
          L.pos[row] = tau + mine; L.Tidx[tau + mine] = row; L.Jsg[tau + mine] = -1.f; L.tslot[tau + mine] = sSlot[mine];
        } else {
          double cg[BT], zy[BT];
          if (ps >= 0) {
            const double sg = (double)L.Jsg[ps];
#pragma unroll
            for (int a = 0; a < BT; a++) { cg[a] = sg * sX[a * LAZY_TM + ps]; zy[a] = sg * sU[a * LAZY_TM + ps]; }
          } else {
            double wt[BT];
#pragma unroll
            for (int a = 0; a < BT; a++) wt[a] = (a < t) ? grow[a] - dw[a] : 0.0;
#pragma unroll
            for (int a = 0; a < BT; a++) {
              double w = 0;
#pragma unroll
              for (int bb = 0; bb < BT; bb++) w += sD[a * BT + bb] * wt[bb];
              cg[a] = nrow[a] - dx[a];
              zy[a] = w - du[a];
            }
          }
          double lin = 0, quadY = 0, quadD = 0;
#pragma unroll
          for (int a = 0; a < BT; a++) {
            lin += cg[a] * zy[a];
            double sy = 0, sd = 0;
#pragma unroll
            for (int bb = 0; bb < BT; bb++) { sy += sYY[a * BT + bb] * cg[bb]; sd += sD[a * BT + bb] * cg[bb]; }
            quadY += cg[a] * sy; quadD += cg[a] * sd;
          }
          r = rho[row] - 2.0 * lin + quadY;
          if (r < 0.0) r = 0.0;
          dn = diag[row] - quadD;
          kp = kept[row];
        }
        rho[row] = r; diag[row] = dn; kept[row] = kp;
        const double sc = r / fabs(dn);
        score[row] = sc;
        if (kp) { mn1 = sc; imn = row; } else { mx1 = sc; imx = row; }
      }
    }
    double mn2 = INFINITY, mx2 = -INFINITY;
    wave_merge(mn1, mn2, imn, mx1, mx2, imx);          // lanes that lead no row hold the neutral record
    if ((tid & 63) == 63) { const int w = tid >> 6; w_mn1[w] = mn1; w_mn2[w] = mn2; w_imn[w] = imn; w_mx1[w] = mx1; w_mx2[w] = mx2; w_imx[w] = imx; }
    __syncthreads();
    if (tid == 0) {
      mn1 = w_mn1[0]; mn2 = w_mn2[0]; imn = w_imn[0]; mx1 = w_mx1[0]; mx2 = w_mx2[0]; imx = w_imx[0];
      for (int w = 1; w < 4; w++) { merge_min(mn1, mn2, imn, w_mn1[w], w_mn2[w], w_imn[w]); merge_max(mx1, mx2, imx, w_mx1[w], w_mx2[w], w_imx[w]); }
      SelRec rec; rec.mn1 = mn1; rec.mn2 = mn2; rec.mx1 = mx1; rec.mx2 = mx2; rec.imn = imn; rec.imx = imx;
      L.sel[rbk] = rec;
    }
    __syncthreads();
    }
  } else if (b < row_wgs + col_blocks) {
    const int cb = b - row_wgs, slice = tid >> 6, col = cb * COLS_PER_BLOCK + (tid & 63);
    for (int idx = tid; idx < LAZY_TM * BT; idx += 256) sX[idx] = L.bX[idx];
    __syncthreads();
    if (col < m) {
      double y[BT];
#pragma unroll
      for (int a = 0; a < BT; a++) y[a] = (a < t) ? L.bY[(int64_t)a * m + col] : 0.0;
      for (int r = slice; r < tau; r += 4) {
        double v = 0;
#pragma unroll
        for (int a = 0; a < BT; a++) v += sX[r * BT + a] * y[a];
        L.ZT[(int64_t)r * m + col] -= v;
      }
      for (int a = slice; a < t; a += 4) L.ZT[(int64_t)(tau + a) * m + col] = y[a];
    }
  } else {
    const int mb = b - row_wgs - col_blocks, nmb = gridDim.x - row_wgs - col_blocks;
    double* Mi = L.Minv;
    for (int idx = mb * 256 + tid; idx < tau * tau; idx += nmb * 256) {
      const int r = idx / tau, s = idx % tau;
      double v = 0;
      for (int a = 0; a < t; a++) {
        double xd = 0;
        for (int bb = 0; bb < t; bb++) xd += L.bX[r * BT + bb] * L.bD[bb * BT + a];
        v += xd * L.bX[s * BT + a];
      }
      Mi[r * LAZY_TM + s] += v;
    }
    if (mb == 0) {
      for (int idx = tid; idx < tau * t; idx += 256) {
        const int r = idx / t, a = idx % t;
        double v = 0;
        for (int bb = 0; bb < t; bb++) v -= L.bX[r * BT + bb] * L.bD[bb * BT + a];
        Mi[r * LAZY_TM + tau + a] = v; Mi[(tau + a) * LAZY_TM + r] = v;
      }
      for (int idx = tid; idx < t * t; idx += 256) { const int a = idx / t, bb = idx % t; Mi[(tau + a) * LAZY_TM + tau + bb] = L.bD[a * BT + bb]; }
    }
  }
}

hipError_t launch_lazy_block_remove(const TabDims& d, const TabPtrs& t, const LazyPtrs& L, int take, const int32_t* pick,
                                    hipStream_t s) {
  if (take < 1 || take > BT) return hipErrorInvalidValue;
  const int rb = (d.d1 + ROWS_PER_BLOCK - 1) / ROWS_PER_BLOCK, cb = (d.m + COLS_PER_BLOCK - 1) / COLS_PER_BLOCK;
  hipLaunchKernelGGL(blk_prep_kernel, dim3(1), dim3(256), 0, s, L, t.N, d.d1, take, pick, t.kept, t.ctrl);
  hipLaunchKernelGGL(blk_cols_kernel, dim3(cb), dim3(256), 0, s, L, t.Z, d.m, take, t.ctrl);
  hipLaunchKernelGGL(blk_gemv_kernel, dim3(LAZY_TM + 1), dim3(256), 0, s, L, d.m, take, cb, t.ctrl, t.trace_out);
  const int row_wgs = std::min(rb, 256);
  hipLaunchKernelGGL(blk_update_kernel, dim3(row_wgs + cb + 16), dim3(256), 0, s, L, t.N, d.d1, d.m, take, rb, row_wgs, cb, t.ctrl,
                     t.kept, t.gram, t.dblk, t.score);
  return hipGetLastError();
}

hipError_t launch_lazy_init(const TabDims& d, const TabPtrs& t, const LazyPtrs& L, hipStream_t s, int mode) {
  hipError_t e = hipMemsetAsync(L.pos, 0xFF, (size_t)d.d1 * 4, s);
  if (e != hipSuccess) return e;
  e = hipMemsetAsync(L.Minv, 0, (size_t)LAZY_TM * LAZY_TM * 8, s);
  if (e != hipSuccess) return e;
  e = hipMemsetAsync(L.C0R, 0, (size_t)d.d1 * LAZY_TM * 4, s);
  if (e != hipSuccess) return e;
  e = launch_partials(d, t, L, s);
  if (e != hipSuccess) return e;
  return launch_candidates(d, t, L, s, mode);
}

}  // namespace osscar
