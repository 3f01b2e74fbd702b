// Internal declarations shared by the translation units of libosscar (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>
#include <vector>

namespace osscar {

// message of the last failure of a call that takes no context, per host thread (returned by osscar_last_error(NULL))
void set_contextless_error(const char* msg);

// ----------------------------------------------------------------------------------------------
// gemm.hip : C = alpha * A * B + beta * Cin (+ diag_add on the diagonal), all row-major float32
// storage, products accumulated in float64 on the matrix cores (v_mfma_f64_16x16x4_f64).
// ----------------------------------------------------------------------------------------------
struct GemmArgs {
  int M, N, K;
  const float* A; int64_t lda;   // M x K
  const float* B; int64_t ldb;   // K x N
  const float* Cin; int64_t ldcin;  // M x N or nullptr (treated as zero)
  void* C; int64_t ldc;          // M x N, float or double
  double alpha, beta, diag_add;
  int c_is_f64;                  // output (and Cin) element type: 0 float, 1 double
  int lower_only;                // 1: compute only tiles that touch the lower triangle (row >= col)
  int trans_b;                   // 1: B is given as N x K row-major (C = alpha * A * B^T + ...)
  int acc_f32;                   // 1: accumulate in float32 (v_mfma_f32_32x32x2_f32); float32 output only
  // hints for the int8-digit product only (i8gemm.hip; any other kernel ignores them): A (B) is square with a diagonal far
  // above the rest of its rows (columns), to be kept out of the fixed-point digits and added in float64
  int i8_diag_a, i8_diag_b;
  // and a levelling of the contraction index: A is used as A 2^(ksign kexp[k]), B as 2^(-ksign kexp[k]) B (nullptr: none)
  const int* i8_kexp; int i8_ksign;
};
hipError_t launch_gemm_f64acc(const GemmArgs& a, hipStream_t s);
// diagnostic log of the launches above: enable (1) / disable and clear (0); read = rows of {M, N, K, kind, ms} with
// kind = 1 float32 accumulation | 2 float64 output | 4 lower triangle only | 8 B transposed; returns the number of rows
// kind also carries 16 = the int8-digit product of i8gemm.hip
void gemm_log_enable(int on);
int gemm_log_read(double* out, int capacity);
void gemm_log_open(int M, int N, int K, int kind, hipStream_t s, int* slot);
void gemm_log_close(int slot, hipStream_t s);

// ----------------------------------------------------------------------------------------------
// i8gemm.hip : the same product C = alpha A B + beta Cin (+ diag_add on the diagonal; lower_only) for float32 A, B, Cin, C
// with the accuracy of float64 accumulation, computed on the int8 matrix cores from I8_S seven-bit digits per operand
// ----------------------------------------------------------------------------------------------
constexpr int I8_S = 5;
size_t i8_pack_bytes(int64_t rows, int64_t K);          // packed size of an operand with `rows` rows (A) or columns (B)
bool i8_gemm_fits(const GemmArgs& g);
// kexp[k] = round(log2 sqrt(D_kk)) from the diagonal of a Gram block (device, n ints)
hipError_t launch_i8_kexp(const float* D, int n, int64_t ld, int* kexp, hipStream_t s);
// packA / packB: scratch for the two packed operands (capacities in bytes), mx: M + N words for the scaling exponents
hipError_t launch_i8_gemm(const GemmArgs& g, void* packA, size_t capA, void* packB, size_t capB, unsigned* mx, size_t mx_entries,
                          hipStream_t s);

// ----------------------------------------------------------------------------------------------
// gram.hip : H64 (+)= Xc^T Xc on the lower-triangle tiles (bf16 X, d1 % 8 == 0, ldx % 8 == 0, 16-byte aligned)
// ----------------------------------------------------------------------------------------------
// Repacks `pack_rows`-token chunks of Xc into MFMA operand order in pack_buf (pack_rows * 128*ceil(d1/128) * 2 bytes)
// and accumulates them into H64.
// tiles: the tile schedule on the device (gram_tile_list_host for the symmetric product, rect_tile_list_host for a
// rectangular one), uploaded once by the caller; no call here waits for the stream.
// Patch geometry of a convolutional layer: row (b*Hout + oy)*Wout + ox, column (c*kh + dy)*kw + dx of the patch matrix is
// F[b][c][oy*stride + dy - pad][ox*stride + dx - pad] (zero outside the map).
struct ConvSpec { int B, C, Hin, Win, kh, kw, stride, pad, Hout, Wout; };
hipError_t launch_gram_packed(const void* Xc, int64_t n_c, int64_t ldx, int d1, double* H64, const int2* tiles,
                              size_t tile_entries, void* pack_buf, int64_t pack_rows, hipStream_t s,
                              const void* Yc = nullptr, int64_t ldy = 0, int m = 0, double* G64 = nullptr,
                              const int2* tiles_y = nullptr, size_t tile_y_entries = 0, void* pack_buf_y = nullptr,
                              const ConvSpec* conv = nullptr, hipEvent_t* ev = nullptr, int ev_pairs = 0, int* ev_used = nullptr);
// ev (optional, 2 * ev_pairs events): recorded before and after each launch of the symmetric product kernel (one per
// pack_rows chunk), *ev_used = pairs recorded
// host-side schedules: lower-triangle tiles of a d1 x d1 result / all tiles of a d1 x m result (128 x 128 tiles)
void gram_tile_list_host(int d1, std::vector<int2>& out);
void rect_tile_list_host(int d1, int m, std::vector<int2>& out);
// conv (optional): Xc is a feature map (NCHW, bf16) and the rows are its patches
// Xt[c][r - r0] = patch matrix entry (r, c) as float32 for rows r0 .. r0 + nr (generic path of convolutional layers)
hipError_t launch_im2col_transpose(const void* F, int is_bf16, const ConvSpec& cs, int64_t r0, int64_t nr, int d1, float* Xt,
                                   int64_t ldxt, hipStream_t s);
// Yc (optional, bf16 n_c x m): also G64 (d1 x m, float64) += Xc^T Yc, with its own tile list (>= 8 * (ceil(d1/128) *
// ceil(m/128) / 8 + 64) entries) and pack buffer (pack_rows * 128*ceil(m/128) * 2 bytes)
int gram_tile_schedule(int tiles_per_side, int32_t* out, int capacity);   // host only: the tile order of the SYRK kernel
// G64 (zeroed by the caller) += H W for bf16 W through three bf16 pieces of the float32 H (see gram.hip)
hipError_t launch_hw_split(const float* H, int d1, const void* W, int64_t ldw, int m, double* G64, const int2* tiles,
                           size_t tile_entries, void* pack_h, void* pack_w, int64_t pack_rows, hipStream_t s);
// Products of float32 matrices on the bf16 matrix cores through three bf16 pieces per operand (see gram.hip).  Operands are
// row-major with the contraction along their rows (C = A^T B).  pack: split_pack_bytes(K, cols) bytes, 256-byte aligned.
size_t split_pack_bytes(int64_t K, int64_t cols);
hipError_t launch_pack_pieces(const float* A, int64_t lda, int64_t K, int cols, void* pack, hipStream_t s);   // cols % 8 == 0, lda % 4 == 0
// acc (M x N float64, dense; cleared here) = A^T B.  tiles: rect_tile_list_host(M, N), or gram_tile_list_host(M) for the lower
// triangle of a square result (ntiles = number of real tiles in the list, for the split of the contraction over workgroups)
hipError_t launch_split_product(const void* packA, int M, const void* packB, int N, int64_t K, int nprod, double* acc,
                                const int2* tiles, size_t tile_entries, int ntiles, hipStream_t s);
// C = float(beta * Cin + alpha * acc)
hipError_t launch_split_epilogue(const double* acc, int M, int N, const float* Cin, int64_t ldcin, float* C, int64_t ldc, double alpha,
                                 double beta, hipStream_t s);
hipError_t launch_sumsq(const void* A, int is_bf16, int64_t rows, int64_t cols, int64_t ld, double* acc, double* partial,
                        hipStream_t s);   // partial: 1024 doubles
hipError_t launch_finalize_G(const double* G64, const float* Wf, const double* lambda_dev, float* G, int64_t n, hipStream_t s);
hipError_t launch_transpose_to_f32(const void* X, int is_bf16, int64_t rows, int64_t cols, int64_t ldx, float* Xt,
                                   int64_t ldxt, hipStream_t s);
// H = float(mirror(H64) + lam*I); also usable with lam = 0
hipError_t launch_finalize_H(const double* H64, float* H, int d1, const double* lam_dev, hipStream_t s);
// out[0] = sum_i H64[i][i]
hipError_t launch_trace64(const double* H64, int d1, double* out, hipStream_t s);
hipError_t launch_convert_to_f32(const void* src, int is_bf16, int64_t rows, int64_t cols, int64_t lds, float* dst,
                                 hipStream_t s);
// norms2[j] = sum over group j of W^2 (float64); c0 = sum W*G
hipError_t launch_group_norms(const float* Wf, int p, int q, int m, double* norms2, hipStream_t s);
hipError_t launch_dot64(const float* a, const float* b, int64_t n, double* out, double* partial, hipStream_t s);
// out = sum_i <a[rows[i], :], b[i, :]>, a with leading dimension m, b dense nrows x m (partial: 1024 doubles)
hipError_t launch_dot64_rows(const float* a, const int32_t* rows, const float* b, int nrows, int m, double* out, double* partial,
                             hipStream_t s);

// ----------------------------------------------------------------------------------------------
// tableau.hip : the swept tableau N (d1 x d1, lower triangle valid) and Z (d1 x m)
//   N_KK = -P, N_{K,Kc} = V, N_{Kc,Kc} = S (Schur complement), Z_K = B, Z_Kc = R.
// ----------------------------------------------------------------------------------------------
struct SearchCtrl {          // lives in device memory
  int32_t done;              // set when a swap is rejected (or nothing left to swap)
  int32_t iters;             // iterations run
  int32_t accepted;          // swaps applied
  int32_t notpd;             // a pivot block was not definite
  int32_t g_out, g_in;       // current selection (group ids), -1 if none
  int32_t pause;             // delayed-update search: the host must flush before the search can go on
  int32_t tau;               // delayed-update search: number of pending pivots that every kernel of an iteration works with
  int32_t tau_inc;           // pivots that the iteration just applied adds to it: folded into tau by the next one-workgroup
  int32_t misses;            // kernel (prep), so that no kernel changes tau while its own workgroups read it.
                             // misses: delayed-update search, pivots so far whose products with Z0 had not been computed ahead
  double obj;                // tracked objective
  double rel_tol;
  double delta;              // exact change of the current pair
  double gap_rem, gap_add;
};

struct TabDims { int d1, m, p, q; };

hipError_t launch_gather(const float* src, int64_t lds, const int32_t* rows, int nrows, const int32_t* cols, int ncols,
                         float* dst, int64_t ldd, hipStream_t s);
// dst[rows[i]][cols[j]] = sign * src[i][j], only where rows[i] >= cols[j] if lower_only
hipError_t launch_scatter(const float* src, int64_t lds, const int32_t* rows, int nrows, const int32_t* cols, int ncols,
                          float* dst, int64_t ldd, float sign, int lower_only, hipStream_t s);
hipError_t launch_mirror_lower(float* A, int n, int64_t lda, hipStream_t s);
hipError_t launch_absmax(const float* A, int64_t n, double* out, hipStream_t s);

constexpr int INV_NB = 128;   // pivot block width of the sweep inverse
// In-place inverse of the symmetric positive definite n x n matrix A (full storage on entry and exit)
// by block sweeps of width INV_NB; panel/work buffers are caller-provided: panel (n*INV_NB), panelD (2*n*INV_NB),
// small (INV_NB*INV_NB doubles).  notpd_flag (device int) is set if a pivot block is not definite.
// The same with the working matrix in float64 (A64: n x n, panels: 5 n INV_NB float64): P = H^-1 rounded to float32 once.
// side (optional): a second stream with two events, on which the bulk of each panel's update runs beside the next panel's
// small kernels; every launch is joined back into s before the call returns.
struct SideStream;
hipError_t spd_inverse_f64(const float* H, int64_t ldh, int n, float* P, double* A64, double* panels, double* small,
                           int32_t* notpd_flag, hipStream_t s, const SideStream* side = nullptr);
hipError_t spd_inverse_inplace(float* A, int n, float* panel, float* panelD, double* small, int32_t* notpd_flag,
                               hipStream_t s);

struct TabPtrs {
  float* N; float* Z;              // tableau
  int32_t* kept;                   // p flags: 1 kept, 0 candidate
  double* score;                   // p scores: removal cost (kept) / addition gain (candidate)
  double* gram;                    // p * q*q : Z_g Z_g^T per group (float64)
  double* dblk;                    // p * q*q : float64 copy of the diagonal blocks N_gg
  float* C1; float* C2;            // d1 x q panels
  float* C1D; float* C2D;          // d1 x q panels times D
  float* rZ1; float* rZ2;          // q x m
  double* small;                   // scratch for q x q algebra (>= 16*q*q doubles)
  double* dpart;                   // ceil(m / 16) partial sums of the exact change of a pair (column blocks, fixed order)
  double* cross; double* xgram; double* xdblk; double* xscore;   // exact entering rule: d1*q, p*q*q, p*q*q, p
  SearchCtrl* ctrl;
  int32_t* trace_out; int32_t* trace_in; float* trace_gap; double* trace_obj;
};

hipError_t launch_refresh_scores(const TabDims& d, const TabPtrs& t, hipStream_t s);
hipError_t launch_refresh_blocks(const TabDims& d, const TabPtrs& t, hipStream_t s);        // first half: Gram and diagonal blocks
hipError_t launch_refresh_from_blocks(const TabDims& d, const TabPtrs& t, hipStream_t s);   // second half: the scores from them   // gram, dblk, score from N, Z
// ev (optional): three events recorded before the bulk update of N, after it, and after the update of Z.
// single (optional, device): removal of the one group *single instead of a swap (Case 1 alone; no selection kernel).
// exact_in: the entering group is the argmax of the exact gain of the pair with the selected leaving group.
hipError_t launch_search_iteration(const TabDims& d, const TabPtrs& t, int forced_out, int forced_in, int always_accept,
                                   hipStream_t s, hipEvent_t* ev = nullptr, const int32_t* single = nullptr, int exact_in = 0);
// pick[0..take) = the kept groups of smallest removal cost (ascending), *gap = relative gap to the next one; take <= 64
// side 1: the groups outside the kept set with the largest addition gain (descending) instead
hipError_t launch_greedy_pick(const TabDims& d, const TabPtrs& t, int take, int32_t* pick, float* gap, hipStream_t s,
                              int side = 0);
hipError_t launch_select(const TabDims& d, const TabPtrs& t, int forced_out, int forced_in, hipStream_t s);

// ----------------------------------------------------------------------------------------------
// lazy.hip : delayed-update search for q = 1
// ----------------------------------------------------------------------------------------------
constexpr int LAZY_TM = 128;     // capacity of the pending pivot set (two per swap)
constexpr int LAZY_NC = 256;     // rows of Z0 whose products with all of Z0 are computed ahead, after every flush
constexpr int LAZY_NS = 64;      // spare slots for pivots that were not among them
constexpr int LAZY_NPICK_OUT = 88;  // swap search: kept rows picked by cost of removal ...
constexpr int LAZY_NPICK_IN = 72;   // ... and rows outside the kept set picked by gain; together a multiple of 32
constexpr int LAZY_BT = 16;      // rows that one block removal of the nested schedule takes at most
struct SelRec { double mn1, mn2, mx1, mx2; int32_t imn, imx; };   // best / second-best scores of a block of rows
struct LazyPtrs {
  int32_t* pos;     // d1: position in the pending set or -1
  int32_t* Tidx;    // LAZY_TM pivot indices
  float* Jsg;       // LAZY_TM: -1 for pivots that left the kept set, +1 for pivots that entered
  float* C0R;       // d1 x LAZY_TM row-major: base columns N0[:, T_s]
  double* Minv;     // LAZY_TM x LAZY_TM: inverse of N0[T, T]
  float* Minv32;    // float copy for the flush
  double* ZT;       // LAZY_TM x m: Minv * Z0[T, :]
  float* ZT32;      // LAZY_TM x m (flush)
  float* E;         // d1 x LAZY_TM: C0 * Minv (flush)
  double* xg; double* xj; double* u1; double* u2;   // LAZY_TM
  double* cg; double* cj; double* w1; double* w2;   // d1
  double* y1; double* y2; float* y1f; float* y2f;   // m
  double* part;     // ceil(m/64) * 5 partial sums
  double* ls;       // 16 scalars
  SelRec* sel;      // ceil(d1/32) per-block score records
  // products of Z0 with the rows of Z0 that are likely to become pivots before the next flush
  double* GbT;      // (LAZY_NC + LAZY_NS) x d1: row s = Z0 Z0[cand[s], :]^T
  double* rowsq;    // 2 ceil(m / 128) x d1: sums of squares of every row's 64-column stretches, left by Z0's update in the flush
  float* Zc;        // LAZY_NC x m: the gathered rows (shapes that take the general matrix-product kernel)
  // flush: E, C0 and ZT cut into three bf16 pieces in matrix-core operand order (768 bytes per padded row / column), and the
  // tile schedules of the two updates (the Gram kernel's: lower triangle of d1 x d1, all of d1 x m), uploaded at create
  void* Epk; void* Cpk; void* Zpk;
  const int2* tiles_sym; size_t n_tiles_sym; const int2* tiles_rect; size_t n_tiles_rect;
  void* ZcP;        // LAZY_NC x 32*ceil(m/32) x 3 bf16: the candidate rows cut into three bf16 pieces, in matrix-core operand order
  int32_t* cslot;   // d1: slot of a row in GbT or -1
  int32_t* cand;    // LAZY_NC + LAZY_NS: row held by a slot or -1
  int32_t* tslot;   // LAZY_TM: slot of each pending pivot
  int32_t* misc;    // [0] spare slots in use, [1] miss mask of the current pair (1: g, 2: j), [2] slot of g, [3] slot of j
  double* lkey; int32_t* lidx;   // 2 x 64 x 32: per-block winners of the candidate selection
  // block removal (nested schedule): b = N0[T, G], X = M^-1 b (LAZY_TM x LAZY_BT each), U = ZT Y^T (four partial sums of that
  // shape, one per quarter of the columns), D, Y Y^T (LAZY_BT^2),
  // Y (LAZY_BT x m), per-column-block partial sums, the changes of the objective, the picks
  double* bB; double* bX; double* bU; double* bD; double* bYY; double* bY; double* bpart; double* bdl; int32_t* bG;
};
// mode: which rows get their products with Z0 computed ahead: 0 = LAZY_NC/2 cheapest removals + LAZY_NC/2 largest gains,
// 1 = LAZY_NC cheapest removals (removal-only loops), 2 = none (every pivot then costs a pass over Z0)
hipError_t launch_lazy_init(const TabDims& d, const TabPtrs& t, const LazyPtrs& L, hipStream_t s, int mode = 0);
// ev (optional): events recorded before and after the pass over Z0, and at the end of the iteration
// single (optional, device): removal of the one row *single instead of a swap; adds one pending pivot instead of two
hipError_t launch_lazy_iteration(const TabDims& d, const TabPtrs& t, const LazyPtrs& L, int always_accept, hipStream_t s,
                                 hipEvent_t* ev = nullptr, const int32_t* single = nullptr, int forced_out = -1,
                                 int forced_in = -1);
// A second stream and two events: the flush runs its update of N0 there, beside the candidate selection and the look-ahead
// product on the main stream (they touch disjoint data), and joins before the scores are refreshed.
// The `take` <= LAZY_BT rows in pick (device) leave the kept set as one block pivot (nested schedule, q = 1); does nothing
// but set ctrl->pause if a pick is pending, is not among the rows whose products were computed ahead, or the pending set
// has no room for all of them.
hipError_t launch_lazy_block_remove(const TabDims& d, const TabPtrs& t, const LazyPtrs& L, int take, const int32_t* pick,
                                    hipStream_t s);

struct SideStream { hipStream_t stream = nullptr; hipEvent_t fork = nullptr, join = nullptr; };
// side == nullptr (or no stream in it): everything in order on s
hipError_t launch_lazy_flush(const TabDims& d, const TabPtrs& t, const LazyPtrs& L, hipStream_t s, int mode = 0,
                             const SideStream* side = nullptr);

hipError_t launch_scatter_rows(const float* src, int64_t lds, const int32_t* rows, int nrows, int ncols, void* dst,
                               int64_t ldd, int dst_is_bf16, hipStream_t s);
hipError_t launch_fill_rows_zero(void* dst, int64_t ldd, int nrows_total, int ncols, int dst_is_bf16, hipStream_t s);

}  // namespace osscar
