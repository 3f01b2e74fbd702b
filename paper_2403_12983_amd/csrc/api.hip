// C interface of libosscar: context, workspace carve-up and host-side orchestration of the kernels.
#include "../../include/osscar.h"
#include "internal.h"

#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <numeric>
#include <string>
#include <vector>

using namespace osscar;

namespace {

constexpr int64_t XT_ROWS = 4096;   // calibration rows per sub-step of the generic (non-MFMA-bf16) Gram path
constexpr int64_t PACK_ROWS = 16384;   // calibration rows repacked at a time on the bf16 MFMA path
// staging buffer of the Gram phase: float32 X^T sub-step (generic path) or repacked bf16 rows (MFMA path)
size_t rect_tile_entries(int64_t d1, int64_t m) { return (size_t)(((d1 + 127) / 128 + 3) / 4 * (((m + 127) / 128 + 7) / 8) + 8) * 32; }
// staging of a target chunk: repacked bf16 rows (MFMA path) or a float32 sub-step (generic path)
size_t target_stage_bytes(int64_t m) { return (size_t)std::max<int64_t>(XT_ROWS * m * 4, PACK_ROWS * ((m + 127) / 128 * 128) * 2); }
size_t gram_stage_bytes(int64_t d1) { return (size_t)std::max<int64_t>(d1 * XT_ROWS * 4, PACK_ROWS * ((d1 + 127) / 128 * 128) * 2); }
constexpr int EV_SAMPLES = 64;

size_t align_up(size_t x, size_t a = 256) { return (x + a - 1) / a * a; }
// buffers of the two corrections that run on the bf16 matrix cores: packed pieces of P and of the residual (a x a for the
// inverse, a x m for the weights), and the float64 accumulator of the result (kept rows a, m columns)
size_t split_acc_elems(size_t a, size_t b, size_t m) { (void)b; return std::max(a * a, a * m); }
size_t split_x_cols(size_t a, size_t b, size_t m) { (void)b; return std::max(a, m); }
// scratch of the int8-digit products (i8gemm.hip): the A side is P, H_KK or H_cK (max(a, b) rows), the B side P, G_K, B, H_Kc
// or V (max(a, b, m) columns); the contraction always runs over the a kept rows
size_t i8_rows(size_t a, size_t b) { return std::max(a, b); }
size_t i8_cols(size_t a, size_t b, size_t m) { return std::max(std::max(a, b), m); }
size_t i8_bytes(size_t a, size_t b, size_t m) {
  return align_up(i8_pack_bytes(i8_rows(a, b), a)) + align_up(i8_pack_bytes(i8_cols(a, b, m), a)) + align_up((i8_rows(a, b) + i8_cols(a, b, m)) * 4) +
         align_up(a * 4);
}
size_t split_bytes(size_t a, size_t b, size_t m) {
  return align_up(split_pack_bytes(a, a)) + align_up(split_pack_bytes(a, split_x_cols(a, b, m))) + align_up(split_acc_elems(a, b, m) * 8);
}
size_t gram_tile_entries(int64_t d1) { size_t t = (size_t)(d1 + 127) / 128; return 8 * (t * t / 2 + t + 8); }
// room for any tile list of the state build: shapes up to d1 x max(d1, m), rectangular or lower triangle
size_t state_tile_entries(int64_t d1, int64_t m) { return std::max(rect_tile_entries(d1, std::max(d1, m)), gram_tile_entries(d1)); }

struct Carve {
  char* base; size_t off;
  explicit Carve(void* b) : base(reinterpret_cast<char*>(b)), off(0) {}
  template <typename T> T* take(size_t count) {
    T* p = base ? reinterpret_cast<T*>(base + off) : nullptr;
    off += align_up(count * sizeof(T));
    return p;
  }
};

__global__ void fill_f64_kernel(double* p, int64_t n, double v) {
  for (int64_t i = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x) p[i] = v;
}
// out = the symmetric matrix whose lower triangle is that of A
__global__ void mirror_from_lower_kernel(const float* __restrict__ A, float* __restrict__ out, int n) {
  int64_t tot = (int64_t)n * n;
  for (int64_t idx = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; idx < tot; idx += (int64_t)gridDim.x * blockDim.x) {
    int i = (int)(idx / n), j = (int)(idx % n);
    out[idx] = (j <= i) ? A[idx] : A[(int64_t)j * n + i];
  }
}
__global__ void add_inplace_kernel(float* __restrict__ a, const float* __restrict__ b, int64_t n) {
  for (int64_t i = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x) a[i] += b[i];
}
// dst[i][j] = sign * Nsym(rows[i], cols[j])
__global__ void gather_sym_kernel(const float* __restrict__ N, int64_t ld, const int32_t* __restrict__ rows, int nrows,
                                  const int32_t* __restrict__ cols, int ncols, float* __restrict__ dst, float sign) {
  int64_t tot = (int64_t)nrows * ncols;
  for (int64_t idx = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; idx < tot; idx += (int64_t)gridDim.x * blockDim.x) {
    int i = (int)(idx / ncols), j = (int)(idx % ncols);
    int64_t r = rows[i], c = cols[j];
    int64_t hi = r > c ? r : c, lo = r > c ? c : r;
    dst[idx] = sign * N[hi * ld + lo];
  }
}
int grid_for(int64_t n) { int64_t b = (n + 1023) / 1024; return (int)std::min<int64_t>(std::max<int64_t>(b, 1), 131072); }

}  // namespace

static thread_local std::string g_contextless_error = "no error recorded";
namespace osscar { void set_contextless_error(const char* msg) { g_contextless_error = msg ? msg : ""; } }

struct osscar_ctx {
  osscar_desc desc;
  hipStream_t stream;
  int d1, m, p, q, k, kr, cr;
  bool poisoned = false;
  std::string err;
  enum Phase { FRESH, ACCUM, FINAL, READY } phase = FRESH;

  // persistent device arrays
  float *H, *G, *N, *Z;
  double *norms2, *score, *gram, *dblk, *small, *scal, *partial, *dpart;
  double *cross, *xgram, *xdblk, *xscore;   // exact entering rule
  int32_t *kept, *rowsK, *rowsC, *notpd;
  float *C1, *C2, *Cblk, *rZ1, *rZ2;
  SearchCtrl* ctrl;
  int32_t *trace_out, *trace_in; float* trace_gap; double* trace_obj;
  int32_t *g_pick, *g_removed; float* g_gap;   // nested schedule from the dense layer
  int2 *tiles_sym, *tiles_rect;                // tile schedules of the bf16 matrix-core products (uploaded once at create)
  size_t n_tiles_sym = 0, n_tiles_rect = 0;
  int2* tiles_state;                           // two schedules of the corrections' products (shapes follow the kept count)
  std::vector<int2> tl_host[2];                // their host copies stay alive while the copies to the device are in flight
  int64_t counters[8] = {0, 0, 0, 0, 0, 0, 0, 0};
  float* Wdense = nullptr;       // float32 copy of W kept from finalize: the dense layer's exact weights (nested schedule), and
  bool have_Wdense = false;      // the pruned rows' weights for the objective of a kept set (build_state)
  LazyPtrs lazy;
  // phase-shared scratch
  char* scratch; size_t scratch_bytes;

  double lambda = 0, c0 = 0;
  int accum_target = 0;          // the layer being accumulated takes its chunks through osscar_gram_target
  bool dense_is_exact = true;    // the dense layer has objective 0 (false for a target output or a caller-supplied quadratic form)
  std::vector<double> norms_host;
  std::vector<int32_t> kept_host;
  double timers[16] = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
  hipEvent_t ev_a = nullptr, ev_b = nullptr;
  hipEvent_t ev_s[EV_SAMPLES][3];
  hipEvent_t ev_g[2 * EV_SAMPLES];   // pairs around the launches of the Gram kernel of the last chunk call
  SearchCtrl* snap = nullptr;         // pinned host memory for reading the control block
  int ev_g_used = 0; int64_t ev_g_rows = 0;
  SideStream side;   // the flush of the delayed-update search overlaps two of its products
  bool ev_ok = false;
};

namespace {

struct Layout {
  size_t total = 0, scratch_bytes = 0;
};

// Carves (or just sizes, when base == nullptr) the workspace for a description.
Layout carve_all(const osscar_desc& ds, void* base, osscar_ctx* c) {
  const int64_t d1 = ds.d1, m = ds.m, p = ds.p, q = ds.q, kr = (int64_t)ds.k * q, cr = d1 - kr;
  const int64_t ms = std::max<int32_t>(ds.max_swaps, 1);
  Carve cv(base);
  float* H = cv.take<float>(d1 * d1);
  float* G = cv.take<float>(d1 * m);
  float* N = cv.take<float>(d1 * d1);
  float* Z = cv.take<float>(d1 * m);
  double* norms2 = cv.take<double>(p);
  double* score = cv.take<double>(p);
  double* gram = cv.take<double>(p * q * q);
  double* dblk = cv.take<double>(p * q * q);
  double* small = cv.take<double>(std::max<int64_t>(16 * q * q, INV_NB * INV_NB));
  double* cross = cv.take<double>(d1 * q);
  double* xgram = cv.take<double>(p * q * q);
  double* xdblk = cv.take<double>(p * q * q);
  double* xscore = cv.take<double>(p);
  double* scal = cv.take<double>(1024);
  double* partial = cv.take<double>(2048);
  double* dpart = cv.take<double>((m + 15) / 16 + 64);
  int32_t* kept = cv.take<int32_t>(p);
  int32_t* rowsK = cv.take<int32_t>(d1);
  int32_t* rowsC = cv.take<int32_t>(d1);
  int32_t* notpd = cv.take<int32_t>(64);
  float* C1 = cv.take<float>(d1 * q);
  float* C2 = cv.take<float>(d1 * q);
  float* Cblk = cv.take<float>(4 * d1 * q);
  float* rZ1 = cv.take<float>(q * m);
  float* rZ2 = cv.take<float>(q * m);
  SearchCtrl* ctrl = cv.take<SearchCtrl>(4);
  int32_t* trace_out = cv.take<int32_t>(ms);
  int32_t* trace_in = cv.take<int32_t>(ms);
  float* trace_gap = cv.take<float>(2 * ms);
  double* trace_obj = cv.take<double>(ms);
  int32_t* g_pick = cv.take<int32_t>(128);      // 64 leaving + 64 entering picks of a block move
  int32_t* g_removed = cv.take<int32_t>(p);
  float* g_gap = cv.take<float>(p);
  float* Wdense = cv.take<float>(d1 * m);
  int2* tiles_sym = cv.take<int2>(gram_tile_entries(d1));
  int2* tiles_rect = cv.take<int2>(rect_tile_entries(d1, m));
  int2* tiles_state = cv.take<int2>(2 * state_tile_entries(d1, m));
  LazyPtrs L{};
  if (q == 1) {
    const int64_t TM = LAZY_TM;
    L.pos = cv.take<int32_t>(d1); L.Tidx = cv.take<int32_t>(TM); L.Jsg = cv.take<float>(TM);
    L.C0R = cv.take<float>(d1 * TM); L.Minv = cv.take<double>(TM * TM); L.Minv32 = cv.take<float>(TM * TM);
    L.ZT = cv.take<double>(TM * m); L.ZT32 = cv.take<float>(TM * m); L.E = cv.take<float>(d1 * TM);
    L.xg = cv.take<double>(TM); L.xj = cv.take<double>(TM); L.u1 = cv.take<double>(4 * TM); L.u2 = cv.take<double>(4 * TM);      // GEMV_SPLIT partial sums per pending row
    L.cg = cv.take<double>(d1); L.cj = cv.take<double>(d1); L.w1 = cv.take<double>(d1); L.w2 = cv.take<double>(d1);
    L.y1 = cv.take<double>(m); L.y2 = cv.take<double>(m); L.y1f = cv.take<float>(m); L.y2f = cv.take<float>(m);
    L.part = cv.take<double>(((m + 63) / 64) * 5); L.ls = cv.take<double>(16);
    L.sel = cv.take<SelRec>((d1 + 31) / 32);
    L.GbT = cv.take<double>((int64_t)(LAZY_NC + LAZY_NS) * d1); L.Zc = cv.take<float>((int64_t)LAZY_NC * m);
    L.rowsq = cv.take<double>((int64_t)2 * ((m + 127) / 128) * d1);
    L.ZcP = cv.take<char>((int64_t)LAZY_NC * ((m + 31) / 32 * 32) * 6);
    L.Epk = cv.take<char>((int64_t)768 * ((d1 + 127) / 128 * 128)); L.Cpk = cv.take<char>((int64_t)768 * ((d1 + 127) / 128 * 128));
    L.Zpk = cv.take<char>((int64_t)768 * ((m + 127) / 128 * 128));
    L.cslot = cv.take<int32_t>(d1); L.cand = cv.take<int32_t>(LAZY_NC + LAZY_NS); L.tslot = cv.take<int32_t>(LAZY_TM);
    L.misc = cv.take<int32_t>(8); L.lkey = cv.take<double>(2 * 64 * 32); L.lidx = cv.take<int32_t>(2 * 64 * 32);
    L.bB = cv.take<double>(TM * LAZY_BT); L.bX = cv.take<double>(TM * LAZY_BT); L.bU = cv.take<double>(4 * TM * LAZY_BT);
    L.bD = cv.take<double>(LAZY_BT * LAZY_BT); L.bYY = cv.take<double>(LAZY_BT * LAZY_BT); L.bY = cv.take<double>((int64_t)LAZY_BT * m);
    L.bpart = cv.take<double>(((m + 63) / 64) * (LAZY_BT * LAZY_BT + LAZY_BT)); L.bdl = cv.take<double>(LAZY_BT);
    L.bG = cv.take<int32_t>(LAZY_BT);
  }
  // scratch: the larger of the Gram phase and the init / refresh / backsolve phase
  size_t gram_phase = align_up((size_t)d1 * d1 * 8) + align_up((size_t)d1 * m * 4) + align_up(gram_stage_bytes(d1));
  if (ds.target_output) gram_phase += align_up((size_t)d1 * m * 8) + align_up(target_stage_bytes(m));
  auto init_bytes = [&](size_t a, size_t b) {   // kept rows a, candidate rows b
    return 4 * align_up(a * a * 4) + 3 * align_up(a * b * 4) + align_up(b * b * 4) + 4 * align_up(a * m * 4) + align_up(b * m * 4) +
           align_up(10 * a * INV_NB * 4) + split_bytes(a, b, m) + i8_bytes(a, b, m) + 4096;
  };
  size_t init_phase = init_bytes(kr, cr);
  if (ds.from_dense) {   // the nested schedule visits every kept-row count from d1 down to kr
    init_phase = std::max(init_phase, init_bytes(d1, 0));
    init_phase = std::max(init_phase, init_bytes(d1 / 2, d1 - d1 / 2));
  }
  size_t scratch_bytes = std::max(gram_phase, init_phase);
  char* scratch = cv.take<char>(scratch_bytes);
  if (c) {
    c->H = H; c->G = G; c->N = N; c->Z = Z; c->norms2 = norms2; c->score = score; c->gram = gram; c->dblk = dblk;
    c->cross = cross; c->xgram = xgram; c->xdblk = xdblk; c->xscore = xscore;
    c->small = small; c->scal = scal; c->partial = partial; c->dpart = dpart; c->kept = kept; c->rowsK = rowsK; c->rowsC = rowsC;
    c->notpd = notpd; c->C1 = C1; c->C2 = C2; c->Cblk = Cblk; c->rZ1 = rZ1; c->rZ2 = rZ2; c->ctrl = ctrl;
    c->trace_out = trace_out; c->trace_in = trace_in; c->trace_gap = trace_gap; c->trace_obj = trace_obj;
    c->g_pick = g_pick; c->g_removed = g_removed; c->g_gap = g_gap; c->Wdense = Wdense;
    c->tiles_sym = tiles_sym; c->tiles_rect = tiles_rect; c->tiles_state = tiles_state;
    c->scratch = scratch; c->scratch_bytes = scratch_bytes; c->lazy = L;
  }
  Layout lay; lay.total = cv.off; lay.scratch_bytes = scratch_bytes;
  return lay;
}

bool desc_ok(const osscar_desc* d) {
  if (!d) return false;
  if (d->d1 <= 0 || d->m <= 0 || d->p <= 0 || d->q <= 0 || d->q > 64) return false;
  if ((int64_t)d->p * d->q != d->d1) return false;
  if (d->k < 1 || d->k > d->p) return false;
  if (d->d1 > 65536 || d->m > 65536 || d->max_swaps < 0) return false;
  if (d->x_dtype != OSSCAR_F32 && d->x_dtype != OSSCAR_BF16) return false;
  if (d->w_dtype != OSSCAR_F32 && d->w_dtype != OSSCAR_BF16) return false;
  return true;
}

osscar_status fail(osscar_ctx* c, osscar_status st, const char* fmt, ...) {
  char buf[512];
  va_list ap; va_start(ap, fmt); vsnprintf(buf, sizeof buf, fmt, ap); va_end(ap);
  if (c) { c->err = buf; if (st != OSSCAR_EINVAL && st != OSSCAR_ESTATE) c->poisoned = true; }
  return st;
}

#define HIPCHK(c, expr)                                                                           \
  do {                                                                                            \
    hipError_t e__ = (expr);                                                                      \
    if (e__ != hipSuccess) return fail((c), OSSCAR_EHIP, "%s failed: %s", #expr, hipGetErrorString(e__)); \
  } while (0)

TabDims dims(const osscar_ctx* c) { return TabDims{c->d1, c->m, c->p, c->q}; }
TabPtrs ptrs(const osscar_ctx* c) {
  TabPtrs t{};
  t.N = c->N; t.Z = c->Z; t.kept = c->kept; t.score = c->score; t.gram = c->gram; t.dblk = c->dblk;
  t.C1 = c->C1; t.C2 = c->C2; t.C1D = c->Cblk; t.C2D = c->Cblk + (int64_t)c->d1 * c->q;
  t.rZ1 = c->rZ1; t.rZ2 = c->rZ2; t.small = c->small; t.dpart = c->dpart; t.ctrl = c->ctrl;
  t.cross = c->cross; t.xgram = c->xgram; t.xdblk = c->xdblk; t.xscore = c->xscore;
  t.trace_out = c->trace_out; t.trace_in = c->trace_in; t.trace_gap = c->trace_gap; t.trace_obj = c->trace_obj;
  return t;
}

hipError_t gemm(hipStream_t s, int M, int N, int K, const float* A, int64_t lda, const float* B, int64_t ldb, const float* Cin,
                int64_t ldcin, float* C, int64_t ldc, double alpha, double beta, double diag_add = 0.0, int lower_only = 0,
                int trans_b = 0, int acc_f32 = 0) {
  GemmArgs g{};
  g.M = M; g.N = N; g.K = K; g.A = A; g.lda = lda; g.B = B; g.ldb = ldb; g.Cin = Cin; g.ldcin = ldcin; g.C = C; g.ldc = ldc;
  g.alpha = alpha; g.beta = beta; g.diag_add = diag_add; g.c_is_f64 = 0; g.lower_only = lower_only; g.trans_b = trans_b;
  g.acc_f32 = acc_f32;
  return launch_gemm_f64acc(g, s);
}

// The large products that define the state (B = P G_K, V, S, R): on the int8 matrix cores (i8gemm.hip) when every dimension
// is at least I8_MIN_DIM and the scratch is there, else on the float64-accumulating kernel, which also keeps the residuals
// that involve P (of the Newton-Schulz route of the inverse, of the weight correction).  osscar_debug_int_products(0) sends
// everything there (tests).
struct I8Bufs {
  void* packA = nullptr; void* packB = nullptr; unsigned* mx = nullptr; size_t capA = 0, capB = 0, mx_entries = 0;
  int* kexp = nullptr;      // round(log2 sqrt(H_kk)) of the kept rows (the contraction index of every large product), once per state build
};
constexpr int I8_MIN_DIM = 1024;
bool g_i8_products = true;
hipError_t big_gemm(hipStream_t s, const I8Bufs* ib, int M, int N, int K, const float* A, int64_t lda, const float* B, int64_t ldb,
                    const float* Cin, int64_t ldcin, float* C, int64_t ldc, double alpha, double beta, double diag_add = 0.0,
                    int lower_only = 0, int diag_a = 0, int diag_b = 0, int ksign = 0) {
  GemmArgs g{};
  g.i8_diag_a = diag_a; g.i8_diag_b = diag_b;
  if (ib && ib->kexp && ksign != 0) { g.i8_kexp = ib->kexp; g.i8_ksign = ksign; }
  g.M = M; g.N = N; g.K = K; g.A = A; g.lda = lda; g.B = B; g.ldb = ldb; g.Cin = Cin; g.ldcin = ldcin; g.C = C; g.ldc = ldc;
  g.alpha = alpha; g.beta = beta; g.diag_add = diag_add; g.lower_only = lower_only;
  if (g_i8_products && ib && ib->packA && M >= I8_MIN_DIM && N >= I8_MIN_DIM && K >= I8_MIN_DIM && i8_gemm_fits(g) &&
      i8_pack_bytes(M, K) <= ib->capA && i8_pack_bytes(N, K) <= ib->capB && (size_t)M + (size_t)N <= ib->mx_entries)
    return launch_i8_gemm(g, ib->packA, ib->capA, ib->packB, ib->capB, ib->mx, ib->mx_entries, s);
  return launch_gemm_f64acc(g, s);
}

// Host copy of the membership flags -> sorted row lists on the device.
osscar_status upload_rows(osscar_ctx* c) {
  std::vector<int32_t> rk, rc;
  rk.reserve(c->kr); rc.reserve(c->cr);
  for (int g = 0; g < c->p; g++)
    for (int r = 0; r < c->q; r++) (c->kept_host[g] ? rk : rc).push_back(g * c->q + r);
  if ((int)rk.size() != c->kr) return fail(c, OSSCAR_ESTATE, "internal: kept set has %zu rows, expected %d", rk.size(), c->kr);
  HIPCHK(c, hipMemcpyAsync(c->rowsK, rk.data(), rk.size() * 4, hipMemcpyHostToDevice, c->stream));
  if (!rc.empty()) HIPCHK(c, hipMemcpyAsync(c->rowsC, rc.data(), rc.size() * 4, hipMemcpyHostToDevice, c->stream));
  HIPCHK(c, hipStreamSynchronize(c->stream));   // the vectors die at return
  return OSSCAR_OK;
}

// P = (H_KK)^-1 (full, symmetric) and B = P G_K (with one float64-residual refinement step if P is not yet exact), for the rows in
// c->rowsK.  Buffers come from the scratch region: HKK (kept), P, T1, T2 (kr x kr each), GK, B (kr x m), T3, T4.
// sp != nullptr: the two small corrections (P (I - H_KK P) of the inverse, P (G_K - H_KK B) of the weights) run on the bf16
// matrix cores through three-piece splits.  The products that define the state -- B = P G_K, V, S, R -- do not: with
// float32 sums inside the matrix cores they came out 3e-5 (B, V) and 1e-3 (R) away from the float64-accumulated
// results on the 28672-row layer, whose H has large entries of one sign that cancel in these products.
struct SplitBufs { void *packP, *packX; double* acc; size_t capP, capX, cap_acc; };   // capacities in bytes / elements
struct InvBufs { float *HKK, *P, *T1, *T2, *GK, *B, *T3, *T4, *panels; const SplitBufs* sp = nullptr; const I8Bufs* i8 = nullptr; };

// Are the shapes fit for the packed bf16 products (8-element packets)?
bool split_ok(const osscar_ctx* c) { return c->kr % 8 == 0 && c->m % 8 == 0; }

// Tile schedule `slot` of the state build for an M x N result (lower: the lower triangle of a square result): built on the
// host, copied behind the stream's earlier work.
struct TileRef { const int2* dev; size_t entries; int ntiles; };
osscar_status stage_tiles(osscar_ctx* c, int slot, int M, int N, bool lower, TileRef* out) {
  std::vector<int2>& v = c->tl_host[slot];
  if (lower) gram_tile_list_host(M, v); else rect_tile_list_host(M, N, v);
  const size_t cap = state_tile_entries(c->d1, c->m);
  if (v.size() > cap) return fail(c, OSSCAR_ENOMEM, "internal: tile schedule of a %d x %d product exceeds its buffer", M, N);
  int2* dev = c->tiles_state + (size_t)slot * cap;
  HIPCHK(c, hipMemcpyAsync(dev, v.data(), v.size() * sizeof(int2), hipMemcpyHostToDevice, c->stream));
  const int tm = (M + 127) / 128, tn = (N + 127) / 128;
  out->dev = dev; out->entries = v.size(); out->ntiles = lower ? tm * (tm + 1) / 2 : tm * tn;
  return OSSCAR_OK;
}

// the three bf16 pieces of A (K x cols, contraction along the rows) into one of the pack buffers, capacity checked
osscar_status pack_into(osscar_ctx* c, const SplitBufs& sp, void* pack, const float* A, int64_t lda, int K, int cols) {
  const size_t cap = pack == sp.packP ? sp.capP : pack == sp.packX ? sp.capX : 0;
  if (split_pack_bytes(K, cols) > cap) return fail(c, OSSCAR_ENOMEM, "internal: packed operand %d x %d exceeds its buffer", K, cols);
  HIPCHK(c, launch_pack_pieces(A, lda, K, cols, pack, c->stream));
  return OSSCAR_OK;
}

// C = beta Cin + alpha A^T B from packed pieces (see gram.hip: launch_split_product)
osscar_status split_gemm(osscar_ctx* c, const SplitBufs& sp, const void* packA, int M, const void* packB, int N, int K, int nprod,
                         const TileRef& t, const float* Cin, int64_t ldcin, float* C, int64_t ldc, double alpha, double beta) {
  if ((size_t)M * N > sp.cap_acc) return fail(c, OSSCAR_ENOMEM, "internal: %d x %d product exceeds the accumulator", M, N);
  HIPCHK(c, launch_split_product(packA, M, packB, N, K, nprod, sp.acc, t.dev, t.entries, t.ntiles, c->stream));
  HIPCHK(c, launch_split_epilogue(sp.acc, M, N, Cin, ldcin, C, ldc, alpha, beta, c->stream));
  return OSSCAR_OK;
}

// out[0] = max_i P_ii H_ii (the largest variance inflation factor 1 / (1 - R_i^2) of a kept row: how much of row i the other
// kept rows explain), out[1] = 1 if any entry of the diagonal of P is not finite.  One workgroup.
__global__ __launch_bounds__(1024) void vif_max_kernel(const float* __restrict__ P, const float* __restrict__ H, int n, double* __restrict__ out) {
  __shared__ double sh[16];
  __shared__ int bad[16];
  double v = 0.0; int b = 0;
  for (int i = threadIdx.x; i < n; i += 1024) {
    const double x = (double)P[(int64_t)i * n + i] * (double)H[(int64_t)i * n + i];
    if (!(x == x) || !(fabs(x) < 1e300)) b = 1; else v = fmax(v, x);
  }
  for (int o = 32; o > 0; o >>= 1) { v = fmax(v, __shfl_down(v, o, 64)); b |= __shfl_down(b, o, 64); }
  if ((threadIdx.x & 63) == 0) { sh[threadIdx.x >> 6] = v; bad[threadIdx.x >> 6] = b; }
  __syncthreads();
  if (threadIdx.x == 0) {
    for (int i = 1; i < 16; i++) { v = fmax(v, sh[i]); b |= bad[i]; }
    out[0] = v; out[1] = (double)b;
  }
}

// The inverse by the float64-storage sweep (default), or by the float32 sweep refined by Newton-Schulz
// (osscar_debug_refined_inverse(1): the two are held against each other in the tests).
bool g_refined_inverse = false;
// osscar_debug_side_stream(0): no second stream anywhere (tests hold the overlapped schedules against the in-order ones)
bool g_side_stream = true;
static const SideStream* side_of(const osscar_ctx* c) { return (g_side_stream && c->ev_ok) ? &c->side : nullptr; }

// B_known (optional, kr x m): the weights are known exactly (dense layer: B = W), only G_K is gathered beside them.
osscar_status inverse_and_weights(osscar_ctx* c, const InvBufs& b, const float* B_known = nullptr) {
  hipStream_t s = c->stream;
  const int kr = c->kr, m = c->m;
  HIPCHK(c, launch_gather(c->H, c->d1, c->rowsK, kr, c->rowsK, kr, b.HKK, kr, s));
  if (b.i8 && b.i8->kexp) HIPCHK(c, launch_i8_kexp(b.HKK, kr, kr, b.i8->kexp, s));
  HIPCHK(c, hipMemsetAsync(c->notpd, 0, 64 * 4, s));
  const SplitBufs* sp = b.sp;
  osscar_status st = OSSCAR_OK;
  bool correct = false;          // does B = P G_K get its residual correction?
  TileRef t_low{}, t_b{};
  if (sp) {
    if ((st = stage_tiles(c, 0, kr, kr, true, &t_low)) != OSSCAR_OK) return st;
    if ((st = stage_tiles(c, 1, kr, m, false, &t_b)) != OSSCAR_OK) return st;
  }
  if (!g_refined_inverse) {
    // The sweep on a float64 copy of H_KK (in the memory of T1 and T2), rounded to float32 once: exact to that rounding.
    HIPCHK(c, hipEventRecord(c->ev_s[2][0], s));
    HIPCHK(c, spd_inverse_f64(b.HKK, kr, kr, b.P, reinterpret_cast<double*>(b.T1), reinterpret_cast<double*>(b.panels), c->small, c->notpd, s,
                              side_of(c)));
    HIPCHK(c, hipEventRecord(c->ev_s[2][1], s));
    HIPCHK(c, launch_absmax(b.P, (int64_t)kr * kr, c->partial, s));
    hipLaunchKernelGGL(vif_max_kernel, dim3(1), dim3(1024), 0, s, b.P, b.HKK, kr, c->scal + 20);
    double part[256], vif[2] = {0, 0}; int32_t bad = 0;
    HIPCHK(c, hipMemcpyAsync(part, c->partial, sizeof part, hipMemcpyDeviceToHost, s));
    HIPCHK(c, hipMemcpyAsync(vif, c->scal + 20, 16, hipMemcpyDeviceToHost, s));
    HIPCHK(c, hipMemcpyAsync(&bad, c->notpd, 4, hipMemcpyDeviceToHost, s));
    HIPCHK(c, hipStreamSynchronize(s));
    { float ms = 0; hipEventElapsedTime(&ms, c->ev_s[2][0], c->ev_s[2][1]); c->timers[9] = ms; }
    c->timers[10] = 0; c->timers[11] = vif[0];
    double pmax = 0;
    for (double v : part) if (v > pmax || v != v) pmax = v;      // a NaN anywhere in P makes pmax NaN
    if (bad || vif[1] != 0.0 || !(pmax < 1e300) || !(vif[0] >= 0.999))
      return fail(c, OSSCAR_ENOTPD, "H restricted to the kept rows is not positive definite to working precision "
                                     "(pivot flag %d, largest |P| %.3g, largest P_ii H_ii %.3g)", bad, pmax, vif[0]);
    // P is exact to its float32 rounding, which still costs B = P G_K about 6e-8 times the cancellation in that product.
    // The largest P_ii H_ii measures it: 1.5 - 25 on the benchmark recipes and the correlated test layers, 270 and 1800 on
    // the two test layers where B without the correction left the objective off by more than 1e-5; from 100 on B is
    // corrected against its float64 residual.
    correct = vif[0] >= 100.0;
  } else {
  HIPCHK(c, launch_gather(c->H, c->d1, c->rowsK, kr, c->rowsK, kr, b.P, kr, s));
  HIPCHK(c, spd_inverse_inplace(b.P, kr, b.panels, b.panels + (int64_t)kr * INV_NB, c->small, c->notpd, s));
  // Newton-Schulz: P <- P + P (I - H_KK P), residual accumulated in float64
  double last_resid = 1.0;
  for (int step = 0; step < 3; step++) {
    HIPCHK(c, hipEventRecord(c->ev_s[2][0], s));
    // The residual stays on the float64 matrix-core instruction: what the step needs from it is the error of P along the
    // few dominant directions of H (where P is 1e-4 and less of its norm), and five 7-bit digits per operand do not carry that:
    // with this one product on the int8 path the addition gains of the 28672-row benchmark layer came out 4 times further
    // from the float64 state (8e-5 against 2e-5), with all the others there they are unchanged.
    HIPCHK(c, gemm(s, kr, kr, kr, b.HKK, kr, b.P, kr, nullptr, 0, b.T1, kr, -1.0, 0.0, 1.0));
    HIPCHK(c, hipEventRecord(c->ev_s[2][1], s));
    HIPCHK(c, launch_absmax(b.T1, (int64_t)kr * kr, c->partial, s));
    // P + P (I - H P) is symmetric up to rounding: compute its lower triangle and mirror it.  The correction P (I - H P) is
    // about 1e-5 of P, so it needs only a few digits: float32 accumulation, or the three leading products of the bf16
    // pieces (2^-16 of the correction), are far below P's own rounding.
    HIPCHK(c, hipEventRecord(c->ev_s[1][0], s));
    if (sp) {
      if ((st = pack_into(c, *sp, sp->packP, b.P, kr, kr, kr)) != OSSCAR_OK) return st;
      if ((st = pack_into(c, *sp, sp->packX, b.T1, kr, kr, kr)) != OSSCAR_OK) return st;
      if ((st = split_gemm(c, *sp, sp->packP, kr, sp->packX, kr, kr, 3, t_low, b.P, kr, b.T2, kr, 1.0, 1.0)) != OSSCAR_OK) return st;
    } else {
      HIPCHK(c, gemm(s, kr, kr, kr, b.P, kr, b.T1, kr, b.P, kr, b.T2, kr, 1.0, 1.0, 0.0, 1, 0, 1));
    }
    HIPCHK(c, hipEventRecord(c->ev_s[1][1], s));
    hipLaunchKernelGGL(mirror_from_lower_kernel, dim3(grid_for((int64_t)kr * kr)), dim3(256), 0, s, b.T2, b.P, kr);
    double part[256]; int32_t bad = 0;
    HIPCHK(c, hipMemcpyAsync(part, c->partial, sizeof part, hipMemcpyDeviceToHost, s));
    HIPCHK(c, hipMemcpyAsync(&bad, c->notpd, 4, hipMemcpyDeviceToHost, s));
    HIPCHK(c, hipStreamSynchronize(s));
    { float ms = 0; hipEventElapsedTime(&ms, c->ev_s[1][0], c->ev_s[1][1]); c->timers[10] = ms; }
    { float ms = 0; hipEventElapsedTime(&ms, c->ev_s[2][0], c->ev_s[2][1]); c->timers[9] = ms; }
    double resid = 0;
    for (double v : part) if (v > resid || v != v) resid = v;      // a NaN anywhere in I - H P makes resid NaN
    if (bad || !(resid < 0.9))
      return fail(c, OSSCAR_ENOTPD, "H restricted to the kept rows is not positive definite to working precision "
                                     "(pivot flag %d, |I - H P|_max = %.3g)", bad, resid);
    last_resid = resid;
    c->timers[11] = resid;
    if (resid < 1e-3) break;     // the step just taken squares it below float32 resolution
    if (step == 2)                // three steps and still above: the last one leaves about resid^2, not good enough to call P exact
      return fail(c, OSSCAR_ENOTPD, "the inverse of H on the kept rows did not converge (|I - H P|_max = %.3g after three "
                                     "Newton-Schulz steps): H_KK is too ill-conditioned for float32 storage", resid);
  }
  // the residual before the last step is this path's measure of the conditioning (2e-5 on the benchmark layers)
  correct = !(last_resid < 4e-5);
  }

  // B = P G_K, then B += P (G_K - H_KK B)
  HIPCHK(c, launch_gather(c->G, m, c->rowsK, kr, nullptr, m, b.GK, m, s));
  if (B_known) {
    HIPCHK(c, hipMemcpyAsync(b.B, B_known, (size_t)kr * m * 4, hipMemcpyDeviceToDevice, s));
    return OSSCAR_OK;
  }
  float* B0 = correct ? b.T3 : b.B;
  HIPCHK(c, big_gemm(s, b.i8, kr, m, kr, b.P, kr, b.GK, m, nullptr, 0, B0, m, 1.0, 0.0, 0.0, 0, 1, 0, 1));
  if (!correct) return OSSCAR_OK;
  HIPCHK(c, gemm(s, kr, m, kr, b.HKK, kr, b.T3, m, b.GK, m, b.T4, m, -1.0, 1.0));      // the residual: float64 accumulation
  if (sp) {
    if ((st = pack_into(c, *sp, sp->packP, b.P, kr, kr, kr)) != OSSCAR_OK) return st;      // the refined inverse
    if ((st = pack_into(c, *sp, sp->packX, b.T4, m, kr, m)) != OSSCAR_OK) return st;
    if ((st = split_gemm(c, *sp, sp->packP, kr, sp->packX, m, kr, 3, t_b, b.T3, m, b.B, m, 1.0, 1.0)) != OSSCAR_OK) return st;
  } else {
    HIPCHK(c, gemm(s, kr, m, kr, b.P, kr, b.T4, m, b.T3, m, b.B, m, 1.0, 1.0));
  }
  return OSSCAR_OK;
}

SplitBufs carve_split(osscar_ctx* c, Carve& cv) {
  const size_t a = c->kr, bb = c->cr, m = c->m;
  SplitBufs sp;
  sp.capP = split_pack_bytes(a, a); sp.capX = split_pack_bytes(a, split_x_cols(a, bb, m));
  sp.cap_acc = split_acc_elems(a, bb, m);
  sp.packP = cv.take<char>(sp.capP);
  sp.packX = cv.take<char>(sp.capX);
  sp.acc = cv.take<double>(sp.cap_acc);
  return sp;
}

I8Bufs carve_i8(osscar_ctx* c, Carve& cv) {
  const size_t a = c->kr, bb = c->cr, m = c->m;
  I8Bufs ib;
  ib.capA = i8_pack_bytes(i8_rows(a, bb), a); ib.capB = i8_pack_bytes(i8_cols(a, bb, m), a);
  ib.mx_entries = i8_rows(a, bb) + i8_cols(a, bb, m);
  ib.packA = cv.take<char>(ib.capA);
  ib.packB = cv.take<char>(ib.capB);
  ib.mx = cv.take<unsigned>(ib.mx_entries);
  ib.kexp = cv.take<int>(a);
  return ib;
}

InvBufs carve_inv(osscar_ctx* c, Carve& cv) {
  const int64_t kr = c->kr, m = c->m;
  InvBufs b;
  b.HKK = cv.take<float>(kr * kr); b.P = cv.take<float>(kr * kr);
  b.T1 = cv.take<float>(2 * kr * kr); b.T2 = b.T1 + kr * kr;      // together: the kr x kr float64 work matrix of the sweep inverse
  b.GK = cv.take<float>(kr * m); b.B = cv.take<float>(kr * m); b.T3 = cv.take<float>(kr * m); b.T4 = cv.take<float>(kr * m);
  b.panels = cv.take<float>(10 * kr * INV_NB);                     // five panels of float64
  return b;
}

// obj = c0 - <G_K, B>
osscar_status objective_from(osscar_ctx* c, const float* GK, const float* B, double* obj) {
  HIPCHK(c, launch_dot64(GK, B, (int64_t)c->kr * c->m, c->scal + 8, c->partial, c->stream));
  double dot = 0;
  HIPCHK(c, hipMemcpyAsync(&dot, c->scal + 8, 8, hipMemcpyDeviceToHost, c->stream));
  HIPCHK(c, hipStreamSynchronize(c->stream));
  *obj = c->c0 - dot;
  return OSSCAR_OK;
}

// Builds N, Z, the scores and the tracked objective for the kept set in c->kept_host.
osscar_status build_state(osscar_ctx* c, double* obj_out, const float* B_known = nullptr) {
  hipStream_t s = c->stream;
  const int d1 = c->d1, m = c->m, kr = c->kr, cr = c->cr;
  osscar_status st = upload_rows(c);
  if (st != OSSCAR_OK) return st;
  HIPCHK(c, hipMemcpyAsync(c->kept, c->kept_host.data(), c->p * 4, hipMemcpyHostToDevice, s));
  Carve cv(c->scratch);
  InvBufs b = carve_inv(c, cv);
  float* HKC = cv.take<float>((int64_t)kr * cr);
  float* V = cv.take<float>((int64_t)kr * cr);
  float* HCK = cv.take<float>((int64_t)cr * kr);
  float* S = cv.take<float>((int64_t)cr * cr);
  float* R = cv.take<float>((int64_t)cr * m);
  SplitBufs sp = carve_split(c, cv);
  I8Bufs ib = carve_i8(c, cv);
  if (cv.off > c->scratch_bytes) return fail(c, OSSCAR_ENOMEM, "internal: scratch carve-up exceeds the workspace");
  const bool split = split_ok(c);
  if (split) b.sp = &sp;
  b.i8 = &ib;
  st = inverse_and_weights(c, b, B_known);
  if (st != OSSCAR_OK) return st;
  if (cr > 0) {
    HIPCHK(c, launch_gather(c->H, d1, c->rowsK, kr, c->rowsC, cr, HKC, cr, s));
    HIPCHK(c, launch_gather(c->H, d1, c->rowsC, cr, c->rowsC, cr, S, cr, s));
    HIPCHK(c, launch_gather(c->G, m, c->rowsC, cr, nullptr, m, R, m, s));
    HIPCHK(c, hipEventRecord(c->ev_s[0][0], s));
    HIPCHK(c, launch_gather(c->H, d1, c->rowsC, cr, c->rowsK, kr, HCK, kr, s));
    HIPCHK(c, big_gemm(s, b.i8, kr, cr, kr, b.P, kr, HKC, cr, nullptr, 0, V, cr, 1.0, 0.0, 0.0, 0, 1, 0, 1));   // V = P H_{K,Kc}
    HIPCHK(c, big_gemm(s, b.i8, cr, cr, kr, HCK, kr, V, cr, S, cr, S, cr, -1.0, 1.0, 0.0, 1, 0, 0, -1));   // S = H_cc - H_cK V (lower)
    HIPCHK(c, big_gemm(s, b.i8, cr, m, kr, HCK, kr, b.B, m, R, m, R, m, -1.0, 1.0, 0.0, 0, 0, 0, -1));     // R = G_c - H_cK B
    HIPCHK(c, hipEventRecord(c->ev_s[0][1], s));
    HIPCHK(c, launch_scatter(V, cr, c->rowsK, kr, c->rowsC, cr, c->N, d1, 1.f, 0, s));
    HIPCHK(c, launch_scatter(S, cr, c->rowsC, cr, c->rowsC, cr, c->N, d1, 1.f, 1, s));
    HIPCHK(c, launch_scatter_rows(R, m, c->rowsC, cr, m, c->Z, m, 0, s));
  }
  HIPCHK(c, launch_scatter(b.P, kr, c->rowsK, kr, c->rowsK, kr, c->N, d1, -1.f, 1, s));
  HIPCHK(c, launch_scatter_rows(b.B, m, c->rowsK, kr, m, c->Z, m, 0, s));
  HIPCHK(c, launch_refresh_scores(dims(c), ptrs(c), s));
  double obj = 0;
  if (c->have_Wdense && c->dense_is_exact) {
    // obj(K) = c0 - <G_K, B> = <W_c, R_c> over the pruned rows c (B = W_K + V W_c, so <G_K, B> = <G_K, W_K> + <V^T G_K, W_c>).
    // The first form subtracts two numbers of the size of c0 and inherits the float32 rounding of B at that size; the
    // second has terms of the size of the loss itself, which matters when the kept rows carry most of Tr(W^T H W).
    if (cr > 0) {
      HIPCHK(c, launch_dot64_rows(c->Wdense, c->rowsC, R, cr, m, c->scal + 8, c->partial, s));
      HIPCHK(c, hipMemcpyAsync(&obj, c->scal + 8, 8, hipMemcpyDeviceToHost, s));
    }
    HIPCHK(c, hipStreamSynchronize(s));
  } else {
    st = objective_from(c, b.GK, b.B, &obj);     // synchronises the stream
    if (st != OSSCAR_OK) return st;
  }
  if (cr > 0) { float ms = 0; hipEventElapsedTime(&ms, c->ev_s[0][0], c->ev_s[0][1]); c->timers[12] = ms; }
  if (obj_out) *obj_out = obj;
  return OSSCAR_OK;
}

osscar_status read_kept(osscar_ctx* c) {
  c->kept_host.resize(c->p);
  HIPCHK(c, hipMemcpyAsync(c->kept_host.data(), c->kept, c->p * 4, hipMemcpyDeviceToHost, c->stream));
  HIPCHK(c, hipStreamSynchronize(c->stream));
  return OSSCAR_OK;
}

osscar_status check_ctx(osscar_ctx* c) {
  if (!c) return OSSCAR_EINVAL;
  if (c->poisoned) return OSSCAR_ESTATE;
  return OSSCAR_OK;
}

double elapsed(osscar_ctx* c) {
  float ms = 0;
  if (c->ev_ok && hipEventSynchronize(c->ev_b) == hipSuccess) hipEventElapsedTime(&ms, c->ev_a, c->ev_b);
  return ms;
}

}  // namespace

extern "C" {

size_t osscar_workspace_bytes(const osscar_desc* desc) {
  if (!desc_ok(desc)) return 0;
  return carve_all(*desc, nullptr, nullptr).total + 256;
}

osscar_status osscar_create(osscar_ctx** out, const osscar_desc* desc, void* workspace_dev, size_t workspace_bytes,
                            void* hip_stream) {
  if (!out) return OSSCAR_EINVAL;
  *out = nullptr;
  if (!desc_ok(desc) || !workspace_dev) return OSSCAR_EINVAL;
  if ((reinterpret_cast<uintptr_t>(workspace_dev) & 255) != 0) return OSSCAR_EINVAL;
  size_t need = carve_all(*desc, nullptr, nullptr).total + 256;
  if (workspace_bytes < need) return OSSCAR_ENOMEM;
  osscar_ctx* c = new (std::nothrow) osscar_ctx();
  if (!c) return OSSCAR_ENOMEM;
  c->desc = *desc;
  c->stream = reinterpret_cast<hipStream_t>(hip_stream);
  c->d1 = (int)desc->d1; c->m = (int)desc->m; c->p = desc->p; c->q = desc->q; c->k = desc->k;
  c->kr = desc->k * desc->q; c->cr = c->d1 - c->kr;
  carve_all(*desc, workspace_dev, c);
  {   // tile schedules of the packed matrix-core products: built and uploaded once, so that no chunk call waits for the stream
    std::vector<int2> ts, tr;
    gram_tile_list_host(c->d1, ts);
    rect_tile_list_host(c->d1, c->m, tr);
    if (ts.size() > gram_tile_entries(c->d1) || tr.size() > rect_tile_entries(c->d1, c->m)) { delete c; return OSSCAR_ENOMEM; }
    if (hipMemcpy(c->tiles_sym, ts.data(), ts.size() * sizeof(int2), hipMemcpyHostToDevice) != hipSuccess ||
        hipMemcpy(c->tiles_rect, tr.data(), tr.size() * sizeof(int2), hipMemcpyHostToDevice) != hipSuccess) { delete c; return OSSCAR_EHIP; }
    c->n_tiles_sym = ts.size(); c->n_tiles_rect = tr.size();
    c->lazy.tiles_sym = c->tiles_sym; c->lazy.n_tiles_sym = ts.size(); c->lazy.tiles_rect = c->tiles_rect; c->lazy.n_tiles_rect = tr.size();
  }
  c->ev_ok = (hipEventCreate(&c->ev_a) == hipSuccess) && (hipEventCreate(&c->ev_b) == hipSuccess);
  for (int i = 0; i < EV_SAMPLES && c->ev_ok; i++)
    for (int j = 0; j < 3; j++) c->ev_ok = c->ev_ok && (hipEventCreate(&c->ev_s[i][j]) == hipSuccess);
  for (int i = 0; i < 2 * EV_SAMPLES && c->ev_ok; i++) c->ev_ok = c->ev_ok && (hipEventCreate(&c->ev_g[i]) == hipSuccess);
  c->ev_ok = c->ev_ok && hipHostMalloc(reinterpret_cast<void**>(&c->snap), sizeof(SearchCtrl), hipHostMallocDefault) == hipSuccess;
  c->ev_ok = c->ev_ok && hipStreamCreateWithFlags(&c->side.stream, hipStreamNonBlocking) == hipSuccess &&
             hipEventCreateWithFlags(&c->side.fork, hipEventDisableTiming) == hipSuccess &&
             hipEventCreateWithFlags(&c->side.join, hipEventDisableTiming) == hipSuccess;
  if (!c->ev_ok) { osscar_destroy(c); return OSSCAR_EHIP; }
  *out = c;
  return OSSCAR_OK;
}

osscar_status osscar_destroy(osscar_ctx* c) {
  if (!c) return OSSCAR_EINVAL;
  hipStreamSynchronize(c->stream);
  if (c->side.stream) { hipStreamSynchronize(c->side.stream); hipStreamDestroy(c->side.stream); }
  if (c->side.fork) hipEventDestroy(c->side.fork);
  if (c->side.join) hipEventDestroy(c->side.join);
  if (c->ev_a) hipEventDestroy(c->ev_a);
  if (c->ev_b) hipEventDestroy(c->ev_b);
  for (int i = 0; i < EV_SAMPLES; i++)
    for (int j = 0; j < 3; j++) if (c->ev_s[i][j]) hipEventDestroy(c->ev_s[i][j]);
  for (int i = 0; i < 2 * EV_SAMPLES; i++) if (c->ev_g[i]) hipEventDestroy(c->ev_g[i]);
  if (c->snap) hipHostFree(c->snap);
  delete c;
  return OSSCAR_OK;
}

const char* osscar_last_error(const osscar_ctx* c) { return c ? c->err.c_str() : g_contextless_error.c_str(); }

// Shared body of osscar_gram (Yc == nullptr, target == 0) and osscar_gram_target.
static osscar_status gram_impl(osscar_ctx* c, const char* who, int target, const void* Xc, const void* Yc, int64_t n_c, int64_t ldx,
                               int64_t ldy, int finalize, const void* W, int64_t ldw, double lambda_abs, double lambda_rel,
                               const ConvSpec* conv = nullptr) {
  osscar_status st = check_ctx(c);
  if (st != OSSCAR_OK) return st;
  if (n_c < 0 || (n_c > 0 && (!Xc || ldx < c->d1))) return fail(c, OSSCAR_EINVAL, "%s: bad chunk (n_c=%lld, ldx=%lld)", who, (long long)n_c, (long long)ldx);
  if (target && n_c > 0 && (!Yc || ldy < c->m)) return fail(c, OSSCAR_EINVAL, "%s: bad target chunk (ldy=%lld)", who, (long long)ldy);
  if (target && !c->desc.target_output) return fail(c, OSSCAR_EINVAL, "%s: the context was created without desc.target_output", who);
  if (finalize && (!W || ldw < c->m)) return fail(c, OSSCAR_EINVAL, "%s: finalize needs W with ldw >= m", who);
  if (c->phase == osscar_ctx::ACCUM && c->accum_target != target)
    return fail(c, OSSCAR_ESTATE, "%s: a layer takes all its chunks through osscar_gram or all through osscar_gram_target", who);
  hipStream_t s = c->stream;
  const int d1 = c->d1, m = c->m;
  Carve cv(c->scratch);
  double* H64 = cv.take<double>((int64_t)d1 * d1);
  float* Wf = cv.take<float>((int64_t)d1 * m);
  float* Xt = reinterpret_cast<float*>(cv.take<char>(gram_stage_bytes(d1)));
  double* G64 = nullptr; float* Ys = nullptr;
  if (c->desc.target_output) {
    G64 = cv.take<double>((int64_t)d1 * m);
    Ys = reinterpret_cast<float*>(cv.take<char>(target_stage_bytes(m)));
  }
  if (c->phase != osscar_ctx::ACCUM) {   // first chunk of a layer
    hipLaunchKernelGGL(fill_f64_kernel, dim3(grid_for((int64_t)d1 * d1)), dim3(256), 0, s, H64, (int64_t)d1 * d1, 0.0);
    if (target) {
      hipLaunchKernelGGL(fill_f64_kernel, dim3(grid_for((int64_t)d1 * m)), dim3(256), 0, s, G64, (int64_t)d1 * m, 0.0);
      hipLaunchKernelGGL(fill_f64_kernel, dim3(1), dim3(64), 0, s, c->scal + 12, (int64_t)1, 0.0);
    }
    c->phase = osscar_ctx::ACCUM;
    c->accum_target = target;
    c->timers[0] = 0;
  }
  if (n_c > 0) {
    HIPCHK(c, hipEventRecord(c->ev_a, s));
    const bool bf16 = c->desc.x_dtype == OSSCAR_BF16;
    bool fast = bf16 && (d1 % 8 == 0) && (conv || ((ldx % 8 == 0) && ((reinterpret_cast<uintptr_t>(Xc) & 15) == 0)));
    if (target) fast = fast && (m % 8 == 0) && (ldy % 8 == 0) && ((reinterpret_cast<uintptr_t>(Yc) & 15) == 0);
    if (target) HIPCHK(c, launch_sumsq(Yc, bf16, n_c, m, ldy, c->scal + 12, c->partial, s));
    if (fast) {
      if (target) HIPCHK(c, launch_gram_packed(Xc, n_c, ldx, d1, H64, c->tiles_sym, c->n_tiles_sym, Xt, PACK_ROWS, s, Yc, ldy, m, G64,
                                               c->tiles_rect, c->n_tiles_rect, Ys));
      else {
        HIPCHK(c, launch_gram_packed(Xc, n_c, ldx, d1, H64, c->tiles_sym, c->n_tiles_sym, Xt, PACK_ROWS, s, nullptr, 0, 0, nullptr,
                                     nullptr, 0, nullptr, conv, c->ev_g, EV_SAMPLES, &c->ev_g_used));
        c->ev_g_rows = n_c;
      }
    } else {
      const size_t esz = bf16 ? 2 : 4;
      for (int64_t r0 = 0; r0 < n_c; r0 += XT_ROWS) {
        int64_t nr = std::min<int64_t>(XT_ROWS, n_c - r0);
        const char* src = reinterpret_cast<const char*>(Xc) + (size_t)r0 * ldx * esz;
        if (conv) HIPCHK(c, launch_im2col_transpose(Xc, bf16, *conv, r0, nr, d1, Xt, XT_ROWS, s));
        else HIPCHK(c, launch_transpose_to_f32(src, bf16, nr, d1, ldx, Xt, XT_ROWS, s));
        GemmArgs g{};
        g.M = d1; g.N = d1; g.K = (int)nr; g.A = Xt; g.lda = XT_ROWS; g.B = Xt; g.ldb = XT_ROWS; g.trans_b = 1;
        g.Cin = reinterpret_cast<const float*>(H64); g.ldcin = d1; g.C = H64; g.ldc = d1; g.alpha = 1.0; g.beta = 1.0;
        g.c_is_f64 = 1; g.lower_only = 1;
        HIPCHK(c, launch_gemm_f64acc(g, s));
        if (target) {   // G64 += Xt (d1 x nr) * Yc (nr x m)
          const char* srcy = reinterpret_cast<const char*>(Yc) + (size_t)r0 * ldy * esz;
          HIPCHK(c, launch_convert_to_f32(srcy, bf16, nr, m, ldy, Ys, s));
          GemmArgs y{};
          y.M = d1; y.N = m; y.K = (int)nr; y.A = Xt; y.lda = XT_ROWS; y.B = Ys; y.ldb = m;
          y.Cin = reinterpret_cast<const float*>(G64); y.ldcin = m; y.C = G64; y.ldc = m; y.alpha = 1.0; y.beta = 1.0; y.c_is_f64 = 1;
          HIPCHK(c, launch_gemm_f64acc(y, s));
        }
      }
    }
    HIPCHK(c, hipEventRecord(c->ev_b, s));
    if (finalize) c->timers[0] += elapsed(c);
  }
  if (!finalize) return OSSCAR_OK;

  HIPCHK(c, hipEventRecord(c->ev_a, s));
  HIPCHK(c, launch_trace64(H64, d1, c->scal, s));
  double tr = 0;
  HIPCHK(c, hipMemcpyAsync(&tr, c->scal, 8, hipMemcpyDeviceToHost, s));
  HIPCHK(c, hipStreamSynchronize(s));
  c->lambda = lambda_abs + lambda_rel * tr / d1;
  HIPCHK(c, hipMemcpyAsync(c->scal + 1, &c->lambda, 8, hipMemcpyHostToDevice, s));
  HIPCHK(c, launch_finalize_H(H64, c->H, d1, c->scal + 1, s));
  HIPCHK(c, launch_convert_to_f32(W, c->desc.w_dtype == OSSCAR_BF16, d1, m, ldw, Wf, s));
  double yy = 0;
  if (target) {
    // G = X^T Y + lambda W, c0 = ||Y||^2 + lambda ||W||^2
    HIPCHK(c, launch_finalize_G(G64, Wf, c->scal + 1, c->G, (int64_t)d1 * m, s));
    HIPCHK(c, launch_dot64(Wf, Wf, (int64_t)d1 * m, c->scal + 2, c->partial, s));
    HIPCHK(c, hipMemcpyAsync(&yy, c->scal + 12, 8, hipMemcpyDeviceToHost, s));
  } else {
    // G = H W.  bf16 W: three bf16-MFMA products with the pieces of H, in the memory the float64 Gram accumulator has
    // just left; otherwise (or if that memory is too small) the float64-accumulating GEMM.
    const int64_t prow = std::min<int64_t>(PACK_ROWS, ((int64_t)d1 + 63) / 64 * 64);
    const size_t ph_bytes = align_up((size_t)prow * ((d1 + 127) / 128 * 128) * 2), pw_bytes = align_up((size_t)prow * ((m + 127) / 128 * 128) * 2);
    const size_t g64_bytes = align_up((size_t)d1 * m * 8);
    const bool split_ok = c->desc.w_dtype == OSSCAR_BF16 && (d1 % 8 == 0) && (m % 8 == 0) && (ldw % 8 == 0) &&
                          ((reinterpret_cast<uintptr_t>(W) & 15) == 0) &&
                          g64_bytes + ph_bytes + pw_bytes <= (size_t)d1 * d1 * 8;
    HIPCHK(c, hipEventRecord(c->ev_s[0][0], s));
    if (split_ok) {
      char* base = reinterpret_cast<char*>(H64);
      double* Gacc = reinterpret_cast<double*>(base);
      void* pack_h = base + g64_bytes;
      void* pack_w = base + g64_bytes + ph_bytes;
      hipLaunchKernelGGL(fill_f64_kernel, dim3(grid_for((int64_t)d1 * m)), dim3(256), 0, s, Gacc, (int64_t)d1 * m, 0.0);
      hipLaunchKernelGGL(fill_f64_kernel, dim3(1), dim3(64), 0, s, c->scal + 13, (int64_t)1, 0.0);
      HIPCHK(c, launch_hw_split(c->H, d1, W, ldw, m, Gacc, c->tiles_rect, c->n_tiles_rect, pack_h, pack_w, prow, s));
      HIPCHK(c, launch_finalize_G(Gacc, Wf, c->scal + 13, c->G, (int64_t)d1 * m, s));
    } else {
      HIPCHK(c, gemm(s, d1, m, d1, c->H, d1, Wf, m, nullptr, 0, c->G, m, 1.0, 0.0));
    }
    HIPCHK(c, hipEventRecord(c->ev_s[0][1], s));
    HIPCHK(c, launch_dot64(Wf, c->G, (int64_t)d1 * m, c->scal + 2, c->partial, s));
  }
  HIPCHK(c, launch_group_norms(Wf, c->p, c->q, m, c->norms2, s));
  c->norms_host.resize(c->p);
  HIPCHK(c, hipMemcpyAsync(&c->c0, c->scal + 2, 8, hipMemcpyDeviceToHost, s));
  HIPCHK(c, hipMemcpyAsync(c->norms_host.data(), c->norms2, c->p * 8, hipMemcpyDeviceToHost, s));
  HIPCHK(c, hipEventRecord(c->ev_b, s));
  HIPCHK(c, hipStreamSynchronize(s));
  c->have_Wdense = false;
  if (!target) {
    HIPCHK(c, hipMemcpyAsync(c->Wdense, Wf, (size_t)d1 * m * 4, hipMemcpyDeviceToDevice, s));
    HIPCHK(c, hipStreamSynchronize(s));
    c->have_Wdense = true;
  }
  if (target) c->c0 = yy + c->lambda * c->c0;
  else { float ms = 0; hipEventElapsedTime(&ms, c->ev_s[0][0], c->ev_s[0][1]); c->timers[8] = ms; }
  c->dense_is_exact = !target;
  c->timers[1] = elapsed(c);
  {   // mean duration of the Gram kernel's launches in the last chunk call that took the matrix-core path
    double tot = 0; int n = 0;
    for (int i = 0; i < c->ev_g_used; i++) {
      float ms = 0;
      if (hipEventElapsedTime(&ms, c->ev_g[2 * i], c->ev_g[2 * i + 1]) == hipSuccess) { tot += ms; n++; }
    }
    c->timers[13] = n ? tot / n : 0; c->timers[14] = n; c->timers[15] = (double)c->ev_g_rows;
    c->ev_g_used = 0;
  }
  for (auto& v : c->norms_host) v = std::sqrt(v);
  c->phase = osscar_ctx::FINAL;
  return OSSCAR_OK;
}

osscar_status osscar_gram(osscar_ctx* c, const void* Xc, int64_t n_c, int64_t ldx, int finalize, const void* W, int64_t ldw,
                          double lambda_abs, double lambda_rel) {
  return gram_impl(c, "osscar_gram", 0, Xc, nullptr, n_c, ldx, 0, finalize, W, ldw, lambda_abs, lambda_rel);
}

osscar_status osscar_gram_target(osscar_ctx* c, const void* Xc, const void* Yc, int64_t n_c, int64_t ldx, int64_t ldy, int finalize,
                                 const void* W, int64_t ldw, double lambda_abs, double lambda_rel) {
  return gram_impl(c, "osscar_gram_target", 1, Xc, Yc, n_c, ldx, ldy, finalize, W, ldw, lambda_abs, lambda_rel);
}

osscar_status osscar_gram_conv(osscar_ctx* c, const void* F, int32_t batch, int32_t channels, int32_t h_in, int32_t w_in, int32_t kh,
                               int32_t kw, int32_t stride, int32_t pad, int finalize, const void* W, int64_t ldw, double lambda_abs,
                               double lambda_rel) {
  osscar_status st = check_ctx(c);
  if (st != OSSCAR_OK) return st;
  if (batch < 0 || channels < 1 || h_in < 1 || w_in < 1 || kh < 1 || kw < 1 || stride < 1 || pad < 0 ||
      (int64_t)channels * kh * kw != c->d1 || h_in + 2 * pad < kh || w_in + 2 * pad < kw || (batch > 0 && !F))
    return fail(c, OSSCAR_EINVAL, "osscar_gram_conv: bad geometry (channels * kh * kw must equal d1 = %d)", c->d1);
  ConvSpec cs{batch, channels, h_in, w_in, kh, kw, stride, pad, (h_in + 2 * pad - kh) / stride + 1, (w_in + 2 * pad - kw) / stride + 1};
  const int64_t n_c = (int64_t)batch * cs.Hout * cs.Wout;
  return gram_impl(c, "osscar_gram_conv", 0, F, nullptr, n_c, c->d1, 0, finalize, W, ldw, lambda_abs, lambda_rel, &cs);
}

osscar_status osscar_set_quadratic(osscar_ctx* c, const float* H_dev, const float* G_dev, double c0, const double* norms) {
  osscar_status st = check_ctx(c);
  if (st != OSSCAR_OK) return st;
  if (!H_dev || !G_dev || !norms) return fail(c, OSSCAR_EINVAL, "osscar_set_quadratic: NULL argument");
  hipStream_t s = c->stream;
  HIPCHK(c, hipMemcpyAsync(c->H, H_dev, (size_t)c->d1 * c->d1 * 4, hipMemcpyDeviceToDevice, s));
  HIPCHK(c, hipMemcpyAsync(c->G, G_dev, (size_t)c->d1 * c->m * 4, hipMemcpyDeviceToDevice, s));
  HIPCHK(c, hipStreamSynchronize(s));
  c->c0 = c0; c->lambda = 0; c->dense_is_exact = false; c->have_Wdense = false;
  c->norms_host.assign(norms, norms + c->p);
  c->phase = osscar_ctx::FINAL;
  return OSSCAR_OK;
}

osscar_status osscar_init_support(osscar_ctx* c, int mode, const int32_t* groups, double* obj_host) {
  osscar_status st = check_ctx(c);
  if (st != OSSCAR_OK) return st;
  if (c->phase != osscar_ctx::FINAL && c->phase != osscar_ctx::READY)
    return fail(c, OSSCAR_ESTATE, "osscar_init_support: no quadratic form yet (call osscar_gram with finalize first)");
  c->kept_host.assign(c->p, 0);
  if (mode == OSSCAR_INIT_MAGNITUDE) {
    std::vector<int32_t> order(c->p);
    std::iota(order.begin(), order.end(), 0);
    std::stable_sort(order.begin(), order.end(), [&](int a, int b) { return c->norms_host[a] > c->norms_host[b]; });
    for (int i = 0; i < c->k; i++) c->kept_host[order[i]] = 1;
  } else if (mode == OSSCAR_INIT_GIVEN) {
    if (!groups) return fail(c, OSSCAR_EINVAL, "osscar_init_support: groups_host is NULL");
    for (int i = 0; i < c->k; i++) {
      int g = groups[i];
      if (g < 0 || g >= c->p || c->kept_host[g]) return fail(c, OSSCAR_EINVAL, "osscar_init_support: group %d out of range or repeated", g);
      c->kept_host[g] = 1;
    }
  } else {
    return fail(c, OSSCAR_EINVAL, "osscar_init_support: unknown mode %d", mode);
  }
  HIPCHK(c, hipEventRecord(c->ev_a, c->stream));
  double obj = 0;
  st = build_state(c, &obj);
  if (st != OSSCAR_OK) return st;
  SearchCtrl h{};
  h.obj = obj; h.g_out = -1; h.g_in = -1;
  HIPCHK(c, hipMemcpyAsync(c->ctrl, &h, sizeof h, hipMemcpyHostToDevice, c->stream));
  HIPCHK(c, hipEventRecord(c->ev_b, c->stream));
  HIPCHK(c, hipStreamSynchronize(c->stream));
  c->timers[2] = elapsed(c);
  if (obj_host) *obj_host = obj;
  c->phase = osscar_ctx::READY;
  return OSSCAR_OK;
}

static osscar_status read_ctrl(osscar_ctx* c, SearchCtrl* h) {
  // through pinned memory: the search waits on this copy once per 64 swaps with the device idle meanwhile
  SearchCtrl* dst = c->snap ? c->snap : h;
  HIPCHK(c, hipMemcpyAsync(dst, c->ctrl, sizeof *h, hipMemcpyDeviceToHost, c->stream));
  HIPCHK(c, hipStreamSynchronize(c->stream));
  if (dst != h) *h = *dst;
  return OSSCAR_OK;
}

osscar_status osscar_init_greedy(osscar_ctx* c, int32_t t_hat, int32_t refresh_every, uint32_t flags, int32_t* removed_host,
                                 float* gaps_host, double* obj_host) {
  osscar_status st = check_ctx(c);
  if (st != OSSCAR_OK) return st;
  if (c->phase != osscar_ctx::FINAL && c->phase != osscar_ctx::READY)
    return fail(c, OSSCAR_ESTATE, "osscar_init_greedy: no quadratic form yet (call osscar_gram with finalize first)");
  if (!c->desc.from_dense) return fail(c, OSSCAR_EINVAL, "osscar_init_greedy: the context was created without desc.from_dense");
  if (t_hat < 1 || t_hat > 64 || refresh_every < 0) return fail(c, OSSCAR_EINVAL, "osscar_init_greedy: t_hat %d outside [1, 64] or refresh_every < 0", t_hat);
  hipStream_t s = c->stream;
  const int q = c->q, k = c->k, p = c->p;
  // the loop below visits every kept-row count from d1 down to k q; whatever way this call ends, the context's counts
  // are those of the description again
  struct RestoreCounts { osscar_ctx* c; int kr, cr; ~RestoreCounts() { c->kr = kr; c->cr = cr; } } restore{c, k * q, c->d1 - k * q};
  HIPCHK(c, hipEventRecord(c->ev_a, s));
  // dense layer: every group kept
  c->kept_host.assign(p, 1);
  c->kr = c->d1; c->cr = 0;
  double obj = 0;
  st = build_state(c, &obj, (c->dense_is_exact && c->have_Wdense) ? c->Wdense : nullptr);
  if (st != OSSCAR_OK) return st;
  SearchCtrl h{};
  h.obj = c->dense_is_exact ? 0.0 : obj;   // the dense layer reproduces its own output exactly; a target output it does not
  h.g_out = -1; h.g_in = -1; h.tau = 0; h.tau_inc = 0; h.pause = 0;
  HIPCHK(c, hipMemcpyAsync(c->ctrl, &h, sizeof h, hipMemcpyHostToDevice, s));
  TabDims d = dims(c);
  TabPtrs t = ptrs(c);
  t.trace_out = c->g_removed; t.trace_in = nullptr; t.trace_gap = nullptr; t.trace_obj = nullptr;
  // groups of one row: delayed updates (the removals accumulate as pending pivots and reach N, Z by matrix products
  // once LAZY_TM of them are pending); larger groups: in-place rank-q updates
  const bool use_lazy = (q == 1) && !(flags & OSSCAR_SEARCH_EAGER);
  const LazyPtrs& L = c->lazy;
  const int la_mode = (flags & OSSCAR_SEARCH_NO_LOOKAHEAD) ? 2 : 1;
  if (use_lazy) HIPCHK(c, launch_lazy_init(d, t, L, s, la_mode));
  // Work is enqueued one batch at a time (a batch = the iterations that fit the pending set, or 256 removals in place) and
  // then checked: the delayed-update kernels may stop (pause) when a removed row was not among the rows whose products
  // were computed ahead and the spare slots ran out; the batch is then resumed after a flush from where it stopped.
  // With the products computed ahead, the rows of one iteration leave as one block pivot (four launches per iteration
  // instead of four per row; LAZY_BT rows per pivot at most); a block whose rows are not all among those products stops
  // the batch like a miss does, and the rest of its iteration is then applied row by row, which can fetch the missing
  // products.
  const bool use_block = use_lazy && la_mode == 1;
  int kept_now = p, iter = 0, since_refresh = 0, pending = 0, expected = 0;
  std::vector<int> takes;
  auto step = [&](int i) -> hipError_t {
    return use_lazy ? launch_lazy_iteration(d, t, L, 1, s, nullptr, c->g_pick + i)
                    : launch_search_iteration(d, t, -1, -1, 1, s, nullptr, c->g_pick + i);
  };
  while (kept_now > k) {
    takes.clear();
    int batch = 0, kept_b = kept_now;
    while (kept_b > k) {
      const int take = std::min<int>(t_hat, kept_b - k);
      if (use_lazy ? (pending + batch + take > LAZY_TM) : (batch >= 256)) break;
      HIPCHK(c, launch_greedy_pick(d, t, take, c->g_pick, c->g_gap + iter + (int)takes.size(), s));
      if (use_block) {
        for (int off = 0; off < take; off += LAZY_BT)      // more than LAZY_BT rows: several block pivots, same result
          HIPCHK(c, launch_lazy_block_remove(d, t, L, std::min(LAZY_BT, take - off), c->g_pick + off, s));
      } else {
        for (int i = 0; i < take; i++) HIPCHK(c, step(i));
      }
      takes.push_back(take); batch += take; kept_b -= take;
    }
    if (takes.empty()) {   // the pending set is full: apply it and try again
      HIPCHK(c, launch_lazy_flush(d, t, L, s, la_mode, side_of(c)));
      pending = 0;
      continue;
    }
    st = read_ctrl(c, &h);
    if (st != OSSCAR_OK) return st;
    if (h.notpd) return fail(c, OSSCAR_ENOTPD, "osscar_init_greedy: a pivot block lost definiteness after %d removals", h.iters);
    int done = h.iters - expected;
    if (done < 0 || done > batch) return fail(c, OSSCAR_ESTATE, "internal: osscar_init_greedy lost count of its removals");
    if (done < batch) {
      if (!use_lazy || !h.pause) return fail(c, OSSCAR_ESTATE, "internal: osscar_init_greedy stopped without a reason");
      int acc = 0, it_idx = 0;
      while (acc + takes[it_idx] <= done) { acc += takes[it_idx]; it_idx++; }
      const int off = done - acc;                       // removals of iteration it_idx already applied
      HIPCHK(c, launch_lazy_flush(d, t, L, s, la_mode, side_of(c)));       // also clears pause
      for (int i = off; i < takes[it_idx]; i++) HIPCHK(c, step(i));   // its pick list is still on the device
      pending = takes[it_idx] - off;
      batch = acc + takes[it_idx];
      iter += it_idx + 1;
    } else {
      pending += batch;
      iter += (int)takes.size();
    }
    expected += batch;
    kept_now -= batch;
    since_refresh += batch;
    const bool refresh = refresh_every > 0 && since_refresh >= refresh_every && kept_now > k;
    if (use_lazy && (refresh || kept_now == k) && pending > 0) { HIPCHK(c, launch_lazy_flush(d, t, L, s, la_mode, side_of(c))); pending = 0; }
    if (refresh) {
      st = read_kept(c);
      if (st != OSSCAR_OK) return st;
      c->kr = kept_now * q; c->cr = c->d1 - c->kr;
      st = build_state(c, &obj);
      if (st != OSSCAR_OK) return st;
      HIPCHK(c, hipMemcpyAsync(reinterpret_cast<char*>(c->ctrl) + offsetof(SearchCtrl, obj), &obj, 8, hipMemcpyHostToDevice, s));
      if (use_lazy) HIPCHK(c, launch_lazy_init(d, t, L, s, la_mode));
      since_refresh = 0;
    }
  }
  c->kr = k * q; c->cr = c->d1 - c->kr;
  st = read_ctrl(c, &h);
  if (st != OSSCAR_OK) return st;
  if (h.notpd) return fail(c, OSSCAR_ENOTPD, "osscar_init_greedy: a pivot block lost definiteness after %d removals", h.iters);
  if (h.iters != expected) return fail(c, OSSCAR_ESTATE, "internal: osscar_init_greedy applied %d of %d removals", h.iters, expected);
  st = read_kept(c);
  if (st != OSSCAR_OK) return st;
  st = upload_rows(c);
  if (st != OSSCAR_OK) return st;
  h.done = 0; h.iters = 0; h.accepted = 0;
  HIPCHK(c, hipMemcpyAsync(c->ctrl, &h, sizeof h, hipMemcpyHostToDevice, s));
  if (removed_host && p > k) HIPCHK(c, hipMemcpyAsync(removed_host, c->g_removed, (size_t)(p - k) * 4, hipMemcpyDeviceToHost, s));
  if (gaps_host && iter > 0) HIPCHK(c, hipMemcpyAsync(gaps_host, c->g_gap, (size_t)iter * 4, hipMemcpyDeviceToHost, s));
  HIPCHK(c, hipEventRecord(c->ev_b, s));
  HIPCHK(c, hipStreamSynchronize(s));
  c->timers[2] = elapsed(c);
  if (obj_host) *obj_host = h.obj;
  c->phase = osscar_ctx::READY;
  return OSSCAR_OK;
}

osscar_status osscar_local_search(osscar_ctx* c, int32_t max_swaps, double rel_tol, uint32_t flags, int32_t refresh_every,
                                  osscar_search_result* res, int32_t* t_out, int32_t* t_in, float* t_gap, double* t_obj) {
  osscar_status st = check_ctx(c);
  if (st != OSSCAR_OK) return st;
  if (c->phase != osscar_ctx::READY) return fail(c, OSSCAR_ESTATE, "osscar_local_search: call osscar_init_support first");
  if (max_swaps < 0 || max_swaps > c->desc.max_swaps || rel_tol < 0)
    return fail(c, OSSCAR_EINVAL, "osscar_local_search: max_swaps %d outside [0, desc.max_swaps = %d] or rel_tol < 0", max_swaps, c->desc.max_swaps);
  hipStream_t s = c->stream;
  SearchCtrl h{};
  st = read_ctrl(c, &h);
  if (st != OSSCAR_OK) return st;
  const double obj0 = h.obj;
  h.done = (c->cr == 0) ? 1 : 0; h.iters = 0; h.accepted = 0; h.notpd = 0; h.rel_tol = rel_tol; h.g_out = h.g_in = -1;
  h.pause = 0; h.tau = 0; h.tau_inc = 0; h.misses = 0;
  for (auto& v : c->counters) v = 0;
  HIPCHK(c, hipMemcpyAsync(c->ctrl, &h, sizeof h, hipMemcpyHostToDevice, s));
  HIPCHK(c, hipStreamSynchronize(s));
  const int always = (flags & OSSCAR_SEARCH_ALWAYS_ACCEPT) ? 1 : 0;
  TabDims d = dims(c);
  TabPtrs t = ptrs(c);
  HIPCHK(c, hipEventRecord(c->ev_a, s));
  int launched = 0, since_refresh_base = 0, samples = 0;
  double refresh_ms = 0, upd_n_ms = 0, upd_z_ms = 0;
  const int exact_in = (flags & OSSCAR_SEARCH_EXACT_IN) ? 1 : 0;      // runs on the in-place path
  const bool use_lazy = (c->q == 1) && !(flags & OSSCAR_SEARCH_EAGER) && !exact_in;
  if (use_lazy) {
    // delayed-update search: the tableau in HBM is only touched by a flush every FLUSH iterations
    const LazyPtrs& L = c->lazy;
    // The host waits once per flush interval (to read the control block); the flush and the next interval's iterations are
    // enqueued behind it without another wait, and the flush's time is read at the next wait.
    const int FLUSH = LAZY_TM / 2, BATCH = FLUSH;
    const int la_mode = (flags & OSSCAR_SEARCH_NO_LOOKAHEAD) ? 2 : 0;
    HIPCHK(c, launch_lazy_init(d, t, L, s, la_mode));
    int since_flush = 0;
    double flush_ms = 0; int flushes = 0, pauses = 0;
    bool flush_open = false;                 // a flush whose events have not been read yet
    auto collect = [&]() {                   // only after the stream has been waited for
      if (!flush_open) return;
      float ms = 0; hipEventElapsedTime(&ms, c->ev_s[0][0], c->ev_s[0][1]); flush_ms += ms; flush_open = false;
    };
    auto flush = [&]() -> osscar_status {
      HIPCHK(c, hipEventRecord(c->ev_s[0][0], s));
      HIPCHK(c, launch_lazy_flush(d, t, L, s, la_mode, side_of(c)));
      HIPCHK(c, hipEventRecord(c->ev_s[0][1], s));
      flush_open = true; flushes++;
      since_flush = 0;
      return OSSCAR_OK;
    };
    while (h.iters < max_swaps && !h.done) {
      int nb = std::min(std::min(BATCH, max_swaps - h.iters), FLUSH - since_flush);
      if (refresh_every > 0) nb = std::min(nb, std::max(1, refresh_every - (h.accepted - since_refresh_base)));
      const bool sample = samples + 1 < EV_SAMPLES;
      for (int i = 0; i < nb; i++)
        HIPCHK(c, launch_lazy_iteration(d, t, L, always, s, (i == 0 && sample) ? c->ev_s[samples + 1] : nullptr));
      const int before = h.iters;
      st = read_ctrl(c, &h);
      if (st != OSSCAR_OK) return st;
      collect();
      if (h.notpd) return fail(c, OSSCAR_ENOTPD, "osscar_local_search: a pivot lost definiteness at iteration %d", h.iters);
      since_flush += h.iters - before;
      if (sample && h.iters > before) {
        float a = 0, b = 0;
        hipEventElapsedTime(&a, c->ev_s[samples + 1][0], c->ev_s[samples + 1][1]);
        hipEventElapsedTime(&b, c->ev_s[samples + 1][0], c->ev_s[samples + 1][2]);
        upd_n_ms += a; upd_z_ms += b; samples++;
      }
      const bool want_refresh = !h.done && refresh_every > 0 && h.accepted - since_refresh_base >= refresh_every && h.iters < max_swaps;
      if (h.pause) pauses++;
      if (h.pause || since_flush >= FLUSH || h.done || want_refresh || h.iters >= max_swaps) {
        if (h.tau + h.tau_inc > 0 || h.pause) { st = flush(); if (st != OSSCAR_OK) return st; }
        h.pause = 0; h.tau = 0; h.tau_inc = 0;
      }
      if (want_refresh) {
        if (flush_open) { HIPCHK(c, hipStreamSynchronize(s)); collect(); }      // the refresh times itself with the same events
        hipEvent_t r0 = c->ev_s[0][0], r1 = c->ev_s[0][1];
        HIPCHK(c, hipEventRecord(r0, s));
        st = read_kept(c);
        if (st != OSSCAR_OK) return st;
        double obj = 0;
        st = build_state(c, &obj);
        if (st != OSSCAR_OK) return st;
        HIPCHK(c, hipMemcpyAsync(reinterpret_cast<char*>(c->ctrl) + offsetof(SearchCtrl, obj), &obj, 8, hipMemcpyHostToDevice, s));
        HIPCHK(c, launch_lazy_init(d, t, L, s, la_mode));     // selection records and look-ahead products of the rebuilt state
        HIPCHK(c, hipEventRecord(r1, s));
        HIPCHK(c, hipStreamSynchronize(s));
        float ms = 0; hipEventElapsedTime(&ms, r0, r1); refresh_ms += ms;
        since_refresh_base = h.accepted;
        h.obj = obj;
      }
    }
    if (h.tau + h.tau_inc > 0) { st = flush(); if (st != OSSCAR_OK) return st; }
    if (flush_open) { HIPCHK(c, hipStreamSynchronize(s)); collect(); }
    c->timers[6] = refresh_ms + flush_ms;
    c->counters[0] = flushes; c->counters[1] = pauses; c->counters[2] = h.misses; c->counters[3] = h.iters;
  } else {
  const int BATCH = 32;
  while (launched < max_swaps && !h.done) {
    int nb = std::min(BATCH, max_swaps - launched);
    if (refresh_every > 0) nb = std::min(nb, std::max(1, refresh_every - (h.accepted - since_refresh_base)));
    const bool sample = samples + 1 < EV_SAMPLES;
    for (int i = 0; i < nb; i++) {
      HIPCHK(c, launch_search_iteration(d, t, -1, -1, always, s, (i == 0 && sample) ? c->ev_s[samples + 1] : nullptr, nullptr,
                                        exact_in));
    }
    launched += nb;
    st = read_ctrl(c, &h);
    if (st != OSSCAR_OK) return st;
    if (sample) {   // the sampled iteration ran its updates unless the search had already stopped before it
      float a = 0, b = 0;
      hipEventElapsedTime(&a, c->ev_s[samples + 1][0], c->ev_s[samples + 1][1]);
      hipEventElapsedTime(&b, c->ev_s[samples + 1][1], c->ev_s[samples + 1][2]);
      upd_n_ms += a; upd_z_ms += b; samples++;
    }
    if (h.notpd) return fail(c, OSSCAR_ENOTPD, "osscar_local_search: a pivot block lost definiteness at iteration %d", h.iters);
    if (!h.done && refresh_every > 0 && h.accepted - since_refresh_base >= refresh_every && launched < max_swaps) {
      hipEvent_t r0 = c->ev_s[0][0], r1 = c->ev_s[0][1];
      HIPCHK(c, hipEventRecord(r0, s));
      st = read_kept(c);
      if (st != OSSCAR_OK) return st;
      double obj = 0;
      st = build_state(c, &obj);
      if (st != OSSCAR_OK) return st;
      HIPCHK(c, hipMemcpyAsync(reinterpret_cast<char*>(c->ctrl) + offsetof(SearchCtrl, obj), &obj, 8, hipMemcpyHostToDevice, s));
      HIPCHK(c, hipEventRecord(r1, s));
      HIPCHK(c, hipStreamSynchronize(s));
      float ms = 0; hipEventElapsedTime(&ms, r0, r1); refresh_ms += ms;
      since_refresh_base = h.accepted;
      h.obj = obj;
    }
  }
  c->timers[6] = refresh_ms;
  }
  HIPCHK(c, hipEventRecord(c->ev_b, s));
  st = read_ctrl(c, &h);
  if (st != OSSCAR_OK) return st;
  c->timers[3] = elapsed(c);
  c->timers[5] = samples ? upd_n_ms / samples : 0;
  c->timers[7] = samples ? upd_z_ms / samples : 0;
  if (res) { res->iters = h.iters; res->accepted = h.accepted; res->obj_initial = obj0; res->obj_final = h.obj; }
  const int n = h.iters;
  if (n > 0) {
    if (t_out) HIPCHK(c, hipMemcpyAsync(t_out, c->trace_out, n * 4, hipMemcpyDeviceToHost, s));
    if (t_in) HIPCHK(c, hipMemcpyAsync(t_in, c->trace_in, n * 4, hipMemcpyDeviceToHost, s));
    if (t_gap) HIPCHK(c, hipMemcpyAsync(t_gap, c->trace_gap, n * 8, hipMemcpyDeviceToHost, s));
    if (t_obj) HIPCHK(c, hipMemcpyAsync(t_obj, c->trace_obj, n * 8, hipMemcpyDeviceToHost, s));
    HIPCHK(c, hipStreamSynchronize(s));
  }
  return OSSCAR_OK;
}

osscar_status osscar_block_search(osscar_ctx* c, int32_t max_iters, int32_t block, double rel_tol, uint32_t flags,
                                  osscar_search_result* res, int32_t* t_out, int32_t* t_in, float* t_gap, double* t_obj) {
  osscar_status st = check_ctx(c);
  if (st != OSSCAR_OK) return st;
  if (c->phase != osscar_ctx::READY) return fail(c, OSSCAR_ESTATE, "osscar_block_search: call osscar_init_support first");
  if (max_iters < 0 || block < 1 || block > 64 || rel_tol < 0)
    return fail(c, OSSCAR_EINVAL, "osscar_block_search: max_iters %d < 0, block %d outside [1, 64] or rel_tol < 0", max_iters, block);
  hipStream_t s = c->stream;
  SearchCtrl h{};
  st = read_ctrl(c, &h);
  if (st != OSSCAR_OK) return st;
  const double obj0 = h.obj;
  h.done = 0; h.iters = 0; h.accepted = 0; h.notpd = 0; h.rel_tol = rel_tol; h.g_out = h.g_in = -1; h.pause = 0; h.tau = 0; h.tau_inc = 0;
  HIPCHK(c, hipMemcpyAsync(c->ctrl, &h, sizeof h, hipMemcpyHostToDevice, s));
  HIPCHK(c, hipStreamSynchronize(s));
  const bool always = (flags & OSSCAR_SEARCH_ALWAYS_ACCEPT) != 0;
  const bool use_lazy = (c->q == 1) && !(flags & OSSCAR_SEARCH_EAGER);
  const int la_mode = (flags & OSSCAR_SEARCH_NO_LOOKAHEAD) ? 2 : 0;
  const int take = std::min<int>(block, std::min(c->k, c->p - c->k));
  TabDims d = dims(c);
  TabPtrs t = ptrs(c);
  t.trace_out = nullptr; t.trace_in = nullptr; t.trace_gap = nullptr; t.trace_obj = nullptr;   // pairs are recorded on the host
  const LazyPtrs& L = c->lazy;
  HIPCHK(c, hipEventRecord(c->ev_a, s));
  if (use_lazy) HIPCHK(c, launch_lazy_init(d, t, L, s, la_mode));
  int pending = 0, done_pairs = 0, blocks = 0, accepted = 0;
  // applies the pairs one after the other (each unconditionally); resumes after a flush when the kernels had to stop
  auto run_pairs = [&](const std::vector<int32_t>& out, const std::vector<int32_t>& inn) -> osscar_status {
    size_t idx = 0;
    while (idx < out.size()) {
      for (size_t r = idx; r < out.size(); r++) {
        if (use_lazy) HIPCHK(c, launch_lazy_iteration(d, t, L, 1, s, nullptr, nullptr, out[r], inn[r]));
        else HIPCHK(c, launch_search_iteration(d, t, out[r], inn[r], 1, s));
      }
      osscar_status q = read_ctrl(c, &h);
      if (q != OSSCAR_OK) return q;
      if (h.notpd) return fail(c, OSSCAR_ENOTPD, "osscar_block_search: a pivot lost definiteness in move %d", blocks);
      const int did = h.iters - done_pairs;
      if (did < 0 || did > (int)(out.size() - idx)) return fail(c, OSSCAR_ESTATE, "internal: osscar_block_search lost count of its pairs");
      done_pairs += did; idx += did; pending += 2 * did;
      if (idx < out.size()) {
        if (!use_lazy || !h.pause) return fail(c, OSSCAR_ESTATE, "internal: osscar_block_search stopped without a reason");
        HIPCHK(c, launch_lazy_flush(d, t, L, s, la_mode, side_of(c)));
        pending = 0;
      }
    }
    return OSSCAR_OK;
  };
  std::vector<int32_t> out(take), inn(take);
  float gaps[2] = {0, 0};
  while (take > 0 && blocks < max_iters) {
    if (use_lazy && pending + 2 * take > LAZY_TM) { HIPCHK(c, launch_lazy_flush(d, t, L, s, la_mode, side_of(c))); pending = 0; }
    HIPCHK(c, launch_greedy_pick(d, t, take, c->g_pick, c->g_gap, s, 0));
    HIPCHK(c, launch_greedy_pick(d, t, take, c->g_pick + 64, c->g_gap + 1, s, 1));
    HIPCHK(c, hipMemcpyAsync(out.data(), c->g_pick, (size_t)take * 4, hipMemcpyDeviceToHost, s));
    HIPCHK(c, hipMemcpyAsync(inn.data(), c->g_pick + 64, (size_t)take * 4, hipMemcpyDeviceToHost, s));
    HIPCHK(c, hipMemcpyAsync(gaps, c->g_gap, 8, hipMemcpyDeviceToHost, s));
    HIPCHK(c, hipStreamSynchronize(s));
    const double obj_before = h.obj;
    st = run_pairs(out, inn);
    if (st != OSSCAR_OK) return st;
    const double delta = h.obj - obj_before;
    const bool ok = always || delta < -rel_tol * obj_before;
    if (t_out) std::copy(out.begin(), out.end(), t_out + (size_t)blocks * block);
    if (t_in) std::copy(inn.begin(), inn.end(), t_in + (size_t)blocks * block);
    if (t_out) std::fill(t_out + (size_t)blocks * block + take, t_out + (size_t)(blocks + 1) * block, -1);
    if (t_in) std::fill(t_in + (size_t)blocks * block + take, t_in + (size_t)(blocks + 1) * block, -1);
    if (t_gap) { t_gap[2 * blocks] = gaps[0]; t_gap[2 * blocks + 1] = gaps[1]; }
    if (t_obj) t_obj[blocks] = ok ? h.obj : obj_before;
    blocks++;
    if (!ok) {
      // take the move back: the same pairs in reverse (the pending pivots must reach the tableau first)
      if (use_lazy && pending > 0) { HIPCHK(c, launch_lazy_flush(d, t, L, s, la_mode, side_of(c))); pending = 0; }
      std::vector<int32_t> bo(inn.rbegin(), inn.rend()), bi(out.rbegin(), out.rend());
      st = run_pairs(bo, bi);
      if (st != OSSCAR_OK) return st;
      h.obj = obj_before;
      HIPCHK(c, hipMemcpyAsync(reinterpret_cast<char*>(c->ctrl) + offsetof(SearchCtrl, obj), &h.obj, 8, hipMemcpyHostToDevice, s));
      break;
    }
    accepted++;
  }
  if (use_lazy && pending > 0) HIPCHK(c, launch_lazy_flush(d, t, L, s, la_mode, side_of(c)));
  HIPCHK(c, hipEventRecord(c->ev_b, s));
  HIPCHK(c, hipStreamSynchronize(s));
  c->timers[3] = elapsed(c);
  if (res) { res->iters = blocks; res->accepted = accepted; res->obj_initial = obj0; res->obj_final = h.obj; }
  return OSSCAR_OK;
}

osscar_status osscar_apply_swap(osscar_ctx* c, int32_t g_out, int32_t g_in) {
  osscar_status st = check_ctx(c);
  if (st != OSSCAR_OK) return st;
  if (c->phase != osscar_ctx::READY) return fail(c, OSSCAR_ESTATE, "osscar_apply_swap: call osscar_init_support first");
  if (g_out < 0 || g_out >= c->p || g_in < 0 || g_in >= c->p) return fail(c, OSSCAR_EINVAL, "osscar_apply_swap: group out of range");
  st = read_kept(c);
  if (st != OSSCAR_OK) return st;
  if (!c->kept_host[g_out] || c->kept_host[g_in]) return fail(c, OSSCAR_EINVAL, "osscar_apply_swap: %d must be kept and %d must not", g_out, g_in);
  SearchCtrl h{};
  st = read_ctrl(c, &h);
  if (st != OSSCAR_OK) return st;
  h.done = 0; h.iters = 0; h.notpd = 0; h.pause = 0; h.tau = 0; h.tau_inc = 0;
  HIPCHK(c, hipMemcpyAsync(c->ctrl, &h, sizeof h, hipMemcpyHostToDevice, c->stream));
  HIPCHK(c, hipStreamSynchronize(c->stream));
  TabPtrs t = ptrs(c);
  t.trace_out = nullptr;
  HIPCHK(c, launch_search_iteration(dims(c), t, g_out, g_in, 1, c->stream));
  st = read_ctrl(c, &h);
  if (st != OSSCAR_OK) return st;
  if (h.notpd) return fail(c, OSSCAR_ENOTPD, "osscar_apply_swap: pivot block not definite");
  return OSSCAR_OK;
}

osscar_status osscar_backsolve(osscar_ctx* c, void* What, int64_t ldw_hat, int32_t out_dtype, int32_t* support, double* obj_host) {
  osscar_status st = check_ctx(c);
  if (st != OSSCAR_OK) return st;
  if (c->phase != osscar_ctx::READY) return fail(c, OSSCAR_ESTATE, "osscar_backsolve: call osscar_init_support first");
  if (!What || ldw_hat < c->m || (out_dtype != OSSCAR_F32 && out_dtype != OSSCAR_BF16))
    return fail(c, OSSCAR_EINVAL, "osscar_backsolve: bad output buffer");
  hipStream_t s = c->stream;
  HIPCHK(c, hipEventRecord(c->ev_a, s));
  st = read_kept(c);
  if (st != OSSCAR_OK) return st;
  st = upload_rows(c);
  if (st != OSSCAR_OK) return st;
  Carve cv(c->scratch);
  InvBufs b = carve_inv(c, cv);
  SplitBufs sp = carve_split(c, cv);
  I8Bufs ib = carve_i8(c, cv);      // for the state build of the fallback below
  if (cv.off > c->scratch_bytes) return fail(c, OSSCAR_ENOMEM, "internal: scratch carve-up exceeds the workspace");
  const bool split = split_ok(c);
  if (split) b.sp = &sp;
  b.i8 = &ib;
  // Refine the maintained weights instead of refactorising: B <- B + P (G_K - H_KK B) with the maintained inverse P
  // and a float64-accumulated residual.  One step shrinks the error by |I - P H_KK| (about 1e-3 after thousands of
  // swaps, so after a correction of relative size r the error left is about 1e-3 r); a second step is taken if the
  // first correction was not small, and a fresh inverse if it was large.
  {
    const int kr = c->kr, m = c->m;
    HIPCHK(c, launch_gather(c->H, c->d1, c->rowsK, kr, c->rowsK, kr, b.HKK, kr, s));
    HIPCHK(c, launch_i8_kexp(b.HKK, kr, kr, ib.kexp, s));
    HIPCHK(c, launch_gather(c->G, m, c->rowsK, kr, nullptr, m, b.GK, m, s));
    hipLaunchKernelGGL(gather_sym_kernel, dim3(grid_for((int64_t)kr * kr)), dim3(256), 0, s, c->N, (int64_t)c->d1, c->rowsK, kr,
                       c->rowsK, kr, b.P, -1.f);
    HIPCHK(c, launch_gather(c->Z, m, c->rowsK, kr, nullptr, m, b.B, m, s));
    TileRef t_b{};
    if (split) {
      if ((st = stage_tiles(c, 1, kr, m, false, &t_b)) != OSSCAR_OK) return st;
      if ((st = pack_into(c, sp, sp.packP, b.P, kr, kr, kr)) != OSSCAR_OK) return st;
    }
    bool ok = false;
    for (int step = 0; step < 3 && !ok; step++) {
      // residual, sums exact: H_KK levelled along k and the weights B have no entries far below their row / column maxima,
      // so the int8 digits carry both operands whole (unlike a residual that involves P)
      HIPCHK(c, big_gemm(s, b.i8, kr, m, kr, b.HKK, kr, b.B, m, b.GK, m, b.T4, m, -1.0, 1.0, 0.0, 0, 0, 0, -1));
      // the correction is small, a few digits of it are enough: float32 accumulation, or the three leading products of
      // the bf16 pieces
      if (split) {
        if ((st = pack_into(c, sp, sp.packX, b.T4, m, kr, m)) != OSSCAR_OK) return st;
        if ((st = split_gemm(c, sp, sp.packP, kr, sp.packX, m, kr, 3, t_b, nullptr, 0, b.T3, m, 1.0, 0.0)) != OSSCAR_OK) return st;
      } else {
        HIPCHK(c, gemm(s, kr, m, kr, b.P, kr, b.T4, m, nullptr, 0, b.T3, m, 1.0, 0.0, 0.0, 0, 0, 1));
      }
      HIPCHK(c, launch_dot64(b.T3, b.T3, (int64_t)kr * m, c->scal + 9, c->partial, s));
      HIPCHK(c, launch_dot64(b.B, b.B, (int64_t)kr * m, c->scal + 10, c->partial + 1024, s));
      hipLaunchKernelGGL(add_inplace_kernel, dim3(grid_for((int64_t)kr * m)), dim3(256), 0, s, b.B, b.T3, (int64_t)kr * m);
      double nn[2] = {0, 0};
      HIPCHK(c, hipMemcpyAsync(nn, c->scal + 9, 16, hipMemcpyDeviceToHost, s));
      HIPCHK(c, hipStreamSynchronize(s));
      const double ratio = std::sqrt(nn[0] / std::max(nn[1], 1e-300));
      if (!(ratio < 1e-2)) break;             // the maintained inverse is not good enough: refactorise
      if (ratio < 1e-4) ok = true;            // what is left is ratio * |I - P H_KK| <= 1e-6: below the float32 storage of B
    }
    if (!ok) {
      st = inverse_and_weights(c, b);
      if (st != OSSCAR_OK) return st;
    }
  }
  HIPCHK(c, launch_fill_rows_zero(What, ldw_hat, c->d1, c->m, out_dtype == OSSCAR_BF16, s));
  HIPCHK(c, launch_scatter_rows(b.B, c->m, c->rowsK, c->kr, c->m, What, ldw_hat, out_dtype == OSSCAR_BF16, s));
  double obj = 0;
  st = objective_from(c, b.GK, b.B, &obj);
  if (st != OSSCAR_OK) return st;
  HIPCHK(c, hipEventRecord(c->ev_b, s));
  HIPCHK(c, hipStreamSynchronize(s));
  c->timers[4] = elapsed(c);
  if (obj_host) *obj_host = obj;
  if (support) {
    int n = 0;
    for (int g = 0; g < c->p; g++) if (c->kept_host[g]) support[n++] = g;
  }
  return OSSCAR_OK;
}

osscar_status osscar_get_tensor(osscar_ctx* c, int which, void* dst, size_t dst_bytes) {
  osscar_status st = check_ctx(c);
  if (st != OSSCAR_OK) return st;
  if (!dst) return fail(c, OSSCAR_EINVAL, "osscar_get_tensor: NULL destination");
  hipStream_t s = c->stream;
  const int64_t d1 = c->d1, m = c->m, kr = c->kr, cr = c->cr;
  auto need = [&](size_t b) { return dst_bytes >= b; };
  if (which == OSSCAR_T_H || which == OSSCAR_T_G) {
    if (c->phase != osscar_ctx::FINAL && c->phase != osscar_ctx::READY) return fail(c, OSSCAR_ESTATE, "no quadratic form yet");
    size_t b = (which == OSSCAR_T_H ? d1 * d1 : d1 * m) * 4;
    if (!need(b)) return fail(c, OSSCAR_EINVAL, "osscar_get_tensor: destination too small");
    HIPCHK(c, hipMemcpyAsync(dst, which == OSSCAR_T_H ? c->H : c->G, b, hipMemcpyDeviceToDevice, s));
    HIPCHK(c, hipStreamSynchronize(s));
    return OSSCAR_OK;
  }
  if (c->phase != osscar_ctx::READY) return fail(c, OSSCAR_ESTATE, "osscar_get_tensor: no search state yet");
  st = read_kept(c);
  if (st != OSSCAR_OK) return st;
  if (which == OSSCAR_T_REM || which == OSSCAR_T_ADD) {
    if (!need((size_t)c->p * 8)) return fail(c, OSSCAR_EINVAL, "osscar_get_tensor: destination too small");
    std::vector<double> sc(c->p);
    HIPCHK(c, hipMemcpyAsync(sc.data(), c->score, c->p * 8, hipMemcpyDeviceToHost, s));
    HIPCHK(c, hipStreamSynchronize(s));
    for (int g = 0; g < c->p; g++) {
      if (which == OSSCAR_T_REM && !c->kept_host[g]) sc[g] = INFINITY;
      if (which == OSSCAR_T_ADD && c->kept_host[g]) sc[g] = -INFINITY;
    }
    HIPCHK(c, hipMemcpy(dst, sc.data(), c->p * 8, hipMemcpyHostToDevice));
    return OSSCAR_OK;
  }
  if (which == OSSCAR_T_KEPT_SLOTS || which == OSSCAR_T_CAND_SLOTS) {
    std::vector<int32_t> ids;
    for (int g = 0; g < c->p; g++) if ((c->kept_host[g] != 0) == (which == OSSCAR_T_KEPT_SLOTS)) ids.push_back(g);
    if (!need(ids.size() * 4)) return fail(c, OSSCAR_EINVAL, "osscar_get_tensor: destination too small");
    if (!ids.empty()) HIPCHK(c, hipMemcpy(dst, ids.data(), ids.size() * 4, hipMemcpyHostToDevice));
    return OSSCAR_OK;
  }
  st = upload_rows(c);
  if (st != OSSCAR_OK) return st;
  float* out = reinterpret_cast<float*>(dst);
  switch (which) {
    case OSSCAR_T_P:
      if (!need(kr * kr * 4)) return fail(c, OSSCAR_EINVAL, "osscar_get_tensor: destination too small");
      hipLaunchKernelGGL(gather_sym_kernel, dim3(grid_for(kr * kr)), dim3(256), 0, s, c->N, d1, c->rowsK, (int)kr, c->rowsK, (int)kr, out, -1.f);
      break;
    case OSSCAR_T_V:
      if (!need(kr * cr * 4)) return fail(c, OSSCAR_EINVAL, "osscar_get_tensor: destination too small");
      if (cr > 0) hipLaunchKernelGGL(gather_sym_kernel, dim3(grid_for(kr * cr)), dim3(256), 0, s, c->N, d1, c->rowsK, (int)kr, c->rowsC, (int)cr, out, 1.f);
      break;
    case OSSCAR_T_B:
      if (!need(kr * m * 4)) return fail(c, OSSCAR_EINVAL, "osscar_get_tensor: destination too small");
      HIPCHK(c, launch_gather(c->Z, m, c->rowsK, (int)kr, nullptr, (int)m, out, m, s));
      break;
    case OSSCAR_T_R:
      if (!need(cr * m * 4)) return fail(c, OSSCAR_EINVAL, "osscar_get_tensor: destination too small");
      if (cr > 0) HIPCHK(c, launch_gather(c->Z, m, c->rowsC, (int)cr, nullptr, (int)m, out, m, s));
      break;
    default:
      return fail(c, OSSCAR_EINVAL, "osscar_get_tensor: unknown tensor id %d", which);
  }
  HIPCHK(c, hipGetLastError());
  HIPCHK(c, hipStreamSynchronize(s));
  return OSSCAR_OK;
}

osscar_status osscar_get_scalars(osscar_ctx* c, double* lambda_host, double* c0_host) {
  if (!c) return OSSCAR_EINVAL;
  if (lambda_host) *lambda_host = c->lambda;
  if (c0_host) *c0_host = c->c0;
  return OSSCAR_OK;
}

int32_t osscar_debug_tile_schedule(int64_t d1, int32_t* out_host, int32_t capacity) {
  if (d1 <= 0 || d1 > 65536) return -1;
  return gram_tile_schedule((int)((d1 + 127) / 128), out_host, capacity);
}

osscar_status osscar_debug_gemm_log(int32_t enable) { gemm_log_enable(enable); return OSSCAR_OK; }
osscar_status osscar_debug_int_products(int32_t enable) { g_i8_products = enable != 0; return OSSCAR_OK; }
osscar_status osscar_debug_refined_inverse(int32_t enable) { g_refined_inverse = enable != 0; return OSSCAR_OK; }
osscar_status osscar_debug_side_stream(int32_t enable) { g_side_stream = enable != 0; return OSSCAR_OK; }
int32_t osscar_debug_gemm_log_read(double* out_host, int32_t capacity) {
  if (!out_host || capacity < 0) return -1;
  return gemm_log_read(out_host, capacity);
}

osscar_status osscar_get_counters(osscar_ctx* c, int64_t* out) {
  if (!c || !out) return OSSCAR_EINVAL;
  for (int i = 0; i < 8; i++) out[i] = c->counters[i];
  return OSSCAR_OK;
}

osscar_status osscar_get_timers(osscar_ctx* c, double* out) {
  if (!c || !out) return OSSCAR_EINVAL;
  for (int i = 0; i < 16; i++) out[i] = c->timers[i];
  return OSSCAR_OK;
}

}  // extern "C"
