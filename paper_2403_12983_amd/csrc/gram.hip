// Quadratic-form construction (Section 3, dense-layer paragraph): H = X^T X accumulated over chunks of
// calibration rows, then the ridge, G = H W and c0.
//
// gram_pack_kernel + gram_packed_kernel: SYRK-style product on the lower-triangle tiles of H with
//   v_mfma_f32_32x32x16_bf16.  Both MFMA operands are column panels of the same row-major chunk Xc (rows =
//   tokens), so every lane needs 8 consecutive TOKENS of one column in a register quad: the chunk is first
//   rewritten once into that order (8 x 8 register transposes, HBM-bound, a few percent of the product's
//   time), and the product kernel then only copies contiguous blocks into LDS and issues MFMAs.
//   Tile order: the host lays the tiles out so that the workgroups that run together on one XCD (block
//   index modulo 8) form 4 x 8 blocks of tiles sharing their 12 column panels in that XCD's L2, and deals
//   the strips of tile rows to the XCDs in alternating direction so that all eight get equal work.
#include "internal.h"
#include <cstdlib>
#include <vector>

namespace osscar {

typedef float f16v __attribute__((ext_vector_type(16)));
typedef __bf16 bf8 __attribute__((ext_vector_type(8)));

constexpr int GBK = 64;            // tokens per LDS stage

// Tile order: strips of 4 tile rows are dealt to the 8 XCDs (block index modulo 8 selects the XCD), largest strip first to
// the XCD with the least work so far, so that all eight finish together; within a strip the tiles are walked in 4 x 8
// blocks.  Lists are padded with (-1, -1) to equal length.
static void build_tile_list(int tm_count, std::vector<int2>& out) {
  constexpr int NX = 8, RB = 4, CB = 8;
  std::vector<std::vector<int2>> lists(NX);
  const int strips = (tm_count + RB - 1) / RB;
  std::vector<int> owner(strips, 0);
  std::vector<long> load(NX, 0);
  for (int sidx = strips - 1; sidx >= 0; sidx--) {            // strips grow with the row index: last = largest
    const int r0 = sidx * RB, r1 = std::min(tm_count, r0 + RB);
    long tiles = 0;
    for (int r = r0; r < r1; r++) tiles += r + 1;
    int best = 0;
    for (int x = 1; x < NX; x++) if (load[x] < load[best]) best = x;
    owner[sidx] = best; load[best] += tiles;
  }
  for (int sidx = 0; sidx < strips; sidx++) {
    std::vector<int2>& L = lists[owner[sidx]];
    int r0 = sidx * RB, r1 = std::min(tm_count, r0 + RB);
    for (int c0 = 0; c0 < r1; c0 += CB)
      for (int r = r0; r < r1; r++)
        for (int c = c0; c < c0 + CB && c <= r; c++) L.push_back(int2{r, c});
  }
  size_t len = 0;
  for (auto& L : lists) len = std::max(len, L.size());
  out.assign(len * NX, int2{-1, -1});
  for (int x = 0; x < NX; x++)
    for (size_t i = 0; i < lists[x].size(); i++) out[i * NX + x] = lists[x][i];
}

// ------------------------------------------------------------------------------------------------
// gram_pack_kernel rewrites a chunk of X once into the operand format of the MFMA: for every stage
// (64 tokens) and every panel (128 columns) one contiguous 16 KB block of 16-byte packets, packet (kg, c) = the 8
// tokens kg*8..kg*8+7 of column c, at slot kg*128 + c.  Tokens past the chunk and columns past d1 are zero.
// gram_packed_kernel then copies whole blocks global -> LDS (linear, no transposes or masks in the hot loop) and
// reads MFMA operands as single ds_read_b128: 16 neighbouring lanes read 16 neighbouring packets.
// Accuracy: the MFMA accumulators are added (v_add_f32, round to nearest) to a second float32 register set every
// `window` stages and restarted from zero, so the accumulation inside the matrix core never spans more than
// window*64 tokens; the second set is added to the float64 H once per launch.
// ------------------------------------------------------------------------------------------------
constexpr int PK_SLOTS = 8 * 128;   // packets per (stage, panel)

__global__ __launch_bounds__(256) void gram_pack_kernel(const uint16_t* __restrict__ X, int64_t n_c, int64_t ldx, int d1,
                                                         int npanels, uint4* __restrict__ Xp) {
  const int tid = threadIdx.x;
  const int panel = blockIdx.x * 2 + (tid >> 7);
  if (panel >= npanels) return;
  const int kg = (tid & 127) >> 4, cg = tid & 15;
  const int col = panel * 128 + cg * 8;
  const bool live = col < d1;
  const int64_t row0 = (int64_t)blockIdx.y * GBK + kg * 8;
  const uint16_t* src = X + (live ? col : 0);
  uint4 st[8];
#pragma unroll
  for (int r = 0; r < 8; r++) {
    const int64_t row = row0 + r;
    const int64_t rowc = row < n_c ? row : n_c - 1;
    st[r] = *reinterpret_cast<const uint4*>(src + rowc * ldx);
  }
#pragma unroll
  for (int r = 0; r < 8; r++)
    if (!live || row0 + r >= n_c) st[r] = uint4{0u, 0u, 0u, 0u};
  uint4* out = Xp + ((int64_t)blockIdx.y * npanels + panel) * PK_SLOTS + kg * 128 + cg * 8;
#define OSSCAR_PACK_LO(F) uint4{(st[0].F & 0xFFFFu) | (st[1].F << 16), (st[2].F & 0xFFFFu) | (st[3].F << 16), \
                                (st[4].F & 0xFFFFu) | (st[5].F << 16), (st[6].F & 0xFFFFu) | (st[7].F << 16)}
#define OSSCAR_PACK_HI(F) uint4{(st[0].F >> 16) | (st[1].F & 0xFFFF0000u), (st[2].F >> 16) | (st[3].F & 0xFFFF0000u), \
                                (st[4].F >> 16) | (st[5].F & 0xFFFF0000u), (st[6].F >> 16) | (st[7].F & 0xFFFF0000u)}
  out[0] = OSSCAR_PACK_LO(x); out[1] = OSSCAR_PACK_HI(x);
  out[2] = OSSCAR_PACK_LO(y); out[3] = OSSCAR_PACK_HI(y);
  out[4] = OSSCAR_PACK_LO(z); out[5] = OSSCAR_PACK_HI(z);
  out[6] = OSSCAR_PACK_LO(w); out[7] = OSSCAR_PACK_HI(w);
#undef OSSCAR_PACK_LO
#undef OSSCAR_PACK_HI
}

// The same repacking for a convolutional layer: the 8 x 8 blocks are gathered from the feature map, patch by patch.
__global__ __launch_bounds__(256) void gram_pack_conv_kernel(const uint16_t* __restrict__ F, ConvSpec cs, int64_t r0, int64_t n_c,
                                                              int d1, int npanels, uint4* __restrict__ Xp) {
  const int tid = threadIdx.x;
  const int panel = blockIdx.x * 2 + (tid >> 7);
  if (panel >= npanels) return;
  const int kg = (tid & 127) >> 4, cg = tid & 15;
  const int col0 = panel * 128 + cg * 8;
  const int64_t row0 = (int64_t)blockIdx.y * GBK + kg * 8;
  const int kk = cs.kh * cs.kw;
  uint32_t v[8][4];                       // v[j][r/2]: rows r, r+1 of column j
#pragma unroll
  for (int j = 0; j < 8; j++)
#pragma unroll
    for (int h = 0; h < 4; h++) v[j][h] = 0u;
#pragma unroll
  for (int r = 0; r < 8; r++) {
    const int64_t row = row0 + r;
    if (row >= n_c) continue;
    const int64_t pr = r0 + row;
    const int ox = (int)(pr % cs.Wout), oy = (int)((pr / cs.Wout) % cs.Hout), b = (int)(pr / ((int64_t)cs.Wout * cs.Hout));
#pragma unroll
    for (int j = 0; j < 8; j++) {
      const int col = col0 + j;
      if (col >= d1) continue;
      const int c = col / kk, dy = (col % kk) / cs.kw, dx = col % cs.kw;
      const int y = oy * cs.stride + dy - cs.pad, x = ox * cs.stride + dx - cs.pad;
      if (y < 0 || y >= cs.Hin || x < 0 || x >= cs.Win) continue;
      const uint32_t e = F[(((int64_t)b * cs.C + c) * cs.Hin + y) * cs.Win + x];
      v[j][r >> 1] |= (r & 1) ? (e << 16) : e;
    }
  }
  uint4* out = Xp + ((int64_t)blockIdx.y * npanels + panel) * PK_SLOTS + kg * 128 + cg * 8;
#pragma unroll
  for (int j = 0; j < 8; j++) out[j] = uint4{v[j][0], v[j][1], v[j][2], v[j][3]};
}

// Out (+)= A^T B for packed operands Ap (rows of the result) and Bp (columns of the result); symmetric: Ap == Bp and only
// tiles on or below the diagonal are listed, the diagonal ones loading one panel.
__global__ __launch_bounds__(256, 2) __attribute__((amdgpu_waves_per_eu(2, 2))) void gram_packed_kernel(
    const uint4* __restrict__ Ap, int64_t a_sstride, const uint4* __restrict__ Bp, int64_t b_sstride, int nstages, int rows_out,
    int cols_out, int ldo, double* __restrict__ H64, const int2* __restrict__ tile_list, int stages_per_split, int window,
    int symmetric, int split) {
  constexpr int WT = 2, TS = 128;
  extern __shared__ uint4 lds[];             // [2 buffers][2 panels][PK_SLOTS]
  const int2 tile = tile_list[blockIdx.x];
  if (tile.x < 0) return;
  const int tm = tile.x, tn = tile.y;
  const bool diag = symmetric && (tm == tn);
  const int i0 = tm * TS, j0 = tn * TS;
  const int s_begin = split * stages_per_split;
  const int s_end = (s_begin + stages_per_split < nstages) ? s_begin + stages_per_split : nstages;
  if (s_begin >= s_end) return;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;

  f16v acc[WT][WT], acc2[WT][WT];
#pragma unroll
  for (int a = 0; a < WT; a++)
#pragma unroll
    for (int b = 0; b < WT; b++)
#pragma unroll
      for (int r = 0; r < 16; r++) { acc[a][b][r] = 0.f; acc2[a][b][r] = 0.f; }

  const uint4* ga = Ap + (int64_t)tm * PK_SLOTS + tid;
  const uint4* gb = Bp + (int64_t)tn * PK_SLOTS + tid;
  uint4 ra0, ra1, ra2, ra3, rb0, rb1, rb2, rb3;
  rb0 = rb1 = rb2 = rb3 = uint4{0u, 0u, 0u, 0u};
#define OSSCAR_GLOAD(st)                                                                         \
  {                                                                                              \
    const uint4* pa_ = ga + (st) * a_sstride;                                                    \
    ra0 = pa_[0]; ra1 = pa_[256]; ra2 = pa_[512]; ra3 = pa_[768];                                \
    if (!diag) {                                                                                 \
      const uint4* pb_ = gb + (st) * b_sstride;                                                  \
      rb0 = pb_[0]; rb1 = pb_[256]; rb2 = pb_[512]; rb3 = pb_[768];                              \
    }                                                                                            \
  }
#define OSSCAR_SSTORE(buf)                                                                       \
  {                                                                                              \
    uint4* la_ = lds + ((buf) * 2 + 0) * PK_SLOTS + tid;                                         \
    la_[0] = ra0; la_[256] = ra1; la_[512] = ra2; la_[768] = ra3;                                \
    if (!diag) {                                                                                 \
      uint4* lb_ = lds + ((buf) * 2 + 1) * PK_SLOTS + tid;                                       \
      lb_[0] = rb0; lb_[256] = rb1; lb_[512] = rb2; lb_[768] = rb3;                              \
    }                                                                                            \
  }
  const int oa = wm * 64 + (lane & 31), ob = wn * 64 + (lane & 31);

  OSSCAR_GLOAD(s_begin);
  OSSCAR_SSTORE(0);
  __syncthreads();
  int in_window = 0;
  int buf = 0;
  for (int st = s_begin; st < s_end; st++) {
    const bool more = (st + 1 < s_end);
    if (more) OSSCAR_GLOAD(st + 1);
    const uint4* pa = lds + (buf * 2 + 0) * PK_SLOTS;
    const uint4* pb = diag ? pa : lds + (buf * 2 + 1) * PK_SLOTS;
    __builtin_amdgcn_s_setprio(1);        // the wave that is multiplying goes first; the other wave of the SIMD issues its loads and stores in between
#pragma unroll
    for (int ks = 0; ks < GBK / 16; ks++) {
      const int kgo = (ks * 2 + (lane >> 5)) * 128;
      bf8 fa[WT], fb[WT];
#pragma unroll
      for (int a = 0; a < WT; a++) {
        uint4 v = pa[kgo + oa + a * 32];
        fa[a] = *reinterpret_cast<bf8*>(&v);
      }
#pragma unroll
      for (int b = 0; b < WT; b++) {
        uint4 v = pb[kgo + ob + b * 32];
        fb[b] = *reinterpret_cast<bf8*>(&v);
      }
#pragma unroll
      for (int a = 0; a < WT; a++)
#pragma unroll
        for (int b = 0; b < WT; b++)
          acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[a], fb[b], acc[a][b], 0, 0, 0);
    }
    __builtin_amdgcn_s_setprio(0);
    if (++in_window >= window && more) {
      in_window = 0;
#pragma unroll
      for (int a = 0; a < WT; a++)
#pragma unroll
        for (int b = 0; b < WT; b++)
#pragma unroll
          for (int r = 0; r < 16; r++) { acc2[a][b][r] += acc[a][b][r]; acc[a][b][r] = 0.f; }
    }
    if (more) OSSCAR_SSTORE(buf ^ 1);
    __syncthreads();
    buf ^= 1;
  }
#undef OSSCAR_GLOAD
#undef OSSCAR_SSTORE

  // C layout of the 32 x 32 MFMA: register r = rr*4 + r3 holds row rr*8 + (lane/32)*4 + r3, column lane%32
  // (the opaque copy of d1 keeps the compiler from computing the 64 output addresses ahead of the main loop)
  int d1v = ldo;
  asm volatile("" : "+s"(d1v));
  const int rbase = i0 + wm * 64 + (lane >> 5) * 4;
  const int cbase = j0 + wn * 64 + (lane & 31);
  double* hbase = H64 + (int64_t)rbase * d1v + cbase;
#pragma unroll
  for (int a = 0; a < WT; a++)
#pragma unroll
    for (int rr = 0; rr < 4; rr++) {
#pragma unroll
      for (int r3 = 0; r3 < 4; r3++) {
        const int ro = a * 32 + rr * 8 + r3;
        double* hrow = hbase + (int64_t)ro * d1v;
        const bool rok = (rbase + ro < rows_out);
#pragma unroll
        for (int b = 0; b < WT; b++)
          if (rok && cbase + b * 32 < cols_out)
            unsafeAtomicAdd(hrow + b * 32, (double)acc[a][b][rr * 4 + r3] + (double)acc2[a][b][rr * 4 + r3]);
      }
      asm volatile("" ::: "memory");
    }
}

// Xt[c][r - r0] = patch matrix entry (r, c) as float32 (32 x 32 tiles through LDS so that the writes are contiguous)
__global__ __launch_bounds__(256) void im2col_transpose_kernel(const void* __restrict__ F, int is_bf16, ConvSpec cs, int64_t r0,
                                                                int64_t nr, int d1, float* __restrict__ Xt, int64_t ldxt) {
  __shared__ float tile[32][33];
  const int64_t c0 = (int64_t)blockIdx.x * 32, q0 = (int64_t)blockIdx.y * 32;
  const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
  const int kk = cs.kh * cs.kw;
  for (int i = ty; i < 32; i += 8) {
    const int64_t r = q0 + i;
    const int col = (int)(c0 + tx);
    float val = 0.f;
    if (r < nr && col < d1) {
      const int64_t pr = r0 + r;
      const int ox = (int)(pr % cs.Wout), oy = (int)((pr / cs.Wout) % cs.Hout), b = (int)(pr / ((int64_t)cs.Wout * cs.Hout));
      const int c = col / kk, dy = (col % kk) / cs.kw, dx = col % cs.kw;
      const int y = oy * cs.stride + dy - cs.pad, x = ox * cs.stride + dx - cs.pad;
      if (y >= 0 && y < cs.Hin && x >= 0 && x < cs.Win) {
        const int64_t idx = (((int64_t)b * cs.C + c) * cs.Hin + y) * cs.Win + x;
        val = is_bf16 ? __uint_as_float(((uint32_t)reinterpret_cast<const uint16_t*>(F)[idx]) << 16) : reinterpret_cast<const float*>(F)[idx];
      }
    }
    tile[i][tx] = val;
  }
  __syncthreads();
  for (int i = ty; i < 32; i += 8) {
    const int64_t col = c0 + i, r = q0 + tx;
    if (col < d1 && r < nr) Xt[col * ldxt + r] = tile[tx][i];
  }
}
hipError_t launch_im2col_transpose(const void* F, int is_bf16, const ConvSpec& cs, int64_t r0, int64_t nr, int d1, float* Xt,
                                   int64_t ldxt, hipStream_t s) {
  if (nr <= 0) return hipSuccess;
  hipLaunchKernelGGL(im2col_transpose_kernel, dim3((d1 + 31) / 32, (unsigned)((nr + 31) / 32)), dim3(256), 0, s, F, is_bf16, cs, r0, nr, d1,
                     Xt, ldxt);
  return hipGetLastError();
}

// host-only view of the schedule for tests: fills out[0 .. 2*count) with (row, column) pairs, returns the list length
int gram_tile_schedule(int tiles_per_side, int32_t* out, int capacity) {
  std::vector<int2> t;
  build_tile_list(tiles_per_side, t);
  if (out)
    for (size_t i = 0; i < t.size() && (int)i < capacity; i++) { out[2 * i] = t[i].x; out[2 * i + 1] = t[i].y; }
  return (int)t.size();
}

// all tiles of an R x C grid, in 4 x 8 blocks dealt to the XCDs in turn
static void build_rect_tile_list(int R, int C, std::vector<int2>& out) {
  constexpr int NX = 8, RB = 4, CB = 8;
  std::vector<std::vector<int2>> lists(NX);
  int blk = 0;
  for (int r0 = 0; r0 < R; r0 += RB)
    for (int c0 = 0; c0 < C; c0 += CB, blk++)
      for (int r = r0; r < std::min(R, r0 + RB); r++)
        for (int c = c0; c < std::min(C, c0 + CB); c++) lists[blk % NX].push_back(int2{r, c});
  size_t len = 0;
  for (auto& L : lists) len = std::max(len, L.size());
  out.assign(len * NX, int2{-1, -1});
  for (int x = 0; x < NX; x++)
    for (size_t i = 0; i < lists[x].size(); i++) out[i * NX + x] = lists[x][i];
}

static int split_stages(int ntiles, int nstages, int* per_out) {
  int splits = 1;
  if (ntiles < 1024) splits = std::min(nstages, (2048 + ntiles - 1) / ntiles);
  int per = (nstages + splits - 1) / splits;
  per = std::max(per, std::min(nstages, 8));
  *per_out = per;
  return (nstages + per - 1) / per;
}

void gram_tile_list_host(int d1, std::vector<int2>& out) { build_tile_list((d1 + 127) / 128, out); }
void rect_tile_list_host(int d1, int m, std::vector<int2>& out) { build_rect_tile_list((d1 + 127) / 128, (m + 127) / 128, out); }

// Out += A^T B over all stages.  When the contraction is cut into several ranges (few tiles: small layers), the ranges run
// as launches one after the other, so that every element of Out receives its additions in one fixed order (each launch
// adds once per element: the atomic adds never meet).
static void launch_packed_splits(const uint4* Ap, int64_t a_ss, const uint4* Bp, int64_t b_ss, int nstages, int rows_out, int cols_out,
                                 int ldo, double* Out, const int2* tiles, size_t tile_entries, int ntiles, int window, int symmetric,
                                 hipStream_t s) {
  int per = 0;
  const int splits = split_stages(ntiles, nstages, &per);
  const size_t shmem = (size_t)2 * 2 * PK_SLOTS * 16;
  for (int sp = 0; sp < splits; sp++)
    hipLaunchKernelGGL(gram_packed_kernel, dim3((unsigned)tile_entries), dim3(256), shmem, s, Ap, a_ss, Bp, b_ss, nstages, rows_out,
                       cols_out, ldo, Out, tiles, per, window, symmetric, sp);
}

hipError_t launch_gram_packed(const void* Xc, int64_t n_c, int64_t ldx, int d1, double* H64, const int2* tiles,
                              size_t tile_entries, void* pack_buf, int64_t pack_rows, hipStream_t s, const void* Yc,
                              int64_t ldy, int m, double* G64, const int2* tiles_y, size_t tile_y_entries, void* pack_buf_y,
                              const ConvSpec* conv, hipEvent_t* ev, int ev_pairs, int* ev_used) {
  if (ev_used) *ev_used = 0;
  if (n_c <= 0) return hipSuccess;
  if (pack_rows < GBK || pack_rows % GBK || !tiles || tile_entries == 0) return hipErrorInvalidValue;
  if (Yc && (!tiles_y || tile_y_entries == 0)) return hipErrorInvalidValue;
  const int npanels = (d1 + 127) / 128, npanels_y = Yc ? (m + 127) / 128 : 0;
  const int ntiles = npanels * (npanels + 1) / 2;
  const int window = 16;   // 1024 tokens per MFMA accumulation window
  for (int64_t r0 = 0; r0 < n_c; r0 += pack_rows) {
    const int64_t nr = std::min<int64_t>(pack_rows, n_c - r0);
    const int nstages = (int)((nr + GBK - 1) / GBK);
    const uint16_t* src = reinterpret_cast<const uint16_t*>(Xc) + r0 * ldx;
    const uint4* Xp = reinterpret_cast<const uint4*>(pack_buf);
    if (conv)
      hipLaunchKernelGGL(gram_pack_conv_kernel, dim3((npanels + 1) / 2, nstages), dim3(256), 0, s, reinterpret_cast<const uint16_t*>(Xc),
                         *conv, r0, nr, d1, npanels, reinterpret_cast<uint4*>(pack_buf));
    else
      hipLaunchKernelGGL(gram_pack_kernel, dim3((npanels + 1) / 2, nstages), dim3(256), 0, s, src, nr, ldx, d1, npanels,
                         reinterpret_cast<uint4*>(pack_buf));
    const int64_t xs = (int64_t)npanels * PK_SLOTS;
    const bool timed = ev && ev_used && *ev_used < ev_pairs;
    if (timed) hipEventRecord(ev[2 * *ev_used], s);
    launch_packed_splits(Xp, xs, Xp, xs, nstages, d1, d1, d1, H64, tiles, tile_entries, ntiles, window, 1, s);
    if (timed) { hipEventRecord(ev[2 * *ev_used + 1], s); ++*ev_used; }
    if (Yc) {
      const uint16_t* srcy = reinterpret_cast<const uint16_t*>(Yc) + r0 * ldy;
      const uint4* Yp = reinterpret_cast<const uint4*>(pack_buf_y);
      hipLaunchKernelGGL(gram_pack_kernel, dim3((npanels_y + 1) / 2, nstages), dim3(256), 0, s, srcy, nr, ldy, m, npanels_y,
                         reinterpret_cast<uint4*>(pack_buf_y));
      launch_packed_splits(Xp, xs, Yp, (int64_t)npanels_y * PK_SLOTS, nstages, d1, m, m, G64, tiles_y, tile_y_entries,
                           npanels * npanels_y, window, 0, s);
    }
  }
  return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// G = H W on the bf16 matrix cores for bf16 W: H (float32) is split into three bf16 pieces H = H1 + H2 + H3 (each the
// round-to-nearest bf16 of what the previous ones left, so the sum is exact to 2^-25), and H_i^T W = H_i W (H is
// symmetric) runs on the packed kernel above: products of two bf16 numbers are exact in float32, the accumulation is
// restarted every 1024 rows and ends in float64, as for the Gram.
// ------------------------------------------------------------------------------------------------
__device__ __forceinline__ uint32_t bf16_rne_bits(float x) {
  const uint32_t u = __float_as_uint(x);
  return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
}
// piece 0, 1, 2 of the split, packed like gram_pack_kernel packs a bf16 matrix (rows = the contraction index)
__global__ __launch_bounds__(256) void gram_pack_split_kernel(const float* __restrict__ A, int64_t n_c, int64_t lda, int cols,
                                                               int npanels, int piece, uint4* __restrict__ Xp) {
  const int tid = threadIdx.x;
  const int panel = blockIdx.x * 2 + (tid >> 7);
  if (panel >= npanels) return;
  const int kg = (tid & 127) >> 4, cg = tid & 15;
  const int col = panel * 128 + cg * 8;
  const bool live = col < cols;
  const int64_t row0 = (int64_t)blockIdx.y * GBK + kg * 8;
  uint32_t h[8][8];
#pragma unroll
  for (int r = 0; r < 8; r++) {
    const int64_t row = row0 + r;
    float v[8];
    if (live && row < n_c) {
      const float4 a = *reinterpret_cast<const float4*>(A + row * lda + col);
      const float4 b = *reinterpret_cast<const float4*>(A + row * lda + col + 4);
      v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w; v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
    } else {
#pragma unroll
      for (int j = 0; j < 8; j++) v[j] = 0.f;
    }
#pragma unroll
    for (int j = 0; j < 8; j++) {
      float x = v[j];
      uint32_t bits = bf16_rne_bits(x);
      for (int p = 0; p < piece; p++) { x -= __uint_as_float(bits << 16); bits = bf16_rne_bits(x); }
      h[r][j] = bits;
    }
  }
  uint4* out = Xp + ((int64_t)blockIdx.y * npanels + panel) * PK_SLOTS + kg * 128 + cg * 8;
#pragma unroll
  for (int j = 0; j < 8; j++)
    out[j] = uint4{h[0][j] | (h[1][j] << 16), h[2][j] | (h[3][j] << 16), h[4][j] | (h[5][j] << 16), h[6][j] | (h[7][j] << 16)};
}

// G64 (d1 x m, float64, zeroed by the caller) += H W.  H: d1 x d1 float32 (ld = d1, d1 % 8 == 0, 16-byte aligned), W: d1 x m bf16
// (m % 8 == 0, ldw % 8 == 0, 16-byte aligned).  pack_h: pack_rows * 128*ceil(d1/128) * 2 bytes, pack_w likewise for m.
hipError_t launch_hw_split(const float* H, int d1, const void* W, int64_t ldw, int m, double* G64, const int2* tiles,
                           size_t tile_entries, void* pack_h, void* pack_w, int64_t pack_rows, hipStream_t s) {
  if (pack_rows < GBK || pack_rows % GBK || !tiles || tile_entries == 0) return hipErrorInvalidValue;
  const int npanels = (d1 + 127) / 128, npanels_w = (m + 127) / 128;
  const int window = 16;
  for (int64_t r0 = 0; r0 < d1; r0 += pack_rows) {
    const int64_t nr = std::min<int64_t>(pack_rows, d1 - r0);
    const int nstages = (int)((nr + GBK - 1) / GBK);
    hipLaunchKernelGGL(gram_pack_kernel, dim3((npanels_w + 1) / 2, nstages), dim3(256), 0, s,
                       reinterpret_cast<const uint16_t*>(W) + r0 * ldw, nr, ldw, m, npanels_w, reinterpret_cast<uint4*>(pack_w));
    for (int piece = 0; piece < 3; piece++) {
      hipLaunchKernelGGL(gram_pack_split_kernel, dim3((npanels + 1) / 2, nstages), dim3(256), 0, s, H + r0 * d1, nr, (int64_t)d1, d1,
                         npanels, piece, reinterpret_cast<uint4*>(pack_h));
      launch_packed_splits(reinterpret_cast<const uint4*>(pack_h), (int64_t)npanels * PK_SLOTS, reinterpret_cast<const uint4*>(pack_w),
                           (int64_t)npanels_w * PK_SLOTS, nstages, d1, m, m, G64, tiles, tile_entries, npanels * npanels_w, window, 0, s);
    }
  }
  return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// General products of float32 matrices on the bf16 matrix cores: C = beta Cin + alpha A^T B with A (K x M) and B (K x N)
// row-major, the contraction running over their rows.  Each operand is cut into three bf16 pieces (a = a1 + a2 + a3, each the
// round-to-nearest bf16 of what the pieces before it leave: together 24 significand bits), and the six products whose
// weight is at least 2^-16 of the leading one -- a1 b1, a1 b2, a2 b1, a2 b2, a1 b3, a3 b1 -- run on the packed kernel above:
// products of bf16 numbers are exact in float32, sums restart every 1024 rows and end in float64.  What is dropped (a2 b3,
// a3 b2, a3 b3) is below 2^-24 of |a| |b| term by term, the size of the operands' own float32 rounding.
// ------------------------------------------------------------------------------------------------
static int64_t split_kpad(int64_t K) { return (K + GBK - 1) / GBK * GBK; }
size_t split_pack_bytes(int64_t K, int64_t cols) { return (size_t)3 * split_kpad(K) * ((cols + 127) / 128 * 128) * 2; }

hipError_t launch_pack_pieces(const float* A, int64_t lda, int64_t K, int cols, void* pack, hipStream_t s) {
  if (K <= 0 || cols <= 0) return hipSuccess;
  if (cols % 8 || lda % 4 || (reinterpret_cast<uintptr_t>(A) & 15)) return hipErrorInvalidValue;
  const int npanels = (cols + 127) / 128, nstages = (int)(split_kpad(K) / GBK);
  const size_t piece = (size_t)nstages * npanels * PK_SLOTS;      // uint4 packets per piece
  for (int pc = 0; pc < 3; pc++)
    hipLaunchKernelGGL(gram_pack_split_kernel, dim3((npanels + 1) / 2, nstages), dim3(256), 0, s, A, K, lda, cols, npanels, pc,
                       reinterpret_cast<uint4*>(pack) + pc * piece);
  return hipGetLastError();
}

__global__ void split_epilogue_kernel(const double* __restrict__ acc, int M, int N, const float* __restrict__ Cin, int64_t ldcin,
                                      float* __restrict__ C, int64_t ldc, double alpha, double beta) {
  const int64_t tot = (int64_t)M * N;
  for (int64_t idx = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; idx < tot; idx += (int64_t)gridDim.x * blockDim.x) {
    const int64_t i = idx / N, j = idx % N;
    double v = alpha * acc[idx];
    if (Cin) v += beta * (double)Cin[i * ldcin + j];
    C[i * ldc + j] = (float)v;
  }
}

// acc (M x N float64, dense) = A^T B from packed pieces; nprod = 6 (full float32 accuracy) or 3 (a1 b1 + a1 b2 + a2 b1: 2^-16)
hipError_t launch_split_product(const void* packA, int M, const void* packB, int N, int64_t K, int nprod, double* acc,
                                const int2* tiles, size_t tile_entries, int ntiles, hipStream_t s) {
  if (M <= 0 || N <= 0) return hipSuccess;
  if (!tiles || tile_entries == 0 || (nprod != 6 && nprod != 3)) return hipErrorInvalidValue;
  const int npa = (M + 127) / 128, npb = (N + 127) / 128, nstages = (int)(split_kpad(K) / GBK);
  const size_t pieceA = (size_t)nstages * npa * PK_SLOTS, pieceB = (size_t)nstages * npb * PK_SLOTS;
  hipError_t e = hipMemsetAsync(acc, 0, (size_t)M * N * 8, s);
  if (e != hipSuccess) return e;
  if (K <= 0) return hipSuccess;
  static const int combo[6][2] = {{0, 0}, {0, 1}, {1, 0}, {1, 1}, {0, 2}, {2, 0}};
  for (int c = 0; c < nprod; c++)
    launch_packed_splits(reinterpret_cast<const uint4*>(packA) + combo[c][0] * pieceA, (int64_t)npa * PK_SLOTS,
                         reinterpret_cast<const uint4*>(packB) + combo[c][1] * pieceB, (int64_t)npb * PK_SLOTS, nstages, M, N, N, acc,
                         tiles, tile_entries, ntiles, 16, 0, s);
  return hipGetLastError();
}

hipError_t launch_split_epilogue(const double* acc, int M, int N, const float* Cin, int64_t ldcin, float* C, int64_t ldc, double alpha,
                                 double beta, hipStream_t s) {
  if (M <= 0 || N <= 0) return hipSuccess;
  hipLaunchKernelGGL(split_epilogue_kernel, dim3(2048), dim3(256), 0, s, acc, M, N, (beta != 0.0) ? Cin : nullptr, ldcin, C, ldc, alpha, beta);
  return hipGetLastError();
}

// sum of squares of a rows x cols matrix (float32 or bf16), added to *acc
__global__ __launch_bounds__(256) void sumsq_kernel(const void* __restrict__ A, int is_bf16, int64_t rows, int64_t cols, int64_t ld,
                                                     double* __restrict__ part) {
  __shared__ double red[4];
  double v = 0;
  const int64_t tot = rows * cols;
  for (int64_t idx = blockIdx.x * 256 + threadIdx.x; idx < tot; idx += (int64_t)gridDim.x * 256) {
    const int64_t r = idx / cols, c = idx % cols;
    const float x = is_bf16 ? __uint_as_float(((uint32_t)reinterpret_cast<const uint16_t*>(A)[r * ld + c]) << 16)
                            : reinterpret_cast<const float*>(A)[r * ld + c];
    v += (double)x * (double)x;
  }
  for (int o = 32; o > 0; o >>= 1) v += __shfl_down(v, o, 64);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
  __syncthreads();
  if (threadIdx.x == 0) part[blockIdx.x] = red[0] + red[1] + red[2] + red[3];
}
// *acc += the 1024 partial sums, in a fixed order
__global__ __launch_bounds__(1024) void sumsq_add_kernel(const double* __restrict__ part, double* __restrict__ acc);
hipError_t launch_sumsq(const void* A, int is_bf16, int64_t rows, int64_t cols, int64_t ld, double* acc, double* partial, hipStream_t s) {
  if (rows <= 0 || cols <= 0) return hipSuccess;
  hipLaunchKernelGGL(sumsq_kernel, dim3(1024), dim3(256), 0, s, A, is_bf16, rows, cols, ld, partial);
  hipLaunchKernelGGL(sumsq_add_kernel, dim3(1), dim3(1024), 0, s, partial, acc);
  return hipGetLastError();
}

// G = float32(G64 + lambda W)
__global__ void finalize_G_kernel(const double* __restrict__ G64, const float* __restrict__ Wf, const double* __restrict__ lambda,
                                  float* __restrict__ G, int64_t n) {
  const double lam = *lambda;
  for (int64_t i = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x)
    G[i] = (float)(G64[i] + lam * (double)Wf[i]);
}
hipError_t launch_finalize_G(const double* G64, const float* Wf, const double* lambda_dev, float* G, int64_t n, hipStream_t s) {
  hipLaunchKernelGGL(finalize_G_kernel, dim3(2048), dim3(256), 0, s, G64, Wf, lambda_dev, G, n);
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

// H[i][j] = float(H64[max(i,j)][min(i,j)] + (i == j ? lam : 0)).  One workgroup per 64 x 64 tile on or below the
// diagonal: it reads the tile of H64 along its rows, writes it to H, and writes the mirrored tile from LDS, so that both
// the reads and the writes run along rows.
__global__ __launch_bounds__(256) void finalize_H_kernel(const double* __restrict__ H64, float* __restrict__ H, int d1,
                                                          const double* __restrict__ lam_dev) {
  __shared__ float tile[64][65];
  const double lam = lam_dev ? lam_dev[0] : 0.0;
  // tile index -> (tr, tc), tc <= tr
  const int t = blockIdx.x;
  int tr = (int)((sqrtf(8.f * (float)t + 1.f) - 1.f) * 0.5f);
  while ((int64_t)(tr + 1) * (tr + 2) / 2 <= t) tr++;
  while ((int64_t)tr * (tr + 1) / 2 > t) tr--;
  const int tc = t - tr * (tr + 1) / 2;
  const int r0 = tr * 64, c0 = tc * 64;
  const int lx = threadIdx.x & 63, ly = threadIdx.x >> 6;
  for (int k = 0; k < 16; k++) {
    const int i = r0 + ly + 4 * k, j = c0 + lx;
    float v = 0.f;
    if (i < d1 && j < d1) {
      // on a diagonal tile the entries above the diagonal come from their mirror images
      double x = (i >= j) ? H64[(int64_t)i * d1 + j] : H64[(int64_t)j * d1 + i];
      if (i == j) x += lam;
      v = (float)x;
      H[(int64_t)i * d1 + j] = v;
    }
    tile[ly + 4 * k][lx] = v;
  }
  if (tr == tc) return;
  __syncthreads();
  for (int k = 0; k < 16; k++) {
    const int i = c0 + ly + 4 * k, j = r0 + lx;      // row of the mirrored tile, column along the lanes
    if (i < d1 && j < d1) H[(int64_t)i * d1 + j] = tile[lx][ly + 4 * k];
  }
}

hipError_t launch_finalize_H(const double* H64, float* H, int d1, const double* lam_dev, hipStream_t s) {
  const int64_t nt = (d1 + 63) / 64;
  hipLaunchKernelGGL(finalize_H_kernel, dim3((unsigned)(nt * (nt + 1) / 2)), dim3(256), 0, s, H64, H, d1, lam_dev);
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

// out = sum_i <a[rows[i], :], b[i, :]> (a: row-major with leading dimension m, b: dense nrows x m), float64, fixed order
__global__ __launch_bounds__(256) void dot64_rows_stage1(const float* __restrict__ a, const int32_t* __restrict__ rows,
                                                          const float* __restrict__ b, int nrows, int m, double* __restrict__ partial) {
  __shared__ double sh[4];
  double v = 0;
  for (int i = blockIdx.x; i < nrows; i += gridDim.x) {
    const float* ar = a + (int64_t)rows[i] * m;
    const float* br = b + (int64_t)i * m;
    for (int c = threadIdx.x; c < m; c += 256) v += (double)ar[c] * (double)br[c];
  }
  double t = block_sum(v, sh);
  if (threadIdx.x == 0) partial[blockIdx.x] = t;
}
hipError_t launch_dot64_rows(const float* a, const int32_t* rows, const float* b, int nrows, int m, double* out, double* partial,
                             hipStream_t s) {
  hipLaunchKernelGGL(dot64_rows_stage1, dim3(1024), dim3(256), 0, s, a, rows, b, nrows, m, partial);
  hipLaunchKernelGGL(dot64_stage2, dim3(1), dim3(1024), 0, s, partial, 1024, out);
  return hipGetLastError();
}

__global__ __launch_bounds__(1024) void sumsq_add_kernel(const double* __restrict__ part, double* __restrict__ acc) {
  __shared__ double sh[16];
  double t = block_sum(part[threadIdx.x], sh);
  if (threadIdx.x == 0) acc[0] += t;
}

hipError_t launch_dot64(const float* a, const float* b, int64_t n, double* out, double* partial, hipStream_t s) {
  hipLaunchKernelGGL(dot64_stage1, dim3(1024), dim3(256), 0, s, a, b, n, partial);
  hipLaunchKernelGGL(dot64_stage2, dim3(1), dim3(1024), 0, s, partial, 1024, out);
  return hipGetLastError();
}

}  // namespace osscar
