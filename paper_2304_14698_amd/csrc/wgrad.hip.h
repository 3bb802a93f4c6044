// Weight gradients of one affine layer, dW = X^T dZ and db = 1^T dZ, over a very tall X
// (rows = edges or nodes), deterministic: the rows are cut into chunks, every (column tile,
// chunk) block accumulates its partial [64, H] tile on the matrix cores in fp32, and a second
// kernel adds the chunk partials in chunk order onto the caller's gradient vector.
//
// The contraction runs over rows, so both MFMA operands need "lane = column, elements = rows".
// Row-major tiles are therefore transposed on their way into LDS: element (row, col) of a tile
// of TC columns lives at ((row / V) * TC' + col + col / V) * V + row % V (one pad column after
// every V keeps the transposing writes free of bank conflicts), which makes a lane's V rows of
// one column one 16-byte LDS read. The bias gradient comes from an extra all-ones column of X.
#pragma once
#include "mlp2.hip.h"

enum { WG_PLAIN = 0, WG_EDGE = 1, WG_NODE = 2, WG_EMBED = 3 };

struct WgradArgs {
  int64_t n_rows;
  int rows_per_chunk, n_chunks;
  int Ka;                   // real columns of X; column Ka is the all-ones bias column
  const void *A;            // PLAIN: [rows, Ka] operand type (Ka == H)
  const void *h, *agg;      // EDGE / NODE sources, operand type
  const int32_t *agg_src;   // NODE, transpose-read kernel: [N] row of agg per node, -1 = none (zeros are read)
  const void *zero_row;     // 1 KB of zeros
  const int32_t *in_ptr, *in_src, *in_dst;
  const float *edge_feat;
  const int32_t *node_op;
  const float *node_dense;
  int De, Tn, Dd;
  const void *dZ;           // [rows, H] operand type
  float *partial;           // [n_chunks, KaP, H], KaP = 64 * gridDim.x
};

// V consecutive columns (col0 .. col0+V-1, col0 a multiple of V) of row `row` of the virtual X.
template <typename T, int H, int KIND>
__device__ __forceinline__ typename Operand<T>::vec wgrad_load_x(const WgradArgs &a, int64_t row,
                                                                 int col0) {
  using Opd = Operand<T>;
  constexpr int V = Opd::V;
  typename Opd::vec x;
  if constexpr (KIND == WG_PLAIN) {
    if (col0 + V <= a.Ka) return *(const typename Opd::vec *)((const T *)a.A + (size_t)row * a.Ka + col0);
#pragma unroll
    for (int j = 0; j < V; ++j) x[j] = Opd::from_float(col0 + j == a.Ka ? 1.f : 0.f);
    return x;
  } else if constexpr (KIND == WG_EDGE) {
    if (col0 + V <= H) return *(const typename Opd::vec *)((const T *)a.h + (size_t)a.in_src[row] * H + col0);
    if (col0 + V <= 2 * H)
      return *(const typename Opd::vec *)((const T *)a.h + (size_t)a.in_dst[row] * H + (col0 - H));
#pragma unroll
    for (int j = 0; j < V; ++j) {
      const int k = col0 + j - 2 * H;
      x[j] = Opd::from_float(k < a.De ? a.edge_feat[(size_t)row * a.De + k] : (k == a.De ? 1.f : 0.f));
    }
    return x;
  } else if constexpr (KIND == WG_NODE) {
    if (col0 + V <= H) return *(const typename Opd::vec *)((const T *)a.h + (size_t)row * H + col0);
    if (col0 + V <= 2 * H) {
      if (a.in_ptr[row + 1] > a.in_ptr[row])
        return *(const typename Opd::vec *)((const T *)a.agg + (size_t)row * H + (col0 - H));
      return Opd::zero();
    }
#pragma unroll
    for (int j = 0; j < V; ++j) x[j] = Opd::from_float(col0 + j == 2 * H ? 1.f : 0.f);
    return x;
  } else {
    const int op = a.node_op[row];
#pragma unroll
    for (int j = 0; j < V; ++j) {
      const int k = col0 + j;
      float v = 0.f;
      if (k < a.De) {
        for (int e = a.in_ptr[row]; e < a.in_ptr[row + 1]; ++e) v += a.edge_feat[(size_t)e * a.De + k];
      } else if (k < a.De + a.Tn) v = (k - a.De == op) ? 1.f : 0.f;
      else if (k < a.De + a.Tn + a.Dd) v = a.node_dense[(size_t)row * a.Dd + (k - a.De - a.Tn)];
      else if (k == a.De + a.Tn + a.Dd) v = 1.f;
      x[j] = Opd::from_float(v);
    }
    return x;
  }
}

template <typename T, int H, int KIND>
__global__ __launch_bounds__(256) void wgrad_kernel(const WgradArgs a) {
  using Opd = Operand<T>;
  using vec = typename Opd::vec;
  constexpr int V = Opd::V;            // rows per lane per MFMA step; a step covers 2V rows
  constexpr int TA = 64;               // X columns per block
  constexpr int RS = 8 * V;            // rows per stage (64 bf16, 32 fp32: LDS stays under 48 KB)
  constexpr int NB = H / 64;           // 32-column blocks of dZ per wave
  __shared__ T As[RS / V][TA + TA / V][V];
  __shared__ T Bs[RS / V][H + H / V][V];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, l32 = lane & 31, g = lane >> 5;
  const int ka0 = blockIdx.x * TA;
  const int chunk = blockIdx.y;
  const int64_t r_begin = (int64_t)chunk * a.rows_per_chunk;
  int64_t r_end = r_begin + a.rows_per_chunk;
  if (r_end > a.n_rows) r_end = a.n_rows;
  const int kab = wave & 1;            // this wave's 32-column block of X inside the tile
  const int kbb0 = wave >> 1;          // its dZ blocks: kbb0, kbb0 + 2, ...

  f32x16 acc[NB];
#pragma unroll
  for (int i = 0; i < NB; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[i][r] = 0.f;

  for (int64_t rs = r_begin; rs < r_end; rs += RS) {
    // ---- stage X tile: RS rows x TA columns, V-column vectors; lanes run over column chunks
    for (int vi = tid; vi < RS * (TA / V); vi += 256) {
      const int cc = vi % (TA / V), rl = vi / (TA / V);
      const int64_t row = rs + rl;
      vec x = row < r_end ? wgrad_load_x<T, H, KIND>(a, row, ka0 + cc * V) : Opd::zero();
#pragma unroll
      for (int j = 0; j < V; ++j) As[rl / V][cc * (V + 1) + j][rl % V] = x[j];
    }
    for (int vi = tid; vi < RS * (H / V); vi += 256) {
      const int cc = vi % (H / V), rl = vi / (H / V);
      const int64_t row = rs + rl;
      vec x = row < r_end ? *(const vec *)((const T *)a.dZ + (size_t)row * H + cc * V) : Opd::zero();
#pragma unroll
      for (int j = 0; j < V; ++j) Bs[rl / V][cc * (V + 1) + j][rl % V] = x[j];
    }
    __syncthreads();
    // ---- contraction over the stage's rows, 2V rows per step
#pragma unroll
    for (int st = 0; st < RS / (2 * V); ++st) {
      const int ca = 32 * kab + l32;
      const vec xa = *(const vec *)&As[2 * st + g][ca + ca / V][0];
#pragma unroll
      for (int i = 0; i < NB; ++i) {
        const int cb = 32 * (kbb0 + 2 * i) + l32;
        const vec xb = *(const vec *)&Bs[2 * st + g][cb + cb / V][0];
        Opd::mma(xa, xb, acc[i]);
      }
    }
    __syncthreads();
  }
  const int KaP = TA * gridDim.x;
  float *out = a.partial + ((size_t)chunk * KaP + ka0 + 32 * kab) * H;
#pragma unroll
  for (int i = 0; i < NB; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r)
      out[(size_t)acc_row(r, g) * H + 32 * (kbb0 + 2 * i) + l32] = acc[i][r];
}

// ---------------------------------------------------------------------------------------------
// bf16 variant built on the LDS transpose read (ds_read_b64_tr_b16): tiles go into LDS row-major,
// 16 bytes per lane, and an operand "lane = column, elements = 8 consecutive rows" is two reads.
// In a group of 16 lanes, lane L passes the address of 4 consecutive 16-bit elements -- lanes
// 4j .. 4j+3 together one 16-element piece of row j -- and receives element L of each of the four
// rows; so lane L points at tile[k0 + L / 4][c0 + 4 * (L % 4)] and gets tile[k0 .. k0+3][c0 + L].
//
// A block owns 128 columns of X and all H columns of dZ over one contiguous slice of the rows
// (wave (wa, wb): X columns 64 wa .., dZ columns H/2 wb ..), stages 32 rows at a time, and keeps
// the next stage's global loads in flight while the matrix cores work on the current one (one
// barrier per stage); the row indices of gathered X columns are fetched two stages ahead. The
// 128-column tiles of one row slice run on the same XCD, so dZ is fetched into that L2 once.
// Rows of an LDS tile are 64 bytes longer than their data: with a row stride of 16 (mod 64)
// dwords the four rows a transpose read touches fall on different banks.
struct Wgrad2Plan {
  int kt, ny, rows_per_slot;     // column tiles of X, row slices, rows per slice (multiple of 32)
};
// kt column tiles; blocks_per_cu = how many blocks of the kernel variant a CU holds
inline Wgrad2Plan wgrad2_plan(int64_t n_rows, int kt, int n_cu, int blocks_per_cu) {
  Wgrad2Plan p;
  p.kt = kt;
  int per = (blocks_per_cu * n_cu / 8) / p.kt;            // row slices per XCD
  if (per < 1) per = 1;
  int64_t want = (n_rows + 63) / 64;                      // at least 64 rows per slice
  want = (want + 7) / 8;
  if (want < 1) want = 1;
  if (per > want) per = (int)want;
  p.ny = 8 * per;
  int64_t rps = (n_rows + p.ny - 1) / p.ny;
  p.rows_per_slot = (int)((rps + 31) / 32 * 32);
  return p;
}

typedef short s16x4 __attribute__((ext_vector_type(4)));

// 8 rows (k0 .. k0+7) of one column as an MFMA operand; p = this lane's address for rows k0 .. k0+3
__device__ __forceinline__ bf16x8 lds_tr_operand(const char *p, int row_stride) {
  typedef s16x4 __attribute__((address_space(3))) * lp;
  const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lp)(p));
  const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lp)(p + 4 * row_stride));
  const s16x8 v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
  return __builtin_bit_cast(bf16x8, v);
}

// The stage loop of one block. Every global load is unconditional, from a clamped (always valid)
// address, and masked afterwards: divergent or conditional loads would put waits for memory in
// the middle of the loop. TAIL = the tile holds columns past the gathered / direct ones (edge
// attributes, the all-ones bias column, padding); such tiles are whole for the EDGE and NODE
// kinds (2H is a multiple of 128), PLAIN uses the one formulation for all its tiles.
template <int H, int KIND, bool TAIL, int TA, int RS>
__device__ __forceinline__ void wgrad2_run(const WgradArgs &a, int ka0, int64_t r_begin, int64_t r_end,
                                           char (*Xs)[RS * (TA * 2 + 64)], char (*Zs)[RS * (H * 2 + 64)],
                                           f32x16 (&acc)[2][H / 64 > 0 ? H / 64 : 1], bool do_bias,
                                           float (&bsum)[8]) {
  using T = bf16_t;
  using vec = bf16x8;
  constexpr int NT = 2 * TA;                               // TA / 64 x 2 waves
  constexpr int XV = RS / 16;                              // X vectors per thread per stage
  constexpr int XS = TA * 2 + 64, ZS = H * 2 + 64;         // LDS row strides, bytes
  constexpr int NB = H / 64 > 0 ? H / 64 : 1;              // 32-column blocks of dZ per wave
  constexpr int ZV = RS * (H / 8) / NT;                    // dZ vectors per thread per stage
  static_assert(ZV >= 1, "a stage of dZ gives every thread at least one vector");
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, g = lane >> 5;
  const int wa = wave % (TA / 64), wb = wave / (TA / 64);
  const int n_stage = (int)((r_end - r_begin + RS - 1) / RS);

  // ---- this thread's XV X vectors per stage: rows xr, xr + 16, .. of the stage, columns xc .. xc+7
  const int xr = tid / (TA / 8), xcl = tid % (TA / 8), xc = ka0 + 8 * xcl;
  const bool second = xc >= H;                             // EDGE: receiver's state; NODE: aggregate
  [[maybe_unused]] const int32_t *idx_arr = second ? a.in_dst : a.in_src;
  [[maybe_unused]] const T *gbase = (const T *)a.h + (second ? xc - H : xc);
  [[maybe_unused]] const T *nbase = second ? (const T *)a.agg + (xc - H) : (const T *)a.h + xc;
  vec ones = Operand<T>::zero();                           // the bias column, when this thread holds it
  if (xc == a.Ka) ones[0] = (T)1.0f;

  auto row_of = [&](int st, int c) {
    int64_t row = r_begin + (int64_t)st * RS + xr + 16 * c;
    return row < r_end ? row : r_end - 1;
  };
  auto live = [&](int st, int c) { return r_begin + (int64_t)st * RS + xr + 16 * c < r_end; };
  // row indices (EDGE) of stage st, which may be past the end
  auto load_idx = [&](int st, int (&ix)[XV]) {
#pragma unroll
    for (int c = 0; c < XV; ++c) {
      ix[c] = 0;
      if constexpr (!TAIL && KIND == WG_EDGE) ix[c] = idx_arr[row_of(st, c)];
      if constexpr (!TAIL && KIND == WG_NODE) {
        ix[c] = a.agg_src[row_of(st, c)];   // (every thread, under no condition: see load_x)
      }
    }
  };
  auto load_x = [&](int st, const int (&ix)[XV], vec (&x)[XV]) {
#pragma unroll
    for (int c = 0; c < XV; ++c) {
      const int64_t row = row_of(st, c);
      const bool on = live(st, c);
      if constexpr (KIND == WG_PLAIN) {
        const int cc = xc + 8 <= a.Ka ? xc : a.Ka - 8;
        const vec v = *(const vec *)((const T *)a.A + (size_t)row * a.Ka + cc);
        x[c] = !on ? Operand<T>::zero() : (xc + 8 <= a.Ka ? v : ones);
      } else if constexpr (!TAIL && KIND == WG_EDGE) {
        const vec v = *(const vec *)(gbase + (size_t)ix[c] * H);
        x[c] = on ? v : Operand<T>::zero();
      } else if constexpr (!TAIL && KIND == WG_NODE) {
        // (the received sum of a node without in-edges is read from a row of zeros: the select
        // is on the address, formed from an index requested a stage earlier. A select on the
        // loaded value here made the compiler wait for the load on the spot.)
        const int64_t srow = second ? (int64_t)ix[c] : row;
        const T *p = srow < 0 ? (const T *)a.zero_row + (xc - H) : nbase + (size_t)srow * H;
        const vec v = *(const vec *)p;
        x[c] = on ? v : Operand<T>::zero();
      } else if constexpr (KIND == WG_EDGE) {              // [edge attributes | 1 | 0 ...]
        // every lane loads and uses an attribute (times 0 or 1, plus the bias column's 1): a
        // select would let the compiler move the loads into branches with waits behind them
        vec v;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          const int k = xc - 2 * H + j;
          const float f = a.De > 0 ? a.edge_feat[(size_t)row * a.De + (k < a.De ? k : a.De - 1)] : 0.f;
          v[j] = (T)fmaf(f, k < a.De ? 1.f : 0.f, k == a.De ? 1.f : 0.f);
        }
        x[c] = on ? v : Operand<T>::zero();
      } else {                                             // NODE: [1 | 0 ...]
        x[c] = on ? ones : Operand<T>::zero();
      }
    }
  };
  auto load_z = [&](int st, vec (&z)[ZV]) {
#pragma unroll
    for (int c = 0; c < ZV; ++c) {
      const int vi = tid + NT * c, rl = vi / (H / 8), cc = vi % (H / 8);
      int64_t row = r_begin + (int64_t)st * RS + rl;
      const bool on = row < r_end;
      if (!on) row = r_end - 1;
      const vec v = *(const vec *)((const T *)a.dZ + (size_t)row * H + cc * 8);
      z[c] = on ? v : Operand<T>::zero();
    }
  };
  auto commit = [&](int buf, const vec (&x)[XV], const vec (&z)[ZV]) {
#pragma unroll
    for (int c = 0; c < XV; ++c) *(vec *)(Xs[buf] + (xr + 16 * c) * XS + xcl * 16) = x[c];
#pragma unroll
    for (int c = 0; c < ZV; ++c) {
      const int vi = tid + NT * c, rl = vi / (H / 8), cc = vi % (H / 8);
      *(vec *)(Zs[buf] + rl * ZS + cc * 16) = z[c];
    }
  };

  // column sums of dZ (the bias gradient) from the vectors this thread stages: all of them cover
  // the same eight columns (NT is a multiple of H / 8)
  auto add_bias = [&](const vec (&z)[ZV]) {
#pragma unroll
    for (int c = 0; c < ZV; ++c)
#pragma unroll
      for (int j = 0; j < 8; ++j) bsum[j] += (float)z[c][j];
  };
  int ix0[XV], ix1[XV];
  vec xn[XV], zn[ZV];
  load_idx(0, ix0);
  load_idx(1, ix1);
  load_x(0, ix0, xn);
  load_z(0, zn);
  commit(0, xn, zn);
  if (do_bias) add_bias(zn);
  __syncthreads();
  // per-lane offsets of the transpose reads: row 8 g + L / 4, 8 bytes at 16-bit column 16 half + 4 (L % 4)
  const int L = lane & 15, half = (lane >> 4) & 1;
  const int xoff = (8 * g + L / 4) * XS + (32 * (2 * wa) + 16 * half + 4 * (L % 4)) * 2;
  const int zoff = (8 * g + L / 4) * ZS + (32 * (wb * NB) + 16 * half + 4 * (L % 4)) * 2;
  for (int st = 0; st < n_stage; ++st) {
    int ix2[XV];
    load_idx(st + 2 < n_stage ? st + 2 : st, ix2);
    const int sn = st + 1 < n_stage ? st + 1 : st;         // (the last iteration re-reads its own stage)
    load_x(sn, ix1, xn);
    load_z(sn, zn);
    const char *xs = Xs[st & 1] + xoff, *zs = Zs[st & 1] + zoff;
#pragma unroll
    for (int k = 0; k < RS / 16; ++k) {
      vec xa[2], xb[NB];
#pragma unroll
      for (int m = 0; m < 2; ++m) xa[m] = lds_tr_operand(xs + 16 * k * XS + 64 * m, XS);
#pragma unroll
      for (int i = 0; i < NB; ++i) xb[i] = lds_tr_operand(zs + 16 * k * ZS + 64 * i, ZS);
#pragma unroll
      for (int m = 0; m < 2; ++m)
#pragma unroll
        for (int i = 0; i < NB; ++i) Operand<T>::mma(xa[m], xb[i], acc[m][i]);
    }
    commit((st + 1) & 1, xn, zn);
    if (do_bias && st + 1 < n_stage) add_bias(zn);
    __syncthreads();
#pragma unroll
    for (int c = 0; c < XV; ++c) ix1[c] = ix2[c];
  }
}

// TA = X columns per block: 128 (four waves, two blocks per CU) or 256 (eight waves, one block
// per CU: X enters once, dZ once per 256 instead of once per 128 columns). ka_base = first column
// of the launch's tiles (a launch may cover only the columns past the H-wide parts).
// bias_row >= 0: the column sums of dZ are taken on the vector ALU by the first tile's block of
// every row slice and stored as row bias_row of the slice's partial (then no tile has to hold the
// all-ones column); KaP = rows per slice of the partial array.
// RS = rows per stage, 32 or 64: a stage is what a block has in flight from memory while it
// multiplies the previous one, and 32 rows are too few to cover the latency with one block per CU.
template <int H, int KIND, int TA, int RS = 32>
__global__ __launch_bounds__(2 * TA) void wgrad2_kernel(const WgradArgs a, int kt, int ny, int ka_base, int KaP,
                                                        int bias_row) {
  constexpr int XS = TA * 2 + 64, ZS = H * 2 + 64;
  constexpr int NB = H / 64 > 0 ? H / 64 : 1;
  static_assert(KIND != WG_EMBED, "the embed layer's input rows are written out first and go through WG_PLAIN");
  extern __shared__ __align__(16) char smem[];              // wgrad2_lds_bytes<H, TA>()
  char(*Xs)[RS * XS] = reinterpret_cast<char(*)[RS * XS]>(smem);
  char(*Zs)[RS * ZS] = reinterpret_cast<char(*)[RS * ZS]>(smem + 2 * RS * XS);
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, l32 = lane & 31, g = lane >> 5;
  const int wa = wave % (TA / 64), wb = wave / (TA / 64);
  // blocks are dealt round-robin to the 8 XCDs: the kt tiles of a row slice stay on one XCD
  const int xcd = blockIdx.x % 8, q = blockIdx.x / 8;
  const int kq = q % kt, y = xcd + 8 * (q / kt);
  const int ka0 = ka_base + kq * TA;
  const int64_t r_begin = (int64_t)y * a.rows_per_chunk;
  int64_t r_end = r_begin + a.rows_per_chunk;
  if (r_end > a.n_rows) r_end = a.n_rows;

  f32x16 acc[2][NB];
#pragma unroll
  for (int m = 0; m < 2; ++m)
#pragma unroll
    for (int i = 0; i < NB; ++i)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[m][i][r] = 0.f;
  const bool do_bias = bias_row >= 0 && kq == 0;
  float bsum[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  if (r_end > r_begin) {
    if (KIND != WG_PLAIN && ka0 >= 2 * H) wgrad2_run<H, KIND, true, TA, RS>(a, ka0, r_begin, r_end, Xs, Zs, acc, do_bias, bsum);
    else wgrad2_run<H, KIND, false, TA, RS>(a, ka0, r_begin, r_end, Xs, Zs, acc, do_bias, bsum);
  }
  if (do_bias) {
    // thread t holds columns 8 (t % (H / 8)) ..; the 2 TA / (H / 8) threads of a column chunk are
    // added in thread order (the stage loop ended with a barrier: the tile buffers are free)
    constexpr int NT = 2 * TA, CH = H / 8, NG = NT / CH;
    float *red = reinterpret_cast<float *>(smem);          // [NG][H]
    const int t = threadIdx.x;
#pragma unroll
    for (int j = 0; j < 8; ++j) red[(t / CH) * H + 8 * (t % CH) + j] = bsum[j];
    __syncthreads();
    for (int f = t; f < H; f += NT) {
      float sum = red[f];
      for (int k = 1; k < NG; ++k) sum += red[k * H + f];
      a.partial[((size_t)y * KaP + bias_row) * H + f] = sum;
    }
  }
  // partial[y][column - ka_base][f]
  float *out = a.partial + ((size_t)y * KaP + kq * TA + 32 * (2 * wa)) * H + 32 * (wb * NB) + l32;
#pragma unroll
  for (int m = 0; m < 2; ++m)
#pragma unroll
    for (int i = 0; i < NB; ++i)
#pragma unroll
      for (int r = 0; r < 16; ++r)
        out[(size_t)(32 * m + acc_row(r, g)) * H + 32 * i] = acc[m][i][r];
}

template <int H, int TA, int RS = 32>
constexpr size_t wgrad2_lds_bytes() { return 2 * RS * (size_t)(TA * 2 + 64) + 2 * RS * (size_t)(H * 2 + 64); }

// dW[k, f] += sum over chunks of partial[chunk, k, f] for k < Ka; db[f] += row Ka (db may be null:
// a product without a bias row). A block handles
// 32 consecutive entries; its 8 thread groups take every eighth chunk (eight loads in flight
// each) and their sums are added in group order, so the result has one fixed summation order.
__global__ __launch_bounds__(256) void wgrad_reduce_kernel(const float *partial, int n_chunks, int KaP, int Ka,
                                                           int H, float *dW, float *db) {
  __shared__ float part[8][32];
  const int e = threadIdx.x & 31, g = threadIdx.x >> 5;
  const int64_t i = (int64_t)blockIdx.x * 32 + e;
  const bool live = i < (int64_t)(Ka + (db ? 1 : 0)) * H;   // (db null: no bias row)
  const int k = live ? (int)(i / H) : 0, f = live ? (int)(i - (int64_t)k * H) : 0;
  const float *p = partial + (size_t)k * H + f;
  const size_t cs = (size_t)KaP * H;
  float s = 0.f;
  int c = g;
  for (; c + 56 < n_chunks; c += 64) {
    float v[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) v[j] = p[(size_t)(c + 8 * j) * cs];
#pragma unroll
    for (int j = 0; j < 8; ++j) s += v[j];
  }
  for (; c < n_chunks; c += 8) s += p[(size_t)c * cs];
  part[g][e] = s;
  __syncthreads();
  if (g == 0 && live) {
    float t = part[0][e];
#pragma unroll
    for (int j = 1; j < 8; ++j) t += part[j][e];
    if (k < Ka) dW[(size_t)k * H + f] += t;
    else db[f] += t;
  }
}
