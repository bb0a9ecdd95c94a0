// Recurrent memory cells (GRU, LSTM), one time step per launch: the hidden-side contraction on the matrix cores with
// the gate stage (forward) or the gate derivatives (back-propagation through time) as its epilogue, and the index
// plumbing of column-wise minibatches.  The input-side contractions and the weight gradients run in the GEMM kernel.
#include "kernels.h"

namespace rslx {
namespace {

typedef float f4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ float sigmoidf_(float a) { return 1.0f / (1.0f + __expf(-a)); }
// tanh through the exponential of -2|a| (never overflows): (1 - e) / (1 + e) with the sign of a
__device__ __forceinline__ float tanhf_(float a) {
  const float e = __expf(-2.0f * fabsf(a));
  const float t = (1.0f - e) / (1.0f + e);
  return a < 0.f ? -t : t;
}

__device__ __forceinline__ f4 ld4(const float* p) { return *reinterpret_cast<const f4*>(p); }
__device__ __forceinline__ void st4(float* p, f4 v) { *reinterpret_cast<f4*>(p) = v; }

// ---- fused step kernels ----------------------------------------------------------------------------------
// A workgroup of 2 x 2 wavefronts owns 32 rows and 32 hidden units: wavefront (wr, wj) takes rows 16 wr .. 16 wr + 15
// and hidden units 16 wj .. 16 wj + 15 and accumulates NTW tiles of 16 output columns with
// v_mfma_f32_16x16x4_f32, D[row, col] += sum_k A[row, k] B[k, col(tile)]; the tiles' columns come from `col0[]`
// (forward: the r, z and n columns of its 16 hidden units; backward: the 16 hidden units themselves).  Accumulator
// register q of lane l belongs to row 4 * (l / 16) + q and column l % 16 in every tile, so the gate stage finds all
// its operands in the lane's own registers.  Operands are staged through LDS in chunks of KC contraction steps; the
// next chunk's global loads are in flight while the current one is multiplied.  One step moves little data per
// workgroup and every chunk costs a full memory latency, so the chunks are long rather than many, and two
// wavefronts share each SIMD so that one's LDS reads overlap the other's matrix instructions.
constexpr int GS_JB = 32;          // hidden units per workgroup
constexpr int GS_ROWS = 32;        // rows per workgroup
constexpr int GS_THREADS = 256;

template <int NTW, int KC>
struct StepTile {
  static constexpr int NT = 2 * NTW;            // tiles per workgroup: wavefront column wj owns tiles wj * NTW ...
  static constexpr int APITCH = KC + 4;         // floats per staged A row (16-byte aligned, spreads the banks)
  static constexpr int COLS = 16 * NT, BPITCH = COLS + 8;
  static constexpr int A_VECS = GS_ROWS * KC / 4, B_VECS = KC * COLS / 4;
  static constexpr int A_PER = (A_VECS + GS_THREADS - 1) / GS_THREADS, B_PER = (B_VECS + GS_THREADS - 1) / GS_THREADS;
  static constexpr int LDS_FLOATS = GS_ROWS * APITCH + KC * BPITCH;

  // acc[u] += A[row0 + 16 wr .., 0 .. K) * B[0 .. K, col0[wj * NTW + u] .. + 16).  Rows >= n_rows read as zero and so
  // do the columns of tile t from col_end[t] on.  K, lda, ldb, col0[], col_end[] are multiples of 4 and A, B are
  // 16-byte aligned, so every 16-byte fetch is entirely inside or entirely outside.
  static __device__ __forceinline__ void mma(const float* __restrict__ A, int lda, int row0, int n_rows,
                                             const float* __restrict__ B, int ldb, const int (&col0)[NT],
                                             const int (&col_end)[NT], int K, float* smem, f4 (&acc)[NTW]) {
    float* As = smem;
    float* Bs = smem + GS_ROWS * APITCH;
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wr = wave & 1, wj = wave >> 1;
    const int m = lane & 15, kq = lane >> 4;
    // what this lane fetches of every chunk: fixed (row, k offset) pairs of A and (k, column) pairs of B
    int a_off[A_PER], a_kc[A_PER], b_col[B_PER], b_k[B_PER];
    bool a_ok[A_PER], b_ok[B_PER];
#pragma unroll
    for (int i = 0; i < A_PER; ++i) {
      const int v = tid + i * GS_THREADS;
      const int r = v / (KC / 4);
      a_kc[i] = (v % (KC / 4)) * 4;
      a_ok[i] = v < A_VECS && row0 + r < n_rows;
      a_off[i] = min(row0 + r, n_rows - 1) * lda;
    }
#pragma unroll
    for (int i = 0; i < B_PER; ++i) {
      const int v = tid + i * GS_THREADS;
      const int c4 = v % (COLS / 4), t = c4 / 4;
      b_k[i] = v / (COLS / 4);
      int c0 = col0[0], ce = col_end[0];
#pragma unroll
      for (int u = 1; u < NT; ++u) { c0 = t == u ? col0[u] : c0; ce = t == u ? col_end[u] : ce; }
      const int col = c0 + (c4 % 4) * 4;
      b_ok[i] = v < B_VECS && col < ce;
      b_col[i] = b_ok[i] ? col : 0;
    }
    // Loads are issued unconditionally from clamped (always valid) addresses and the out-of-range parts are zeroed
    // only when the chunk is written to LDS, so nothing waits on a load before the chunk is needed.
    f4 ra[A_PER], rb[B_PER];
    auto fetch = [&](int k0) {
#pragma unroll
      for (int i = 0; i < A_PER; ++i) ra[i] = ld4(A + (long)a_off[i] + min(k0 + a_kc[i], K - 4));
#pragma unroll
      for (int i = 0; i < B_PER; ++i) rb[i] = ld4(B + (long)min(k0 + b_k[i], K - 1) * ldb + b_col[i]);
    };
    auto stage = [&](int k0) {
#pragma unroll
      for (int i = 0; i < A_PER; ++i) {
        const int v = tid + i * GS_THREADS;
        const f4 x = (a_ok[i] && k0 + a_kc[i] < K) ? ra[i] : f4{0.f, 0.f, 0.f, 0.f};
        if (A_VECS % GS_THREADS == 0 || v < A_VECS) st4(As + (v / (KC / 4)) * APITCH + a_kc[i], x);
      }
#pragma unroll
      for (int i = 0; i < B_PER; ++i) {
        const int v = tid + i * GS_THREADS;
        const f4 x = (b_ok[i] && k0 + b_k[i] < K) ? rb[i] : f4{0.f, 0.f, 0.f, 0.f};
        if (B_VECS % GS_THREADS == 0 || v < B_VECS) st4(Bs + b_k[i] * BPITCH + (v % (COLS / 4)) * 4, x);
      }
    };
    fetch(0);
    const float* ap = As + (wr * 16 + m) * APITCH + kq;
    const float* bp = Bs + kq * BPITCH + wj * NTW * 16 + m;
    for (int k0 = 0; k0 < K; k0 += KC) {
      __syncthreads();               // the previous chunk has been consumed
      stage(k0);
      __syncthreads();
      fetch(k0 + KC);                // past the end this re-reads the last rows (clamped); never staged
      __builtin_amdgcn_sched_barrier(0);
      // operands of contraction step s + 1 are read from LDS while the matrix instructions of step s run
      float a_cur = ap[0], b_cur[NTW];
#pragma unroll
      for (int u = 0; u < NTW; ++u) b_cur[u] = bp[16 * u];
#pragma unroll
      for (int s4 = 0; s4 < KC / 4; ++s4) {
        float a_nxt = 0.f, b_nxt[NTW];
        if (s4 + 1 < KC / 4) {
          a_nxt = ap[4 * (s4 + 1)];
#pragma unroll
          for (int u = 0; u < NTW; ++u) b_nxt[u] = bp[4 * (s4 + 1) * BPITCH + 16 * u];
        }
#pragma unroll
        for (int u = 0; u < NTW; ++u) acc[u] = __builtin_amdgcn_mfma_f32_16x16x4f32(a_cur, b_cur[u], acc[u], 0, 0, 0);
        __builtin_amdgcn_sched_group_barrier(0x100, 1 + NTW, 0);    // next step's LDS reads ...
        __builtin_amdgcn_sched_group_barrier(0x008, NTW, 0);        // ... then this step's matrix instructions
        if (s4 + 1 < KC / 4) {
          a_cur = a_nxt;
#pragma unroll
          for (int u = 0; u < NTW; ++u) b_cur[u] = b_nxt[u];
        }
      }
    }
  }
};

// The same accumulation for an operand pair that is contiguous along the contraction on BOTH sides: A[row, k] and
// Bt[col, k] (D[row, col] += sum_k A[row, k] Bt[col, k]).  Both are staged row-major with the contraction index
// innermost, so one 16-byte LDS read per operand feeds four matrix instructions: lane (m, kq) of group g reads
// k = 16 g + 4 kq .. + 3 and uses component i in instruction i, which then contracts over {16 g + 4 kq' + i} - the
// order of the sum inside a group of 16 is permuted, nothing else.  The backward step uses it (A = dgh of the next
// step, Bt = the rows of W_hh itself), where one instruction per contraction step would leave the LDS latency bare.
template <int NTW, int KC>
struct StepTileKK {
  static constexpr int NT = 2 * NTW;
  static constexpr int PITCH = KC + 4;
  static constexpr int BROWS = 16 * NT;
  static constexpr int A_VECS = GS_ROWS * KC / 4, B_VECS = BROWS * KC / 4;
  static constexpr int A_PER = (A_VECS + GS_THREADS - 1) / GS_THREADS, B_PER = (B_VECS + GS_THREADS - 1) / GS_THREADS;
  static constexpr int LDS_FLOATS = (GS_ROWS + BROWS) * PITCH;
  static_assert(KC % 16 == 0 && A_VECS % GS_THREADS == 0 && B_VECS % GS_THREADS == 0, "chunk shape");

  // acc[u] += A[row0 + 16 wr .., 0 .. K) * Bt[col0[wj * NTW + u] .. + 16, 0 .. K)^T.  Rows >= n_rows and Bt rows from
  // col_end[t] on read as zero; K, lda, ldbt multiples of 4, A and Bt 16-byte aligned.
  static __device__ __forceinline__ void mma(const float* __restrict__ A, int lda, int row0, int n_rows,
                                             const float* __restrict__ Bt, int ldbt, const int (&col0)[NT],
                                             const int (&col_end)[NT], int K, float* smem, f4 (&acc)[NTW]) {
    float* As = smem;
    float* Bs = smem + GS_ROWS * PITCH;
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wr = wave & 1, wj = wave >> 1;
    const int m = lane & 15, kq = lane >> 4;
    int a_off[A_PER], a_kc[A_PER], b_off[B_PER], b_kc[B_PER];
    bool a_ok[A_PER], b_ok[B_PER];
#pragma unroll
    for (int i = 0; i < A_PER; ++i) {
      const int v = tid + i * GS_THREADS;
      const int r = v / (KC / 4);
      a_kc[i] = (v % (KC / 4)) * 4;
      a_ok[i] = row0 + r < n_rows;
      a_off[i] = min(row0 + r, n_rows - 1) * lda;
    }
#pragma unroll
    for (int i = 0; i < B_PER; ++i) {
      const int v = tid + i * GS_THREADS;
      const int c = v / (KC / 4), t = c / 16;
      b_kc[i] = (v % (KC / 4)) * 4;
      int c0 = col0[0], ce = col_end[0];
#pragma unroll
      for (int u = 1; u < NT; ++u) { c0 = t == u ? col0[u] : c0; ce = t == u ? col_end[u] : ce; }
      const int col = c0 + (c % 16);
      b_ok[i] = col < ce;
      b_off[i] = min(col, ce - 1) * ldbt;           // clamped: always a valid row
    }
    f4 ra[A_PER], rb[B_PER];
    auto fetch = [&](int k0) {      // unconditional loads from clamped addresses; zeroing happens at staging time
#pragma unroll
      for (int i = 0; i < A_PER; ++i) ra[i] = ld4(A + (long)a_off[i] + min(k0 + a_kc[i], K - 4));
#pragma unroll
      for (int i = 0; i < B_PER; ++i) rb[i] = ld4(Bt + (long)b_off[i] + min(k0 + b_kc[i], K - 4));
    };
    auto stage = [&](int k0) {
#pragma unroll
      for (int i = 0; i < A_PER; ++i) {
        const int v = tid + i * GS_THREADS;
        st4(As + (v / (KC / 4)) * PITCH + a_kc[i], (a_ok[i] && k0 + a_kc[i] < K) ? ra[i] : f4{0.f, 0.f, 0.f, 0.f});
      }
#pragma unroll
      for (int i = 0; i < B_PER; ++i) {
        const int v = tid + i * GS_THREADS;
        st4(Bs + (v / (KC / 4)) * PITCH + b_kc[i], (b_ok[i] && k0 + b_kc[i] < K) ? rb[i] : f4{0.f, 0.f, 0.f, 0.f});
      }
    };
    const float* ap = As + (wr * 16 + m) * PITCH + 4 * kq;
    const float* bp = Bs + (wj * NTW * 16 + m) * PITCH + 4 * kq;
    fetch(0);
    for (int k0 = 0; k0 < K; k0 += KC) {
      __syncthreads();               // the previous chunk has been consumed
      stage(k0);
      __syncthreads();
      fetch(k0 + KC);                // past the end this re-reads clamped addresses; never staged
      __builtin_amdgcn_sched_barrier(0);
      f4 a_cur = ld4(ap), b_cur[NTW];
#pragma unroll
      for (int u = 0; u < NTW; ++u) b_cur[u] = ld4(bp + u * 16 * PITCH);
#pragma unroll
      for (int g = 0; g < KC / 16; ++g) {
        f4 a_nxt = a_cur, b_nxt[NTW];
#pragma unroll
        for (int u = 0; u < NTW; ++u) b_nxt[u] = b_cur[u];
        if (g + 1 < KC / 16) {
          a_nxt = ld4(ap + 16 * (g + 1));
#pragma unroll
          for (int u = 0; u < NTW; ++u) b_nxt[u] = ld4(bp + u * 16 * PITCH + 16 * (g + 1));
        }
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
          for (int u = 0; u < NTW; ++u) acc[u] = __builtin_amdgcn_mfma_f32_16x16x4f32(a_cur[i], b_cur[u][i], acc[u], 0, 0, 0);
        a_cur = a_nxt;
#pragma unroll
        for (int u = 0; u < NTW; ++u) b_cur[u] = b_nxt[u];
      }
    }
  }
};

// Workgroup -> (row block, hidden-unit block).  Consecutive workgroup ids are dealt round-robin to the 8 XCDs, each
// with an L2 of its own: all hidden-unit blocks of a row block go to one XCD, so a row block's operand rows are
// fetched into one L2 only (the weights, shared by every row block, fit in each L2).
constexpr int GS_XCDS = 8;
__device__ __forceinline__ void step_block(int H, int& rb, int& jb) {
  const int jblocks = (H + GS_JB - 1) / GS_JB;
  const int xcd = (int)blockIdx.x % GS_XCDS, i = (int)blockIdx.x / GS_XCDS;
  rb = (i / jblocks) * GS_XCDS + xcd;
  jb = i % jblocks;
}

template <int CELL> struct CellShape;
template <> struct CellShape<CELL_GRU> { static constexpr int G = 3, KC = 128; };
template <> struct CellShape<CELL_LSTM> { static constexpr int G = 4, KC = 64; };   // shorter chunks: 8 tiles of weights in LDS

template <int CELL>
__global__ __launch_bounds__(GS_THREADS) void step_fwd_kernel(const StepFwdArgs a) {
  constexpr int G = CellShape<CELL>::G;
  using Tile = StepTile<G, CellShape<CELL>::KC>;
  __shared__ __attribute__((aligned(16))) float smem[Tile::LDS_FLOATS];
  const int z = blockIdx.y;
  const StepFwdNet& n = a.net[z];
  const int H = n.H, nb = a.nb, S = CELL == CELL_LSTM ? 2 * H : H;
  int rb, jb;
  step_block(H, rb, jb);
  const int row0 = rb * GS_ROWS, j0 = jb * GS_JB;
  if (row0 >= nb) return;
  int col0[2 * G], col_end[2 * G];      // tile wj * G + g: gate g of hidden units j0 + 16 wj ...
#pragma unroll
  for (int t = 0; t < 2 * G; ++t) { col0[t] = (t % G) * H + j0 + (t / G) * 16; col_end[t] = (t % G) * H + H; }
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wr = wave & 1, wj = wave >> 1;
  const int j = j0 + wj * 16 + (lane & 15), jc = min(j, H - 1);
  const int rbase = row0 + wr * 16 + 4 * (lane >> 4);
  // the gate stage's own operands do not depend on the contraction: fetch them first (clamped addresses, no
  // branches) so their latency hides behind it
  float pgi[4][G], pst[4];      // pst: the state entry the gates blend with (GRU: h, LSTM: c)
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    const int row = min(rbase + q, nb - 1);
    const long og = (long)row * G * H + jc;
#pragma unroll
    for (int g = 0; g < G; ++g) pgi[q][g] = n.gi[og + g * H];
    pst[q] = n.sin[(long)row * S + (CELL == CELL_LSTM ? H : 0) + jc];
  }
  float bias[G];
#pragma unroll
  for (int g = 0; g < G; ++g) bias[g] = n.b_hh[g * H + jc];
  f4 acc[G];
#pragma unroll
  for (int t = 0; t < G; ++t) acc[t] = f4{0.f, 0.f, 0.f, 0.f};
  Tile::mma(n.sin, S, row0, nb, n.w_hh, G * H, col0, col_end, H, smem, acc);
  if (j >= H) return;
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    const int row = rbase + q;
    if (row >= nb) continue;
    const long og = (long)row * G * H + j;
    float keep = 1.0f;
    if (n.sin_next != nullptr && a.done != nullptr) keep = a.done[a.done_idx ? a.done_idx[row] : row] ? 0.0f : 1.0f;
    if (CELL == CELL_GRU) {
      const float ghr = acc[0][q] + bias[0], ghz = acc[1][q] + bias[1], ghn = acc[2][q] + bias[2];
      const float r = sigmoidf_(pgi[q][0] + ghr);
      const float zz = sigmoidf_(pgi[q][1] + ghz);
      const float nn = tanhf_(pgi[q][2] + r * ghn);
      const float h = (1.0f - zz) * nn + zz * pst[q];
      n.h_out[(long)row * n.ld_out + j] = h;
      if (n.sin_next != nullptr) n.sin_next[(long)row * S + j] = h * keep;
      if (n.pre_out != nullptr) { n.pre_out[og] = ghr; n.pre_out[og + H] = ghz; n.pre_out[og + 2 * H] = ghn; }
    } else {
      float pre[G];
#pragma unroll
      for (int g = 0; g < G; ++g) pre[g] = pgi[q][g] + acc[g][q] + bias[g];
      const float ii = sigmoidf_(pre[0]), ff = sigmoidf_(pre[1]), gg = tanhf_(pre[2]), oo = sigmoidf_(pre[3]);
      const float c = ff * pst[q] + ii * gg;
      const float h = oo * tanhf_(c);
      n.h_out[(long)row * n.ld_out + j] = h;
      if (n.c_out != nullptr) n.c_out[(long)row * n.ld_out + j] = c;
      if (n.sin_next != nullptr) { n.sin_next[(long)row * S + j] = h * keep; n.sin_next[(long)row * S + H + j] = c * keep; }
      if (n.pre_out != nullptr) {
#pragma unroll
        for (int g = 0; g < G; ++g) n.pre_out[og + g * H] = pre[g];
      }
    }
  }
}

template <int CELL>
__global__ __launch_bounds__(GS_THREADS) void step_bwd_kernel(const StepBwdArgs a) {
  constexpr int G = CellShape<CELL>::G;
  using Tile = StepTileKK<1, 128>;
  __shared__ __attribute__((aligned(16))) float smem[Tile::LDS_FLOATS];
  const int z = blockIdx.y;
  const StepBwdNet& n = a.net[z];
  const int H = n.H, nb = a.nb, S = CELL == CELL_LSTM ? 2 * H : H;
  int rb, jb;
  step_block(H, rb, jb);
  const int row0 = rb * GS_ROWS, j0 = jb * GS_JB;
  if (row0 >= nb) return;
  const bool has_next = n.dg_next != nullptr;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wr = wave & 1, wj = wave >> 1;
  const int j = j0 + wj * 16 + (lane & 15), jc = min(j, H - 1);
  const int rbase = row0 + wr * 16 + 4 * (lane >> 4);
  // the gate stage's own operands, fetched ahead of the contraction (clamped addresses, no branches)
  float pgi[4][G], ppre[4][G], pst[4], pdh[4], pcarry[4];
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    const int row = min(rbase + q, nb - 1);
    const long o = (long)row * H + jc, og = (long)row * G * H + jc;
#pragma unroll
    for (int g = 0; g < G; ++g) {
      ppre[q][g] = n.pre[og + g * H];
      pgi[q][g] = CELL == CELL_GRU ? n.gi[og + g * H] : 0.f;
    }
    pst[q] = n.sin[(long)row * S + (CELL == CELL_LSTM ? H : 0) + jc];
    pdh[q] = n.dh_ext[o];
    pcarry[q] = has_next ? n.carry[o] : 0.f;
  }
  f4 acc[1] = {f4{0.f, 0.f, 0.f, 0.f}};
  if (has_next) {
    const int col0[2] = {j0, j0 + 16}, col_end[2] = {H, H};      // rows of W_hh = hidden units
    Tile::mma(n.dg_next, G * H, row0, nb, n.w_hh, G * H, col0, col_end, G * H, smem, acc);
  }
  if (j >= H) return;
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    const int row = rbase + q;
    if (row >= nb) continue;
    const long o = (long)row * H + j, og = (long)row * G * H + j;
    float keep = 1.0f;
    if (has_next && a.done != nullptr) keep = a.done[a.done_idx ? a.done_idx[row] : row] ? 0.0f : 1.0f;
    if (CELL == CELL_GRU) {
      float dh = pdh[q];
      if (has_next) dh += (acc[0][q] + pcarry[q]) * keep;
      const float ghn = ppre[q][2];
      const float r = sigmoidf_(pgi[q][0] + ppre[q][0]);
      const float zz = sigmoidf_(pgi[q][1] + ppre[q][1]);
      const float nn = tanhf_(pgi[q][2] + r * ghn);
      const float dn = dh * (1.0f - zz);
      const float dz = dh * (pst[q] - nn);
      const float dn_pre = dn * (1.0f - nn * nn);
      const float dr_pre = dn_pre * ghn * r * (1.0f - r);
      const float dz_pre = dz * zz * (1.0f - zz);
      n.carry[o] = dh * zz;
      n.dgi[og] = dr_pre; n.dgi[og + H] = dz_pre; n.dgi[og + 2 * H] = dn_pre;
      n.dg[og] = dr_pre; n.dg[og + H] = dz_pre; n.dg[og + 2 * H] = dn_pre * r;
    } else {
      float dh = pdh[q], dc = 0.f;
      if (has_next) { dh += acc[0][q] * keep; dc = pcarry[q] * keep; }
      const float ii = sigmoidf_(ppre[q][0]), ff = sigmoidf_(ppre[q][1]), gg = tanhf_(ppre[q][2]), oo = sigmoidf_(ppre[q][3]);
      const float tc = tanhf_(ff * pst[q] + ii * gg);
      const float d_o = dh * tc;
      const float dct = dc + dh * oo * (1.0f - tc * tc);
      n.carry[o] = dct * ff;
      n.dg[og] = dct * gg * ii * (1.0f - ii);
      n.dg[og + H] = dct * pst[q] * ff * (1.0f - ff);
      n.dg[og + 2 * H] = dct * ii * (1.0f - gg * gg);
      n.dg[og + 3 * H] = d_o * oo * (1.0f - oo);
    }
  }
}

__global__ __launch_bounds__(256) void row_gather_kernel(const RowGatherArgs a) {
  const RowGatherJob& J = a.job[blockIdx.y];
  const int q = J.H >> 2;
  const long e = (long)blockIdx.x * 256 + threadIdx.x;
  if (e >= (long)a.nb * q) return;
  const int i = (int)(e / q), j = (int)(e - (long)i * q) * 4;
  const int src = a.idx ? a.idx[i] : i;
  f4 v = ld4(J.src + (long)src * J.H + j);
  if (a.reset != nullptr && a.reset[i]) v = f4{0.f, 0.f, 0.f, 0.f};
  st4(J.dst + (long)i * J.H + j, v);
  if (J.dst2 != nullptr) st4(J.dst2 + (long)i * J.H + j, v);
}

__global__ __launch_bounds__(256) void copy_matrix_kernel(const float* __restrict__ src, int ld_src, int rows, int cols,
                                                          float* __restrict__ dst) {
  const int q = cols >> 2;
  const long e = (long)blockIdx.x * 256 + threadIdx.x;
  if (e >= (long)rows * q) return;
  const int r = (int)(e / q), c = (int)(e - (long)r * q) * 4;
  st4(dst + (long)r * cols + c, ld4(src + (long)r * ld_src + c));
}

__global__ __launch_bounds__(256) void column_rows_kernel(const int32_t* __restrict__ perm, int E, int M, int T, int N,
                                                          int32_t* __restrict__ rows_out) {
  const long total = (long)E * T * N;
  const long o = (long)blockIdx.x * 256 + threadIdx.x;
  if (o >= total) return;
  const int nb = N / M;
  const int i = (int)(o % nb);
  long r = o / nb;
  const int t = (int)(r % T); r /= T;
  const int m = (int)(r % M);
  const int e = (int)(r / M);
  rows_out[o] = t * N + perm[(long)e * N + (long)m * nb + i];
}

}  // namespace

static dim3 step_grid(int nb, const int* H, int n_nets) {
  int blocks = 0;
  for (int k = 0; k < n_nets; ++k) {
    const int rblocks = ((nb + GS_ROWS - 1) / GS_ROWS + GS_XCDS - 1) / GS_XCDS * GS_XCDS;   // see step_block
    const int b = rblocks * ((H[k] + GS_JB - 1) / GS_JB);
    blocks = b > blocks ? b : blocks;
  }
  return dim3(blocks, n_nets);
}

hipError_t launch_step_fwd(const StepFwdArgs& a, hipStream_t stream) {
  if (a.nb <= 0 || a.n_nets <= 0) return hipSuccess;
  const int G = a.cell == CELL_LSTM ? 4 : 3;
  int H[2] = {a.net[0].H, a.net[1].H};
  double flops = 0.0;
  for (int k = 0; k < a.n_nets; ++k) flops += 2.0 * a.nb * H[k] * (double)G * H[k];
  TraceScope ts(stream, a.cell == CELL_LSTM ? "lstm_step_fwd" : "gru_step_fwd", flops, 0.0);
  const dim3 grid = step_grid(a.nb, H, a.n_nets);
  if (a.cell == CELL_LSTM) hipLaunchKernelGGL(step_fwd_kernel<CELL_LSTM>, grid, dim3(GS_THREADS), 0, stream, a);
  else hipLaunchKernelGGL(step_fwd_kernel<CELL_GRU>, grid, dim3(GS_THREADS), 0, stream, a);
  return hipGetLastError();
}

hipError_t launch_step_bwd(const StepBwdArgs& a, hipStream_t stream) {
  if (a.nb <= 0 || a.n_nets <= 0) return hipSuccess;
  const int G = a.cell == CELL_LSTM ? 4 : 3;
  int H[2] = {a.net[0].H, a.net[1].H};
  double flops = 0.0;
  for (int k = 0; k < a.n_nets; ++k) flops += a.net[k].dg_next ? 2.0 * a.nb * H[k] * (double)G * H[k] : 0.0;
  TraceScope ts(stream, a.cell == CELL_LSTM ? "lstm_step_bwd" : "gru_step_bwd", flops, 0.0);
  const dim3 grid = step_grid(a.nb, H, a.n_nets);
  if (a.cell == CELL_LSTM) hipLaunchKernelGGL(step_bwd_kernel<CELL_LSTM>, grid, dim3(GS_THREADS), 0, stream, a);
  else hipLaunchKernelGGL(step_bwd_kernel<CELL_GRU>, grid, dim3(GS_THREADS), 0, stream, a);
  return hipGetLastError();
}

hipError_t launch_row_gather(const RowGatherArgs& a, hipStream_t stream) {
  long work = 0;
  for (int k = 0; k < a.n_jobs; ++k) { const long w = (long)a.nb * (a.job[k].H >> 2); work = w > work ? w : work; }
  if (work == 0) return hipSuccess;
  hipLaunchKernelGGL(row_gather_kernel, dim3((unsigned)((work + 255) / 256), a.n_jobs), dim3(256), 0, stream, a);
  return hipGetLastError();
}

hipError_t launch_copy_matrix(const float* src, int32_t ld_src, int32_t rows, int32_t cols, float* dst, hipStream_t stream) {
  const long total = (long)rows * (cols >> 2);
  if (total == 0) return hipSuccess;
  hipLaunchKernelGGL(copy_matrix_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, stream, src, ld_src, rows, cols, dst);
  return hipGetLastError();
}

hipError_t launch_column_rows(const int32_t* perm, int32_t E, int32_t M, int32_t T, int32_t N, int32_t* rows_out,
                              hipStream_t stream) {
  const long total = (long)E * T * N;
  if (total == 0) return hipSuccess;
  hipLaunchKernelGGL(column_rows_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, stream, perm, E, M, T, N, rows_out);
  return hipGetLastError();
}

}  // namespace rslx
