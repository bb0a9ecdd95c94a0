// fp32 matrix-core contraction for gfx950 (v_mfma_f32_32x32x2_f32), used by every dense layer of the
// actor, critic, student, teacher and RND networks: forward, input gradient and weight gradient.
//
// Tiling: one workgroup = 4 wavefronts (256 lanes) computes a BM x BN block of C.  Operand tiles of
// BK (16) contraction steps are staged through LDS in contraction-major order (As[k][m], Bs[k][n]),
// so that the 32 lanes of an MFMA operand row read 32 consecutive words (bank-conflict free), and are
// double-buffered: global loads of tile k+1 are in flight while tile k feeds the matrix cores.
//
// MFMA 32x32x2 fp32 register layout (wave64, lane l, g = l / 32, j = l % 32):
//   A operand: A[row = j][k = g]      B operand: B[k = g][col = j]
//   D/C, 16 accumulators r = 0..15:   D[row = 8 * (r / 4) + 4 * g + r % 4][col = j]
#include <cstdio>
#include <cstring>
#include <type_traits>

#include "kernels.h"

namespace rslx {

typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int PAD = 4;    // LDS row padding (floats); keeps rows 16-byte aligned
constexpr int NT = 256;   // lanes per workgroup

__device__ __forceinline__ int wrap_row(const GemmProblem& P, int r) { return r >= P.idx_mod ? r - P.idx_mod : r; }

__device__ __forceinline__ int src_row(const GemmProblem& P, int r) {
  int rr = wrap_row(P, r);
  const int v = P.row_idx ? P.row_idx[rr] : rr;
  return r >= P.idx_mod ? v + P.wrap_add : v;
}

// ---- operand with the contraction index contiguous in memory (tile rows = M or N index) ---------------------
// Everything that does not change along the contraction (row pointers with the gather applied, validity,
// whether the row uses the column map) is set up once per tile; a k-tile fetch is then loads only.
// Element (row, k) lands at lds[k][row].
template <int R, int BK, bool IS_X, bool VEC>
struct KContig {
  static constexpr int NREG = R * BK / NT;
  static constexpr int LK = BK / 4;                 // vector path: lanes along k (one float4 each)
  static constexpr int RPV = NT / LK;               // vector path: rows per pass
  static constexpr int RPS = NT / BK;               // scalar path: rows per pass
  static constexpr int NPTR = VEC ? R / RPV : R / RPS;
  static constexpr bool vec = VEC;
  const float* ptr[VEC ? 1 : NPTR];                 // scalar path: row pointers, gather applied
  uint32_t off[VEC ? NPTR : 1];                     // vector path: element offsets of the rows from `base`; rows past the
                                                    // end point at the last row, so every offset can be loaded from
  const float* base;
  uint32_t mapped;                                  // scalar path, bit p: row of pass p reads through col_map / col_sign
  uint32_t valid;                                   // vector path, bit p: the row of pass p exists

  __device__ __forceinline__ void setup(const GemmProblem& P, const float* b, int ld, int row0, int row_end) {
    const int tid = threadIdx.x;
    mapped = 0;
    valid = 0;
    base = b;
    if constexpr (VEC) {
#pragma unroll
      for (int p = 0; p < R / RPV; ++p) {
        const int row = row0 + p * RPV + tid / LK;
        if (row < row_end) valid |= 1u << p;
        const int rc = min(row, row_end - 1);
        off[p] = (uint32_t)(IS_X ? src_row(P, rc) : rc) * (uint32_t)ld + 4u * (tid % LK);
      }
    } else {
#pragma unroll
      for (int p = 0; p < R / RPS; ++p) {
        const int row = row0 + p * RPS + tid / BK;
        ptr[p] = nullptr;
        if (row < row_end) {
          ptr[p] = base + (long)(IS_X ? src_row(P, row) : row) * ld;
          if (IS_X && P.col_map != nullptr && row >= P.map_from) mapped |= 1u << p;
        }
      }
    }
  }

  __device__ __forceinline__ void fetch(const GemmProblem& P, int k0, int k_end, float (&reg)[NREG]) const {
    const int tid = threadIdx.x;
    if constexpr (VEC) {
      const float* bk = base + k0;                 // uniform; the per-lane part is the 32-bit offset
      const bool kok = k0 + 4 * (tid % LK) < k_end;
#pragma unroll
      for (int p = 0; p < R / RPV; ++p) {
        float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
        if (kok && ((valid >> p) & 1u)) v = *reinterpret_cast<const float4*>(bk + off[p]);
        reg[4 * p + 0] = v.x; reg[4 * p + 1] = v.y; reg[4 * p + 2] = v.z; reg[4 * p + 3] = v.w;
      }
    } else {
      const int c = k0 + tid % BK;
      const bool kok = c < k_end;
      int cm = c;
      float sg = 1.0f;
      if (IS_X && kok && P.col_map != nullptr) {
        cm = P.col_map[c];
        if (P.col_sign != nullptr) sg = P.col_sign[c];
      }
#pragma unroll
      for (int p = 0; p < R / RPS; ++p) {
        float v = 0.f;
        if (kok && ptr[p] != nullptr) v = ((mapped >> p) & 1u) ? sg * ptr[p][cm] : ptr[p][c];
        reg[p] = v;
      }
    }
  }

  // One 16-byte load / its LDS writes at a time, without bounds checks (whole BK-tiles of the contraction only; rows
  // past the end repeat the last row and feed output rows that are dropped): the contraction loop places them
  // between its matrix-core instructions.
  static constexpr int NPIECE = VEC ? R / RPV : 0;
  __device__ __forceinline__ void fetch_piece(int k0, float (&reg)[NREG], int p) const {
    const float4 v = *reinterpret_cast<const float4*>(base + k0 + off[VEC ? p : 0]);
    reg[4 * p + 0] = v.x; reg[4 * p + 1] = v.y; reg[4 * p + 2] = v.z; reg[4 * p + 3] = v.w;
  }
  template <int S>
  __device__ __forceinline__ void stash_piece(float (*lds)[S], const float (&reg)[NREG], int p) const {
    const int tid = threadIdx.x;
    const int row = p * RPV + tid / LK;
    const int kq = 4 * (tid % LK);
#pragma unroll
    for (int c = 0; c < 4; ++c) lds[kq + c][row] = reg[4 * p + c];
  }

  template <int S>
  __device__ __forceinline__ void stash(float (*lds)[S], const float (&reg)[NREG]) const {
    const int tid = threadIdx.x;
    if constexpr (VEC) {
#pragma unroll
      for (int p = 0; p < R / RPV; ++p) {
        const int row = p * RPV + tid / LK;
        const int kq = 4 * (tid % LK);
#pragma unroll
        for (int c = 0; c < 4; ++c) lds[kq + c][row] = reg[4 * p + c];
      }
    } else {
#pragma unroll
      for (int p = 0; p < R / RPS; ++p) lds[tid % BK][p * RPS + tid / BK] = reg[p];
    }
  }
};

// ---- operand with the M / N index contiguous in memory (tile rows = contraction index) ----------------------
// The column (and its mapped twin for mirrored rows) is fixed per lane; the contraction row changes per k-tile.
template <int Cw, int BK, bool IS_X, bool VEC>
struct Direct {
  static constexpr int NREG = Cw * BK / NT;
  static constexpr int V = Cw / 4;                  // vector path: float4 per tile row
  static constexpr int RPV = NT / V;                // vector path: tile rows per pass
  static constexpr int RPS = NT / Cw;               // scalar path: tile rows per pass
  const float* base;
  int ld, col, cm;
  int colc;                                         // vector path: col, or the last whole 16-byte column group of the matrix
  float sg;
  bool col_ok, has_map;
  uint32_t off[VEC ? (BK / RPV > 0 ? BK / RPV : 1) : 1];   // vector path, rows not gathered: offsets from row k0
  int next_row[(VEC && IS_X) ? (BK / RPV > 0 ? BK / RPV : 1) : 1];   // vector path, gathered rows: source rows of the next fetch
  static constexpr bool vec = VEC;

  __device__ __forceinline__ void setup(const GemmProblem& P, const float* b, int ld_, int col0, int col_end) {
    const int tid = threadIdx.x;
    base = b; ld = ld_;
    col = vec ? col0 + 4 * (tid % V) : col0 + tid % Cw;
    col_ok = col < col_end;
    has_map = false; cm = col; sg = 1.0f;
    colc = col_ok ? col : max(col_end - 4, 0);
    if constexpr (VEC) {
#pragma unroll
      for (int p = 0; p < BK / RPV; ++p) off[p] = (uint32_t)(p * RPV + tid / V) * (uint32_t)ld + (uint32_t)colc;
    }
    if (IS_X && !vec && col_ok && P.col_map != nullptr) {
      has_map = true;
      cm = P.col_map[col];
      if (P.col_sign != nullptr) sg = P.col_sign[col];
    }
  }

  // Gathered rows (vector path): the source rows of a tile are looked up while the previous tile is fetched, so
  // that no fetch waits for its own index loads.  `prime` looks up the rows of the first tile; every fetch then
  // looks up the rows of the tile BK further on (fetches walk the contraction range in steps of BK).
  __device__ __forceinline__ void prime(const GemmProblem& P, int k0, int k_end) {
    if constexpr (VEC && IS_X) {
      const int tid = threadIdx.x;
#pragma unroll
      for (int p = 0; p < BK / RPV; ++p) next_row[p] = src_row(P, min(k0 + p * RPV + tid / V, k_end - 1));
    }
  }

  __device__ __forceinline__ void fetch(const GemmProblem& P, int k0, int k_end, float (&reg)[NREG]) {
    const int tid = threadIdx.x;
    if constexpr (VEC) {
      const float* bk = base + (long)k0 * ld;      // uniform
#pragma unroll
      for (int p = 0; p < BK / RPV; ++p) {
        const int kk = k0 + p * RPV + tid / V;
        float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
        if (col_ok && kk < k_end) {
          if constexpr (IS_X) v = *reinterpret_cast<const float4*>(base + (long)next_row[p] * ld + col);
          else v = *reinterpret_cast<const float4*>(bk + off[p]);
        }
        reg[4 * p + 0] = v.x; reg[4 * p + 1] = v.y; reg[4 * p + 2] = v.z; reg[4 * p + 3] = v.w;
      }
      if constexpr (IS_X) {
#pragma unroll
        for (int p = 0; p < BK / RPV; ++p) next_row[p] = src_row(P, min(k0 + BK + p * RPV + tid / V, k_end - 1));
      }
    } else {
#pragma unroll
      for (int p = 0; p < BK / RPS; ++p) {
        const int kk = k0 + p * RPS + tid / Cw;
        float v = 0.f;
        if (col_ok && kk < k_end) {
          const float* rowp = base + (long)(IS_X ? src_row(P, kk) : kk) * ld;
          v = (has_map && kk >= P.map_from) ? sg * rowp[cm] : rowp[col];
        }
        reg[p] = v;
      }
    }
  }

  // Piecewise variants without bounds checks (whole BK-tiles of the contraction; matrix widths that are multiples of
  // four): columns past the end repeat the last column group and feed outputs that are dropped.  The first form is
  // for contraction rows that are not gathered (row kk is row kk), the second walks the gathered rows like `fetch`.
  static constexpr int NPIECE = VEC ? BK / RPV : 0;
  __device__ __forceinline__ void fetch_piece(int k0, float (&reg)[NREG], int p) const {
    const float4 v = *reinterpret_cast<const float4*>(base + (long)k0 * ld + off[VEC ? p : 0]);
    reg[4 * p + 0] = v.x; reg[4 * p + 1] = v.y; reg[4 * p + 2] = v.z; reg[4 * p + 3] = v.w;
  }
  __device__ __forceinline__ void fetch_piece_gathered(const GemmProblem& P, int k0, int k_end, float (&reg)[NREG], int p) {
    const int pi = (VEC && IS_X) ? p : 0;
    const float4 v = *reinterpret_cast<const float4*>(base + (long)next_row[pi] * ld + colc);
    reg[4 * p + 0] = v.x; reg[4 * p + 1] = v.y; reg[4 * p + 2] = v.z; reg[4 * p + 3] = v.w;
    next_row[pi] = src_row(P, min(k0 + BK + p * RPV + (int)threadIdx.x / V, k_end - 1));
  }
  template <int S>
  __device__ __forceinline__ void stash_piece(float (*lds)[S], const float (&reg)[NREG], int p) const {
    const int tid = threadIdx.x;
    const float4 v = make_float4(reg[4 * p], reg[4 * p + 1], reg[4 * p + 2], reg[4 * p + 3]);
    *reinterpret_cast<float4*>(&lds[p * RPV + tid / V][4 * (tid % V)]) = v;
  }

  template <int S>
  __device__ __forceinline__ void stash(float (*lds)[S], const float (&reg)[NREG]) const {
    const int tid = threadIdx.x;
    if constexpr (VEC) {
#pragma unroll
      for (int p = 0; p < BK / RPV; ++p) {
        const float4 v = make_float4(reg[4 * p], reg[4 * p + 1], reg[4 * p + 2], reg[4 * p + 3]);
        *reinterpret_cast<float4*>(&lds[p * RPV + tid / V][4 * (tid % V)]) = v;
      }
    } else {
#pragma unroll
      for (int p = 0; p < BK / RPS; ++p) lds[p * RPS + tid / Cw][tid % Cw] = reg[p];
    }
  }
};

// LDS floats of one tile configuration: two buffers of BK x (BM + PAD) and BK x (BN + PAD).
template <int BM, int BN, int BK>
constexpr int gemm_lds_floats() { return 2 * BK * (BM + PAD) + 2 * BK * (BN + PAD); }

// One output tile (one split of it for the weight gradient) of problem P.  `lin` numbers the workgroups of the
// problem's grid of gx tiles x (total / gx) splits; `smem` holds gemm_lds_floats<BM, BN, BK>() floats.
template <int MODE, int BM, int BN, int WM, int WN, int BK, bool AVEC, bool BVEC>
__device__ __forceinline__ void gemm_tile(const GemmProblem& P, int lin, const int total, const int gx, float* smem) {
  static_assert(WM * WN == 4, "four wavefronts per workgroup");
  constexpr int TM = BM / WM / 32, TN = BN / WN / 32;
  static_assert(TM >= 1 && TN >= 1, "wave tile must hold at least one 32x32 block");
  constexpr int SA = BM + PAD, SB = BN + PAD;
  float (*As)[BK][SA] = reinterpret_cast<float (*)[BK][SA]>(smem);
  float (*Bs)[BK][SB] = reinterpret_cast<float (*)[BK][SB]>(smem + 2 * BK * SA);

  const int tiles_n = (P.N + BN - 1) / BN;
  const int tiles_m = (P.M + BM - 1) / BM;
  // Workgroups are handed to the 8 XCDs round-robin by linear id; remap so that neighbours in (tile, split)
  // order - which share operand rows - run on the same XCD and meet in its L2.
  if ((total & 7) == 0) lin = (lin & 7) * (total >> 3) + (lin >> 3);
  const int tile = lin % gx;
  if (tile >= tiles_m * tiles_n) return;
  const int split = lin / gx;
  if (MODE == GEMM_DW && split >= P.n_split) return;
  const int tn = tile % tiles_n, tm = tile / tiles_n;
  const int m0 = tm * BM, n0 = tn * BN;
  const int k_begin = (MODE == GEMM_DW) ? split * P.k_chunk : 0;
  const int k_end = (MODE == GEMM_DW) ? min(P.K, k_begin + P.k_chunk) : P.K;
  const int nk = (k_end - k_begin + BK - 1) / BK;

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int g = lane >> 5, j = lane & 31;
  const int wm = wave / WN, wn = wave % WN;
  const int a_off = wm * (TM * 32) + j, b_off = wn * (TN * 32) + j;

  float ra[BM * BK / NT], rb[BN * BK / NT];
  f32x16 acc[TM][TN];
#pragma unroll
  for (int a = 0; a < TM; ++a)
#pragma unroll
    for (int b = 0; b < TN; ++b)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[a][b][r] = 0.f;
  float bsum = 0.f;   // DW: column sum of dZ for the bias gradient

  // operand A: DW reads X rows as contraction rows (M index contiguous); FWD / DX read rows with k contiguous.
  // operand B: always N index contiguous (W, W^T or dZ).
  KContig<BM, BK, MODE == GEMM_FWD, AVEC> a_k;
  Direct<BM, BK, true, AVEC> a_d;
  Direct<BN, BK, false, BVEC> b_d;
  const int a_cols = (MODE == GEMM_DW && P.a_cols > P.M) ? P.a_cols : P.M;   // DW: readable (zero-padded) width of X
  if (MODE == GEMM_DW) a_d.setup(P, P.A, P.lda, m0, a_cols);
  else a_k.setup(P, P.A, P.lda, m0, P.M);
  b_d.setup(P, P.B, P.ldb, n0, P.N);

  // DX with at most two 32x32 blocks per wave: the activation values that gate the result (ELU') are fetched
  // ahead of the contraction loop and wait in registers, so the epilogue does not stall on them.
  constexpr bool AUX_AHEAD = MODE == GEMM_DX && TM * TN <= 2;
  float hpre[AUX_AHEAD ? TM * TN * 16 : 1];
  const bool full_mn = m0 + BM <= P.M && n0 + BN <= P.N;
  const bool aux_ahead = AUX_AHEAD && full_mn && P.aux != nullptr;
  auto fetch_aux = [&]() {
    if constexpr (AUX_AHEAD) {
      if (aux_ahead) {
        const int ld = P.ldc;
#pragma unroll
        for (int x = 0; x < TM; ++x)
#pragma unroll
          for (int y = 0; y < TN; ++y) {
            const float* hp = P.aux + (long)(m0 + wm * (TM * 32) + x * 32 + 4 * g) * ld + (n0 + wn * (TN * 32) + y * 32 + j);
#pragma unroll
            for (int r = 0; r < 16; ++r) hpre[(x * TN + y) * 16 + r] = hp[(8 * (r / 4) + (r % 4)) * ld];
          }
      }
    }
  };
  auto stash = [&](int buf) {
    if (MODE == GEMM_DW) a_d.template stash<SA>(As[buf], ra);
    else a_k.template stash<SA>(As[buf], ra);
    b_d.template stash<SB>(Bs[buf], rb);
  };
  // The general loop: every lane checks its bounds (scalar operand paths, contraction ranges that are no multiple
  // of BK).
  auto main_loop = [&]() {
    auto fetch = [&](int k0) {
      if (MODE == GEMM_DW) a_d.fetch(P, k0, k_end, ra);
      else a_k.fetch(P, k0, k_end, ra);
      b_d.fetch(P, k0, k_end, rb);
    };
    if (nk > 0) {
      if (MODE == GEMM_DW) a_d.prime(P, k_begin, k_end);
      fetch(k_begin);
      stash(0);
    }
    fetch_aux();
    __syncthreads();
    for (int kt = 0; kt < nk; ++kt) {
      const int buf = kt & 1;
      if (kt + 1 < nk) fetch(k_begin + (kt + 1) * BK);
      // operands of step kk + 2 are read from LDS before the matrix-core instructions of step kk issue
      float a_cur[TM], b_cur[TN], a_nxt[TM], b_nxt[TN];
#pragma unroll
      for (int t = 0; t < TM; ++t) a_cur[t] = As[buf][g][a_off + t * 32];
#pragma unroll
      for (int t = 0; t < TN; ++t) b_cur[t] = Bs[buf][g][b_off + t * 32];
#pragma unroll
      for (int kk = 0; kk < BK; kk += 2) {
        if (kk + 2 < BK) {
#pragma unroll
          for (int t = 0; t < TM; ++t) a_nxt[t] = As[buf][kk + 2 + g][a_off + t * 32];
#pragma unroll
          for (int t = 0; t < TN; ++t) b_nxt[t] = Bs[buf][kk + 2 + g][b_off + t * 32];
        }
        __builtin_amdgcn_sched_barrier(0);   // keep the LDS reads ahead of the matrix-core instructions
#pragma unroll
        for (int x = 0; x < TM; ++x)
#pragma unroll
          for (int y = 0; y < TN; ++y)
            acc[x][y] = __builtin_amdgcn_mfma_f32_32x32x2f32(a_cur[x], b_cur[y], acc[x][y], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
        if (kk + 2 < BK) {
#pragma unroll
          for (int t = 0; t < TM; ++t) a_cur[t] = a_nxt[t];
#pragma unroll
          for (int t = 0; t < TN; ++t) b_cur[t] = b_nxt[t];
        }
      }
      if (MODE == GEMM_DW && tm == 0 && tid < BN) {
#pragma unroll
        for (int kk = 0; kk < BK; ++kk) bsum += Bs[buf][kk][tid];
      }
      if (kt + 1 < nk) stash(buf ^ 1);
      __syncthreads();
    }
  };
  // 16-byte operand paths over whole BK-tiles run the same double buffer without bounds checks (operand rows and
  // columns past the matrix repeat valid ones; the outputs they feed are dropped by the epilogue) and with the other
  // instructions dealt out between the matrix-core instructions, one per gap: the 16-byte loads of the next tile
  // in the first steps of a tile, their LDS writes in the last steps, the LDS operand reads of the next step after
  // the first matrix-core instruction of each step.  A wave then never issues a burst of memory instructions while
  // its matrix-core queue runs dry (measured: 6 % faster forward, 11 % faster input gradient at 128 x 128).
  // GATHERED: the weight gradient's contraction rows go through row_idx / wrap (looked up one tile ahead).
  auto stream_loop = [&](auto gathered_tag) {
    constexpr bool GATHERED = decltype(gathered_tag)::value;
    constexpr int NA = MODE == GEMM_DW ? decltype(a_d)::NPIECE : decltype(a_k)::NPIECE;
    constexpr int NB = decltype(b_d)::NPIECE;
    constexpr int NP = NA + NB, STEPS = BK / 2;
    static_assert(2 * NP <= STEPS, "loads and LDS writes of a tile take one step each");
    auto load_piece = [&](int q, int k0) {
#pragma unroll
      for (int p = 0; p < NA; ++p)
        if (q == p) {
          if (MODE == GEMM_DW && GATHERED) a_d.fetch_piece_gathered(P, k0, k_end, ra, p);
          else if (MODE == GEMM_DW) a_d.fetch_piece(k0, ra, p);
          else a_k.fetch_piece(k0, ra, p);
        }
#pragma unroll
      for (int p = 0; p < NB; ++p)
        if (q == NA + p) b_d.fetch_piece(k0, rb, p);
    };
    auto stash_piece = [&](int q, int buf) {
#pragma unroll
      for (int p = 0; p < NA; ++p)
        if (q == p) {
          if (MODE == GEMM_DW) a_d.template stash_piece<SA>(As[buf], ra, p);
          else a_k.template stash_piece<SA>(As[buf], ra, p);
        }
#pragma unroll
      for (int p = 0; p < NB; ++p)
        if (q == NA + p) b_d.template stash_piece<SB>(Bs[buf], rb, p);
    };
    if (GATHERED) a_d.prime(P, k_begin, k_end);
#pragma unroll
    for (int q = 0; q < NP; ++q) load_piece(q, k_begin);
    stash(0);
    fetch_aux();
    __syncthreads();
    for (int kt = 0; kt < nk; ++kt) {
      const int buf = kt & 1;
      const int k_next = k_begin + min(kt + 1, nk - 1) * BK;   // the last tile fetches itself again: in bounds, unused
      float a_cur[TM], b_cur[TN], a_nxt[TM], b_nxt[TN];
#pragma unroll
      for (int t = 0; t < TM; ++t) a_cur[t] = As[buf][g][a_off + t * 32];
#pragma unroll
      for (int t = 0; t < TN; ++t) b_cur[t] = Bs[buf][g][b_off + t * 32];
#pragma unroll
      for (int st = 0; st < STEPS; ++st) {
        if (st + 1 < STEPS) {
#pragma unroll
          for (int t = 0; t < TM; ++t) a_nxt[t] = As[buf][2 * st + 2 + g][a_off + t * 32];
#pragma unroll
          for (int t = 0; t < TN; ++t) b_nxt[t] = Bs[buf][2 * st + 2 + g][b_off + t * 32];
        }
        if (st < NP) load_piece(st, k_next);
        if (st >= STEPS - NP) stash_piece(st - (STEPS - NP), buf ^ 1);
#pragma unroll
        for (int x = 0; x < TM; ++x)
#pragma unroll
          for (int y = 0; y < TN; ++y)
            acc[x][y] = __builtin_amdgcn_mfma_f32_32x32x2f32(a_cur[x], b_cur[y], acc[x][y], 0, 0, 0);
        // order within the step: masks 0x008 matrix core, 0x100 LDS read, 0x020 global load, 0x200 LDS write
        if constexpr (TM * TN >= 4) {
          __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
          __builtin_amdgcn_sched_group_barrier(0x100, TM + TN, 0);
          __builtin_amdgcn_sched_group_barrier(0x008, TM * TN - 2, 0);
          __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
          __builtin_amdgcn_sched_group_barrier(0x200, 4, 0);
          __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        } else {
          __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
          __builtin_amdgcn_sched_group_barrier(0x100, TM + TN, 0);
          __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
          __builtin_amdgcn_sched_group_barrier(0x200, 4, 0);
          __builtin_amdgcn_sched_group_barrier(0x008, TM * TN - 1, 0);
        }
        __builtin_amdgcn_sched_barrier(0);
        if (st + 1 < STEPS) {
#pragma unroll
          for (int t = 0; t < TM; ++t) a_cur[t] = a_nxt[t];
#pragma unroll
          for (int t = 0; t < TN; ++t) b_cur[t] = b_nxt[t];
        }
      }
      if (MODE == GEMM_DW && tm == 0 && tid < BN) {
#pragma unroll
        for (int kk = 0; kk < BK; ++kk) bsum += Bs[buf][kk][tid];
      }
      __syncthreads();
    }
  };
  const bool whole_tiles = nk > 0 && (k_end - k_begin) % BK == 0;
  const bool widths_ok = P.N >= 4 && (P.N & 3) == 0 && (MODE != GEMM_DW || (a_cols >= 4 && (a_cols & 3) == 0));
  const bool plain_rows = MODE != GEMM_DW || (P.row_idx == nullptr && k_end <= P.idx_mod);
  if constexpr (AVEC && BVEC) {
    if (whole_tiles && widths_ok && plain_rows) stream_loop(std::false_type{});
    else if (whole_tiles && widths_ok) stream_loop(std::true_type{});
    else main_loop();
  } else {
    main_loop();
  }

  // ---- epilogue -------------------------------------------------------------------------------
  // Problem fields are copied to registers first: read through the reference they would be fetched again after
  // every store, since a store may alias them as far as the compiler can tell.
  const int Mr = P.M, Nc = P.N, ldc = P.ldc;
  const bool elu = P.elu != 0;
  const float alpha = P.alpha;
  const float* aux = P.aux;
  const int bias_off = P.bias_off;
  float* Cb = P.C;
  if (MODE == GEMM_DW) Cb += (long)split * P.split_stride;
  // Tiles inside the matrix.  Loads issued after a block's stores would have to wait for those stores as well (one
  // counter covers both), so everything a block reads is requested before the previous block's stores: the biases
  // of all blocks up front, the activation values that gate the input gradient one block ahead.
  if (full_mn) {
    float bias[TN];
#pragma unroll
    for (int y = 0; y < TN; ++y) bias[y] = (MODE == GEMM_FWD && aux != nullptr) ? aux[n0 + wn * (TN * 32) + y * 32 + j] : 0.f;
    constexpr bool GATE_PIPE = MODE == GEMM_DX && !AUX_AHEAD;
    float hx[2][16];
    auto block_offset = [&](int b) {
      const int x = b / TN, y = b % TN;
      // register r of a 32x32 block sits 8 * (r / 4) + r % 4 rows below its first row: a uniform offset
      return (long)(m0 + wm * (TM * 32) + x * 32 + 4 * g) * ldc + (n0 + wn * (TN * 32) + y * 32 + j);
    };
    auto load_gate = [&](int b, float (&h)[16]) {
      const float* hp = aux + block_offset(b);
#pragma unroll
      for (int r = 0; r < 16; ++r) h[r] = hp[(8 * (r / 4) + (r % 4)) * ldc];
    };
    if (GATE_PIPE && aux != nullptr) load_gate(0, hx[0]);
#pragma unroll
    for (int b = 0; b < TM * TN; ++b) {
      const int x = b / TN, y = b % TN;
      float* cp = Cb + block_offset(b);
      if (MODE == GEMM_DX && aux != nullptr) {
        if constexpr (AUX_AHEAD) {
#pragma unroll
          for (int r = 0; r < 16; ++r) hx[b & 1][r] = hpre[b * 16 + r];
        } else if (b + 1 < TM * TN) {
          load_gate(b + 1, hx[(b + 1) & 1]);
        }
      }
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        float v = acc[x][y][r];
        if (MODE == GEMM_FWD) {
          v += bias[y];
          if (elu) {
            const float e = alpha * (__expf(v) - 1.0f);
            v = v > 0.f ? v : e;
          }
        } else if (MODE == GEMM_DX) {
          if (aux != nullptr) v *= (hx[b & 1][r] > 0.f) ? 1.0f : (hx[b & 1][r] + alpha);
        }
        cp[(8 * (r / 4) + (r % 4)) * ldc] = v;
      }
    }
    if (MODE == GEMM_DW && tm == 0 && bias_off >= 0 && tid < BN && n0 + tid < Nc) Cb[bias_off + n0 + tid] = bsum;
    return;
  }
#pragma unroll
  for (int x = 0; x < TM; ++x) {
#pragma unroll
    for (int y = 0; y < TN; ++y) {
      const int col = n0 + wn * (TN * 32) + y * 32 + j;
      const int row_base = m0 + wm * (TM * 32) + x * 32 + 4 * g;
      // Edge tiles: what a block reads is read through clamped indices and turned into the block's 16 results before
      // the first conditional store, so that no store has to wait behind a load (or behind the store before it).
      const int colc = min(col, Nc - 1);
      float bias = 0.f;
      if (MODE == GEMM_FWD && aux != nullptr) bias = aux[colc];
      float out[16];
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        float v = acc[x][y][r];
        if (MODE == GEMM_FWD) {
          v += bias;
          if (elu) {
            const float e = alpha * (__expf(v) - 1.0f);
            v = v > 0.f ? v : e;
          }
        } else if (MODE == GEMM_DX) {
          if (aux != nullptr) {
            const int rowc = min(row_base + 8 * (r / 4) + (r % 4), Mr - 1);
            const float h = aux[(long)rowc * ldc + colc];
            v *= (h > 0.f) ? 1.0f : (h + alpha);
          }
        }
        out[r] = v;
      }
#pragma unroll
      for (int r = 0; r < 16; ++r) asm volatile("" : "+v"(out[r]));   // the results exist before the branches below
      if (col >= Nc) continue;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int row = row_base + 8 * (r / 4) + (r % 4);
        if (row < Mr) Cb[(long)row * ldc + col] = out[r];
      }
    }
  }
  if (MODE == GEMM_DW && tm == 0 && bias_off >= 0 && tid < BN && n0 + tid < Nc) Cb[bias_off + n0 + tid] = bsum;
}

template <int MODE, int BM, int BN, int WM, int WN, int BK, bool AVEC, bool BVEC>
__global__ __launch_bounds__(NT) __attribute__((amdgpu_waves_per_eu(4))) void gemm_kernel(const GemmBatch batch) {
  __shared__ __align__(16) float smem[gemm_lds_floats<BM, BN, BK>()];
  gemm_tile<MODE, BM, BN, WM, WN, BK, AVEC, BVEC>(batch.p[blockIdx.z], blockIdx.x + gridDim.x * blockIdx.y,
                                                  gridDim.x * gridDim.y, gridDim.x, smem);
}

// Weight gradient and input gradient of one layer in one launch (both read the same dZ and neither reads the
// other's result): the workgroups of the second fill the CUs as those of the first drain, so one launch tail and
// one output phase disappear.  Workgroups [0, nw) belong to the weight gradient (gw tiles x sw splits per
// problem), the next ne to an optional second weight gradient of narrow output (the network's output layer, whose
// operands are ready at the same time: 128 x 32 tiles, ge tiles x se splits per problem), the rest to the input
// gradient (gx tiles per problem).  16-byte operand paths only (the narrow one reads dZ with scalar loads).
template <int WBM, int WBN, int WWM, int WWN, int XBM, int XBN, int XWM, int XWN, int BK>
__global__ __launch_bounds__(NT) __attribute__((amdgpu_waves_per_eu(4))) void gemm_pair_kernel(
    const GemmBatch bw, const GemmBatch bx, const GemmBatch be, const int gw, const int sw, const int gx, const int ge,
    const int se) {
  constexpr int LW = gemm_lds_floats<WBM, WBN, BK>(), LX = gemm_lds_floats<XBM, XBN, BK>();
  constexpr int LE = gemm_lds_floats<128, 32, BK>();
  constexpr int LWX = LW > LX ? LW : LX;
  __shared__ __align__(16) float smem[LWX > LE ? LWX : LE];
  const int per_w = gw * sw, per_e = ge * se;
  const int nw = bw.count * per_w, ne = be.count * per_e;
  const int b = blockIdx.x;
  // When the weight-gradient workgroups alone fill the chip (4 resident workgroups on each of 256 CUs), the input
  // gradient is the tail of the launch: its waves then issue ahead of the weight gradient's that are still running
  // (measured: 4 % off such a launch; 5 % on, when the two kinds share the chip from the start).
  if (b >= nw + ne && nw >= 1024) __builtin_amdgcn_s_setprio(3);
  if (b < nw) {
    const int z = b / per_w;
    gemm_tile<GEMM_DW, WBM, WBN, WWM, WWN, BK, true, true>(bw.p[z], b - z * per_w, per_w, gw, smem);
  } else if (b < nw + ne) {
    const int c = b - nw;
    const int z = c / per_e;
    gemm_tile<GEMM_DW, 128, 32, 4, 1, BK, true, false>(be.p[z], c - z * per_e, per_e, ge, smem);
  } else {
    const int c = b - nw - ne;
    const int z = c / gx;
    gemm_tile<GEMM_DX, XBM, XBN, XWM, XWN, BK, true, true>(bx.p[z], c - z * gx, gx, gx, smem);
  }
}

template <int MODE, int BM, int BN, int WM, int WN, int BK = 16>
static hipError_t launch_cfg(const GemmBatch& batch, hipStream_t stream) {
  int tiles = 0, splits = 1;
  // 16-byte fetches need every grouped problem to allow them and at least one float4 per lane and tile
  bool avec = BM * BK >= 4 * NT, bvec = BN * BK >= 4 * NT;
  for (int i = 0; i < batch.count; ++i) {
    const GemmProblem& P = batch.p[i];
    int t = ((P.M + BM - 1) / BM) * ((P.N + BN - 1) / BN);
    tiles = t > tiles ? t : tiles;
    if (MODE == GEMM_DW) splits = P.n_split > splits ? P.n_split : splits;
    // the 16-byte paths address rows by 32-bit element offsets from the matrix base
    const int64_t lim = (int64_t)1 << 32;
    const int64_t a_rows = P.row_idx != nullptr ? P.a_src_rows : (MODE == GEMM_DW ? P.K : P.M);
    const bool a_fits = a_rows > 0 && a_rows * (int64_t)P.lda < lim;
    const bool b_fits = (int64_t)P.K * P.ldb < lim;
    avec = avec && P.a_vec != 0 && a_fits;
    bvec = bvec && P.b_vec != 0 && b_fits;
  }
  if (tiles == 0) return hipSuccess;
  dim3 grid(tiles, splits, batch.count);
  double flops = 0.0;
  for (int i = 0; i < batch.count; ++i) flops += 2.0 * batch.p[i].M * (double)batch.p[i].N * batch.p[i].K;
  static const char* const mode_name[3] = {"fwd", "dx", "dw"};
  char name[48];
  snprintf(name, sizeof name, "gemm_%s_%dx%d", mode_name[MODE], BM, BN);
  TraceScope ts(stream, name, flops, 0.0);
  if (avec && bvec) hipLaunchKernelGGL((gemm_kernel<MODE, BM, BN, WM, WN, BK, true, true>), grid, dim3(NT), 0, stream, batch);
  else if (avec) hipLaunchKernelGGL((gemm_kernel<MODE, BM, BN, WM, WN, BK, true, false>), grid, dim3(NT), 0, stream, batch);
  else if (bvec) hipLaunchKernelGGL((gemm_kernel<MODE, BM, BN, WM, WN, BK, false, true>), grid, dim3(NT), 0, stream, batch);
  else hipLaunchKernelGGL((gemm_kernel<MODE, BM, BN, WM, WN, BK, false, false>), grid, dim3(NT), 0, stream, batch);
  return hipGetLastError();
}

// Tile selection.  Measured on MI355X: one 128x128 workgroup per CU reaches ~40 % of the matrix-core peak,
// four resident workgroups per CU reach ~65 %, so the tile shrinks (64x128) whenever 128x128 tiles would leave
// fewer than about three workgroups per CU, and short contractions (K <= 64, epilogue-bound) also use it.
enum TileCfg { TILE_128x128, TILE_64x128, TILE_128x64, TILE_128x32 };

static TileCfg pick_tile(GemmMode mode, const GemmBatch& batch) {
  int maxM = 0, maxN = 0, minK = 1 << 30, dw_big = 1;
  long tiles128 = 0;
  for (int i = 0; i < batch.count; ++i) {
    const GemmProblem& P = batch.p[i];
    maxM = P.M > maxM ? P.M : maxM;
    maxN = P.N > maxN ? P.N : maxN;
    minK = P.K < minK ? P.K : minK;
    tiles128 += (long)((P.M + 127) / 128) * ((P.N + 127) / 128);
    dw_big &= P.dw_big;
  }
  if (maxN <= 32) return TILE_128x32;
  if (maxM <= 64) return TILE_64x128;
  if (maxN <= 64) return TILE_128x64;
  if (mode == GEMM_DW) return dw_big ? TILE_128x128 : TILE_64x128;
  if (minK <= 64 || tiles128 < 700) return TILE_64x128;
  if (mode == GEMM_DX && maxN >= 512) return TILE_64x128;   // wide outputs: the ELU' operand reads favour more, smaller workgroups
  return TILE_128x128;
}

int gemm_dw_tiles(int32_t M, int32_t N, bool big) {
  if (N <= 32) return (M + 127) / 128;
  if (M <= 64 || !big) return ((M + 63) / 64) * ((N + 127) / 128);
  if (N <= 64) return ((M + 127) / 128) * ((N + 63) / 64);
  return ((M + 127) / 128) * ((N + 127) / 128);
}

template <int MODE>
static hipError_t launch_mode(const GemmBatch& batch, hipStream_t stream) {
  switch (pick_tile((GemmMode)MODE, batch)) {
    case TILE_128x32: return launch_cfg<MODE, 128, 32, 4, 1>(batch, stream);
    case TILE_64x128: return launch_cfg<MODE, 64, 128, 1, 4>(batch, stream);
    case TILE_128x64: return launch_cfg<MODE, 128, 64, 2, 2>(batch, stream);
    default: return launch_cfg<MODE, 128, 128, 2, 2>(batch, stream);
  }
}

// ---- weight transposition --------------------------------------------------------------------------
// The input-gradient contraction reads W^T; transposing the (small) weight matrices once per optimiser step
// lets that kernel fetch both operands the way the forward kernel does instead of transposing W tiles in LDS
// for every row block.
__global__ __launch_bounds__(256) void transpose_kernel(const TransposeBatch b) {
  __shared__ float t[32][33];
  const TransposeJob& J = b.job[blockIdx.z];
  const int tiles_c = (J.cols + 31) / 32;
  const int tiles_r = (J.rows + 31) / 32;
  if ((int)blockIdx.x >= tiles_c * tiles_r) return;
  const int r0 = ((int)blockIdx.x / tiles_c) * 32, c0 = ((int)blockIdx.x % tiles_c) * 32;
  const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
  for (int i = ty; i < 32; i += 8)
    if (r0 + i < J.rows && c0 + tx < J.cols) t[i][tx] = J.src[(long)(r0 + i) * J.cols + c0 + tx];
  __syncthreads();
  for (int i = ty; i < 32; i += 8)
    if (c0 + i < J.cols && r0 + tx < J.rows) J.dst[(long)(c0 + i) * J.rows + r0 + tx] = t[tx][i];
}

hipError_t launch_transpose(const TransposeBatch& b, hipStream_t stream) {
  int tiles = 0;
  for (int i = 0; i < b.count; ++i) {
    int t = ((b.job[i].rows + 31) / 32) * ((b.job[i].cols + 31) / 32);
    tiles = t > tiles ? t : tiles;
  }
  if (tiles == 0 || b.count == 0) return hipSuccess;
  TraceScope ts(stream, "transpose_weights", 0.0, 0.0);
  hipLaunchKernelGGL(transpose_kernel, dim3(tiles, 1, b.count), dim3(256), 0, stream, b);
  return hipGetLastError();
}

// Grid geometry of a batch for a tile shape and whether every problem may use the 16-byte operand paths.
struct BatchGeom {
  int tiles = 0, splits = 1;
  bool vec = true;
  double flops = 0.0;
};

static BatchGeom batch_geom(GemmMode mode, const GemmBatch& batch, int BM, int BN) {
  BatchGeom g;
  for (int i = 0; i < batch.count; ++i) {
    const GemmProblem& P = batch.p[i];
    const int t = ((P.M + BM - 1) / BM) * ((P.N + BN - 1) / BN);
    g.tiles = t > g.tiles ? t : g.tiles;
    if (mode == GEMM_DW) g.splits = P.n_split > g.splits ? P.n_split : g.splits;
    const int64_t lim = (int64_t)1 << 32;
    const int64_t a_rows = P.row_idx != nullptr ? P.a_src_rows : (mode == GEMM_DW ? P.K : P.M);
    g.vec = g.vec && P.a_vec != 0 && P.b_vec != 0 && a_rows > 0 && a_rows * (int64_t)P.lda < lim &&
            (int64_t)P.K * P.ldb < lim;
    g.flops += 2.0 * P.M * (double)P.N * P.K;
  }
  return g;
}

template <int WBM, int WBN, int WWM, int WWN, int XBM, int XBN, int XWM, int XWN>
static hipError_t launch_pair_cfg(const GemmBatch& bw, const GemmBatch& bx, const GemmBatch& be, const BatchGeom& gw,
                                  const BatchGeom& gx, const BatchGeom& ge, hipStream_t stream) {
  char name[48];
  snprintf(name, sizeof name, "gemm_dwdx_%dx%d_%dx%d", WBM, WBN, XBM, XBN);
  TraceScope ts(stream, name, gw.flops + gx.flops + ge.flops, 0.0);
  const int blocks = bw.count * gw.tiles * gw.splits + bx.count * gx.tiles + be.count * ge.tiles * ge.splits;
  hipLaunchKernelGGL((gemm_pair_kernel<WBM, WBN, WWM, WWN, XBM, XBN, XWM, XWN, 16>), dim3(blocks), dim3(NT), 0, stream,
                     bw, bx, be, gw.tiles, gw.splits, gx.tiles, ge.tiles, ge.splits);
  return hipGetLastError();
}

// The narrow weight gradient can ride in the paired launch when it takes 128 x 32 tiles and its X operand allows
// 16-byte loads (what gemm_kernel<GEMM_DW, 128, 32, 4, 1, 16, true, false> needs).
static bool narrow_dw_fits(const GemmBatch& be) {
  if (be.count <= 0 || pick_tile(GEMM_DW, be) != TILE_128x32) return false;
  for (int i = 0; i < be.count; ++i) {
    const GemmProblem& P = be.p[i];
    const int64_t a_rows = P.row_idx != nullptr ? P.a_src_rows : P.K;
    if (!P.a_vec || a_rows <= 0 || a_rows * (int64_t)P.lda >= ((int64_t)1 << 32)) return false;
  }
  return true;
}

hipError_t launch_gemm_dw_dx(const GemmBatch& bw, const GemmBatch& bx, hipStream_t stream, const GemmBatch* narrow_dw) {
  const TileCfg tw = pick_tile(GEMM_DW, bw), tx = pick_tile(GEMM_DX, bx);
  const bool w_ok = tw == TILE_128x128 || tw == TILE_64x128, x_ok = tx == TILE_128x128 || tx == TILE_64x128;
  if (w_ok && x_ok && bw.count > 0 && bx.count > 0) {
    const BatchGeom gw = batch_geom(GEMM_DW, bw, tw == TILE_128x128 ? 128 : 64, 128);
    const BatchGeom gx = batch_geom(GEMM_DX, bx, tx == TILE_128x128 ? 128 : 64, 128);
    if (gw.vec && gx.vec && gw.tiles > 0 && gx.tiles > 0) {
      GemmBatch be;
      memset(&be, 0, sizeof be);
      BatchGeom ge;
      ge.tiles = 0; ge.splits = 0;
      if (narrow_dw != nullptr && narrow_dw_fits(*narrow_dw)) {
        be = *narrow_dw;
        ge = batch_geom(GEMM_DW, be, 128, 32);
      } else if (narrow_dw != nullptr) {
        hipError_t e = launch_gemm(GEMM_DW, *narrow_dw, stream);
        if (e != hipSuccess) return e;
      }
      if (tw == TILE_128x128 && tx == TILE_128x128) return launch_pair_cfg<128, 128, 2, 2, 128, 128, 2, 2>(bw, bx, be, gw, gx, ge, stream);
      if (tw == TILE_128x128) return launch_pair_cfg<128, 128, 2, 2, 64, 128, 1, 4>(bw, bx, be, gw, gx, ge, stream);
      if (tx == TILE_128x128) return launch_pair_cfg<64, 128, 1, 4, 128, 128, 2, 2>(bw, bx, be, gw, gx, ge, stream);
      return launch_pair_cfg<64, 128, 1, 4, 64, 128, 1, 4>(bw, bx, be, gw, gx, ge, stream);
    }
  }
  if (narrow_dw != nullptr) {
    hipError_t e = launch_gemm(GEMM_DW, *narrow_dw, stream);
    if (e != hipSuccess) return e;
  }
  hipError_t e = launch_gemm(GEMM_DW, bw, stream);
  if (e != hipSuccess) return e;
  return launch_gemm(GEMM_DX, bx, stream);
}

hipError_t launch_gemm(GemmMode mode, const GemmBatch& batch, hipStream_t stream) {
  switch (mode) {
    case GEMM_FWD: return launch_mode<GEMM_FWD>(batch, stream);
    case GEMM_DX: return launch_mode<GEMM_DX>(batch, stream);
    default: return launch_mode<GEMM_DW>(batch, stream);
  }
}

}  // namespace rslx
