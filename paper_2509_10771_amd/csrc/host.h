// Host-side helpers shared by the entry-point files of librslx (api.hip, api_recurrent.hip): error reporting,
// workspace carving, launch sequencing of MLP forward / backward passes, split-gradient planning and reduction.
// Not part of the public ABI (that is include/rslx.h).
#pragma once

#include <climits>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <string>
#include <vector>

#include "../../include/rslx.h"
#include "kernels.h"

namespace rslx {
namespace host {

inline thread_local std::string g_last_error;

inline int32_t fail(int32_t code, const char* fmt, ...) {
  char buf[512];
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(buf, sizeof buf, fmt, ap);
  va_end(ap);
  g_last_error = buf;
  return code;
}

#define RSLX_HIP(expr)                                                                    \
  do {                                                                                    \
    hipError_t e_ = (expr);                                                               \
    if (e_ != hipSuccess) return fail(RSLX_ERR_HIP, "%s: %s", #expr, hipGetErrorString(e_)); \
  } while (0)

#define RSLX_TRY(expr)             \
  do {                             \
    int32_t rc_ = (expr);          \
    if (rc_ != RSLX_OK) return rc_; \
  } while (0)

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

inline uint64_t mix64_host(uint64_t x) {
  x += 0x9E3779B97F4A7C15ull;
  x = (x ^ (x >> 30)) * 0xBF58476D1CE4E5B9ull;
  x = (x ^ (x >> 27)) * 0x94D049BB133111EBull;
  return x ^ (x >> 31);
}

// ---- workspace carving: the same code sizes the workspace (base == nullptr) and hands out pointers ----
struct Carver {
  char* base;
  size_t off = 0;
  explicit Carver(void* b) : base(static_cast<char*>(b)) {}
  template <typename T>
  T* take(size_t count) {
    off = (off + 255) / 256 * 256;
    T* p = base ? reinterpret_cast<T*>(base + off) : nullptr;
    off += count * sizeof(T);
    return p;
  }
};

// ---- network helpers ---------------------------------------------------------------------------------
inline int64_t layer_offset(const rslx_mlp& n, int l) {
  int64_t o = 0;
  for (int i = 0; i < l; ++i) o += (int64_t)n.dims[i] * n.dims[i + 1] + n.dims[i + 1];
  return o;
}
inline int64_t weight_count(const rslx_mlp& n) { return layer_offset(n, n.n_layers); }
inline int64_t param_count(const rslx_mlp& n) { return weight_count(n) + (n.has_log_std ? n.dims[n.n_layers] : 0); }

inline int32_t check_mlp(const rslx_mlp* n, const char* name, bool trainable) {
  if (!n) return fail(RSLX_ERR_INVALID_ARG, "%s: null network", name);
  if (n->n_layers < 1 || n->n_layers > RSLX_MAX_LAYERS) return fail(RSLX_ERR_SHAPE, "%s: n_layers %d out of range", name, n->n_layers);
  for (int i = 0; i <= n->n_layers; ++i)
    if (n->dims[i] < 1 || n->dims[i] > (1 << 20)) return fail(RSLX_ERR_SHAPE, "%s: dims[%d] = %d", name, i, n->dims[i]);
  if (!n->params || !aligned16(n->params)) return fail(RSLX_ERR_INVALID_ARG, "%s: params null or not 16-byte aligned", name);
  if (trainable) {
    if (!n->grads || !n->adam_m || !n->adam_v) return fail(RSLX_ERR_INVALID_ARG, "%s: grads / adam_m / adam_v required", name);
    if (!aligned16(n->grads) || !aligned16(n->adam_m) || !aligned16(n->adam_v))
      return fail(RSLX_ERR_INVALID_ARG, "%s: optimiser buffers not 16-byte aligned", name);
  }
  return RSLX_OK;
}

// View of a network's input matrix (see GemmProblem in kernels.h).
struct XView {
  const float* base = nullptr;
  int ld = 0;
  const int32_t* row_idx = nullptr;
  const int32_t* col_map = nullptr;
  const float* col_sign = nullptr;
  int idx_mod = INT_MAX;
  int map_from = INT_MAX;
  int64_t src_rows = 0;     // rows of the matrix behind row_idx
  int wrap_add = 0;         // rows past idx_mod read this many rows further down (staged mirrored copy)
  int cols = 0;             // staged input: zero-padded width of the rows (a multiple of 16), 0 = the network's input width
};

// Staged network input (see launch_stage_input): worth it when the rows cannot be fetched 16 bytes at a time, when
// their width is no whole number of contraction tiles, or when mirrored rows would go through a column map.  The
// first layer then contracts over the padded width, which reads rows of W past its end: those meet zero columns,
// but they must lie inside the parameter buffer.
inline int staged_width(const rslx_mlp& n, int32_t ld, bool mirrored) {
  const int D = n.dims[0];
  if (!mirrored && D % 16 == 0 && ld % 4 == 0) return 0;
  const int Dp = (D + 15) / 16 * 16;
  if ((int64_t)Dp * n.dims[1] > weight_count(n)) return 0;
  return Dp;
}

// Per-network activation storage for `rows` rows: out[l] = output of layer l, dz[l] = gradient w.r.t. the
// pre-activation of hidden layer l.  The caller may point out[last] at its own buffer.
struct NetBufs {
  float* out[RSLX_MAX_LAYERS] = {};
  float* dz[RSLX_MAX_LAYERS] = {};
};

inline void carve_net(Carver& c, const rslx_mlp& n, int64_t rows, bool backward, NetBufs& b) {
  for (int l = 0; l < n.n_layers; ++l) b.out[l] = c.take<float>((size_t)rows * n.dims[l + 1]);
  if (backward)
    for (int l = 0; l + 1 < n.n_layers; ++l) b.dz[l] = c.take<float>((size_t)rows * n.dims[l + 1]);
}

inline GemmProblem blank_problem() {
  GemmProblem p;
  memset(&p, 0, sizeof p);
  p.idx_mod = INT_MAX;
  p.map_from = INT_MAX;
  p.bias_off = -1;
  p.n_split = 1;
  return p;
}

inline void set_x(GemmProblem& p, const XView& x) {
  p.A = x.base; p.lda = x.ld; p.row_idx = x.row_idx; p.col_map = x.col_map; p.col_sign = x.col_sign;
  p.idx_mod = x.idx_mod; p.map_from = x.map_from; p.a_src_rows = x.src_rows; p.wrap_add = x.wrap_add;
}

struct NetJob {
  const rslx_mlp* net;
  XView x;
  int32_t rows;
  NetBufs* bufs;
};

// Forward of up to two networks of equal depth, one grouped launch per layer.
// With skip_last the output layer is left to the caller (fused output-layer + loss kernel).
inline int32_t forward_nets(const NetJob* jobs, int count, hipStream_t stream, bool skip_last = false) {
  if (count == 2 && jobs[0].net->n_layers != jobs[1].net->n_layers) {
    RSLX_TRY(forward_nets(jobs, 1, stream, skip_last));
    return forward_nets(jobs + 1, 1, stream, skip_last);
  }
  const int L = jobs[0].net->n_layers;
  for (int l = 0; l < (skip_last ? L - 1 : L); ++l) {
    GemmBatch b;
    b.count = count;
    for (int i = 0; i < count; ++i) {
      const rslx_mlp& n = *jobs[i].net;
      GemmProblem p = blank_problem();
      if (l == 0) {
        set_x(p, jobs[i].x);
      } else {
        p.A = jobs[i].bufs->out[l - 1];
        p.lda = n.dims[l];
      }
      const float* W = n.params + layer_offset(n, l);
      p.B = W; p.ldb = n.dims[l + 1];
      p.aux = W + (int64_t)n.dims[l] * n.dims[l + 1];
      p.C = jobs[i].bufs->out[l]; p.ldc = n.dims[l + 1];
      p.M = jobs[i].rows; p.N = n.dims[l + 1]; p.K = (l == 0 && jobs[i].x.cols) ? jobs[i].x.cols : n.dims[l];
      p.elu = (l + 1 < L) ? 1 : 0;
      p.alpha = n.elu_alpha;
      p.a_vec = (p.K % 4 == 0 && p.lda % 4 == 0 && aligned16(p.A) && p.col_map == nullptr) ? 1 : 0;
      p.b_vec = (p.N % 4 == 0 && aligned16(p.B)) ? 1 : 0;
      b.p[i] = p;
    }
    RSLX_HIP(launch_gemm(GEMM_FWD, b, stream));
  }
  return RSLX_OK;
}

// Split plan of one trained network's weight gradients: layer l is reduced over `split[l]` row chunks of
// `chunk[l]` rows; its partial results (W then b, `size[l]` floats per split) start at `part_off[l]`.
struct SplitPlan {
  int32_t split[RSLX_MAX_LAYERS];
  int32_t chunk[RSLX_MAX_LAYERS];
  int32_t big[RSLX_MAX_LAYERS];
  int64_t size[RSLX_MAX_LAYERS];
  int64_t pitch[RSLX_MAX_LAYERS];     // floats between consecutive split buffers of a layer
  int64_t part_off[RSLX_MAX_LAYERS];
  int64_t total = 0;       // floats
  int32_t blocks = 0;      // workgroups of the reduction = entries of the squared-norm list
};

// Enough workgroups to fill the 256 CUs once, but at least 128 rows per split: four 64-row-tile workgroups per CU,
// three of the 128x128 ones (measured: 768 of those beat 1024).  A weight gradient that shares its launch with the
// layer's input gradient (every layer but the first) needs fewer - the input gradient's workgroups take the other
// slots - which also shrinks its partial sums: two per CU for 128x128 tiles, one per CU for 64-row tiles (measured
// on the 256x128 layer at 24 576 rows: 256 weight-gradient + 768 input-gradient workgroups are one resident round
// of 1024; 192 and 320..1024 are all slower, 128 makes the weight gradient the launch's long pole).
constexpr int DW_TARGET_WGS = 1024;
constexpr int DW_TARGET_WGS_PAIRED = 256;
constexpr int DW_TARGET_WGS_BIG = 768;
constexpr int DW_TARGET_WGS_BIG_PAIRED = 512;

// Plans layer l (an [M, N] weight reduced over `rows` rows) and appends it to p.
inline void plan_layer(SplitPlan& p, int l, int M, int N, int32_t rows, int group, bool paired) {
  const int tiles_big = ((M + 127) / 128) * ((N + 127) / 128);
  p.big[l] = (tiles_big * group >= 16) ? 1 : 0;
  const int tiles = gemm_dw_tiles(M, N, p.big[l] != 0);
  // 64-row tiles share a launch only where the paired kernel exists for both tile shapes (both widths above 64) or
  // as the narrow output layer that rides in the next layer's paired launch
  const bool small_shares = paired && ((M > 64 && N > 64) || N <= 32);
  const int target = p.big[l] ? (paired ? DW_TARGET_WGS_BIG_PAIRED : DW_TARGET_WGS_BIG)
                              : (small_shares ? DW_TARGET_WGS_PAIRED : DW_TARGET_WGS);
  int s = (target + tiles * group - 1) / (tiles * group);
  const int smax = rows / 128 > 1 ? rows / 128 : 1;
  if (s > smax) s = smax;
  if (s < 1) s = 1;
  int c = (rows + s - 1) / s;
  c = (c + 15) / 16 * 16;
  s = (rows + c - 1) / c;            // drop splits that would be empty
  p.split[l] = s;
  p.chunk[l] = c;
  p.size[l] = (int64_t)M * N + N;
  p.pitch[l] = (p.size[l] + 3) / 4 * 4;      // 16-byte aligned split buffers
  p.part_off[l] = p.total;
  p.total += p.pitch[l] * s;
  p.blocks += (int32_t)((p.size[l] + REDUCE_BLOCK_FLOATS - 1) / REDUCE_BLOCK_FLOATS);
}

inline SplitPlan plan_splits(const rslx_mlp& n, int32_t rows, int group, bool first_has_dx = false) {
  SplitPlan p;
  for (int l = 0; l < n.n_layers; ++l) plan_layer(p, l, n.dims[l], n.dims[l + 1], rows, group, l > 0 || first_has_dx);
  return p;
}

struct BwdJob {
  const rslx_mlp* net;
  XView x;
  int32_t rows;
  NetBufs* bufs;
  const float* d_out;    // [rows, dims[L]]
  float* wt;             // scratch for the transposed weights (flat parameter layout)
  float* partials;       // split partials, laid out by `plan`
  const SplitPlan* plan;
  float* dx0 = nullptr;  // optional [rows, dims[0]]: gradient w.r.t. the network input (a memory in front of it)
};

// Backward of up to two networks of equal depth: per layer one grouped weight-gradient launch (split over
// rows, partial sums) and one grouped input-gradient launch.
// With skip_last_dx the input gradient of the output layer (dz of the last hidden layer) already exists.
// Transposed copies of the weight matrices that the input-gradient contractions of backward_nets read.
inline int32_t transpose_weights(const BwdJob* jobs, int count, hipStream_t stream, bool skip_last_dx) {
  TransposeBatch tb;
  tb.count = 0;
  for (int i = 0; i < count; ++i) {
    const rslx_mlp& n = *jobs[i].net;
    for (int l = jobs[i].dx0 != nullptr ? 0 : 1; l < (skip_last_dx ? n.n_layers - 1 : n.n_layers); ++l)
      tb.job[tb.count++] = TransposeJob{n.params + layer_offset(n, l), jobs[i].wt + layer_offset(n, l), n.dims[l], n.dims[l + 1]};
  }
  RSLX_HIP(launch_transpose(tb, stream));
  return RSLX_OK;
}

// Lets the Adam launch keep a job's transposed weights current (see AdamSegment::wt).
inline void adam_keeps_transposed(AdamSegment& sg, const rslx_mlp& n, float* wt, bool first_has_dx = false) {
  sg.wt = wt;
  sg.n_layers = n.n_layers;
  sg.wt_from = first_has_dx ? 0 : 1;
  for (int i = 0; i <= n.n_layers; ++i) sg.dims[i] = n.dims[i];
}

// wt_ready: the transposed weights in jobs[i].wt are current (transpose_weights at the start of the call, kept up
// to date by the Adam launches since), so no transposition is launched here.
inline int32_t backward_nets(const BwdJob* jobs, int count, hipStream_t stream, bool skip_last_dx = false,
                             bool wt_ready = false) {
  if (count == 2 && jobs[0].net->n_layers != jobs[1].net->n_layers) {
    RSLX_TRY(backward_nets(jobs, 1, stream, skip_last_dx, wt_ready));
    return backward_nets(jobs + 1, 1, stream, skip_last_dx, wt_ready);
  }
  const int L = jobs[0].net->n_layers;
  const bool dx_in = jobs[0].dx0 != nullptr;     // all jobs of a call agree on this
  if (!wt_ready) RSLX_TRY(transpose_weights(jobs, count, stream, skip_last_dx));
  GemmBatch pending;
  bool has_pending = false;
  for (int l = L - 1; l >= 0; --l) {
    GemmBatch bw, bx;
    bw.count = bx.count = count;
    for (int i = 0; i < count; ++i) {
      const rslx_mlp& n = *jobs[i].net;
      const float* dz = (l == L - 1) ? jobs[i].d_out : jobs[i].bufs->dz[l];
      GemmProblem p = blank_problem();
      if (l == 0) {
        set_x(p, jobs[i].x);
      } else {
        p.A = jobs[i].bufs->out[l - 1];
        p.lda = n.dims[l];
      }
      p.B = dz; p.ldb = n.dims[l + 1];
      const SplitPlan& sp = *jobs[i].plan;
      p.C = jobs[i].partials + sp.part_off[l]; p.ldc = n.dims[l + 1];
      p.M = n.dims[l]; p.N = n.dims[l + 1]; p.K = jobs[i].rows;
      if (l == 0) p.a_cols = jobs[i].x.cols;
      p.n_split = sp.split[l];
      p.k_chunk = sp.chunk[l];
      p.split_stride = sp.pitch[l];
      p.bias_off = n.dims[l] * n.dims[l + 1];
      p.dw_big = sp.big[l];
      p.a_vec = ((p.a_cols ? p.a_cols : p.M) % 4 == 0 && p.lda % 4 == 0 && aligned16(p.A) && p.col_map == nullptr) ? 1 : 0;
      p.b_vec = (p.N % 4 == 0 && aligned16(p.B)) ? 1 : 0;
      bw.p[i] = p;
      if ((l > 0 || dx_in) && !(skip_last_dx && l == L - 1)) {
        GemmProblem q = blank_problem();
        q.A = dz; q.lda = n.dims[l + 1];
        q.B = jobs[i].wt + layer_offset(n, l); q.ldb = n.dims[l];
        q.C = l > 0 ? jobs[i].bufs->dz[l - 1] : jobs[i].dx0; q.ldc = n.dims[l];
        q.aux = l > 0 ? jobs[i].bufs->out[l - 1] : nullptr;      // the network input is not an ELU output
        q.M = jobs[i].rows; q.N = n.dims[l]; q.K = n.dims[l + 1];
        q.alpha = n.elu_alpha;
        q.a_vec = (q.K % 4 == 0 && aligned16(q.A)) ? 1 : 0;
        q.b_vec = (q.N % 4 == 0 && aligned16(q.B)) ? 1 : 0;
        bx.p[i] = q;
      }
    }
    if ((l > 0 || dx_in) && !(skip_last_dx && l == L - 1)) {
      RSLX_HIP(launch_gemm_dw_dx(bw, bx, stream, has_pending ? &pending : nullptr));
      has_pending = false;
    } else if (skip_last_dx && l == L - 1 && l > 0) {
      // the output layer's weight gradient (its input gradient exists already): it joins the next layer's launch
      pending = bw;
      has_pending = true;
    } else {
      if (has_pending) RSLX_HIP(launch_gemm(GEMM_DW, pending, stream));
      has_pending = false;
      RSLX_HIP(launch_gemm(GEMM_DW, bw, stream));
    }
  }
  if (has_pending) RSLX_HIP(launch_gemm(GEMM_DW, pending, stream));
  return RSLX_OK;
}

inline FusedNet fused_net(const rslx_mlp& n, const float* x, int ldx, const int32_t* col_map, float* out, bool head) {
  FusedNet f;
  memset(&f, 0, sizeof f);
  f.params = n.params; f.x = x; f.ldx = ldx; f.col_map = col_map; f.out = out;
  f.n_layers = n.n_layers;
  for (int i = 0; i <= n.n_layers; ++i) f.dims[i] = n.dims[i];
  f.alpha = n.elu_alpha;
  f.head = head ? 1 : 0;
  return f;
}

// The layer-fused launch holds one workgroup per CU and walks 32 rows through all layers as one dependent chain:
// unbeatable while a network's row blocks fit the chip once (two networks: two rounds), but each further round costs the whole
// chain again, and the tiled per-layer launches then do the same work faster (measured at 16 384 rows, two
// networks [48, 512, 256, 128, 12]: 4 rounds, 176 us fused against 127 us layered).
// The choice depends on the row count alone, so that a values-only call and a full call on the same batch take the
// same path and return bit-identical values.
inline bool fused_forward_pays(const FusedForwardArgs& fa) {
  return fused_forward_supported(fa) && (fa.n_rows + 31) / 32 <= 256;
}

inline int max_dim_of(const rslx_mlp& n) {
  int m = 0;
  for (int i = 0; i <= n.n_layers; ++i) m = n.dims[i] > m ? n.dims[i] : m;
  return m;
}

inline bool involution_ok(const int32_t* perm, const float* sign, int n) {
  if (!perm || !sign) return false;
  for (int j = 0; j < n; ++j) {
    if (perm[j] < 0 || perm[j] >= n) return false;
    if (sign[j] != 1.0f && sign[j] != -1.0f) return false;
  }
  for (int j = 0; j < n; ++j) {
    if (perm[perm[j]] != j) return false;
    if (sign[j] * sign[perm[j]] != 1.0f) return false;
  }
  return true;
}

inline float bias_correction(float beta, int64_t t) { return (float)(1.0 - std::pow((double)beta, (double)t)); }

inline int64_t round4(int64_t n) { return (n + 3) / 4 * 4; }


struct TrainBufs {        // per trained network
  NetBufs act;
  float* d_out = nullptr;
  float* wt = nullptr;
  float* partials = nullptr;
  SplitPlan plan;
  double* sumsq = nullptr;
  int n_sumsq = 0;
};

inline void carve_train(Carver& c, const rslx_mlp& n, int32_t rows, int group, TrainBufs& t, bool first_has_dx = false) {
  carve_net(c, n, rows, true, t.act);
  t.d_out = c.take<float>((size_t)rows * n.dims[n.n_layers]);
  t.wt = c.take<float>((size_t)round4(weight_count(n)));
  t.plan = plan_splits(n, rows, group, first_has_dx);
  t.partials = c.take<float>((size_t)t.plan.total);
  t.n_sumsq = t.plan.blocks;
}

// Appends one network's layers to a reduce launch; the network's sumsq blocks must start at entry a.blocks of
// a.sumsq_blocks.
inline void reduce_add_net(ReduceArgs& a, const rslx_mlp& n, const TrainBufs& t) {
  for (int l = 0; l < n.n_layers; ++l) {
    ReduceSeg& sg = a.seg[a.n_seg++];
    sg.partials = t.partials + t.plan.part_off[l];
    sg.grads = n.grads + layer_offset(n, l);
    sg.size = t.plan.size[l];
    sg.pitch = t.plan.pitch[l];
    sg.split = t.plan.split[l];
    sg.block_start = a.blocks;
    a.blocks += (int)((t.plan.size[l] + REDUCE_BLOCK_FLOATS - 1) / REDUCE_BLOCK_FLOATS);
  }
}

inline int32_t reduce_net(const rslx_mlp& n, const TrainBufs& t, hipStream_t s) {
  ReduceArgs a;
  memset(&a, 0, sizeof a);
  a.sumsq_blocks = t.sumsq;
  reduce_add_net(a, n, t);
  RSLX_HIP(launch_reduce_partials(a, s));
  return RSLX_OK;
}


static_assert(sizeof(rslx_dev_counters) == 4 * sizeof(int64_t), "rslx_dev_counters is four 64-bit words");
inline hipError_t advance_counters(rslx_dev_counters* c, int64_t act, int64_t call, int64_t adam, int64_t rnd, hipStream_t s) {
  const int64_t d[4] = {act, call, adam, rnd};
  return launch_counter_add(reinterpret_cast<int64_t*>(c), d, 4, s);
}


// One act() step of an actor / critic pair of MLPs on given input matrices (defined in api.hip).  ld_actor /
// ld_critic: row strides of the input matrices when they are wider than the networks' inputs (the hidden part of a
// packed recurrent state); 0 = dense.
int32_t act_impl(const rslx_mlp* actor, const rslx_mlp* critic, const float* obs_actor, const float* obs_critic,
                 int32_t N, uint64_t seed, uint64_t step, rslx_dev_counters* counters, const float* eps_or_null,
                 float* actions, float* logp, float* values, float* mu, float* sigma, uint32_t flags, void* ws,
                 size_t ws_bytes, void* stream, int32_t ld_actor = 0, int32_t ld_critic = 0);

}  // namespace host
}  // namespace rslx
