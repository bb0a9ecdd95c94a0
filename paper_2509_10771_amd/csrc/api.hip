// Host side of librslx: argument validation, workspace carving and launch sequencing for the C ABI
// declared in include/rslx.h.  No entry point synchronises with the host or allocates device memory.
#include <climits>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <string>
#include <vector>

#include "../../include/rslx.h"
#include "kernels.h"

namespace {

using namespace rslx;

thread_local std::string g_last_error;

int32_t fail(int32_t code, const char* fmt, ...) {
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

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

uint64_t mix64_host(uint64_t x) {
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
int64_t layer_offset(const rslx_mlp& n, int l) {
  int64_t o = 0;
  for (int i = 0; i < l; ++i) o += (int64_t)n.dims[i] * n.dims[i + 1] + n.dims[i + 1];
  return o;
}
int64_t weight_count(const rslx_mlp& n) { return layer_offset(n, n.n_layers); }
int64_t param_count(const rslx_mlp& n) { return weight_count(n) + (n.has_log_std ? n.dims[n.n_layers] : 0); }

int32_t check_mlp(const rslx_mlp* n, const char* name, bool trainable) {
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
};

// Per-network activation storage for `rows` rows: out[l] = output of layer l, dz[l] = gradient w.r.t. the
// pre-activation of hidden layer l.  The caller may point out[last] at its own buffer.
struct NetBufs {
  float* out[RSLX_MAX_LAYERS] = {};
  float* dz[RSLX_MAX_LAYERS] = {};
};

void carve_net(Carver& c, const rslx_mlp& n, int64_t rows, bool backward, NetBufs& b) {
  for (int l = 0; l < n.n_layers; ++l) b.out[l] = c.take<float>((size_t)rows * n.dims[l + 1]);
  if (backward)
    for (int l = 0; l + 1 < n.n_layers; ++l) b.dz[l] = c.take<float>((size_t)rows * n.dims[l + 1]);
}

GemmProblem blank_problem() {
  GemmProblem p;
  memset(&p, 0, sizeof p);
  p.idx_mod = INT_MAX;
  p.map_from = INT_MAX;
  p.bias_off = -1;
  p.n_split = 1;
  return p;
}

void set_x(GemmProblem& p, const XView& x) {
  p.A = x.base; p.lda = x.ld; p.row_idx = x.row_idx; p.col_map = x.col_map; p.col_sign = x.col_sign;
  p.idx_mod = x.idx_mod; p.map_from = x.map_from; p.a_src_rows = x.src_rows;
}

struct NetJob {
  const rslx_mlp* net;
  XView x;
  int32_t rows;
  NetBufs* bufs;
};

// Forward of up to two networks of equal depth, one grouped launch per layer.
// With skip_last the output layer is left to the caller (fused output-layer + loss kernel).
int32_t forward_nets(const NetJob* jobs, int count, hipStream_t stream, bool skip_last = false) {
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
      p.M = jobs[i].rows; p.N = n.dims[l + 1]; p.K = n.dims[l];
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
// three of the 128x128 ones (measured: 768 of those beat 1024).  A 128x128 weight gradient that shares its launch
// with the layer's input gradient (every layer but the first) only needs two per CU - the input gradient's
// workgroups take the other slots - which also halves its partial sums.
constexpr int DW_TARGET_WGS = 1024;
constexpr int DW_TARGET_WGS_BIG = 768;
constexpr int DW_TARGET_WGS_BIG_PAIRED = 512;

// Plans layer l (an [M, N] weight reduced over `rows` rows) and appends it to p.
void plan_layer(SplitPlan& p, int l, int M, int N, int32_t rows, int group, bool paired) {
  const int tiles_big = ((M + 127) / 128) * ((N + 127) / 128);
  p.big[l] = (tiles_big * group >= 16) ? 1 : 0;
  const int tiles = gemm_dw_tiles(M, N, p.big[l] != 0);
  const int target = p.big[l] ? (paired ? DW_TARGET_WGS_BIG_PAIRED : DW_TARGET_WGS_BIG) : DW_TARGET_WGS;
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

SplitPlan plan_splits(const rslx_mlp& n, int32_t rows, int group, bool first_has_dx = false) {
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
int32_t backward_nets(const BwdJob* jobs, int count, hipStream_t stream, bool skip_last_dx = false) {
  if (count == 2 && jobs[0].net->n_layers != jobs[1].net->n_layers) {
    RSLX_TRY(backward_nets(jobs, 1, stream, skip_last_dx));
    return backward_nets(jobs + 1, 1, stream, skip_last_dx);
  }
  const int L = jobs[0].net->n_layers;
  TransposeBatch tb;
  tb.count = 0;
  const bool dx_in = jobs[0].dx0 != nullptr;     // all jobs of a call agree on this
  for (int i = 0; i < count; ++i)
    for (int l = dx_in ? 0 : 1; l < (skip_last_dx ? L - 1 : L); ++l) {
      const rslx_mlp& n = *jobs[i].net;
      tb.job[tb.count++] = TransposeJob{n.params + layer_offset(n, l), jobs[i].wt + layer_offset(n, l), n.dims[l], n.dims[l + 1]};
    }
  RSLX_HIP(launch_transpose(tb, stream));
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
      p.n_split = sp.split[l];
      p.k_chunk = sp.chunk[l];
      p.split_stride = sp.pitch[l];
      p.bias_off = n.dims[l] * n.dims[l + 1];
      p.dw_big = sp.big[l];
      p.a_vec = (p.M % 4 == 0 && p.lda % 4 == 0 && aligned16(p.A) && p.col_map == nullptr) ? 1 : 0;
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
    if ((l > 0 || dx_in) && !(skip_last_dx && l == L - 1)) RSLX_HIP(launch_gemm_dw_dx(bw, bx, stream));
    else RSLX_HIP(launch_gemm(GEMM_DW, bw, stream));
  }
  return RSLX_OK;
}

FusedNet fused_net(const rslx_mlp& n, const float* x, int ldx, const int32_t* col_map, float* out, bool head) {
  FusedNet f;
  memset(&f, 0, sizeof f);
  f.params = n.params; f.x = x; f.ldx = ldx; f.col_map = col_map; f.out = out;
  f.n_layers = n.n_layers;
  for (int i = 0; i <= n.n_layers; ++i) f.dims[i] = n.dims[i];
  f.alpha = n.elu_alpha;
  f.head = head ? 1 : 0;
  return f;
}

int max_dim_of(const rslx_mlp& n) {
  int m = 0;
  for (int i = 0; i <= n.n_layers; ++i) m = n.dims[i] > m ? n.dims[i] : m;
  return m;
}

bool involution_ok(const int32_t* perm, const float* sign, int n) {
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

float bias_correction(float beta, int64_t t) { return (float)(1.0 - std::pow((double)beta, (double)t)); }

int64_t round4(int64_t n) { return (n + 3) / 4 * 4; }

struct TraceRec {
  hipEvent_t a, b;
  char kernel[48];
  double flops, bytes;
};
bool g_trace_on = false;
size_t g_trace_cap = 0;
std::vector<TraceRec> g_trace;

}  // namespace

namespace rslx {
void trace_open(hipStream_t stream, const char* kernel, double flops, double bytes) {
  if (!g_trace_on || g_trace.size() >= g_trace_cap) return;
  TraceRec r;
  if (hipEventCreate(&r.a) != hipSuccess) return;
  if (hipEventCreate(&r.b) != hipSuccess) { (void)hipEventDestroy(r.a); return; }
  snprintf(r.kernel, sizeof r.kernel, "%s", kernel);
  r.flops = flops; r.bytes = bytes;
  (void)hipEventRecord(r.a, stream);
  g_trace.push_back(r);
}
void trace_close(hipStream_t stream) {
  if (!g_trace_on || g_trace.empty()) return;
  (void)hipEventRecord(g_trace.back().b, stream);
}
}  // namespace rslx

// ======================================================================================================
extern "C" {

int32_t rslx_trace_begin(int32_t max_records) {
  if (max_records < 1) return fail(RSLX_ERR_INVALID_ARG, "rslx_trace_begin: max_records = %d", max_records);
  for (TraceRec& r : g_trace) { (void)hipEventDestroy(r.a); (void)hipEventDestroy(r.b); }
  g_trace.clear();
  g_trace.reserve(max_records);
  g_trace_cap = (size_t)max_records;
  g_trace_on = true;
  return RSLX_OK;
}

int32_t rslx_trace_end(rslx_trace_record* out, int32_t cap, int32_t* n_out) {
  g_trace_on = false;
  if (!n_out) return fail(RSLX_ERR_INVALID_ARG, "rslx_trace_end: null n_out");
  int32_t n = 0;
  for (TraceRec& r : g_trace) {
    float ms = 0.f;
    hipError_t e = hipEventSynchronize(r.b);
    if (e == hipSuccess) e = hipEventElapsedTime(&ms, r.a, r.b);
    if (e != hipSuccess) return fail(RSLX_ERR_HIP, "rslx_trace_end: %s", hipGetErrorString(e));
    if (out && n < cap) {
      memcpy(out[n].kernel, r.kernel, sizeof r.kernel);
      out[n].flops = r.flops; out[n].bytes = r.bytes; out[n].ms = ms;
    }
    ++n;
  }
  *n_out = n;
  if (out) {
    for (TraceRec& r : g_trace) { (void)hipEventDestroy(r.a); (void)hipEventDestroy(r.b); }
    g_trace.clear();
  } else {
    g_trace_on = false;
  }
  return RSLX_OK;
}

int32_t rslx_version(void) { return 100; }

const char* rslx_last_error(void) { return g_last_error.c_str(); }

int32_t rslx_device_check(void) {
  int dev = 0;
  RSLX_HIP(hipGetDevice(&dev));
  hipDeviceProp_t prop;
  RSLX_HIP(hipGetDeviceProperties(&prop, dev));
  if (strncmp(prop.gcnArchName, "gfx950", 6) != 0)
    return fail(RSLX_ERR_UNSUPPORTED, "device %d is %s, this library is built for gfx950", dev, prop.gcnArchName);
  return RSLX_OK;
}

// ---- permutation ---------------------------------------------------------------------------------------
size_t rslx_permutation_workspace_bytes(int32_t B) { return B > 0 ? perm_workspace_bytes(B) + 256 : 256; }

int32_t rslx_permutation(uint64_t seed, uint64_t call_index, int32_t epoch, int32_t B, int32_t* perm_out, void* ws,
                         size_t ws_bytes, void* stream) {
  if (B < 0 || epoch < 0) return fail(RSLX_ERR_SHAPE, "rslx_permutation: B = %d, epoch = %d", B, epoch);
  if (B == 0) return RSLX_OK;
  if (!perm_out || !ws) return fail(RSLX_ERR_INVALID_ARG, "rslx_permutation: null pointer");
  if (ws_bytes < rslx_permutation_workspace_bytes(B)) return fail(RSLX_ERR_WORKSPACE, "rslx_permutation: workspace too small");
  Carver c(ws);
  void* w = c.take<char>(perm_workspace_bytes(B));
  const uint64_t base = mix64_host(mix64_host(mix64_host(seed) ^ call_index) ^ (uint64_t)epoch);
  RSLX_HIP(launch_permutations(&base, 1, B, perm_out, w, (hipStream_t)stream));
  return RSLX_OK;
}

// ---- act ---------------------------------------------------------------------------------------------------
static size_t act_carve(Carver& c, const rslx_mlp* actor, const rslx_mlp* critic, int32_t N, NetBufs* ba, NetBufs* bc) {
  NetBufs ta, tc;
  if (actor) carve_net(c, *actor, N, false, ta);
  if (critic) carve_net(c, *critic, N, false, tc);
  if (ba) *ba = ta;
  if (bc) *bc = tc;
  return c.off + 256;
}

size_t rslx_act_workspace_bytes(const rslx_mlp* actor, const rslx_mlp* critic, int32_t N) {
  if (N <= 0) return 256;
  Carver c(nullptr);
  return act_carve(c, actor, critic, N, nullptr, nullptr);
}

}  // extern "C"

namespace {
static_assert(sizeof(rslx_dev_counters) == 4 * sizeof(int64_t), "rslx_dev_counters is four 64-bit words");
hipError_t advance_counters(rslx_dev_counters* c, int64_t act, int64_t call, int64_t adam, int64_t rnd, hipStream_t s) {
  const int64_t d[4] = {act, call, adam, rnd};
  return launch_counter_add(reinterpret_cast<int64_t*>(c), d, 4, s);
}

// Shared body of rslx_act and rslx_act_dc: with `counters` the noise position comes from device memory.
int32_t act_impl(const rslx_mlp* actor, const rslx_mlp* critic, const float* obs_actor, const float* obs_critic,
                 int32_t N, uint64_t seed, uint64_t step, rslx_dev_counters* counters, const float* eps_or_null,
                 float* actions, float* logp, float* values, float* mu, float* sigma, uint32_t flags, void* ws,
                 size_t ws_bytes, void* stream, int32_t ld_actor = 0, int32_t ld_critic = 0) {
  // ld_actor / ld_critic: row strides of the input matrices when they are wider than the networks' inputs (the
  // hidden part of a packed recurrent state); 0 = dense.
  const bool values_only = (flags & RSLX_ACT_VALUES_ONLY) != 0;
  const int64_t* step_dev = counters ? &counters->act_step : nullptr;
  const uint64_t noise_pre = mix64_host(seed ^ 0xAC7ull);
  if (N < 0) return fail(RSLX_ERR_SHAPE, "rslx_act: N = %d", N);
  RSLX_TRY(check_mlp(critic, "rslx_act critic", false));
  if (critic->dims[critic->n_layers] != 1) return fail(RSLX_ERR_SHAPE, "rslx_act: critic output width must be 1");
  if (!values_only) {
    RSLX_TRY(check_mlp(actor, "rslx_act actor", false));
    if (!actor->has_log_std) return fail(RSLX_ERR_INVALID_ARG, "rslx_act: actor needs log_std");
    if (actor->dims[actor->n_layers] > RSLX_MAX_ACTIONS) return fail(RSLX_ERR_SHAPE, "rslx_act: action width > %d", RSLX_MAX_ACTIONS);
    if (!obs_actor || !actions || !logp || !mu || !sigma) return fail(RSLX_ERR_INVALID_ARG, "rslx_act: null actor input / output");
  }
  if (!obs_critic || !values) return fail(RSLX_ERR_INVALID_ARG, "rslx_act: null critic input / output");
  if (N == 0) return RSLX_OK;
  const rslx_mlp* a = values_only ? nullptr : actor;
  if (!ws || ws_bytes < rslx_act_workspace_bytes(a, critic, N)) return fail(RSLX_ERR_WORKSPACE, "rslx_act: workspace too small");
  hipStream_t s = (hipStream_t)stream;
  // Fast path: one layer-fused launch for both networks and the Gaussian head.
  {
    FusedForwardArgs fa;
    memset(&fa, 0, sizeof fa);
    fa.n_rows = N;
    fa.max_dim = max_dim_of(*critic);
    if (a) {
      fa.net[fa.n_nets++] = fused_net(*a, obs_actor, ld_actor ? ld_actor : a->dims[0], nullptr, mu, true);
      fa.max_dim = max_dim_of(*a) > fa.max_dim ? max_dim_of(*a) : fa.max_dim;
    }
    fa.net[fa.n_nets++] = fused_net(*critic, obs_critic, ld_critic ? ld_critic : critic->dims[0], nullptr, values, false);
    fa.deterministic = (flags & RSLX_ACT_DETERMINISTIC) ? 1 : 0;
    fa.eps = eps_or_null;
    fa.noise_base = mix64_host(noise_pre ^ step);
    fa.step_dev = step_dev; fa.noise_pre = noise_pre;
    fa.actions = actions; fa.logp = logp; fa.sigma = sigma;
    if (fused_forward_supported(fa)) {
      RSLX_HIP(launch_fused_forward(fa, s));
      if (counters && !values_only) RSLX_HIP(advance_counters(counters, 1, 0, 0, 0, s));
      return RSLX_OK;
    }
  }
  // General path (layers wider than the fused kernel's LDS budget): one grouped launch per layer.
  Carver c(ws);
  NetBufs ba, bc;
  act_carve(c, a, critic, N, &ba, &bc);
  bc.out[critic->n_layers - 1] = values;              // [N, 1] lands directly in the caller's buffer
  NetJob jobs[2];
  int nj = 0;
  if (a) {
    ba.out[a->n_layers - 1] = mu;
    XView xa; xa.base = obs_actor; xa.ld = ld_actor ? ld_actor : a->dims[0];
    jobs[nj++] = NetJob{a, xa, N, &ba};
  }
  XView xc; xc.base = obs_critic; xc.ld = ld_critic ? ld_critic : critic->dims[0];
  jobs[nj++] = NetJob{critic, xc, N, &bc};
  RSLX_TRY(forward_nets(jobs, nj, s));
  if (a) {
    const int A = a->dims[a->n_layers];
    const uint64_t base = mix64_host(noise_pre ^ step);
    RSLX_HIP(launch_act_head(mu, a->params + weight_count(*a), eps_or_null, base, N, A,
                             (flags & RSLX_ACT_DETERMINISTIC) ? 1 : 0, actions, logp, mu, sigma, s, step_dev, noise_pre));
    if (counters) RSLX_HIP(advance_counters(counters, 1, 0, 0, 0, s));
  }
  return RSLX_OK;
}
}  // namespace

extern "C" {

int32_t rslx_act(const rslx_mlp* actor, const rslx_mlp* critic, const float* obs_actor, const float* obs_critic,
                 int32_t N, uint64_t seed, uint64_t step, const float* eps_or_null, float* actions, float* logp,
                 float* values, float* mu, float* sigma, uint32_t flags, void* ws, size_t ws_bytes, void* stream) {
  return act_impl(actor, critic, obs_actor, obs_critic, N, seed, step, nullptr, eps_or_null, actions, logp, values, mu,
                  sigma, flags, ws, ws_bytes, stream);
}

int32_t rslx_act_dc(const rslx_mlp* actor, const rslx_mlp* critic, const float* obs_actor, const float* obs_critic,
                    int32_t N, uint64_t seed, rslx_dev_counters* counters, const float* eps_or_null, float* actions,
                    float* logp, float* values, float* mu, float* sigma, uint32_t flags, void* ws, size_t ws_bytes,
                    void* stream) {
  if (!counters) return fail(RSLX_ERR_INVALID_ARG, "rslx_act_dc: null counters");
  return act_impl(actor, critic, obs_actor, obs_critic, N, seed, 0, counters, eps_or_null, actions, logp, values, mu,
                  sigma, flags, ws, ws_bytes, stream);
}

// ---- GAE -----------------------------------------------------------------------------------------------------
size_t rslx_gae_workspace_bytes(int32_t T, int32_t N) {
  (void)T;
  if (N <= 0) return 256;
  return (size_t)gae_num_blocks(N) * 16 + 16 + 512;
}

int32_t rslx_gae(const float* rewards, const float* values, const float* last_values, const uint8_t* dones,
                 const uint8_t* timeouts_or_null, int32_t T, int32_t N, float gamma, float lam, int32_t normalize_adv,
                 float* advantages, float* returns, void* ws, size_t ws_bytes, void* stream) {
  if (T < 0 || N < 0) return fail(RSLX_ERR_SHAPE, "rslx_gae: T = %d, N = %d", T, N);
  if (T == 0 || N == 0) return RSLX_OK;
  if (!rewards || !values || !last_values || !dones || !advantages || !returns)
    return fail(RSLX_ERR_INVALID_ARG, "rslx_gae: null pointer");
  if (!aligned16(advantages)) return fail(RSLX_ERR_INVALID_ARG, "rslx_gae: advantages not 16-byte aligned");
  if ((int64_t)T * N > (int64_t)INT_MAX * 4) return fail(RSLX_ERR_SHAPE, "rslx_gae: T*N too large");
  double* partials = nullptr;
  if (normalize_adv) {
    if (!ws || ws_bytes < rslx_gae_workspace_bytes(T, N)) return fail(RSLX_ERR_WORKSPACE, "rslx_gae: workspace too small");
    Carver c(ws);
    partials = c.take<double>((size_t)gae_num_blocks(N) * 2 + 2);
  }
  RSLX_HIP(launch_gae(rewards, values, last_values, dones, timeouts_or_null, T, N, gamma, lam, normalize_adv ? 1 : 0,
                      advantages, returns, partials, (hipStream_t)stream));
  return RSLX_OK;
}

// ---- Adam ----------------------------------------------------------------------------------------------------
size_t rslx_adam_workspace_bytes(int64_t n) { return n > 0 ? ((size_t)reduce_num_blocks(n) + 1) * 8 + 512 : 256; }

int32_t rslx_adam_step(float* params, const float* grads, float* m, float* v, int64_t n, float lr, float beta1,
                       float beta2, float eps, float max_grad_norm, int64_t* adam_step, float* grad_norm_out, void* ws,
                       size_t ws_bytes, void* stream) {
  if (n < 0) return fail(RSLX_ERR_SHAPE, "rslx_adam_step: n = %lld", (long long)n);
  if (!adam_step) return fail(RSLX_ERR_INVALID_ARG, "rslx_adam_step: null adam_step");
  if (n == 0) { ++*adam_step; return RSLX_OK; }
  if (!params || !grads || !m || !v) return fail(RSLX_ERR_INVALID_ARG, "rslx_adam_step: null pointer");
  if (!aligned16(params) || !aligned16(grads) || !aligned16(m) || !aligned16(v))
    return fail(RSLX_ERR_INVALID_ARG, "rslx_adam_step: buffers not 16-byte aligned");
  if (!ws || ws_bytes < rslx_adam_workspace_bytes(n)) return fail(RSLX_ERR_WORKSPACE, "rslx_adam_step: workspace too small");
  hipStream_t s = (hipStream_t)stream;
  Carver c(ws);
  const int nb = reduce_num_blocks(n);
  double* sumsq = c.take<double>((size_t)nb + 1);
  RSLX_HIP(launch_sumsq(grads, n, sumsq, s));
  const int64_t t = *adam_step + 1;
  AdamArgs a;
  memset(&a, 0, sizeof a);
  a.seg[0] = AdamSegment{params, grads, m, v, n};
  a.n_seg = 1;
  a.sumsq_blocks = sumsq; a.n_sumsq = nb;
  a.max_grad_norm = max_grad_norm;
  a.lr = lr; a.beta1 = beta1; a.beta2 = beta2; a.eps = eps;
  a.bc1 = bias_correction(beta1, t); a.bc2 = bias_correction(beta2, t);
  a.grad_norm_out = grad_norm_out;
  RSLX_HIP(launch_adam(a, s));
  *adam_step = t;
  return RSLX_OK;
}

// ---- PPO update ------------------------------------------------------------------------------------------------
namespace {

struct TrainBufs {        // per trained network
  NetBufs act;
  float* d_out = nullptr;
  float* wt = nullptr;
  float* partials = nullptr;
  SplitPlan plan;
  double* sumsq = nullptr;
  int n_sumsq = 0;
};

struct PpoPlan {
  int32_t B, mb, rows;
  bool fused_head = false;           // output layers + loss + their input gradient in one launch
  int32_t loss_blocks = 0;
  int32_t* perms = nullptr;          // [E, B]
  void* perm_ws = nullptr;
  TrainBufs actor, critic, pred;
  NetBufs targ;
  double* sumsq_all = nullptr;       // actor blocks, critic blocks, log_std slot
  double* loss_partials = nullptr;
  double* mse_partials = nullptr;
  size_t bytes = 0;
};

void carve_train(Carver& c, const rslx_mlp& n, int32_t rows, int group, TrainBufs& t, bool first_has_dx = false) {
  carve_net(c, n, rows, true, t.act);
  t.d_out = c.take<float>((size_t)rows * n.dims[n.n_layers]);
  t.wt = c.take<float>((size_t)round4(weight_count(n)));
  t.plan = plan_splits(n, rows, group, first_has_dx);
  t.partials = c.take<float>((size_t)t.plan.total);
  t.n_sumsq = t.plan.blocks;
}

void ppo_plan(Carver& c, const rslx_mlp* actor, const rslx_mlp* critic, const rslx_rollout* ro, const rslx_ppo_cfg* cfg,
              const rslx_sym* sym, const rslx_rnd_train* rnd, PpoPlan& p) {
  p.B = ro->T * ro->N;
  p.mb = p.B / cfg->minibatches;
  p.rows = sym ? 2 * p.mb : p.mb;
  p.perms = c.take<int32_t>((size_t)cfg->epochs * p.B);
  p.perm_ws = c.take<char>(perm_workspace_bytes(p.B));
  carve_train(c, *actor, p.rows, 2, p.actor);
  carve_train(c, *critic, p.rows, 2, p.critic);
  p.sumsq_all = c.take<double>((size_t)p.actor.n_sumsq + p.critic.n_sumsq + 2);
  p.actor.sumsq = p.sumsq_all;
  p.critic.sumsq = p.sumsq_all + p.actor.n_sumsq;
  p.fused_head = actor->n_layers >= 2 && critic->n_layers >= 2 &&
                 ppo_head_supported(actor->dims[actor->n_layers - 1], critic->dims[critic->n_layers - 1], ro->A);
  p.loss_blocks = p.fused_head ? ppo_head_num_blocks(p.mb, sym != nullptr) : ppo_loss_num_blocks(p.mb);
  p.loss_partials = c.take<double>((size_t)p.loss_blocks * (PPO_NPART_FIXED + ro->A));
  if (rnd) {
    carve_train(c, *rnd->predictor, p.mb, 1, p.pred);
    p.pred.sumsq = c.take<double>((size_t)p.pred.n_sumsq + 1);
    carve_net(c, *rnd->target, p.mb, false, p.targ);
    const int K = rnd->target->dims[rnd->target->n_layers];
    p.mse_partials = c.take<double>(mse_num_blocks((int64_t)p.mb * K));
  }
  p.bytes = c.off + 256;
}

int32_t ppo_validate(const rslx_mlp* actor, const rslx_mlp* critic, const rslx_rollout* ro, const rslx_ppo_cfg* cfg,
                     const rslx_sym* sym, const rslx_rnd_train* rnd, bool need_buffers) {
  if (!ro || !cfg) return fail(RSLX_ERR_INVALID_ARG, "rslx_ppo_update: null rollout or cfg");
  RSLX_TRY(check_mlp(actor, "rslx_ppo_update actor", need_buffers));
  RSLX_TRY(check_mlp(critic, "rslx_ppo_update critic", need_buffers));
  if (!actor->has_log_std) return fail(RSLX_ERR_INVALID_ARG, "rslx_ppo_update: actor needs log_std");
  if (ro->T < 1 || ro->N < 1 || (int64_t)ro->T * ro->N > (1 << 30)) return fail(RSLX_ERR_SHAPE, "rslx_ppo_update: T = %d, N = %d", ro->T, ro->N);
  if (ro->Da != actor->dims[0] || ro->Dc != critic->dims[0] || ro->A != actor->dims[actor->n_layers] ||
      critic->dims[critic->n_layers] != 1)
    return fail(RSLX_ERR_SHAPE, "rslx_ppo_update: rollout widths do not match the networks");
  if (ro->A > 32) return fail(RSLX_ERR_UNSUPPORTED, "rslx_ppo_update: action width %d > 32", ro->A);
  if (cfg->epochs < 0 || cfg->minibatches < 1) return fail(RSLX_ERR_SHAPE, "rslx_ppo_update: epochs / minibatches");
  if ((ro->T * ro->N) % cfg->minibatches != 0)
    return fail(RSLX_ERR_SHAPE, "rslx_ppo_update: T*N = %d is not a multiple of minibatches = %d", ro->T * ro->N, cfg->minibatches);
  if (need_buffers) {
    if (!ro->obs_actor || !ro->obs_critic || !ro->actions || !ro->logp || !ro->values || !ro->mu || !ro->sigma ||
        !ro->advantages || !ro->returns)
      return fail(RSLX_ERR_INVALID_ARG, "rslx_ppo_update: null rollout buffer");
  }
  if (sym) {
    if (!involution_ok(sym->perm_obs_a_host, sym->sign_obs_a_host, ro->Da) ||
        !involution_ok(sym->perm_obs_c_host, sym->sign_obs_c_host, ro->Dc) ||
        !involution_ok(sym->perm_act_host, sym->sign_act_host, ro->A))
      return fail(RSLX_ERR_INVALID_ARG, "rslx_ppo_update: mirror map is not an involutive signed permutation");
    if (need_buffers && (!sym->perm_obs_a || !sym->sign_obs_a || !sym->perm_obs_c || !sym->sign_obs_c || !sym->perm_act || !sym->sign_act))
      return fail(RSLX_ERR_INVALID_ARG, "rslx_ppo_update: null device mirror map");
  }
  if (rnd) {
    RSLX_TRY(check_mlp(rnd->target, "rslx_ppo_update rnd target", false));
    RSLX_TRY(check_mlp(rnd->predictor, "rslx_ppo_update rnd predictor", need_buffers));
    if (rnd->target->n_layers != rnd->predictor->n_layers) return fail(RSLX_ERR_SHAPE, "rslx_ppo_update: rnd nets differ in depth");
    for (int i = 0; i <= rnd->target->n_layers; ++i)
      if (rnd->target->dims[i] != rnd->predictor->dims[i]) return fail(RSLX_ERR_SHAPE, "rslx_ppo_update: rnd nets differ in shape");
    if (rnd->n_subset != rnd->target->dims[0] || (!rnd->subset_idx && rnd->n_subset != ro->Da))
      return fail(RSLX_ERR_SHAPE, "rslx_ppo_update: rnd subset width");
  }
  return RSLX_OK;
}

// Appends one network's layers to a reduce launch; the network's sumsq blocks must start at entry a.blocks of
// a.sumsq_blocks.
void reduce_add_net(ReduceArgs& a, const rslx_mlp& n, const TrainBufs& t) {
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

int32_t reduce_net(const rslx_mlp& n, const TrainBufs& t, hipStream_t s) {
  ReduceArgs a;
  memset(&a, 0, sizeof a);
  a.sumsq_blocks = t.sumsq;
  reduce_add_net(a, n, t);
  RSLX_HIP(launch_reduce_partials(a, s));
  return RSLX_OK;
}

}  // namespace

size_t rslx_ppo_update_workspace_bytes(const rslx_mlp* actor, const rslx_mlp* critic, const rslx_rollout* ro,
                                       const rslx_ppo_cfg* cfg, const rslx_sym* sym, const rslx_rnd_train* rnd) {
  if (ppo_validate(actor, critic, ro, cfg, sym, rnd, false) != RSLX_OK) return 0;
  Carver c(nullptr);
  PpoPlan p;
  ppo_plan(c, actor, critic, ro, cfg, sym, rnd, p);
  return p.bytes;
}

}  // extern "C"

namespace {
// Shared body of rslx_ppo_update and rslx_ppo_update_dc: with `counters` the permutation stream index and the
// optimiser step counts are read from device memory by the kernels and advanced at the end of the call.
int32_t ppo_update_impl(rslx_mlp* actor, rslx_mlp* critic, const rslx_rollout* ro, const rslx_ppo_cfg* cfg,
                        const rslx_sym* sym, const rslx_rnd_train* rnd, int64_t* adam_step, rslx_dev_counters* counters,
                        float* stats, void* ws, size_t ws_bytes, void* stream) {
  RSLX_TRY(ppo_validate(actor, critic, ro, cfg, sym, rnd, true));
  if ((!adam_step && !counters) || !stats) return fail(RSLX_ERR_INVALID_ARG, "rslx_ppo_update: null adam_step or stats");
  int64_t host_step = 0, host_rnd_step = 0;      // stand-ins for the host counters in the device-counter variant
  if (counters) adam_step = &host_step;
  int64_t* rnd_step = rnd ? (counters ? &host_rnd_step : rnd->adam_step) : nullptr;
  if (rnd && !rnd_step) return fail(RSLX_ERR_INVALID_ARG, "rslx_ppo_update: rnd adam_step null");
  hipStream_t s = (hipStream_t)stream;
  Carver c(ws);
  PpoPlan p;
  ppo_plan(c, actor, critic, ro, cfg, sym, rnd, p);
  if (!ws || ws_bytes < p.bytes) return fail(RSLX_ERR_WORKSPACE, "rslx_ppo_update: workspace %zu < %zu bytes", ws_bytes, p.bytes);
  const int A = ro->A, L_a = actor->n_layers, L_c = critic->n_layers;

  {
    std::vector<uint64_t> bases(cfg->epochs);
    for (int e = 0; e < cfg->epochs; ++e)
      bases[e] = mix64_host(mix64_host(mix64_host(cfg->seed) ^ cfg->call_index) ^ (uint64_t)(e + cfg->epoch_offset));
    RSLX_HIP(launch_permutations(bases.data(), cfg->epochs, p.B, p.perms, p.perm_ws, s, mix64_host(cfg->seed),
                                 counters ? &counters->call_index : nullptr, cfg->epoch_offset));
  }

  for (int e = 0; e < cfg->epochs; ++e) {
    for (int m = 0; m < cfg->minibatches; ++m) {
      const int32_t* idx = p.perms + (size_t)e * p.B + (size_t)m * p.mb;
      float* stats_row = stats + ((size_t)e * cfg->minibatches + m) * RSLX_NSTATS;

      XView xa, xc;
      xa.base = ro->obs_actor; xa.ld = ro->Da; xa.row_idx = idx; xa.src_rows = p.B;
      xc.base = ro->obs_critic; xc.ld = ro->Dc; xc.row_idx = idx; xc.src_rows = p.B;
      if (sym) {
        xa.idx_mod = xc.idx_mod = p.mb;
        xa.map_from = xc.map_from = p.mb;
        xa.col_map = sym->perm_obs_a; xa.col_sign = sym->sign_obs_a;
        xc.col_map = sym->perm_obs_c; xc.col_sign = sym->sign_obs_c;
      }
      NetJob fj[2] = {NetJob{actor, xa, p.rows, &p.actor.act}, NetJob{critic, xc, p.rows, &p.critic.act}};
      RSLX_TRY(forward_nets(fj, 2, s, p.fused_head));

      PpoLossArgs la;
      memset(&la, 0, sizeof la);
      la.mu = p.actor.act.out[L_a - 1];
      la.v = p.critic.act.out[L_c - 1];
      la.log_std = actor->params + weight_count(*actor);
      la.idx = idx;
      la.actions = ro->actions; la.logp_old = ro->logp; la.adv = ro->advantages; la.returns = ro->returns;
      la.v_old = ro->values; la.mu_old = ro->mu; la.sigma_old = ro->sigma;
      la.perm_act = sym ? sym->perm_act : nullptr;
      la.sign_act = sym ? sym->sign_act : nullptr;
      la.mb = p.mb; la.rows = p.rows; la.A = A;
      la.clip = cfg->clip; la.value_coef = cfg->value_coef; la.entropy_coef = cfg->entropy_coef;
      la.mirror_coef = sym ? sym->mirror_loss_coef : 0.f;
      la.clipped_value = cfg->use_clipped_value_loss;
      la.d_mu = p.actor.d_out; la.d_v = p.critic.d_out;
      la.partials = p.loss_partials;
      if (p.fused_head) {
        PpoHeadArgs ha;
        ha.loss = la;
        ha.h_a = p.actor.act.out[L_a - 2]; ha.h_c = p.critic.act.out[L_c - 2];
        ha.w_a = actor->params + layer_offset(*actor, L_a - 1); ha.w_c = critic->params + layer_offset(*critic, L_c - 1);
        ha.dz_a = p.actor.act.dz[L_a - 2]; ha.dz_c = p.critic.act.dz[L_c - 2];
        ha.Ha = actor->dims[L_a - 1]; ha.Hc = critic->dims[L_c - 1];
        ha.alpha_a = actor->elu_alpha; ha.alpha_c = critic->elu_alpha;
        RSLX_HIP(launch_ppo_head(ha, s));
      } else {
        RSLX_HIP(launch_ppo_loss(la, s));
      }
      BwdJob bj[2] = {BwdJob{actor, xa, p.rows, &p.actor.act, p.actor.d_out, p.actor.wt, p.actor.partials, &p.actor.plan},
                      BwdJob{critic, xc, p.rows, &p.critic.act, p.critic.d_out, p.critic.wt, p.critic.partials, &p.critic.plan}};
      RSLX_TRY(backward_nets(bj, 2, s, p.fused_head));
      {   // one launch: both networks' split sums and the loss head's sums
        ReduceArgs ra;
        memset(&ra, 0, sizeof ra);
        ra.sumsq_blocks = p.sumsq_all;
        reduce_add_net(ra, *actor, p.actor);
        reduce_add_net(ra, *critic, p.critic);
        ra.finish.partials = p.loss_partials; ra.finish.blocks = p.loss_blocks;
        ra.finish.rows = p.rows; ra.finish.mb = p.mb; ra.finish.A = A;
        ra.finish.log_std = la.log_std; ra.finish.entropy_coef = cfg->entropy_coef;
        ra.finish.d_log_std = actor->grads + weight_count(*actor);
        ra.finish.stats_row = stats_row;
        ra.finish.sumsq_slot = p.sumsq_all + p.actor.n_sumsq + p.critic.n_sumsq;
        RSLX_HIP(launch_reduce_partials(ra, s));
      }

      const int64_t t = *adam_step + 1;
      AdamArgs aa;
      memset(&aa, 0, sizeof aa);
      aa.seg[0] = AdamSegment{actor->params, actor->grads, actor->adam_m, actor->adam_v, param_count(*actor)};
      aa.seg[1] = AdamSegment{critic->params, critic->grads, critic->adam_m, critic->adam_v, param_count(*critic)};
      aa.n_seg = 2;
      aa.sumsq_blocks = p.sumsq_all; aa.n_sumsq = p.actor.n_sumsq + p.critic.n_sumsq + 1;
      aa.max_grad_norm = cfg->max_grad_norm;
      aa.lr = cfg->lr; aa.beta1 = cfg->beta1; aa.beta2 = cfg->beta2; aa.eps = cfg->adam_eps;
      aa.bc1 = bias_correction(cfg->beta1, t); aa.bc2 = bias_correction(cfg->beta2, t);
      if (counters) { aa.step_dev = &counters->adam_step; aa.step_off = (int32_t)t; }
      aa.grad_norm_out = stats_row + RSLX_STAT_GRAD_NORM;
      RSLX_HIP(launch_adam(aa, s));
      *adam_step = t;

      if (rnd) {
        const rslx_mlp& pr = *rnd->predictor;
        const int K = pr.dims[pr.n_layers];
        XView xr;
        xr.base = ro->obs_actor; xr.ld = ro->Da; xr.row_idx = idx; xr.src_rows = p.B;
        if (rnd->subset_idx) { xr.col_map = rnd->subset_idx; xr.map_from = 0; }
        NetJob rj[2] = {NetJob{&pr, xr, p.mb, &p.pred.act}, NetJob{rnd->target, xr, p.mb, &p.targ}};
        RSLX_TRY(forward_nets(rj, 2, s));
        const int nbm = mse_num_blocks((int64_t)p.mb * K);
        RSLX_HIP(launch_mse(p.pred.act.out[pr.n_layers - 1], p.targ.out[pr.n_layers - 1], nullptr, p.mb, K,
                            p.pred.d_out, p.mse_partials, s));
        RSLX_HIP(launch_mse_finish(p.mse_partials, nbm, (int64_t)p.mb * K, stats_row + RSLX_STAT_RND_LOSS, s));
        BwdJob rb{&pr, xr, p.mb, &p.pred.act, p.pred.d_out, p.pred.wt, p.pred.partials, &p.pred.plan};
        RSLX_TRY(backward_nets(&rb, 1, s));
        RSLX_TRY(reduce_net(pr, p.pred, s));
        const int64_t tr = *rnd_step + 1;
        AdamArgs ar;
        memset(&ar, 0, sizeof ar);
        ar.seg[0] = AdamSegment{pr.params, pr.grads, pr.adam_m, pr.adam_v, param_count(pr)};
        ar.n_seg = 1;
        ar.sumsq_blocks = p.pred.sumsq; ar.n_sumsq = 0;
        ar.max_grad_norm = 0.f;
        ar.lr = rnd->lr; ar.beta1 = cfg->beta1; ar.beta2 = cfg->beta2; ar.eps = cfg->adam_eps;
        ar.bc1 = bias_correction(cfg->beta1, tr); ar.bc2 = bias_correction(cfg->beta2, tr);
        if (counters) { ar.step_dev = &counters->rnd_adam_step; ar.step_off = (int32_t)tr; }
        RSLX_HIP(launch_adam(ar, s));
        *rnd_step = tr;
      }
    }
  }
  if (counters) RSLX_HIP(advance_counters(counters, 0, 1, host_step, host_rnd_step, s));
  return RSLX_OK;
}
}  // namespace

extern "C" {

int32_t rslx_ppo_update(rslx_mlp* actor, rslx_mlp* critic, const rslx_rollout* ro, const rslx_ppo_cfg* cfg,
                        const rslx_sym* sym, const rslx_rnd_train* rnd, int64_t* adam_step, float* stats, void* ws,
                        size_t ws_bytes, void* stream) {
  if (!adam_step) return fail(RSLX_ERR_INVALID_ARG, "rslx_ppo_update: null adam_step or stats");
  return ppo_update_impl(actor, critic, ro, cfg, sym, rnd, adam_step, nullptr, stats, ws, ws_bytes, stream);
}

int32_t rslx_ppo_update_dc(rslx_mlp* actor, rslx_mlp* critic, const rslx_rollout* ro, const rslx_ppo_cfg* cfg,
                           const rslx_sym* sym, const rslx_rnd_train* rnd, rslx_dev_counters* counters, float* stats,
                           void* ws, size_t ws_bytes, void* stream) {
  if (!counters) return fail(RSLX_ERR_INVALID_ARG, "rslx_ppo_update_dc: null counters");
  return ppo_update_impl(actor, critic, ro, cfg, sym, rnd, nullptr, counters, stats, ws, ws_bytes, stream);
}

// ---- behaviour cloning ---------------------------------------------------------------------------------------------
namespace {
struct BcPlan {
  int32_t mb;
  int32_t* perms = nullptr;
  void* perm_ws = nullptr;
  TrainBufs student;
  NetBufs teacher;
  float* targets = nullptr;
  double* mse_partials = nullptr;
  size_t bytes = 0;
};

void bc_plan(Carver& c, const rslx_mlp* student, const rslx_mlp* teacher, int32_t B, const rslx_bc_cfg* cfg, BcPlan& p) {
  p.mb = B / cfg->minibatches;
  p.perms = c.take<int32_t>((size_t)cfg->epochs * B);
  p.perm_ws = c.take<char>(perm_workspace_bytes(B));
  carve_train(c, *student, p.mb, 1, p.student);
  p.student.sumsq = c.take<double>((size_t)p.student.n_sumsq + 1);
  const int A = student->dims[student->n_layers];
  if (teacher) {
    carve_net(c, *teacher, p.mb, false, p.teacher);
    p.targets = c.take<float>((size_t)B * A);
  }
  p.mse_partials = c.take<double>(mse_num_blocks((int64_t)p.mb * A));
  p.bytes = c.off + 256;
}

int32_t bc_validate(const rslx_mlp* student, const rslx_mlp* teacher, int32_t B, const rslx_bc_cfg* cfg, bool need_buffers) {
  if (!cfg) return fail(RSLX_ERR_INVALID_ARG, "rslx_bc_update: null cfg");
  RSLX_TRY(check_mlp(student, "rslx_bc_update student", need_buffers));
  if (teacher) {
    RSLX_TRY(check_mlp(teacher, "rslx_bc_update teacher", false));
    if (teacher->dims[teacher->n_layers] != student->dims[student->n_layers])
      return fail(RSLX_ERR_SHAPE, "rslx_bc_update: teacher and student action widths differ");
  }
  if (B < 1 || cfg->minibatches < 1 || cfg->epochs < 0 || B % cfg->minibatches != 0)
    return fail(RSLX_ERR_SHAPE, "rslx_bc_update: B = %d is not a positive multiple of minibatches = %d", B, cfg->minibatches);
  return RSLX_OK;
}
}  // namespace

size_t rslx_bc_update_workspace_bytes(const rslx_mlp* student, const rslx_mlp* teacher, int32_t B, const rslx_bc_cfg* cfg) {
  if (bc_validate(student, teacher, B, cfg, false) != RSLX_OK) return 0;
  Carver c(nullptr);
  BcPlan p;
  bc_plan(c, student, teacher, B, cfg, p);
  return p.bytes;
}

}  // extern "C"

namespace {
// Shared body of rslx_bc_update and rslx_bc_update_dc (permutation stream and Adam step count from device memory).
int32_t bc_update_impl(rslx_mlp* student, const rslx_mlp* teacher, const float* obs_student, const float* obs_teacher,
                       const float* targets_or_null, int32_t B, const rslx_bc_cfg* cfg, int64_t* adam_step,
                       rslx_dev_counters* counters, float* stats, void* ws, size_t ws_bytes, void* stream) {
  int64_t host_step = 0;
  if (counters) adam_step = &host_step;
  const rslx_mlp* tch = targets_or_null ? nullptr : teacher;
  if (!targets_or_null && !teacher) return fail(RSLX_ERR_INVALID_ARG, "rslx_bc_update: need a teacher or precomputed targets");
  RSLX_TRY(bc_validate(student, tch, B, cfg, true));
  if (!obs_student || !stats) return fail(RSLX_ERR_INVALID_ARG, "rslx_bc_update: null pointer");
  if (tch && !obs_teacher) return fail(RSLX_ERR_INVALID_ARG, "rslx_bc_update: null teacher observations");
  hipStream_t s = (hipStream_t)stream;
  Carver c(ws);
  BcPlan p;
  bc_plan(c, student, tch, B, cfg, p);
  if (!ws || ws_bytes < p.bytes) return fail(RSLX_ERR_WORKSPACE, "rslx_bc_update: workspace %zu < %zu bytes", ws_bytes, p.bytes);
  const int A = student->dims[student->n_layers];
  const int Ls = student->n_layers;

  const float* targets = targets_or_null;
  if (tch) {                           // teacher means for every row, one minibatch-sized slab at a time
    for (int k = 0; k < cfg->minibatches; ++k) {
      NetBufs tb = p.teacher;
      tb.out[tch->n_layers - 1] = p.targets + (size_t)k * p.mb * A;
      XView xt; xt.base = obs_teacher + (size_t)k * p.mb * tch->dims[0]; xt.ld = tch->dims[0];
      NetJob j{tch, xt, p.mb, &tb};
      RSLX_TRY(forward_nets(&j, 1, s));
    }
    targets = p.targets;
  }
  {
    std::vector<uint64_t> bases(cfg->epochs);
    for (int e = 0; e < cfg->epochs; ++e)
      bases[e] = mix64_host(mix64_host(mix64_host(cfg->seed) ^ cfg->call_index) ^ (uint64_t)(e + cfg->epoch_offset));
    RSLX_HIP(launch_permutations(bases.data(), cfg->epochs, B, p.perms, p.perm_ws, s, mix64_host(cfg->seed),
                                 counters ? &counters->call_index : nullptr, cfg->epoch_offset));
  }
  const int nbm = mse_num_blocks((int64_t)p.mb * A);
  for (int e = 0; e < cfg->epochs; ++e) {
    for (int m = 0; m < cfg->minibatches; ++m) {
      const int32_t* idx = p.perms + (size_t)e * B + (size_t)m * p.mb;
      float* stats_row = stats + ((size_t)e * cfg->minibatches + m) * RSLX_NSTATS;
      RSLX_HIP(launch_fill(stats_row, RSLX_NSTATS, 0.f, s));
      XView xs; xs.base = obs_student; xs.ld = student->dims[0]; xs.row_idx = idx; xs.src_rows = B;
      NetJob fj{student, xs, p.mb, &p.student.act};
      RSLX_TRY(forward_nets(&fj, 1, s));
      RSLX_HIP(launch_mse(p.student.act.out[Ls - 1], targets, idx, p.mb, A, p.student.d_out, p.mse_partials, s));
      RSLX_HIP(launch_mse_finish(p.mse_partials, nbm, (int64_t)p.mb * A, stats_row, s));
      BwdJob bj{student, xs, p.mb, &p.student.act, p.student.d_out, p.student.wt, p.student.partials, &p.student.plan};
      RSLX_TRY(backward_nets(&bj, 1, s));
      RSLX_TRY(reduce_net(*student, p.student, s));
      const int64_t t = *adam_step + 1;
      AdamArgs aa;
      memset(&aa, 0, sizeof aa);
      aa.seg[0] = AdamSegment{student->params, student->grads, student->adam_m, student->adam_v, weight_count(*student)};
      aa.n_seg = 1;
      aa.sumsq_blocks = p.student.sumsq; aa.n_sumsq = p.student.n_sumsq;
      aa.max_grad_norm = cfg->max_grad_norm;
      aa.lr = cfg->lr; aa.beta1 = cfg->beta1; aa.beta2 = cfg->beta2; aa.eps = cfg->adam_eps;
      aa.bc1 = bias_correction(cfg->beta1, t); aa.bc2 = bias_correction(cfg->beta2, t);
      if (counters) { aa.step_dev = &counters->adam_step; aa.step_off = (int32_t)t; }
      aa.grad_norm_out = stats_row + RSLX_STAT_GRAD_NORM;
      RSLX_HIP(launch_adam(aa, s));
      *adam_step = t;
    }
  }
  if (counters) RSLX_HIP(advance_counters(counters, 0, 1, host_step, 0, s));
  return RSLX_OK;
}
}  // namespace

extern "C" {

int32_t rslx_bc_update(rslx_mlp* student, const rslx_mlp* teacher, const float* obs_student, const float* obs_teacher,
                       const float* targets_or_null, int32_t B, const rslx_bc_cfg* cfg, int64_t* adam_step, float* stats,
                       void* ws, size_t ws_bytes, void* stream) {
  if (!adam_step) return fail(RSLX_ERR_INVALID_ARG, "rslx_bc_update: null pointer");
  return bc_update_impl(student, teacher, obs_student, obs_teacher, targets_or_null, B, cfg, adam_step, nullptr, stats, ws,
                        ws_bytes, stream);
}

int32_t rslx_bc_update_dc(rslx_mlp* student, const rslx_mlp* teacher, const float* obs_student, const float* obs_teacher,
                          const float* targets_or_null, int32_t B, const rslx_bc_cfg* cfg, rslx_dev_counters* counters,
                          float* stats, void* ws, size_t ws_bytes, void* stream) {
  if (!counters) return fail(RSLX_ERR_INVALID_ARG, "rslx_bc_update_dc: null counters");
  return bc_update_impl(student, teacher, obs_student, obs_teacher, targets_or_null, B, cfg, nullptr, counters, stats, ws,
                        ws_bytes, stream);
}

// ---- one collection step of the distillation loop ---------------------------------------------------------------------
size_t rslx_bc_collect_workspace_bytes(const rslx_mlp* student, const rslx_mlp* teacher, int32_t N) {
  if (N <= 0 || !student || !teacher) return 256;
  Carver c(nullptr);
  return act_carve(c, student, teacher, N, nullptr, nullptr);
}

int32_t rslx_bc_collect(const rslx_mlp* student, const rslx_mlp* teacher, const float* obs_student, const float* obs_teacher,
                        int32_t N, float* actions, float* targets, void* ws, size_t ws_bytes, void* stream) {
  if (N < 0) return fail(RSLX_ERR_SHAPE, "rslx_bc_collect: N = %d", N);
  RSLX_TRY(check_mlp(student, "rslx_bc_collect student", false));
  RSLX_TRY(check_mlp(teacher, "rslx_bc_collect teacher", false));
  if (student->dims[student->n_layers] != teacher->dims[teacher->n_layers])
    return fail(RSLX_ERR_SHAPE, "rslx_bc_collect: student and teacher action widths differ");
  if (!obs_student || !obs_teacher || !actions || !targets) return fail(RSLX_ERR_INVALID_ARG, "rslx_bc_collect: null pointer");
  if (N == 0) return RSLX_OK;
  if (!ws || ws_bytes < rslx_bc_collect_workspace_bytes(student, teacher, N))
    return fail(RSLX_ERR_WORKSPACE, "rslx_bc_collect: workspace too small");
  hipStream_t s = (hipStream_t)stream;
  {
    FusedForwardArgs fa;
    memset(&fa, 0, sizeof fa);
    fa.n_rows = N;
    fa.n_nets = 2;
    fa.max_dim = max_dim_of(*student) > max_dim_of(*teacher) ? max_dim_of(*student) : max_dim_of(*teacher);
    fa.net[0] = fused_net(*student, obs_student, student->dims[0], nullptr, actions, false);
    fa.net[1] = fused_net(*teacher, obs_teacher, teacher->dims[0], nullptr, targets, false);
    if (fused_forward_supported(fa)) {
      RSLX_HIP(launch_fused_forward(fa, s));
      return RSLX_OK;
    }
  }
  Carver c(ws);
  NetBufs bs, bt;
  act_carve(c, student, teacher, N, &bs, &bt);
  bs.out[student->n_layers - 1] = actions;
  bt.out[teacher->n_layers - 1] = targets;
  XView xs; xs.base = obs_student; xs.ld = student->dims[0];
  XView xt; xt.base = obs_teacher; xt.ld = teacher->dims[0];
  NetJob jobs[2] = {NetJob{student, xs, N, &bs}, NetJob{teacher, xt, N, &bt}};
  RSLX_TRY(forward_nets(jobs, 2, s));
  return RSLX_OK;
}


// ---- symmetry augmentation ---------------------------------------------------------------------------------------------
int32_t rslx_sym_augment(const rslx_sym* sym, const float* obs_in, const float* act_in, int32_t B, int32_t D, int32_t A,
                         float* obs_out, float* act_out, void* stream) {
  if (!sym) return fail(RSLX_ERR_INVALID_ARG, "rslx_sym_augment: null sym");
  if (B < 0 || D < 0 || A < 0) return fail(RSLX_ERR_SHAPE, "rslx_sym_augment: negative size");
  hipStream_t s = (hipStream_t)stream;
  if (obs_in) {
    if (!involution_ok(sym->perm_obs_a_host, sym->sign_obs_a_host, D))
      return fail(RSLX_ERR_INVALID_ARG, "rslx_sym_augment: observation map is not an involutive signed permutation");
    if (!obs_out || !sym->perm_obs_a || !sym->sign_obs_a) return fail(RSLX_ERR_INVALID_ARG, "rslx_sym_augment: null pointer");
  }
  if (act_in) {
    if (!involution_ok(sym->perm_act_host, sym->sign_act_host, A))
      return fail(RSLX_ERR_INVALID_ARG, "rslx_sym_augment: action map is not an involutive signed permutation");
    if (!act_out || !sym->perm_act || !sym->sign_act) return fail(RSLX_ERR_INVALID_ARG, "rslx_sym_augment: null pointer");
  }
  if (obs_in) RSLX_HIP(launch_sym_augment(obs_in, B, D, sym->perm_obs_a, sym->sign_obs_a, obs_out, s));
  if (act_in) RSLX_HIP(launch_sym_augment(act_in, B, A, sym->perm_act, sym->sign_act, act_out, s));
  return RSLX_OK;
}

// ---- RND reward -----------------------------------------------------------------------------------------------------
static size_t rnd_carve(Carver& c, const rslx_mlp* net, int32_t N, NetBufs* bp, NetBufs* bt, double** partials) {
  NetBufs p, t;
  carve_net(c, *net, N, false, p);
  carve_net(c, *net, N, false, t);
  double* pp = c.take<double>((size_t)rnd_num_blocks(N) * 2 + 2);
  if (bp) *bp = p;
  if (bt) *bt = t;
  if (partials) *partials = pp;
  return c.off + 256;
}

size_t rslx_rnd_workspace_bytes(const rslx_mlp* target, int32_t N) {
  if (!target || N <= 0 || target->n_layers < 1 || target->n_layers > RSLX_MAX_LAYERS) return 256;
  Carver c(nullptr);
  return rnd_carve(c, target, N, nullptr, nullptr, nullptr);
}

int32_t rslx_rnd(const rslx_mlp* target, const rslx_mlp* predictor, const float* obs, int32_t N, int32_t D,
                 const int32_t* subset_idx_or_null, int32_t n_subset, float* running, float weight, int32_t update_stats,
                 float* r_int_out, float* rewards_inout_or_null, void* ws, size_t ws_bytes, void* stream) {
  RSLX_TRY(check_mlp(target, "rslx_rnd target", false));
  RSLX_TRY(check_mlp(predictor, "rslx_rnd predictor", false));
  if (target->n_layers != predictor->n_layers) return fail(RSLX_ERR_SHAPE, "rslx_rnd: networks differ in depth");
  for (int i = 0; i <= target->n_layers; ++i)
    if (target->dims[i] != predictor->dims[i]) return fail(RSLX_ERR_SHAPE, "rslx_rnd: networks differ in shape");
  if (N < 0 || D < 1) return fail(RSLX_ERR_SHAPE, "rslx_rnd: N = %d, D = %d", N, D);
  if (n_subset != target->dims[0] || (!subset_idx_or_null && n_subset != D)) return fail(RSLX_ERR_SHAPE, "rslx_rnd: subset width");
  if (!obs || !running || !r_int_out) return fail(RSLX_ERR_INVALID_ARG, "rslx_rnd: null pointer");
  if (N == 0) return RSLX_OK;
  if (!ws || ws_bytes < rslx_rnd_workspace_bytes(target, N)) return fail(RSLX_ERR_WORKSPACE, "rslx_rnd: workspace too small");
  hipStream_t s = (hipStream_t)stream;
  Carver c(ws);
  NetBufs bp, bt;
  double* partials = nullptr;
  rnd_carve(c, target, N, &bp, &bt, &partials);
  XView x;
  x.base = obs; x.ld = D;
  if (subset_idx_or_null) { x.col_map = subset_idx_or_null; x.map_from = 0; }
  const int L = target->n_layers;
  FusedForwardArgs fa;
  memset(&fa, 0, sizeof fa);
  fa.n_rows = N; fa.n_nets = 2; fa.max_dim = max_dim_of(*target);
  fa.net[0] = fused_net(*predictor, obs, D, subset_idx_or_null, bp.out[L - 1], false);
  fa.net[1] = fused_net(*target, obs, D, subset_idx_or_null, bt.out[L - 1], false);
  if (fused_forward_supported(fa)) {
    RSLX_HIP(launch_fused_forward(fa, s));
  } else {
    NetJob jobs[2] = {NetJob{predictor, x, N, &bp}, NetJob{target, x, N, &bt}};
    RSLX_TRY(forward_nets(jobs, 2, s));
  }
  RSLX_HIP(launch_rnd_reward(bp.out[L - 1], bt.out[L - 1], N, target->dims[L], running, weight, update_stats ? 1 : 0,
                             r_int_out, rewards_inout_or_null, partials, s));
  return RSLX_OK;
}

}  // extern "C"

// ======================================================================================================
// Recurrent actor-critic: GRU or LSTM memories in front of the MLPs, back-propagation through time.
// ======================================================================================================
namespace {

int gates(const rslx_memory& g) { return g.cell == RSLX_CELL_LSTM ? 4 : 3; }
int gate_width(const rslx_memory& g) { return gates(g) * g.hidden; }                              // G H
int state_width(const rslx_memory& g) { return g.cell == RSLX_CELL_LSTM ? 2 * g.hidden : g.hidden; }   // S
int64_t gru_off_bih(const rslx_memory& g) { return (int64_t)g.in_dim * gate_width(g); }
int64_t gru_off_whh(const rslx_memory& g) { return gru_off_bih(g) + gate_width(g); }
int64_t gru_off_bhh(const rslx_memory& g) { return gru_off_whh(g) + (int64_t)g.hidden * gate_width(g); }
int64_t gru_count(const rslx_memory& g) { return gru_off_bhh(g) + gate_width(g); }

int32_t check_gru(const rslx_memory* g, const char* name, bool trainable) {
  if (!g) return fail(RSLX_ERR_INVALID_ARG, "%s: null memory", name);
  if (g->cell != RSLX_CELL_GRU && g->cell != RSLX_CELL_LSTM) return fail(RSLX_ERR_INVALID_ARG, "%s: unknown cell %d", name, g->cell);
  if (g->in_dim < 1 || g->in_dim > (1 << 20) || g->hidden < 4 || g->hidden > (1 << 16) || g->hidden % 4 != 0)
    return fail(RSLX_ERR_SHAPE, "%s: in_dim = %d, hidden = %d (hidden must be a multiple of 4)", name, g->in_dim, g->hidden);
  if (!g->params || !aligned16(g->params)) return fail(RSLX_ERR_INVALID_ARG, "%s: params null or not 16-byte aligned", name);
  if (trainable) {
    if (!g->grads || !g->adam_m || !g->adam_v) return fail(RSLX_ERR_INVALID_ARG, "%s: grads / adam_m / adam_v required", name);
    if (!aligned16(g->grads) || !aligned16(g->adam_m) || !aligned16(g->adam_v))
      return fail(RSLX_ERR_INVALID_ARG, "%s: optimiser buffers not 16-byte aligned", name);
  }
  return RSLX_OK;
}

// C[M, G H] = X W + b for one side of a memory's gates (X given as a view or as a plain matrix).
GemmProblem gate_problem(const XView& x, int K, const float* W, const float* b, float* C, int M, int H3) {
  GemmProblem p = blank_problem();
  set_x(p, x);
  p.B = W; p.ldb = H3; p.aux = b;
  p.C = C; p.ldc = H3;
  p.M = M; p.N = H3; p.K = K;
  p.elu = 0; p.alpha = 1.f;
  p.a_vec = (K % 4 == 0 && p.lda % 4 == 0 && aligned16(p.A) && p.col_map == nullptr) ? 1 : 0;
  p.b_vec = (H3 % 4 == 0 && aligned16(W)) ? 1 : 0;
  return p;
}

XView plain_view(const float* base, int ld) {
  XView x;
  x.base = base; x.ld = ld;
  return x;
}

struct StepBufs {     // one memory's buffers of a single act step
  float* hin = nullptr;     // [N, S] state the step starts from (after reset)
  float* gi = nullptr;      // [N, G H]
  float* hnew = nullptr;    // [N, S] values-only: the state is not written back
};

size_t act_recurrent_carve(Carver& c, const rslx_memory* ga, const rslx_memory* gc, int32_t N, StepBufs* ba, StepBufs* bc) {
  const rslx_memory* g[2] = {ga, gc};
  StepBufs* b[2] = {ba, bc};
  for (int k = 0; k < 2; ++k) {
    if (!g[k]) continue;
    StepBufs t;
    t.hin = c.take<float>((size_t)N * state_width(*g[k]));
    t.gi = c.take<float>((size_t)N * gate_width(*g[k]));
    t.hnew = c.take<float>((size_t)N * state_width(*g[k]));
    if (b[k]) *b[k] = t;
  }
  return c.off;
}

// hin -> gi -> new state (hidden-side contraction fused with the gates), for the memories listed (1 or 2), each with its own input matrix.
int32_t gru_step(const rslx_memory* const* g, const float* const* obs, const StepBufs* b, float* const* h_out, int count,
                 int32_t N, hipStream_t s) {
  GemmBatch bi;
  bi.count = count;
  StepFwdArgs sa;
  memset(&sa, 0, sizeof sa);
  sa.n_nets = count; sa.nb = N; sa.cell = g[0]->cell;
  for (int k = 0; k < count; ++k) {
    const rslx_memory& m = *g[k];
    bi.p[k] = gate_problem(plain_view(obs[k], m.in_dim), m.in_dim, m.params, m.params + gru_off_bih(m), b[k].gi, N, gate_width(m));
    // the new packed state goes to h_out[k] ([N, S]): h in its first H columns, an LSTM's c behind it
    sa.net[k] = StepFwdNet{b[k].gi, b[k].hin, h_out[k], m.cell == RSLX_CELL_LSTM ? h_out[k] + m.hidden : nullptr, nullptr,
                           m.params + gru_off_whh(m), m.params + gru_off_bhh(m), nullptr, m.hidden, state_width(m)};
  }
  RSLX_HIP(launch_gemm(GEMM_FWD, bi, s));
  RSLX_HIP(launch_step_fwd(sa, s));
  return RSLX_OK;
}

int32_t act_recurrent_validate(const rslx_memory* ga, const rslx_mlp* actor, const rslx_memory* gc, const rslx_mlp* critic,
                               bool values_only) {
  RSLX_TRY(check_gru(gc, "rslx_act_recurrent critic memory", false));
  RSLX_TRY(check_mlp(critic, "rslx_act_recurrent critic", false));
  if (critic->dims[0] != gc->hidden) return fail(RSLX_ERR_SHAPE, "rslx_act_recurrent: critic input width != memory width");
  if (!values_only) {
    RSLX_TRY(check_gru(ga, "rslx_act_recurrent actor memory", false));
    RSLX_TRY(check_mlp(actor, "rslx_act_recurrent actor", false));
    if (actor->dims[0] != ga->hidden) return fail(RSLX_ERR_SHAPE, "rslx_act_recurrent: actor input width != memory width");
    if (ga->cell != gc->cell) return fail(RSLX_ERR_UNSUPPORTED, "rslx_act_recurrent: the two memories use different cells");
  }
  return RSLX_OK;
}

}  // namespace

extern "C" {

size_t rslx_act_recurrent_workspace_bytes(const rslx_memory* gru_actor, const rslx_mlp* actor, const rslx_memory* gru_critic,
                                          const rslx_mlp* critic, int32_t N) {
  if (N <= 0 || !gru_critic || !critic) return 256;
  Carver c(nullptr);
  act_recurrent_carve(c, gru_actor, gru_critic, N, nullptr, nullptr);
  return (c.off + 255) / 256 * 256 + rslx_act_workspace_bytes(actor, critic, N);
}

}  // extern "C"

namespace {
// Shared body of rslx_act_recurrent and rslx_act_recurrent_dc (noise position from device memory).
int32_t act_recurrent_impl(const rslx_memory* gru_actor, const rslx_mlp* actor, const rslx_memory* gru_critic,
                           const rslx_mlp* critic, const float* obs_actor, const float* obs_critic, int32_t N,
                           float* h_actor, float* h_critic, const uint8_t* reset_or_null, float* h0_actor_out,
                           float* h0_critic_out, uint64_t seed, uint64_t step, rslx_dev_counters* counters,
                           const float* eps_or_null, float* actions, float* logp, float* values, float* mu, float* sigma,
                           uint32_t flags, void* ws, size_t ws_bytes, void* stream) {
  const bool values_only = (flags & RSLX_ACT_VALUES_ONLY) != 0;
  if (N < 0) return fail(RSLX_ERR_SHAPE, "rslx_act_recurrent: N = %d", N);
  RSLX_TRY(act_recurrent_validate(gru_actor, actor, gru_critic, critic, values_only));
  if (!obs_critic || !h_critic || !values) return fail(RSLX_ERR_INVALID_ARG, "rslx_act_recurrent: null critic input / state / output");
  if (!values_only && (!obs_actor || !h_actor)) return fail(RSLX_ERR_INVALID_ARG, "rslx_act_recurrent: null actor input / state");
  // everything the MLP stage would reject is rejected here, before the memories advance the caller's states
  if (!values_only && (!actions || !logp || !mu || !sigma)) return fail(RSLX_ERR_INVALID_ARG, "rslx_act_recurrent: null actor output");
  if (!values_only && !actor->has_log_std) return fail(RSLX_ERR_INVALID_ARG, "rslx_act_recurrent: actor needs log_std");
  if (critic->dims[critic->n_layers] != 1) return fail(RSLX_ERR_SHAPE, "rslx_act_recurrent: critic output width must be 1");
  if (!values_only && actor->dims[actor->n_layers] > RSLX_MAX_ACTIONS)
    return fail(RSLX_ERR_SHAPE, "rslx_act_recurrent: action width > %d", RSLX_MAX_ACTIONS);
  if (!aligned16(h_critic) || (!values_only && !aligned16(h_actor)) || (h0_actor_out && !aligned16(h0_actor_out)) ||
      (h0_critic_out && !aligned16(h0_critic_out)))
    return fail(RSLX_ERR_INVALID_ARG, "rslx_act_recurrent: state buffers not 16-byte aligned");
  if (N == 0) return RSLX_OK;
  const rslx_memory* ga = values_only ? nullptr : gru_actor;
  const rslx_mlp* a = values_only ? nullptr : actor;
  if (!ws || ws_bytes < rslx_act_recurrent_workspace_bytes(ga, a, gru_critic, critic, N))
    return fail(RSLX_ERR_WORKSPACE, "rslx_act_recurrent: workspace too small");
  hipStream_t s = (hipStream_t)stream;
  Carver c(ws);
  StepBufs ba, bc;
  act_recurrent_carve(c, ga, gru_critic, N, &ba, &bc);
  const size_t used = (c.off + 255) / 256 * 256;

  RowGatherArgs rg;
  memset(&rg, 0, sizeof rg);
  rg.nb = N; rg.reset = reset_or_null;
  if (ga) rg.job[rg.n_jobs++] = RowGatherJob{h_actor, ba.hin, values_only ? nullptr : h0_actor_out, state_width(*ga)};
  rg.job[rg.n_jobs++] = RowGatherJob{h_critic, bc.hin, values_only ? nullptr : h0_critic_out, state_width(*gru_critic)};
  RSLX_HIP(launch_row_gather(rg, s));

  const float* h_in_actor_mlp = h_actor;
  const float* h_in_critic_mlp = values_only ? bc.hnew : h_critic;
  if (ga) {
    const rslx_memory* g[2] = {ga, gru_critic};
    const float* obs[2] = {obs_actor, obs_critic};
    const StepBufs b[2] = {ba, bc};
    float* out[2] = {h_actor, h_critic};
    RSLX_TRY(gru_step(g, obs, b, out, 2, N, s));
  } else {
    const rslx_memory* g[1] = {gru_critic};
    const float* obs[1] = {obs_critic};
    const StepBufs b[1] = {bc};
    float* out[1] = {bc.hnew};
    RSLX_TRY(gru_step(g, obs, b, out, 1, N, s));
  }
  return act_impl(a, critic, h_in_actor_mlp, h_in_critic_mlp, N, seed, step, counters, eps_or_null, actions, logp, values,
                  mu, sigma, flags, static_cast<char*>(ws) + used, ws_bytes - used, stream, ga ? state_width(*ga) : 0,
                  state_width(*gru_critic));
}
}  // namespace

extern "C" {

int32_t rslx_act_recurrent(const rslx_memory* mem_actor, const rslx_mlp* actor, const rslx_memory* mem_critic,
                           const rslx_mlp* critic, const float* obs_actor, const float* obs_critic, int32_t N,
                           float* h_actor, float* h_critic, const uint8_t* reset_or_null, float* h0_actor_out,
                           float* h0_critic_out, uint64_t seed, uint64_t step, const float* eps_or_null, float* actions,
                           float* logp, float* values, float* mu, float* sigma, uint32_t flags, void* ws, size_t ws_bytes,
                           void* stream) {
  return act_recurrent_impl(mem_actor, actor, mem_critic, critic, obs_actor, obs_critic, N, h_actor, h_critic, reset_or_null,
                            h0_actor_out, h0_critic_out, seed, step, nullptr, eps_or_null, actions, logp, values, mu, sigma,
                            flags, ws, ws_bytes, stream);
}

int32_t rslx_act_recurrent_dc(const rslx_memory* mem_actor, const rslx_mlp* actor, const rslx_memory* mem_critic,
                              const rslx_mlp* critic, const float* obs_actor, const float* obs_critic, int32_t N,
                              float* h_actor, float* h_critic, const uint8_t* reset_or_null, float* h0_actor_out,
                              float* h0_critic_out, uint64_t seed, rslx_dev_counters* counters, const float* eps_or_null,
                              float* actions, float* logp, float* values, float* mu, float* sigma, uint32_t flags, void* ws,
                              size_t ws_bytes, void* stream) {
  if (!counters) return fail(RSLX_ERR_INVALID_ARG, "rslx_act_recurrent_dc: null counters");
  return act_recurrent_impl(mem_actor, actor, mem_critic, critic, obs_actor, obs_critic, N, h_actor, h_critic, reset_or_null,
                            h0_actor_out, h0_critic_out, seed, 0, counters, eps_or_null, actions, logp, values, mu, sigma,
                            flags, ws, ws_bytes, stream);
}

}  // extern "C"

namespace {

struct RnnBufs {          // per memory, one column-wise minibatch (rows = T * nb)
  float* gi = nullptr;    // [rows, G H] input-side gate terms
  float* gh = nullptr;    // [rows, G H] what the forward steps store for the backward pass (GRU: gh, LSTM: a)
  float* dgi = nullptr;   // [rows, G H] GRU only: gradient w.r.t. gi
  float* dgh = nullptr;   // [rows, G H] gradient w.r.t. the hidden-side terms (LSTM: w.r.t. a, serves both sides)
  float* hin = nullptr;   // [rows, S] packed state every step starts from
  float* hs = nullptr;    // [rows, H] new hidden states = input of the MLP
  float* dh = nullptr;    // [rows, H] gradient from the MLP
  float* direct = nullptr;  // [nb, H] carried between backward steps (GRU: dh z, LSTM: gradient w.r.t. c)
  SplitPlan plan;           // layer 0: W_ih / b_ih, layer 1: W_hh / b_hh
  float* partials = nullptr;
};

struct RnnPlan {
  int32_t T, N, nb, rows;
  bool fused_head = false;
  int32_t loss_blocks = 0;
  int32_t* perms = nullptr;      // [E, N]
  void* perm_ws = nullptr;
  int32_t* rows_all = nullptr;   // [E, M, T, nb] roll-out rows of every minibatch
  TrainBufs actor, critic;
  RnnBufs ma, mc;
  double* sumsq_all = nullptr;
  int32_t n_sumsq = 0;
  double* loss_partials = nullptr;
  size_t bytes = 0;
};

void carve_memory(Carver& c, const rslx_memory& g, int32_t rows, int32_t nb, RnnBufs& b, int group = 2) {
  const size_t H = g.hidden, GH = gate_width(g), S = state_width(g);
  b.gi = c.take<float>(rows * GH); b.gh = c.take<float>(rows * GH);
  b.dgi = g.cell == RSLX_CELL_GRU ? c.take<float>(rows * GH) : nullptr;
  b.dgh = c.take<float>(rows * GH);
  b.hin = c.take<float>(rows * S); b.hs = c.take<float>(rows * H); b.dh = c.take<float>(rows * H);
  b.direct = c.take<float>(nb * H);
  plan_layer(b.plan, 0, g.in_dim, (int)GH, rows, group, false);
  plan_layer(b.plan, 1, g.hidden, (int)GH, rows, group, false);
  b.partials = c.take<float>((size_t)b.plan.total);
}

void rnn_plan(Carver& c, const rslx_memory* ga, const rslx_mlp* actor, const rslx_memory* gc, const rslx_mlp* critic,
              const rslx_rollout* ro, const rslx_ppo_cfg* cfg, RnnPlan& p) {
  p.T = ro->T; p.N = ro->N;
  p.nb = ro->N / cfg->minibatches;
  p.rows = p.T * p.nb;
  p.perms = c.take<int32_t>((size_t)cfg->epochs * p.N);
  p.perm_ws = c.take<char>(perm_workspace_bytes(p.N));
  p.rows_all = c.take<int32_t>((size_t)cfg->epochs * p.T * p.N);
  carve_train(c, *actor, p.rows, 2, p.actor, true);
  carve_train(c, *critic, p.rows, 2, p.critic, true);
  carve_memory(c, *ga, p.rows, p.nb, p.ma);
  carve_memory(c, *gc, p.rows, p.nb, p.mc);
  p.n_sumsq = p.actor.n_sumsq + p.critic.n_sumsq + p.ma.plan.blocks + p.mc.plan.blocks + 1;
  p.sumsq_all = c.take<double>((size_t)p.n_sumsq + 1);
  p.fused_head = actor->n_layers >= 2 && critic->n_layers >= 2 &&
                 ppo_head_supported(actor->dims[actor->n_layers - 1], critic->dims[critic->n_layers - 1], ro->A);
  p.loss_blocks = p.fused_head ? ppo_head_num_blocks(p.rows, false) : ppo_loss_num_blocks(p.rows);
  p.loss_partials = c.take<double>((size_t)p.loss_blocks * (PPO_NPART_FIXED + ro->A));
  p.bytes = c.off + 256;
}

int32_t rnn_validate(const rslx_memory* ga, const rslx_mlp* actor, const rslx_memory* gc, const rslx_mlp* critic,
                     const rslx_rollout* ro, const rslx_ppo_cfg* cfg, bool need_buffers) {
  if (!ro || !cfg) return fail(RSLX_ERR_INVALID_ARG, "rslx_ppo_update_recurrent: null rollout or cfg");
  RSLX_TRY(check_gru(ga, "rslx_ppo_update_recurrent actor memory", need_buffers));
  RSLX_TRY(check_gru(gc, "rslx_ppo_update_recurrent critic memory", need_buffers));
  RSLX_TRY(check_mlp(actor, "rslx_ppo_update_recurrent actor", need_buffers));
  RSLX_TRY(check_mlp(critic, "rslx_ppo_update_recurrent critic", need_buffers));
  if (!actor->has_log_std) return fail(RSLX_ERR_INVALID_ARG, "rslx_ppo_update_recurrent: actor needs log_std");
  if (ro->T < 1 || ro->N < 1 || (int64_t)ro->T * ro->N > (1 << 30))
    return fail(RSLX_ERR_SHAPE, "rslx_ppo_update_recurrent: T = %d, N = %d", ro->T, ro->N);
  if (ro->Da != ga->in_dim || ro->Dc != gc->in_dim || actor->dims[0] != ga->hidden || critic->dims[0] != gc->hidden ||
      ro->A != actor->dims[actor->n_layers] || critic->dims[critic->n_layers] != 1)
    return fail(RSLX_ERR_SHAPE, "rslx_ppo_update_recurrent: rollout, memory and network widths do not match");
  if (ga->cell != gc->cell) return fail(RSLX_ERR_UNSUPPORTED, "rslx_ppo_update_recurrent: the two memories use different cells");
  if (ro->A > 32) return fail(RSLX_ERR_UNSUPPORTED, "rslx_ppo_update_recurrent: action width %d > 32", ro->A);
  if (actor->n_layers + critic->n_layers + 4 > 16)
    return fail(RSLX_ERR_UNSUPPORTED, "rslx_ppo_update_recurrent: more than 12 MLP layers in total");
  if (cfg->epochs < 0 || cfg->minibatches < 1) return fail(RSLX_ERR_SHAPE, "rslx_ppo_update_recurrent: epochs / minibatches");
  if (ro->N % cfg->minibatches != 0)
    return fail(RSLX_ERR_SHAPE, "rslx_ppo_update_recurrent: N = %d is not a multiple of minibatches = %d", ro->N, cfg->minibatches);
  if (need_buffers && (!ro->obs_actor || !ro->obs_critic || !ro->actions || !ro->logp || !ro->values || !ro->mu ||
                       !ro->sigma || !ro->advantages || !ro->returns))
    return fail(RSLX_ERR_INVALID_ARG, "rslx_ppo_update_recurrent: null rollout buffer");
  return RSLX_OK;
}

// Weight-gradient problem of one side of a memory's gates: partials[l] = X^T dG over the row splits.
GemmProblem gate_dw_problem(const XView& x, int M, const float* dG, int H3, int32_t rows, const RnnBufs& b, int l) {
  GemmProblem p = blank_problem();
  set_x(p, x);
  p.B = dG; p.ldb = H3;
  p.C = b.partials + b.plan.part_off[l]; p.ldc = H3;
  p.M = M; p.N = H3; p.K = rows;
  p.n_split = b.plan.split[l];
  p.k_chunk = b.plan.chunk[l];
  p.split_stride = b.plan.pitch[l];
  p.bias_off = M * H3;
  p.dw_big = b.plan.big[l];
  p.a_vec = (M % 4 == 0 && p.lda % 4 == 0 && aligned16(p.A) && p.col_map == nullptr) ? 1 : 0;
  p.b_vec = (H3 % 4 == 0 && aligned16(dG)) ? 1 : 0;
  return p;
}

// Memories forward over one column-wise minibatch: the input-side gates of all T steps in one GEMM (rows gathered
// from the roll-out through ridx), then one fused step launch per time step for all `count` memories.
int32_t memories_forward(const rslx_memory* const* mem, RnnBufs* const* mb, int count, const float* const* obs,
                         const float* const* h0, const int32_t* envs, const int32_t* ridx, const uint8_t* dones, int T,
                         int nb, int N, hipStream_t s) {
  const int rows = T * nb;
  RowGatherArgs rg;
  memset(&rg, 0, sizeof rg);
  rg.n_jobs = count; rg.nb = nb; rg.idx = envs;
  for (int k = 0; k < count; ++k) rg.job[k] = RowGatherJob{h0[k], mb[k]->hin, nullptr, state_width(*mem[k])};
  RSLX_HIP(launch_row_gather(rg, s));
  GemmBatch bi;
  bi.count = count;
  for (int k = 0; k < count; ++k) {
    XView x;
    x.base = obs[k]; x.ld = mem[k]->in_dim; x.row_idx = ridx; x.src_rows = (int64_t)T * N;
    bi.p[k] = gate_problem(x, mem[k]->in_dim, mem[k]->params, mem[k]->params + gru_off_bih(*mem[k]), mb[k]->gi, rows,
                           gate_width(*mem[k]));
  }
  RSLX_HIP(launch_gemm(GEMM_FWD, bi, s));
  for (int t = 0; t < T; ++t) {
    StepFwdArgs sa;
    memset(&sa, 0, sizeof sa);
    sa.n_nets = count; sa.nb = nb; sa.cell = mem[0]->cell; sa.done = dones; sa.done_idx = ridx + (size_t)t * nb;
    for (int k = 0; k < count; ++k) {
      const rslx_memory& g = *mem[k];
      const size_t H = g.hidden, GH = gate_width(g), S = state_width(g), r0 = (size_t)t * nb;
      sa.net[k] = StepFwdNet{mb[k]->gi + r0 * GH, mb[k]->hin + r0 * S, mb[k]->hs + r0 * H, nullptr,
                             t + 1 < T ? mb[k]->hin + (r0 + nb) * S : nullptr, g.params + gru_off_whh(g),
                             g.params + gru_off_bhh(g), mb[k]->gh + r0 * GH, g.hidden, g.hidden};
    }
    RSLX_HIP(launch_step_fwd(sa, s));
  }
  return RSLX_OK;
}

// Back-propagation through time from mb[k]->dh (the gradient w.r.t. every step's new hidden state): one fused step
// launch per time step, last to first, then the weight gradients of both sides of the gates over all steps at once
// (split partials, to be summed by the caller's reduction).
int32_t memories_backward(const rslx_memory* const* mem, RnnBufs* const* mb, int count, const float* const* obs,
                          const int32_t* ridx, const uint8_t* dones, int T, int nb, int N, hipStream_t s) {
  const int rows = T * nb;
  for (int t = T - 1; t >= 0; --t) {
    StepBwdArgs sb;
    memset(&sb, 0, sizeof sb);
    sb.n_nets = count; sb.nb = nb; sb.cell = mem[0]->cell; sb.done = dones; sb.done_idx = ridx + (size_t)t * nb;
    for (int k = 0; k < count; ++k) {
      const rslx_memory& g = *mem[k];
      const size_t H = g.hidden, GH = gate_width(g), S = state_width(g), r0 = (size_t)t * nb;
      const bool last = t == T - 1;
      sb.net[k] = StepBwdNet{mb[k]->dh + r0 * H, last ? nullptr : mb[k]->dgh + (r0 + nb) * GH, mb[k]->direct,
                             g.params + gru_off_whh(g), mb[k]->gi + r0 * GH, mb[k]->gh + r0 * GH, mb[k]->hin + r0 * S,
                             mb[k]->dgi ? mb[k]->dgi + r0 * GH : nullptr, mb[k]->dgh + r0 * GH, g.hidden};
    }
    RSLX_HIP(launch_step_bwd(sb, s));
  }
  GemmBatch bwi, bwh;
  bwi.count = bwh.count = count;
  for (int k = 0; k < count; ++k) {
    const rslx_memory& g = *mem[k];
    XView x;
    x.base = obs[k]; x.ld = g.in_dim; x.row_idx = ridx; x.src_rows = (int64_t)T * N;
    // an LSTM's two sides of the gates share one gradient
    bwi.p[k] = gate_dw_problem(x, g.in_dim, mb[k]->dgi ? mb[k]->dgi : mb[k]->dgh, gate_width(g), rows, *mb[k], 0);
    bwh.p[k] = gate_dw_problem(plain_view(mb[k]->hin, state_width(g)), g.hidden, mb[k]->dgh, gate_width(g), rows, *mb[k], 1);
  }
  RSLX_HIP(launch_gemm(GEMM_DW, bwi, s));
  RSLX_HIP(launch_gemm(GEMM_DW, bwh, s));
  return RSLX_OK;
}

void reduce_add_memory(ReduceArgs& a, const rslx_memory& g, const RnnBufs& b) {
  for (int l = 0; l < 2; ++l) {
    ReduceSeg& sg = a.seg[a.n_seg++];
    sg.partials = b.partials + b.plan.part_off[l];
    sg.grads = g.grads + (l == 0 ? 0 : gru_off_whh(g));
    sg.size = b.plan.size[l];
    sg.pitch = b.plan.pitch[l];
    sg.split = b.plan.split[l];
    sg.block_start = a.blocks;
    a.blocks += (int)((b.plan.size[l] + REDUCE_BLOCK_FLOATS - 1) / REDUCE_BLOCK_FLOATS);
  }
}

}  // namespace

extern "C" {

size_t rslx_ppo_update_recurrent_workspace_bytes(const rslx_memory* gru_actor, const rslx_mlp* actor, const rslx_memory* gru_critic,
                                                 const rslx_mlp* critic, const rslx_rollout* ro, const rslx_ppo_cfg* cfg) {
  if (rnn_validate(gru_actor, actor, gru_critic, critic, ro, cfg, false) != RSLX_OK) return 0;
  Carver c(nullptr);
  RnnPlan p;
  rnn_plan(c, gru_actor, actor, gru_critic, critic, ro, cfg, p);
  return p.bytes;
}

}  // extern "C"

namespace {
// Shared body of rslx_ppo_update_recurrent and its device-counter variant.
int32_t ppo_update_recurrent_impl(rslx_memory* gru_actor, rslx_mlp* actor, rslx_memory* gru_critic, rslx_mlp* critic,
                                  const rslx_rollout* ro, const uint8_t* dones, const float* h0_actor, const float* h0_critic,
                                  const rslx_ppo_cfg* cfg, int64_t* adam_step, rslx_dev_counters* counters, float* stats,
                                  void* ws, size_t ws_bytes, void* stream) {
  RSLX_TRY(rnn_validate(gru_actor, actor, gru_critic, critic, ro, cfg, true));
  int64_t host_step = 0;
  if (counters) adam_step = &host_step;
  if (!dones || !h0_actor || !h0_critic || !adam_step || !stats)
    return fail(RSLX_ERR_INVALID_ARG, "rslx_ppo_update_recurrent: null dones, h0, adam_step or stats");
  if (!aligned16(h0_actor) || !aligned16(h0_critic)) return fail(RSLX_ERR_INVALID_ARG, "rslx_ppo_update_recurrent: h0 not 16-byte aligned");
  hipStream_t s = (hipStream_t)stream;
  Carver c(ws);
  RnnPlan p;
  rnn_plan(c, gru_actor, actor, gru_critic, critic, ro, cfg, p);
  if (!ws || ws_bytes < p.bytes) return fail(RSLX_ERR_WORKSPACE, "rslx_ppo_update_recurrent: workspace %zu < %zu bytes", ws_bytes, p.bytes);
  const int A = ro->A, L_a = actor->n_layers, L_c = critic->n_layers;
  const int T = p.T, nb = p.nb, rows = p.rows;
  const rslx_memory* mem[2] = {gru_actor, gru_critic};
  RnnBufs* mb[2] = {&p.ma, &p.mc};
  const float* obs[2] = {ro->obs_actor, ro->obs_critic};
  const float* h0[2] = {h0_actor, h0_critic};

  {
    std::vector<uint64_t> bases(cfg->epochs);
    for (int e = 0; e < cfg->epochs; ++e)
      bases[e] = mix64_host(mix64_host(mix64_host(cfg->seed) ^ cfg->call_index) ^ (uint64_t)(e + cfg->epoch_offset));
    RSLX_HIP(launch_permutations(bases.data(), cfg->epochs, p.N, p.perms, p.perm_ws, s, mix64_host(cfg->seed),
                                 counters ? &counters->call_index : nullptr, cfg->epoch_offset));
    RSLX_HIP(launch_column_rows(p.perms, cfg->epochs, cfg->minibatches, T, p.N, p.rows_all, s));
  }

  for (int e = 0; e < cfg->epochs; ++e) {
    for (int m = 0; m < cfg->minibatches; ++m) {
      const int32_t* envs = p.perms + (size_t)e * p.N + (size_t)m * nb;
      const int32_t* ridx = p.rows_all + ((size_t)e * cfg->minibatches + m) * rows;
      float* stats_row = stats + ((size_t)e * cfg->minibatches + m) * RSLX_NSTATS;

      RSLX_TRY(memories_forward(mem, mb, 2, obs, h0, envs, ridx, dones, T, nb, p.N, s));

      // ---- MLPs on the hidden states, loss head, MLP backward down to the hidden states ----
      XView xa = plain_view(p.ma.hs, gru_actor->hidden), xc = plain_view(p.mc.hs, gru_critic->hidden);
      NetJob fj[2] = {NetJob{actor, xa, rows, &p.actor.act}, NetJob{critic, xc, rows, &p.critic.act}};
      RSLX_TRY(forward_nets(fj, 2, s, p.fused_head));
      PpoLossArgs la;
      memset(&la, 0, sizeof la);
      la.mu = p.actor.act.out[L_a - 1];
      la.v = p.critic.act.out[L_c - 1];
      la.log_std = actor->params + weight_count(*actor);
      la.idx = ridx;
      la.actions = ro->actions; la.logp_old = ro->logp; la.adv = ro->advantages; la.returns = ro->returns;
      la.v_old = ro->values; la.mu_old = ro->mu; la.sigma_old = ro->sigma;
      la.mb = rows; la.rows = rows; la.A = A;
      la.clip = cfg->clip; la.value_coef = cfg->value_coef; la.entropy_coef = cfg->entropy_coef;
      la.clipped_value = cfg->use_clipped_value_loss;
      la.d_mu = p.actor.d_out; la.d_v = p.critic.d_out;
      la.partials = p.loss_partials;
      if (p.fused_head) {
        PpoHeadArgs ha;
        ha.loss = la;
        ha.h_a = p.actor.act.out[L_a - 2]; ha.h_c = p.critic.act.out[L_c - 2];
        ha.w_a = actor->params + layer_offset(*actor, L_a - 1); ha.w_c = critic->params + layer_offset(*critic, L_c - 1);
        ha.dz_a = p.actor.act.dz[L_a - 2]; ha.dz_c = p.critic.act.dz[L_c - 2];
        ha.Ha = actor->dims[L_a - 1]; ha.Hc = critic->dims[L_c - 1];
        ha.alpha_a = actor->elu_alpha; ha.alpha_c = critic->elu_alpha;
        RSLX_HIP(launch_ppo_head(ha, s));
      } else {
        RSLX_HIP(launch_ppo_loss(la, s));
      }
      BwdJob bj[2] = {BwdJob{actor, xa, rows, &p.actor.act, p.actor.d_out, p.actor.wt, p.actor.partials, &p.actor.plan, p.ma.dh},
                      BwdJob{critic, xc, rows, &p.critic.act, p.critic.d_out, p.critic.wt, p.critic.partials, &p.critic.plan, p.mc.dh}};
      RSLX_TRY(backward_nets(bj, 2, s, p.fused_head));

      RSLX_TRY(memories_backward(mem, mb, 2, obs, ridx, dones, T, nb, p.N, s));
      {   // one launch: every split sum and the loss head's sums
        ReduceArgs ra;
        memset(&ra, 0, sizeof ra);
        ra.sumsq_blocks = p.sumsq_all;
        reduce_add_net(ra, *actor, p.actor);
        reduce_add_net(ra, *critic, p.critic);
        reduce_add_memory(ra, *gru_actor, p.ma);
        reduce_add_memory(ra, *gru_critic, p.mc);
        ra.finish.partials = p.loss_partials; ra.finish.blocks = p.loss_blocks;
        ra.finish.rows = rows; ra.finish.mb = rows; ra.finish.A = A;
        ra.finish.log_std = la.log_std; ra.finish.entropy_coef = cfg->entropy_coef;
        ra.finish.d_log_std = actor->grads + weight_count(*actor);
        ra.finish.stats_row = stats_row;
        ra.finish.sumsq_slot = p.sumsq_all + (p.n_sumsq - 1);
        RSLX_HIP(launch_reduce_partials(ra, s));
      }
      const int64_t t1 = *adam_step + 1;
      AdamArgs aa;
      memset(&aa, 0, sizeof aa);
      aa.seg[0] = AdamSegment{actor->params, actor->grads, actor->adam_m, actor->adam_v, param_count(*actor)};
      aa.seg[1] = AdamSegment{critic->params, critic->grads, critic->adam_m, critic->adam_v, param_count(*critic)};
      aa.seg[2] = AdamSegment{gru_actor->params, gru_actor->grads, gru_actor->adam_m, gru_actor->adam_v, gru_count(*gru_actor)};
      aa.seg[3] = AdamSegment{gru_critic->params, gru_critic->grads, gru_critic->adam_m, gru_critic->adam_v, gru_count(*gru_critic)};
      aa.n_seg = 4;
      aa.sumsq_blocks = p.sumsq_all; aa.n_sumsq = p.n_sumsq;
      aa.max_grad_norm = cfg->max_grad_norm;
      aa.lr = cfg->lr; aa.beta1 = cfg->beta1; aa.beta2 = cfg->beta2; aa.eps = cfg->adam_eps;
      aa.bc1 = bias_correction(cfg->beta1, t1); aa.bc2 = bias_correction(cfg->beta2, t1);
      if (counters) { aa.step_dev = &counters->adam_step; aa.step_off = (int32_t)t1; }
      aa.grad_norm_out = stats_row + RSLX_STAT_GRAD_NORM;
      RSLX_HIP(launch_adam(aa, s));
      *adam_step = t1;
    }
  }
  if (counters) RSLX_HIP(advance_counters(counters, 0, 1, host_step, 0, s));
  return RSLX_OK;
}
}  // namespace

extern "C" {

int32_t rslx_ppo_update_recurrent(rslx_memory* mem_actor, rslx_mlp* actor, rslx_memory* mem_critic, rslx_mlp* critic,
                                  const rslx_rollout* ro, const uint8_t* dones, const float* h0_actor, const float* h0_critic,
                                  const rslx_ppo_cfg* cfg, int64_t* adam_step, float* stats, void* ws, size_t ws_bytes,
                                  void* stream) {
  if (!adam_step) return fail(RSLX_ERR_INVALID_ARG, "rslx_ppo_update_recurrent: null adam_step");
  return ppo_update_recurrent_impl(mem_actor, actor, mem_critic, critic, ro, dones, h0_actor, h0_critic, cfg, adam_step, nullptr,
                                   stats, ws, ws_bytes, stream);
}

int32_t rslx_ppo_update_recurrent_dc(rslx_memory* mem_actor, rslx_mlp* actor, rslx_memory* mem_critic, rslx_mlp* critic,
                                     const rslx_rollout* ro, const uint8_t* dones, const float* h0_actor,
                                     const float* h0_critic, const rslx_ppo_cfg* cfg, rslx_dev_counters* counters,
                                     float* stats, void* ws, size_t ws_bytes, void* stream) {
  if (!counters) return fail(RSLX_ERR_INVALID_ARG, "rslx_ppo_update_recurrent_dc: null counters");
  return ppo_update_recurrent_impl(mem_actor, actor, mem_critic, critic, ro, dones, h0_actor, h0_critic, cfg, nullptr, counters,
                                   stats, ws, ws_bytes, stream);
}

}  // extern "C"

// ---- a single memory: one step, and behaviour cloning of a recurrent student ---------------------------------
namespace {

struct RnnBcPlan {
  int32_t nb, rows;
  int32_t* perms = nullptr;      // [E, N]
  void* perm_ws = nullptr;
  int32_t* rows_all = nullptr;   // [E, M, T, nb]
  TrainBufs student;
  RnnBufs mem;
  double* sumsq_all = nullptr;
  int32_t n_sumsq = 0;
  double* mse_partials = nullptr;
  size_t bytes = 0;
};

void rnn_bc_plan(Carver& c, const rslx_memory* g, const rslx_mlp* student, int32_t T, int32_t N, const rslx_bc_cfg* cfg, RnnBcPlan& p) {
  p.nb = N / cfg->minibatches;
  p.rows = T * p.nb;
  p.perms = c.take<int32_t>((size_t)cfg->epochs * N);
  p.perm_ws = c.take<char>(perm_workspace_bytes(N));
  p.rows_all = c.take<int32_t>((size_t)cfg->epochs * T * N);
  carve_train(c, *student, p.rows, 1, p.student, true);
  carve_memory(c, *g, p.rows, p.nb, p.mem, 1);
  p.n_sumsq = p.student.n_sumsq + p.mem.plan.blocks;
  p.sumsq_all = c.take<double>((size_t)p.n_sumsq + 1);
  p.mse_partials = c.take<double>(mse_num_blocks((int64_t)p.rows * student->dims[student->n_layers]));
  p.bytes = c.off + 256;
}

int32_t rnn_bc_validate(const rslx_memory* g, const rslx_mlp* student, int32_t T, int32_t N, const rslx_bc_cfg* cfg, bool need_buffers) {
  if (!cfg) return fail(RSLX_ERR_INVALID_ARG, "rslx_bc_update_recurrent: null cfg");
  RSLX_TRY(check_gru(g, "rslx_bc_update_recurrent memory", need_buffers));
  RSLX_TRY(check_mlp(student, "rslx_bc_update_recurrent student", need_buffers));
  if (student->dims[0] != g->hidden) return fail(RSLX_ERR_SHAPE, "rslx_bc_update_recurrent: student input width != memory width");
  if (student->n_layers + 2 > 16) return fail(RSLX_ERR_UNSUPPORTED, "rslx_bc_update_recurrent: too many layers");
  if (T < 1 || N < 1 || (int64_t)T * N > (1 << 30)) return fail(RSLX_ERR_SHAPE, "rslx_bc_update_recurrent: T = %d, N = %d", T, N);
  if (cfg->minibatches < 1 || cfg->epochs < 0 || N % cfg->minibatches != 0)
    return fail(RSLX_ERR_SHAPE, "rslx_bc_update_recurrent: N = %d is not a multiple of minibatches = %d", N, cfg->minibatches);
  return RSLX_OK;
}

}  // namespace

extern "C" {

size_t rslx_memory_step_workspace_bytes(const rslx_memory* mem, int32_t N) {
  if (!mem || N <= 0) return 256;
  Carver c(nullptr);
  act_recurrent_carve(c, mem, nullptr, N, nullptr, nullptr);
  return c.off + 256;
}

int32_t rslx_memory_step(const rslx_memory* mem, const float* obs, int32_t N, float* state, const uint8_t* reset_or_null,
                         float* s0_out, float* h_dense_out, void* ws, size_t ws_bytes, void* stream) {
  if (N < 0) return fail(RSLX_ERR_SHAPE, "rslx_memory_step: N = %d", N);
  RSLX_TRY(check_gru(mem, "rslx_memory_step memory", false));
  if (!obs || !state) return fail(RSLX_ERR_INVALID_ARG, "rslx_memory_step: null input or state");
  if (!aligned16(state) || (s0_out && !aligned16(s0_out)) || (h_dense_out && !aligned16(h_dense_out)))
    return fail(RSLX_ERR_INVALID_ARG, "rslx_memory_step: state buffers not 16-byte aligned");
  if (N == 0) return RSLX_OK;
  if (!ws || ws_bytes < rslx_memory_step_workspace_bytes(mem, N)) return fail(RSLX_ERR_WORKSPACE, "rslx_memory_step: workspace too small");
  hipStream_t s = (hipStream_t)stream;
  Carver c(ws);
  StepBufs b;
  act_recurrent_carve(c, mem, nullptr, N, &b, nullptr);
  RowGatherArgs rg;
  memset(&rg, 0, sizeof rg);
  rg.n_jobs = 1; rg.nb = N; rg.reset = reset_or_null;
  rg.job[0] = RowGatherJob{state, b.hin, s0_out, state_width(*mem)};
  RSLX_HIP(launch_row_gather(rg, s));
  const rslx_memory* g[1] = {mem};
  const float* o[1] = {obs};
  const StepBufs bb[1] = {b};
  float* out[1] = {state};
  RSLX_TRY(gru_step(g, o, bb, out, 1, N, s));
  if (h_dense_out) RSLX_HIP(launch_copy_matrix(state, state_width(*mem), N, mem->hidden, h_dense_out, s));
  return RSLX_OK;
}

size_t rslx_bc_update_recurrent_workspace_bytes(const rslx_memory* gru, const rslx_mlp* student, int32_t T, int32_t N,
                                                const rslx_bc_cfg* cfg) {
  if (rnn_bc_validate(gru, student, T, N, cfg, false) != RSLX_OK) return 0;
  Carver c(nullptr);
  RnnBcPlan p;
  rnn_bc_plan(c, gru, student, T, N, cfg, p);
  return p.bytes;
}

int32_t rslx_bc_update_recurrent(rslx_memory* gru, rslx_mlp* student, const float* obs_student, const float* targets,
                                 const uint8_t* dones, const float* h0, int32_t T, int32_t N, const rslx_bc_cfg* cfg,
                                 int64_t* adam_step, float* stats, void* ws, size_t ws_bytes, void* stream) {
  RSLX_TRY(rnn_bc_validate(gru, student, T, N, cfg, true));
  if (!obs_student || !targets || !dones || !h0 || !adam_step || !stats)
    return fail(RSLX_ERR_INVALID_ARG, "rslx_bc_update_recurrent: null pointer");
  if (!aligned16(h0)) return fail(RSLX_ERR_INVALID_ARG, "rslx_bc_update_recurrent: h0 not 16-byte aligned");
  hipStream_t s = (hipStream_t)stream;
  Carver c(ws);
  RnnBcPlan p;
  rnn_bc_plan(c, gru, student, T, N, cfg, p);
  if (!ws || ws_bytes < p.bytes) return fail(RSLX_ERR_WORKSPACE, "rslx_bc_update_recurrent: workspace %zu < %zu bytes", ws_bytes, p.bytes);
  const int A = student->dims[student->n_layers], Ls = student->n_layers;
  const int nb = p.nb, rows = p.rows;
  const rslx_memory* mem[1] = {gru};
  RnnBufs* mb[1] = {&p.mem};
  const float* obs[1] = {obs_student};
  const float* h0s[1] = {h0};
  {
    std::vector<uint64_t> bases(cfg->epochs);
    for (int e = 0; e < cfg->epochs; ++e)
      bases[e] = mix64_host(mix64_host(mix64_host(cfg->seed) ^ cfg->call_index) ^ (uint64_t)(e + cfg->epoch_offset));
    RSLX_HIP(launch_permutations(bases.data(), cfg->epochs, N, p.perms, p.perm_ws, s));
    RSLX_HIP(launch_column_rows(p.perms, cfg->epochs, cfg->minibatches, T, N, p.rows_all, s));
  }
  const int nbm = mse_num_blocks((int64_t)rows * A);
  for (int e = 0; e < cfg->epochs; ++e) {
    for (int m = 0; m < cfg->minibatches; ++m) {
      const int32_t* envs = p.perms + (size_t)e * N + (size_t)m * nb;
      const int32_t* ridx = p.rows_all + ((size_t)e * cfg->minibatches + m) * rows;
      float* stats_row = stats + ((size_t)e * cfg->minibatches + m) * RSLX_NSTATS;
      RSLX_HIP(launch_fill(stats_row, RSLX_NSTATS, 0.f, s));
      RSLX_TRY(memories_forward(mem, mb, 1, obs, h0s, envs, ridx, dones, T, nb, N, s));
      XView xs = plain_view(p.mem.hs, gru->hidden);
      NetJob fj{student, xs, rows, &p.student.act};
      RSLX_TRY(forward_nets(&fj, 1, s));
      RSLX_HIP(launch_mse(p.student.act.out[Ls - 1], targets, ridx, rows, A, p.student.d_out, p.mse_partials, s));
      RSLX_HIP(launch_mse_finish(p.mse_partials, nbm, (int64_t)rows * A, stats_row, s));
      BwdJob bj{student, xs, rows, &p.student.act, p.student.d_out, p.student.wt, p.student.partials, &p.student.plan, p.mem.dh};
      RSLX_TRY(backward_nets(&bj, 1, s));
      RSLX_TRY(memories_backward(mem, mb, 1, obs, ridx, dones, T, nb, N, s));
      {
        ReduceArgs ra;
        memset(&ra, 0, sizeof ra);
        ra.sumsq_blocks = p.sumsq_all;
        reduce_add_net(ra, *student, p.student);
        reduce_add_memory(ra, *gru, p.mem);
        RSLX_HIP(launch_reduce_partials(ra, s));
      }
      const int64_t t1 = *adam_step + 1;
      AdamArgs aa;
      memset(&aa, 0, sizeof aa);
      aa.seg[0] = AdamSegment{student->params, student->grads, student->adam_m, student->adam_v, weight_count(*student)};
      aa.seg[1] = AdamSegment{gru->params, gru->grads, gru->adam_m, gru->adam_v, gru_count(*gru)};
      aa.n_seg = 2;
      aa.sumsq_blocks = p.sumsq_all; aa.n_sumsq = p.n_sumsq;
      aa.max_grad_norm = cfg->max_grad_norm;
      aa.lr = cfg->lr; aa.beta1 = cfg->beta1; aa.beta2 = cfg->beta2; aa.eps = cfg->adam_eps;
      aa.bc1 = bias_correction(cfg->beta1, t1); aa.bc2 = bias_correction(cfg->beta2, t1);
      aa.grad_norm_out = stats_row + RSLX_STAT_GRAD_NORM;
      RSLX_HIP(launch_adam(aa, s));
      *adam_step = t1;
    }
  }
  return RSLX_OK;
}

}  // extern "C"
