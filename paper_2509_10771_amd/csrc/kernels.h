// Internal interface between the host-side entry points and the HIP kernels of librslx.
// Not part of the public ABI (that is include/rslx.h).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace rslx {

// ---------------------------------------------------------------------------------------------
// Optional launch trace: while enabled, every kernel launch site brackets its launch with a pair of HIP
// events on the launch stream and tags it with its algorithmic flops / bytes.  Disabled by default
// (then these calls do nothing).
// ---------------------------------------------------------------------------------------------
// trace_open returns the index of the record it opened, or -1 when none was opened (trace off, record limit
// reached, event creation failed); trace_close records the end event of exactly that record.
int trace_open(hipStream_t stream, const char* kernel, double flops, double bytes);
void trace_close(hipStream_t stream, int record);
struct TraceScope {
  hipStream_t s;
  int record;
  TraceScope(hipStream_t stream, const char* kernel, double flops, double bytes)
      : s(stream), record(trace_open(stream, kernel, flops, bytes)) {}
  ~TraceScope() { trace_close(s, record); }
};

// ---------------------------------------------------------------------------------------------
// Dense fp32 contraction on the matrix cores, three operand arrangements of one kernel:
//   GEMM_FWD  C[r, n]   = act( sum_k X(r, k) W[k, n] + bias[n] )          (layer forward)
//   GEMM_DX   C[r, kin] = ( sum_n dZ[r, n] Wt[n, kin] ) * ELU'(H[r, kin])  (input gradient; Wt = W^T,
//             transposed once per step by launch_transpose)
//   GEMM_DW   C_s[kin, n] = sum_{r in split s} X(r, kin) dZ[r, n]          (weight gradient, split
//             over rows; the block row holding kin = 0 also emits the column sums of dZ = db)
// X(r, c) is a view of a row-major matrix with an optional row gather and column map:
//   src_row = row_idx ? row_idx[r mod idx_mod] : r mod idx_mod
//   X(r, c) = (r >= map_from && col_map) ? col_sign[c] * A[src_row, col_map[c]] : A[src_row, c]
// which covers minibatch gathering, mirrored copies and feature subsets without materialising them.
// ---------------------------------------------------------------------------------------------
enum GemmMode : int { GEMM_FWD = 0, GEMM_DX = 1, GEMM_DW = 2 };

struct GemmProblem {
  const float* A;           // FWD/DW: X storage; DX: dZ
  const float* B;           // FWD: W [K_in, N_out] row-major; DX: W^T [N_out, K_in] row-major; DW: dZ
  float* C;                 // FWD/DX: output; DW: base of split partial 0
  const float* aux;         // FWD: bias[N] or null; DX: H at C's coordinates (ldc) or null
  const int32_t* row_idx;   // optional row gather for X (device)
  const int32_t* col_map;   // optional column map for X (device)
  const float* col_sign;    // optional column sign for X (device, with col_map)
  int32_t idx_mod;          // rows r >= idx_mod wrap to r - idx_mod (INT32_MAX = no wrap)
  int32_t wrap_add;         // added to the source row of a wrapped row (a second copy of the matrix further down)
  int32_t map_from;         // rows >= map_from use col_map / col_sign
  int32_t M, N, K;          // GEMM extents (K is the contraction length)
  int32_t lda, ldb, ldc;
  int32_t elu;              // FWD: 1 = ELU epilogue, 0 = linear
  float alpha;              // ELU parameter
  int32_t k_chunk;          // DW: contraction rows per split
  int32_t n_split;          // DW: number of splits (grid.y)
  int64_t split_stride;     // DW: floats between consecutive partial buffers
  int32_t bias_off;         // DW: offset of the db partial inside a partial buffer, -1 = none
  int32_t dw_big;           // DW: 1 = 128x128 tiles were planned for this layer, 0 = 64x128
  int32_t a_vec, b_vec;     // 1 = operand may be fetched with 16-byte loads
  int64_t a_src_rows;       // rows of the matrix that row_idx gathers from (0 = unknown)
  int32_t a_cols;           // DW: readable width of X's rows when it exceeds M (zero-padded storage), 0 = M
};

struct GemmBatch {
  GemmProblem p[2];
  int32_t count;
};

hipError_t launch_gemm(GemmMode mode, const GemmBatch& batch, hipStream_t stream);
// Weight gradient (bw) and input gradient (bx) of one layer; one launch when both fit the paired kernel.
// narrow_dw: optional further weight gradient whose operands are ready as well (the output layer's, a few columns
// wide); it rides in the same launch when it can, else it is launched on its own first.
hipError_t launch_gemm_dw_dx(const GemmBatch& bw, const GemmBatch& bx, hipStream_t stream, const GemmBatch* narrow_dw = nullptr);
// Out-of-place transposes of up to 16 row-major matrices in one launch: dst[c, r] = src[r, c].
struct TransposeJob { const float* src; float* dst; int32_t rows, cols; };
struct TransposeBatch { TransposeJob job[16]; int32_t count; };
hipError_t launch_transpose(const TransposeBatch& b, hipStream_t stream);
// Number of output tiles the weight-gradient kernel uses for an [M, N] layer (big = 128x128 tiles allowed).
int gemm_dw_tiles(int32_t M, int32_t N, bool big);

// ---------------------------------------------------------------------------------------------
// Layer-fused inference of up to two networks over the same batch rows (fused_forward.hip).
// ---------------------------------------------------------------------------------------------
struct FusedNet {
  const float* params;      // flat layout; a `head` network's log_std follows its last bias
  const float* x;           // input matrix [n_rows, ldx] row-major
  const int32_t* col_map;   // optional: input column k reads x[:, col_map[k]]
  float* out;               // last layer's output [n_rows, dims[n_layers]]
  int32_t ldx;
  int32_t n_layers;
  int32_t dims[9];
  float alpha;
  int32_t head;             // 1: run the Gaussian head on this network's output
  // per-layer work split, filled in by launch_fused_forward: a layer's 64-column groups are shared by
  // 1 << split_shift wavefronts each, `split_steps` contraction steps apiece, of which `split_parts` have work
  int32_t split_shift[8], split_steps[8], split_parts[8];
};
struct FusedForwardArgs {
  FusedNet net[2];
  int32_t n_nets, n_rows, max_dim, deterministic;
  const float* eps;         // optional caller noise [n_rows, A]
  uint64_t noise_base;
  const int64_t* step_dev;  // optional device counter: noise_base = mix64(noise_pre ^ *step_dev)
  uint64_t noise_pre;
  float* actions; float* logp; float* sigma;
};
bool fused_forward_supported(const FusedForwardArgs& a);
hipError_t launch_fused_forward(const FusedForwardArgs& a, hipStream_t stream);

// ---------------------------------------------------------------------------------------------
// Streaming / reduction kernels (elementwise.hip)
// ---------------------------------------------------------------------------------------------
int gae_num_blocks(int32_t N);
hipError_t launch_gae(const float* rewards, const float* values, const float* last_values,
                      const uint8_t* dones, const uint8_t* timeouts, int32_t T, int32_t N, float gamma,
                      float lam, int32_t normalize, float* adv, float* ret, double* partials,
                      hipStream_t stream);

// Permutation by sorting 64-bit hash keys (bucket scatter + in-bucket ranking).
size_t perm_workspace_bytes(int32_t B);
// perm_out [n_perm, B]; base_keys (host) holds one hashed stream key per permutation.
// call_index_dev != null: base_keys[e] is ignored and the key base of permutation e is
// mix64(mix64(seed_mixed ^ *call_index_dev) ^ (epoch0 + e)), formed in the kernels.
hipError_t launch_permutations(const uint64_t* base_keys, int32_t n_perm, int32_t B, int32_t* perm_out, void* ws,
                               hipStream_t stream, uint64_t seed_mixed = 0, const uint64_t* call_index_dev = nullptr,
                               int32_t epoch0 = 0);

// Sum the split partials of one network's gradient, layer by layer, into the flat gradient buffer and emit
// per-block sums of squares.  Layer l owns `split[l]` partial buffers of `size[l]` floats each, `pitch[l]` floats
// apart from `part_off[l]` on; its gradient starts at `grad_off[l]`.
// Sums of the PPO loss partials: stats row, log_std gradient and its squared norm (see launch_reduce_partials).
struct LossFinishArgs {
  const double* partials;   // [blocks][5 + A]; blocks == 0: nothing to finish
  int32_t blocks, rows, mb, A;
  const float* log_std;
  float entropy_coef;
  float* d_log_std;
  float* stats_row;
  double* sumsq_slot;
};
// One segment = the split-buffers of one layer of one network.
struct ReduceSeg {
  const float* partials;    // first split buffer of the layer
  float* grads;             // the layer's slice of the flat gradient
  int64_t size;             // floats per split (W then b)
  int64_t pitch;            // floats between consecutive split buffers (multiple of 4)
  int32_t split;
  int32_t block_start;      // first workgroup of the segment
};
struct ReduceArgs {
  ReduceSeg seg[16];
  int32_t n_seg;
  int32_t blocks;           // workgroups over all segments; block b writes sumsq_blocks[b]
  double* sumsq_blocks;
  LossFinishArgs finish;    // handled by one extra workgroup of the same launch
};
constexpr int REDUCE_BLOCK_FLOATS = 256;
hipError_t launch_reduce_partials(const ReduceArgs& a, hipStream_t stream);
// Per-block sums of squares of an existing gradient buffer (reduce_num_blocks(n) entries).
int reduce_num_blocks(int64_t n);
hipError_t launch_sumsq(const float* g, int64_t n, double* sumsq_blocks, hipStream_t stream);

struct AdamSegment {
  float* params; const float* grads; float* m; float* v;
  int64_t n;
  // Optional: every updated weight of layers >= wt_from is also written to its place in `wt`, the flat buffer of
  // transposed weight matrices the input-gradient contraction reads (W_l^T at the layer's parameter offset), so
  // that no transposition launch is needed before the next optimiser step.  dims: the MLP's layer widths.
  float* wt;
  int32_t n_layers, wt_from;
  int32_t dims[9];
};
struct AdamArgs {
  AdamSegment seg[4];
  int32_t n_seg;
  const double* sumsq_blocks;  // per-block sums of squares covering every clipped tensor
  int32_t n_sumsq;
  float max_grad_norm;         // <= 0: no clipping
  float lr, beta1, beta2, eps;
  float bc1, bc2;              // 1 - beta1^t, 1 - beta2^t (used when step_dev is null)
  const int64_t* step_dev;     // optional device counter: t = *step_dev + step_off, corrections formed in the kernel
  int32_t step_off;
  float* grad_norm_out;        // optional device scalar (stats column)
};
// Lists longer than this are folded by an extra single-workgroup launch into the slot sumsq_blocks[n_sumsq],
// which the caller must have reserved.
constexpr int ADAM_MAX_INLINE_SUMSQ = 4096;
hipError_t launch_adam(const AdamArgs& a, hipStream_t stream);

// Gaussian head of act(): noise, action, log-density.
// step_dev != null: the noise base is mix64(noise_pre ^ *step_dev) instead of noise_base.
hipError_t launch_act_head(const float* mu_in, const float* log_std, const float* eps, uint64_t noise_base,
                           int32_t N, int32_t A, int32_t deterministic, float* actions, float* logp, float* mu_out,
                           float* sigma_out, hipStream_t stream, const int64_t* step_dev = nullptr, uint64_t noise_pre = 0);
// counters[i] += delta[i] for i < n <= 4 (one small launch); for callers whose counters live in device memory.
hipError_t launch_counter_add(int64_t* counters, const int64_t* delta, int32_t n, hipStream_t stream);
hipError_t launch_copy_column(const float* src, int32_t n, float* dst, hipStream_t stream);

// PPO loss head: per-row loss terms, d loss / d mu and d loss / d V, block partial sums.
struct PpoLossArgs {
  const float* mu;        // [rows, A] new means (rows = mb or 2*mb)
  const float* v;         // [rows]
  const float* log_std;   // [A]
  const int32_t* idx;     // [mb] rollout rows of this minibatch
  const float* actions; const float* logp_old; const float* adv; const float* returns; const float* v_old;
  const float* mu_old; const float* sigma_old;
  const int32_t* perm_act; const float* sign_act;  // mirror map of actions (null without symmetry)
  int32_t mb, rows, A;
  float clip, value_coef, entropy_coef, mirror_coef;
  int32_t clipped_value;
  float* d_mu;            // [rows, A]
  float* d_v;             // [rows]
  double* partials;       // [blocks, PPO_NPART]
};
constexpr int PPO_NPART_FIXED = 5;  // surrogate, value, kl, clip count, mirror ; then A entries of dlog_std
int ppo_loss_num_blocks(int32_t mb);
hipError_t launch_ppo_loss(const PpoLossArgs& a, hipStream_t stream);
// Fused output layers + loss head + input gradient of the output layers (needs the last hidden widths to be
// 32, 64, 128 or 256; ppo_head_supported tells).  loss.mu / loss.v are not read; loss.partials needs
// ppo_head_num_blocks entries.
struct PpoHeadArgs {
  PpoLossArgs loss;
  const float* h_a; const float* h_c;   // last hidden activations [rows, Ha], [rows, Hc]
  const float* w_a; const float* w_c;   // output layers: W [H, out] row-major followed by the bias
  float* dz_a; float* dz_c;             // gradients w.r.t. the last hidden pre-activations
  int32_t Ha, Hc;
  float alpha_a, alpha_c;
};
bool ppo_head_supported(int32_t Ha, int32_t Hc, int32_t A);
int ppo_head_num_blocks(int32_t mb, bool sym);
hipError_t launch_ppo_head(const PpoHeadArgs& h, hipStream_t stream);

// Mean-squared-error head: d = 2 (y - target) / (rows * width), block partial sums of squared error.
int mse_num_blocks(int64_t n);
hipError_t launch_mse(const float* y, const float* target, const int32_t* target_idx, int32_t rows, int32_t width,
                      float* d_y, double* partials, hipStream_t stream);
hipError_t launch_mse_finish(const double* partials, int32_t blocks, int64_t count, float* stat_out, hipStream_t stream);

hipError_t launch_sym_augment(const float* in, int32_t B, int32_t D, const int32_t* perm, const float* sign,
                              float* out, hipStream_t stream);
// Network input staged for the 16-byte operand paths: out [B (+ B), Dp] holds in [B, D] (row stride ld) with the
// columns D..Dp-1 zero and, when perm is given, below it the mirrored rows sign[j] * in[r, perm[j]].
hipError_t launch_stage_input(const float* in, int32_t ld, int32_t B, int32_t D, int32_t Dp, const int32_t* perm,
                              const float* sign, float* out, hipStream_t stream);

// RND reward: row sums of squared differences, batch moments, running-stat merge, normalisation.
int rnd_num_blocks(int32_t N);
hipError_t launch_rnd_reward(const float* yp, const float* yt, int32_t N, int32_t K, float* running, float weight,
                             int32_t update_stats, float* r_int, float* rewards, double* partials, hipStream_t stream);

hipError_t launch_fill(float* p, int64_t n, float value, hipStream_t stream);

// ---------------------------------------------------------------------------------------------
// Recurrent memory cells (recurrent.hip), one time step per launch for up to two networks (the actor's and the
// critic's memory, same cell type); H % 4 == 0.  G gates, packed state rows of width S:
//   GRU  (G = 3: r, z, n; S = H, state h):   gi = x W_ih + b_ih (from the GEMM kernel),  gh = h W_hh + b_hh
//        r = sigmoid(gi_r + gh_r), z = sigmoid(gi_z + gh_z), n = tanh(gi_n + r gh_n), h' = (1 - z) n + z h
//   LSTM (G = 4: i, f, g, o; S = 2H, state [h | c]):   a = gi + h W_hh + b_hh
//        i, f, o = sigmoid(a_i, a_f, a_o), g = tanh(a_g), c' = f c + i g, h' = o tanh(c')
// Forward: h W_hh is formed tile by tile on the matrix cores, the gates are the epilogue.  pre_out (when set;
// the backward pass reads it) receives gh for the GRU and the whole pre-activation a for the LSTM.
// ---------------------------------------------------------------------------------------------
enum CellKind : int { CELL_GRU = 0, CELL_LSTM = 1 };
struct StepFwdNet {
  const float* gi;        // [nb, G H] this step's rows
  const float* sin;       // [nb, S] packed state the step starts from
  float* h_out;           // new hidden state, row stride ld_out
  float* c_out;           // LSTM: new cell state, row stride ld_out; null = not stored
  float* sin_next;        // [nb, S] or null: new state * (1 - done), what the next step starts from
  const float* w_hh;      // [H, G H] row-major
  const float* b_hh;      // [G H]
  float* pre_out;         // [nb, G H] or null
  int32_t H, ld_out;
};
struct StepFwdArgs {
  StepFwdNet net[2];
  int32_t n_nets, nb, cell;
  const uint8_t* done;      // episode-end flags (null = none); row i reads done[done_idx ? done_idx[i] : i]
  const int32_t* done_idx;
};
hipError_t launch_step_fwd(const StepFwdArgs& a, hipStream_t stream);

// One step of back-propagation through time.  back = dg_next W_hh^T (what step t + 1 sends to its input hidden
// state through the hidden-side contraction) is formed tile by tile and never stored.  With keep = 1 - done:
//   GRU:  dh = dh_ext + keep (back + carry);  writes dgi = [dr_pre, dz_pre, dn_pre], dg = [dr_pre, dz_pre, dn_pre r],
//         carry <- dh z  (the direct path into the input state)
//   LSTM: dh = dh_ext + keep back, dc' = keep carry;  writes dg = d loss / d a (the same for both sides of the
//         gates; dgi is not used), carry <- (dc' + dh o (1 - tanh^2 c')) f
struct StepBwdNet {
  const float* dh_ext;    // [nb, H] gradient arriving from the layers above
  const float* dg_next;   // [nb, G H] this network's dg of step t + 1, null on the last step
  float* carry;           // [nb, H] in / out (not read on the last step)
  const float* w_hh;      // [H, G H] row-major: back[row, j] = sum_k dg_next[row, k] W_hh[j, k]
  const float* gi;        // [nb, G H] (GRU only)
  const float* pre;       // [nb, G H] what the forward step stored in pre_out
  const float* sin;       // [nb, S]
  float* dgi;             // [nb, G H] (GRU only)
  float* dg;              // [nb, G H]
  int32_t H;
};
struct StepBwdArgs {
  StepBwdNet net[2];
  int32_t n_nets, nb, cell;
  const uint8_t* done;      // flags of THIS step (they gate what step t + 1 sends back); null = none
  const int32_t* done_idx;
};
hipError_t launch_step_bwd(const StepBwdArgs& a, hipStream_t stream);

// dst[i, :] = src[idx ? idx[i] : i, :] * (reset && reset[i] ? 0 : 1) for up to two [*, H] matrices; a second
// copy of the result goes to dst2 when it is not null.
struct RowGatherJob { const float* src; float* dst; float* dst2; int32_t H; };
struct RowGatherArgs {
  RowGatherJob job[2];
  int32_t n_jobs, nb;
  const int32_t* idx;
  const uint8_t* reset;
};
hipError_t launch_row_gather(const RowGatherArgs& a, hipStream_t stream);

// dst[r, 0 .. cols) = src[r * ld_src + 0 .. cols) for r < rows (cols % 4 == 0): the hidden part of packed states as a
// dense matrix.
hipError_t launch_copy_matrix(const float* src, int32_t ld_src, int32_t rows, int32_t cols, float* dst, hipStream_t stream);

// rows_out[((e * M + m) * T + t) * nb + i] = t * N + perm[e * N + m * nb + i]: the roll-out rows of every
// column-wise minibatch, step-major.
hipError_t launch_column_rows(const int32_t* perm, int32_t E, int32_t M, int32_t T, int32_t N, int32_t* rows_out,
                              hipStream_t stream);

}  // namespace rslx
