// Layer-fused MLP inference for gfx950: the latency-critical path of act() and of the RND reward, where the
// batch is a few thousand rows and per-layer launches would cost more than the arithmetic.
//
// One workgroup (8 wavefronts, two per SIMD) carries 32 batch rows of one network through every layer.
// Activations stay in LDS, contraction-major, in two ping-pong buffers; weights are not staged at all but
// streamed from L2 into the A operand of v_mfma_f32_16x16x4_f32.  A layer is cut into tasks of 64 output columns;
// when a layer has fewer than 8 such groups the contraction range of a group is split over 2, 4 or 8 wavefronts,
// so all 8 stay busy down to the narrow output layer.  Lane (m, kq) of a task owns columns col0 + 4 m .. + 3 at
// contraction index k + kq: one 16-byte load per step of four indices feeds eight matrix-core instructions (four
// column blocks x two 16-row halves of the batch tile), and the 16 lanes of a row read 256 contiguous bytes.
// Partial sums meet in LDS; all 512 lanes then add them up in a fixed order, apply bias and ELU and leave the
// result in the layout the next layer reads.  The last layer is also written to global memory; for the actor
// the Gaussian head (noise, action, log-density) runs in the same launch, one lane per (row, action component).
#include "kernels.h"
#include <algorithm>
#include <type_traits>

namespace rslx {

typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int FF_ROWS = 32;
constexpr int FF_THREADS = 512;
constexpr int FF_WAVES = FF_THREADS / 64;
constexpr int FF_GROUP = 64;                   // output columns per task
constexpr int FF_STEPS = 8;                    // contraction steps (of four indices) per weight chunk
constexpr int FF_CHUNK = 4 * FF_STEPS;         // weight values per lane held in flight per register buffer
constexpr int FF_MAX_DIM = 512;
constexpr int FF_BUF = FF_MAX_DIM * FF_ROWS;   // floats per LDS buffer: one activation matrix or all partial sums
constexpr float FF_LOG_2PI = 1.8378770664093453f;

__device__ __forceinline__ uint64_t ff_mix64(uint64_t x) {
  x += 0x9E3779B97F4A7C15ull;
  x = (x ^ (x >> 30)) * 0xBF58476D1CE4E5B9ull;
  x = (x ^ (x >> 27)) * 0x94D049BB133111EBull;
  return x ^ (x >> 31);
}

// LDS position of activation (k, row): the two 16-row halves are interleaved so that one 8-byte read gives a lane
// its B operand for both halves, and 64 lanes read or write 512 contiguous bytes.
__device__ __forceinline__ int ff_at(int k, int row) { return k * FF_ROWS + ((row & 15) << 1) + (row >> 4); }

// ELU with the hardware exponential: alpha (e^x - 1) for x <= 0.  The absolute error (about 1e-7) is what
// matters for a value that feeds the next layer's sums; the relative error near zero does not.
__device__ __forceinline__ float ff_elu(float x, float alpha) { return x > 0.f ? x : alpha * (__expf(x) - 1.0f); }

// Work of one wavefront in one layer: 64 columns from col0 and contraction steps [s_begin, s_end), a step being
// four contraction indices.  Every part spans a whole number of chunk pairs (16 steps); the last one of a group
// runs into zero activations (the LDS rows from K up to the next multiple of 64 are kept at zero), so no chunk
// needs a partial form.
struct FfTask {
  int col0, kpart, parts, s_begin, s_end;   // parts: how many wavefronts share a group's contraction
  bool active;
};

__host__ __device__ inline int ff_groups(int N) { return (N + FF_GROUP - 1) / FF_GROUP; }

// The split of a layer is planned on the host (it needs integer divisions): see FusedNet::split_*.
__device__ __forceinline__ FfTask ff_task(const FusedNet& net, int l, int wave) {
  const int K = net.dims[l], N = net.dims[l + 1];
  const int shift = net.split_shift[l], per = net.split_steps[l];
  FfTask t;
  const int group = wave >> shift;
  t.kpart = wave & ((1 << shift) - 1);
  t.col0 = group * FF_GROUP;
  t.parts = net.split_parts[l];
  const int steps = (K + 3) / 4;
  t.s_begin = min(steps, t.kpart * per);
  t.s_end = min(steps, t.s_begin + per);
  t.active = group < ff_groups(N) && t.kpart < t.parts;
  return t;
}

// Weight stream of a task.  Register 4 s + cb of the chunk at step s0 is W[4 (s0 + s) + kq][col0 + 4 m + cb].
// Rows and columns are clamped into the matrix: rows past K meet zero activations, columns past N only feed
// accumulator rows that are dropped later.
struct FfWeights {
  const float* W;
  int ldw, K, N, m, kq;
  bool vec;             // rows are 16-byte aligned and N % 4 == 0: one 16-byte load per step
  int col[4];           // clamped columns col0 + 4 m + cb

  __device__ __forceinline__ void setup(const float* W_, int K_, int N_, int col0, int m_, int kq_) {
    W = W_; ldw = N_; K = K_; N = N_; m = m_; kq = kq_;
    vec = (N_ & 3) == 0 && (reinterpret_cast<uintptr_t>(W_) & 15) == 0;
    const int c = vec ? min(col0 + 4 * m, N - 4) : col0 + 4 * m;
#pragma unroll
    for (int cb = 0; cb < 4; ++cb) col[cb] = min(c + cb, N - 1);
  }
  template <bool VEC>
  __device__ __forceinline__ void load(int s0, float (&dst)[FF_CHUNK]) const {
    if constexpr (VEC) {
#pragma unroll
      for (int s = 0; s < FF_STEPS; ++s) {
        const int row = min(4 * (s0 + s) + kq, K - 1);
        const float4 v = *reinterpret_cast<const float4*>(W + (long)row * ldw + col[0]);
        dst[4 * s + 0] = v.x; dst[4 * s + 1] = v.y; dst[4 * s + 2] = v.z; dst[4 * s + 3] = v.w;
      }
    } else {
#pragma unroll
      for (int s = 0; s < FF_STEPS; ++s) {
        const float* wr = W + (long)min(4 * (s0 + s) + kq, K - 1) * ldw;
#pragma unroll
        for (int cb = 0; cb < 4; ++cb) dst[4 * s + cb] = wr[col[cb]];
      }
    }
  }
};

// acc[cb][h] += W[:, col0 + 4 m + cb]^T (A operand) x activations of row half h (B operand) over the task's
// contraction range.  `w0` arrives holding the task's first chunk, fetched by the caller ahead of time.  Two
// register buffers alternate without copies so that the loads of chunk c + 1 stay in flight under the matrix-core
// instructions of chunk c.
template <bool VEC>
__device__ __forceinline__ void ff_contract(const FfWeights& wt, const FfTask& task, const float* actIn,
                                            float (&w0)[FF_CHUNK], f32x4 (&acc)[4][2]) {
  float w1[FF_CHUNK];
  const float* bp = actIn + (task.s_begin * 4 + wt.kq) * FF_ROWS + 2 * wt.m;
  const int nch = (task.s_end - task.s_begin + FF_STEPS - 1) / FF_STEPS;
  auto read_b = [&](int c, int s) { return *reinterpret_cast<const float2*>(bp + (c * FF_STEPS + s) * 4 * FF_ROWS); };
  // One chunk: its matrix-core instructions with, dealt out between them, the loads of the following chunk into
  // the other register buffer and the LDS reads of the activations two steps ahead; the first two steps' activations
  // arrive in `bh`, read under the previous chunk (the last chunk reads its own again).
  float2 bh[2] = {read_b(0, 0), read_b(0, 1)};
  auto chunk = [&](int c, int s_next, const float (&src)[FF_CHUNK], float (&dst)[FF_CHUNK]) {
    wt.load<VEC>(s_next, dst);
    float2 b[FF_STEPS + 2];
    b[0] = bh[0]; b[1] = bh[1];
    const int cn = min(c + 1, ((nch + 1) & ~1) - 1);   // chunks come in pairs; an odd count's twin meets zero activations
#pragma unroll
    for (int s = 2; s < FF_STEPS + 2; ++s) b[s] = s < FF_STEPS ? read_b(c, s) : read_b(cn, s - FF_STEPS);
#pragma unroll
    for (int s = 0; s < FF_STEPS; ++s)
#pragma unroll
      for (int cb = 0; cb < 4; ++cb) {
        acc[cb][0] = __builtin_amdgcn_mfma_f32_16x16x4f32(src[4 * s + cb], b[s].x, acc[cb][0], 0, 0, 0);
        acc[cb][1] = __builtin_amdgcn_mfma_f32_16x16x4f32(src[4 * s + cb], b[s].y, acc[cb][1], 0, 0, 0);
      }
    bh[0] = b[FF_STEPS]; bh[1] = b[FF_STEPS + 1];
    // masks: 0x008 matrix core, 0x100 LDS read, 0x020 global load.  Per pair of steps (16 matrix-core instructions):
    // the LDS read of the pair after next, then two groups of loads (one 16-byte load, or four 4-byte loads, per step)
#pragma unroll
    for (int pr = 0; pr < FF_STEPS / 2; ++pr) {
      __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);
      __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
      __builtin_amdgcn_sched_group_barrier(0x008, 4, 0);
      __builtin_amdgcn_sched_group_barrier(0x020, VEC ? 1 : 4, 0);
      __builtin_amdgcn_sched_group_barrier(0x008, 6, 0);
      __builtin_amdgcn_sched_group_barrier(0x020, VEC ? 1 : 4, 0);
      __builtin_amdgcn_sched_group_barrier(0x008, 4, 0);
    }
    __builtin_amdgcn_sched_barrier(0);
  };
  // A task spans an even number of chunks (see the split plan), and the fetch of the following chunk is issued
  // without a test (rows are clamped: a chunk past the range reads valid memory and is not used).  The loop body
  // is therefore free of branches, and the compiler's count of the loads in flight is exact: the matrix-core
  // instructions of one buffer wait for that buffer's loads only, not for the ones just issued into the other.
  for (int c = 0; c < nch; c += 2) {
    chunk(c, task.s_begin + (c + 1) * FF_STEPS, w0, w1);
    chunk(c + 1, task.s_begin + (c + 2) * FF_STEPS, w1, w0);
  }
}

// First weight chunk of a task.
__device__ __forceinline__ void ff_first_chunk(const float* __restrict__ W, int K, int N, const FfTask& task, int m,
                                               int kq, float (&w)[FF_CHUNK]) {
  if (!task.active) return;
  FfWeights wt;
  wt.setup(W, K, N, task.col0, m, kq);
  if (wt.vec) wt.load<true>(task.s_begin, w);
  else wt.load<false>(task.s_begin, w);
}

__global__ __launch_bounds__(FF_THREADS) void fused_forward_kernel(const FusedForwardArgs args) {
  extern __shared__ float lds[];
  const FusedNet& net = args.net[blockIdx.y];
  const int row0 = blockIdx.x * FF_ROWS;
  if (row0 >= args.n_rows) return;
  const int tid = threadIdx.x, lane = tid & 63;
  // the wavefront index decides which columns and contraction range a wavefront works on: held in a scalar
  // register, every test on it is a scalar branch
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int m = lane & 15, kq = lane >> 4;
  float* bufA = lds;
  float* bufB = lds + FF_BUF;

  // The first weight chunk of the first layer and the head's per-component inputs do not depend on any
  // activation: they are requested before the input rows, so their latency passes under the staging.
  float wpre[FF_CHUNK];
  FfTask task = ff_task(net, 0, wave);
  ff_first_chunk(net.params, net.dims[0], net.dims[1], task, m, kq, wpre);
  const int A = net.dims[net.n_layers];
  float head_ls = 0.f, head_eps = 0.f;
  if (net.head && tid < FF_ROWS * A) {
    long woff_ls = 0;
    for (int l = 0; l < net.n_layers; ++l) woff_ls += (long)net.dims[l] * net.dims[l + 1] + net.dims[l + 1];
    head_ls = net.params[woff_ls + (tid >> 5)];
    const long n = row0 + (tid & 31);
    if (!args.deterministic && args.eps != nullptr && n < args.n_rows) head_eps = args.eps[n * A + (tid >> 5)];
  }

  // ---- input rows -> LDS; rows from K0 to the next multiple of 64 are zero ----
  {
    const int K0 = net.dims[0];
    const int Kp = (K0 + 63) & ~63;
    if (net.col_map == nullptr && (net.ldx & 3) == 0 && (K0 & 3) == 0 && (reinterpret_cast<uintptr_t>(net.x) & 15) == 0) {
      // 16-byte loads, lanes along a row; every load is issued before the first one is used
      const int q4 = K0 >> 2;                           // float4 per row
      constexpr int PASS = FF_MAX_DIM * FF_ROWS / 4 / FF_THREADS;
      float4 v[PASS];
#pragma unroll
      for (int i = 0; i < PASS; ++i) {
        const int e = tid + FF_THREADS * i;
        if (FF_THREADS * i >= FF_ROWS * q4) break;
        const int r = e / q4, c4 = e - r * q4;
        v[i] = make_float4(0.f, 0.f, 0.f, 0.f);
        if (e < FF_ROWS * q4 && row0 + r < args.n_rows)
          v[i] = *reinterpret_cast<const float4*>(net.x + (long)(row0 + r) * net.ldx + 4 * c4);
      }
#pragma unroll
      for (int i = 0; i < PASS; ++i) {
        const int e = tid + FF_THREADS * i;
        if (FF_THREADS * i >= FF_ROWS * q4) break;
        if (e < FF_ROWS * q4) {
          const int r = e / q4, c4 = e - r * q4;
          bufA[ff_at(4 * c4 + 0, r)] = v[i].x; bufA[ff_at(4 * c4 + 1, r)] = v[i].y;
          bufA[ff_at(4 * c4 + 2, r)] = v[i].z; bufA[ff_at(4 * c4 + 3, r)] = v[i].w;
        }
      }
      for (int e = tid; e < (Kp - K0) * FF_ROWS; e += FF_THREADS) bufA[K0 * FF_ROWS + e] = 0.f;
    } else {
      const int r = tid & 31;
      const int row = row0 + r;
      for (int k = tid >> 5; k < Kp; k += FF_THREADS / 32) {
        float v = 0.f;
        if (row < args.n_rows && k < K0) {
          const int c = net.col_map ? net.col_map[k] : k;
          v = net.x[(long)row * net.ldx + c];
        }
        bufA[ff_at(k, r)] = v;
      }
    }
  }
  __syncthreads();

  float* in = bufA;
  float* out = bufB;
  long woff = 0;
  for (int l = 0; l < net.n_layers; ++l) {
    const int K = net.dims[l], N = net.dims[l + 1];
    const float* W = net.params + woff;
    const float* bias = W + (long)K * N;
    const bool last = (l + 1 == net.n_layers);
    float* gout = last ? net.out : nullptr;
    const int plane = ff_groups(N) * FF_GROUP * FF_ROWS;     // floats between the partial sums of two parts

    // bias values of the outputs this lane finishes, requested ahead of the contraction: with the contraction of
    // a group shared among wavefronts, the sums are finished by all lanes after an exchange through LDS (lane ->
    // outputs tid + 512 i); otherwise each wavefront finishes its own accumulators in registers
    const bool shared = task.parts > 1;
    constexpr int FIN = FF_MAX_DIM * (FF_ROWS / 2) / FF_THREADS;   // outputs (column, row pair) per lane at most
    float bfin[FIN];
    if (shared) {
#pragma unroll
      for (int i = 0; i < FIN; ++i) {
        if (FF_THREADS * i >= N * 16) break;
        const int e = tid + FF_THREADS * i;
        bfin[i] = bias[min(e >> 4, N - 1)];
      }
    } else if (task.active) {
#pragma unroll
      for (int cb = 0; cb < 4; ++cb)
#pragma unroll
        for (int r = 0; r < 4; ++r) bfin[4 * cb + r] = bias[min(task.col0 + 16 * kq + 4 * r + cb, N - 1)];
    }
    const FfTask next = last ? task : ff_task(net, l + 1, wave);
    if (task.active) {
      f32x4 acc[4][2];
#pragma unroll
      for (int cb = 0; cb < 4; ++cb)
#pragma unroll
        for (int h = 0; h < 2; ++h) acc[cb][h] = f32x4{0.f, 0.f, 0.f, 0.f};
      FfWeights wt;
      wt.setup(W, K, N, task.col0, m, kq);
      if (wt.vec) ff_contract<true>(wt, task, in, wpre, acc);
      else ff_contract<false>(wt, task, in, wpre, acc);
      // the next layer's first chunk is requested before this layer's sums are exchanged
      if (!last) ff_first_chunk(bias + N, N, net.dims[l + 2], next, m, kq, wpre);
      // accumulator register r of block cb: column col0 + 16 kq + 4 r + cb, batch rows m (half 0) and 16 + m
      float* part = out + task.kpart * plane;
#pragma unroll
      for (int cb = 0; cb < 4; ++cb)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const int c = task.col0 + 16 * kq + 4 * r + cb;
          float2 v = make_float2(acc[cb][0][r], acc[cb][1][r]);
          if (!shared) {
            v.x += bfin[4 * cb + r]; v.y += bfin[4 * cb + r];
            if (!last) {
              v.x = ff_elu(v.x, net.alpha);
              v.y = ff_elu(v.y, net.alpha);
            }
            if (gout != nullptr && c < N) {
              if (row0 + m < args.n_rows) gout[(long)(row0 + m) * N + c] = v.x;
              if (row0 + 16 + m < args.n_rows) gout[(long)(row0 + 16 + m) * N + c] = v.y;
            }
          }
          *reinterpret_cast<float2*>(part + c * FF_ROWS + 2 * m) = v;
        }
    } else if (!last) {
      ff_first_chunk(bias + N, N, net.dims[l + 2], next, m, kq, wpre);
    }
    __syncthreads();

    // ---- all lanes: sum the parts in order, bias, activation; result in place of part 0 ----
    // (reads first, then arithmetic, then writes: the LDS latency is paid once, not per output)
    const int parts = task.parts;
    if (shared) {
      float2 fv[FIN];
#pragma unroll
      for (int i = 0; i < FIN; ++i) {
        if (FF_THREADS * i >= N * 16) break;
        const int e = min(tid + FF_THREADS * i, N * 16 - 1);
        const float* p0 = out + (e >> 4) * FF_ROWS + 2 * (e & 15);
        float2 v = *reinterpret_cast<const float2*>(p0);
        for (int p = 1; p < parts; ++p) {
          const float2 u = *reinterpret_cast<const float2*>(p0 + p * plane);
          v.x += u.x; v.y += u.y;
        }
        fv[i] = v;
      }
#pragma unroll
      for (int i = 0; i < FIN; ++i) {
        if (FF_THREADS * i >= N * 16) break;
        const int e = tid + FF_THREADS * i;
        if (e < N * 16) {
          const int c = e >> 4, mp = e & 15;
          float2 v = fv[i];
          v.x += bfin[i]; v.y += bfin[i];
          if (!last) {
            v.x = ff_elu(v.x, net.alpha);
            v.y = ff_elu(v.y, net.alpha);
          }
          *reinterpret_cast<float2*>(out + c * FF_ROWS + 2 * mp) = v;
          if (gout != nullptr) {
            if (row0 + mp < args.n_rows) gout[(long)(row0 + mp) * N + c] = v.x;
            if (row0 + 16 + mp < args.n_rows) gout[(long)(row0 + 16 + mp) * N + c] = v.y;
          }
        }
      }
    }
    // rows from N to the next multiple of 64 are the zero padding the next layer's last chunks run into
    for (int e = tid; e < (((N + 63) & ~63) - N) * 16; e += FF_THREADS)
      *reinterpret_cast<float2*>(out + (N + (e >> 4)) * FF_ROWS + 2 * (e & 15)) = make_float2(0.f, 0.f);
    __syncthreads();
    task = next;
    float* tmp = in; in = out; out = tmp;
    woff += (long)K * N + N;
  }

  // ---- Gaussian head (actor only): `in` now holds mu; one lane per (row, action component) ----
  if (net.head) {
    const float* log_std = net.params + woff;
    float* z2 = out;                       // [A][32]; the other activation buffer is free by now
    float* lsb = z2 + FF_ROWS * A;         // [A] log_std, for the per-row sums
    for (int e = tid; e < FF_ROWS * A; e += FF_THREADS) {
      const int r = e & 31, jj = e >> 5;
      const long n = row0 + r;
      const float ls = e == tid ? head_ls : log_std[jj];
      if (r == 0) lsb[jj] = ls;
      float zz = 0.f;
      if (n < args.n_rows) {
        const long o = n * A + jj;
        const float sg = expf(ls);
        const float mu = in[ff_at(jj, r)];
        float eps;
        if (args.deterministic) {
          eps = 0.f;
        } else if (args.eps != nullptr) {
          eps = e == tid ? head_eps : args.eps[o];
        } else {
          const uint64_t nb = args.step_dev != nullptr ? ff_mix64(args.noise_pre ^ (uint64_t)*args.step_dev) : args.noise_base;
          const uint64_t h = ff_mix64(nb ^ (uint64_t)o);
          const float u1 = (float)((uint32_t)(h >> 40) + 1u) * 5.9604644775390625e-08f;
          const float u2 = (float)((uint32_t)(h >> 8) & 0xFFFFFFu) * 5.9604644775390625e-08f;
          eps = sqrtf(-2.0f * logf(u1)) * cospif(2.0f * u2);
        }
        const float act = mu + sg * eps;
        const float z = (act - mu) / sg;
        zz = z * z;
        args.actions[o] = act;
        args.sigma[o] = sg;
      }
      z2[jj * FF_ROWS + r] = zz;
    }
    __syncthreads();
    if (tid < FF_ROWS && row0 + tid < args.n_rows) {
      float zz = 0.f, sum_ls = 0.f;
      for (int jj = 0; jj < A; ++jj) {
        zz += z2[jj * FF_ROWS + tid];
        sum_ls += lsb[jj];
      }
      args.logp[row0 + tid] = -0.5f * zz - sum_ls - 0.5f * (float)A * FF_LOG_2PI;
    }
  }
}

bool fused_forward_supported(const FusedForwardArgs& a) {
  if (a.max_dim > FF_MAX_DIM || a.n_nets < 1 || a.n_nets > 2) return false;
  return true;
}

hipError_t launch_fused_forward(const FusedForwardArgs& a, hipStream_t stream) {
  if (a.n_rows <= 0) return hipSuccess;
  const size_t lds_bytes = (size_t)2 * FF_BUF * sizeof(float);
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(fused_forward_kernel),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, 2 * FF_BUF * (int)sizeof(float));
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  double flops = 0.0;
  for (int i = 0; i < a.n_nets; ++i)
    for (int l = 0; l < a.net[i].n_layers; ++l) flops += 2.0 * a.n_rows * a.net[i].dims[l] * (double)a.net[i].dims[l + 1];
  TraceScope ts(stream, "fused_forward", flops, 0.0);
  FusedForwardArgs b = a;
  for (int i = 0; i < b.n_nets; ++i)
    for (int l = 0; l < b.net[i].n_layers; ++l) {
      const int g = ff_groups(b.net[i].dims[l + 1]);
      const int shift = g > FF_WAVES / 2 ? 0 : g > FF_WAVES / 4 ? 1 : g > FF_WAVES / 8 ? 2 : 3;
      const int steps = (b.net[i].dims[l] + 3) / 4;
      const int per = (((steps + (1 << shift) - 1) >> shift) + 2 * FF_STEPS - 1) / (2 * FF_STEPS) * (2 * FF_STEPS);
      b.net[i].split_shift[l] = shift;
      b.net[i].split_steps[l] = per;
      b.net[i].split_parts[l] = std::max(1, (steps + per - 1) / per);
    }
  dim3 grid((b.n_rows + FF_ROWS - 1) / FF_ROWS, b.n_nets);
  hipLaunchKernelGGL(fused_forward_kernel, grid, dim3(FF_THREADS), lds_bytes, stream, b);
  return hipGetLastError();
}

}  // namespace rslx
