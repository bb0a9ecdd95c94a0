// Layer-fused MLP inference for gfx950: the latency-critical path of act() and of the RND reward, where the
// batch is a few thousand rows and per-layer launches would cost more than the arithmetic.
//
// One workgroup (8 wavefronts, two per SIMD) carries 32 batch rows of one network through every layer.
// Activations stay in LDS, contraction-major, in two ping-pong buffers; weights are not staged at all: each
// wavefront owns a contiguous range of output columns and streams its slice of W straight from L2 into the A
// operand of v_mfma_f32_16x16x4_f32 (16 consecutive columns of four contraction rows per load), one chunk of 32
// values per lane ahead of the matrix-core instructions that consume it.  A weight value fetched once feeds both
// 16-row halves of the batch tile.  Feeding W as the A operand makes the accumulator layout [output column]
// [batch row], so the epilogue (bias, ELU) writes LDS in the layout the next layer reads.
// The last layer is written to global memory; for the actor the Gaussian head (noise, action, log-density)
// runs in the same launch, one lane per (row, action component).
#include "kernels.h"
#include <type_traits>

namespace rslx {

typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int FF_ROWS = 32;
constexpr int FF_THREADS = 512;
constexpr int FF_WAVES = FF_THREADS / 64;
constexpr int FF_CHUNK = 32;    // weight values per lane held in flight per register buffer
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

// expm1 for the ELU branch (x <= 0): series near zero, where exp(x) - 1 cancels; the hardware exponential elsewhere.
__device__ __forceinline__ float ff_expm1_neg(float x) {
  const float p = x * (1.0f + x * (0.5f + x * (0.16666667f + x * (0.041666668f + x * 0.0083333338f))));
  const float e = __expf(x) - 1.0f;
  return x > -0.125f ? p : e;
}

// The contraction of a column group runs in steps of four indices.  Weight chunk c holds steps [c S, (c + 1) S),
// S = FF_CHUNK / CB: register s * CB + cb of lane (m, kq) is W[4 (c S + s) + kq][col0 + 16 cb + m].  A chunk is
// fetched as the matrix pointer plus a 32-bit offset: a fixed lane part and a uniform part per step.  Steps past
// the last whole one (K / 4) are skipped under a uniform test; the K % 4 indices that remain form one ragged step with clamped rows.  Columns are clamped into the matrix: columns past N only feed
// accumulator rows the epilogue drops.
template <int CB>
struct FfWeights {
  static constexpr int S = FF_CHUNK / CB;
  const float* W;
  int ldw, K, N, col0, m, kq, steps;
  unsigned lo[CB];      // byte offset of W[kq][col0 + 16 cb + m]

  __device__ __forceinline__ void setup(const float* W_, int K_, int N_, int col0_, int m_, int kq_) {
    W = W_; ldw = N_; K = K_; N = N_; col0 = col0_; m = m_; kq = kq_; steps = K_ / 4;
#pragma unroll
    for (int cb = 0; cb < CB; ++cb) lo[cb] = (unsigned)(kq * ldw + min(col0 + 16 * cb + m, N - 1)) * 4u;
  }
  __device__ __forceinline__ int chunks() const { return (steps + S - 1) / S; }
  __device__ __forceinline__ bool whole(int c) const { return (c + 1) * S <= steps; }

  // Step (c, s): uniform byte offset of its four rows, made opaque so that every address is formed next to its
  // load (one add) instead of living in a register of its own across the whole contraction.
  __device__ __forceinline__ unsigned step_off(int c, int s) const {
    return __builtin_amdgcn_readfirstlane((unsigned)((c * S + s) * 4 * ldw) * 4u);
  }

  __device__ __forceinline__ void load(int c, float (&dst)[FF_CHUNK]) const {
    if (c * S >= steps) return;                 // past the end: never consumed
    const char* wb = reinterpret_cast<const char*>(W);
    if (whole(c)) {
#pragma unroll
      for (int s = 0; s < S; ++s) {
        const unsigned so = step_off(c, s);
#pragma unroll
        for (int cb = 0; cb < CB; ++cb) dst[s * CB + cb] = *reinterpret_cast<const float*>(wb + (lo[cb] + so));
      }
    } else {
#pragma unroll
      for (int s = 0; s < S; ++s) {
        if (c * S + s < steps) {
          const unsigned so = step_off(c, s);
#pragma unroll
          for (int cb = 0; cb < CB; ++cb) dst[s * CB + cb] = *reinterpret_cast<const float*>(wb + (lo[cb] + so));
        }
      }
    }
  }
};

// acc[cb][h] += W[:, col0 + 16 cb .. + 15]^T (A operand) x activations of row half h (B operand), cb < CB.
// Lane (m = lane % 16, kq = lane / 16) supplies column col0 + 16 cb + m and batch rows m, 16 + m at contraction
// index k + kq.  `w0` arrives holding chunk 0, fetched by the caller ahead of time.  Two register buffers
// alternate without copies so that the loads of chunk c + 1 stay in flight under the matrix-core instructions of
// chunk c.
template <int CB>
__device__ __forceinline__ void ff_contract(const FfWeights<CB>& wt, const float* actIn, float (&w0)[FF_CHUNK],
                                            f32x4 (&acc)[CB][2]) {
  constexpr int S = FF_CHUNK / CB;      // 4-wide contraction steps per chunk
  constexpr int SB = S < 8 ? S : 8;     // steps whose activation operands are read from LDS together
  const int m = wt.m, kq = wt.kq;
  float w1[FF_CHUNK];
  auto mfma_step = [&](const float* wv, float2 b) {
#pragma unroll
    for (int cb = 0; cb < CB; ++cb) {
      acc[cb][0] = __builtin_amdgcn_mfma_f32_16x16x4f32(wv[cb], b.x, acc[cb][0], 0, 0, 0);
      acc[cb][1] = __builtin_amdgcn_mfma_f32_16x16x4f32(wv[cb], b.y, acc[cb][1], 0, 0, 0);
    }
  };
  auto compute = [&](int c, const float (&src)[FF_CHUNK]) {
    const float* bp = actIn + (c * (4 * S) + kq) * FF_ROWS + 2 * m;
    if (wt.whole(c)) {
#pragma unroll
      for (int s0 = 0; s0 < S; s0 += SB) {
        float2 b[SB];
#pragma unroll
        for (int s = 0; s < SB; ++s) b[s] = *reinterpret_cast<const float2*>(bp + 4 * (s0 + s) * FF_ROWS);
#pragma unroll
        for (int s = 0; s < SB; ++s) mfma_step(&src[(s0 + s) * CB], b[s]);
      }
    } else {
#pragma unroll
      for (int s = 0; s < S; ++s)
        if (c * S + s < wt.steps) mfma_step(&src[s * CB], *reinterpret_cast<const float2*>(bp + 4 * s * FF_ROWS));
    }
  };
  const int nch = wt.chunks();
  for (int c = 0; c < nch; c += 2) {
    wt.load(c + 1, w1);
    compute(c, w0);
    if (c + 1 < nch) {
      wt.load(c + 2, w0);
      compute(c + 1, w1);
    }
  }
  if (wt.K & 3) {     // ragged last step: rows clamped, activations past K read as zero
    const int ka = 4 * wt.steps + kq;
    float wv[CB];
#pragma unroll
    for (int cb = 0; cb < CB; ++cb)
      wv[cb] = wt.W[(long)min(ka, wt.K - 1) * wt.ldw + min(wt.col0 + 16 * cb + m, wt.N - 1)];
    float2 b = *reinterpret_cast<const float2*>(actIn + min(ka, wt.K - 1) * FF_ROWS + 2 * m);
    if (ka >= wt.K) b = make_float2(0.f, 0.f);
    mfma_step(wv, b);
  }
}

// bias + activation, store to LDS and, for the last layer, to global ([row][n]).  Accumulator register r of lane
// (m, kq) holds output column col0 + 16 cb + 4 kq + r for batch rows m (half 0) and 16 + m (half 1).
template <int CB>
__device__ __forceinline__ void ff_epilogue(const f32x4 (&acc)[CB][2], const float (&bv)[CB][4], int N,
                                            int col0, bool elu, float alpha, float* actOut, float* __restrict__ gout,
                                            int ldo, int row0, int n_rows, int m, int kq) {
#pragma unroll
  for (int cb = 0; cb < CB; ++cb) {
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int n = col0 + 16 * cb + 4 * kq + r;
      float v0 = acc[cb][0][r] + bv[cb][r], v1 = acc[cb][1][r] + bv[cb][r];
      if (elu) {
        v0 = v0 > 0.f ? v0 : alpha * ff_expm1_neg(v0);
        v1 = v1 > 0.f ? v1 : alpha * ff_expm1_neg(v1);
      }
      if (n < N) {
        *reinterpret_cast<float2*>(actOut + n * FF_ROWS + 2 * m) = make_float2(v0, v1);
        if (gout != nullptr) {
          if (row0 + m < n_rows) gout[(long)(row0 + m) * ldo + n] = v0;
          if (row0 + 16 + m < n_rows) gout[(long)(row0 + 16 + m) * ldo + n] = v1;
        }
      }
    }
  }
}

// Column-tile group of one wavefront in a layer: `count` (4, 2 or 1) 16-column tiles from column col0; 0 = none.
struct FfGroup {
  int col0, count;
};

__device__ __forceinline__ FfGroup ff_group(int N, int wave, int t_done) {
  const int tiles = (N + 15) / 16;
  const int tpw = (tiles + FF_WAVES - 1) / FF_WAVES;   // 16-column tiles per wavefront, contiguous
  const int t0 = wave * tpw + t_done;
  const int left = min(tiles, (wave + 1) * tpw) - t0;
  FfGroup gr;
  gr.col0 = t0 * 16;
  gr.count = left >= 4 ? 4 : left >= 2 ? 2 : left >= 1 ? 1 : 0;
  return gr;
}

// First weight chunk of a group, in the register order ff_contract<count> expects.
__device__ __forceinline__ void ff_first_chunk(const float* __restrict__ W, int K, int N, FfGroup gr, int m, int kq,
                                               float (&w)[FF_CHUNK]) {
  if (gr.count == 4) {
    FfWeights<4> wt; wt.setup(W, K, N, gr.col0, m, kq); wt.load(0, w);
  } else if (gr.count == 2) {
    FfWeights<2> wt; wt.setup(W, K, N, gr.col0, m, kq); wt.load(0, w);
  } else if (gr.count == 1) {
    FfWeights<1> wt; wt.setup(W, K, N, gr.col0, m, kq); wt.load(0, w);
  }
}

template <int CB>
__device__ __forceinline__ void ff_tile(const float* __restrict__ W, const float* __restrict__ bias, int K, int N,
                                        int col0, const float* in, float (&w0)[FF_CHUNK], f32x4 (&acc)[CB][2],
                                        float (&bv)[CB][4], int m, int kq) {
  // the bias values travel with the weight stream, long before the epilogue needs them
#pragma unroll
  for (int cb = 0; cb < CB; ++cb)
#pragma unroll
    for (int r = 0; r < 4; ++r) bv[cb][r] = bias[min(col0 + 16 * cb + 4 * kq + r, N - 1)];
#pragma unroll
  for (int cb = 0; cb < CB; ++cb)
#pragma unroll
    for (int h = 0; h < 2; ++h) acc[cb][h] = f32x4{0.f, 0.f, 0.f, 0.f};
  FfWeights<CB> wt;
  wt.setup(W, K, N, col0, m, kq);
  ff_contract<CB>(wt, in, w0, acc);
}

__global__ __launch_bounds__(FF_THREADS) void fused_forward_kernel(const FusedForwardArgs args) {
  extern __shared__ float lds[];
  const FusedNet& net = args.net[blockIdx.y];
  const int row0 = blockIdx.x * FF_ROWS;
  if (row0 >= args.n_rows) return;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int m = lane & 15, kq = lane >> 4;
  float* bufA = lds;
  float* bufB = lds + args.max_dim * FF_ROWS;

  // The first weight chunk of the first layer and the head's per-component inputs do not depend on any
  // activation: they are requested before the input rows, so their latency passes under the staging.
  float wpre[FF_CHUNK];
  FfGroup gr = ff_group(net.dims[1], wave, 0);
  ff_first_chunk(net.params, net.dims[0], net.dims[1], gr, m, kq, wpre);
  const int A = net.dims[net.n_layers];
  float head_ls = 0.f, head_eps = 0.f;
  if (net.head && tid < FF_ROWS * A) {
    long woff_ls = 0;
    for (int l = 0; l < net.n_layers; ++l) woff_ls += (long)net.dims[l] * net.dims[l + 1] + net.dims[l + 1];
    head_ls = net.params[woff_ls + (tid >> 5)];
    const long n = row0 + (tid & 31);
    if (!args.deterministic && args.eps != nullptr && n < args.n_rows) head_eps = args.eps[n * A + (tid >> 5)];
  }

  // ---- input rows -> LDS (lanes run over rows) ----
  {
    const int K0 = net.dims[0];
    const int r = tid & 31;
    const int row = row0 + r;
    for (int k = tid >> 5; k < K0; k += FF_THREADS / 32) {
      float v = 0.f;
      if (row < args.n_rows) {
        const int c = net.col_map ? net.col_map[k] : k;
        v = net.x[(long)row * net.ldx + c];
      }
      bufA[ff_at(k, r)] = v;
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
    // weights of the group that follows the current one: the next group of this layer, else the first group of
    // the next layer; its first chunk is requested before the current group's epilogue
    int t_done = 0;
    while (gr.count > 0) {
      t_done += gr.count;
      FfGroup nx = ff_group(N, wave, t_done);
      const float* Wn = W;
      int Kn = K, Nn = N;
      if (nx.count == 0 && !last) {
        Wn = bias + N; Kn = N; Nn = net.dims[l + 2];
        nx = ff_group(Nn, wave, 0);
      }
      auto run = [&](auto cb_tag) {
        constexpr int CB = decltype(cb_tag)::value;
        f32x4 acc[CB][2];
        float bv[CB][4];
        ff_tile<CB>(W, bias, K, N, gr.col0, in, wpre, acc, bv, m, kq);
        ff_first_chunk(Wn, Kn, Nn, nx, m, kq, wpre);
        ff_epilogue<CB>(acc, bv, N, gr.col0, !last, net.alpha, out, gout, N, row0, args.n_rows, m, kq);
      };
      if (gr.count == 4) run(std::integral_constant<int, 4>{});
      else if (gr.count == 2) run(std::integral_constant<int, 2>{});
      else run(std::integral_constant<int, 1>{});
      if (Wn != W) break;          // nx belongs to the next layer
      gr = nx;
    }
    if (gr.count == 0 && !last) {  // this wavefront had no columns in this layer: fetch for the next one now
      gr = ff_group(net.dims[l + 2], wave, 0);
      ff_first_chunk(bias + N, N, net.dims[l + 2], gr, m, kq, wpre);
    } else if (!last) {
      gr = ff_group(net.dims[l + 2], wave, 0);
    }
    __syncthreads();
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
          const uint64_t h = ff_mix64(args.noise_base ^ (uint64_t)o);
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
  if (a.max_dim > 512 || a.n_nets < 1 || a.n_nets > 2) return false;
  return true;
}

hipError_t launch_fused_forward(const FusedForwardArgs& a, hipStream_t stream) {
  if (a.n_rows <= 0) return hipSuccess;
  const size_t lds_bytes = (size_t)2 * a.max_dim * FF_ROWS * sizeof(float);
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(fused_forward_kernel),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, 2 * 512 * FF_ROWS * (int)sizeof(float));
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  double flops = 0.0;
  for (int i = 0; i < a.n_nets; ++i)
    for (int l = 0; l < a.net[i].n_layers; ++l) flops += 2.0 * a.n_rows * a.net[i].dims[l] * (double)a.net[i].dims[l + 1];
  TraceScope ts(stream, "fused_forward", flops, 0.0);
  dim3 grid((a.n_rows + FF_ROWS - 1) / FF_ROWS, a.n_nets);
  hipLaunchKernelGGL(fused_forward_kernel, grid, dim3(FF_THREADS), lds_bytes, stream, a);
  return hipGetLastError();
}

}  // namespace rslx
