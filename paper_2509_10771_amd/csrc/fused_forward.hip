// Layer-fused MLP inference for gfx950: the latency-critical path of act() and of the RND reward, where the
// batch is a few thousand rows and per-layer launches would cost more than the arithmetic.
//
// One workgroup (4 wavefronts) carries 32 batch rows of one network through every layer.  Activations stay in
// LDS, contraction-major ([k][32 rows], two ping-pong buffers); weights are not staged at all: each wavefront
// owns a contiguous range of output columns and streams its slice of W straight from L2 into the A operand of
// v_mfma_f32_32x32x2_f32 (lanes 0..31 read 32 consecutive columns = one 128-byte line per contraction step),
// prefetching one 16-step chunk ahead.  Feeding W as the A operand makes the accumulator layout
// [output column][batch row], so the epilogue's LDS stores (bias, ELU) are conflict-free without padding.
// The last layer is written to global memory; for the actor the Gaussian head (noise, action, log-density)
// runs in the same launch.
#include "kernels.h"

namespace rslx {

typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int FF_ROWS = 32;
constexpr int FF_PREFETCH = 32; // weight values per lane held in flight per buffer (chunk = 32 / NT steps)
constexpr float FF_LOG_2PI = 1.8378770664093453f;

__device__ __forceinline__ uint64_t ff_mix64(uint64_t x) {
  x += 0x9E3779B97F4A7C15ull;
  x = (x ^ (x >> 30)) * 0xBF58476D1CE4E5B9ull;
  x = (x ^ (x >> 27)) * 0x94D049BB133111EBull;
  return x ^ (x >> 31);
}

// acc[t] += W[:, col0 + 32 t .. +31]^T (as A operand) x actIn (as B operand), t < NT.
// Weight loads are unconditional (indices clamped into the matrix): columns past N only feed accumulator rows
// the epilogue drops, and contraction steps past K are cancelled by a zero activation operand.  Two register
// buffers alternate without copies so that the loads of chunk c + 1 stay in flight under the MFMAs of chunk c.
template <int NT>
__device__ __forceinline__ void ff_contract(const float* __restrict__ W, int ldw, int K, int N, int col0,
                                            const float* actIn, int g, int j, f32x16 (&acc)[NT]) {
  constexpr int KC = FF_PREFETCH / NT;      // 2-wide contraction steps per chunk
  float w0[KC][NT], w1[KC][NT];
  int colc[NT];
#pragma unroll
  for (int t = 0; t < NT; ++t) colc[t] = min(col0 + 32 * t + j, N - 1);
  auto load_w = [&](int kbase, float (&dst)[KC][NT]) {
#pragma unroll
    for (int s = 0; s < KC; ++s) {
      const long ka = min(kbase + 2 * s + g, K - 1);
#pragma unroll
      for (int t = 0; t < NT; ++t) dst[s][t] = W[ka * ldw + colc[t]];
    }
  };
  auto compute = [&](int kbase, const float (&src)[KC][NT]) {
    float a[KC];
#pragma unroll
    for (int s = 0; s < KC; ++s) {
      const int ka = kbase + 2 * s + g;
      a[s] = actIn[min(ka, K - 1) * FF_ROWS + j];
      if (ka >= K) a[s] = 0.f;
    }
#pragma unroll
    for (int s = 0; s < KC; ++s)
#pragma unroll
      for (int t = 0; t < NT; ++t) acc[t] = __builtin_amdgcn_mfma_f32_32x32x2f32(src[s][t], a[s], acc[t], 0, 0, 0);
  };
  constexpr int STEP = 2 * KC;
  load_w(0, w0);
  for (int kb = 0; kb < K; kb += 2 * STEP) {
    load_w(kb + STEP, w1);
    compute(kb, w0);
    if (kb + STEP < K) {
      load_w(kb + 2 * STEP, w0);
      compute(kb + STEP, w1);
    }
  }
}

// bias + activation, store to LDS ([n][row]) and, for the last layer, to global ([row][n]).
template <int NT>
__device__ __forceinline__ void ff_epilogue(const f32x16 (&acc)[NT], const float* __restrict__ bias, int N, int col0,
                                            bool elu, float alpha, float* actOut, float* __restrict__ gout, int ldo,
                                            int row0, int n_rows, int g, int j) {
  float bv[NT][16];      // all bias loads are issued before any of them is consumed
#pragma unroll
  for (int t = 0; t < NT; ++t)
#pragma unroll
    for (int r = 0; r < 16; ++r) bv[t][r] = bias[min(col0 + 32 * t + 8 * (r / 4) + 4 * g + (r % 4), N - 1)];
#pragma unroll
  for (int t = 0; t < NT; ++t) {
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int n = col0 + 32 * t + 8 * (r / 4) + 4 * g + (r % 4);
      float v = acc[t][r] + bv[t][r];
      if (elu) v = v > 0.f ? v : alpha * expm1f(v);
      if (n < N) {
        actOut[n * FF_ROWS + j] = v;
        if (gout != nullptr && row0 + j < n_rows) gout[(long)(row0 + j) * ldo + n] = v;
      }
    }
  }
}

__global__ __launch_bounds__(256) void fused_forward_kernel(const FusedForwardArgs args) {
  extern __shared__ float lds[];
  const FusedNet& net = args.net[blockIdx.y];
  const int row0 = blockIdx.x * FF_ROWS;
  if (row0 >= args.n_rows) return;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int g = lane >> 5, j = lane & 31;
  float* bufA = lds;
  float* bufB = lds + args.max_dim * FF_ROWS;

  // ---- input rows -> LDS [k][row] (lanes run over rows so the LDS stores are conflict-free) ----
  {
    const int K0 = net.dims[0];
    const int row = row0 + (tid & 31);
    for (int k = tid >> 5; k < K0; k += 8) {
      float v = 0.f;
      if (row < args.n_rows) {
        const int c = net.col_map ? net.col_map[k] : k;
        v = net.x[(long)row * net.ldx + c];
      }
      bufA[k * FF_ROWS + (tid & 31)] = v;
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
    const int tiles = (N + 31) / 32;
    const int tpw = (tiles + 3) / 4;                   // column tiles per wavefront, contiguous
    const int t_begin = wave * tpw;
    const int t_end = min(tiles, t_begin + tpw);
    for (int t0 = t_begin; t0 < t_end; t0 += 4) {
      const int nt = min(4, t_end - t0);
      const int col0 = t0 * 32;
      if (nt == 4) {
        f32x16 acc[4];
#pragma unroll
        for (int t = 0; t < 4; ++t)
#pragma unroll
          for (int r = 0; r < 16; ++r) acc[t][r] = 0.f;
        ff_contract<4>(W, N, K, N, col0, in, g, j, acc);
        ff_epilogue<4>(acc, bias, N, col0, !last, net.alpha, out, gout, N, row0, args.n_rows, g, j);
      } else if (nt >= 2) {
        f32x16 acc[2];
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
          for (int r = 0; r < 16; ++r) acc[t][r] = 0.f;
        ff_contract<2>(W, N, K, N, col0, in, g, j, acc);
        ff_epilogue<2>(acc, bias, N, col0, !last, net.alpha, out, gout, N, row0, args.n_rows, g, j);
        if (nt == 3) {
          f32x16 acc1[1];
#pragma unroll
          for (int r = 0; r < 16; ++r) acc1[0][r] = 0.f;
          ff_contract<1>(W, N, K, N, col0 + 64, in, g, j, acc1);
          ff_epilogue<1>(acc1, bias, N, col0 + 64, !last, net.alpha, out, gout, N, row0, args.n_rows, g, j);
        }
      } else {
        f32x16 acc1[1];
#pragma unroll
        for (int r = 0; r < 16; ++r) acc1[0][r] = 0.f;
        ff_contract<1>(W, N, K, N, col0, in, g, j, acc1);
        ff_epilogue<1>(acc1, bias, N, col0, !last, net.alpha, out, gout, N, row0, args.n_rows, g, j);
      }
    }
    __syncthreads();
    float* tmp = in; in = out; out = tmp;
    woff += (long)K * N + N;
  }

  // ---- Gaussian head (actor only): `in` now holds mu as [A][row] ----
  if (net.head && tid < FF_ROWS && row0 + tid < args.n_rows) {
    const int A = net.dims[net.n_layers];
    const long n = row0 + tid;
    const float* log_std = net.params + woff;
    float zz = 0.f, sum_ls = 0.f;
    for (int jj = 0; jj < A; ++jj) {
      const long o = n * A + jj;
      const float ls = log_std[jj];
      const float sg = expf(ls);
      const float mu = in[jj * FF_ROWS + tid];
      float e;
      if (args.deterministic) {
        e = 0.f;
      } else if (args.eps != nullptr) {
        e = args.eps[o];
      } else {
        const uint64_t h = ff_mix64(args.noise_base ^ (uint64_t)o);
        const float u1 = (float)((uint32_t)(h >> 40) + 1u) * 5.9604644775390625e-08f;
        const float u2 = (float)((uint32_t)(h >> 8) & 0xFFFFFFu) * 5.9604644775390625e-08f;
        e = sqrtf(-2.0f * logf(u1)) * cospif(2.0f * u2);
      }
      const float act = mu + sg * e;
      const float z = (act - mu) / sg;
      zz += z * z;
      sum_ls += ls;
      args.actions[o] = act;
      args.sigma[o] = sg;
    }
    args.logp[n] = -0.5f * zz - sum_ls - 0.5f * (float)A * FF_LOG_2PI;
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
  hipLaunchKernelGGL(fused_forward_kernel, grid, dim3(256), lds_bytes, stream, a);
  return hipGetLastError();
}

}  // namespace rslx
