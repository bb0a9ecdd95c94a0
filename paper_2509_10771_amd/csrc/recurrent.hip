// Element-wise stages of the gated recurrent unit (forward gates, back-propagation through time) and the
// index plumbing of column-wise minibatches.  The contractions around them run in the GEMM kernel.
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

__global__ __launch_bounds__(256) void gru_gates_fwd_kernel(const GruFwdArgs a) {
  const GruFwdNet& n = a.net[blockIdx.y];
  const int H = n.H, q = H >> 2;
  const long e = (long)blockIdx.x * 256 + threadIdx.x;
  if (e >= (long)a.nb * q) return;
  const int i = (int)(e / q), j = (int)(e - (long)i * q) * 4;
  const float* gi = n.gi + (long)i * 3 * H + j;
  const float* gh = n.gh + (long)i * 3 * H + j;
  const f4 gir = ld4(gi), giz = ld4(gi + H), gin = ld4(gi + 2 * H);
  const f4 ghr = ld4(gh), ghz = ld4(gh + H), ghn = ld4(gh + 2 * H);
  const f4 hin = ld4(n.hin + (long)i * H + j);
  float keep = 1.0f;
  if (n.hin_next != nullptr && a.done != nullptr) keep = a.done[a.done_idx ? a.done_idx[i] : i] ? 0.0f : 1.0f;
  f4 h;
#pragma unroll
  for (int c = 0; c < 4; ++c) {
    const float r = sigmoidf_(gir[c] + ghr[c]);
    const float z = sigmoidf_(giz[c] + ghz[c]);
    const float nn = tanhf_(gin[c] + r * ghn[c]);
    h[c] = (1.0f - z) * nn + z * hin[c];
  }
  st4(n.h_out + (long)i * H + j, h);
  if (n.hin_next != nullptr) st4(n.hin_next + (long)i * H + j, h * keep);
}

__global__ __launch_bounds__(256) void gru_gates_bwd_kernel(const GruBwdArgs a) {
  const GruBwdNet& n = a.net[blockIdx.y];
  const int H = n.H, q = H >> 2;
  const long e = (long)blockIdx.x * 256 + threadIdx.x;
  if (e >= (long)a.nb * q) return;
  const int i = (int)(e / q), j = (int)(e - (long)i * q) * 4;
  const long o = (long)i * H + j, o3 = (long)i * 3 * H + j;
  f4 dh = ld4(n.dh_ext + o);
  if (n.back != nullptr) {
    float keep = 1.0f;
    if (a.done != nullptr) keep = a.done[a.done_idx ? a.done_idx[i] : i] ? 0.0f : 1.0f;
    dh += (ld4(n.back + o) + ld4(n.direct_in + o)) * keep;
  }
  const f4 gir = ld4(n.gi + o3), giz = ld4(n.gi + o3 + H), gin = ld4(n.gi + o3 + 2 * H);
  const f4 ghr = ld4(n.gh + o3), ghz = ld4(n.gh + o3 + H), ghn = ld4(n.gh + o3 + 2 * H);
  const f4 hin = ld4(n.hin + o);
  f4 dr_pre, dz_pre, dn_pre, dn_r, direct;
#pragma unroll
  for (int c = 0; c < 4; ++c) {
    const float r = sigmoidf_(gir[c] + ghr[c]);
    const float z = sigmoidf_(giz[c] + ghz[c]);
    const float nn = tanhf_(gin[c] + r * ghn[c]);
    const float dn = dh[c] * (1.0f - z);
    const float dz = dh[c] * (hin[c] - nn);
    direct[c] = dh[c] * z;
    dn_pre[c] = dn * (1.0f - nn * nn);
    dr_pre[c] = dn_pre[c] * ghn[c] * r * (1.0f - r);
    dz_pre[c] = dz * z * (1.0f - z);
    dn_r[c] = dn_pre[c] * r;
  }
  st4(n.dgi + o3, dr_pre); st4(n.dgi + o3 + H, dz_pre); st4(n.dgi + o3 + 2 * H, dn_pre);
  st4(n.dgh + o3, dr_pre); st4(n.dgh + o3 + H, dz_pre); st4(n.dgh + o3 + 2 * H, dn_r);
  st4(n.direct_out + o, direct);
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

hipError_t launch_gru_gates_fwd(const GruFwdArgs& a, hipStream_t stream) {
  long work = 0;
  for (int k = 0; k < a.n_nets; ++k) { const long w = (long)a.nb * (a.net[k].H >> 2); work = w > work ? w : work; }
  if (work == 0) return hipSuccess;
  double bytes = 0.0;
  for (int k = 0; k < a.n_nets; ++k) bytes += 4.0 * a.nb * a.net[k].H * (6 + 1 + 1 + (a.net[k].hin_next ? 1 : 0));
  TraceScope ts(stream, "gru_gates_fwd", 0.0, bytes);
  hipLaunchKernelGGL(gru_gates_fwd_kernel, dim3((unsigned)((work + 255) / 256), a.n_nets), dim3(256), 0, stream, a);
  return hipGetLastError();
}

hipError_t launch_gru_gates_bwd(const GruBwdArgs& a, hipStream_t stream) {
  long work = 0;
  for (int k = 0; k < a.n_nets; ++k) { const long w = (long)a.nb * (a.net[k].H >> 2); work = w > work ? w : work; }
  if (work == 0) return hipSuccess;
  double bytes = 0.0;
  for (int k = 0; k < a.n_nets; ++k) bytes += 4.0 * a.nb * a.net[k].H * (6 + 2 + (a.net[k].back ? 2 : 0) + 6 + 1);
  TraceScope ts(stream, "gru_gates_bwd", 0.0, bytes);
  hipLaunchKernelGGL(gru_gates_bwd_kernel, dim3((unsigned)((work + 255) / 256), a.n_nets), dim3(256), 0, stream, a);
  return hipGetLastError();
}

hipError_t launch_row_gather(const RowGatherArgs& a, hipStream_t stream) {
  long work = 0;
  for (int k = 0; k < a.n_jobs; ++k) { const long w = (long)a.nb * (a.job[k].H >> 2); work = w > work ? w : work; }
  if (work == 0) return hipSuccess;
  hipLaunchKernelGGL(row_gather_kernel, dim3((unsigned)((work + 255) / 256), a.n_jobs), dim3(256), 0, stream, a);
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
