// Streaming, reduction and bookkeeping kernels of librslx for gfx950: GAE reverse scan, advantage
// normalisation, minibatch permutation (hash keys + bucket sort), split-K gradient reduction with the
// squared-norm, fused clip + Adam, Gaussian policy head, PPO loss head, MSE head, mirror augmentation,
// RND reward normalisation.  Wavefronts are 64 lanes wide throughout.
#include "kernels.h"

namespace rslx {

constexpr int WAVE = 64;

// ---- reductions -----------------------------------------------------------------------------------
constexpr float LOG_2PI = 1.8378770664093453f;

__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
  for (int o = WAVE / 2; o > 0; o >>= 1) v += __shfl_down(v, o, WAVE);
  return v;
}

// Sum over the workgroup; result valid in thread 0.  `smem` holds one double per wavefront.
__device__ __forceinline__ double block_sum(double v, double* smem) {
  const int lane = threadIdx.x & (WAVE - 1), w = threadIdx.x / WAVE;
  const int nw = (blockDim.x + WAVE - 1) / WAVE;
  v = wave_sum(v);
  __syncthreads();
  if (lane == 0) smem[w] = v;
  __syncthreads();
  double t = 0.0;
  if (threadIdx.x == 0)
    for (int i = 0; i < nw; ++i) t += smem[i];
  return t;
}

__global__ void fill_kernel(float* p, long n, float value) {
  long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = value;
}

hipError_t launch_fill(float* p, int64_t n, float value, hipStream_t stream) {
  if (n <= 0) return hipSuccess;
  hipLaunchKernelGGL(fill_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, stream, p, (long)n, value);
  return hipGetLastError();
}

// ---- GAE ----------------------------------------------------------------------------------------------
// One lane per environment column: loads are coalesced across n, the T-step recurrence runs in registers.
template <int BLOCK>
__global__ __launch_bounds__(BLOCK) void gae_scan_kernel(const float* __restrict__ rewards, const float* __restrict__ values,
                                                         const float* __restrict__ last_values,
                                                         const uint8_t* __restrict__ dones,
                                                         const uint8_t* __restrict__ timeouts, int T, int N, float gamma,
                                                         float lam, float* __restrict__ adv, float* __restrict__ ret,
                                                         double* __restrict__ partials) {
  __shared__ double smem[BLOCK / WAVE];
  const int n = blockIdx.x * BLOCK + threadIdx.x;
  double s = 0.0, q = 0.0;
  if (n < N) {
    float a_next = 0.f;
    float v_next = last_values[n];
    const float gl = gamma * lam;
#pragma unroll 8
    for (int t = T - 1; t >= 0; --t) {
      const long o = (long)t * N + n;
      float r = rewards[o];
      const float v = values[o];
      const float nd = dones[o] ? 0.f : 1.f;
      if (timeouts != nullptr && timeouts[o]) r += gamma * v;
      const float delta = r + gamma * nd * v_next - v;
      a_next = delta + gl * nd * a_next;
      adv[o] = a_next;
      ret[o] = a_next + v;
      s += (double)a_next;
      q += (double)a_next * (double)a_next;
      v_next = v;
    }
  }
  if (partials != nullptr) {
    double ts = block_sum(s, smem);
    double tq = block_sum(q, smem);
    if (threadIdx.x == 0) {
      partials[2 * blockIdx.x] = ts;
      partials[2 * blockIdx.x + 1] = tq;
    }
  }
}

// Single workgroup: total sum / sum of squares -> mean and 1 / (std + 1e-8), unbiased std.
__global__ __launch_bounds__(256) void adv_stats_kernel(const double* __restrict__ partials, int nblocks, long count,
                                                        float* __restrict__ mean_inv) {
  __shared__ double smem[4];
  double s = 0.0, q = 0.0;
  for (int i = threadIdx.x; i < nblocks; i += 256) {
    s += partials[2 * i];
    q += partials[2 * i + 1];
  }
  double ts = block_sum(s, smem);
  double tq = block_sum(q, smem);
  if (threadIdx.x == 0) {
    double mean = ts / (double)count;
    double var = count > 1 ? (tq - ts * mean) / (double)(count - 1) : 0.0;
    if (var < 0.0) var = 0.0;
    mean_inv[0] = (float)mean;
    mean_inv[1] = (float)(1.0 / (sqrt(var) + 1e-8));
  }
}

// mean_inv != null: mean and 1 / (std + 1e-8) were formed by adv_stats_kernel.  mean_inv == null: every workgroup
// forms them itself from the scan's block partials, in the same order and arithmetic as adv_stats_kernel (short
// lists only: saves a launch where the whole problem is a few MB).
__global__ __launch_bounds__(256) void adv_normalize_kernel(float* __restrict__ adv, long count,
                                                            const float* __restrict__ mean_inv,
                                                            const double* __restrict__ partials, int nblocks) {
  __shared__ double smem[4];
  __shared__ float s_mi[2];
  float mean, inv;
  if (mean_inv != nullptr) {
    mean = mean_inv[0]; inv = mean_inv[1];
  } else {
    double s = 0.0, q = 0.0;
    for (int i = threadIdx.x; i < nblocks; i += 256) {
      s += partials[2 * i];
      q += partials[2 * i + 1];
    }
    const double ts = block_sum(s, smem);
    const double tq = block_sum(q, smem);
    if (threadIdx.x == 0) {
      const double m = ts / (double)count;
      double var = count > 1 ? (tq - ts * m) / (double)(count - 1) : 0.0;
      if (var < 0.0) var = 0.0;
      s_mi[0] = (float)m;
      s_mi[1] = (float)(1.0 / (sqrt(var) + 1e-8));
    }
    __syncthreads();
    mean = s_mi[0]; inv = s_mi[1];
  }
  long i = ((long)blockIdx.x * 256 + threadIdx.x) * 4;
  if (i + 3 < count) {
    float4 v = *reinterpret_cast<float4*>(adv + i);
    v.x = (v.x - mean) * inv; v.y = (v.y - mean) * inv; v.z = (v.z - mean) * inv; v.w = (v.w - mean) * inv;
    *reinterpret_cast<float4*>(adv + i) = v;
  } else {
    for (; i < count; ++i) adv[i] = (adv[i] - mean) * inv;
  }
}

static int gae_block(int32_t N) { return N >= 65536 ? 256 : 64; }
int gae_num_blocks(int32_t N) { int b = gae_block(N); return (N + b - 1) / b; }

hipError_t launch_gae(const float* rewards, const float* values, const float* last_values, const uint8_t* dones,
                      const uint8_t* timeouts, int32_t T, int32_t N, float gamma, float lam, int32_t normalize,
                      float* adv, float* ret, double* partials, hipStream_t stream) {
  const int nb = gae_num_blocks(N);
  double* part = normalize ? partials : nullptr;
  TraceScope ts(stream, normalize ? "gae_scan+normalize" : "gae_scan", 0.0,
                (double)T * N * (normalize ? 25.0 : 17.0) + 4.0 * N);
  if (gae_block(N) == 256)
    hipLaunchKernelGGL((gae_scan_kernel<256>), dim3(nb), dim3(256), 0, stream, rewards, values, last_values, dones,
                       timeouts, T, N, gamma, lam, adv, ret, part);
  else
    hipLaunchKernelGGL((gae_scan_kernel<64>), dim3(nb), dim3(64), 0, stream, rewards, values, last_values, dones,
                       timeouts, T, N, gamma, lam, adv, ret, part);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess || !normalize) return e;
  const long count = (long)T * N;
  const unsigned blocks = (unsigned)((count + 1023) / 1024);
  if (nb <= 512) {      // short partial list: the normalisation launch sums it itself
    hipLaunchKernelGGL(adv_normalize_kernel, dim3(blocks), dim3(256), 0, stream, adv, count, (const float*)nullptr, partials, nb);
    return hipGetLastError();
  }
  float* mean_inv = reinterpret_cast<float*>(partials + 2 * (size_t)nb);
  hipLaunchKernelGGL(adv_stats_kernel, dim3(1), dim3(256), 0, stream, partials, nb, count, mean_inv);
  hipLaunchKernelGGL(adv_normalize_kernel, dim3(blocks), dim3(256), 0, stream, adv, count, mean_inv, (const double*)nullptr, 0);
  return hipGetLastError();
}

// ---- permutation ------------------------------------------------------------------------------------
__device__ __forceinline__ uint64_t mix64(uint64_t x) {
  x += 0x9E3779B97F4A7C15ull;
  x = (x ^ (x >> 30)) * 0xBF58476D1CE4E5B9ull;
  x = (x ^ (x >> 27)) * 0x94D049BB133111EBull;
  return x ^ (x >> 31);
}

// Keys are uniform 64-bit hashes, so their top bits spread the B items evenly over nb buckets
// (about 32 per bucket).  Bucket membership is order independent; the order inside a bucket is then
// fixed by ranking on (key, index), which makes the result independent of atomic scheduling.
constexpr int PERM_BATCH = 8;   // permutations per launch
struct PermPlan {
  int32_t nb;      // buckets (power of two)
  int32_t shift;   // key >> shift = bucket
};
static PermPlan perm_plan(int32_t B) {
  PermPlan p;
  int lg = 0;
  while ((1 << (lg + 1)) * 32 <= B && lg < 24) ++lg;
  p.nb = 1 << lg;
  p.shift = 64 - lg;
  return p;
}
__device__ __forceinline__ int bucket_of(uint64_t key, int shift) { return shift >= 64 ? 0 : (int)(key >> shift); }

// All kernels below process up to PERM_BATCH permutations (epochs) per launch: blockIdx.y selects the epoch,
// whose scratch arrays sit `*_stride` elements apart.
struct PermBases {
  uint64_t base[PERM_BATCH];
  uint64_t seed_mixed;           // with call_dev: base of entry e = mix64(mix64(seed_mixed ^ *call_dev) ^ epoch[e])
  const uint64_t* call_dev;
  int32_t epoch[PERM_BATCH];
};
__device__ __forceinline__ uint64_t perm_base(const PermBases& pb, int e) {
  if (pb.call_dev == nullptr) return pb.base[e];
  return mix64(mix64(pb.seed_mixed ^ *pb.call_dev) ^ (uint64_t)pb.epoch[e]);
}

__global__ void perm_zero_kernel(int* counts, int n, long stride) {
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) counts[blockIdx.y * stride + i] = 0;
}
__global__ void perm_hist_kernel(const PermBases pb, int B, int shift, int* counts, long stride) {
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < B) atomicAdd(&counts[blockIdx.y * stride + bucket_of(mix64(perm_base(pb, blockIdx.y) ^ (uint64_t)i), shift)], 1);
}
// Exclusive scan of counts[0..nb) by one workgroup per epoch; offsets has nb + 1 entries; cursors are reset.
__global__ __launch_bounds__(1024) void perm_scan_kernel(const int* counts_all, int nb, int* offsets_all, int* cursor_all,
                                                         long stride) {
  __shared__ int wsum[16];
  __shared__ int carry;
  const int* counts = counts_all + blockIdx.y * stride;
  int* offsets = offsets_all + blockIdx.y * stride;
  int* cursor = cursor_all + blockIdx.y * stride;
  if (threadIdx.x == 0) carry = 0;
  __syncthreads();
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  for (int base = 0; base < nb; base += 1024) {
    int i = base + threadIdx.x;
    int c = i < nb ? counts[i] : 0;
    int x = c;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
      int y = __shfl_up(x, o, 64);
      if (lane >= o) x += y;
    }
    if (lane == 63) wsum[w] = x;
    __syncthreads();
    int before = 0;
    for (int k = 0; k < w; ++k) before += wsum[k];
    int excl = carry + before + x - c;
    if (i < nb) {
      offsets[i] = excl;
      cursor[i] = 0;
    }
    __syncthreads();
    if (threadIdx.x == 1023) carry = excl + c;
    __syncthreads();
  }
  if (threadIdx.x == 0) offsets[nb] = carry;
}
__global__ void perm_scatter_kernel(const PermBases pb, int B, int shift, const int* offsets, int* cursor, long stride,
                                    uint64_t* keys, int* idx, long kstride) {
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= B) return;
  const int e = blockIdx.y;
  uint64_t k = mix64(perm_base(pb, e) ^ (uint64_t)i);
  int b = bucket_of(k, shift);
  int pos = offsets[e * stride + b] + atomicAdd(&cursor[e * stride + b], 1);
  keys[e * kstride + pos] = k;
  idx[e * kstride + pos] = i;
}
__global__ void perm_rank_kernel(int B, int shift, const int* offsets_all, long stride, const uint64_t* keys_all,
                                 const int* idx_all, long kstride, int* perm_all) {
  int el = blockIdx.x * blockDim.x + threadIdx.x;
  if (el >= B) return;
  const int e = blockIdx.y;
  const uint64_t* keys = keys_all + e * kstride;
  const int* idx = idx_all + e * kstride;
  const int* offsets = offsets_all + e * stride;
  const uint64_t k = keys[el];
  const int i = idx[el];
  const int b = bucket_of(k, shift);
  const int s = offsets[b], t = offsets[b + 1];
  int rank = 0;
  for (int o = s; o < t; ++o) {
    uint64_t ko = keys[o];
    rank += (ko < k || (ko == k && idx[o] < i)) ? 1 : 0;
  }
  perm_all[(long)e * B + s + rank] = i;
}

static size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

size_t perm_workspace_bytes(int32_t B) {
  PermPlan p = perm_plan(B);
  const size_t seg = align_up((size_t)(p.nb + 1) * 4, 256);
  const size_t kseg = align_up((size_t)B * 8, 256);
  return (size_t)PERM_BATCH * (3 * seg + kseg + kseg / 2 + 256);
}

hipError_t launch_permutations(const uint64_t* base_keys, int32_t n_perm, int32_t B, int32_t* perm_out, void* ws,
                               hipStream_t stream, uint64_t seed_mixed, const uint64_t* call_index_dev, int32_t epoch0) {
  if (B <= 0 || n_perm <= 0) return hipSuccess;
  TraceScope ts(stream, "permutation", 0.0, 0.0);
  PermPlan p = perm_plan(B);
  char* w = static_cast<char*>(ws);
  const size_t seg = align_up((size_t)(p.nb + 1) * 4, 256);
  const size_t kseg = align_up((size_t)B * 8, 256);
  int* counts = reinterpret_cast<int*>(w);
  int* offsets = reinterpret_cast<int*>(w + PERM_BATCH * seg);
  int* cursor = reinterpret_cast<int*>(w + 2 * PERM_BATCH * seg);
  uint64_t* keys = reinterpret_cast<uint64_t*>(w + 3 * PERM_BATCH * seg);
  int* idx = reinterpret_cast<int*>(w + 3 * PERM_BATCH * seg + PERM_BATCH * kseg);
  const long stride = (long)(seg / 4), kstride = (long)(kseg / 8);
  const unsigned gb = (unsigned)((B + 255) / 256);
  for (int e0 = 0; e0 < n_perm; e0 += PERM_BATCH) {
    const int ne = n_perm - e0 < PERM_BATCH ? n_perm - e0 : PERM_BATCH;
    PermBases pb;
    pb.seed_mixed = seed_mixed;
    pb.call_dev = call_index_dev;
    for (int e = 0; e < PERM_BATCH; ++e) {
      pb.base[e] = (e < ne && call_index_dev == nullptr) ? base_keys[e0 + e] : 0;
      pb.epoch[e] = epoch0 + e0 + e;
    }
    int32_t* out = perm_out + (size_t)e0 * B;
    hipLaunchKernelGGL(perm_zero_kernel, dim3((p.nb + 256) / 256, ne), dim3(256), 0, stream, counts, p.nb + 1, stride);
    hipLaunchKernelGGL(perm_hist_kernel, dim3(gb, ne), dim3(256), 0, stream, pb, B, p.shift, counts, stride);
    hipLaunchKernelGGL(perm_scan_kernel, dim3(1, ne), dim3(1024), 0, stream, counts, p.nb, offsets, cursor, stride);
    hipLaunchKernelGGL(perm_scatter_kernel, dim3(gb, ne), dim3(256), 0, stream, pb, B, p.shift, offsets, cursor, stride, keys,
                       idx, kstride);
    hipLaunchKernelGGL(perm_rank_kernel, dim3(gb, ne), dim3(256), 0, stream, B, p.shift, offsets, stride, keys, idx, kstride,
                       out);
  }
  return hipGetLastError();
}

// ---- split-K reduction + squared norm ---------------------------------------------------------------
constexpr int RED_PER_BLOCK = 1024;  // floats per workgroup of the plain squared-norm kernel
int reduce_num_blocks(int64_t n) { return (int)((n + RED_PER_BLOCK - 1) / RED_PER_BLOCK); }

// Sums the per-block partial sums of the PPO loss head in a fixed order: the 256 lanes form 256 / ncomp groups of
// ncomp lanes (one lane per component, so a group reads one block's partials as consecutive words), group g takes
// blocks g, g + G, ..; the groups' sums are then added in index order.  Wavefront 0 writes the statistics row and the
// log_std gradient (two components per lane cover the widest action vector).
__device__ void loss_finish_block(const LossFinishArgs& f) {
  constexpr int NC = PPO_NPART_FIXED + 64;          // components at the widest action vector
  static_assert(NC <= 2 * 64, "two components per lane cover every action width");
  __shared__ double gpart[256];
  __shared__ double total[2 * 64];
  const int t = threadIdx.x, lane = t & 63, w = t >> 6;
  const int A = f.A, ncomp = PPO_NPART_FIXED + A;
  const int G = 256 / ncomp;
  const int grp = t / ncomp, c_own = t - grp * ncomp;
  double acc = 0.0;
  if (grp < G) {
#pragma unroll 8
    for (int b = grp; b < f.blocks; b += G) acc += f.partials[(long)b * ncomp + c_own];
  }
  gpart[t] = acc;
  __syncthreads();
  if (t < 2 * 64) {
    double s = 0.0;
    if (t < ncomp)
      for (int g = 0; g < G; ++g) s += gpart[g * ncomp + t];
    total[t] = s;
  }
  __syncthreads();
  if (w != 0) return;
  double g2 = 0.0, ent = 0.0;
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    const int c = lane + 64 * h;
    if (c >= PPO_NPART_FIXED && c < ncomp) {
      const float g = (float)total[c] - f.entropy_coef;
      f.d_log_std[c - PPO_NPART_FIXED] = g;
      g2 += (double)g * (double)g;
    }
  }
  g2 = wave_sum(g2);
  if (lane < A) ent = 0.5 + 0.5 * (double)LOG_2PI + (double)f.log_std[lane];
  ent = wave_sum(ent);
  const int rows = f.rows, mb = f.mb;
  const int c = lane;
  const double s = total[lane];
  if (c == 0) {
    *f.sumsq_slot = g2;
    f.stats_row[0] = (float)(s / rows);
    f.stats_row[2] = (float)ent;
  }
  if (c == 1) f.stats_row[1] = (float)(s / rows);
  if (c == 2) f.stats_row[3] = (float)(s / mb);
  if (c == 3) f.stats_row[5] = (float)(s / rows);
  if (c == 4) f.stats_row[6] = rows > mb ? (float)(s / ((double)mb * A)) : 0.f;
  if (c == 5) f.stats_row[7] = 0.f;
}

// One workgroup sums 256 consecutive gradient entries of one layer over all of that layer's splits: 64 lanes
// cover the 256 floats with one 16-byte load each, the 4 wavefronts take every 4th split, LDS combines them
// in a fixed order (deterministic result).  The layers of all networks trained in a step share one launch; its
// first workgroup finishes the loss sums instead.
__global__ __launch_bounds__(256) void reduce_partials_kernel(const ReduceArgs a) {
  // the loss sums are a chain of dependent loads in one workgroup: it goes first so that it runs beside the others
  const int has_finish = a.finish.blocks > 0 ? 1 : 0;
  if (has_finish && blockIdx.x == 0) {
    loss_finish_block(a.finish);
    return;
  }
  const int bid = (int)blockIdx.x - has_finish;
  __shared__ float4 part[4][64];
  __shared__ double smem[4];
  int si = 0;
  while (si + 1 < a.n_seg && bid >= a.seg[si + 1].block_start) ++si;
  const ReduceSeg& sg = a.seg[si];
  const long size = sg.size;
  const int n_split = sg.split;
  const float* src = sg.partials;
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const long j0 = ((long)(bid - sg.block_start) * 64 + lane) * 4;
  float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
  if (j0 < size) {      // pitch is a multiple of 4, so the 16-byte load stays inside the split buffer's padding
    const long pitch = sg.pitch;
#pragma unroll 4
    for (int k = w; k < n_split; k += 4) {
      const float4 v = *reinterpret_cast<const float4*>(src + (long)k * pitch + j0);
      s.x += v.x; s.y += v.y; s.z += v.z; s.w += v.w;
    }
  }
  part[w][lane] = s;
  __syncthreads();
  double q = 0.0;
  if (w == 0 && j0 < size) {
    float4 t = part[0][lane];
    for (int g = 1; g < 4; ++g) { t.x += part[g][lane].x; t.y += part[g][lane].y; t.z += part[g][lane].z; t.w += part[g][lane].w; }
    const float* tp = &t.x;
    float* dst = sg.grads + j0;
    for (int c = 0; c < 4; ++c)
      if (j0 + c < size) {
        dst[c] = tp[c];
        q += (double)tp[c] * (double)tp[c];
      }
  }
  double tot = block_sum(q, smem);
  if (threadIdx.x == 0) a.sumsq_blocks[bid] = tot;
}

hipError_t launch_reduce_partials(const ReduceArgs& a, hipStream_t stream) {
  const int extra = a.finish.blocks > 0 ? 1 : 0;
  if (a.blocks + extra <= 0) return hipSuccess;
  double bytes = 0.0;
  for (int i = 0; i < a.n_seg; ++i) bytes += 4.0 * (double)a.seg[i].size * (a.seg[i].split + 1);
  TraceScope ts(stream, "reduce_partials", 0.0, bytes);
  hipLaunchKernelGGL(reduce_partials_kernel, dim3(a.blocks + extra), dim3(256), 0, stream, a);
  return hipGetLastError();
}

__global__ __launch_bounds__(256) void sumsq_kernel(const float* __restrict__ g, long n, double* __restrict__ out) {
  __shared__ double smem[4];
  const long i0 = ((long)blockIdx.x * 256 + threadIdx.x) * 4;
  double q = 0.0;
#pragma unroll
  for (int c = 0; c < 4; ++c)
    if (i0 + c < n) q += (double)g[i0 + c] * (double)g[i0 + c];
  double t = block_sum(q, smem);
  if (threadIdx.x == 0) out[blockIdx.x] = t;
}

hipError_t launch_sumsq(const float* g, int64_t n, double* sumsq_blocks, hipStream_t stream) {
  if (n <= 0) return hipSuccess;
  hipLaunchKernelGGL(sumsq_kernel, dim3(reduce_num_blocks(n)), dim3(256), 0, stream, g, (long)n, sumsq_blocks);
  return hipGetLastError();
}

// ---- fused clip + Adam ------------------------------------------------------------------------------
// Every workgroup re-reduces the (short) list of per-block squared norms in the same order, so the clip
// scale is identical everywhere and no extra launch or atomic is needed.
// Writes the updated weight with flat parameter index i to its transposed position (biases and the layers below
// wt_from have none).
__device__ __forceinline__ void adam_store_transposed(const AdamSegment& sg, long i, float value) {
  long o = 0;
  for (int l = 0; l < sg.n_layers; ++l) {
    const int rows = sg.dims[l], cols = sg.dims[l + 1];
    const long w = (long)rows * cols;
    if (i < o + w) {
      if (l >= sg.wt_from) {
        const int e = (int)(i - o);
        const int r = e / cols, c = e - r * cols;
        sg.wt[o + (long)c * rows + r] = value;
      }
      return;
    }
    o += w + cols;
    if (i < o) return;
  }
}

__global__ __launch_bounds__(256) void adam_kernel(const AdamArgs a) {
  __shared__ double smem[4];
  __shared__ float s_scale, s_bc1, s_bc2;
  // the lane's parameter, gradient and moment loads are requested before the squared-norm list is summed, so the
  // two memory latencies overlap
  const AdamSegment& sg = a.seg[blockIdx.y];
  const long i0 = ((long)blockIdx.x * 256 + threadIdx.x) * 4;
  const bool whole = i0 + 3 < sg.n;
  float4 p = make_float4(0.f, 0.f, 0.f, 0.f), g = p, m = p, v = p;
  if (whole) {
    p = *reinterpret_cast<const float4*>(sg.params + i0);
    g = *reinterpret_cast<const float4*>(sg.grads + i0);
    m = *reinterpret_cast<const float4*>(sg.m + i0);
    v = *reinterpret_cast<const float4*>(sg.v + i0);
  }
  double q = 0.0;
  for (int i = threadIdx.x; i < a.n_sumsq; i += 256) q += a.sumsq_blocks[i];
  double tot = block_sum(q, smem);
  if (threadIdx.x == 0) {
    float bc1 = a.bc1, bc2 = a.bc2;
    if (a.step_dev != nullptr) {          // step counter in device memory: bias corrections formed here
      const double t = (double)(*a.step_dev + a.step_off);
      bc1 = (float)(1.0 - pow((double)a.beta1, t));
      bc2 = (float)(1.0 - pow((double)a.beta2, t));
    }
    s_bc1 = bc1; s_bc2 = bc2;
    float norm = (float)sqrt(tot);
    float s = 1.0f;
    if (a.max_grad_norm > 0.f && a.max_grad_norm < 3.0e38f) s = fminf(1.0f, a.max_grad_norm / (norm + 1e-6f));
    s_scale = s;
    if (a.grad_norm_out != nullptr && blockIdx.x == 0 && blockIdx.y == 0) *a.grad_norm_out = norm;
  }
  __syncthreads();
  const float scale = s_scale;
  const float ob1 = 1.0f - a.beta1, ob2 = 1.0f - a.beta2;
  const float inv_bc1 = 1.0f / s_bc1, inv_bc2 = 1.0f / s_bc2;
  if (i0 >= sg.n) return;
  if (whole) {
    float* pp = &p.x; float* gp = &g.x; float* mp = &m.x; float* vp = &v.x;
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      const float gg = gp[c] * scale;
      mp[c] = a.beta1 * mp[c] + ob1 * gg;
      vp[c] = a.beta2 * vp[c] + ob2 * gg * gg;
      pp[c] -= a.lr * (mp[c] * inv_bc1) / (sqrtf(vp[c] * inv_bc2) + a.eps);
    }
    *reinterpret_cast<float4*>(sg.params + i0) = p;
    *reinterpret_cast<float4*>(sg.m + i0) = m;
    *reinterpret_cast<float4*>(sg.v + i0) = v;
    if (sg.wt != nullptr) {
#pragma unroll
      for (int c = 0; c < 4; ++c) adam_store_transposed(sg, i0 + c, pp[c]);
    }
  } else {
    for (long i = i0; i < sg.n; ++i) {
      const float gg = sg.grads[i] * scale;
      const float m = a.beta1 * sg.m[i] + ob1 * gg;
      const float v = a.beta2 * sg.v[i] + ob2 * gg * gg;
      sg.m[i] = m;
      sg.v[i] = v;
      const float pn = sg.params[i] - a.lr * (m * inv_bc1) / (sqrtf(v * inv_bc2) + a.eps);
      sg.params[i] = pn;
      if (sg.wt != nullptr) adam_store_transposed(sg, i, pn);
    }
  }
}

// Long squared-norm lists (large flat buffers) are first folded to one value by a single workgroup, so that the
// per-block re-reduction in adam_kernel stays short.
__global__ __launch_bounds__(1024) void sumsq_fold_kernel(const double* __restrict__ in, int n, double* __restrict__ out) {
  __shared__ double smem[16];
  double q = 0.0;
  for (int i = threadIdx.x; i < n; i += 1024) q += in[i];
  double t = block_sum(q, smem);
  if (threadIdx.x == 0) *out = t;
}

hipError_t launch_adam(const AdamArgs& a_in, hipStream_t stream) {
  AdamArgs a = a_in;
  if (a.n_sumsq > ADAM_MAX_INLINE_SUMSQ) {     // caller reserved one extra slot behind the list
    double* total = const_cast<double*>(a.sumsq_blocks) + a.n_sumsq;
    hipLaunchKernelGGL(sumsq_fold_kernel, dim3(1), dim3(1024), 0, stream, a.sumsq_blocks, a.n_sumsq, total);
    a.sumsq_blocks = total;
    a.n_sumsq = 1;
  }
  int64_t nmax = 0;
  for (int i = 0; i < a.n_seg; ++i) nmax = a.seg[i].n > nmax ? a.seg[i].n : nmax;
  if (nmax <= 0) return hipSuccess;
  double n_all = 0.0;
  for (int i = 0; i < a.n_seg; ++i) n_all += (double)a.seg[i].n;
  TraceScope ts(stream, "adam", 0.0, 28.0 * n_all);
  dim3 grid((unsigned)((nmax + 1023) / 1024), a.n_seg);
  hipLaunchKernelGGL(adam_kernel, grid, dim3(256), 0, stream, a);
  return hipGetLastError();
}

// ---- Gaussian head of act() -------------------------------------------------------------------------

__global__ __launch_bounds__(256) void act_head_kernel(const float* __restrict__ mu_in, const float* __restrict__ log_std,
                                                       const float* __restrict__ eps_in, uint64_t noise_base, int N,
                                                       int A, int deterministic, float* __restrict__ actions,
                                                       float* __restrict__ logp, float* __restrict__ mu_out,
                                                       float* __restrict__ sigma_out, const int64_t* __restrict__ step_dev,
                                                       uint64_t noise_pre) {
  const int n = blockIdx.x * 256 + threadIdx.x;
  if (n >= N) return;
  if (step_dev != nullptr) noise_base = mix64(noise_pre ^ (uint64_t)*step_dev);
  float acc = 0.f, sum_ls = 0.f;
  for (int jj = 0; jj < A; ++jj) {
    const long o = (long)n * A + jj;
    const float ls = log_std[jj];
    const float sg = expf(ls);
    const float mu = mu_in[o];
    float e;
    if (deterministic) {
      e = 0.f;
    } else if (eps_in != nullptr) {
      e = eps_in[o];
    } else {
      const uint64_t h = mix64(noise_base ^ (uint64_t)o);
      const float u1 = (float)((uint32_t)(h >> 40) + 1u) * 5.9604644775390625e-08f;   // 2^-24
      const float u2 = (float)((uint32_t)(h >> 8) & 0xFFFFFFu) * 5.9604644775390625e-08f;
      e = sqrtf(-2.0f * logf(u1)) * cospif(2.0f * u2);
    }
    const float act = mu + sg * e;
    const float z = (act - mu) / sg;
    acc += z * z;
    sum_ls += ls;
    actions[o] = act;
    mu_out[o] = mu;
    sigma_out[o] = sg;
  }
  logp[n] = -0.5f * acc - sum_ls - 0.5f * (float)A * LOG_2PI;
}

hipError_t launch_act_head(const float* mu_in, const float* log_std, const float* eps, uint64_t noise_base, int32_t N,
                           int32_t A, int32_t deterministic, float* actions, float* logp, float* mu_out,
                           float* sigma_out, hipStream_t stream, const int64_t* step_dev, uint64_t noise_pre) {
  hipLaunchKernelGGL(act_head_kernel, dim3((N + 255) / 256), dim3(256), 0, stream, mu_in, log_std, eps, noise_base, N, A,
                     deterministic, actions, logp, mu_out, sigma_out, step_dev, noise_pre);
  return hipGetLastError();
}

// counters[i] += delta.d[i] for i < n: advances the call-to-call counters that live in device memory.
struct CounterDeltas { int64_t d[4]; };
__global__ void counter_add_kernel(int64_t* counters, CounterDeltas delta, int n) {
  if (blockIdx.x == 0 && (int)threadIdx.x < n) counters[threadIdx.x] += delta.d[threadIdx.x];
}
hipError_t launch_counter_add(int64_t* counters, const int64_t* delta, int32_t n, hipStream_t stream) {
  CounterDeltas cd{};
  for (int i = 0; i < n && i < 4; ++i) cd.d[i] = delta[i];
  hipLaunchKernelGGL(counter_add_kernel, dim3(1), dim3(64), 0, stream, counters, cd, n < 4 ? n : 4);
  return hipGetLastError();
}

__global__ void copy_kernel(const float* __restrict__ src, int n, float* __restrict__ dst) {
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) dst[i] = src[i];
}
hipError_t launch_copy_column(const float* src, int32_t n, float* dst, hipStream_t stream) {
  hipLaunchKernelGGL(copy_kernel, dim3((n + 255) / 256), dim3(256), 0, stream, src, n, dst);
  return hipGetLastError();
}

// ---- PPO loss head -------------------------------------------------------------------------------------
// One lane per minibatch row i (and, with symmetry, its mirrored twin at row i + mb).
constexpr int AMAX = 32;
int ppo_loss_num_blocks(int32_t mb) { return (mb + 255) / 256; }

struct RowTerms { float surr, vloss, clipped; };

__device__ __forceinline__ RowTerms ppo_row(const PpoLossArgs& a, float logp_new, float logp_old, float adv, float v,
                                            float v_old, float ret, float inv_rows, float* d_logp, float* d_v) {
  RowTerms t;
  const float ratio = expf(logp_new - logp_old);
  const float rc = fminf(fmaxf(ratio, 1.0f - a.clip), 1.0f + a.clip);
  const float s1 = -adv * ratio, s2 = -adv * rc;
  t.surr = fmaxf(s1, s2);
  const bool ratio_in = ratio >= 1.0f - a.clip && ratio <= 1.0f + a.clip;
  *d_logp = ((ratio_in || s1 >= s2) ? -adv : 0.f) * inv_rows * ratio;
  t.clipped = fabsf(ratio - 1.0f) > a.clip ? 1.f : 0.f;
  if (a.clipped_value) {
    const float vc = v_old + fminf(fmaxf(v - v_old, -a.clip), a.clip);
    const float e1 = (v - ret) * (v - ret), e2 = (vc - ret) * (vc - ret);
    t.vloss = fmaxf(e1, e2);
    const bool v_in = fabsf(v - v_old) <= a.clip;   // inside the clip range the clipped branch equals the plain one
    *d_v = ((v_in || e1 >= e2) ? 2.0f * (v - ret) : 0.f) * inv_rows * a.value_coef;
  } else {
    t.vloss = (ret - v) * (ret - v);
    *d_v = 2.0f * (v - ret) * inv_rows * a.value_coef;
  }
  return t;
}

// Per-thread partial sums of the loss head.
template <int AM>
struct PpoAcc {
  float surr = 0.f, vloss = 0.f, kl = 0.f, clipped = 0.f, mirror = 0.f;
  float dls[AM];
};

// Rollout quantities of one minibatch row, gathered through the permutation.
template <int AM>
struct PpoRowIn {
  float adv, ret, v_old, logp_old;
  float act[AM], mu_old[AM], sigma_old[AM];
  float act_m[AM];     // mirrored action (symmetry only)
};

template <int AM>
__device__ __forceinline__ void ppo_row_load(const PpoLossArgs& a, int i, PpoRowIn<AM>& in) {
  const int A = a.A;
  const long b = a.idx[i];
  in.adv = a.adv[b]; in.ret = a.returns[b]; in.v_old = a.v_old[b]; in.logp_old = a.logp_old[b];
#pragma unroll
  for (int jj = 0; jj < AM; ++jj) {
    if (jj < A) {
      in.act[jj] = a.actions[b * A + jj];
      in.mu_old[jj] = a.mu_old[b * A + jj];
      in.sigma_old[jj] = a.sigma_old[b * A + jj];
      if (a.rows > a.mb) in.act_m[jj] = a.sign_act[jj] * a.actions[b * A + a.perm_act[jj]];
    }
  }
}

// Loss terms and output gradients of one minibatch row (and, with symmetry, of its mirrored twin).  mu / d_mu
// pointers address one row of A values each (global memory or LDS); v / d_v are scalars.
template <int AM>
__device__ __forceinline__ void ppo_loss_row(const PpoLossArgs& a, const PpoRowIn<AM>& in, const float* mu_row,
                                             const float* mu_twin, float v_row, float v_twin, float* dmu_row,
                                             float* dmu_twin, float* dv_row, float* dv_twin, PpoAcc<AM>& acc) {
  const int A = a.A;
  const bool sym = a.rows > a.mb;
  const float inv_rows = 1.0f / (float)a.rows;
  const float adv = in.adv, ret = in.ret, v_old = in.v_old, logp_old = in.logp_old;
  float mu[AM], sg[AM];
  const float (&act)[AM] = in.act;
  float zz = 0.f, sum_ls = 0.f;
#pragma unroll
  for (int jj = 0; jj < AM; ++jj) {
    if (jj < A) {
      const float ls = a.log_std[jj];
      sg[jj] = expf(ls);
      mu[jj] = mu_row[jj];
      const float z = (act[jj] - mu[jj]) / sg[jj];
      zz += z * z;
      sum_ls += ls;
      const float so = in.sigma_old[jj], mo = in.mu_old[jj];
      acc.kl += logf(sg[jj] / so) + (so * so + (mo - mu[jj]) * (mo - mu[jj])) / (2.0f * sg[jj] * sg[jj]) - 0.5f;
    }
  }
  const float logp_new = -0.5f * zz - sum_ls - 0.5f * (float)A * LOG_2PI;
  float d_logp, d_v;
  RowTerms t = ppo_row(a, logp_new, logp_old, adv, v_row, v_old, ret, inv_rows, &d_logp, &d_v);
  acc.surr += t.surr; acc.vloss += t.vloss; acc.clipped += t.clipped;
  *dv_row = d_v;
#pragma unroll
  for (int jj = 0; jj < AM; ++jj) {
    if (jj < A) {
      const float z = (act[jj] - mu[jj]) / sg[jj];
      dmu_row[jj] = d_logp * z / sg[jj];
      acc.dls[jj] += d_logp * (z * z - 1.0f);
    }
  }
  if (sym) {
    float zz2 = 0.f;
    float mum[AM], zm[AM];
#pragma unroll
    for (int jj = 0; jj < AM; ++jj) {
      if (jj < A) {
        mum[jj] = mu_twin[jj];
        const float am = in.act_m[jj];
        zm[jj] = (am - mum[jj]) / sg[jj];
        zz2 += zm[jj] * zm[jj];
      }
    }
    const float logp_m = -0.5f * zz2 - sum_ls - 0.5f * (float)A * LOG_2PI;
    float d_logp_m, d_v_m;
    RowTerms tm = ppo_row(a, logp_m, logp_old, adv, v_twin, v_old, ret, inv_rows, &d_logp_m, &d_v_m);
    acc.surr += tm.surr; acc.vloss += tm.vloss; acc.clipped += tm.clipped;
    *dv_twin = d_v_m;
    const float msc = a.mirror_coef * 2.0f / ((float)a.mb * (float)A);
#pragma unroll
    for (int jj = 0; jj < AM; ++jj) {
      if (jj < A) {
        const float target = a.sign_act[jj] * mu_row[a.perm_act[jj]];
        const float diff = mum[jj] - target;
        acc.mirror += diff * diff;
        dmu_twin[jj] = d_logp_m * zm[jj] / sg[jj] + msc * diff;
        acc.dls[jj] += d_logp_m * (zm[jj] * zm[jj] - 1.0f);
      }
    }
  }
}

// Workgroup reduction of the partial sums: wavefront shuffle reduction, one LDS exchange, then thread c adds the
// wavefronts' values of component c and writes it to this block's slot.
template <int AM>
__device__ __forceinline__ void ppo_acc_reduce(const PpoAcc<AM>& acc, int A, double* block_out) {
  __shared__ double wpart[4][PPO_NPART_FIXED + AM];
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  auto put = [&](int c, float v) {
    double r = wave_sum((double)v);
    if (lane == 0) wpart[w][c] = r;
  };
  put(0, acc.surr); put(1, acc.vloss); put(2, acc.kl); put(3, acc.clipped); put(4, acc.mirror);
#pragma unroll
  for (int jj = 0; jj < AM; ++jj)
    if (jj < A) put(PPO_NPART_FIXED + jj, acc.dls[jj]);
  __syncthreads();
  const int ncomp = PPO_NPART_FIXED + A;
  if (threadIdx.x < ncomp)
    block_out[threadIdx.x] = wpart[0][threadIdx.x] + wpart[1][threadIdx.x] + wpart[2][threadIdx.x] + wpart[3][threadIdx.x];
}

template <int AM>
__global__ __launch_bounds__(256) void ppo_loss_kernel(const PpoLossArgs a) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  const int A = a.A;
  PpoAcc<AM> acc;
#pragma unroll
  for (int jj = 0; jj < AM; ++jj) acc.dls[jj] = 0.f;
  if (i < a.mb) {
    const long im = (long)i + a.mb;
    const bool sym = a.rows > a.mb;
    PpoRowIn<AM> in;
    ppo_row_load(a, i, in);
    ppo_loss_row(a, in, a.mu + (long)i * A, a.mu + im * A, a.v[i], sym ? a.v[im] : 0.f, a.d_mu + (long)i * A,
                 a.d_mu + im * A, a.d_v + i, a.d_v + im, acc);
  }
  ppo_acc_reduce(acc, A, a.partials + (long)blockIdx.x * (PPO_NPART_FIXED + A));
}

// ---- fused output layer + loss head + input gradient of the output layer --------------------------------------
// One workgroup owns 32 activation rows (32 minibatch rows, or 16 rows and their 16 mirrored twins): it loads the
// last hidden activations of actor and critic into LDS, applies both output layers (A + 1 dot products per row),
// evaluates the PPO loss terms, and back-propagates through the output layers into the pre-activation gradient of
// the last hidden layer.  Three launches and two passes over the activations collapse into one.
// Every phase spreads over all 256 lanes: global loads are issued together before the first one is used, the
// output-layer dot products are cut into 8 contraction ranges per row, the loss runs on (row, action component)
// pairs with the row sums taken through LDS in a fixed order, and the input gradient reads a row's d_mu with
// 16-byte broadcasts.
constexpr int HEAD_ROWS = 32;
constexpr int HEAD_KPARTS = 8;      // lanes that share one row's output-layer dot products (and: 256 / HEAD_ROWS)
constexpr int HEAD_PAD = 4;         // LDS row padding of the activations: rows stay 16-byte aligned, and the lanes
                                    // (row, part) of the output-layer phase spread evenly over the banks

// LDS plan (floats), shared by the kernel and the host-side size check.
struct HeadLds {
  int A4, gp;
  int ha, hc, wa, wc, mu, dmu, vv, dv, gat, pact, cst, dlp, scr, dls, total;
  // A4: padded number of action components = the kernel's template width (rows of W, mu, d_mu in LDS)
  __host__ __device__ HeadLds(int Ha, int Hc, int A, int AP) {
    A4 = AP;
    gp = (4 + 3 * A) | 1;
    int o = 0;
    auto take = [&](int n) { const int r = o; o += (n + 3) & ~3; return r; };
    ha = take(HEAD_ROWS * (Ha + HEAD_PAD));
    hc = take(HEAD_ROWS * (Hc + HEAD_PAD));
    wa = take(Ha * AP + AP);            // W rows padded with zeros to AP, then the bias
    wc = take(Hc + 1);
    mu = take(HEAD_ROWS * A4);
    dmu = take(HEAD_ROWS * A4);
    vv = take(HEAD_ROWS);
    dv = take(HEAD_ROWS);
    gat = take(HEAD_ROWS * gp);
    pact = take(A4);                    // mirror map of the action components
    cst = take(4 * A4);                 // per component: log_std, 1 / sigma, 1 / (2 sigma^2), mirror sign
    dlp = take(2 * HEAD_ROWS);          // d loss / d log-prob of the rows (and of their twins)
    scr = take(2 * A4 * HEAD_ROWS);     // squared standard scores of rows and twins
    dls = take(2 * A4);
    total = o;
  }
};

template <int AM>
__global__ __launch_bounds__(256) void ppo_head_kernel(const PpoHeadArgs h) {
  extern __shared__ float lds[];
  const PpoLossArgs& a = h.loss;
  const int A = a.A, Ha = h.Ha, Hc = h.Hc;
  const HeadLds L(Ha, Hc, A, AM);
  constexpr int A4 = AM;
  const int gp = L.gp;
  const bool sym = a.rows > a.mb;
  const int r_orig = sym ? HEAD_ROWS / 2 : HEAD_ROWS;
  const int i0 = blockIdx.x * r_orig;
  const int sa = Ha + HEAD_PAD, sc = Hc + HEAD_PAD;         // padded LDS row strides
  float* ha = lds + L.ha;
  float* hc = lds + L.hc;
  float* wa = lds + L.wa;
  float* wc = lds + L.wc;
  float* mu = lds + L.mu;
  float* dmu = lds + L.dmu;
  float* vv = lds + L.vv;
  float* dv = lds + L.dv;
  float* gat = lds + L.gat;       // [row][adv, ret, v_old, logp_old, actions[A], mu_old[A], sigma_old[A]]
  int* pact = reinterpret_cast<int*>(lds + L.pact);
  float* cst = lds + L.cst;
  float* dlp = lds + L.dlp;
  float* scr = lds + L.scr;
  float* dls_out = lds + L.dls;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  // local row lr -> activation row (twins live mb rows further down), or -1 past the minibatch
  auto grow = [&](int lr) -> long {
    const int o = lr < r_orig ? lr : lr - r_orig;
    if (i0 + o >= a.mb) return -1;
    return lr < r_orig ? (long)(i0 + o) : (long)a.mb + i0 + o;
  };

  // ---- phase 1: every global read of the block.  Order of issue = order of arrival as far as the wave's load
  //      counter can tell, so: the permutation entries of the rows this wave gathers (needed first, for the
  //      addresses of the gather), the output-layer weights (cached, short), the activations (the long HBM reads),
  //      then, once the permutation entries are there, the gathered rollout rows.  Each group is written to LDS in
  //      the same order, so no wait covers more than it has to. ----
  constexpr int GROWS = HEAD_ROWS / 4;                    // rows gathered per wave: r = wave + 4 i
  int gb[GROWS];
#pragma unroll
  for (int i = 0; i < GROWS; ++i) {
    const int r = wave + 4 * i;
    gb[i] = (r < r_orig && i0 + r < a.mb) ? a.idx[i0 + r] : -1;
  }
  constexpr int WROUND = 8;                               // weight loads in flight per lane
  const int w_elems = (Ha + 1) * AM;
  float wv[WROUND];
#pragma unroll
  for (int i = 0; i < WROUND; ++i) {                      // first round (all of W for A <= 12 at 128 hidden units)
    const int e = tid + 256 * i;
    const int k = e / AM, jj = e - k * AM;
    wv[i] = (e < w_elems && jj < A) ? h.w_a[k * A + jj] : 0.f;
  }
  constexpr int HP = 8;                                   // 16-byte pieces per lane and network (H <= 256)
  float4 ra[HP], rc[HP];
  const int pa = Ha >> 2, pc = Hc >> 2;                   // pieces per row (powers of two)
  const int sha = __ffs(pa) - 1, shc = __ffs(pc) - 1;
#pragma unroll
  for (int i = 0; i < HP; ++i) {
    const int e = tid + 256 * i;
    ra[i] = make_float4(0.f, 0.f, 0.f, 0.f);
    rc[i] = make_float4(0.f, 0.f, 0.f, 0.f);
    if (e < HEAD_ROWS * pa) {
      const long gr = grow(e >> sha);
      if (gr >= 0) ra[i] = *reinterpret_cast<const float4*>(h.h_a + gr * Ha + 4 * (e & (pa - 1)));
    }
    if (e < HEAD_ROWS * pc) {
      const long gr = grow(e >> shc);
      if (gr >= 0) rc[i] = *reinterpret_cast<const float4*>(h.h_c + gr * Hc + 4 * (e & (pc - 1)));
    }
  }
  // rollout rows, gathered through the permutation: wavefront w takes rows w, w + 4, ..; lanes run over the row
  // [adv, ret, v_old, logp_old, actions[A], mu_old[A], sigma_old[A]]; the loads of all 8 rows are in flight together
  const int gw = 4 + 3 * A;
  auto gather_src = [&](int c, const float*& src, int& stride, int& off) {
    stride = 1; off = 0;
    if (c < 4) {
      src = c == 0 ? a.adv : c == 1 ? a.returns : c == 2 ? a.v_old : a.logp_old;
    } else {
      const int q = (c - 4) / A;
      src = q == 0 ? a.actions : q == 1 ? a.mu_old : a.sigma_old;
      stride = A; off = (c - 4) - q * A;
    }
  };
  float gv[GROWS];
  {
    const float* src = a.adv; int stride = 1, off = 0;
    if (lane < gw) gather_src(lane, src, stride, off);
#pragma unroll
    for (int i = 0; i < GROWS; ++i) gv[i] = (lane < gw && gb[i] >= 0) ? src[(long)gb[i] * stride + off] : 0.f;
  }
#pragma unroll
  for (int i = 0; i < WROUND; ++i) {
    const int e = tid + 256 * i;
    if (e < w_elems) wa[e] = wv[i];
  }
  for (int e0 = 256 * WROUND; e0 < w_elems; e0 += 256 * WROUND) {   // wider heads: the rest of W, rows padded with zeros
#pragma unroll
    for (int i = 0; i < WROUND; ++i) {
      const int e = e0 + tid + 256 * i;
      const int k = e / AM, jj = e - k * AM;
      wv[i] = (e < w_elems && jj < A) ? h.w_a[k * A + jj] : 0.f;
    }
#pragma unroll
    for (int i = 0; i < WROUND; ++i) {
      const int e = e0 + tid + 256 * i;
      if (e < w_elems) wa[e] = wv[i];
    }
  }
  for (int e = tid; e < Hc + 1; e += 256) wc[e] = h.w_c[e];
  if (tid < A) {
    const float ls = a.log_std[tid];
    const float inv = expf(-ls);
    cst[4 * tid + 0] = ls; cst[4 * tid + 1] = inv; cst[4 * tid + 2] = 0.5f * inv * inv;
    cst[4 * tid + 3] = sym ? a.sign_act[tid] : 1.0f;
    pact[tid] = sym ? a.perm_act[tid] : tid;
  }
  for (int e = tid; e < HEAD_ROWS * A4; e += 256) dmu[e] = 0.f;    // also the padding the 16-byte reads touch
#pragma unroll
  for (int i = 0; i < HP; ++i) {
    const int e = tid + 256 * i;
    if (e < HEAD_ROWS * pa) {
      *reinterpret_cast<float4*>(ha + (e >> sha) * sa + 4 * (e & (pa - 1))) = ra[i];
    }
    if (e < HEAD_ROWS * pc) {
      *reinterpret_cast<float4*>(hc + (e >> shc) * sc + 4 * (e & (pc - 1))) = rc[i];
    }
  }
  if (lane < gw) {
#pragma unroll
    for (int i = 0; i < GROWS; ++i) {
      const int r = wave + 4 * i;
      if (r < r_orig) gat[r * gp + lane] = gv[i];
    }
  }
  for (int c = lane + 64; c < gw; c += 64) {              // more than 20 action components: the columns past the 64th
    const float* src; int stride, off;
    gather_src(c, src, stride, off);
#pragma unroll
    for (int i = 0; i < GROWS; ++i) gv[i] = gb[i] >= 0 ? src[(long)gb[i] * stride + off] : 0.f;
#pragma unroll
    for (int i = 0; i < GROWS; ++i) {
      const int r = wave + 4 * i;
      if (r < r_orig) gat[r * gp + c] = gv[i];
    }
  }
  __syncthreads();

  // ---- phase 2: output layers.  The 8 lanes (row, p) of a row take every 8th hidden unit each and form the
  //      A + 1 dot products over them; a butterfly over the 8 lanes adds the parts in a fixed order ----
  {
    const int p8 = lane & (HEAD_KPARTS - 1), row = wave * 8 + (lane >> 3);
    float acc[AM + 1];
#pragma unroll
    for (int jj = 0; jj <= AM; ++jj) acc[jj] = 0.f;
    // trip counts are uniform (the lane only shifts the start), so the loops carry no lane mask
#pragma unroll 4
    for (int i = 0; i < Ha / HEAD_KPARTS; ++i) {
      const int k = HEAD_KPARTS * i + p8;
      const float hv = ha[row * sa + k];
      const float4* wr = reinterpret_cast<const float4*>(wa + k * AM);
#pragma unroll
      for (int q = 0; q < AM / 4; ++q) {
        const float4 w4 = wr[q];
        acc[4 * q] += hv * w4.x; acc[4 * q + 1] += hv * w4.y; acc[4 * q + 2] += hv * w4.z; acc[4 * q + 3] += hv * w4.w;
      }
    }
#pragma unroll 4
    for (int i = 0; i < Hc / HEAD_KPARTS; ++i) {
      const int k = HEAD_KPARTS * i + p8;
      acc[AM] += hc[row * sc + k] * wc[k];
    }
    // butterfly over the 8 lanes of a row; all exchanges of a step are issued together
#pragma unroll
    for (int off = 1; off < HEAD_KPARTS; off <<= 1) {
      float t[AM + 1];
#pragma unroll
      for (int jj = 0; jj <= AM; ++jj) t[jj] = __shfl_xor(acc[jj], off, 64);
#pragma unroll
      for (int jj = 0; jj <= AM; ++jj) acc[jj] += t[jj];
    }
    if (p8 == 0) {
#pragma unroll
      for (int jj = 0; jj < AM; ++jj) mu[row * A4 + jj] = acc[jj] + wa[Ha * AM + jj];
      vv[row] = acc[AM] + wc[Hc];
    }
  }
  __syncthreads();

  // ---- phase 3: loss.  Lane (row, jg) handles components jg, jg + 8, .. of a row (and of its twin) ----
  constexpr int JPT = (AM + HEAD_KPARTS - 1) / HEAD_KPARTS;
  const int lr = tid & (HEAD_ROWS - 1), jg = tid >> 5;
  const bool row_ok = lr < r_orig && i0 + lr < a.mb;
  const int lt = lr + r_orig;                       // twin's local row (symmetry only)
  float* z2 = scr;                                  // [A4][32] rows, then [A4][32] twins
  float* z2m = scr + A4 * HEAD_ROWS;
  float zj[JPT], zmj[JPT], diffj[JPT];
  double kl_acc = 0.0, mir_acc = 0.0;
#pragma unroll
  for (int t = 0; t < JPT; ++t) {
    const int jj = jg + HEAD_KPARTS * t;
    zj[t] = 0.f; zmj[t] = 0.f; diffj[t] = 0.f;
    if (jj < A) {
      float zz = 0.f, zzm = 0.f;
      if (row_ok) {
        const float* gr = gat + lr * gp;
        const float ls = cst[4 * jj], inv = cst[4 * jj + 1], inv2 = cst[4 * jj + 2];
        const float act = gr[4 + jj], mo = gr[4 + A + jj], so = gr[4 + 2 * A + jj];
        const float m_ = mu[lr * A4 + jj];
        const float z = (act - m_) * inv;
        zj[t] = z; zz = z * z;
        kl_acc += (double)((ls - logf(so)) + (so * so + (mo - m_) * (mo - m_)) * inv2 - 0.5f);
        if (sym) {
          const float sgn = cst[4 * jj + 3];
          const int pj = pact[jj];
          const float am = sgn * gr[4 + pj];
          const float mm = mu[lt * A4 + jj];
          const float zm = (am - mm) * inv;
          zmj[t] = zm; zzm = zm * zm;
          const float target = sgn * mu[lr * A4 + pj];
          diffj[t] = mm - target;
          mir_acc += (double)(diffj[t] * diffj[t]);
        }
      }
      z2[jj * HEAD_ROWS + lr] = zz;
      if (sym) z2m[jj * HEAD_ROWS + lr] = zzm;
    }
  }
  __syncthreads();
  double surr_acc = 0.0, vl_acc = 0.0, clip_acc = 0.0;
  if (tid < HEAD_ROWS) {
    float dl = 0.f, dlm = 0.f;
    if (row_ok) {
      const float* gr = gat + lr * gp;
      const float inv_rows = 1.0f / (float)a.rows;
      float zz = 0.f, zzm = 0.f, sum_ls = 0.f;
      for (int jj = 0; jj < A; ++jj) {
        zz += z2[jj * HEAD_ROWS + lr];
        if (sym) zzm += z2m[jj * HEAD_ROWS + lr];
        sum_ls += cst[4 * jj];
      }
      const float cl = sum_ls + 0.5f * (float)A * LOG_2PI;
      float d_v;
      RowTerms t = ppo_row(a, -0.5f * zz - cl, gr[3], gr[0], vv[lr], gr[2], gr[1], inv_rows, &dl, &d_v);
      surr_acc = t.surr; vl_acc = t.vloss; clip_acc = t.clipped;
      dv[lr] = d_v;
      if (sym) {
        float d_vm;
        RowTerms tm = ppo_row(a, -0.5f * zzm - cl, gr[3], gr[0], vv[lt], gr[2], gr[1], inv_rows, &dlm, &d_vm);
        surr_acc += tm.surr; vl_acc += tm.vloss; clip_acc += tm.clipped;
        dv[lt] = d_vm;
      }
    } else if (lr < r_orig) {
      dv[lr] = 0.f;
      if (sym) dv[lt] = 0.f;
    }
    dlp[lr] = dl;
    dlp[HEAD_ROWS + lr] = dlm;
  }
  __syncthreads();
  {
    const float dl = dlp[lr], dlm = dlp[HEAD_ROWS + lr];
    const float msc = sym ? a.mirror_coef * 2.0f / ((float)a.mb * (float)A) : 0.f;
#pragma unroll
    for (int t = 0; t < JPT; ++t) {
      const int jj = jg + HEAD_KPARTS * t;
      double g = 0.0;
      if (jj < A && lr < r_orig) {
        const float inv = cst[4 * jj + 1];
        dmu[lr * A4 + jj] = dl * zj[t] * inv;
        float gl = dl * (zj[t] * zj[t] - 1.0f);
        if (sym) {
          dmu[lt * A4 + jj] = dlm * zmj[t] * inv + msc * diffj[t];
          gl += dlm * (zmj[t] * zmj[t] - 1.0f);
        }
        g = row_ok ? (double)gl : 0.0;
      }
      // lanes of a half-wavefront share jj and run over the rows: sum them, one value per component
      for (int off = 16; off > 0; off >>= 1) g += __shfl_xor(g, off, 64);
      if ((lane & 31) == 0 && jj < A) reinterpret_cast<double*>(dls_out)[jj] = g;
    }
  }
  {
    __shared__ double wpart[4][PPO_NPART_FIXED];
    const double v5[PPO_NPART_FIXED] = {surr_acc, vl_acc, kl_acc, clip_acc, mir_acc};
#pragma unroll
    for (int c = 0; c < PPO_NPART_FIXED; ++c) {
      const double r = wave_sum(v5[c]);
      if (lane == 0) wpart[wave][c] = r;
    }
    __syncthreads();
    double* block_out = a.partials + (long)blockIdx.x * (PPO_NPART_FIXED + A);
    if (tid < PPO_NPART_FIXED) block_out[tid] = wpart[0][tid] + wpart[1][tid] + wpart[2][tid] + wpart[3][tid];
    else if (tid < PPO_NPART_FIXED + A) block_out[tid] = reinterpret_cast<const double*>(dls_out)[tid - PPO_NPART_FIXED];
  }

  // ---- phase 4: output-layer gradients for the weight-gradient contraction (d_mu, d_v to global memory) ----
  for (int e = tid; e < HEAD_ROWS * A; e += 256) {
    const int r = e / A, jj = e - r * A;
    const long gr = grow(r);
    if (gr >= 0) a.d_mu[gr * A + jj] = dmu[r * A4 + jj];
  }
  if (tid < HEAD_ROWS) {
    const long gr = grow(tid);
    if (gr >= 0) a.d_v[gr] = dv[tid];
  }
  // ---- input gradient of the output layers, times ELU'(h): lane = hidden unit, its weight row in registers, a
  //      row's d_mu read with 16-byte broadcasts ----
  {
    const int k = tid % Ha, rstep = 256 / Ha;
    float wrow[AM];
#pragma unroll
    for (int q = 0; q < AM / 4; ++q) {
      const float4 w4 = *reinterpret_cast<const float4*>(wa + k * AM + 4 * q);
      wrow[4 * q] = w4.x; wrow[4 * q + 1] = w4.y; wrow[4 * q + 2] = w4.z; wrow[4 * q + 3] = w4.w;
    }
#pragma unroll 4
    for (int i = 0; i < HEAD_ROWS / rstep; ++i) {      // uniform trip count; the lane only shifts the first row
      const int r = tid / Ha + i * rstep;
      const long gr = grow(r);
      if (gr < 0) continue;
      float s = 0.f;
#pragma unroll
      for (int q = 0; q < AM / 4; ++q) {
        const float4 d = *reinterpret_cast<const float4*>(dmu + r * A4 + 4 * q);
        s += d.x * wrow[4 * q] + d.y * wrow[4 * q + 1] + d.z * wrow[4 * q + 2] + d.w * wrow[4 * q + 3];
      }
      const float hv = ha[r * sa + k];
      h.dz_a[gr * Ha + k] = s * (hv > 0.f ? 1.0f : hv + h.alpha_a);
    }
  }
  {
    const int k = tid % Hc, rstep = 256 / Hc;
    const float wk = wc[k];
#pragma unroll 4
    for (int i = 0; i < HEAD_ROWS / rstep; ++i) {
      const int r = tid / Hc + i * rstep;
      const long gr = grow(r);
      if (gr < 0) continue;
      const float hv = hc[r * sc + k];
      h.dz_c[gr * Hc + k] = dv[r] * wk * (hv > 0.f ? 1.0f : hv + h.alpha_c);
    }
  }
}

static int head_width(int A) { return A <= 4 ? 4 : A <= 8 ? 8 : A <= 12 ? 12 : A <= 16 ? 16 : 32; }

size_t ppo_head_lds_bytes(int32_t Ha, int32_t Hc, int32_t A) {
  return sizeof(float) * (size_t)HeadLds(Ha, Hc, A, head_width(A)).total;
}

bool ppo_head_supported(int32_t Ha, int32_t Hc, int32_t A) {
  auto ok = [](int h) { return h == 32 || h == 64 || h == 128 || h == 256; };
  return ok(Ha) && ok(Hc) && A >= 1 && A <= 32 && ppo_head_lds_bytes(Ha, Hc, A) <= 150 * 1024;
}

int ppo_head_num_blocks(int32_t mb, bool sym) { const int r = sym ? HEAD_ROWS / 2 : HEAD_ROWS; return (mb + r - 1) / r; }

template <int AM>
static hipError_t launch_ppo_head_width(const PpoHeadArgs& h, size_t lds_bytes, hipStream_t stream) {
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(ppo_head_kernel<AM>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, 150 * 1024);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  const dim3 grid(ppo_head_num_blocks(h.loss.mb, h.loss.rows > h.loss.mb));
  hipLaunchKernelGGL(ppo_head_kernel<AM>, grid, dim3(256), lds_bytes, stream, h);
  return hipGetLastError();
}

hipError_t launch_ppo_head(const PpoHeadArgs& h, hipStream_t stream) {
  const size_t lds_bytes = ppo_head_lds_bytes(h.Ha, h.Hc, h.loss.A);
  TraceScope ts(stream, "ppo_head", 0.0, 0.0);
  switch (head_width(h.loss.A)) {
    case 4: return launch_ppo_head_width<4>(h, lds_bytes, stream);
    case 8: return launch_ppo_head_width<8>(h, lds_bytes, stream);
    case 12: return launch_ppo_head_width<12>(h, lds_bytes, stream);
    case 16: return launch_ppo_head_width<16>(h, lds_bytes, stream);
    default: return launch_ppo_head_width<32>(h, lds_bytes, stream);
  }
}

hipError_t launch_ppo_loss(const PpoLossArgs& a, hipStream_t stream) {
  TraceScope ts(stream, "ppo_loss", 0.0, 0.0);
  // the widest variant keeps a row's per-component values in per-lane scratch memory: correct, and only reached by
  // action vectors wider than any locomotion or manipulation task of the paper uses
  if (a.A <= 16) hipLaunchKernelGGL(ppo_loss_kernel<16>, dim3(ppo_loss_num_blocks(a.mb)), dim3(256), 0, stream, a);
  else if (a.A <= AMAX) hipLaunchKernelGGL(ppo_loss_kernel<AMAX>, dim3(ppo_loss_num_blocks(a.mb)), dim3(256), 0, stream, a);
  else hipLaunchKernelGGL(ppo_loss_kernel<64>, dim3(ppo_loss_num_blocks(a.mb)), dim3(256), 0, stream, a);
  return hipGetLastError();
}

// ---- MSE head -----------------------------------------------------------------------------------------
int mse_num_blocks(int64_t n) { return (int)((n + 1023) / 1024); }

__global__ __launch_bounds__(256) void mse_kernel(const float* __restrict__ y, const float* __restrict__ target,
                                                  const int32_t* __restrict__ target_idx, int rows, int width,
                                                  float* __restrict__ d_y, double* __restrict__ partials) {
  __shared__ double smem[4];
  const long n = (long)rows * width;
  const float sc = 2.0f / (float)n;
  const long i0 = ((long)blockIdx.x * 256 + threadIdx.x) * 4;
  double q = 0.0;
#pragma unroll
  for (int c = 0; c < 4; ++c) {
    const long i = i0 + c;
    if (i < n) {
      const long r = i / width;
      const long col = i - r * width;
      const long tr = target_idx ? (long)target_idx[r] : r;
      const float d = y[i] - target[tr * width + col];
      d_y[i] = sc * d;
      q += (double)d * (double)d;
    }
  }
  double t = block_sum(q, smem);
  if (threadIdx.x == 0) partials[blockIdx.x] = t;
}

hipError_t launch_mse(const float* y, const float* target, const int32_t* target_idx, int32_t rows, int32_t width,
                      float* d_y, double* partials, hipStream_t stream) {
  const int64_t n = (int64_t)rows * width;
  hipLaunchKernelGGL(mse_kernel, dim3(mse_num_blocks(n)), dim3(256), 0, stream, y, target, target_idx, rows, width, d_y,
                     partials);
  return hipGetLastError();
}

__global__ __launch_bounds__(256) void mse_finish_kernel(const double* __restrict__ partials, int blocks, long count,
                                                         float* __restrict__ stat_out) {
  __shared__ double smem[4];
  double s = 0.0;
  for (int i = threadIdx.x; i < blocks; i += 256) s += partials[i];
  double t = block_sum(s, smem);
  if (threadIdx.x == 0) *stat_out = (float)(t / (double)count);
}

hipError_t launch_mse_finish(const double* partials, int32_t blocks, int64_t count, float* stat_out, hipStream_t stream) {
  hipLaunchKernelGGL(mse_finish_kernel, dim3(1), dim3(256), 0, stream, partials, blocks, (long)count, stat_out);
  return hipGetLastError();
}

// ---- symmetry augmentation ----------------------------------------------------------------------------
__global__ __launch_bounds__(256) void sym_augment_kernel(const float* __restrict__ in, long B, int D,
                                                          const int32_t* __restrict__ perm, const float* __restrict__ sign,
                                                          float* __restrict__ out) {
  const long i = (long)blockIdx.x * 256 + threadIdx.x;
  const long n = B * D;
  if (i >= n) return;
  const long r = i / D;
  const int jj = (int)(i - r * D);
  out[i] = in[i];
  out[n + i] = sign[jj] * in[r * D + perm[jj]];
}

hipError_t launch_sym_augment(const float* in, int32_t B, int32_t D, const int32_t* perm, const float* sign, float* out,
                              hipStream_t stream) {
  const long n = (long)B * D;
  if (n <= 0) return hipSuccess;
  hipLaunchKernelGGL(sym_augment_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, stream, in, (long)B, D, perm,
                     sign, out);
  return hipGetLastError();
}

// One lane per group of four output columns (Dp is a multiple of four, out is 16-byte aligned).
__global__ __launch_bounds__(256) void stage_input_kernel(const float* __restrict__ in, int ld, long B, int D, int Dp,
                                                          const int32_t* __restrict__ perm, const float* __restrict__ sign,
                                                          float* __restrict__ out, long groups) {
  const long i = (long)blockIdx.x * 256 + threadIdx.x;
  if (i >= groups) return;
  const int q = Dp / 4;
  const long r = i / q;
  const int c0 = 4 * (int)(i - r * q);
  const bool mirrored = r >= B;
  const float* row = in + (mirrored ? r - B : r) * (long)ld;
  float v[4];
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    const int c = c0 + k;
    v[k] = 0.f;
    if (c < D) v[k] = mirrored ? sign[c] * row[perm[c]] : row[c];
  }
  *reinterpret_cast<float4*>(out + r * (long)Dp + c0) = make_float4(v[0], v[1], v[2], v[3]);
}

hipError_t launch_stage_input(const float* in, int32_t ld, int32_t B, int32_t D, int32_t Dp, const int32_t* perm,
                              const float* sign, float* out, hipStream_t stream) {
  const long groups = (long)B * (perm ? 2 : 1) * (Dp / 4);
  if (groups <= 0) return hipSuccess;
  TraceScope ts(stream, "stage_input", 0.0, 4.0 * (double)B * (perm ? 2 : 1) * (D + Dp));
  hipLaunchKernelGGL(stage_input_kernel, dim3((unsigned)((groups + 255) / 256)), dim3(256), 0, stream, in, ld, (long)B, D, Dp,
                     perm, sign, out, groups);
  return hipGetLastError();
}

// ---- RND reward ---------------------------------------------------------------------------------------
int rnd_num_blocks(int32_t N) { return (N + 255) / 256; }

__global__ __launch_bounds__(256) void rnd_raw_kernel(const float* __restrict__ yp, const float* __restrict__ yt, int N,
                                                      int K, float* __restrict__ raw, double* __restrict__ partials) {
  __shared__ double smem[4];
  const int n = blockIdx.x * 256 + threadIdx.x;
  double s = 0.0, q = 0.0;
  if (n < N) {
    float acc = 0.f;
    for (int k = 0; k < K; ++k) {
      const float d = yp[(long)n * K + k] - yt[(long)n * K + k];
      acc += d * d;
    }
    raw[n] = acc;
    s = (double)acc;
    q = s * s;
  }
  double ts = block_sum(s, smem);
  double tq = block_sum(q, smem);
  if (threadIdx.x == 0) {
    partials[2 * blockIdx.x] = ts;
    partials[2 * blockIdx.x + 1] = tq;
  }
}

// Single workgroup: batch moments, pairwise merge into running = {mean, var, count}, 1/sqrt(var + 1e-8).
__global__ __launch_bounds__(256) void rnd_stats_kernel(const double* __restrict__ partials, int blocks, int N,
                                                        float* __restrict__ running, int update,
                                                        float* __restrict__ inv_out) {
  __shared__ double smem[4];
  double s = 0.0, q = 0.0;
  for (int i = threadIdx.x; i < blocks; i += 256) {
    s += partials[2 * i];
    q += partials[2 * i + 1];
  }
  double ts = block_sum(s, smem);
  double tq = block_sum(q, smem);
  if (threadIdx.x == 0) {
    double mean = running[0], var = running[1], count = running[2];
    if (update) {
      const double nb = (double)N;
      const double mb = ts / nb;
      double vb = tq / nb - mb * mb;
      if (vb < 0.0) vb = 0.0;
      const double tot = count + nb;
      const double delta = mb - mean;
      const double m2 = var * count + vb * nb + delta * delta * count * nb / tot;
      mean = mean + delta * nb / tot;
      var = m2 / tot;
      count = tot;
      running[0] = (float)mean;
      running[1] = (float)var;
      running[2] = (float)count;
    }
    *inv_out = (float)(1.0 / sqrt(var + 1e-8));
  }
}

__global__ __launch_bounds__(256) void rnd_apply_kernel(float* __restrict__ r_int, int N, const float* __restrict__ inv,
                                                        float weight, float* __restrict__ rewards) {
  const int n = blockIdx.x * 256 + threadIdx.x;
  if (n >= N) return;
  const float r = r_int[n] * inv[0];
  r_int[n] = r;
  if (rewards != nullptr) rewards[n] += weight * r;
}

hipError_t launch_rnd_reward(const float* yp, const float* yt, int32_t N, int32_t K, float* running, float weight,
                             int32_t update_stats, float* r_int, float* rewards, double* partials, hipStream_t stream) {
  const int nb = rnd_num_blocks(N);
  float* inv = reinterpret_cast<float*>(partials + 2 * (size_t)nb);
  hipLaunchKernelGGL(rnd_raw_kernel, dim3(nb), dim3(256), 0, stream, yp, yt, N, K, r_int, partials);
  hipLaunchKernelGGL(rnd_stats_kernel, dim3(1), dim3(256), 0, stream, partials, nb, N, running, update_stats, inv);
  hipLaunchKernelGGL(rnd_apply_kernel, dim3(nb), dim3(256), 0, stream, r_int, N, inv, weight, rewards);
  return hipGetLastError();
}

}  // namespace rslx
