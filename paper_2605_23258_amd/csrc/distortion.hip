// Diagnostics.  Distortion of Section 4: E = sum over evicted tokens of w_i plus sum over
// approximated tokens of w_i * eps_i / ||v_i||^2, the mean relative error over the
// approximated set (1 - R^2_approx), and the quantities of Proposition 1.
//
//   distortion_partial_kernel : grid (chunks of 1024 tokens, kv heads), one thread per token
//                               (four tokens per thread).  Only approximated tokens read
//                               their value row (for ||v||^2).  Sums are kept in fp64 and
//                               leave the workgroup as one partial per chunk.
//   distortion_final_kernel   : one wave per head adds the partials in chunk order (so the
//                               result does not depend on scheduling) and derives the report.
#include "common.hpp"
#include "launch.hpp"

namespace vec {

namespace {

constexpr int kDistThreads = 256;
constexpr int kDistTokens = 1024;          // per workgroup
constexpr int kDistPartial = 8;            // doubles per partial

struct DistParams {
  const float* w; const uint8_t* tier; const float* eps; const void* v;
  int64_t v_sh, v_st;                      // element strides
  int n, n_chunks;
  double* part;                            // [Hkv, n_chunks, kDistPartial]
  double* out;                             // [Hkv, VECTOR_DISTORTION_FIELDS]
};

__device__ __forceinline__ double wave_sum_f64(double x) {
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) x += __shfl_xor(x, o, kWave);
  return x;
}
__device__ __forceinline__ double wave_max_f64(double x) {
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) x = fmax(x, __shfl_xor(x, o, kWave));
  return x;
}

template <typename T, int D>
__global__ __launch_bounds__(kDistThreads) void distortion_partial_kernel(DistParams p) {
  constexpr int E = Elem<T>::kPerChunk;
  __shared__ double red[kDistThreads / kWave][kDistPartial];
  const int h = blockIdx.y, chunk = blockIdx.x;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const T* v_head = reinterpret_cast<const T*>(p.v) + (int64_t)h * p.v_sh;
  double w_ev = 0.0, w_ap = 0.0, e_ap = 0.0, rel_sum = 0.0, n_ap = 0.0, n_ev = 0.0, w_ev_max = 0.0;
  for (int t = chunk * kDistTokens + threadIdx.x; t < min(p.n, (chunk + 1) * kDistTokens); t += kDistThreads) {
    const size_t at = (size_t)h * p.n + t;
    const int tr = p.tier[at];
    const double w = (double)p.w[at];
    if (tr == VECTOR_TIER_EVICT) {
      w_ev += w; n_ev += 1.0; w_ev_max = fmax(w_ev_max, w);
    } else if (tr == VECTOR_TIER_APPROX) {
      const T* row = v_head + (int64_t)t * p.v_st;
      float sq = 0.f;
#pragma unroll 4
      for (int c = 0; c < D / E; ++c) {
        float f[8];
        Unpack16<T>::run(load_chunk(row + c * E), f);
#pragma unroll
        for (int e = 0; e < E; ++e) sq = fmaf(f[e], f[e], sq);
      }
      const double rel = (double)p.eps[at] / (double)sq;
      w_ap += w; e_ap += w * rel; rel_sum += rel; n_ap += 1.0;
    }
  }
  const double vals[kDistPartial] = {wave_sum_f64(w_ev), wave_sum_f64(w_ap), wave_sum_f64(e_ap), wave_sum_f64(rel_sum),
                                     wave_sum_f64(n_ap), wave_sum_f64(n_ev), wave_max_f64(w_ev_max), 0.0};
  if (lane == 0)
#pragma unroll
    for (int i = 0; i < kDistPartial; ++i) red[wave][i] = vals[i];
  __syncthreads();
  if (threadIdx.x < kDistPartial) {
    double x = red[0][threadIdx.x];
    for (int wv = 1; wv < kDistThreads / kWave; ++wv) x = (threadIdx.x == 6) ? fmax(x, red[wv][threadIdx.x]) : x + red[wv][threadIdx.x];
    p.part[((size_t)h * p.n_chunks + chunk) * kDistPartial + threadIdx.x] = x;
  }
}

__global__ __launch_bounds__(kWave) void distortion_final_kernel(DistParams p) {
  const int h = blockIdx.x;
  if (threadIdx.x != 0) return;
  double s[kDistPartial] = {0, 0, 0, 0, 0, 0, 0, 0};
  for (int c = 0; c < p.n_chunks; ++c)
    for (int i = 0; i < kDistPartial; ++i) {
      const double x = p.part[((size_t)h * p.n_chunks + c) * kDistPartial + i];
      s[i] = (i == 6) ? fmax(s[i], x) : s[i] + x;
    }
  const double w_ev = s[0], w_ap = s[1], e_ap = s[2], rel_sum = s[3], n_ap = s[4], n_ev = s[5], w_ev_max = s[6];
  const double mu = n_ap > 0.0 ? rel_sum / n_ap : 0.0;
  const double pool_frac = ((double)p.n - n_ev) / (double)p.n;
  const double w_bar = (1.0 - w_ev) / pool_frac;
  const double w_star = (double)p.n * w_ev_max;
  double* o = p.out + (size_t)h * VECTOR_DISTORTION_FIELDS;
  o[0] = w_ev + e_ap; o[1] = w_ev; o[2] = w_ap; o[3] = mu; o[4] = 1.0 - mu; o[5] = w_bar; o[6] = w_star;
  o[7] = w_bar / (w_star + w_bar); o[8] = n_ap; o[9] = n_ev;
}

// ---------------------------------------------------------------------------
// R^2 of the value map on a token set (Section 3.1): residuals come from the residual kernel;
// here the totals.  r2_partial_kernel: grid (chunks of 1024 tokens, heads); thread j (and its
// partner j + D) accumulates sum v_j and sum v_j^2 over every other token of the chunk in
// fp64, the workgroup also sums the chunk's residuals.  r2_final_kernel adds the chunks in order.
// ---------------------------------------------------------------------------
struct R2Params {
  const float* eps; const void* v;
  int64_t v_sh, v_st;
  int n, n_chunks;
  double* part;                            // [Hkv, n_chunks, 2 D + 1]
  double* out;                             // [Hkv, VECTOR_R2_FIELDS]
};

template <typename T, int D>
__global__ __launch_bounds__(kDistThreads) void r2_partial_kernel(R2Params p) {
  static_assert(kDistThreads % D == 0, "token groups");
  constexpr int TG = kDistThreads / D;
  __shared__ double red[TG][2][D];
  __shared__ double eps_red[kDistThreads / kWave];
  const int h = blockIdx.y, chunk = blockIdx.x;
  const int j = threadIdx.x % D, tg = threadIdx.x / D;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const T* v_head = reinterpret_cast<const T*>(p.v) + (int64_t)h * p.v_sh;
  const int t_end = min(p.n, (chunk + 1) * kDistTokens);
  double s1 = 0.0, s2 = 0.0, se = 0.0;
  for (int t = chunk * kDistTokens + tg; t < t_end; t += TG) {
    const double x = (double)to_float(v_head[(int64_t)t * p.v_st + j]);
    s1 += x;
    s2 += x * x;
  }
  for (int t = chunk * kDistTokens + threadIdx.x; t < t_end; t += kDistThreads) se += (double)p.eps[(size_t)h * p.n + t];
  red[tg][0][j] = s1;
  red[tg][1][j] = s2;
  se = wave_sum_f64(se);
  if (lane == 0) eps_red[wave] = se;
  __syncthreads();
  double* out = p.part + ((size_t)h * p.n_chunks + chunk) * (2 * D + 1);
  if (threadIdx.x < 2 * D) {
    const int which = threadIdx.x / D, jj = threadIdx.x % D;
    double x = 0.0;
    for (int g = 0; g < TG; ++g) x += red[g][which][jj];
    out[which * D + jj] = x;
  }
  if (threadIdx.x == 0) {
    double x = 0.0;
    for (int wv = 0; wv < kDistThreads / kWave; ++wv) x += eps_red[wv];
    out[2 * D] = x;
  }
}

template <int D>
__global__ __launch_bounds__(2 * D) void r2_final_kernel(R2Params p) {
  __shared__ double tot[2][D];
  __shared__ double sse_lds;
  const int h = blockIdx.x;
  const int which = threadIdx.x / D, j = threadIdx.x % D;
  const double* part = p.part + (size_t)h * p.n_chunks * (2 * D + 1);
  double x = 0.0;
  for (int c = 0; c < p.n_chunks; ++c) x += part[(size_t)c * (2 * D + 1) + which * D + j];
  tot[which][j] = x;
  if (threadIdx.x == 0) {
    double e = 0.0;
    for (int c = 0; c < p.n_chunks; ++c) e += part[(size_t)c * (2 * D + 1) + 2 * D];
    sse_lds = e;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    double raw = 0.0, cen = 0.0;
    for (int d = 0; d < D; ++d) {
      raw += tot[1][d];
      cen += tot[1][d] - tot[0][d] * tot[0][d] / (double)p.n;
    }
    double* o = p.out + (size_t)h * VECTOR_R2_FIELDS;
    o[0] = 1.0 - sse_lds / cen; o[1] = 1.0 - sse_lds / raw; o[2] = sse_lds; o[3] = cen; o[4] = raw;
  }
}

}  // namespace

size_t r2_workspace_bytes(int n_kv_heads, int seq_len, int head_dim) {
  return align_up((size_t)n_kv_heads * seq_len * sizeof(float), 256) +
         align_up((size_t)n_kv_heads * ((seq_len + kDistTokens - 1) / kDistTokens) * (2 * head_dim + 1) * sizeof(double), 256);
}

// eps [Hkv, n] (already computed into the head of ws by the residual kernel) -> report
int launch_r2(const vector_shape& s, const float* eps, const void* v, double* out, void* part_ws, hipStream_t stream) {
  R2Params p;
  p.eps = eps; p.v = v; p.n = s.seq_len; p.out = out;
  p.v_st = s.v_stride_tok ? s.v_stride_tok : s.head_dim;
  p.v_sh = s.v_stride_head ? s.v_stride_head : (int64_t)s.seq_len * p.v_st;
  p.n_chunks = (s.seq_len + kDistTokens - 1) / kDistTokens;
  p.part = reinterpret_cast<double*>(part_ws);
  const dim3 grid(p.n_chunks, s.n_kv_heads);
  if (s.dtype == VECTOR_BF16 && s.head_dim == 128) hipLaunchKernelGGL((r2_partial_kernel<bf16_t, 128>), grid, dim3(kDistThreads), 0, stream, p);
  else if (s.dtype == VECTOR_BF16 && s.head_dim == 64) hipLaunchKernelGGL((r2_partial_kernel<bf16_t, 64>), grid, dim3(kDistThreads), 0, stream, p);
  else if (s.dtype == VECTOR_F32 && s.head_dim == 128) hipLaunchKernelGGL((r2_partial_kernel<float, 128>), grid, dim3(kDistThreads), 0, stream, p);
  else if (s.dtype == VECTOR_F32 && s.head_dim == 64) hipLaunchKernelGGL((r2_partial_kernel<float, 64>), grid, dim3(kDistThreads), 0, stream, p);
  else return s.dtype == VECTOR_BF16 || s.dtype == VECTOR_F32 ? VECTOR_ERR_SHAPE : VECTOR_ERR_DTYPE;
  if (s.head_dim == 128) hipLaunchKernelGGL(r2_final_kernel<128>, dim3(s.n_kv_heads), dim3(256), 0, stream, p);
  else hipLaunchKernelGGL(r2_final_kernel<64>, dim3(s.n_kv_heads), dim3(128), 0, stream, p);
  VEC_HIP(hipGetLastError());
  return VECTOR_OK;
}

size_t distortion_workspace_bytes(int n_kv_heads, int seq_len) {
  return align_up((size_t)n_kv_heads * ((seq_len + kDistTokens - 1) / kDistTokens) * kDistPartial * sizeof(double), 256);
}

int launch_distortion(const vector_shape& s, const float* w, const uint8_t* tier, const float* eps, const void* v,
                      double* out, void* ws, hipStream_t stream) {
  DistParams p;
  p.w = w; p.tier = tier; p.eps = eps; p.v = v; p.n = s.seq_len; p.out = out;
  p.v_st = s.v_stride_tok ? s.v_stride_tok : s.head_dim;
  p.v_sh = s.v_stride_head ? s.v_stride_head : (int64_t)s.seq_len * p.v_st;
  p.n_chunks = (s.seq_len + kDistTokens - 1) / kDistTokens;
  p.part = reinterpret_cast<double*>(ws);
  const dim3 grid(p.n_chunks, s.n_kv_heads);
  if (s.dtype == VECTOR_BF16 && s.head_dim == 128) hipLaunchKernelGGL((distortion_partial_kernel<bf16_t, 128>), grid, dim3(kDistThreads), 0, stream, p);
  else if (s.dtype == VECTOR_BF16 && s.head_dim == 64) hipLaunchKernelGGL((distortion_partial_kernel<bf16_t, 64>), grid, dim3(kDistThreads), 0, stream, p);
  else if (s.dtype == VECTOR_F32 && s.head_dim == 128) hipLaunchKernelGGL((distortion_partial_kernel<float, 128>), grid, dim3(kDistThreads), 0, stream, p);
  else if (s.dtype == VECTOR_F32 && s.head_dim == 64) hipLaunchKernelGGL((distortion_partial_kernel<float, 64>), grid, dim3(kDistThreads), 0, stream, p);
  else return s.dtype == VECTOR_BF16 || s.dtype == VECTOR_F32 ? VECTOR_ERR_SHAPE : VECTOR_ERR_DTYPE;
  hipLaunchKernelGGL(distortion_final_kernel, dim3(s.n_kv_heads), dim3(kWave), 0, stream, p);
  VEC_HIP(hipGetLastError());
  return VECTOR_OK;
}

}  // namespace vec
