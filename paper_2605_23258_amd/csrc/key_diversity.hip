// A query-agnostic importance score: the negative cosine of a key to the mean direction of
// its head's unit-normalised keys (a reading of the "key geometric diversity" scorers that
// Section 5 names without a formula).  Two streaming passes over K, both bound by HBM:
//   anchor_partial_kernel : grid (chunks of 512 tokens, kv heads).  A row is read by
//                           row_bytes/16 adjacent lanes; the row norm is a rotate-add across
//                           them; every lane accumulates its 16 bytes of k / ||k|| over the
//                           rows it sees; lanes, waves -> one partial sum per chunk.
//   diversity_score_kernel: sums the partials (in chunk order), normalises the anchor, and
//                           writes score[t] = - (k_t . a) / ||k_t||.
#include "common.hpp"
#include "launch.hpp"

namespace vec {

namespace {

constexpr int kDivThreads = 256;
constexpr int kDivTokens = 512;           // per workgroup
constexpr int kDivUnroll = 4;             // rows per lane group in flight

struct DivParams {
  const void* k;
  int64_t k_sh, k_st;
  int n, n_chunks;
  float* part;                            // [Hkv, n_chunks, d]
  float* score;                           // [Hkv, n]
};

template <int LPR> __device__ __forceinline__ float lanes_sum(float x) {
#pragma unroll
  for (int o = LPR / 2; o >= 1; o >>= 1) x += __shfl_xor(x, o, kWave);
  return x;
}

template <typename T, int D>
__global__ __launch_bounds__(kDivThreads) void anchor_partial_kernel(DivParams p) {
  constexpr int E = Elem<T>::kPerChunk;
  constexpr int LPR = D / E;               // lanes per row
  constexpr int RPW = kWave / LPR;         // rows per wave-wide load
  constexpr int NW = kDivThreads / kWave;
  __shared__ float red[NW][RPW][D];
  const int h = blockIdx.y, chunk = blockIdx.x;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int grp = lane / LPR, piece = lane % LPR;
  const T* k_head = reinterpret_cast<const T*>(p.k) + (int64_t)h * p.k_sh;
  const int t_end = min(p.n, (chunk + 1) * kDivTokens);
  float acc[E];
#pragma unroll
  for (int e = 0; e < E; ++e) acc[e] = 0.f;
  for (int t0 = chunk * kDivTokens + wave * RPW; t0 < t_end; t0 += NW * RPW * kDivUnroll) {
    uint4 raw[kDivUnroll];
#pragma unroll
    for (int u = 0; u < kDivUnroll; ++u)
      raw[u] = load_chunk(k_head + (int64_t)min(t0 + u * NW * RPW + grp, p.n - 1) * p.k_st + piece * E);
#pragma unroll
    for (int u = 0; u < kDivUnroll; ++u) {
      const int t = t0 + u * NW * RPW + grp;
      float f[8];
      Unpack16<T>::run(raw[u], f);
      float sq = 0.f;
#pragma unroll
      for (int e = 0; e < E; ++e) sq = fmaf(f[e], f[e], sq);
      sq = lanes_sum<LPR>(sq);
      const float inv = (t < t_end && sq > 0.f) ? 1.0f / sqrtf(sq) : 0.f;      // a zero key has no direction
#pragma unroll
      for (int e = 0; e < E; ++e) acc[e] = fmaf(f[e], inv, acc[e]);
    }
  }
#pragma unroll
  for (int e = 0; e < E; ++e) red[wave][grp][piece * E + e] = acc[e];
  __syncthreads();
  float* out = p.part + ((size_t)h * p.n_chunks + chunk) * D;
  for (int j = threadIdx.x; j < D; j += kDivThreads) {
    float s = 0.f;
#pragma unroll
    for (int wv = 0; wv < NW; ++wv)
#pragma unroll
      for (int g = 0; g < RPW; ++g) s += red[wv][g][j];
    out[j] = s;
  }
}

template <typename T, int D>
__global__ __launch_bounds__(kDivThreads) void diversity_score_kernel(DivParams p) {
  constexpr int E = Elem<T>::kPerChunk;
  constexpr int LPR = D / E;
  constexpr int RPW = kWave / LPR;
  constexpr int NW = kDivThreads / kWave;
  __shared__ float anchor[D];
  __shared__ float norm_lds;
  const int h = blockIdx.y, chunk = blockIdx.x;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int grp = lane / LPR, piece = lane % LPR;
  for (int j = threadIdx.x; j < D; j += kDivThreads) {
    float s = 0.f;
    for (int c = 0; c < p.n_chunks; ++c) s += p.part[((size_t)h * p.n_chunks + c) * D + j];
    anchor[j] = s;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    float sq = 0.f;
    for (int j = 0; j < D; ++j) sq = fmaf(anchor[j], anchor[j], sq);
    norm_lds = sq > 0.f ? 1.0f / sqrtf(sq) : 0.f;
  }
  __syncthreads();
  float a[E];
#pragma unroll
  for (int e = 0; e < E; ++e) a[e] = anchor[piece * E + e] * norm_lds;
  const T* k_head = reinterpret_cast<const T*>(p.k) + (int64_t)h * p.k_sh;
  const int t_end = min(p.n, (chunk + 1) * kDivTokens);
  for (int t0 = chunk * kDivTokens + wave * RPW; t0 < t_end; t0 += NW * RPW * kDivUnroll) {
    uint4 raw[kDivUnroll];
#pragma unroll
    for (int u = 0; u < kDivUnroll; ++u)
      raw[u] = load_chunk(k_head + (int64_t)min(t0 + u * NW * RPW + grp, p.n - 1) * p.k_st + piece * E);
#pragma unroll
    for (int u = 0; u < kDivUnroll; ++u) {
      const int t = t0 + u * NW * RPW + grp;
      float f[8];
      Unpack16<T>::run(raw[u], f);
      float sq = 0.f, dot = 0.f;
#pragma unroll
      for (int e = 0; e < E; ++e) { sq = fmaf(f[e], f[e], sq); dot = fmaf(f[e], a[e], dot); }
      sq = lanes_sum<LPR>(sq);
      dot = lanes_sum<LPR>(dot);
      if (piece == 0 && t < t_end) p.score[(size_t)h * p.n + t] = sq > 0.f ? -dot / sqrtf(sq) : 0.f;
    }
  }
}

template <typename T, int D>
int run_diversity(const vector_shape& s, DivParams& p, hipStream_t stream) {
  const dim3 grid(p.n_chunks, s.n_kv_heads);
  hipLaunchKernelGGL((anchor_partial_kernel<T, D>), grid, dim3(kDivThreads), 0, stream, p);
  hipLaunchKernelGGL((diversity_score_kernel<T, D>), grid, dim3(kDivThreads), 0, stream, p);
  VEC_HIP(hipGetLastError());
  return VECTOR_OK;
}

}  // namespace

size_t diversity_workspace_bytes(const vector_shape& s) {
  return align_up((size_t)s.n_kv_heads * ((s.seq_len + kDivTokens - 1) / kDivTokens) * s.head_dim * sizeof(float), 256);
}

int launch_key_diversity(const vector_shape& s, const void* k, float* score, void* ws, hipStream_t stream) {
  DivParams p;
  p.k = k; p.n = s.seq_len; p.score = score; p.part = reinterpret_cast<float*>(ws);
  p.k_st = s.k_stride_tok ? s.k_stride_tok : s.head_dim;
  p.k_sh = s.k_stride_head ? s.k_stride_head : (int64_t)s.seq_len * p.k_st;
  p.n_chunks = (s.seq_len + kDivTokens - 1) / kDivTokens;
  if (s.dtype == VECTOR_BF16) {
    if (s.head_dim == 128) return run_diversity<bf16_t, 128>(s, p, stream);
    if (s.head_dim == 64) return run_diversity<bf16_t, 64>(s, p, stream);
  } else if (s.dtype == VECTOR_F32) {
    if (s.head_dim == 128) return run_diversity<float, 128>(s, p, stream);
    if (s.head_dim == 64) return run_diversity<float, 64>(s, p, stream);
  } else {
    return VECTOR_ERR_DTYPE;
  }
  return VECTOR_ERR_SHAPE;
}

}  // namespace vec
