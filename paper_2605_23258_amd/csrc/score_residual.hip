// Importance score (observation-window attention mass, pooled) and
// reconstruction residual ||v - k W||^2 for the VECTOR compression pass
// (Section 3.2, Steps 1 and 2).
//
// Data flow per KV head h (R = G*w query rows share the head's keys):
//   pass 1  score_stats   : S = Q_h K_h^T (MFMA), per-row running max / sum-exp
//                           over a chunk of tokens -> partial (m, l) per chunk
//   combine stats_combine : merge the chunks -> one bias per row,
//                           bias_r = log2-domain max + log2(sum-exp)
//   pass 2  mass_residual : S again, p = exp2(S*c - bias_r), column mean -> mass;
//                           fused on the same K registers: v_hat = K W (MFMA),
//                           eps = sum_j (v - v_hat)^2
//   pool    pool_scores   : average pooling of mass over prefix columns, +inf on
//                           the window columns
//
// K rows go straight from HBM into MFMA operand registers (16 bytes per lane);
// Q_h, W_h^T and the row biases live in LDS for the life of a workgroup.
#include "common.hpp"
#include "launch.hpp"

namespace vec {

namespace {

struct PassParams {
  const void* q;        // [Hq, w, d]
  const void* k;
  const void* v;
  const void* W;
  int64_t k_sh, k_st, v_sh, v_st, w_sh;   // element strides
  int n, w, R, R_pad, n_prefix;
  int tokens_per_chunk, n_chunks;
  float c2;             // log2(e) / sqrt(d)
  float inv_R;
  float2* part;         // [Hkv, n_chunks, R_pad]  (max, sum-exp), log2 domain
  float* bias;          // [Hkv, R_pad]
  float* mass;          // [Hkv, n]
  float* eps;           // [Hkv, n]
};

template <typename T, int D> struct Tile {
  static constexpr int E = Elem<T>::kPerChunk;
  static constexpr int NC = D / (2 * E);            // chunks per row
  static constexpr int kRowBytes = D * (int)sizeof(T);
  static constexpr int kLdsStride = kRowBytes + 16;  // pad: conflict-free 16-byte reads down a column of rows
  static constexpr int JB = D / 32;                  // 32-column blocks of the K W product
};

// Copy `rows` rows of D elements from global to LDS with the padded stride;
// rows in [rows, rows_pad) are zero-filled.
template <typename T, int D, int NT>
__device__ __forceinline__ void fill_rows_lds(unsigned char* lds, const T* src, int rows, int rows_pad) {
  constexpr int P = Tile<T, D>::kRowBytes / 16;
  for (int i = threadIdx.x; i < rows_pad * P; i += NT) {
    int row = i / P, piece = i - row * P;
    uint4 x = make_uint4(0, 0, 0, 0);
    if (row < rows) x = *reinterpret_cast<const uint4*>(reinterpret_cast<const unsigned char*>(src) + (size_t)row * Tile<T, D>::kRowBytes + piece * 16);
    *reinterpret_cast<uint4*>(lds + row * Tile<T, D>::kLdsStride + piece * 16) = x;
  }
}

template <typename T, int D>
__device__ __forceinline__ chunk_t lds_chunk(const unsigned char* lds, int row, int c, int half) {
  return *reinterpret_cast<const chunk_t*>(lds + row * Tile<T, D>::kLdsStride + chunk_elem_offset<T>(c, half) * (int)sizeof(T));
}

// K operand registers of a 32-token subtile: lane (l & 31) holds token t0 + (l & 31).
template <typename T, int D>
__device__ __forceinline__ void load_k_subtile(chunk_t* kf, const T* k_head, int64_t k_st, int t0, int n, int lane) {
  int t = min(t0 + (lane & 31), n - 1);
  const T* row = k_head + (int64_t)t * k_st;
#pragma unroll
  for (int c = 0; c < Tile<T, D>::NC; ++c) kf[c] = load_chunk(row + chunk_elem_offset<T>(c, lane >> 5));
}

// ---------------------------------------------------------------------------
// pass 1: per-row softmax statistics over a chunk of tokens
// ---------------------------------------------------------------------------
template <typename T, int D, int NT>
__global__ __launch_bounds__(NT) void score_stats_kernel(PassParams p) {
  using TL = Tile<T, D>;
  constexpr int NW = NT / kWave;
  extern __shared__ __align__(16) unsigned char smem[];
  unsigned char* q_lds = smem;
  float2* st_lds = reinterpret_cast<float2*>(smem + (size_t)p.R_pad * TL::kLdsStride);   // [NW][NRB][64]

  const int h = blockIdx.y, chunk = blockIdx.x;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, half = lane >> 5, l31 = lane & 31;
  const int nrb = p.R_pad / 32;

  fill_rows_lds<T, D, NT>(q_lds, reinterpret_cast<const T*>(p.q) + (size_t)h * p.R * D, p.R, p.R_pad);
  for (int i = threadIdx.x; i < NW * nrb * 64; i += NT) st_lds[i] = make_float2(-INFINITY, 0.f);
  __syncthreads();

  const T* k_head = reinterpret_cast<const T*>(p.k) + (int64_t)h * p.k_sh;
  const int c_begin = chunk * p.tokens_per_chunk;
  const int c_end = min(p.n, c_begin + p.tokens_per_chunk);
  float2* my_st = st_lds + (size_t)wave * nrb * 64 + lane;

  for (int t0 = c_begin + wave * 64; t0 < c_end; t0 += NW * 64) {
    chunk_t kf0[TL::NC], kf1[TL::NC];
    load_k_subtile<T, D>(kf0, k_head, p.k_st, t0, p.n, lane);
    load_k_subtile<T, D>(kf1, k_head, p.k_st, t0 + 32, p.n, lane);
    // a tile needs masking if it reaches past the first window position or past the chunk
    const bool tail = (t0 + 64 > p.n_prefix + 1) || (t0 + 64 > c_end);
    for (int rb = 0; rb < nrb; ++rb) {
      f32x16 a0 = {0}, a1 = {0};
#pragma unroll
      for (int c = 0; c < TL::NC; ++c) {
        chunk_t qf = lds_chunk<T, D>(q_lds, rb * 32 + l31, c, half);
        mma_chunk<T>(a0, kf0[c], qf);     // rows = tokens, columns = query rows
        mma_chunk<T>(a1, kf1[c], qf);
      }
      float x0[16], x1[16];
#pragma unroll
      for (int v = 0; v < 16; ++v) { x0[v] = a0[v] * p.c2; x1[v] = a1[v] * p.c2; }
      if (tail) {
        // query row (g, r) sits at position n - w + r and sees tokens <= that
        const int qrow = rb * 32 + l31;
        const int last = (qrow < p.R) ? min(p.n_prefix + (qrow % p.w), c_end - 1) : c_end - 1;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          int t = t0 + acc_row(v, half);
          if (t > last) x0[v] = -INFINITY;
          if (t + 32 > last) x1[v] = -INFINITY;
        }
      }
      float tmax = fmaxf(x0[0], x1[0]);
#pragma unroll
      for (int v = 1; v < 16; ++v) tmax = fmaxf(tmax, fmaxf(x0[v], x1[v]));
      float2 st = my_st[rb * 64];
      const float m_new = fmaxf(st.x, tmax);
      const float m_safe = (m_new == -INFINITY) ? 0.f : m_new;
      float sum = 0.f;
#pragma unroll
      for (int v = 0; v < 16; ++v) sum += fast_exp2(x0[v] - m_safe) + fast_exp2(x1[v] - m_safe);
      st.y = st.y * fast_exp2(st.x - m_safe) + sum;
      st.x = m_new;
      my_st[rb * 64] = st;
    }
  }
  __syncthreads();
  // merge the NW waves x 2 lane halves that saw different tokens of the same query row
  float2* out = p.part + ((size_t)h * p.n_chunks + chunk) * p.R_pad;
  for (int row = threadIdx.x; row < p.R_pad; row += NT) {
    const int rb = row >> 5, c = row & 31;
    float m = -INFINITY;
    for (int wv = 0; wv < NW; ++wv)
      for (int hf = 0; hf < 2; ++hf) m = fmaxf(m, st_lds[((size_t)wv * nrb + rb) * 64 + hf * 32 + c].x);
    const float m_safe = (m == -INFINITY) ? 0.f : m;
    float l = 0.f;
    for (int wv = 0; wv < NW; ++wv)
      for (int hf = 0; hf < 2; ++hf) {
        float2 s = st_lds[((size_t)wv * nrb + rb) * 64 + hf * 32 + c];
        l += s.y * fast_exp2(s.x - m_safe);
      }
    out[row] = make_float2(m, l);
  }
}

// merge chunk partials into one bias per query row
__global__ void stats_combine_kernel(PassParams p) {
  const int h = blockIdx.y;
  const int row = blockIdx.x * blockDim.x + threadIdx.x;
  if (row >= p.R_pad) return;
  const float2* part = p.part + (size_t)h * p.n_chunks * p.R_pad + row;
  float m = -INFINITY;
  for (int c = 0; c < p.n_chunks; ++c) m = fmaxf(m, part[(size_t)c * p.R_pad].x);
  float l = 0.f;
  for (int c = 0; c < p.n_chunks; ++c) {
    float2 s = part[(size_t)c * p.R_pad];
    l += s.y * fast_exp2(s.x - m);
  }
  // padded rows get +inf so that they add exp2(-inf) = 0 to every column
  p.bias[(size_t)h * p.R_pad + row] = (row < p.R) ? m + __builtin_amdgcn_logf(l) : INFINITY;
}

// ---------------------------------------------------------------------------
// pass 2: column mass of the normalised probabilities, and/or the residual
// ---------------------------------------------------------------------------
// Raw bits of the JB consecutive value elements a lane compares against its accumulator
// column block; element i is extracted by shifting so that i may be a run-time value.
template <int BYTES> struct RawVec;
template <> struct RawVec<4>  { uint32_t x; };
template <> struct RawVec<8>  { uint64_t x; };
template <> struct RawVec<16> { uint64_t lo, hi; };
template <int BYTES> __device__ __forceinline__ RawVec<BYTES> load_raw(const void* p);
template <> __device__ __forceinline__ RawVec<4> load_raw<4>(const void* p) { return RawVec<4>{*reinterpret_cast<const uint32_t*>(p)}; }
template <> __device__ __forceinline__ RawVec<8> load_raw<8>(const void* p) { return RawVec<8>{*reinterpret_cast<const uint64_t*>(p)}; }
template <> __device__ __forceinline__ RawVec<16> load_raw<16>(const void* p) {
  uint4 x = *reinterpret_cast<const uint4*>(p);
  return RawVec<16>{((uint64_t)x.y << 32) | x.x, ((uint64_t)x.w << 32) | x.z};
}
template <typename T, int BYTES> __device__ __forceinline__ float raw_elem(const RawVec<BYTES>& r, int i);
template <> __device__ __forceinline__ float raw_elem<float, 8>(const RawVec<8>& r, int i) { return __uint_as_float((uint32_t)(r.x >> (32 * i))); }
template <> __device__ __forceinline__ float raw_elem<float, 16>(const RawVec<16>& r, int i) {
  uint64_t y = (i & 2) ? r.hi : r.lo;
  return __uint_as_float((uint32_t)(y >> (32 * (i & 1))));
}
template <> __device__ __forceinline__ float raw_elem<bf16_t, 4>(const RawVec<4>& r, int i) { return __uint_as_float((r.x >> (16 * i)) << 16); }
template <> __device__ __forceinline__ float raw_elem<bf16_t, 8>(const RawVec<8>& r, int i) { return __uint_as_float(((uint32_t)(r.x >> (16 * i))) << 16); }

template <typename T, int D, int NT, bool DO_MASS, bool DO_RES>
__global__ __launch_bounds__(NT) void mass_residual_kernel(PassParams p) {
  using TL = Tile<T, D>;
  constexpr int NW = NT / kWave;
  constexpr int JB = TL::JB;
  extern __shared__ __align__(16) unsigned char smem[];
  unsigned char* q_lds = smem;                                               // DO_MASS: [R_pad] rows
  size_t off = DO_MASS ? (size_t)p.R_pad * TL::kLdsStride : 0;
  float* bias_lds = reinterpret_cast<float*>(smem + off);                    // DO_MASS: [R_pad]
  off += DO_MASS ? (size_t)p.R_pad * sizeof(float) : 0;
  unsigned char* wt_lds = smem + off;                                        // DO_RES: [D] rows of W^T, permuted

  const int h = blockIdx.y, chunk = blockIdx.x;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, half = lane >> 5, l31 = lane & 31;
  const int nrb = p.R_pad / 32;

  if (DO_MASS) {
    fill_rows_lds<T, D, NT>(q_lds, reinterpret_cast<const T*>(p.q) + (size_t)h * p.R * D, p.R, p.R_pad);
    for (int i = threadIdx.x; i < p.R_pad; i += NT) bias_lds[i] = p.bias[(size_t)h * p.R_pad + i];
  }
  if (DO_RES) {
    // W^T into LDS: output column j = nn*JB + jb is stored as physical row jb*32 + nn, so
    // that the 32 lanes of an MFMA operand read 32 consecutive padded rows.
    const T* Wh = reinterpret_cast<const T*>(p.W) + (int64_t)h * p.w_sh;
    for (int i = threadIdx.x; i < D * D; i += NT) {
      int din = i / D, j = i - din * D;
      int prow = (j % JB) * 32 + j / JB;
      *reinterpret_cast<T*>(wt_lds + prow * TL::kLdsStride + din * (int)sizeof(T)) = Wh[i];
    }
  }
  __syncthreads();

  const T* k_head = reinterpret_cast<const T*>(p.k) + (int64_t)h * p.k_sh;
  const T* v_head = DO_RES ? reinterpret_cast<const T*>(p.v) + (int64_t)h * p.v_sh : nullptr;
  const int c_begin = chunk * p.tokens_per_chunk;
  const int c_end = min(p.n, c_begin + p.tokens_per_chunk);
  // the mass of window columns is never used: stop the score part at the prefix
  const int mass_end = min(c_end, p.n_prefix);

  for (int t0 = c_begin + wave * 64; t0 < c_end; t0 += NW * 64) {
    chunk_t kf0[TL::NC], kf1[TL::NC];
    load_k_subtile<T, D>(kf0, k_head, p.k_st, t0, p.n, lane);
    load_k_subtile<T, D>(kf1, k_head, p.k_st, t0 + 32, p.n, lane);

    if (DO_MASS && t0 < mass_end) {
      float col0 = 0.f, col1 = 0.f;
      for (int rb = 0; rb < nrb; ++rb) {
        f32x16 a0 = {0}, a1 = {0};
#pragma unroll
        for (int c = 0; c < TL::NC; ++c) {
          chunk_t qf = lds_chunk<T, D>(q_lds, rb * 32 + l31, c, half);
          mma_chunk<T>(a0, qf, kf0[c]);   // rows = query rows, columns = tokens
          mma_chunk<T>(a1, qf, kf1[c]);
        }
#pragma unroll
        for (int g4 = 0; g4 < 4; ++g4) {
          f32x4 b = *reinterpret_cast<const f32x4*>(bias_lds + rb * 32 + g4 * 8 + half * 4);
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            col0 += fast_exp2(a0[g4 * 4 + i] * p.c2 - b[i]);
            col1 += fast_exp2(a1[g4 * 4 + i] * p.c2 - b[i]);
          }
        }
      }
      col0 += __shfl_xor(col0, 32, kWave);
      col1 += __shfl_xor(col1, 32, kWave);
      const int t = t0 + lane;             // lanes 0..31 -> subtile 0, 32..63 -> subtile 1
      if (t < mass_end) p.mass[(size_t)h * p.n + t] = (half ? col1 : col0) * p.inv_R;
    }

    if (DO_RES) {
#pragma unroll
      for (int sub = 0; sub < 2; ++sub) {
        const chunk_t* kf = sub ? kf1 : kf0;
        const int ts = t0 + sub * 32;
        // value elements in accumulator layout: register v <-> token row acc_row(v), lane <-> JB consecutive columns
        constexpr int VB = JB * (int)sizeof(T);
        RawVec<VB> vv[16];
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          int t = min(ts + acc_row(v, half), p.n - 1);
          vv[v] = load_raw<VB>(v_head + (int64_t)t * p.v_st + l31 * JB);
        }
        float e[16];
#pragma unroll
        for (int v = 0; v < 16; ++v) e[v] = 0.f;
#pragma unroll 1
        for (int jb = 0; jb < JB; ++jb) {
          f32x16 a = {0};
#pragma unroll
          for (int c = 0; c < TL::NC; ++c) {
            chunk_t wf = lds_chunk<T, D>(wt_lds, jb * 32 + l31, c, half);
            mma_chunk<T>(a, kf[c], wf);     // rows = tokens, columns = value dims
          }
#pragma unroll
          for (int v = 0; v < 16; ++v) {
            float df = raw_elem<T, VB>(vv[v], jb) - a[v];
            e[v] += df * df;
          }
        }
        // sum over the 32 lanes (value columns) of each half
#pragma unroll
        for (int v = 0; v < 16; ++v) {
#pragma unroll
          for (int o = 16; o >= 1; o >>= 1) e[v] += __shfl_xor(e[v], o, kWave);
        }
        // lane (l & 31) == v of half hf writes token row acc_row(v, hf)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          int t = ts + acc_row(v, half);
          if (l31 == v && t < c_end) p.eps[(size_t)h * p.n + t] = e[v];
        }
      }
    }
  }
}

// ---------------------------------------------------------------------------
// pooling
// ---------------------------------------------------------------------------
__global__ void pool_scores_kernel(const float* __restrict__ mass, float* __restrict__ score, int n, int n_prefix, int kernel) {
  const int h = blockIdx.y;
  const int t = blockIdx.x * blockDim.x + threadIdx.x;
  if (t >= n) return;
  float out = INFINITY;
  if (t < n_prefix) {
    const int half = kernel / 2;
    const int lo = max(0, t - half), hi = min(n_prefix - 1, t + half);
    float s = 0.f;
    for (int j = lo; j <= hi; ++j) s += mass[(size_t)h * n + j];
    out = s / (float)kernel;
  }
  score[(size_t)h * n + t] = out;
}

// ---------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------
constexpr int kThreads = 512;

struct Plan {
  PassParams pp;
  size_t ws_need;
  size_t lds_stats, lds_pass2;
};

int pick_tokens_per_chunk(int n, int n_kv_heads) {
  // aim for at least ~2 workgroups per CU, chunks of at least 64 tokens per wave
  int tpc = 2048;
  while (tpc > 512 && (int64_t)((n + tpc - 1) / tpc) * n_kv_heads < 512) tpc >>= 1;
  return tpc;
}

template <typename T, int D>
int make_plan(const vector_shape& s, bool do_mass, bool do_res, Plan& plan) {
  using TL = Tile<T, D>;
  PassParams& p = plan.pp;
  const int G = s.n_q_heads / s.n_kv_heads;
  p.n = s.seq_len; p.w = s.window; p.R = G * s.window; p.R_pad = (p.R + 31) / 32 * 32;
  p.n_prefix = s.seq_len - s.window;
  p.tokens_per_chunk = pick_tokens_per_chunk(s.seq_len, s.n_kv_heads);
  p.n_chunks = (s.seq_len + p.tokens_per_chunk - 1) / p.tokens_per_chunk;
  p.c2 = kLog2e / sqrtf((float)D);
  p.inv_R = 1.0f / (float)p.R;
  p.k_st = s.k_stride_tok ? s.k_stride_tok : D;
  p.k_sh = s.k_stride_head ? s.k_stride_head : (int64_t)s.seq_len * p.k_st;
  p.v_st = s.v_stride_tok ? s.v_stride_tok : D;
  p.v_sh = s.v_stride_head ? s.v_stride_head : (int64_t)s.seq_len * p.v_st;
  p.w_sh = s.w_shared ? 0 : (s.w_stride_head ? s.w_stride_head : (int64_t)D * D);
  constexpr int NW = kThreads / kWave;
  plan.lds_stats = (size_t)p.R_pad * TL::kLdsStride + (size_t)NW * (p.R_pad / 32) * 64 * sizeof(float2);
  plan.lds_pass2 = (do_mass ? (size_t)p.R_pad * (TL::kLdsStride + sizeof(float)) : 0) + (do_res ? (size_t)D * TL::kLdsStride : 0);
  if (plan.lds_stats > kMaxLdsBytes || plan.lds_pass2 > kMaxLdsBytes) return VECTOR_ERR_SHAPE;
  return VECTOR_OK;
}

}  // namespace

size_t score_workspace_bytes(const vector_shape& s) {
  const int G = s.n_q_heads / s.n_kv_heads;
  const int R_pad = (G * s.window + 31) / 32 * 32;
  const int tpc = pick_tokens_per_chunk(s.seq_len, s.n_kv_heads);
  const int n_chunks = (s.seq_len + tpc - 1) / tpc;
  size_t b = 0;
  b += align_up((size_t)s.n_kv_heads * n_chunks * R_pad * sizeof(float2), 256);
  b += align_up((size_t)s.n_kv_heads * R_pad * sizeof(float), 256);
  b += align_up((size_t)s.n_kv_heads * s.seq_len * sizeof(float), 256);
  return b;
}

template <typename T, int D>
static int run_score_residual(const vector_shape& s, const void* q, const void* k, const void* v, const void* W,
                              float* score, float* eps, void* ws, hipStream_t stream) {
  const bool do_mass = score != nullptr, do_res = eps != nullptr;
  Plan plan;
  int rc = make_plan<T, D>(s, do_mass, do_res, plan);
  if (rc != VECTOR_OK) return rc;
  PassParams& p = plan.pp;
  p.q = q; p.k = k; p.v = v; p.W = W; p.eps = eps;
  unsigned char* w8 = reinterpret_cast<unsigned char*>(ws);
  p.part = reinterpret_cast<float2*>(w8);
  w8 += align_up((size_t)s.n_kv_heads * p.n_chunks * p.R_pad * sizeof(float2), 256);
  p.bias = reinterpret_cast<float*>(w8);
  w8 += align_up((size_t)s.n_kv_heads * p.R_pad * sizeof(float), 256);
  p.mass = reinterpret_cast<float*>(w8);

  dim3 grid(p.n_chunks, s.n_kv_heads);
  if (do_mass) {
    auto k1 = score_stats_kernel<T, D, kThreads>;
    VEC_HIP(set_max_lds(reinterpret_cast<const void*>(k1), plan.lds_stats));
    VEC_LAUNCH(K_SCORE_STATS, k1, grid, dim3(kThreads), plan.lds_stats, stream, p);
    VEC_LAUNCH(K_STATS_COMBINE, stats_combine_kernel, dim3((p.R_pad + 127) / 128, s.n_kv_heads), dim3(128), 0, stream, p);
  }
  if (do_mass && do_res) {
    auto k2 = mass_residual_kernel<T, D, kThreads, true, true>;
    VEC_HIP(set_max_lds(reinterpret_cast<const void*>(k2), plan.lds_pass2));
    VEC_LAUNCH(K_MASS_RESIDUAL, k2, grid, dim3(kThreads), plan.lds_pass2, stream, p);
  } else if (do_mass) {
    auto k2 = mass_residual_kernel<T, D, kThreads, true, false>;
    VEC_HIP(set_max_lds(reinterpret_cast<const void*>(k2), plan.lds_pass2));
    VEC_LAUNCH(K_MASS_RESIDUAL, k2, grid, dim3(kThreads), plan.lds_pass2, stream, p);
  } else {
    auto k2 = mass_residual_kernel<T, D, kThreads, false, true>;
    VEC_HIP(set_max_lds(reinterpret_cast<const void*>(k2), plan.lds_pass2));
    VEC_LAUNCH(K_MASS_RESIDUAL, k2, grid, dim3(kThreads), plan.lds_pass2, stream, p);
  }
  if (do_mass)
    VEC_LAUNCH(K_POOL, pool_scores_kernel, dim3((s.seq_len + 255) / 256, s.n_kv_heads), dim3(256), 0, stream,
                       p.mass, score, s.seq_len, p.n_prefix, s.pool_kernel);
  VEC_HIP(hipGetLastError());
  return VECTOR_OK;
}

int launch_score_residual(const vector_shape& s, const void* q, const void* k, const void* v, const void* W,
                          float* score, float* eps, void* ws, hipStream_t stream) {
  if (s.dtype == VECTOR_BF16) {
    if (s.head_dim == 128) return run_score_residual<bf16_t, 128>(s, q, k, v, W, score, eps, ws, stream);
    if (s.head_dim == 64) return run_score_residual<bf16_t, 64>(s, q, k, v, W, score, eps, ws, stream);
  } else if (s.dtype == VECTOR_F32) {
    if (s.head_dim == 128) return run_score_residual<float, 128>(s, q, k, v, W, score, eps, ws, stream);
    if (s.head_dim == 64) return run_score_residual<float, 64>(s, q, k, v, W, score, eps, ws, stream);
  } else {
    return VECTOR_ERR_DTYPE;
  }
  return VECTOR_ERR_SHAPE;
}

}  // namespace vec
