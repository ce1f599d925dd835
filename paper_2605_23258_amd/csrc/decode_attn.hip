// Decode attention over the packed VECTOR cache (Section 3.2, Step 3: values of
// approximated tokens are rebuilt from their keys, v_hat = k W, at generation time).
//
// One softmax runs over the live retained rows and the approximated rows together.
// Because the rebuilt value is linear in the key, sum_t p_t (k_t W) = (sum_t p_t k_t) W:
// the kernel accumulates z = sum p_t k_t over the approximated rows and applies W once
// per (sequence, KV head) in the combine step, so every cache row is read exactly once
// and no value row is ever materialised.
//
//   decode_split_kernel   : grid (split, kv head, sequence); each wave walks 32-token
//                           tiles: logits by MFMA (K tile x the G query rows of the
//                           head), online softmax, then p . V (or p . K) on the vector
//                           ALU with rows streamed as 16-byte pieces per lane.
//   decode_combine_kernel : merges the splits, applies W to z, normalises, stores.
#include "common.hpp"
#include "launch.hpp"

namespace vec {

namespace {

struct DecodeParams {
  const void* q; const void* k_ret; const void* v_ret; const void* k_apx; const void* W;
  const int32_t* len_retain;
  void* out;
  float* part;            // [B, Hkv, S, 2*G + 2*G*D] floats: m[G], l[G], accV[G][D], accZ[G][D]
  int B, Hq, Hkv, cap_retain, n_approx, n_splits;
  int64_t w_sh;           // element stride between per-head W
  float c2;               // scale * log2(e)
};

constexpr int DT_ = 256;          // threads per workgroup
constexpr int DW = DT_ / kWave;   // waves
constexpr int kMaxSplits = 64;

template <typename T, int D, int G>
__global__ __launch_bounds__(DT_) void decode_split_kernel(DecodeParams p) {
  constexpr int E = Elem<T>::kPerChunk;          // elements per 16-byte piece
  constexpr int NC = D / (2 * E);
  constexpr int P = D / E;                       // 16-byte pieces per row
  constexpr int RPL = kWave / P;                 // rows covered by one wave-wide load
  constexpr int NIT = 32 / RPL;
  constexpr int PSZ = 2 * G + 2 * G * D;

  __shared__ float p_lds[DW][32][G];
  __shared__ float alpha_lds[DW][G];
  __shared__ float ml_lds[DW][2][G];
  __shared__ float red_lds[DW][2][G][D];

  const int split = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, half = lane >> 5, l31 = lane & 31;
  const int len_r = min(max(p.len_retain[b], 0), p.cap_retain);
  const int nt_r = (len_r + 31) / 32, nt_a = (p.n_approx + 31) / 32, nt = nt_r + nt_a;
  const int tile_begin = (int)((int64_t)nt * split / p.n_splits);
  const int tile_end = (int)((int64_t)nt * (split + 1) / p.n_splits);

  const size_t bh = (size_t)b * p.Hkv + h;
  const T* kr = reinterpret_cast<const T*>(p.k_ret) + bh * p.cap_retain * D;
  const T* vr = reinterpret_cast<const T*>(p.v_ret) + bh * p.cap_retain * D;
  const T* ka = reinterpret_cast<const T*>(p.k_apx) + bh * p.n_approx * D;

  // query rows of this KV head as the N-side MFMA operand: lane (l & 31) = g < G
  chunk_t qf[NC];
  {
    const T* qrow = reinterpret_cast<const T*>(p.q) + ((size_t)b * p.Hq + (size_t)h * G + min(l31, G - 1)) * D;
#pragma unroll
    for (int c = 0; c < NC; ++c) {
      qf[c] = load_chunk(qrow + chunk_elem_offset<T>(c, half));
      if (l31 >= G) qf[c] = make_uint4(0, 0, 0, 0);
    }
  }

  float m_run = -INFINITY, l_run = 0.f;         // meaningful in lanes with (l & 31) < G
  float accV[G][E], accZ[G][E];
#pragma unroll
  for (int g = 0; g < G; ++g)
#pragma unroll
    for (int e = 0; e < E; ++e) accV[g][e] = accZ[g][e] = 0.f;

  const int prow = lane / P, piece = lane % P;   // row group and 16-byte piece this lane streams

  for (int tile = tile_begin + wave; tile < tile_end; tile += DW) {
    const bool is_apx = tile >= nt_r;
    const T* kseg = is_apx ? ka : kr;
    const int seg_len = is_apx ? p.n_approx : len_r;
    const int t0 = (is_apx ? tile - nt_r : tile) * 32;

    // logits: rows = tokens, columns = query rows
    f32x16 s = {0};
    {
      const T* krow = kseg + (size_t)min(t0 + l31, seg_len - 1) * D;
#pragma unroll
      for (int c = 0; c < NC; ++c) mma_chunk<T>(s, load_chunk(krow + chunk_elem_offset<T>(c, half)), qf[c]);
    }
    float x[16];
    float tmax = -INFINITY;
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      x[v] = (t0 + acc_row(v, half) < seg_len) ? s[v] * p.c2 : -INFINITY;
      tmax = fmaxf(tmax, x[v]);
    }
    tmax = fmaxf(tmax, __shfl_xor(tmax, 32, kWave));
    const float m_new = fmaxf(m_run, tmax);      // finite: every tile holds a live token
    const float alpha = fast_exp2(m_run - m_new);
    float psum = 0.f;
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      x[v] = fast_exp2(x[v] - m_new);
      psum += x[v];
    }
    psum += __shfl_xor(psum, 32, kWave);
    l_run = l_run * alpha + psum;
    m_run = m_new;
    if (l31 < G) {
#pragma unroll
      for (int v = 0; v < 16; ++v) p_lds[wave][acc_row(v, half)][l31] = x[v];
      if (half == 0) alpha_lds[wave][l31] = alpha;
    }
    // LDS operations of one wave complete in issue order: the reads below see these writes
    __builtin_amdgcn_wave_barrier();

    float al[G];
    bool rescale = false;
#pragma unroll
    for (int g = 0; g < G; ++g) { al[g] = alpha_lds[wave][g]; rescale |= al[g] != 1.f; }
    if (rescale) {
#pragma unroll
      for (int g = 0; g < G; ++g)
#pragma unroll
        for (int e = 0; e < E; ++e) { accV[g][e] *= al[g]; accZ[g][e] *= al[g]; }
    }

    // p . rows: value rows for retained tokens, key rows for approximated ones
    const T* rseg = is_apx ? ka : vr;
    if (is_apx) {
#pragma unroll
      for (int it = 0; it < NIT; ++it) {
        const int r = it * RPL + prow;
        const chunk_t raw = load_chunk(rseg + (size_t)min(t0 + r, seg_len - 1) * D + piece * E);
        float pg[G];
#pragma unroll
        for (int g = 0; g < G; ++g) pg[g] = p_lds[wave][r][g];
        float f[E];
        if constexpr (E == 8) {
          f[0] = bf16_lo(raw.x); f[1] = bf16_hi(raw.x); f[2] = bf16_lo(raw.y); f[3] = bf16_hi(raw.y);
          f[4] = bf16_lo(raw.z); f[5] = bf16_hi(raw.z); f[6] = bf16_lo(raw.w); f[7] = bf16_hi(raw.w);
        } else {
          f[0] = __uint_as_float(raw.x); f[1] = __uint_as_float(raw.y); f[2] = __uint_as_float(raw.z); f[3] = __uint_as_float(raw.w);
        }
#pragma unroll
        for (int g = 0; g < G; ++g)
#pragma unroll
          for (int e = 0; e < E; ++e) accZ[g][e] += pg[g] * f[e];
      }
    } else {
#pragma unroll
      for (int it = 0; it < NIT; ++it) {
        const int r = it * RPL + prow;
        const chunk_t raw = load_chunk(rseg + (size_t)min(t0 + r, seg_len - 1) * D + piece * E);
        float pg[G];
#pragma unroll
        for (int g = 0; g < G; ++g) pg[g] = p_lds[wave][r][g];
        float f[E];
        if constexpr (E == 8) {
          f[0] = bf16_lo(raw.x); f[1] = bf16_hi(raw.x); f[2] = bf16_lo(raw.y); f[3] = bf16_hi(raw.y);
          f[4] = bf16_lo(raw.z); f[5] = bf16_hi(raw.z); f[6] = bf16_lo(raw.w); f[7] = bf16_hi(raw.w);
        } else {
          f[0] = __uint_as_float(raw.x); f[1] = __uint_as_float(raw.y); f[2] = __uint_as_float(raw.z); f[3] = __uint_as_float(raw.w);
        }
#pragma unroll
        for (int g = 0; g < G; ++g)
#pragma unroll
          for (int e = 0; e < E; ++e) accV[g][e] += pg[g] * f[e];
      }
    }
    __builtin_amdgcn_wave_barrier();             // keep the next tile's LDS writes behind these reads
  }

  // ---- merge the row groups of a wave, then the waves of the workgroup ----
#pragma unroll
  for (int g = 0; g < G; ++g)
#pragma unroll
    for (int e = 0; e < E; ++e) {
#pragma unroll
      for (int o = P; o < kWave; o <<= 1) {
        accV[g][e] += __shfl_xor(accV[g][e], o, kWave);
        accZ[g][e] += __shfl_xor(accZ[g][e], o, kWave);
      }
    }
  if (lane < P) {
#pragma unroll
    for (int g = 0; g < G; ++g)
#pragma unroll
      for (int e = 0; e < E; ++e) {
        red_lds[wave][0][g][piece * E + e] = accV[g][e];
        red_lds[wave][1][g][piece * E + e] = accZ[g][e];
      }
  }
  if (lane < G) { ml_lds[wave][0][lane] = m_run; ml_lds[wave][1][lane] = l_run; }
  __syncthreads();

  float* out = p.part + (bh * p.n_splits + split) * PSZ;
  for (int i = threadIdx.x; i < 2 * G * D; i += DT_) {
    const int set = i / (G * D), g = (i / D) % G, j = i % D;
    float m = -INFINITY;
#pragma unroll
    for (int wv = 0; wv < DW; ++wv) m = fmaxf(m, ml_lds[wv][0][g]);
    float acc = 0.f;
#pragma unroll
    for (int wv = 0; wv < DW; ++wv) {
      const float mw = ml_lds[wv][0][g];
      if (mw != -INFINITY) acc += red_lds[wv][set][g][j] * fast_exp2(mw - m);
    }
    out[2 * G + i] = acc;
  }
  if (threadIdx.x < G) {
    const int g = threadIdx.x;
    float m = -INFINITY, l = 0.f;
#pragma unroll
    for (int wv = 0; wv < DW; ++wv) m = fmaxf(m, ml_lds[wv][0][g]);
#pragma unroll
    for (int wv = 0; wv < DW; ++wv) {
      const float mw = ml_lds[wv][0][g];
      if (mw != -INFINITY) l += ml_lds[wv][1][g] * fast_exp2(mw - m);
    }
    out[g] = m;
    out[G + g] = l;
  }
}

template <typename T, int D, int G>
__global__ __launch_bounds__(256) void decode_combine_kernel(DecodeParams p) {
  constexpr int PSZ = 2 * G + 2 * G * D;
  __shared__ float z_lds[G][D];
  __shared__ float v_lds[G][D];
  __shared__ float scale_lds[kMaxSplits][G];   // per split: exp2(m_s - M)
  __shared__ float linv_lds[G];
  const int h = blockIdx.x, b = blockIdx.y;
  const size_t bh = (size_t)b * p.Hkv + h;
  const float* part = p.part + bh * p.n_splits * PSZ;

  if (threadIdx.x < G) {
    const int g = threadIdx.x;
    float m = -INFINITY;
    for (int s = 0; s < p.n_splits; ++s) m = fmaxf(m, part[(size_t)s * PSZ + g]);
    float l = 0.f;
    for (int s = 0; s < p.n_splits; ++s) {
      const float ms = part[(size_t)s * PSZ + g];
      const float sc = (ms == -INFINITY) ? 0.f : fast_exp2(ms - m);
      scale_lds[s][g] = sc;
      l += part[(size_t)s * PSZ + G + g] * sc;
    }
    linv_lds[g] = (l > 0.f) ? 1.f / l : 0.f;
  }
  __syncthreads();
  for (int i = threadIdx.x; i < G * D; i += 256) {
    const int g = i / D;
    float av = 0.f, az = 0.f;
    for (int s = 0; s < p.n_splits; ++s) {
      const float sc = scale_lds[s][g];
      av += part[(size_t)s * PSZ + 2 * G + i] * sc;
      az += part[(size_t)s * PSZ + 2 * G + G * D + i] * sc;
    }
    (&v_lds[0][0])[i] = av;
    (&z_lds[0][0])[i] = az;
  }
  __syncthreads();
  // out[g][j] = (sum_ret p v  +  z[g][:] . W[:, j]) / l
  const T* Wh = reinterpret_cast<const T*>(p.W) + (int64_t)h * p.w_sh;
  T* out = reinterpret_cast<T*>(p.out) + ((size_t)b * p.Hq + (size_t)h * G) * D;
  for (int j = threadIdx.x; j < D; j += 256 / 1) {
    float acc[G];
#pragma unroll
    for (int g = 0; g < G; ++g) acc[g] = v_lds[g][j];
    if (p.n_approx > 0) {
      for (int i = 0; i < D; ++i) {
        const float wij = to_float(Wh[(size_t)i * D + j]);
#pragma unroll
        for (int g = 0; g < G; ++g) acc[g] += z_lds[g][i] * wij;
      }
    }
#pragma unroll
    for (int g = 0; g < G; ++g) store_elem(out + (size_t)g * D + j, acc[g] * linv_lds[g]);
  }
}

int pick_splits(int batch, int n_kv_heads, int cap_retain, int n_approx) {
  // enough workgroups for ~4 per CU, each with at least 4 tiles per wave; at most 64
  const int tiles = (cap_retain + 31) / 32 + (n_approx + 31) / 32;
  int s = (1024 + batch * n_kv_heads - 1) / (batch * n_kv_heads);
  const int max_by_work = tiles / (4 * DW) > 1 ? tiles / (4 * DW) : 1;
  if (s > max_by_work) s = max_by_work;
  if (s > kMaxSplits) s = kMaxSplits;
  if (s < 1) s = 1;
  return s;
}

template <typename T, int D, int G>
int run_decode(const vector_cache& c, DecodeParams& p, hipStream_t stream) {
  VEC_LAUNCH(K_DECODE_SPLIT, (decode_split_kernel<T, D, G>), dim3(p.n_splits, c.n_kv_heads, c.batch), dim3(DT_), 0, stream, p);
  VEC_LAUNCH(K_DECODE_COMBINE, (decode_combine_kernel<T, D, G>), dim3(c.n_kv_heads, c.batch), dim3(256), 0, stream, p);
  VEC_HIP(hipGetLastError());
  return VECTOR_OK;
}

template <typename T, int D>
int run_decode_g(const vector_cache& c, DecodeParams& p, hipStream_t stream) {
  switch (c.n_q_heads / c.n_kv_heads) {
    case 1: return run_decode<T, D, 1>(c, p, stream);
    case 2: return run_decode<T, D, 2>(c, p, stream);
    case 4: return run_decode<T, D, 4>(c, p, stream);
    case 8: return run_decode<T, D, 8>(c, p, stream);
    default: return VECTOR_ERR_SHAPE;
  }
}

}  // namespace

size_t decode_workspace_bytes(int batch, int n_q_heads, int n_kv_heads, int head_dim, int cap_retain, int n_approx) {
  // sized for the largest split count so that the bound holds for any live length
  (void)cap_retain; (void)n_approx;
  const int G = n_q_heads / n_kv_heads;
  return align_up((size_t)batch * n_kv_heads * kMaxSplits * (2 * G + 2 * G * head_dim) * sizeof(float), 256);
}

int launch_decode_attn(const vector_cache& c, const void* q, float scale, void* out, int flags, void* ws,
                       hipStream_t stream) {
  (void)flags;
  DecodeParams p;
  p.q = q; p.k_ret = c.k_ret; p.v_ret = c.v_ret; p.k_apx = c.k_apx; p.W = c.W; p.len_retain = c.len_retain;
  p.out = out; p.part = reinterpret_cast<float*>(ws);
  p.B = c.batch; p.Hq = c.n_q_heads; p.Hkv = c.n_kv_heads; p.cap_retain = c.cap_retain; p.n_approx = c.n_approx;
  p.n_splits = pick_splits(c.batch, c.n_kv_heads, c.cap_retain, c.n_approx);
  p.w_sh = c.w_shared ? 0 : (int64_t)c.head_dim * c.head_dim;
  p.c2 = scale * kLog2e;
  if (c.dtype == VECTOR_BF16) {
    if (c.head_dim == 128) return run_decode_g<bf16_t, 128>(c, p, stream);
    if (c.head_dim == 64) return run_decode_g<bf16_t, 64>(c, p, stream);
  } else if (c.dtype == VECTOR_F32) {
    if (c.head_dim == 128) return run_decode_g<float, 128>(c, p, stream);
    if (c.head_dim == 64) return run_decode_g<float, 64>(c, p, stream);
  } else {
    return VECTOR_ERR_DTYPE;
  }
  return VECTOR_ERR_SHAPE;
}

}  // namespace vec
