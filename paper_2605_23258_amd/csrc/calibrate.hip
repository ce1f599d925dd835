// Least-squares value map (Section 3.1): W_h = argmin_W || K_h W - V_h ||_F^2, no intercept,
// from m calibration tokens per KV head, through the normal equations
//   (K^T K) W = K^T V.
//
//   gram_kernel  : grid (token chunks, kv heads).  The two d x d products contract over
//                  tokens, so the operands are columns of the [token][dim] tiles: a workgroup
//                  stages 32-token tiles of K and V in LDS with coalesced 16-byte loads and
//                  its waves read them back down the columns (eight 2-byte reads per MFMA
//                  operand register set).  Wave w owns the 32-row block w of both products
//                  (d = 128; for d = 64 two waves take K^T K and two K^T V).  fp32 MFMA
//                  accumulation inside a chunk; one fp32 partial pair per chunk.
//   gram_valu_kernel : the same partials for fp32 inputs with plain FMAs (small problems).
//   solve_kernel : one workgroup per head.  Sums the chunk partials in fp64, factors
//                  K^T K = L L^T in LDS (fp64 Cholesky), and solves the d right-hand sides,
//                  one thread per column of W.
#include "common.hpp"
#include "launch.hpp"

namespace vec {

namespace {

constexpr int kCalThreads = 256;
constexpr int kCalTile = 32;                 // tokens per staged tile
constexpr int kCalMaxChunks = 64;

struct CalParams {
  const void* k; const void* v;
  int64_t k_sh, k_st, v_sh, v_st;           // element strides
  int m;                                    // calibration tokens per head
  int tokens_per_chunk, n_chunks;
  float* part;                              // [Hkv, n_chunks, 2, d, d] fp32: K^T K, then K^T V
  double* c64;                              // [Hkv, d, d] fp64 scratch: the Cholesky factor during the solves
  void* W;                                  // [Hkv, d, d] out
  int* status;                              // [Hkv]: 0 ok, 1 not positive definite
};

typedef __attribute__((ext_vector_type(8))) unsigned short cal_u16x8;

template <int D>
__global__ __launch_bounds__(kCalThreads) void gram_kernel(CalParams p) {
  using T = bf16_t;
  constexpr int kRowBytes = D * 2;
  constexpr int kStride = kRowBytes + 16;
  constexpr int kPieces = kRowBytes / 16;
  constexpr int kLoads = kCalTile * kPieces / kCalThreads;       // 16-byte pieces per thread, tile and tensor
  static_assert(kCalTile * kPieces % kCalThreads == 0 && kLoads >= 1, "tile shape");
  constexpr int JB = D / 32;
  constexpr int kTileBytes = kCalTile * kStride;
  // wave -> (row block, which products): d = 128: row block = wave, both products;
  // d = 64: waves 0,1 take K^T K, waves 2,3 take K^T V
  constexpr bool kBoth = (JB == 4);
  __shared__ __align__(16) unsigned char lds[2][2][kTileBytes];   // [buffer][K, V]

  const int h = blockIdx.y, chunk = blockIdx.x;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, l31 = lane & 31, half = lane >> 5;
  const int ib = kBoth ? wave : (wave % JB);
  const bool do_g = kBoth || wave < JB, do_c = kBoth || wave >= JB;
  const T* k_head = reinterpret_cast<const T*>(p.k) + (int64_t)h * p.k_sh;
  const T* v_head = reinterpret_cast<const T*>(p.v) + (int64_t)h * p.v_sh;
  const int c_begin = chunk * p.tokens_per_chunk;
  const int c_end = min(p.m, c_begin + p.tokens_per_chunk);
  const int n_tiles = (c_end - c_begin + kCalTile - 1) / kCalTile;

  f32x16 accg[JB], accc[JB];
#pragma unroll
  for (int jb = 0; jb < JB; ++jb)
#pragma unroll
    for (int x = 0; x < 16; ++x) { accg[jb][x] = 0.f; accc[jb][x] = 0.f; }

  // rows past the chunk are staged as zeros: they add nothing to either product
  auto fetch = [&](uint4* kr, uint4* vr, int tile) {
#pragma unroll
    for (int u = 0; u < kLoads; ++u) {
      const int i = threadIdx.x + u * kCalThreads;
      const int t = c_begin + tile * kCalTile + i / kPieces;
      kr[u] = make_uint4(0, 0, 0, 0);
      vr[u] = make_uint4(0, 0, 0, 0);
      if (t < c_end) {
        kr[u] = load_chunk(reinterpret_cast<const unsigned char*>(k_head + (int64_t)t * p.k_st) + (i % kPieces) * 16);
        vr[u] = load_chunk(reinterpret_cast<const unsigned char*>(v_head + (int64_t)t * p.v_st) + (i % kPieces) * 16);
      }
    }
  };
  auto stash = [&](const uint4* kr, const uint4* vr, int buf) {
#pragma unroll
    for (int u = 0; u < kLoads; ++u) {
      const int i = threadIdx.x + u * kCalThreads;
      const int off = (i / kPieces) * kStride + (i % kPieces) * 16;
      *reinterpret_cast<uint4*>(lds[buf][0] + off) = kr[u];
      *reinterpret_cast<uint4*>(lds[buf][1] + off) = vr[u];
    }
  };
  // operand of one 16-token step: lane (dim 32*blk + l31, half) holds tokens 16*ks + 8*half + e
  auto column = [&](const unsigned char* tile, int blk, int ks) {
    cal_u16x8 a;
#pragma unroll
    for (int e = 0; e < 8; ++e)
      a[e] = *reinterpret_cast<const unsigned short*>(tile + (16 * ks + 8 * half + e) * kStride + (blk * 32 + l31) * 2);
    return __builtin_bit_cast(bf16x8, a);
  };

  uint4 kr[kLoads], vr[kLoads];
  if (n_tiles > 0) { fetch(kr, vr, 0); stash(kr, vr, 0); }
  for (int tile = 0; tile < n_tiles; ++tile) {
    __syncthreads();                         // tile is staged; the other buffer is free
    if (tile + 1 < n_tiles) fetch(kr, vr, tile + 1);
    const unsigned char* kt = lds[tile & 1][0];
    const unsigned char* vt = lds[tile & 1][1];
#pragma unroll
    for (int ks = 0; ks < kCalTile / 16; ++ks) {
      const bf16x8 a = column(kt, ib, ks);
#pragma unroll
      for (int jb = 0; jb < JB; ++jb) {
        if (do_g) accg[jb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, column(kt, jb, ks), accg[jb], 0, 0, 0);
        if (do_c) accc[jb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, column(vt, jb, ks), accc[jb], 0, 0, 0);
      }
    }
    if (tile + 1 < n_tiles) stash(kr, vr, (tile + 1) & 1);
  }
  // accumulator register x of block jb: row 32*ib + acc_row(x, half), column 32*jb + l31
  float* out = p.part + ((size_t)h * p.n_chunks + chunk) * 2 * D * D;
#pragma unroll
  for (int jb = 0; jb < JB; ++jb)
#pragma unroll
    for (int x = 0; x < 16; ++x) {
      const size_t at = (size_t)(32 * ib + acc_row(x, half)) * D + 32 * jb + l31;
      if (do_g) out[at] = accg[jb][x];
      if (do_c) out[(size_t)D * D + at] = accc[jb][x];
    }
}

// fp32 inputs: plain FMAs; a thread owns one column and every other row of both products
template <int D>
__global__ __launch_bounds__(kCalThreads) void gram_valu_kernel(CalParams p) {
  constexpr int kStride = D + 1;
  constexpr int kPer = D * D / kCalThreads;          // outputs per thread and product
  __shared__ float kt[kCalTile][kStride], vt[kCalTile][kStride];
  const int h = blockIdx.y, chunk = blockIdx.x;
  const float* k_head = reinterpret_cast<const float*>(p.k) + (int64_t)h * p.k_sh;
  const float* v_head = reinterpret_cast<const float*>(p.v) + (int64_t)h * p.v_sh;
  const int c_begin = chunk * p.tokens_per_chunk;
  const int c_end = min(p.m, c_begin + p.tokens_per_chunk);
  // outputs o = tid + u * kCalThreads of either product: row o / D, column o % D
  float ag[kPer], ac[kPer];
#pragma unroll
  for (int u = 0; u < kPer; ++u) { ag[u] = 0.f; ac[u] = 0.f; }
  for (int t0 = c_begin; t0 < c_end; t0 += kCalTile) {
    __syncthreads();
    for (int i = threadIdx.x; i < kCalTile * D; i += kCalThreads) {
      const int r = i / D, c = i % D, t = t0 + r;
      kt[r][c] = (t < c_end) ? k_head[(int64_t)t * p.k_st + c] : 0.f;
      vt[r][c] = (t < c_end) ? v_head[(int64_t)t * p.v_st + c] : 0.f;
    }
    __syncthreads();
#pragma unroll 4
    for (int r = 0; r < kCalTile; ++r) {
#pragma unroll
      for (int u = 0; u < kPer; ++u) {
        const int o = threadIdx.x + u * kCalThreads, i = o / D, j = o % D;
        ag[u] = fmaf(kt[r][i], kt[r][j], ag[u]);
        ac[u] = fmaf(kt[r][i], vt[r][j], ac[u]);
      }
    }
  }
  float* out = p.part + ((size_t)h * p.n_chunks + chunk) * 2 * D * D;
#pragma unroll
  for (int u = 0; u < kPer; ++u) {
    const int o = threadIdx.x + u * kCalThreads;
    out[o] = ag[u];
    out[(size_t)D * D + o] = ac[u];
  }
}

template <typename T, int D>
__global__ __launch_bounds__(kCalThreads) void solve_kernel(CalParams p) {
  extern __shared__ __align__(16) unsigned char cal_smem[];
  constexpr int LD = D + 1;                                  // padded row: a column walk hits distinct banks
  double* G = reinterpret_cast<double*>(cal_smem);           // [D][LD]: K^T K, then its Cholesky factor; later K^T V / W
  __shared__ int bad;
  const int h = blockIdx.x;
  const float* part = p.part + (size_t)h * p.n_chunks * 2 * D * D;
  double* Lg = p.c64 + (size_t)h * D * D;                    // the factor, parked in global memory for the solves
  if (threadIdx.x == 0) bad = 0;
  for (int o = threadIdx.x; o < D * D; o += kCalThreads) {
    double g = 0.0;
#pragma unroll 8
    for (int ch = 0; ch < p.n_chunks; ++ch) g += (double)part[(size_t)ch * 2 * D * D + o];
    G[(o / D) * LD + o % D] = g;
  }
  __syncthreads();
  // left-looking Cholesky, one thread per row: column kk of the factor is
  //   L[i][kk] = (G[i][kk] - sum_{q < kk} L[i][q] L[kk][q]) / L[kk][kk],   i >= kk
  for (int kk = 0; kk < D; ++kk) {
    const int i = threadIdx.x;
    double v = 0.0;
    if (i >= kk && i < D) {
      // four running sums and an unrolled body: the loads of several steps are in flight together
      double a0 = 0.0, a1 = 0.0, a2 = 0.0, a3 = 0.0;
      int q = 0;
#pragma unroll 2
      for (; q + 4 <= kk; q += 4) {
        a0 += G[i * LD + q] * G[kk * LD + q];
        a1 += G[i * LD + q + 1] * G[kk * LD + q + 1];
        a2 += G[i * LD + q + 2] * G[kk * LD + q + 2];
        a3 += G[i * LD + q + 3] * G[kk * LD + q + 3];
      }
      for (; q < kk; ++q) a0 += G[i * LD + q] * G[kk * LD + q];
      v = G[i * LD + kk] - ((a0 + a1) + (a2 + a3));
    }
    if (i == kk && !(v > 0.0)) bad = 1;
    __syncthreads();                            // every row has read what it needs of column kk's old values
    if (bad) break;
    if (i == kk) G[kk * LD + kk] = sqrt(v);
    __syncthreads();
    if (i > kk && i < D) G[i * LD + kk] = v / G[kk * LD + kk];
    __syncthreads();
  }
  T* Wh = reinterpret_cast<T*>(p.W) + (size_t)h * D * D;
  if (bad) {                                    // not positive definite: say so, write NaN
    if (threadIdx.x == 0) p.status[h] = 1;
    for (int o = threadIdx.x; o < D * D; o += kCalThreads) store_elem(Wh + o, __builtin_nanf(""));
    return;
  }
  if (threadIdx.x == 0) p.status[h] = 0;
  // Solves out of LDS: the factor is repacked as its lower triangle (through global memory,
  // which avoids an in-place shuffle), and the right-hand sides come in blocks of kCols columns.
  for (int o = threadIdx.x; o < D * D; o += kCalThreads) Lg[o] = G[(o / D) * LD + o % D];
  __syncthreads();
  double* Lp = G;                                             // packed: L[i][q] at i (i + 1) / 2 + q
  for (int o = threadIdx.x; o < D * D; o += kCalThreads) {
    const int i = o / D, q = o % D;
    if (q <= i) Lp[i * (i + 1) / 2 + q] = Lg[o];
  }
  constexpr int kSplit = 4;                                   // adjacent lanes that share a column's inner sums
  constexpr int kCols = kCalThreads / kSplit;                 // columns per block
  static_assert(D % kCols == 0 || kCols % D == 0, "column blocks");
  constexpr int kBlockCols = kCols < D ? kCols : D;
  double* C = Lp + D * (D + 1) / 2;                           // [D][kBlockCols]
  const int jl = threadIdx.x / kSplit, r = threadIdx.x % kSplit;
  auto wave_sync = [&]() {                                    // the lanes of a column sit in one wave
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
  };
  for (int j0 = 0; j0 < D; j0 += kBlockCols) {
    __syncthreads();                                          // packed factor in place / previous block done
    for (int o = threadIdx.x; o < D * kBlockCols; o += kCalThreads) {
      const int i = o / kBlockCols, jj = o % kBlockCols;
      double c = 0.0;
#pragma unroll 8
      for (int ch = 0; ch < p.n_chunks; ++ch) c += (double)part[(size_t)ch * 2 * D * D + D * D + i * D + j0 + jj];
      C[o] = c;
    }
    __syncthreads();
    if (jl < kBlockCols) {
      // L y = c_j
      for (int i = 0; i < D; ++i) {
        const double* Li = Lp + i * (i + 1) / 2;
        double s = 0.0, s1 = 0.0;
        int q = r;
#pragma unroll 4
        for (; q + kSplit < i; q += 2 * kSplit) {
          s += Li[q] * C[q * kBlockCols + jl];
          s1 += Li[q + kSplit] * C[(q + kSplit) * kBlockCols + jl];
        }
        if (q < i) s += Li[q] * C[q * kBlockCols + jl];
        s += s1;
#pragma unroll
        for (int o = 1; o < kSplit; o <<= 1) s += __shfl_xor(s, o, kWave);
        if (r == 0) C[i * kBlockCols + jl] = (C[i * kBlockCols + jl] - s) / Li[i];
        wave_sync();
      }
      // L^T x = y
      for (int i = D - 1; i >= 0; --i) {
        double s = 0.0, s1 = 0.0;
        int q = i + 1 + r;
#pragma unroll 4
        for (; q + kSplit < D; q += 2 * kSplit) {
          s += Lp[q * (q + 1) / 2 + i] * C[q * kBlockCols + jl];
          s1 += Lp[(q + kSplit) * (q + kSplit + 1) / 2 + i] * C[(q + kSplit) * kBlockCols + jl];
        }
        if (q < D) s += Lp[q * (q + 1) / 2 + i] * C[q * kBlockCols + jl];
        s += s1;
#pragma unroll
        for (int o = 1; o < kSplit; o <<= 1) s += __shfl_xor(s, o, kWave);
        const double x = (C[i * kBlockCols + jl] - s) / Lp[i * (i + 1) / 2 + i];
        wave_sync();
        if (r == 0) {
          C[i * kBlockCols + jl] = x;
          store_elem(Wh + (size_t)i * D + j0 + jl, (float)x);
        }
        wave_sync();
      }
    }
  }
}

void calibrate_chunks(int m, int& tokens_per_chunk, int& n_chunks) {
  n_chunks = (m + 1023) / 1024;
  if (n_chunks > kCalMaxChunks) n_chunks = kCalMaxChunks;
  if (n_chunks < 1) n_chunks = 1;
  tokens_per_chunk = ((m + n_chunks - 1) / n_chunks + kCalTile - 1) / kCalTile * kCalTile;
  n_chunks = (m + tokens_per_chunk - 1) / tokens_per_chunk;
  if (n_chunks < 1) n_chunks = 1;
}

template <typename T, int D>
int run_calibrate(const vector_shape& s, CalParams& p, hipStream_t stream) {
  const dim3 grid(p.n_chunks, s.n_kv_heads);
  if constexpr (Elem<T>::kDtype == VECTOR_BF16) hipLaunchKernelGGL(gram_kernel<D>, grid, dim3(kCalThreads), 0, stream, p);
  else hipLaunchKernelGGL(gram_valu_kernel<D>, grid, dim3(kCalThreads), 0, stream, p);
  // padded square for the factorisation; packed triangle plus a block of right-hand sides for the solves
  constexpr int kBlockCols = (kCalThreads / 4) < D ? (kCalThreads / 4) : D;
  constexpr size_t kFactor = (size_t)D * (D + 1), kSolve = (size_t)D * (D + 1) / 2 + (size_t)D * kBlockCols;
  const size_t lds = (kFactor > kSolve ? kFactor : kSolve) * sizeof(double);
  VEC_HIP(set_max_lds(reinterpret_cast<const void*>(solve_kernel<T, D>), lds));
  hipLaunchKernelGGL((solve_kernel<T, D>), dim3(s.n_kv_heads), dim3(kCalThreads), lds, stream, p);
  VEC_HIP(hipGetLastError());
  return VECTOR_OK;
}

}  // namespace

size_t calibrate_workspace_bytes(const vector_shape& s) {
  int tpc, nc;
  calibrate_chunks(s.seq_len, tpc, nc);
  const size_t dd = (size_t)s.head_dim * s.head_dim;
  return align_up((size_t)s.n_kv_heads * nc * 2 * dd * sizeof(float), 256) + align_up((size_t)s.n_kv_heads * dd * sizeof(double), 256) +
         align_up((size_t)s.n_kv_heads * sizeof(int), 256);
}

int launch_calibrate(const vector_shape& s, const void* k, const void* v, void* W, void* ws, hipStream_t stream) {
  CalParams p;
  p.k = k; p.v = v; p.W = W; p.m = s.seq_len;
  const int D = s.head_dim;
  p.k_st = s.k_stride_tok ? s.k_stride_tok : D;
  p.k_sh = s.k_stride_head ? s.k_stride_head : (int64_t)s.seq_len * p.k_st;
  p.v_st = s.v_stride_tok ? s.v_stride_tok : D;
  p.v_sh = s.v_stride_head ? s.v_stride_head : (int64_t)s.seq_len * p.v_st;
  calibrate_chunks(s.seq_len, p.tokens_per_chunk, p.n_chunks);
  const size_t dd = (size_t)D * D;
  unsigned char* w8 = reinterpret_cast<unsigned char*>(ws);
  p.part = reinterpret_cast<float*>(w8);
  w8 += align_up((size_t)s.n_kv_heads * p.n_chunks * 2 * dd * sizeof(float), 256);
  p.c64 = reinterpret_cast<double*>(w8);
  w8 += align_up((size_t)s.n_kv_heads * dd * sizeof(double), 256);
  p.status = reinterpret_cast<int*>(w8);
  if (s.dtype == VECTOR_BF16) {
    if (D == 128) return run_calibrate<bf16_t, 128>(s, p, stream);
    if (D == 64) return run_calibrate<bf16_t, 64>(s, p, stream);
  } else if (s.dtype == VECTOR_F32) {
    if (D == 128) return run_calibrate<float, 128>(s, p, stream);
    if (D == 64) return run_calibrate<float, 64>(s, p, stream);
  } else {
    return VECTOR_ERR_DTYPE;
  }
  return VECTOR_ERR_SHAPE;
}

}  // namespace vec
