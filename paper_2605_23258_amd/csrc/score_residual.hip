// Importance score (observation-window attention mass, pooled) and
// reconstruction residual ||v - k W||^2 for the VECTOR compression pass
// (Section 3.2, Steps 1 and 2).
//
// Data flow per KV head h (R = G*w query rows share the head's keys):
//   pass 1  score_stats   : S = Q_h K_h^T (MFMA), per-row running max / sum-exp
//                           over a chunk of tokens -> partial (m, l) per (row, chunk)
//   pass 2  mass_residual : prologue merges the chunk partials into one bias per row,
//                           bias_r = log2-domain max + log2(sum-exp); then S again,
//                           p = exp2(S*c - bias_r), column mean -> mass; fused on the
//                           same K registers: v_hat^T = W^T K^T (MFMA),
//                           eps = sum_j (v - v_hat)^2
//   pool                  : average or maximum pooling of mass over prefix columns, +inf on the
//                           window columns (route_bucket_kernel in route_compact.hip, which hands
//                           the routing its first histogram and bucket lists in the same launch)
//
// Pass 1 has two kernels: score_stats_tiles_kernel (R_pad = 128 or 256: key tiles through LDS,
// a wave keeps its block of Q_h and the rows' running statistics in registers) and
// score_stats_kernel (any row count: keys straight into operand registers, Q_h in LDS).
// In pass 2 K rows go straight from HBM into MFMA operand registers (16 bytes per lane); the
// next tile's rows are requested as soon as the last MFMA of the current tile has been issued;
// Q_h, W_h^T and the row biases live in LDS for the life of a workgroup.  MFMAs of row block
// i+1 are written between the exponentials of row block i: the vector port is the narrow
// resource of both passes, and a wave's MFMAs only hide under its own vector work when the two
// alternate in the instruction stream.  Both passes put all chunks of a KV head on one XCD, and
// pass 2 walks a chunk backwards, towards what pass 1 left in that XCD's L2.
// Template flags of pass 2: PROBE (repeat a tile's arithmetic on resident operands, for
// measuring the contraction alone), ROPE (keys are un-rotated by position for the residual).
#include "common.hpp"
#include "launch.hpp"

#ifndef VEC_P1_THREADS
#define VEC_P1_THREADS 1024
#define VEC_P1_SUBTILES 1
#endif

namespace vec {

namespace {

struct PassParams {
  const void* q;        // [Hq, w, d]
  const void* k;
  const void* v;
  const void* W;
  int64_t k_sh, k_st, v_sh, v_st, w_sh;   // element strides
  int hps;              // stacked sequences: KV heads per sequence (0: one sequence); head hv of the launch is
  int64_t k_sb, v_sb;   // KV head hv % hps of sequence hv / hps, sequences k_sb / v_sb elements apart
  int n, w, R, R_pad, n_prefix;
  // Query heads of a KV head taken a group at a time (when all G * w rows do not fit at once): this
  // launch sees R rows starting at row q_row0 of the head's q_head_rows = G * w rows, and its
  // column mass is added to what the earlier groups left.
  int q_head_rows, q_row0, accumulate;
  int tokens_per_chunk;  // pass 2: tokens per workgroup
  int tpc1, n_chunks;    // pass 1: tokens per workgroup, and the number of such chunks (= partials per row)
  int threads_per_row;  // pass-2 prologue: lanes that share the merge of one row's partials
  float c2;             // log2(e) / sqrt(d)
  float inv_R;
  float2* part;         // [Hkv, n_chunks, R_pad]  (max, sum-exp), log2 domain
  float* mass;          // [Hkv, n]
  float* eps;           // [Hkv, n]
  float4* range;        // [Hkv, range_stride] or null: every workgroup of pass 2 leaves, over the prefix columns
                        // it stored with a positive mass m, their count and the sums of l and l * l, where
                        // l = log2(m) - log_ref; the routing's bucket launch turns them into the head's
                        // typical score range
  int range_stride;     // entries of `range` per head (the second pass's workgroups per head)
  // Several sequences of different lengths in one launch (template flag RAGGED): the launch's
  // own parameters only say where the sequences' parameter blocks lie; launch head hv belongs
  // to sequence hv / seq_hps and is its head hv % seq_hps, and a workgroup whose chunk
  // index lies beyond its sequence's chunks leaves at once.
  int64_t pos_base;     // post-RoPE keys with a position array: token t of this head is at positions[pos_base + t]
                        // (+ the sequence's share when sequences are stacked)
  const PassParams* seq_table;
  int seq_hps;
  const float* lse;     // null, or the log-sum-exp (natural log, logits scaled by 1/sqrt(d)) of every query row,
  int64_t lse_sh;       // row r of query head hq at lse[hq * lse_sh + r]: then pass 2 needs no pass 1
  float log_ref;        // log2 of the mean mass of a prefix column, -log2(n_prefix): keeps l small
  int repeat;           // probe kernels only: times each tile's arithmetic is run on the same registers
};

// RAGGED launches: swap in the parameters of the sequence this workgroup belongs to
template <bool RAGGED>
__device__ __forceinline__ void take_sequence(PassParams& p, int& h) {
  if constexpr (RAGGED) {
    const int seq = h / p.seq_hps;
    h -= seq * p.seq_hps;
    p = p.seq_table[seq];
  }
}

// element offset of a launch head's keys (or values), and the KV head whose W it uses
__device__ __forceinline__ int64_t head_offset(const PassParams& p, int h, int64_t seq_stride, int64_t head_stride) {
  return p.hps ? (int64_t)(h / p.hps) * seq_stride + (int64_t)(h % p.hps) * head_stride : (int64_t)h * head_stride;
}
__device__ __forceinline__ int w_head(const PassParams& p, int h) { return p.hps ? h % p.hps : h; }

template <typename T, int D> struct Tile {
  static constexpr int E = Elem<T>::kPerChunk;
  static constexpr int NC = D / (2 * E);            // chunks per row
  static constexpr int kRowBytes = D * (int)sizeof(T);
  static constexpr int kLdsStride = kRowBytes + 16;  // pad: conflict-free 16-byte reads down a column of rows
  static constexpr int JB = D / 32;                  // 32-row blocks of the W^T K^T product
  static constexpr int VP = (D / 2) / E;             // 16-byte pieces of half a value row
  static constexpr int kMfmaPerChunk = (sizeof(T) == 2) ? 1 : 4;   // MFMA instructions per operand chunk
};

// Copy `rows` rows of D elements from global to LDS with the padded stride;
// rows in [rows, rows_pad) are zero-filled.  Loads go out eight at a time per thread so
// that their latencies overlap, and each workgroup starts at a different row (`rot`) so
// that the workgroups of one head, which all read the same rows at the same moment, do
// not queue up on the same cache lines.
template <typename T, int D, int NT>
__device__ __forceinline__ void fill_rows_lds(unsigned char* lds, const T* src, int rows, int rows_pad, int rot) {
  constexpr int P = Tile<T, D>::kRowBytes / 16;
  constexpr int U = 8;
  const int total = rows_pad * P;
  const int shift = (rot % rows_pad) * P;
  for (int base = threadIdx.x; base < total; base += NT * U) {
    uint4 x[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      int i = base + u * NT + shift;
      if (i >= total) i -= total;
      const int row = i / P, piece = i - row * P;
      // always load (from a clamped row) and blank afterwards: a load under a branch makes the
      // compiler wait for every earlier load as well
      x[u] = *reinterpret_cast<const uint4*>(reinterpret_cast<const unsigned char*>(src) + (size_t)min(row, rows - 1) * Tile<T, D>::kRowBytes + piece * 16);
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      int i = base + u * NT + shift;
      if (i >= total) i -= total;
      if (!(base + u * NT < total && i / P < rows)) x[u] = make_uint4(0, 0, 0, 0);
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      int i = base + u * NT + shift;
      if (i >= total) i -= total;
      const int row = i / P, piece = i - row * P;
      if (base + u * NT < total) *reinterpret_cast<uint4*>(lds + row * Tile<T, D>::kLdsStride + piece * 16) = x[u];
    }
  }
}

// fill_rows_lds in two halves, for a caller that has other work between the request and the use:
// the first batch of eight loads per thread goes out in fill_rows_request, fill_rows_finish
// stores it and runs the remaining batches (if the block has more than NT * 8 pieces).
template <typename T, int D, int NT>
__device__ __forceinline__ void fill_rows_request(uint4 (&x)[8], const T* src, int rows, int rows_pad, int rot) {
  constexpr int P = Tile<T, D>::kRowBytes / 16;
  const int total = rows_pad * P;
  const int shift = (rot % rows_pad) * P;
#pragma unroll
  for (int u = 0; u < 8; ++u) {
    int i = (int)threadIdx.x + u * NT + shift;
    if (i >= total) i -= total;
    i = min(i, total - 1);                       // threads beyond the block load a duplicate
    const int row = i / P, piece = i - row * P;
    x[u] = *reinterpret_cast<const uint4*>(reinterpret_cast<const unsigned char*>(src) + (size_t)min(row, rows - 1) * Tile<T, D>::kRowBytes + piece * 16);
  }
}
template <typename T, int D, int NT>
__device__ __forceinline__ void fill_rows_finish(uint4 (&x)[8], unsigned char* lds, const T* src, int rows, int rows_pad, int rot) {
  constexpr int P = Tile<T, D>::kRowBytes / 16;
  constexpr int U = 8;
  const int total = rows_pad * P;
  const int shift = (rot % rows_pad) * P;
#pragma unroll
  for (int u = 0; u < U; ++u) {
    int i = (int)threadIdx.x + u * NT + shift;
    if (i >= total) i -= total;
    const int row = i / P, piece = i - row * P;
    if ((int)threadIdx.x + u * NT < total)
      *reinterpret_cast<uint4*>(lds + row * Tile<T, D>::kLdsStride + piece * 16) = row < rows ? x[u] : make_uint4(0, 0, 0, 0);
  }
  for (int base = (int)threadIdx.x + NT * U; base < total; base += NT * U) {
    uint4 y[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      int i = base + u * NT + shift;
      if (i >= total) i -= total;
      const int row = i / P, piece = i - row * P;
      y[u] = *reinterpret_cast<const uint4*>(reinterpret_cast<const unsigned char*>(src) + (size_t)min(row, rows - 1) * Tile<T, D>::kRowBytes + piece * 16);
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      int i = base + u * NT + shift;
      if (i >= total) i -= total;
      const int row = i / P, piece = i - row * P;
      if (base + u * NT < total) *reinterpret_cast<uint4*>(lds + row * Tile<T, D>::kLdsStride + piece * 16) = row < rows ? y[u] : make_uint4(0, 0, 0, 0);
    }
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

__device__ __forceinline__ float max3(float a, float b, float c) { return fmaxf(fmaxf(a, b), c); }

// Pure arithmetic has no position of its own in the instruction stream: the compiler
// would issue a block's MFMAs back to back and its exponentials after them.  An empty
// volatile asm that "uses" an accumulator and the running sum ties both chains to this
// point, so what is written between two pins is also issued between them.
#define VEC_PIN(acc, x) asm volatile("" : "+v"(acc), "+v"(x))
#define VEC_PIN3(acc, x, y) asm volatile("" : "+v"(acc), "+v"(x), "+v"(y))

// ---------------------------------------------------------------------------
// pass 1: per-row softmax statistics over a chunk of tokens
// ---------------------------------------------------------------------------
template <typename T, int D, int NT, int NS, bool RAGGED = false>     // NS subtiles of 32 tokens per wave tile
__global__ __launch_bounds__(NT) void score_stats_kernel(PassParams p) {
  int h = blockIdx.y;
  take_sequence<RAGGED>(p, h);
  if (RAGGED && (int)blockIdx.x >= p.n_chunks) return;
  using TL = Tile<T, D>;
  constexpr int NW = NT / kWave;
  constexpr int TW = 32 * NS;                    // tokens per wave tile
  extern __shared__ __align__(16) unsigned char smem[];
  unsigned char* q_lds = smem;
  float2* st_lds = reinterpret_cast<float2*>(smem + (size_t)p.R_pad * TL::kLdsStride);   // [NW][NRB][64]

  const int chunk = blockIdx.x;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, half = lane >> 5, l31 = lane & 31;
  const int nrb = p.R_pad / 32;

  const T* k_head = reinterpret_cast<const T*>(p.k) + head_offset(p, h, p.k_sb, p.k_sh);
  const int c_begin = chunk * p.tpc1;
  const int c_end = min(p.n, c_begin + p.tpc1);
  constexpr int kStep = NW * TW;

  chunk_t kf[NS][TL::NC];
  auto load_keys = [&](int t) {
#pragma unroll
    for (int sI = 0; sI < NS; ++sI) load_k_subtile<T, D>(kf[sI], k_head, p.k_st, t + 32 * sI, p.n, lane);
  };
  int t0 = c_begin + wave * TW;
  if (t0 < c_end) load_keys(t0);          // first tile's keys fly while Q is staged
  fill_rows_lds<T, D, NT>(q_lds, reinterpret_cast<const T*>(p.q) + ((size_t)h * p.q_head_rows + p.q_row0) * D, p.R, p.R_pad, chunk * 8);
  for (int i = threadIdx.x; i < NW * nrb * 64; i += NT) st_lds[i] = make_float2(-INFINITY, 0.f);
  __syncthreads();

  float2* my_st = st_lds + (size_t)wave * nrb * 64 + lane;

  // logits of one row block against the wave's subtiles: rows = tokens, columns = query rows
  auto mma_rb = [&](f32x16 (&x)[NS], int rb) {
#pragma unroll
    for (int c = 0; c < TL::NC; ++c) {
      chunk_t qf = lds_chunk<T, D>(q_lds, rb * 32 + l31, c, half);
#pragma unroll
      for (int sI = 0; sI < NS; ++sI) {
        if (c == 0) mma_chunk_first<T>(x[sI], kf[sI][c], qf);
        else mma_chunk<T>(x[sI], kf[sI][c], qf);
      }
    }
  };
  auto tile_max = [&](const f32x16 (&x)[NS]) {     // short independent chains, not one long one
    float m = -INFINITY;
#pragma unroll
    for (int sI = 0; sI < NS; ++sI) {
      float m0 = max3(x[sI][0], x[sI][1], x[sI][2]), m1 = max3(x[sI][8], x[sI][9], x[sI][10]);
      m0 = max3(m0, x[sI][3], x[sI][4]); m1 = max3(m1, x[sI][11], x[sI][12]);
      m0 = max3(m0, x[sI][5], x[sI][6]); m1 = max3(m1, x[sI][13], x[sI][14]);
      m = max3(m, fmaxf(m0, x[sI][7]), fmaxf(m1, x[sI][15]));
    }
    return m * p.c2;                              // c2 > 0: scaling commutes with max
  };
  // fold the lane's logits of one row block into the running (max, sum-exp) of its query row
  auto stats_rb = [&](const f32x16 (&x)[NS], int rb) {
    const float tmax = tile_max(x);
    float2 st = my_st[rb * 64];
    const float m_new = fmaxf(st.x, tmax);
    const float m_safe = (m_new == -INFINITY) ? 0.f : m_new;
    float sum[2] = {0.f, 0.f};
#pragma unroll
    for (int sI = 0; sI < NS; ++sI)
#pragma unroll
      for (int v = 0; v < 16; ++v) sum[(sI + v) & 1] += fast_exp2(fmaf(x[sI][v], p.c2, -m_safe));
    st.y = st.y * fast_exp2(st.x - m_safe) + (sum[0] + sum[1]);
    st.x = m_new;
    my_st[rb * 64] = st;
  };
  // One pipelined step: the MFMAs of row block rb_n go out one at a time, each followed by
  // the exponentials of a few logits of row block rb_c, so that the matrix pipe works while
  // the vector ALU does.
  auto step = [&](f32x16 (&nx)[NS], int rb_n, const f32x16 (&cu)[NS], int rb_c) {
    const float tmax = tile_max(cu);
    float2 st = my_st[rb_c * 64];
    const float m_new = fmaxf(st.x, tmax);
    const float m_safe = (m_new == -INFINITY) ? 0.f : m_new;
    float sum0 = 0.f, sum1 = 0.f;
    chunk_t qf = lds_chunk<T, D>(q_lds, rb_n * 32 + l31, 0, half);
#pragma unroll
    for (int c = 0; c < TL::NC; ++c) {
      const chunk_t q_now = qf;
      if (c + 1 < TL::NC) qf = lds_chunk<T, D>(q_lds, rb_n * 32 + l31, c + 1, half);
#pragma unroll
      for (int sI = 0; sI < NS; ++sI) {
        constexpr int kSlots = TL::NC * NS;
        const int slot = c * NS + sI;
        if (c == 0) mma_chunk_first<T>(nx[sI], kf[sI][c], q_now);
        else mma_chunk<T>(nx[sI], kf[sI][c], q_now);
#pragma unroll
        for (int v = slot * 16 / kSlots; v < (slot + 1) * 16 / kSlots; ++v)
#pragma unroll
          for (int s2 = 0; s2 < NS; ++s2) {
            const float e = fast_exp2(fmaf(cu[s2][v], p.c2, -m_safe));
            if ((s2 + v) & 1) sum1 += e; else sum0 += e;
          }
        VEC_PIN3(nx[sI], sum0, sum1);
      }
    }
    st.y = st.y * fast_exp2(st.x - m_safe) + (sum0 + sum1);
    st.x = m_new;
    my_st[rb_c * 64] = st;
  };

  while (t0 < c_end) {
    const int tn = t0 + kStep;
    // a tile needs masking if it reaches past the first window position or past the chunk
    const bool tail = (t0 + TW > p.n_prefix + 1) || (t0 + TW > c_end);
    f32x16 A[NS], B[NS];
    if (!tail) {
      mma_rb(A, 0);
      int rb = 0;
      for (; rb + 2 < nrb; rb += 2) {
        step(B, rb + 1, A, rb);
        step(A, rb + 2, B, rb + 1);
      }
      if (rb + 1 < nrb) {
        step(B, rb + 1, A, rb);
        if (tn < c_end) load_keys(tn);     // every MFMA of the tile is issued: fetch the next keys
        stats_rb(B, rb + 1);
      } else {
        if (tn < c_end) load_keys(tn);
        stats_rb(A, rb);
      }
    } else {
      for (int rb = 0; rb < nrb; ++rb) {
        mma_rb(A, rb);
        // query row (g, r) sits at position n - w + r and sees tokens <= that
        const int qrow = rb * 32 + l31;
        const int last = (qrow < p.R) ? min(p.n_prefix + (qrow % p.w), c_end - 1) : c_end - 1;
#pragma unroll
        for (int sI = 0; sI < NS; ++sI)
#pragma unroll
          for (int v = 0; v < 16; ++v)
            if (t0 + 32 * sI + acc_row(v, half) > last) A[sI][v] = -INFINITY;
        stats_rb(A, rb);
      }
      if (tn < c_end) load_keys(tn);
    }
    t0 = tn;
  }
  __syncthreads();
  // merge the NW waves x 2 lane halves that saw different tokens of the same query row
  float2* out = p.part + ((size_t)h * p.n_chunks + chunk) * p.R_pad;     // [head][chunk][row]: rows of a chunk side by side
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

// ---------------------------------------------------------------------------
// pass 1, key tiles through LDS: for R_pad = 128 or 256 (4 or 8 row blocks)
// ---------------------------------------------------------------------------
// Eight waves; a wave owns one or two 32-row blocks of Q_h for the whole launch and keeps them
// in registers as B operands, so its lanes carry the running (max, sum-exp) of their own
// query rows in registers too.  The keys of the chunk stream through LDS in 64-token
// tiles per token group (the waves that own the same rows form the groups, which work on
// different tiles): all 512 threads load a step's tiles with 16-byte loads, 16 adjacent lanes
// per row, one step ahead of the one being consumed (double buffered, one barrier per step),
// and every wave of a token group reads its tile back in operand order.  With two row blocks
// per wave (256 bf16 rows) an operand chunk read from LDS feeds two MFMAs of independent
// chains: half the LDS traffic per MFMA, and no MFMA waits for the one before it.
// Compared with score_stats_kernel the key loads are fully coalesced, overlap with the
// arithmetic, and no statistics pass through LDS.
constexpr int kV2TileTokens = 64;
constexpr int kV2Threads = 512;
// row blocks per wave, and the token groups that follow from it
constexpr int tiles_blocks_per_wave(int nrb, int elem_bytes) { return (nrb == 8 && elem_bytes == 2) ? 2 : 1; }
constexpr int tiles_token_groups(int nrb, int elem_bytes) {
  return (kV2Threads / kWave) / (nrb / tiles_blocks_per_wave(nrb, elem_bytes));
}

template <typename T, int D, int NRB, bool RAGGED = false>
__global__ __launch_bounds__(kV2Threads) void score_stats_tiles_kernel(PassParams p) {
  int chunk, h;
  if (RAGGED) { chunk = blockIdx.x; h = blockIdx.y; }
  else xcd_chunk_head(chunk, h);
  take_sequence<RAGGED>(p, h);
  if (RAGGED && chunk >= p.n_chunks) return;
  using TL = Tile<T, D>;
  constexpr int NT = kV2Threads;
  constexpr int NW = NT / kWave;
  constexpr int RBW = tiles_blocks_per_wave(NRB, (int)sizeof(T));   // row blocks per wave
  constexpr int NRW = NRB / RBW;                     // waves that cover all rows
  constexpr int TG = NW / NRW;                       // token groups
  constexpr int NC = TL::NC;
  constexpr int kStepTokens = TG * kV2TileTokens;
  constexpr int kPieces = TL::kRowBytes / 16;        // 16-byte pieces per key row
  constexpr int kLoads = kStepTokens * kPieces / NT; // pieces per thread and step
  static_assert(NW % NRW == 0 && (kStepTokens * kPieces) % NT == 0, "tile shape");
  constexpr int kBufBytes = kStepTokens * TL::kLdsStride;
  extern __shared__ __align__(16) unsigned char smem[];

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, half = lane >> 5, l31 = lane & 31;
  const int rw = wave % NRW, tg = wave / NRW;
  const T* k_head = reinterpret_cast<const T*>(p.k) + head_offset(p, h, p.k_sb, p.k_sh);
  const int c_begin = chunk * p.tpc1;
  const int c_end = min(p.n, c_begin + p.tpc1);
  const int n_steps = (c_end - c_begin + kStepTokens - 1) / kStepTokens;

  // piece i of a step: token i / kPieces of the step, 16 bytes at piece i % kPieces.  A thread's
  // pieces sit at fixed byte offsets from the step's first row, worked out once; a step moves
  // them by a whole number of rows (one scalar product per step, no 64-bit vector multiplies in
  // the loop).  Only a step that reaches past the sequence's end clamps its rows one by one.
  int64_t piece_off[kLoads];
#pragma unroll
  for (int u = 0; u < kLoads; ++u) {
    const int i = threadIdx.x + u * NT;
    piece_off[u] = ((int64_t)(i / kPieces) * p.k_st) * (int64_t)sizeof(T) + (i % kPieces) * 16;
  }
  auto fetch = [&](uint4* raw, int step) {
    const int row0 = c_begin + step * kStepTokens;
    if (row0 + kStepTokens <= p.n) {                 // uniform
      const unsigned char* base = reinterpret_cast<const unsigned char*>(k_head + (int64_t)row0 * p.k_st);
#pragma unroll
      for (int u = 0; u < kLoads; ++u) raw[u] = load_chunk(base + piece_off[u]);
    } else {
#pragma unroll
      for (int u = 0; u < kLoads; ++u) {
        const int i = threadIdx.x + u * NT;
        const int t = min(row0 + i / kPieces, p.n - 1);                          // clamped: masked below
        raw[u] = load_chunk(reinterpret_cast<const unsigned char*>(k_head + (int64_t)t * p.k_st) + (i % kPieces) * 16);
      }
    }
  };
  auto stash = [&](const uint4* raw, int buf) {
#pragma unroll
    for (int u = 0; u < kLoads; ++u) {
      const int i = threadIdx.x + u * NT;
      *reinterpret_cast<uint4*>(smem + buf * kBufBytes + (i / kPieces) * TL::kLdsStride + (i % kPieces) * 16) = raw[u];
    }
  };

  // Key tiles are requested kAhead steps before they are consumed (a step's arithmetic is
  // shorter than a trip to HBM); they wait in registers and enter LDS one step ahead.  The first
  // tile is asked for before anything else: the launch's first MFMA waits for it longest.
  constexpr int kAhead = (kLoads > 2) ? 2 : 3;
  uint4 raw[kAhead][kLoads];
  fetch(raw[0], 0);
  // this wave's query rows: B operands, zero beyond R
  chunk_t qf[RBW][NC];
  int qrow[RBW];
#pragma unroll
  for (int j = 0; j < RBW; ++j) {
    qrow[j] = (rw * RBW + j) * 32 + l31;
    const T* qrow_p = reinterpret_cast<const T*>(p.q) + ((size_t)h * p.q_head_rows + p.q_row0 + min(qrow[j], p.R - 1)) * D;
#pragma unroll
    for (int c = 0; c < NC; ++c) {
      qf[j][c] = load_chunk(qrow_p + chunk_elem_offset<T>(c, half));
      if (qrow[j] >= p.R) qf[j][c] = make_uint4(0, 0, 0, 0);
    }
  }
#pragma unroll
  for (int a = 1; a < kAhead; ++a)
    if (a < n_steps) fetch(raw[a], a);
  // of query rows qrow[j], over this lane half's tokens
  float m_run[RBW], l_run[RBW];
#pragma unroll
  for (int j = 0; j < RBW; ++j) { m_run[j] = -INFINITY; l_run[j] = 0.f; }
  // rows = tokens, columns = query rows
  auto tile_max1 = [&](const f32x16& x) {
    float m0 = max3(x[0], x[1], x[2]), m1 = max3(x[8], x[9], x[10]);
    m0 = max3(m0, x[3], x[4]); m1 = max3(m1, x[11], x[12]);
    m0 = max3(m0, x[5], x[6]); m1 = max3(m1, x[13], x[14]);
    return fmaxf(fmaxf(m0, x[7]), fmaxf(m1, x[15])) * p.c2;
  };
  auto fold = [&](const f32x16& x, int j) {
    const float m_new = fmaxf(m_run[j], tile_max1(x));
    const float m_safe = (m_new == -INFINITY) ? 0.f : m_new;
    float s0 = 0.f, s1 = 0.f;
#pragma unroll
    for (int v = 0; v < 16; v += 2) {
      s0 += fast_exp2(fmaf(x[v], p.c2, -m_safe));
      s1 += fast_exp2(fmaf(x[v + 1], p.c2, -m_safe));
    }
    l_run[j] = l_run[j] * fast_exp2(m_run[j] - m_safe) + (s0 + s1);
    m_run[j] = m_new;
  };
  // MFMAs of one subtile (for every row block of the wave), one operand chunk at a time, each
  // followed by its share of the exponentials of a subtile that is already complete: the matrix
  // pipe works through the new products while the vector ALU folds the finished ones into the
  // running statistics
  auto mma_fold = [&](auto refill_tag, f32x16* nx, chunk_t* kf, f32x16* cu, const unsigned char* refill) {
    constexpr bool kRefill = decltype(refill_tag)::value;
    float m_new[RBW], m_safe[RBW], s0[RBW], s1[RBW];
#pragma unroll
    for (int c = 0; c < NC; ++c) {
#pragma unroll
      for (int j = 0; j < RBW; ++j) {
        if (c == 0) mma_chunk_first<T>(nx[j], kf[c], qf[j][c]);
        else mma_chunk<T>(nx[j], kf[c], qf[j][c]);
        // the next subtile's chunk, into the registers just read for the last time
        if (kRefill && j == RBW - 1) kf[c] = lds_chunk<T, D>(refill, 32 + l31, c, half);
        if (c == 0) {
          // the finished subtile's row maxima wait for its last MFMA: taken once the new subtile's
          // first MFMA is in the pipe, not before
          VEC_PIN(nx[j], cu[j]);
          m_new[j] = fmaxf(m_run[j], tile_max1(cu[j]));
          m_safe[j] = (m_new[j] == -INFINITY) ? 0.f : m_new[j];
          s0[j] = 0.f; s1[j] = 0.f;
        }
#pragma unroll
        for (int v = c * 16 / NC; v < (c + 1) * 16 / NC; ++v) {
          const float e = fast_exp2(fmaf(cu[j][v], p.c2, -m_safe[j]));
          if (v & 1) s1[j] += e; else s0[j] += e;
        }
        VEC_PIN3(nx[j], s0[j], s1[j]);
      }
    }
#pragma unroll
    for (int j = 0; j < RBW; ++j) {
      l_run[j] = l_run[j] * fast_exp2(m_run[j] - m_safe[j]) + (s0[j] + s1[j]);
      m_run[j] = m_new[j];
    }
  };

  // The second subtile of a step is folded during the first subtile's MFMAs of the next step,
  // so `pend` carries products across steps; all -inf folds to nothing.
  f32x16 pend[RBW];
#pragma unroll
  for (int j = 0; j < RBW; ++j)
#pragma unroll
    for (int v = 0; v < 16; ++v) pend[j][v] = -INFINITY;
  auto compute = [&](int step) {
    const unsigned char* tile = smem + (step & 1) * kBufBytes + tg * kV2TileTokens * TL::kLdsStride;
    const int t0 = c_begin + step * kStepTokens + tg * kV2TileTokens;
    if (t0 < c_end) {
      // the first subtile in operand order, requested before the first MFMA; the second subtile's
      // chunks follow into the same registers as the first one's are consumed
      chunk_t kf[NC];
#pragma unroll
      for (int c = 0; c < NC; ++c) kf[c] = lds_chunk<T, D>(tile, l31, c, half);
      f32x16 A[RBW];
      // a tile needs masking if it reaches past the first window position or past the chunk
      const bool tail = (t0 + kV2TileTokens > p.n_prefix + 1) || (t0 + kV2TileTokens > c_end);
      if (!tail) {
        mma_fold(std::true_type{}, A, kf, pend, tile);
        mma_fold(std::false_type{}, pend, kf, A, tile);
      } else {
        // query row (g, r) sits at position n - w + r and sees tokens <= that
        int last[RBW];
#pragma unroll
        for (int j = 0; j < RBW; ++j) last[j] = (qrow[j] < p.R) ? min(p.n_prefix + (qrow[j] % p.w), c_end - 1) : c_end - 1;
        mma_fold(std::true_type{}, A, kf, pend, tile);
#pragma unroll
        for (int j = 0; j < RBW; ++j)
#pragma unroll
          for (int v = 0; v < 16; ++v)
            if (t0 + acc_row(v, half) > last[j]) A[j][v] = -INFINITY;
        mma_fold(std::false_type{}, pend, kf, A, tile);
#pragma unroll
        for (int j = 0; j < RBW; ++j)
#pragma unroll
          for (int v = 0; v < 16; ++v)
            if (t0 + 32 + acc_row(v, half) > last[j]) pend[j][v] = -INFINITY;
      }
    }
  };
  stash(raw[0], 0);
  for (int step0 = 0; step0 < n_steps; step0 += kAhead) {
#pragma unroll
    for (int a = 0; a < kAhead; ++a) {               // ring slot a holds tile step0 + a
      const int step = step0 + a;
      if (step < n_steps) {
        __syncthreads();                   // tile `step` is in its buffer; the other buffer is free
        if (step + kAhead < n_steps) fetch(raw[a], step + kAhead);      // slot a was stashed a step ago
        compute(step);
        if (step + 1 < n_steps) stash(raw[(a + 1) % kAhead], (step + 1) & 1);
      }
    }
  }
  // the last pending subtile; then merge the two lane halves, then the token groups: one (max, sum) per (row, chunk)
#pragma unroll
  for (int j = 0; j < RBW; ++j) {
    fold(pend[j], j);
    const float m2 = __shfl_xor(m_run[j], 32, kWave), l2 = __shfl_xor(l_run[j], 32, kWave);
    const float mn = fmaxf(m_run[j], m2);
    const float ms = (mn == -INFINITY) ? 0.f : mn;
    l_run[j] = l_run[j] * fast_exp2(m_run[j] - ms) + l2 * fast_exp2(m2 - ms);
    m_run[j] = mn;
  }
  __syncthreads();                         // tiles are dead: reuse LDS for the group merge
  float2* grp = reinterpret_cast<float2*>(smem);     // [TG][NRB * 32]
#pragma unroll
  for (int j = 0; j < RBW; ++j)
    if (half == 0) grp[tg * (NRB * 32) + qrow[j]] = make_float2(m_run[j], l_run[j]);
  __syncthreads();
  float2* out = p.part + ((size_t)h * p.n_chunks + chunk) * p.R_pad;     // [head][chunk][row]: rows of a chunk side by side
  for (int row = threadIdx.x; row < NRB * 32; row += NT) {
    float m = -INFINITY;
#pragma unroll
    for (int g = 0; g < TG; ++g) m = fmaxf(m, grp[g * (NRB * 32) + row].x);
    const float ms = (m == -INFINITY) ? 0.f : m;
    float l = 0.f;
#pragma unroll
    for (int g = 0; g < TG; ++g) {
      const float2 sv = grp[g * (NRB * 32) + row];
      l += sv.y * fast_exp2(sv.x - ms);
    }
    out[row] = make_float2(m, l);
  }
}

// ---------------------------------------------------------------------------
// pass 2: column mass of the normalised probabilities, and/or the residual
// ---------------------------------------------------------------------------
template <typename T> struct Unpack;
template <> struct Unpack<bf16_t> {   // 16 bytes -> 8 floats
  static __device__ __forceinline__ void run(const uint4& r, float* f) {
    f[0] = bf16_lo(r.x); f[1] = bf16_hi(r.x); f[2] = bf16_lo(r.y); f[3] = bf16_hi(r.y);
    f[4] = bf16_lo(r.z); f[5] = bf16_hi(r.z); f[6] = bf16_lo(r.w); f[7] = bf16_hi(r.w);
  }
};
template <> struct Unpack<float> {    // 16 bytes -> 4 floats
  static __device__ __forceinline__ void run(const uint4& r, float* f) {
    f[0] = __uint_as_float(r.x); f[1] = __uint_as_float(r.y); f[2] = __uint_as_float(r.z); f[3] = __uint_as_float(r.w);
  }
};

// 16 bytes of un-rotated key elements back into operand form.  bf16 operands cannot hold
// the turned-back values exactly, so they go to the matrix core twice: the rounded value and
// the remainder of that rounding (about 2^-17 relative together).
template <typename T> struct SplitPack;
template <> struct SplitPack<bf16_t> {
  static constexpr bool kTwoParts = true;
  static __device__ __forceinline__ void run(const float* f, chunk_t& hi, chunk_t& lo) {
    uint32_t h[4], l[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      h[e] = pack_bf16(f[2 * e], f[2 * e + 1]);
      l[e] = pack_bf16(f[2 * e] - bf16_lo(h[e]), f[2 * e + 1] - bf16_hi(h[e]));
    }
    hi = make_uint4(h[0], h[1], h[2], h[3]);
    lo = make_uint4(l[0], l[1], l[2], l[3]);
  }
};
template <> struct SplitPack<float> {
  static constexpr bool kTwoParts = false;
  static __device__ __forceinline__ void run(const float* f, chunk_t& hi, chunk_t& lo) {
    hi = make_uint4(__float_as_uint(f[0]), __float_as_uint(f[1]), __float_as_uint(f[2]), __float_as_uint(f[3]));
    lo = make_uint4(0, 0, 0, 0);
  }
};

// Operand registers of a 32-token subtile with the rotary embedding of the lane's token
// (at position pos) taken back out.  A lane holds elements c*2E + half*E + e of its row
// (chunk c, element e), so both partners of a rotary pair sit in the same lane: chunks c and
// c + NC/2 for pairs (i, i + d/2), neighbours inside a chunk for pairs (2i, 2i + 1).
template <typename T, int D>
__device__ __forceinline__ void unrotate_subtile(const chunk_t* kf, float pos, const float2* turns, int interleaved, int half,
                                                 chunk_t* kh, chunk_t* kl) {
  constexpr int E = Tile<T, D>::E, NC = Tile<T, D>::NC;
  if (!interleaved) {
#pragma unroll
    for (int c = 0; c < NC / 2; ++c) {
      float a[E], b[E];
      Unpack<T>::run(kf[c], a);
      Unpack<T>::run(kf[c + NC / 2], b);
#pragma unroll
      for (int e = 0; e < E; ++e) {
        float cs, sn;
        const float2 t = turns[c * 2 * E + half * E + e];
        rotary_cos_sin(pos, t.x, t.y, cs, sn);
        rotary_back(a[e], b[e], cs, sn, a[e], b[e]);
      }
      SplitPack<T>::run(a, kh[c], kl[c]);
      SplitPack<T>::run(b, kh[c + NC / 2], kl[c + NC / 2]);
      __builtin_amdgcn_sched_barrier(0);        // one chunk pair at a time: keeps the live set small
    }
  } else {
#pragma unroll
    for (int c = 0; c < NC; ++c) {
      float f[E];
      Unpack<T>::run(kf[c], f);
#pragma unroll
      for (int e = 0; e < E; e += 2) {
        float cs, sn;
        const float2 t = turns[(c * 2 * E + half * E + e) / 2];
        rotary_cos_sin(pos, t.x, t.y, cs, sn);
        rotary_back(f[e], f[e + 1], cs, sn, f[e], f[e + 1]);
      }
      SplitPack<T>::run(f, kh[c], kl[c]);
      __builtin_amdgcn_sched_barrier(0);
    }
  }
}

// Value registers of a 32-token subtile: lane (token l & 31, half l >> 5) holds the
// contiguous half row v[token][half*D/2, +D/2) as VP pieces of 16 bytes.
template <typename T, int D>
__device__ __forceinline__ void load_v_subtile(chunk_t* vf, const T* v_head, int64_t v_st, int t0, int n, int lane) {
  int t = min(t0 + (lane & 31), n - 1);
  const T* row = v_head + (int64_t)t * v_st + (lane >> 5) * (D / 2);
#pragma unroll
  for (int i = 0; i < Tile<T, D>::VP; ++i) vf[i] = load_chunk(row + i * Tile<T, D>::E);
}

// PROBE: the tile loop re-runs each tile's arithmetic p.repeat times on the operands it already
// holds (no further loads), to time the contraction code with memory out of the picture.
// ROPE: the keys are cached after rotary position embedding; the residual un-rotates them
// (the scores use them as cached).
template <typename T, int D, int NT, bool DO_MASS, bool DO_RES, bool PROBE = false, bool ROPE = false, bool RAGGED = false>
__global__ __launch_bounds__(NT) void mass_residual_kernel(PassParams p, RopeParams rp) {
  int chunk, h;
  if (RAGGED) { chunk = blockIdx.x; h = blockIdx.y; }
  else xcd_chunk_head(chunk, h);
  take_sequence<RAGGED>(p, h);
  if (RAGGED && chunk * p.tokens_per_chunk >= p.n) return;
  using TL = Tile<T, D>;
  constexpr int NW = NT / kWave;
  constexpr int JB = TL::JB;
  constexpr int E = TL::E;
  extern __shared__ __align__(16) unsigned char smem[];
  unsigned char* q_lds = smem;                                               // DO_MASS: [R_pad] rows
  size_t off = DO_MASS ? (size_t)p.R_pad * TL::kLdsStride : 0;
  float* bias_lds = reinterpret_cast<float*>(smem + off);                    // DO_MASS: [R_pad]
  off += DO_MASS ? (size_t)p.R_pad * sizeof(float) : 0;
  unsigned char* wt_lds = smem + off;                                        // DO_RES: [D] rows of W^T, permuted
  off += DO_RES ? (size_t)D * TL::kLdsStride : 0;
  float2* turns_lds = reinterpret_cast<float2*>(smem + off);                 // ROPE: [D/2] rotary frequencies (hi, lo)

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, half = lane >> 5, l31 = lane & 31;
  const int nrb = p.R_pad / 32;

  const T* k_head = reinterpret_cast<const T*>(p.k) + head_offset(p, h, p.k_sb, p.k_sh);
  const T* v_head = DO_RES ? reinterpret_cast<const T*>(p.v) + head_offset(p, h, p.v_sb, p.v_sh) : nullptr;
  const int c_begin = chunk * p.tokens_per_chunk;
  const int c_end = min(p.n, c_begin + p.tokens_per_chunk);
  // the mass of window columns is never used: stop the score part at the prefix
  const int mass_end = min(c_end, p.n_prefix);
  constexpr int kStep = NW * 64;

  // A wave takes its tiles from the chunk's end towards its start: the first pass read the chunk
  // forwards on the same XCD, so what is left of the keys in that L2 is the chunk's end.
  chunk_t kf0[TL::NC], kf1[TL::NC];
  const int t_first = c_begin + wave * 64;
  int t0 = t_first < c_end ? t_first + (c_end - t_first - 1) / kStep * kStep : t_first - kStep;

  // Prologue: every global load of the staging below is issued before the first result is
  // used, so the workgroup pays one memory round trip, not one per stage.
  constexpr int WU = (D * D / E + NT - 1) / NT;          // 16-byte pieces of W per thread
  union WPiece { uint4 raw; T el[E]; };
  WPiece wpiece[WU];
  if (DO_RES) {
    const T* Wh = reinterpret_cast<const T*>(p.W) + (int64_t)w_head(p, h) * p.w_sh;
#pragma unroll
    for (int u = 0; u < WU; ++u) {
      const int i = min(threadIdx.x + u * NT, D * D / E - 1);      // clamped: the store below is guarded
      wpiece[u].raw = load_chunk(Wh + (size_t)(i / (D / E)) * D + (i % (D / E)) * E);
    }
  }
  // pass 1's chunk partials of this thread's row: `tpr` adjacent lanes share one row and
  // each takes every tpr-th chunk; the first kPre of them are requested here
  constexpr int kPre = 16;
  const int tpr = p.threads_per_row, sub = threadIdx.x % tpr;
  const int rows_per_sweep = NT / tpr;
  float2 pre[kPre];
  uint4 q_first[8];
  const T* q_rows = reinterpret_cast<const T*>(p.q) + ((size_t)h * p.q_head_rows + p.q_row0) * D;
  if (DO_MASS) {
    if (!p.lse) {
      const int row = min((int)threadIdx.x / tpr, p.R_pad - 1);      // threads beyond R_pad rows load a duplicate
      const float2* part = p.part + (size_t)h * p.n_chunks * p.R_pad + row;
#pragma unroll
      for (int u = 0; u < kPre; ++u) pre[u] = part[(size_t)min(sub + u * tpr, p.n_chunks - 1) * p.R_pad];   // blanked when folded
    }
    fill_rows_request<T, D, NT>(q_first, q_rows, p.R, p.R_pad, chunk * 8);
  }
  // The first tile's keys are asked for after the staged operands (loads return in the order
  // they were issued: ahead of the staging loads, the keys' trip to HBM would hold up everything
  // below); they fly while W^T is laid out, the partials are merged and the query rows stored.
  if (t0 >= t_first) {
    load_k_subtile<T, D>(kf0, k_head, p.k_st, t0, p.n, lane);
    load_k_subtile<T, D>(kf1, k_head, p.k_st, t0 + 32, p.n, lane);
  }
  if (DO_RES) {
    // W^T into LDS as the M-side operand.  MFMA row m of block jb stands for value dim
    //   j = hf*(D/2) + jb*16 + (m >> 3)*4 + (m & 3),  hf = (m >> 2) & 1,
    // which makes accumulator register v of a lane in half hf hold dim hf*(D/2) + jb*16 + v:
    // exactly the contiguous half row of v that the lane loads.
#pragma unroll
    for (int u = 0; u < WU; ++u) {
      const int i = threadIdx.x + u * NT, din = i / (D / E), j0 = (i % (D / E)) * E;
      if (i < D * D / E) {
#pragma unroll
        for (int e = 0; e < E; ++e) {
          const int j = j0 + e;
          const int hf = j / (D / 2), r = j % (D / 2), jb = r >> 4, q16 = r & 15;
          const int m = (q16 >> 2) * 8 + hf * 4 + (q16 & 3);
          *reinterpret_cast<T*>(wt_lds + (jb * 32 + m) * TL::kLdsStride + din * (int)sizeof(T)) = wpiece[u].el[e];
        }
      }
    }
  }
  if (DO_MASS) {
    // Merge the partials: bias = max + log2(sum-exp); padded rows get +inf so that they add
    // exp2(-inf) = 0 to every column.
    auto fold = [](float& m, float& l, float m2, float l2) {
      const float mn = fmaxf(m, m2);
      const float ms = (mn == -INFINITY) ? 0.f : mn;
      l = l * fast_exp2(m - ms) + l2 * fast_exp2(m2 - ms);
      m = mn;
    };
    if (p.lse) {                              // the caller's log-sum-exp, turned into the log2 domain of the logits
      for (int row = threadIdx.x; row < p.R_pad; row += NT) {
        const int qr = p.q_row0 + row, g = qr / p.w, r = qr - g * p.w;
        bias_lds[row] = (row < p.R) ? p.lse[((int64_t)h * (p.q_head_rows / p.w) + g) * p.lse_sh + r] * kLog2e : INFINITY;
      }
    }
    // a batch of partials at once: their maximum first, then the sum against it (independent
    // exponentials, no chain from one partial to the next), then one fold into the running pair
    auto fold_batch = [&](float& m, float& l, const float2* sv, int count_in, int stride_in, int first_in, int nb) {
      float bm = -INFINITY;
#pragma unroll
      for (int u = 0; u < 16; ++u)
        if (u < nb && first_in + u * stride_in < count_in) bm = fmaxf(bm, sv[u].x);
      const float bs = (bm == -INFINITY) ? 0.f : bm;
      float bl = 0.f;
#pragma unroll
      for (int u = 0; u < 16; ++u)
        if (u < nb && first_in + u * stride_in < count_in) bl += sv[u].y * fast_exp2(sv[u].x - bs);
      fold(m, l, bm, bl);
    };
    for (int row0 = 0; !p.lse && row0 < p.R_pad; row0 += rows_per_sweep) {
      const int row = row0 + threadIdx.x / tpr;
      float m = -INFINITY, l = 0.f;
      if (row < p.R_pad) {
        const float2* part = p.part + (size_t)h * p.n_chunks * p.R_pad + row;
        int c_from = sub;
        if (row0 == 0) {                       // the preloaded ones
          fold_batch(m, l, pre, p.n_chunks, tpr, sub, kPre);
          c_from = sub + kPre * tpr;
        }
        for (int c0 = c_from; c0 < p.n_chunks; c0 += 8 * tpr) {       // the rest, eight loads in flight at a time
          float2 sv[16];
#pragma unroll
          for (int u = 0; u < 8; ++u) sv[u] = part[(size_t)min(c0 + u * tpr, p.n_chunks - 1) * p.R_pad];
          fold_batch(m, l, sv, p.n_chunks, tpr, c0, 8);
        }
      }
      for (int o = 1; o < tpr; o <<= 1) {
        const float m2 = __shfl_xor(m, o, kWave), l2 = __shfl_xor(l, o, kWave);
        fold(m, l, m2, l2);
      }
      if (sub == 0 && row < p.R_pad) bias_lds[row] = (row < p.R) ? m + __builtin_amdgcn_logf(l) : INFINITY;
    }
    fill_rows_finish<T, D, NT>(q_first, q_lds, q_rows, p.R, p.R_pad, chunk * 8);
  }
  if (ROPE && threadIdx.x < D / 2) turns_lds[threadIdx.x] = make_float2(rp.turns_hi[threadIdx.x], rp.turns_lo[threadIdx.x]);
  // The first tile's values are asked for before the barrier: memory keeps working while the
  // workgroup waits for its slowest wave, and no wave starts its first tile stuck behind sixteen
  // loads in a queue that the keys of all eight waves still fill.
  chunk_t vf0[TL::VP], vf1[TL::VP];
  bool values_requested = false;
  if (DO_RES && !ROPE && t0 >= t_first) {
    load_v_subtile<T, D>(vf0, v_head, p.v_st, t0, p.n, lane);
    load_v_subtile<T, D>(vf1, v_head, p.v_st, t0 + 32, p.n, lane);
    values_requested = true;
  }
  __syncthreads();

  // ---- score part: rows = query rows, columns = tokens ----
  auto mass_mma = [&](f32x16& x0, f32x16& x1, int rb) {
#pragma unroll
    for (int c = 0; c < TL::NC; ++c) {
      chunk_t qf = lds_chunk<T, D>(q_lds, rb * 32 + l31, c, half);
      if (c == 0) { mma_chunk_first<T>(x0, qf, kf0[c]); mma_chunk_first<T>(x1, qf, kf1[c]); }
      else { mma_chunk<T>(x0, qf, kf0[c]); mma_chunk<T>(x1, qf, kf1[c]); }
    }
  };
  auto mass_valu = [&](const f32x16& x0, const f32x16& x1, int rb, float& col0, float& col1) {
#pragma unroll
    for (int g4 = 0; g4 < 4; ++g4) {
      f32x4 b = *reinterpret_cast<const f32x4*>(bias_lds + rb * 32 + g4 * 8 + half * 4);
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        col0 += fast_exp2(fmaf(x0[g4 * 4 + i], p.c2, -b[i]));
        col1 += fast_exp2(fmaf(x1[g4 * 4 + i], p.c2, -b[i]));
      }
    }
  };
  // MFMAs of row block rb_n one at a time, each followed by exponentials of row block rb_c
  auto mass_step = [&](f32x16& n0, f32x16& n1, int rb_n, const f32x16& c0, const f32x16& c1, int rb_c,
                       float& col0, float& col1) {
    float b[16];
#pragma unroll
    for (int g4 = 0; g4 < 4; ++g4) {
      f32x4 bb = *reinterpret_cast<const f32x4*>(bias_lds + rb_c * 32 + g4 * 8 + half * 4);
#pragma unroll
      for (int i = 0; i < 4; ++i) b[g4 * 4 + i] = bb[i];
    }
    chunk_t qf = lds_chunk<T, D>(q_lds, rb_n * 32 + l31, 0, half);
#pragma unroll
    for (int c = 0; c < TL::NC; ++c) {
      const chunk_t q_now = qf;
      if (c + 1 < TL::NC) qf = lds_chunk<T, D>(q_lds, rb_n * 32 + l31, c + 1, half);
      const int lo = c * 16 / TL::NC, hi = (c + 1) * 16 / TL::NC, mid = lo + (hi - lo + 1) / 2;
      if (c == 0) mma_chunk_first<T>(n0, q_now, kf0[c]);
      else mma_chunk<T>(n0, q_now, kf0[c]);
#pragma unroll
      for (int v = lo; v < mid; ++v) {
        col0 += fast_exp2(fmaf(c0[v], p.c2, -b[v]));
        col1 += fast_exp2(fmaf(c1[v], p.c2, -b[v]));
      }
      VEC_PIN3(n0, col0, col1);
      if (c == 0) mma_chunk_first<T>(n1, q_now, kf1[c]);
      else mma_chunk<T>(n1, q_now, kf1[c]);
#pragma unroll
      for (int v = mid; v < hi; ++v) {
        col0 += fast_exp2(fmaf(c0[v], p.c2, -b[v]));
        col1 += fast_exp2(fmaf(c1[v], p.c2, -b[v]));
      }
      VEC_PIN3(n1, col0, col1);
    }
  };

  // ---- residual part: rows = value dims, columns = tokens; block bi = subtile * JB + jb ----
  auto res_mma = [&](f32x16& a, int bi) {
    const chunk_t* kf = (bi / JB) ? kf1 : kf0;
#pragma unroll
    for (int c = 0; c < TL::NC; ++c) {
      const chunk_t wf = lds_chunk<T, D>(wt_lds, (bi % JB) * 32 + l31, c, half);
      if (c == 0) mma_chunk_first<T>(a, wf, kf[c]);
      else mma_chunk<T>(a, wf, kf[c]);
    }
  };
  // register v of block (sub, jb) pairs with element jb*16 + v of the lane's half row of v
  auto res_diff = [&](const f32x16& a, int bi, int v, float& e) {
    const chunk_t* vf = (bi / JB) ? vf1 : vf0;
    const int el = (bi % JB) * 16 + v;
    float f[E];
    Unpack<T>::run(vf[el / E], f);
    const float df = f[el % E] - a[v];
    e = fmaf(df, df, e);
  };
  auto res_step = [&](f32x16& nx, int bi_n, const f32x16& cu, int bi_c, float& e) {
    const chunk_t* kf = (bi_n / JB) ? kf1 : kf0;
    chunk_t wf = lds_chunk<T, D>(wt_lds, (bi_n % JB) * 32 + l31, 0, half);
#pragma unroll
    for (int c = 0; c < TL::NC; ++c) {
      const chunk_t w_now = wf;
      if (c + 1 < TL::NC) wf = lds_chunk<T, D>(wt_lds, (bi_n % JB) * 32 + l31, c + 1, half);
      if (c == 0) mma_chunk_first<T>(nx, w_now, kf[c]);
      else mma_chunk<T>(nx, w_now, kf[c]);
#pragma unroll
      for (int v = c * 16 / TL::NC; v < (c + 1) * 16 / TL::NC; ++v) res_diff(cu, bi_c, v, e);
      VEC_PIN(nx, e);
    }
  };
  int rep = 0;
  auto load_next = [&](int tn) {
    if (PROBE && rep + 1 < p.repeat) return;
    if (tn >= t_first) {                 // every MFMA of the tile is issued: fetch the next keys
      load_k_subtile<T, D>(kf0, k_head, p.k_st, tn, p.n, lane);
      load_k_subtile<T, D>(kf1, k_head, p.k_st, tn + 32, p.n, lane);
    }
  };
  // one subtile's share of it, as soon as the last MFMA that reads that subtile's keys is issued
  auto load_next_subtile = [&](int tn, int sub) {
    if (PROBE && rep + 1 < p.repeat) return;
    if (tn >= t_first) load_k_subtile<T, D>(sub ? kf1 : kf0, k_head, p.k_st, tn + 32 * sub, p.n, lane);
  };

  float st_n = 0.f, st_l = 0.f, st_ll = 0.f;   // over the columns this lane stores
  while (t0 >= t_first) {
    const int tn = t0 - kStep;
    if (DO_RES && !ROPE && (!PROBE || rep == 0) && !values_requested) {   // values arrive while the score part computes
      load_v_subtile<T, D>(vf0, v_head, p.v_st, t0, p.n, lane);
      load_v_subtile<T, D>(vf1, v_head, p.v_st, t0 + 32, p.n, lane);
    }
    values_requested = false;
    if (DO_MASS && t0 < mass_end) {
      float col0 = 0.f, col1 = 0.f;
      f32x16 A0, A1, B0, B1;
      mass_mma(A0, A1, 0);
      int rb = 0;
      for (; rb + 2 < nrb; rb += 2) {
        mass_step(B0, B1, rb + 1, A0, A1, rb, col0, col1);
        mass_step(A0, A1, rb + 2, B0, B1, rb + 1, col0, col1);
      }
      if (rb + 1 < nrb) {
        mass_step(B0, B1, rb + 1, A0, A1, rb, col0, col1);
        if (!DO_RES) load_next(tn);
        mass_valu(B0, B1, rb + 1, col0, col1);
      } else {
        if (!DO_RES) load_next(tn);
        mass_valu(A0, A1, rb, col0, col1);
      }
      col0 += __shfl_xor(col0, 32, kWave);
      col1 += __shfl_xor(col1, 32, kWave);
      const int t = t0 + lane;             // lanes 0..31 -> subtile 0, 32..63 -> subtile 1
      if (t < mass_end) {
        float* dst = p.mass + (size_t)h * p.n + t;
        float m = (half ? col1 : col0) * p.inv_R;
        if (p.accumulate) m += *dst;
        *dst = m;
        if (m > 0.f) {
          const float l = __log2f(m) - p.log_ref;
          st_n += 1.f;
          st_l += l;
          st_ll = fmaf(l, l, st_ll);
        }
      }
    } else if (DO_MASS && !DO_RES) {
      load_next(tn);
    }
    if constexpr (DO_RES && ROPE) {
      // un-rotate one subtile at a time, then its W^T k products: the MFMAs of block jb + 1
      // are issued before the differences of block jb are taken
      float e01[2] = {0.f, 0.f};
#pragma unroll
      for (int sub = 0; sub < 2; ++sub) {
        const int tok = min(t0 + 32 * sub + l31, p.n - 1);
        const int64_t at = p.pos_base + (p.hps ? (int64_t)(h / p.hps) * p.n : 0) + tok;
        const float pos = (float)((rp.positions ? rp.positions[at] : tok) + rp.pos_offset);
        chunk_t kh[TL::NC], kl[TL::NC];
        const float2* turns = turns_lds;            // re-read per subtile: hoisting the table out of the
        asm volatile("" : "+v"(turns));             // tile loop would pin 64 registers for the whole kernel
        unrotate_subtile<T, D>(sub ? kf1 : kf0, pos, turns, rp.interleaved, half, kh, kl);
        // the values are requested only now: earlier they would sit in registers the un-rotation
        // needs (and be spilled); they arrive while the first block's products run
        chunk_t vsub[TL::VP];
        load_v_subtile<T, D>(vsub, v_head, p.v_st, t0 + 32 * sub, p.n, lane);
        auto mma_block = [&](f32x16& a, int jb) {
#pragma unroll
          for (int c = 0; c < TL::NC; ++c) {
            const chunk_t wf = lds_chunk<T, D>(wt_lds, jb * 32 + l31, c, half);
            if (c == 0) mma_chunk_first<T>(a, wf, kh[c]);
            else mma_chunk<T>(a, wf, kh[c]);
            if (SplitPack<T>::kTwoParts) mma_chunk<T>(a, wf, kl[c]);
          }
        };
        f32x16 RA, RB;
        mma_block(RA, 0);
#pragma unroll
        for (int jb = 0; jb < JB; ++jb) {
          f32x16& cur = (jb & 1) ? RB : RA;
          f32x16& nxt = (jb & 1) ? RA : RB;
          if (jb + 1 < JB) mma_block(nxt, jb + 1);
#pragma unroll
          for (int v = 0; v < 16; ++v) {
            const int el = jb * 16 + v;             // element of the lane's half row of v
            float f[E];
            Unpack<T>::run(vsub[el / E], f);
            const float df = f[el % E] - cur[v];
            e01[sub] = fmaf(df, df, e01[sub]);
          }
        }
      }
      load_next(tn);
      float e0 = e01[0], e1 = e01[1];
      e0 += __shfl_xor(e0, 32, kWave);
      e1 += __shfl_xor(e1, 32, kWave);
      const int t = t0 + lane;
      if (t < c_end) p.eps[(size_t)h * p.n + t] = half ? e1 : e0;
    } else if (DO_RES) {
      float e0 = 0.f, e1 = 0.f;
      f32x16 RA, RB;
      res_mma(RA, 0);
#pragma unroll
      for (int bi = 0; bi + 1 < 2 * JB; ++bi) {
        float& e = (bi / JB) ? e1 : e0;
        if (bi & 1) res_step(RA, bi + 1, RB, bi, e);
        else res_step(RB, bi + 1, RA, bi, e);
        if (bi + 1 == JB - 1) load_next_subtile(tn, 0);     // block JB - 1 was the last one on the first subtile's keys
      }
      load_next_subtile(tn, 1);
#pragma unroll
      for (int v = 0; v < 16; ++v) res_diff(((2 * JB - 1) & 1) ? RB : RA, 2 * JB - 1, v, e1);
      e0 += __shfl_xor(e0, 32, kWave);       // the two halves of the value row
      e1 += __shfl_xor(e1, 32, kWave);
      const int t = t0 + lane;               // lanes 0..31 -> subtile 0, 32..63 -> subtile 1
      if (t < c_end) p.eps[(size_t)h * p.n + t] = half ? e1 : e0;
    }
    if (PROBE && ++rep < p.repeat) continue;
    rep = 0;
    t0 = tn;
  }
  if (DO_MASS && p.range) {                   // uniform: the workgroup's sums, waves added in one fixed order
    st_n = wave_sum_dpp(st_n);
    st_l = wave_sum_dpp(st_l);
    st_ll = wave_sum_dpp(st_ll);
    __syncthreads();                          // every wave is done with the staged query rows
    float* part = reinterpret_cast<float*>(q_lds);
    if (lane == 0) { part[3 * wave] = st_n; part[3 * wave + 1] = st_l; part[3 * wave + 2] = st_ll; }
    __syncthreads();
    if (threadIdx.x == 0) {
      float a = 0.f, b = 0.f, c = 0.f;
#pragma unroll
      for (int w = 0; w < NW; ++w) { a += part[3 * w]; b += part[3 * w + 1]; c += part[3 * w + 2]; }
      p.range[(size_t)h * p.range_stride + chunk] = make_float4(a, b, c, 0.f);
    }
  }
}

// ---------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------
constexpr int kThreads = 512;        // pass 2

constexpr int kThreads1 = VEC_P1_THREADS;   // pass 1
constexpr int kSub1 = VEC_P1_SUBTILES;

struct Plan {
  PassParams pp;
  size_t lds_stats, lds_pass2, lds_tiles;
  bool tiles;           // pass 1 on the kernel that streams key tiles through LDS
};

#ifndef VEC_TILES_MIN_WGS
#define VEC_TILES_MIN_WGS 256
#endif
// pass 1 through LDS tiles: one workgroup per CU where the sequence allows it (more, shorter chunks
// gain a microsecond in pass 1 and lose two in the partial merge of pass 2)
int pick_tokens_per_chunk_tiles(int n, int n_kv_heads) {
  int tpc = 8192;
  while (tpc > 256 && (int64_t)((n + tpc - 1) / tpc) * n_kv_heads < VEC_TILES_MIN_WGS) tpc >>= 1;
  return tpc;
}

size_t stats_tiles_lds(int nrb, int elem_bytes, size_t lds_stride) {
  return (size_t)2 * tiles_token_groups(nrb, elem_bytes) * kV2TileTokens * lds_stride;
}
bool stats_by_tiles(int nrb, int elem_bytes, size_t lds_stride) {
  return (nrb == 8 || nrb == 4) && stats_tiles_lds(nrb, elem_bytes, lds_stride) <= kMaxLdsBytes;
}

int pick_tokens_per_chunk(int n, int n_kv_heads) {
  // at least one workgroup per CU where the sequence allows it, and then as many
  // 64-token tiles per wave as possible so that the key prefetch has something to hide
  int tpc = 8192;
  while (tpc > 512 && (int64_t)((n + tpc - 1) / tpc) * n_kv_heads < 256) tpc >>= 1;
  return tpc;
}

template <typename T, int D>
// plan_heads: the head count the chunk sizes are chosen for.  A stack of sequences plans for one
// sequence's heads, so that every sequence gets the chunking (and with it the order of the
// floating-point sums) it would get alone.
int make_plan(const vector_shape& s, bool do_mass, bool do_res, Plan& plan, int plan_heads = 0) {
  if (plan_heads <= 0) plan_heads = s.n_kv_heads;
  using TL = Tile<T, D>;
  PassParams& p = plan.pp;
  const int G = s.n_q_heads / s.n_kv_heads;
  p.n = s.seq_len; p.w = s.window; p.R = G * s.window; p.R_pad = (p.R + 31) / 32 * 32;
  p.n_prefix = s.seq_len - s.window;
  p.tokens_per_chunk = pick_tokens_per_chunk(s.seq_len, plan_heads);
  plan.tiles = stats_by_tiles(p.R_pad / 32, (int)sizeof(T), (size_t)Tile<T, D>::kLdsStride);
  p.tpc1 = plan.tiles ? pick_tokens_per_chunk_tiles(s.seq_len, plan_heads) : p.tokens_per_chunk;
  p.n_chunks = (s.seq_len + p.tpc1 - 1) / p.tpc1;
  int tpr = 1;
  while (tpr * 2 <= 64 && tpr * 2 * p.R_pad <= kThreads && tpr * 2 <= p.n_chunks) tpr *= 2;
  p.threads_per_row = tpr;
  p.c2 = kLog2e / sqrtf((float)D);
  p.inv_R = 1.0f / (float)p.R;
  p.q_head_rows = p.R; p.q_row0 = 0; p.accumulate = 0; p.range = nullptr; p.range_stride = 0; p.log_ref = 0.f; p.lse = nullptr; p.lse_sh = 0; p.seq_table = nullptr; p.seq_hps = 0; p.pos_base = 0;
  p.k_st = s.k_stride_tok ? s.k_stride_tok : D;
  p.k_sh = s.k_stride_head ? s.k_stride_head : (int64_t)s.seq_len * p.k_st;
  p.v_st = s.v_stride_tok ? s.v_stride_tok : D;
  p.v_sh = s.v_stride_head ? s.v_stride_head : (int64_t)s.seq_len * p.v_st;
  p.w_sh = s.w_shared ? 0 : (s.w_stride_head ? s.w_stride_head : (int64_t)D * D);
  p.hps = 0; p.k_sb = 0; p.v_sb = 0;
  constexpr int NW = kThreads1 / kWave;
  plan.lds_stats = (size_t)p.R_pad * TL::kLdsStride + (size_t)NW * (p.R_pad / 32) * 64 * sizeof(float2);
  plan.lds_pass2 = (do_mass ? (size_t)p.R_pad * (TL::kLdsStride + sizeof(float)) : 0) + (do_res ? (size_t)D * TL::kLdsStride : 0);
  // the pass-1 footprint only matters when the scores are asked for
  if ((do_mass && !plan.tiles && plan.lds_stats > kMaxLdsBytes) || plan.lds_pass2 > kMaxLdsBytes) return VECTOR_ERR_SHAPE;
  return VECTOR_OK;
}

}  // namespace

size_t score_workspace_bytes(const vector_shape& s) {
  const int G = s.n_q_heads / s.n_kv_heads;
  const int R_pad = (G * s.window + 31) / 32 * 32;
  const int n_chunks = (s.seq_len + 255) / 256;      // upper bound over both pass-1 kernels' chunkings
  size_t b = 0;
  b += align_up((size_t)s.n_kv_heads * n_chunks * R_pad * sizeof(float2), 256);
  b += align_up((size_t)s.n_kv_heads * s.seq_len * sizeof(float), 256);
  return b;
}

// One pair of passes over the keys for the query rows [q_row0, q_row0 + rows of `g`) of every KV
// head (g: the shape with the group's query-head count).  accumulate: the column mass is added to
// what earlier groups left.  The residual rides along when eps is given.  prepare_passes fills in
// the parameters, launch_passes enqueues the kernels (RAGGED: one launch for several sequences'
// parameter blocks, see PassParams::seq_table).
struct PassLaunch {
  Plan plan;
  dim3 grid1, grid2;
  size_t lds2;
  bool do_mass, do_res, use_rope;
  RopeParams rp;
};

template <typename T, int D>
static int prepare_passes(const SeqStack* stack, const vector_shape& s, const vector_shape& g, int q_row0, bool accumulate, const void* q,
                          const void* k, const void* v, const void* W, bool do_mass, float* eps, void* ws, const RopeParams* rope,
                          const QueryLse* lse, float4* range, PassLaunch& L) {
  L.do_mass = do_mass;
  L.do_res = eps != nullptr;
  int rc = make_plan<T, D>(g, do_mass, L.do_res, L.plan, stack ? stack->heads_per_seq : 0);
  if (rc != VECTOR_OK) return rc;
  PassParams& p = L.plan.pp;
  p.q = q; p.k = k; p.v = v; p.W = W; p.eps = eps; p.repeat = 1;
  const int rows_all = (s.n_q_heads / s.n_kv_heads) * s.window;
  p.q_head_rows = rows_all; p.q_row0 = q_row0; p.accumulate = accumulate ? 1 : 0;
  p.range = do_mass ? range : nullptr;
  if (lse && do_mass) { p.lse = lse->lse; p.lse_sh = lse->stride_head ? lse->stride_head : s.window; }
  p.log_ref = -log2f((float)(p.n_prefix > 0 ? p.n_prefix : 1));
  p.inv_R = 1.0f / (float)rows_all;
  if (stack) {                      // the strides inside a sequence are the shape's, as for one sequence
    p.hps = stack->heads_per_seq; p.k_sb = stack->k_stride_seq; p.v_sb = stack->v_stride_seq;
  }
  // workspace: partials (sized for all rows of a head, so any group fits), then the mass
  const int rows_all_pad = (rows_all + 31) / 32 * 32;
  unsigned char* w8 = reinterpret_cast<unsigned char*>(ws);
  p.part = reinterpret_cast<float2*>(w8);
  w8 += align_up((size_t)s.n_kv_heads * ((s.seq_len + 255) / 256) * rows_all_pad * sizeof(float2), 256);
  p.mass = reinterpret_cast<float*>(w8);
  L.rp = RopeParams{};
  L.use_rope = rope != nullptr && L.do_res;                // the scores use the keys as cached
  if (L.use_rope) L.rp = *rope;
  L.lds2 = L.plan.lds_pass2 + (L.use_rope ? (D / 2) * sizeof(float2) : 0);
  if (L.lds2 > kMaxLdsBytes) return VECTOR_ERR_SHAPE;
  L.grid1 = dim3(p.n_chunks, s.n_kv_heads);
  L.grid2 = dim3((s.seq_len + p.tokens_per_chunk - 1) / p.tokens_per_chunk, s.n_kv_heads);
  p.range_stride = (int)L.grid2.x;
  return VECTOR_OK;
}

// p: the launch's parameters (RAGGED: only seq_table / seq_hps are looked at); L: what decides the
// kernels and their LDS, the same for every sequence of a ragged launch
template <typename T, int D, bool RAGGED>
static int launch_passes(const PassParams& p, const PassLaunch& L, dim3 grid1, dim3 grid2, hipStream_t stream) {
  if (L.do_mass && !L.plan.pp.lse) {          // pass 1: the rows' (max, sum-exp); not needed when the caller brings them
    const int nrb = L.plan.pp.R_pad / 32;
    if (L.plan.tiles) {
      const size_t lds_tiles = stats_tiles_lds(nrb, (int)sizeof(T), Tile<T, D>::kLdsStride);
      void (*k1)(PassParams) = nrb == 8 ? score_stats_tiles_kernel<T, D, 8, RAGGED> : score_stats_tiles_kernel<T, D, 4, RAGGED>;
      VEC_HIP(set_max_lds(reinterpret_cast<const void*>(k1), lds_tiles));
      VEC_LAUNCH(K_SCORE_STATS, k1, grid1, dim3(kV2Threads), lds_tiles, stream, p);
    } else {
      auto k1 = score_stats_kernel<T, D, kThreads1, kSub1, RAGGED>;
      VEC_HIP(set_max_lds(reinterpret_cast<const void*>(k1), L.plan.lds_stats));
      VEC_LAUNCH(K_SCORE_STATS, k1, grid1, dim3(kThreads1), L.plan.lds_stats, stream, p);
    }
  }
  void (*k2)(PassParams, RopeParams);
  if (RAGGED) k2 = L.use_rope ? mass_residual_kernel<T, D, kThreads, true, true, false, true, RAGGED> : mass_residual_kernel<T, D, kThreads, true, true, false, false, RAGGED>;
  else if (L.do_mass && L.do_res) k2 = L.use_rope ? mass_residual_kernel<T, D, kThreads, true, true, false, true> : mass_residual_kernel<T, D, kThreads, true, true>;
  else if (L.do_mass) k2 = mass_residual_kernel<T, D, kThreads, true, false>;
  else k2 = L.use_rope ? mass_residual_kernel<T, D, kThreads, false, true, false, true> : mass_residual_kernel<T, D, kThreads, false, true>;
  VEC_HIP(set_max_lds(reinterpret_cast<const void*>(k2), L.lds2));
  VEC_LAUNCH(K_MASS_RESIDUAL, k2, grid2, dim3(kThreads), L.lds2, stream, p, L.rp);
  VEC_HIP(hipGetLastError());
  return VECTOR_OK;
}

template <typename T, int D>
static int run_passes(const SeqStack* stack, const vector_shape& s, const vector_shape& g, int q_row0, bool accumulate, const void* q,
                      const void* k, const void* v, const void* W, bool do_mass, float* eps, void* ws, hipStream_t stream,
                      const RopeParams* rope, const QueryLse* lse, float4* range, int* n_range_out, float** mass_out, int* n_prefix_out) {
  PassLaunch L;
  const int rc = prepare_passes<T, D>(stack, s, g, q_row0, accumulate, q, k, v, W, do_mass, eps, ws, rope, lse, range, L);
  if (rc != VECTOR_OK) return rc;
  if (mass_out) *mass_out = L.plan.pp.mass;
  if (n_prefix_out) *n_prefix_out = L.plan.pp.n_prefix;
  if (n_range_out) *n_range_out = (int)L.grid2.x;
  return launch_passes<T, D, false>(L.plan.pp, L, L.grid1, L.grid2, stream);
}

// Query heads per pair of passes: all G of a KV head when their G * w rows fit the kernels' LDS
// layouts, else the largest count that does (0: not even one head's window fits).
template <typename T, int D>
static int heads_per_group(const vector_shape& s, bool do_res) {
  const int G = s.n_q_heads / s.n_kv_heads;
  for (int gh = G; gh >= 1; --gh) {
    vector_shape g = s;
    g.n_q_heads = s.n_kv_heads * gh;
    Plan plan;
    if (make_plan<T, D>(g, true, do_res, plan) == VECTOR_OK) return gh;
  }
  return 0;
}

// Several sequences of different lengths, each with all its query heads in one group and its own
// score workspace: one pair of passes for all of them, then one pooling launch.
template <typename T, int D>
static int run_score_residual_ragged(const vector_shape& s, const RaggedSeq* seqs, int count, const void* W, void* tables,
                                     hipStream_t stream, const RopeParams* rope) {
  if (count < 1 || count > kMaxRaggedSeqs) return VECTOR_ERR_ARG;
  PassParams host[kMaxRaggedSeqs];
  PassLaunch first;
  unsigned g1 = 0, g2 = 0;
  for (int b = 0; b < count; ++b) {
    vector_shape t = seqs[b].shape;
    if (heads_per_group<T, D>(t, true) != t.n_q_heads / t.n_kv_heads) return VECTOR_ERR_SHAPE;
    PassLaunch L;
    float4* range = reinterpret_cast<float4*>(route_mass_range(seqs[b].route_ws, t.n_kv_heads));
    const QueryLse ql = {seqs[b].lse, seqs[b].lse_stride_head};
    const int rc = prepare_passes<T, D>(nullptr, t, t, 0, false, seqs[b].q, seqs[b].k, seqs[b].v, W, true, seqs[b].eps, seqs[b].score_ws,
                                        rope, seqs[b].lse ? &ql : nullptr, range, L);
    if (rc != VECTOR_OK) return rc;
    L.plan.pp.pos_base = seqs[b].pos_base;
    host[b] = L.plan.pp;
    if (b == 0) first = L;
    if (L.grid1.x > g1) g1 = L.grid1.x;
    if (L.grid2.x > g2) g2 = L.grid2.x;
  }
  unsigned char* t8 = reinterpret_cast<unsigned char*>(tables);
  int rc = upload_table(host, sizeof(PassParams) * count, t8, stream);
  if (rc != VECTOR_OK) return rc;
  PassParams lp = host[0];
  lp.seq_table = reinterpret_cast<const PassParams*>(t8);
  lp.seq_hps = s.n_kv_heads;
  const unsigned heads = (unsigned)count * s.n_kv_heads;
  if ((rc = launch_passes<T, D, true>(lp, first, dim3(g1, heads), dim3(g2, heads), stream)) != VECTOR_OK) return rc;
  // pooling + score-key buckets of every sequence
  PoolSeq pool[kMaxRaggedSeqs];
  for (int b = 0; b < count; ++b) {
    pool[b].mass = host[b].mass; pool[b].score = seqs[b].score; pool[b].seq_len = seqs[b].shape.seq_len;
    pool[b].n_prefix = host[b].n_prefix; pool[b].route_ws = seqs[b].route_ws; pool[b].n_range = host[b].range_stride;
  }
  return launch_pool_scores_ragged(pool, count, s.n_kv_heads, s.pool_kernel, s.pool_mode, t8 + align_up(sizeof(PassParams) * count, 256), stream);
}

template <typename T, int D>
static int run_score_residual(const SeqStack* stack, const vector_shape& s, const void* q, const void* k, const void* v, const void* W,
                              float* score, float* eps, void* ws, hipStream_t stream, const RopeParams* rope,
                              void* route_ws, const QueryLse* lse) {
  const bool do_mass = score != nullptr;
  if (!do_mass) return run_passes<T, D>(stack, s, s, 0, false, q, k, v, W, false, eps, ws, stream, rope, nullptr, nullptr, nullptr, nullptr, nullptr);
  // The query heads of a KV head go through the two passes a group at a time; usually one group.
  // The first group's second pass carries the residual.
  const int G = s.n_q_heads / s.n_kv_heads;
  const int gh = heads_per_group<T, D>(s, eps != nullptr);
  if (gh == 0) return VECTOR_ERR_SHAPE;
  float* mass = nullptr;
  int n_prefix = 0, n_range = 0;
  for (int g0 = 0; g0 < G; g0 += gh) {
    vector_shape g = s;
    g.n_q_heads = s.n_kv_heads * (g0 + gh <= G ? gh : G - g0);
    // the last group's second pass sees the finished mass: it leaves its statistics for the routing's buckets
    float4* range = (route_ws && g0 + gh >= G) ? reinterpret_cast<float4*>(route_mass_range(route_ws, s.n_kv_heads)) : nullptr;
    const int rc = run_passes<T, D>(stack, s, g, g0 * s.window, g0 > 0, q, k, v, W, true, g0 == 0 ? eps : nullptr, ws, stream, rope,
                                    lse, range, &n_range, &mass, &n_prefix);
    if (rc != VECTOR_OK) return rc;
  }
  return launch_pool_scores(mass, score, s.n_kv_heads, s.seq_len, n_prefix, s.pool_kernel, s.pool_mode, route_ws, n_range, stream);
}

template <typename T, int D>
static int run_residual_probe(const vector_shape& s, const void* k, const void* v, const void* W, float* eps, int repeat,
                              hipStream_t stream) {
  Plan plan;
  int rc = make_plan<T, D>(s, false, true, plan);
  if (rc != VECTOR_OK) return rc;
  PassParams& p = plan.pp;
  p.q = nullptr; p.k = k; p.v = v; p.W = W; p.eps = eps; p.part = nullptr; p.mass = nullptr; p.repeat = repeat;
  auto k2 = mass_residual_kernel<T, D, kThreads, false, true, true>;
  VEC_HIP(set_max_lds(reinterpret_cast<const void*>(k2), plan.lds_pass2));
  VEC_LAUNCH(K_MASS_RESIDUAL, k2, dim3((s.seq_len + p.tokens_per_chunk - 1) / p.tokens_per_chunk, s.n_kv_heads), dim3(kThreads), plan.lds_pass2,
             stream, p, RopeParams{});
  VEC_HIP(hipGetLastError());
  return VECTOR_OK;
}

int launch_residual_probe(const vector_shape& s, const void* k, const void* v, const void* W, float* eps, int repeat,
                          hipStream_t stream) {
  if (s.dtype != VECTOR_BF16) return VECTOR_ERR_DTYPE;
  if (s.head_dim == 128) return run_residual_probe<bf16_t, 128>(s, k, v, W, eps, repeat, stream);
  if (s.head_dim == 64) return run_residual_probe<bf16_t, 64>(s, k, v, W, eps, repeat, stream);
  return VECTOR_ERR_SHAPE;
}

int launch_score_residual(const vector_shape& s, const void* q, const void* k, const void* v, const void* W,
                          float* score, float* eps, void* ws, hipStream_t stream, const RopeParams* rope,
                          void* route_ws, const SeqStack* stack, const QueryLse* lse) {
  if (s.dtype == VECTOR_BF16) {
    if (s.head_dim == 128) return run_score_residual<bf16_t, 128>(stack, s, q, k, v, W, score, eps, ws, stream, rope, route_ws, lse);
    if (s.head_dim == 64) return run_score_residual<bf16_t, 64>(stack, s, q, k, v, W, score, eps, ws, stream, rope, route_ws, lse);
  } else if (s.dtype == VECTOR_F32) {
    if (s.head_dim == 128) return run_score_residual<float, 128>(stack, s, q, k, v, W, score, eps, ws, stream, rope, route_ws, lse);
    if (s.head_dim == 64) return run_score_residual<float, 64>(stack, s, q, k, v, W, score, eps, ws, stream, rope, route_ws, lse);
  } else {
    return VECTOR_ERR_DTYPE;
  }
  return VECTOR_ERR_SHAPE;
}

bool score_heads_in_one_group(const vector_shape& s) {
  const int G = s.n_q_heads / s.n_kv_heads;
  if (s.dtype == VECTOR_BF16) return s.head_dim == 128 ? heads_per_group<bf16_t, 128>(s, true) == G : heads_per_group<bf16_t, 64>(s, true) == G;
  return s.head_dim == 128 ? heads_per_group<float, 128>(s, true) == G : heads_per_group<float, 64>(s, true) == G;
}

size_t ragged_table_bytes(int count) {
  return align_up(sizeof(PassParams) * count, 256) + route_ragged_table_bytes(count);
}

int launch_score_residual_ragged(const vector_shape& s, const RaggedSeq* seqs, int count, const void* W, void* tables,
                                 hipStream_t stream, const RopeParams* rope) {
  if (s.dtype == VECTOR_BF16) {
    if (s.head_dim == 128) return run_score_residual_ragged<bf16_t, 128>(s, seqs, count, W, tables, stream, rope);
    if (s.head_dim == 64) return run_score_residual_ragged<bf16_t, 64>(s, seqs, count, W, tables, stream, rope);
  } else if (s.dtype == VECTOR_F32) {
    if (s.head_dim == 128) return run_score_residual_ragged<float, 128>(s, seqs, count, W, tables, stream, rope);
    if (s.head_dim == 64) return run_score_residual_ragged<float, 64>(s, seqs, count, W, tables, stream, rope);
  } else {
    return VECTOR_ERR_DTYPE;
  }
  return VECTOR_ERR_SHAPE;
}

}  // namespace vec
