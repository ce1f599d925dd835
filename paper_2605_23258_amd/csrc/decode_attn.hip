// Decode attention over the packed VECTOR cache (Section 3.2, Step 3: values of
// approximated tokens are rebuilt from their keys, v_hat = k W, at generation time).
//
// One softmax runs over the live retained rows and the approximated rows together.
// Because the rebuilt value is linear in the key, sum_t p_t (k_t W) = (sum_t p_t k_t) W:
// the kernel accumulates z = sum p_t k_t over the approximated rows and applies W once
// per (sequence, KV head) in the combine step, so every cache row is read exactly once
// and no value row is ever materialised.
//
// The path is bound by HBM (about 5 flop per byte): a row of the cache is read by
// row_bytes/16 adjacent lanes, 16 bytes each, so every load instruction of a wave covers
// 1 KiB of consecutive memory, and every cache row is read exactly once per step.
//
//   decode_split_mfma_kernel : bf16 caches.  grid (split, kv head, sequence); a workgroup owns
//                           a range of rows of one segment (retained or approximated).  Waves
//                           park 32-row tiles in LDS and run both products (scores, then
//                           weights times rows) on the matrix cores; see the comment above
//                           the kernel.  Variants: ROPE (approximated rows are un-rotated
//                           before they stand in for values), LITERAL (v_hat = k W rebuilt per
//                           row instead of the reassociated sum).
//   decode_split_kernel   : fp32 caches: the same split with vector-ALU dot products (partial
//                           dot product per lane, rotate-add across the lanes of a row,
//                           online softmax per lane group).
//   decode_combine_kernel : merges the splits, applies W to z, normalises, stores.
#include "common.hpp"
#include "launch.hpp"

namespace vec {

namespace {

struct DecodeParams {
  const void* q; const void* k_ret; const void* v_ret; const void* k_apx; const void* W;
  const int32_t* len_retain;
  // per-sequence capacities and first rows of the sequences' blocks (all null: uniform blocks)
  const int32_t* cap_retain_seq; const int32_t* n_approx_seq;
  const int64_t* ret_row_start; const int64_t* apx_row_start;
  // the step's own token (null: none): exact key and value [B, Hkv, D]; it is attended as row
  // len_retain[b] of the retained segment and stored there when the block has room
  const void* k_new; const void* v_new;
  // paged retained segments (null: contiguous): block ids [B, Hkv, blocks_per_seq]; a block is
  // 1 << block_shift rows of the k_ret / v_ret pools
  const int32_t* block_table;
  int block_shift, blocks_per_seq;
  void* out;
  float* part;            // [B, Hkv, S, 2*G + G*D] floats: m[G], l[G], acc[G][D]
  int B, Hq, Hkv, cap_retain, n_approx;
  int splits_ret, splits_apx;   // workgroups per (sequence, head) on each segment
  int64_t w_sh;           // element stride between per-head W
  float c2;               // scale * log2(e)
  int literal;            // approximated rows: rebuild v_hat = k W per row instead of (sum p k) W
  int out_f32;            // store the result as fp32 whatever the cache dtype
};

// Where the rows of one (sequence, KV head) lie: row offsets into k_ret / v_ret and into k_apx,
// the live length of the retained segment and the length of the approximated one.
struct SegmentRows {
  size_t ret_row0, apx_row0;
  int len_retain, n_approx, new_row, cap;
  const int32_t* blocks;      // paged: this (sequence, head)'s block ids; ret_row0 is then 0
  int block_shift;
};
// row r of the retained segment as a row of the k_ret / v_ret arrays.  PAGED is a template
// argument of the kernels: the lookups cost registers that the contiguous layout should not pay.
template <bool PAGED>
__device__ __forceinline__ size_t retained_row(const SegmentRows& s, int r) {
  if (PAGED) return ((size_t)s.blocks[r >> s.block_shift] << s.block_shift) + (size_t)(r & ((1 << s.block_shift) - 1));
  return s.ret_row0 + (size_t)r;
}
__device__ __forceinline__ SegmentRows segment_rows(const DecodeParams& p, int b, int h) {
  SegmentRows s;
  int cap = p.cap_retain;
  s.n_approx = p.n_approx;
  if (p.cap_retain_seq) {
    cap = max(p.cap_retain_seq[b], 0);
    s.n_approx = max(p.n_approx_seq[b], 0);
    s.ret_row0 = (size_t)p.ret_row_start[b] + (size_t)h * cap;
    s.apx_row0 = (size_t)p.apx_row_start[b] + (size_t)h * s.n_approx;
  } else {
    const size_t bh = (size_t)b * p.Hkv + h;
    s.ret_row0 = bh * cap;
    s.apx_row0 = bh * s.n_approx;
  }
  s.blocks = nullptr;
  s.block_shift = 0;
  if (p.block_table) {
    s.blocks = p.block_table + ((size_t)b * p.Hkv + h) * p.blocks_per_seq;
    s.block_shift = p.block_shift;
    s.ret_row0 = 0;
  }
  s.len_retain = min(max(p.len_retain[b], 0), cap);
  s.cap = cap;
  s.new_row = -1;
  if (p.k_new) { s.new_row = s.len_retain; s.len_retain += 1; }      // the new token is the last live row
  return s;
}

// The workgroup whose rows include the step's own token stores it in the cache (when the block has
// room) for the steps to come; this step reads it from the caller's buffers, so nothing waits for
// the store.
template <typename T, int D, bool PAGED>
__device__ __forceinline__ void append_new_row(const DecodeParams& p, const SegmentRows& seg, bool is_apx, int row_begin, int row_end,
                                               const T* k_new, const T* v_new) {
  constexpr int kPieces = D * (int)sizeof(T) / 16;
  if (is_apx || seg.new_row < row_begin || seg.new_row >= row_end || seg.new_row >= seg.cap) return;
  if ((int)threadIdx.x < 2 * kPieces) {
    const int piece = (int)threadIdx.x % kPieces;
    const bool is_v = (int)threadIdx.x >= kPieces;
    unsigned char* dst = reinterpret_cast<unsigned char*>(const_cast<void*>(is_v ? p.v_ret : p.k_ret)) +
                         retained_row<PAGED>(seg, seg.new_row) * D * sizeof(T) + piece * 16;
    const unsigned char* src = reinterpret_cast<const unsigned char*>(is_v ? v_new : k_new) + piece * 16;
    *reinterpret_cast<uint4*>(dst) = *reinterpret_cast<const uint4*>(src);
  }
}

constexpr int DT_ = 256;          // threads per workgroup
constexpr int DW = DT_ / kWave;   // waves
constexpr int kMaxSplits = 64;
constexpr int kUnroll = 4;        // rows per lane group in flight
constexpr int kTargetWorkgroups = 768;
#ifndef VEC_DEC_TARGET
#define VEC_DEC_TARGET 1024
#endif
constexpr int kTargetWorkgroupsMfma = VEC_DEC_TARGET;   // bf16 kernel: two workgroups fit a CU
#ifndef VEC_ROPE_APX_COST
#define VEC_ROPE_APX_COST 2.2
#endif
constexpr double kRopeApxCost = VEC_ROPE_APX_COST;

// sum over the LPR adjacent lanes that share a row; every lane of the group gets the total
template <int LPR> __device__ __forceinline__ float group_sum(float x) {
  if constexpr (LPR == 16) {
    // rotate-add inside a DPP row of 16 lanes: no LDS traffic
#define VEC_ROR_ADD(n) x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x120 + (n), 0xf, 0xf, false))
    VEC_ROR_ADD(8); VEC_ROR_ADD(4); VEC_ROR_ADD(2); VEC_ROR_ADD(1);
#undef VEC_ROR_ADD
    return x;
  } else {
#pragma unroll
    for (int o = LPR / 2; o >= 1; o >>= 1) x += __shfl_xor(x, o, kWave);
    return x;
  }
}

// ROPE: the cache holds keys after their rotary embedding; logits use them as cached, and the rows
// that stand in for values of approximated tokens are the keys turned back by their original
// positions (rp.positions, one per row of k_apx).
template <typename T, int D, int G, bool PAGED = false, bool ROPE = false>
__global__ __launch_bounds__(DT_) void decode_split_kernel(DecodeParams p, RopeParams rp) {
  constexpr int E = Elem<T>::kPerChunk;          // elements per 16-byte piece
  constexpr int LPR = D / E;                     // lanes per row
  constexpr int RPI = kWave / LPR;               // rows per wave-wide load instruction
  constexpr int PSZ = 2 * G + G * D;

  __shared__ float ml_lds[DW][2][G];
  __shared__ float red_lds[DW][G][D];

  const int split = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int grp = lane / LPR, piece = lane % LPR;
  const SegmentRows seg = segment_rows(p, b, h);
  const bool is_apx = split >= p.splits_ret;
  const int seg_len = is_apx ? seg.n_approx : seg.len_retain;
  const int n_sp = is_apx ? p.splits_apx : p.splits_ret;
  const int sp = is_apx ? split - p.splits_ret : split;
  // ranges are multiples of the workgroup's row step so that loads stay aligned to it
  constexpr int kStepRows = DW * RPI * kUnroll;
  const int steps = (seg_len + kStepRows - 1) / kStepRows;
  const int row_begin = (int)((int64_t)steps * sp / n_sp) * kStepRows;
  const int row_end = min(seg_len, (int)((int64_t)steps * (sp + 1) / n_sp) * kStepRows);

  const size_t bh = (size_t)b * p.Hkv + h;
  // a segment's rows: the approximated block, the retained block, or (paged) the retained pool
  const T* kseg = is_apx ? reinterpret_cast<const T*>(p.k_apx) + seg.apx_row0 * D : reinterpret_cast<const T*>(p.k_ret);
  const T* vseg = reinterpret_cast<const T*>(p.v_ret);
  auto seg_row = [&](int r) { return is_apx ? (size_t)r : retained_row<PAGED>(seg, r); };
  const T* k_new = p.k_new ? reinterpret_cast<const T*>(p.k_new) + bh * D : kseg;
  const T* v_new = p.k_new ? reinterpret_cast<const T*>(p.v_new) + bh * D : vseg;
  append_new_row<T, D, PAGED>(p, seg, is_apx, row_begin, row_end, k_new, v_new);

  // this lane's slice of the G query rows, pre-scaled into the log2 domain
  float qf[G][E];
#pragma unroll
  for (int g = 0; g < G; ++g) {
    const uint4 raw = load_chunk(reinterpret_cast<const T*>(p.q) + ((size_t)b * p.Hq + (size_t)h * G + g) * D + piece * E);
    Unpack16<T>::run(raw, qf[g]);
#pragma unroll
    for (int e = 0; e < E; ++e) qf[g][e] *= p.c2;
  }

  float m_run[G], l_run[G], acc[G][E];
#pragma unroll
  for (int g = 0; g < G; ++g) {
    m_run[g] = -INFINITY; l_run[g] = 0.f;
#pragma unroll
    for (int e = 0; e < E; ++e) acc[g][e] = 0.f;
  }

  // ROPE: the rotary pair of each of the lane's E elements, and its frequency.  Pairs (x[2i], x[2i+1])
  // lie inside the lane's piece; pairs (x[i], x[i + D/2]) are split between this lane and the lane
  // LPR/2 further along the row, which holds the same e of the other half.
  const int32_t* pos_seg = (ROPE && is_apx && rp.positions) ? rp.positions + seg.apx_row0 : nullptr;
  const bool lower_half = piece < LPR / 2;
  float t_hi[E], t_lo[E];
  if (ROPE && is_apx) {
#pragma unroll
    for (int e = 0; e < E; ++e) {
      const int i = rp.interleaved ? (piece * E + e) / 2 : (piece % (LPR / 2)) * E + e;
      t_hi[e] = rp.turns_hi[i];
      t_lo[e] = rp.turns_lo[i];
    }
  }
  auto unrotate_row = [&](const float* kf, int pos, float* out) {
    const float pf = (float)pos;
    if (rp.interleaved) {
#pragma unroll
      for (int e = 0; e < E; e += 2) {
        float cs, sn;
        rotary_cos_sin(pf, t_hi[e], t_lo[e], cs, sn);
        rotary_back(kf[e], kf[e + 1], cs, sn, out[e], out[e + 1]);
      }
    } else {
#pragma unroll
      for (int e = 0; e < E; ++e) {
        const float other = __shfl_xor(kf[e], LPR / 2, kWave);
        float cs, sn, a_pre, b_pre;
        rotary_cos_sin(pf, t_hi[e], t_lo[e], cs, sn);
        rotary_back(lower_half ? kf[e] : other, lower_half ? other : kf[e], cs, sn, a_pre, b_pre);
        out[e] = lower_half ? a_pre : b_pre;
      }
    }
  };

  // The loop bound is the same for every lane of a wave; rows past the range are masked.
  // The rows of the next step are requested before the current ones are consumed.
  auto fetch = [&](uint4* kraw, uint4* vraw, int base) {
    const int r0 = base + grp * kUnroll;
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
      const int r = min(r0 + u, seg_len - 1);      // clamped: never reads past the live rows
      const bool fresh = !is_apx && r == seg.new_row;        // the step's own token comes from the caller's buffers
      const size_t at = seg_row(fresh ? 0 : r) * D + piece * E;
      kraw[u] = load_chunk(fresh ? k_new + piece * E : kseg + at);
      if (!is_apx) vraw[u] = load_chunk(fresh ? v_new + piece * E : vseg + at);
      else if (ROPE) vraw[u].x = (uint32_t)((pos_seg ? pos_seg[r] : r) + rp.pos_offset);    // the row's position rides along
    }
  };
  auto consume = [&](const uint4* kraw, const uint4* vraw, int base) {
    const int r0 = base + grp * kUnroll;
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
      float kf[E];
      Unpack16<T>::run(kraw[u], kf);
      float s[G];
#pragma unroll
      for (int g = 0; g < G; ++g) {
        float d = 0.f;
#pragma unroll
        for (int e = 0; e < E; ++e) d = fmaf(qf[g][e], kf[e], d);
        s[g] = group_sum<LPR>(d);
      }
      const bool live = r0 + u < row_end;
      bool grew = false;
#pragma unroll
      for (int g = 0; g < G; ++g) {
        if (!live) s[g] = -INFINITY;
        grew |= s[g] > m_run[g];
      }
      if (__any(grew)) {                             // rare once the running maxima have settled
#pragma unroll
        for (int g = 0; g < G; ++g) {
          const float m_new = fmaxf(m_run[g], s[g]);
          const float alpha = (m_new == -INFINITY) ? 1.f : fast_exp2(m_run[g] - m_new);
          l_run[g] *= alpha;
#pragma unroll
          for (int e = 0; e < E; ++e) acc[g][e] *= alpha;
          m_run[g] = m_new;
        }
      }
      float rowf[E];
      if (is_apx) {
        if (ROPE) {
          unrotate_row(kf, (int)vraw[u].x, rowf);
        } else {
#pragma unroll
          for (int e = 0; e < E; ++e) rowf[e] = kf[e];
        }
      } else {
        Unpack16<T>::run(vraw[u], rowf);
      }
#pragma unroll
      for (int g = 0; g < G; ++g) {
        const float pg = (m_run[g] == -INFINITY) ? 0.f : fast_exp2(s[g] - m_run[g]);
        l_run[g] += pg;
#pragma unroll
        for (int e = 0; e < E; ++e) acc[g][e] = fmaf(pg, rowf[e], acc[g][e]);
      }
    }
  };
  uint4 ka[kUnroll], va[kUnroll], kb[kUnroll], vb[kUnroll];
  int base = row_begin + wave * RPI * kUnroll;
  if (base < row_end) fetch(ka, va, base);
  while (base < row_end) {
    const int b1 = base + kStepRows;
    if (b1 < row_end) fetch(kb, vb, b1);
    consume(ka, va, base);
    if (b1 >= row_end) break;
    const int b2 = b1 + kStepRows;
    if (b2 < row_end) fetch(ka, va, b2);
    consume(kb, vb, b1);
    base = b2;
  }

  // ---- merge the lane groups of a wave (each ran its own softmax), then the waves ----
#pragma unroll
  for (int o = LPR; o < kWave; o <<= 1) {
#pragma unroll
    for (int g = 0; g < G; ++g) {
      const float m2 = __shfl_xor(m_run[g], o, kWave), l2 = __shfl_xor(l_run[g], o, kWave);
      const float mn = fmaxf(m_run[g], m2);
      const float a = (m_run[g] == -INFINITY) ? 0.f : fast_exp2(m_run[g] - mn);
      const float c = (m2 == -INFINITY) ? 0.f : fast_exp2(m2 - mn);
      l_run[g] = l_run[g] * a + l2 * c;
#pragma unroll
      for (int e = 0; e < E; ++e) acc[g][e] = acc[g][e] * a + __shfl_xor(acc[g][e], o, kWave) * c;
      m_run[g] = mn;
    }
  }
  if (lane < LPR) {
#pragma unroll
    for (int g = 0; g < G; ++g)
#pragma unroll
      for (int e = 0; e < E; ++e) red_lds[wave][g][piece * E + e] = acc[g][e];
  }
  if (lane == 0) {
#pragma unroll
    for (int g = 0; g < G; ++g) { ml_lds[wave][0][g] = m_run[g]; ml_lds[wave][1][g] = l_run[g]; }
  }
  __syncthreads();

  float* out = p.part + (bh * (p.splits_ret + p.splits_apx) + split) * PSZ;
  for (int i = threadIdx.x; i < G * D; i += DT_) {
    const int g = i / D, j = i % D;
    float m = -INFINITY;
#pragma unroll
    for (int wv = 0; wv < DW; ++wv) m = fmaxf(m, ml_lds[wv][0][g]);
    float a = 0.f;
#pragma unroll
    for (int wv = 0; wv < DW; ++wv) {
      const float mw = ml_lds[wv][0][g];
      if (mw != -INFINITY) a += red_lds[wv][g][j] * fast_exp2(mw - m);
    }
    out[2 * G + i] = a;
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

// ---------------------------------------------------------------------------
// bf16 caches: the same split, on the matrix cores.  Rows still arrive as 1 KiB
// wave-wide loads (16 bytes per lane, adjacent lanes on one row); a wave parks a tile of
// 32 rows in its own slice of LDS and reads it back in operand order:
//   scores   S[t][g] = sum_e K[t][e] q[g][e]     A = key tile (16-byte reads along a row),
//                                                 B = the G query rows (columns >= G zero)
//   output   O[j][g] += sum_t R[t][j] P[t][g]    A = tile of R read down its columns
//                                                 (R = values, or the keys themselves for
//                                                 approximated rows), B = P
// The accumulator layout of S (column g on lane g, sixteen tokens in the registers of a
// lane) is already the B-operand layout of the second product once the contraction index
// is numbered the way those registers number the tokens, so P never leaves its lane.  P is
// fed to the matrix core as bf16 twice: its rounded value and the remainder of that
// rounding, which keeps the weights to about 2^-16 relative.
// ---------------------------------------------------------------------------
constexpr int kTileRows = 32;

typedef __attribute__((ext_vector_type(8))) unsigned short u16x8;

template <int D> struct MfmaDecodeTile {
  static constexpr int kRowBytes = D * 2;
  static constexpr int kStride = kRowBytes + 16;            // LDS row stride: 16-byte reads of 32 rows hit distinct banks
  static constexpr int kPieces = kRowBytes / 16;            // 16-byte pieces per row
  static constexpr int kRowsPerLoad = kWave / kPieces;
  static constexpr int kLoads = kTileRows / kRowsPerLoad;   // wave-wide loads per tile and tensor
  static constexpr int kTileBytes = kTileRows * kStride;
  static constexpr int kLdsBytes = DW * 2 * kTileBytes;
};

// ROPE: the cached keys carry rotary position embedding.  Logits use them as cached; the
// rows that stand in for values of approximated tokens are the keys turned back by their
// original positions (rp.positions, one per row of k_apx), written to the second tile as bf16.
// LITERAL: approximated rows are rebuilt one by one, v_hat = k W, before they are weighted.
template <int D, int G, bool ROPE, bool LITERAL = false, bool PAGED = false>
__global__ __launch_bounds__(DT_, 2) void decode_split_mfma_kernel(DecodeParams p, RopeParams rp) {
  using T = bf16_t;
  using TL = MfmaDecodeTile<D>;
  constexpr int NC = D / 16;               // 16-element steps of the score contraction
  constexpr int JB = D / 32;               // 32-wide blocks of the output dimension
  constexpr int PSZ = 2 * G + G * D;
  constexpr float kNegBig = -1.0e30f;      // running maximum before any row: finite, so differences stay finite
  static_assert(DW * (G * D + 2 * G) * 4 <= TL::kLdsBytes, "merge area must fit in the tile area");

  extern __shared__ __align__(16) unsigned char dec_lds[];

  const int split = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int l31 = lane & 31, half = lane >> 5;
  const SegmentRows seg = segment_rows(p, b, h);
  const bool is_apx = split >= p.splits_ret;
  const int seg_len = is_apx ? seg.n_approx : seg.len_retain;
  const int n_sp = is_apx ? p.splits_apx : p.splits_ret;
  const int sp = is_apx ? split - p.splits_ret : split;
  constexpr int kStepRows = DW * kTileRows;
  const int steps = (seg_len + kStepRows - 1) / kStepRows;
  const int row_begin = (int)((int64_t)steps * sp / n_sp) * kStepRows;
  const int row_end = min(seg_len, (int)((int64_t)steps * (sp + 1) / n_sp) * kStepRows);

  const size_t bh = (size_t)b * p.Hkv + h;
  // a segment's rows: the approximated block, the retained block, or (paged) the retained pool
  const T* kseg = is_apx ? reinterpret_cast<const T*>(p.k_apx) + seg.apx_row0 * D : reinterpret_cast<const T*>(p.k_ret);
  const T* vseg = reinterpret_cast<const T*>(p.v_ret);
  auto seg_row = [&](int r) { return is_apx ? (size_t)r : retained_row<PAGED>(seg, r); };
  const T* k_new = p.k_new ? reinterpret_cast<const T*>(p.k_new) + bh * D : kseg;
  const T* v_new = p.k_new ? reinterpret_cast<const T*>(p.v_new) + bh * D : vseg;
  append_new_row<T, D, PAGED>(p, seg, is_apx, row_begin, row_end, k_new, v_new);

  unsigned char* k_tile = dec_lds + wave * 2 * TL::kTileBytes;
  unsigned char* v_tile = k_tile + TL::kTileBytes;
  const unsigned char* r_tile = (is_apx && !ROPE) ? k_tile : v_tile;
  const bool literal = LITERAL && is_apx;                    // rebuild every approximated value row

  // B operand of the score product: query row g on lane g, zero beyond G
  chunk_t qf[NC];
#pragma unroll
  for (int c = 0; c < NC; ++c) {
    qf[c] = make_uint4(0, 0, 0, 0);
    if (l31 < G)
      qf[c] = load_chunk(reinterpret_cast<const T*>(p.q) + ((size_t)b * p.Hq + (size_t)h * G + l31) * D + (2 * c + half) * 8);
  }

  f32x16 o[JB];
#pragma unroll
  for (int jb = 0; jb < JB; ++jb)
#pragma unroll
    for (int v = 0; v < 16; ++v) o[jb][v] = 0.f;
  float m_run = kNegBig, l_run = 0.f;

  const int ld_row = lane / TL::kPieces, ld_piece = lane % TL::kPieces;
  const int32_t* pos_seg = (ROPE && is_apx && rp.positions) ? rp.positions + seg.apx_row0 : nullptr;
  // Which 16 bytes of the tile a lane brings in with its i-th load.  Normally 16 adjacent lanes
  // share a row.  For approximated rows that are to be un-rotated with pairs (x[i], x[i + d/2])
  // a lane instead takes both members of its pairs: loads 2u and 2u+1 bring pieces p and
  // p + kPieces/2 of the same row, kPieces/2 adjacent lanes share a row.
  constexpr int HP = TL::kPieces / 2;
  constexpr int kRowsPerPair = kWave / HP;
  const bool paired = ROPE && is_apx && !rp.interleaved;
  const int pr_row = lane / HP, pr_piece = lane % HP;
  auto row_of = [&](int i) { return paired ? (i / 2) * kRowsPerPair + pr_row : i * TL::kRowsPerLoad + ld_row; };
  auto piece_of = [&](int i) { return paired ? pr_piece + (i & 1) * HP : ld_piece; };
  // For an approximated row under ROPE the second register set carries the row's position
  // (in .x) instead of a value row.
  // (the segment is the same for the whole workgroup: one straight-line loop per case, so that
  // all loads of a tile go out together)
  // Paged with blocks of at least a tile's 32 rows: tiles start at multiples of 32 rows, so a tile
  // lies in one block.  The block ids of the workgroup's row range sit in one register across the
  // wave (lane j: block (row_begin / block rows) + j), read once before the loop; a tile's id then
  // comes out of that register instead of memory.
  const bool tile_in_block = PAGED && !is_apx && seg.block_shift >= 5 &&
                             ((row_end - 1) >> seg.block_shift) - (row_begin >> seg.block_shift) < kWave;
  int my_block = 0;
  if (tile_in_block && row_begin < row_end) {
    const int j = min((row_begin >> seg.block_shift) + lane, (row_end - 1) >> seg.block_shift);
    my_block = seg.blocks[j];
  }
  auto fetch = [&](uint4* kraw, uint4* vraw, int base) {
    if (!ROPE || !is_apx) {
      size_t tile_shift = 0;                     // paged, one block per tile: array row = tile_shift + segment row
      if (tile_in_block) {
        const int blk = __builtin_amdgcn_readlane(my_block, (base >> seg.block_shift) - (row_begin >> seg.block_shift));
        tile_shift = ((size_t)blk << seg.block_shift) - (size_t)((base >> seg.block_shift) << seg.block_shift);
      }
#pragma unroll
      for (int i = 0; i < TL::kLoads; ++i) {
        const int r = min(base + i * TL::kRowsPerLoad + ld_row, seg_len - 1);   // clamped: never past the live rows
        const bool fresh = !is_apx && r == seg.new_row;      // the step's own token comes from the caller's buffers
        const size_t at = (tile_in_block ? tile_shift + (size_t)r : seg_row(fresh ? 0 : r)) * D + ld_piece * 8;
        kraw[i] = load_chunk(fresh ? k_new + ld_piece * 8 : kseg + at);
        if (!is_apx) vraw[i] = load_chunk(fresh ? v_new + ld_piece * 8 : vseg + at);
      }
    } else {
#pragma unroll
      for (int i = 0; i < TL::kLoads; ++i) {
        const int r = min(base + row_of(i), seg_len - 1);
        kraw[i] = load_chunk(kseg + (size_t)r * D + piece_of(i) * 8);
        vraw[i].x = (uint32_t)((pos_seg ? pos_seg[r] : r) + rp.pos_offset);
      }
    }
  };
  // the lane's pieces always cover the same rotary pairs: their frequencies stay in registers
  float t_hi[8], t_lo[8];
  if (ROPE && is_apx) {
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const int i = rp.interleaved ? (ld_piece * 8 + e) / 2 : pr_piece * 8 + e;
      t_hi[e] = rp.turns_hi[i];
      t_lo[e] = rp.turns_lo[i];
    }
  }
  auto pack8 = [](const float* f) {
    return make_uint4(pack_bf16(f[0], f[1]), pack_bf16(f[2], f[3]), pack_bf16(f[4], f[5]), pack_bf16(f[6], f[7]));
  };
  // both members of eight pairs (x[i], x[i + d/2]) of a cached key row, turned back by the row's position
  auto unrotate_pair = [&](const uint4& ra, const uint4& rb, int pos, uint4& oa, uint4& ob) {
    float a[8], b[8];
    const float pf = (float)pos;
    Unpack16<T>::run(ra, a);
    Unpack16<T>::run(rb, b);
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      float cs, sn;
      rotary_cos_sin(pf, t_hi[e], t_lo[e], cs, sn);
      rotary_back(a[e], b[e], cs, sn, a[e], b[e]);
    }
    oa = pack8(a);
    ob = pack8(b);
  };
  // pairs (x[2i], x[2i+1]): four of them inside one 16-byte piece
  auto unrotate_piece = [&](const uint4& raw, int pos) {
    float f[8];
    const float pf = (float)pos;
    Unpack16<T>::run(raw, f);
#pragma unroll
    for (int e = 0; e < 8; e += 2) {
      float cs, sn;
      rotary_cos_sin(pf, t_hi[e], t_lo[e], cs, sn);
      rotary_back(f[e], f[e + 1], cs, sn, f[e], f[e + 1]);
    }
    return pack8(f);
  };
  auto stage = [&](const uint4* kraw, const uint4* vraw) {
    if (!is_apx || !ROPE) {
#pragma unroll
      for (int i = 0; i < TL::kLoads; ++i) {
        const int off = (i * TL::kRowsPerLoad + ld_row) * TL::kStride + ld_piece * 16;
        *reinterpret_cast<uint4*>(k_tile + off) = kraw[i];
        if (!is_apx) *reinterpret_cast<uint4*>(v_tile + off) = vraw[i];
      }
    } else {
#pragma unroll
      for (int i = 0; i < TL::kLoads; ++i) {
        const int off = row_of(i) * TL::kStride + piece_of(i) * 16;
        *reinterpret_cast<uint4*>(k_tile + off) = kraw[i];
        if (!paired) {
          *reinterpret_cast<uint4*>(v_tile + off) = unrotate_piece(kraw[i], (int)vraw[i].x);
        } else if (i & 1) {
          uint4 oa, ob;
          unrotate_pair(kraw[i - 1], kraw[i], (int)vraw[i].x, oa, ob);
          *reinterpret_cast<uint4*>(v_tile + row_of(i - 1) * TL::kStride + piece_of(i - 1) * 16) = oa;
          *reinterpret_cast<uint4*>(v_tile + off) = ob;
        }
      }
    }
  };
  // the tile belongs to this wave alone; these keep the compiler from moving LDS accesses of
  // different lanes across the hand-over (the hardware runs a wave's LDS operations in order)
  auto wave_fence = [&]() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
  };

  auto consume = [&](int base) {
    // ---- scores ----
    f32x16 s;
#pragma unroll
    for (int c = 0; c < NC; ++c) {
      const chunk_t a = *reinterpret_cast<const chunk_t*>(k_tile + l31 * TL::kStride + (2 * c + half) * 16);
      if (c == 0) mma_chunk_first<T>(s, a, qf[c]); else mma_chunk<T>(s, a, qf[c]);
    }
    float tmax = kNegBig;
    if (base + kTileRows > row_end) {               // ragged last tile: rows past the range score -inf
#pragma unroll
      for (int v = 0; v < 16; ++v) s[v] = (base + acc_row(v, half) < row_end) ? s[v] * p.c2 : -INFINITY;
    } else {
#pragma unroll
      for (int v = 0; v < 16; ++v) s[v] *= p.c2;
    }
#pragma unroll
    for (int v = 0; v < 16; ++v) tmax = fmaxf(tmax, s[v]);
    tmax = fmaxf(tmax, __shfl_xor(tmax, 32, kWave));
    if (__any(tmax > m_run)) {                       // rare once the running maxima have settled
      const float m_new = fmaxf(m_run, tmax);
      const float alpha = fast_exp2(m_run - m_new);
      l_run *= alpha;
#pragma unroll
      for (int jb = 0; jb < JB; ++jb)
#pragma unroll
        for (int v = 0; v < 16; ++v) o[jb][v] *= alpha;
      m_run = m_new;
    }
    // ---- weights, split into a bf16 value and the bf16 remainder ----
    bf16x8 p_hi[2], p_lo[2];
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const float pv = fast_exp2(s[v] - m_run);
      l_run += pv;
      const __bf16 hi = (__bf16)pv;
      p_hi[v >> 3][v & 7] = hi;
      p_lo[v >> 3][v & 7] = (__bf16)(pv - (float)hi);
    }
    // ---- output: contraction index e of step ks on lane half `half` is tile row
    //      16 ks + 4 half + 8 (e / 4) + e % 4, the row accumulator register 8 ks + e holds ----
    if (LITERAL && literal) {
      // v_hat[t][j] = sum_i K[t][i] W[i][j] per 32-wide block of j: rows = tokens, so that the
      // accumulator of lane j holds its column in exactly the order the second product wants
      // for its A operand; fed as bf16 value + remainder like the weights.
#pragma unroll
      for (int jb = 0; jb < JB; ++jb) {
        const unsigned char* wt = dec_lds + jb * 2 * TL::kTileBytes + TL::kTileBytes;
        f32x16 vh;
#pragma unroll
        for (int c = 0; c < NC; ++c) {
          const chunk_t a = *reinterpret_cast<const chunk_t*>(k_tile + l31 * TL::kStride + (2 * c + half) * 16);
          const chunk_t b = *reinterpret_cast<const chunk_t*>(wt + l31 * TL::kStride + (2 * c + half) * 16);
          if (c == 0) mma_chunk_first<T>(vh, a, b); else mma_chunk<T>(vh, a, b);
        }
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
          bf16x8 v_hi, v_lo;
#pragma unroll
          for (int e = 0; e < 8; ++e) {
            const float x = vh[8 * ks + e];
            const __bf16 hi = (__bf16)x;
            v_hi[e] = hi;
            v_lo[e] = (__bf16)(x - (float)hi);
          }
          o[jb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(v_hi, p_hi[ks], o[jb], 0, 0, 0);
          o[jb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(v_lo, p_hi[ks], o[jb], 0, 0, 0);
          o[jb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(v_hi, p_lo[ks], o[jb], 0, 0, 0);
        }
      }
      return;
    }
#pragma unroll
    for (int jb = 0; jb < JB; ++jb) {
#pragma unroll
      for (int ks = 0; ks < 2; ++ks) {
        u16x8 a;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const int row = 16 * ks + 4 * half + 8 * (e >> 2) + (e & 3);
          a[e] = *reinterpret_cast<const unsigned short*>(r_tile + row * TL::kStride + (jb * 32 + l31) * 2);
        }
        o[jb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), p_hi[ks], o[jb], 0, 0, 0);
        o[jb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), p_lo[ks], o[jb], 0, 0, 0);
      }
    }
  };

  // Literal reconstruction: W^T of the head sits in the value-tile slots, which approximated rows
  // do not use (32 rows of W^T per slot, same row stride as a tile).
  if (LITERAL && literal) {
    const T* Wh = reinterpret_cast<const T*>(p.W) + (int64_t)h * p.w_sh;
    for (int idx = threadIdx.x; idx < D * D / 8; idx += DT_) {
      const int i = idx / (D / 8), j0 = (idx % (D / 8)) * 8;
      union { uint4 raw; unsigned short el[8]; } w;
      w.raw = load_chunk(Wh + (size_t)i * D + j0);
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const int j = j0 + e;
        *reinterpret_cast<unsigned short*>(dec_lds + (j / 32) * 2 * TL::kTileBytes + TL::kTileBytes + (j % 32) * TL::kStride + i * 2) = w.el[e];
      }
    }
    __syncthreads();
  }

  uint4 kraw[TL::kLoads], vraw[TL::kLoads];
  int base = row_begin + wave * kTileRows;
  if (base < row_end) fetch(kraw, vraw, base);
  while (base < row_end) {
    wave_fence();                                    // last tile's reads are done before it is overwritten
    stage(kraw, vraw);
    const int next = base + kStepRows;
    if (next < row_end) fetch(kraw, vraw, next);     // in flight while this tile is consumed
    wave_fence();
    consume(base);
    base = next;
  }

  // ---- merge the waves ----
  const float l_tot = l_run + __shfl_xor(l_run, 32, kWave);
  __syncthreads();                                   // every wave is done with its tiles: reuse the area
  float* red = reinterpret_cast<float*>(dec_lds);                    // [DW][G][D]
  float* ml = red + DW * G * D;                                       // [DW][2][G]
  if (l31 < G) {
#pragma unroll
    for (int jb = 0; jb < JB; ++jb)
#pragma unroll
      for (int v = 0; v < 16; ++v) red[(wave * G + l31) * D + jb * 32 + acc_row(v, half)] = o[jb][v];
    if (half == 0) {
      ml[(wave * 2 + 0) * G + l31] = (l_tot > 0.f) ? m_run : -INFINITY;
      ml[(wave * 2 + 1) * G + l31] = l_tot;
    }
  }
  __syncthreads();
  float* out = p.part + (bh * (p.splits_ret + p.splits_apx) + split) * PSZ;
  for (int i = threadIdx.x; i < G * D; i += DT_) {
    const int g = i / D, j = i % D;
    float m = -INFINITY;
#pragma unroll
    for (int wv = 0; wv < DW; ++wv) m = fmaxf(m, ml[(wv * 2) * G + g]);
    float a = 0.f;
#pragma unroll
    for (int wv = 0; wv < DW; ++wv) {
      const float mw = ml[(wv * 2) * G + g];
      if (mw != -INFINITY) a += red[(wv * G + g) * D + j] * fast_exp2(mw - m);
    }
    out[2 * G + i] = a;
  }
  if (threadIdx.x < G) {
    const int g = threadIdx.x;
    float m = -INFINITY, l = 0.f;
#pragma unroll
    for (int wv = 0; wv < DW; ++wv) m = fmaxf(m, ml[(wv * 2) * G + g]);
#pragma unroll
    for (int wv = 0; wv < DW; ++wv) {
      const float mw = ml[(wv * 2) * G + g];
      if (mw != -INFINITY) l += ml[(wv * 2 + 1) * G + g] * fast_exp2(mw - m);
    }
    out[g] = m;
    out[G + g] = l;
  }
}

template <typename T, int D, int G>
__global__ __launch_bounds__(256) void decode_combine_kernel(DecodeParams p) {
  constexpr int PSZ = 2 * G + G * D;
  constexpr int E = Elem<T>::kPerChunk;    // elements of W per 16-byte load
  constexpr int CG = D / E;                // thread groups along a row of W
  constexpr int RG = 256 / CG;             // thread groups along its rows (the contraction index)
  constexpr int RP = D / RG;               // rows of W per thread
  constexpr int kWavesC = 256 / kWave;
  static_assert(CG <= kWave && D % RG == 0, "a wave holds whole row groups");
  __shared__ float z_lds[G][D];
  __shared__ float v_lds[G][D];
  __shared__ float zw_lds[kWavesC][G][D];
  __shared__ float linv_lds[G];
  const int h = blockIdx.x, b = blockIdx.y;
  const size_t bh = (size_t)b * p.Hkv + h;
  const int n_splits = p.splits_ret + p.splits_apx;
  const float* part = p.part + bh * n_splits * PSZ;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;

  // this thread's block of W (rows rg*RP.., 16 bytes of each) is requested first: it depends on
  // nothing and arrives while the splits are merged
  const int cg = threadIdx.x % CG, rg = threadIdx.x / CG;
  const T* Wh = reinterpret_cast<const T*>(p.W) + (int64_t)h * p.w_sh;
  uint4 wraw[RP];
  const bool use_w = p.n_approx > 0 && !p.literal;      // literal partials are values already
  // the step's own token is now a row of the cache (the split launch has finished): one thread per
  // sequence makes it live, unless the block was full
  if (p.k_new && h == 0 && threadIdx.x == 0) {
    const int cap = p.cap_retain_seq ? max(p.cap_retain_seq[b], 0) : p.cap_retain;
    int* len = const_cast<int*>(p.len_retain) + b;
    *len = min(min(max(*len, 0), cap) + 1, cap);
  }
  if (use_w) {
#pragma unroll
    for (int r = 0; r < RP; ++r) wraw[r] = load_chunk(Wh + (size_t)(rg * RP + r) * D + cg * E);
  }

  // Merge the splits in one round of loads: a thread owns G*D/256 output elements and, for each,
  // reads every split's (m, l, partial) itself (the (m, l) reads of a query row are shared by
  // the lanes that work on that row), folding eight splits at a time into a running maximum.
  constexpr int kFold = 8;
  for (int i = threadIdx.x; i < G * D; i += 256) {
    const int g = i / D;
    float M = -INFINITY, L = 0.f, av = 0.f, az = 0.f;
    for (int s0 = 0; s0 < n_splits; s0 += kFold) {
      float ms[kFold], ls[kFold], xs[kFold];
#pragma unroll
      for (int u = 0; u < kFold; ++u) {
        const int sI = min(s0 + u, n_splits - 1);
        ms[u] = part[(size_t)sI * PSZ + g];
        ls[u] = part[(size_t)sI * PSZ + G + g];
        xs[u] = part[(size_t)sI * PSZ + 2 * G + i];
      }
      float mx = M;
#pragma unroll
      for (int u = 0; u < kFold; ++u)
        if (s0 + u < n_splits) mx = fmaxf(mx, ms[u]);
      const float keep = (M == -INFINITY) ? 0.f : fast_exp2(M - mx);     // mx = -inf only if M is
      L *= keep; av *= keep; az *= keep;
#pragma unroll
      for (int u = 0; u < kFold; ++u) {
        if (s0 + u < n_splits && ms[u] != -INFINITY) {
          const float sc = fast_exp2(ms[u] - mx);
          L = fmaf(ls[u], sc, L);
          if (s0 + u < p.splits_ret || p.literal) av = fmaf(xs[u], sc, av);
          else az = fmaf(xs[u], sc, az);
        }
      }
      M = mx;
    }
    (&v_lds[0][0])[i] = av;
    (&z_lds[0][0])[i] = az;
    if (i % D == 0) linv_lds[g] = (L > 0.f) ? 1.f / L : 0.f;
  }
  __syncthreads();
  // out[g][j] = (sum_ret p v  +  z[g][:] . W[:, j]) / l : partial products over the thread's rows
  // of W, summed over the row groups of a wave by lane exchange, over the waves through LDS
  {
    float a[G][E];
#pragma unroll
    for (int g = 0; g < G; ++g)
#pragma unroll
      for (int e = 0; e < E; ++e) a[g][e] = 0.f;
    if (use_w) {
#pragma unroll
      for (int r = 0; r < RP; ++r) {
        float wf[E];
        Unpack16<T>::run(wraw[r], wf);
#pragma unroll
        for (int g = 0; g < G; ++g) {
          const float zg = z_lds[g][rg * RP + r];
#pragma unroll
          for (int e = 0; e < E; ++e) a[g][e] = fmaf(zg, wf[e], a[g][e]);
        }
      }
    }
#pragma unroll
    for (int o = CG; o < kWave; o <<= 1)
#pragma unroll
      for (int g = 0; g < G; ++g)
#pragma unroll
        for (int e = 0; e < E; ++e) a[g][e] += __shfl_xor(a[g][e], o, kWave);
    if (lane < CG) {
#pragma unroll
      for (int g = 0; g < G; ++g)
#pragma unroll
        for (int e = 0; e < E; ++e) zw_lds[wave][g][cg * E + e] = a[g][e];
    }
  }
  __syncthreads();
  T* out = reinterpret_cast<T*>(p.out) + ((size_t)b * p.Hq + (size_t)h * G) * D;
  for (int i = threadIdx.x; i < G * D; i += 256) {
    const int g = i / D, j = i % D;
    float zw = 0.f;
#pragma unroll
    for (int q = 0; q < kWavesC; ++q) zw += zw_lds[q][g][j];
    const float r = (v_lds[g][j] + zw) * linv_lds[g];
    if (p.out_f32) reinterpret_cast<float*>(p.out)[((size_t)b * p.Hq + (size_t)h * G) * D + i] = r;
    else store_elem(out + i, r);
  }
}

void pick_splits(int target, int batch, int n_kv_heads, int cap_retain, int n_approx, double apx_cost, int& s_ret, int& s_apx) {
  // One round of workgroups: 256 CUs hold three of these workgroups each, and a second,
  // partly filled round would stream with too few loads in flight.  The splits are divided
  // between the segments by their bytes (a retained row is a key and a value); a workgroup
  // gets a few hundred rows at least.
  const int pairs = batch * n_kv_heads;
  int total = target / pairs;
  if (total > kMaxSplits) total = kMaxSplits;
  if (total < 2) total = 2;
  const double w_ret = 2.0 * cap_retain, w_apx = apx_cost * n_approx;
  s_ret = cap_retain > 0 ? (int)(total * w_ret / (w_ret + w_apx) + 0.5) : 0;
  if (cap_retain > 0 && s_ret < 1) s_ret = 1;
  s_apx = n_approx > 0 ? total - s_ret : 0;
  if (n_approx > 0 && s_apx < 1) s_apx = 1;
  const int max_ret = cap_retain / 256 + 1, max_apx = n_approx / 256 + 1;
  if (s_ret > max_ret) s_ret = max_ret;
  if (s_apx > max_apx) s_apx = max_apx;
  if (s_ret + s_apx == 0) s_ret = 1;             // nothing cached: one workgroup writes the empty partial
}

template <typename T, int D, int G, bool PAGED>
int run_decode_layout(const vector_cache& c, DecodeParams& p, hipStream_t stream, const RopeParams* rope) {
  const dim3 grid(p.splits_ret + p.splits_apx, c.n_kv_heads, c.batch);
  if constexpr (Elem<T>::kDtype == VECTOR_BF16) {
    constexpr int lds = MfmaDecodeTile<D>::kLdsBytes;
    if (rope) {
      VEC_HIP(set_max_lds(reinterpret_cast<const void*>(decode_split_mfma_kernel<D, G, true, false, PAGED>), lds));
      VEC_LAUNCH(K_DECODE_SPLIT, (decode_split_mfma_kernel<D, G, true, false, PAGED>), grid, dim3(DT_), lds, stream, p, *rope);
    } else if (p.literal) {
      VEC_HIP(set_max_lds(reinterpret_cast<const void*>(decode_split_mfma_kernel<D, G, false, true, PAGED>), lds));
      VEC_LAUNCH(K_DECODE_SPLIT, (decode_split_mfma_kernel<D, G, false, true, PAGED>), grid, dim3(DT_), lds, stream, p, RopeParams{});
    } else {
      VEC_HIP(set_max_lds(reinterpret_cast<const void*>(decode_split_mfma_kernel<D, G, false, false, PAGED>), lds));
      VEC_LAUNCH(K_DECODE_SPLIT, (decode_split_mfma_kernel<D, G, false, false, PAGED>), grid, dim3(DT_), lds, stream, p, RopeParams{});
    }
  } else {
    if (rope) {
      VEC_LAUNCH(K_DECODE_SPLIT, (decode_split_kernel<T, D, G, PAGED, true>), grid, dim3(DT_), 0, stream, p, *rope);
    } else {
      VEC_LAUNCH(K_DECODE_SPLIT, (decode_split_kernel<T, D, G, PAGED, false>), grid, dim3(DT_), 0, stream, p, RopeParams{});
    }
  }
  VEC_LAUNCH(K_DECODE_COMBINE, (decode_combine_kernel<T, D, G>), dim3(c.n_kv_heads, c.batch), dim3(256), 0, stream, p);
  VEC_HIP(hipGetLastError());
  return VECTOR_OK;
}

template <typename T, int D, int G>
int run_decode(const vector_cache& c, DecodeParams& p, hipStream_t stream, const RopeParams* rope) {
  return p.block_table ? run_decode_layout<T, D, G, true>(c, p, stream, rope) : run_decode_layout<T, D, G, false>(c, p, stream, rope);
}

template <typename T, int D>
int run_decode_g(const vector_cache& c, DecodeParams& p, hipStream_t stream, const RopeParams* rope) {
  switch (c.n_q_heads / c.n_kv_heads) {
    case 1: return run_decode<T, D, 1>(c, p, stream, rope);
    case 2: return run_decode<T, D, 2>(c, p, stream, rope);
    case 3: return run_decode<T, D, 3>(c, p, stream, rope);
    case 4: return run_decode<T, D, 4>(c, p, stream, rope);
    case 5: return run_decode<T, D, 5>(c, p, stream, rope);
    case 6: return run_decode<T, D, 6>(c, p, stream, rope);
    case 7: return run_decode<T, D, 7>(c, p, stream, rope);
    case 8: return run_decode<T, D, 8>(c, p, stream, rope);
    case 10: return run_decode<T, D, 10>(c, p, stream, rope);
    case 12: return run_decode<T, D, 12>(c, p, stream, rope);
    case 16: return run_decode<T, D, 16>(c, p, stream, rope);
    default: return VECTOR_ERR_SHAPE;
  }
}

}  // namespace

size_t decode_workspace_bytes(int batch, int n_q_heads, int n_kv_heads, int head_dim, int cap_retain, int n_approx) {
  // sized for the largest split count so that the bound holds for any live length
  (void)cap_retain; (void)n_approx;
  const int G = n_q_heads / n_kv_heads;
  return align_up((size_t)batch * n_kv_heads * 2 * kMaxSplits * (2 * G + G * head_dim) * sizeof(float), 256);
}

int launch_decode_attn(const vector_cache& c, const void* q, float scale, void* out, int flags, void* ws,
                       hipStream_t stream, const RopeParams* rope, const void* k_new, const void* v_new) {
  DecodeParams p;
  p.literal = (flags & VECTOR_DECODE_LITERAL) ? 1 : 0;
  p.out_f32 = (flags & VECTOR_DECODE_OUT_F32) ? 1 : 0;
  if (p.literal && (rope || c.dtype != VECTOR_BF16)) return VECTOR_ERR_DTYPE;
  p.q = q; p.k_ret = c.k_ret; p.v_ret = c.v_ret; p.k_apx = c.k_apx; p.W = c.W; p.len_retain = c.len_retain;
  p.k_new = k_new; p.v_new = v_new;
  p.block_table = c.ret_block_table; p.block_shift = 0; p.blocks_per_seq = c.ret_blocks_per_seq;
  while (c.ret_block_table && (1 << p.block_shift) < c.ret_block_rows) ++p.block_shift;
  p.cap_retain_seq = c.cap_retain_seq; p.n_approx_seq = c.n_approx_seq;
  p.ret_row_start = c.ret_row_start; p.apx_row_start = c.apx_row_start;
  p.out = out; p.part = reinterpret_cast<float*>(ws);
  p.B = c.batch; p.Hq = c.n_q_heads; p.Hkv = c.n_kv_heads; p.cap_retain = c.cap_retain; p.n_approx = c.n_approx;
  // an approximated row costs its bytes; with the rotary un-rotation its sines and cosines make
  // it cost about as much as two rows' worth of streaming
  pick_splits(c.dtype == VECTOR_BF16 ? kTargetWorkgroupsMfma : kTargetWorkgroups, c.batch, c.n_kv_heads, c.cap_retain, c.n_approx,
              rope ? kRopeApxCost : 1.0, p.splits_ret, p.splits_apx);
  p.w_sh = c.w_shared ? 0 : (int64_t)c.head_dim * c.head_dim;
  p.c2 = scale * kLog2e;
  if (c.dtype == VECTOR_BF16) {
    if (c.head_dim == 128) return run_decode_g<bf16_t, 128>(c, p, stream, rope);
    if (c.head_dim == 64) return run_decode_g<bf16_t, 64>(c, p, stream, rope);
  } else if (c.dtype == VECTOR_F32) {
    if (c.head_dim == 128) return run_decode_g<float, 128>(c, p, stream, rope);
    if (c.head_dim == 64) return run_decode_g<float, 64>(c, p, stream, rope);
  } else {
    return VECTOR_ERR_DTYPE;
  }
  return VECTOR_ERR_SHAPE;
}

}  // namespace vec
