// C ABI of libvector: argument validation and dispatch to the kernel launchers.
// Everything is checked on the host before the first launch, so a failing call
// leaves the outputs untouched.
#include <math.h>
#include <string.h>

#include <algorithm>

#include "../../include/vector.h"
#include "common.hpp"
#include "launch.hpp"

namespace {

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

int check_shape(const vector_shape* s, bool need_window) {
  if (!s) return VECTOR_ERR_ARG;
  if (s->dtype != VECTOR_F32 && s->dtype != VECTOR_BF16) return VECTOR_ERR_DTYPE;
  if (s->head_dim != 64 && s->head_dim != 128) return VECTOR_ERR_SHAPE;
  if (s->n_kv_heads < 1 || s->n_kv_heads > 65535 || s->n_q_heads < s->n_kv_heads || s->n_q_heads % s->n_kv_heads) return VECTOR_ERR_SHAPE;
  if (s->seq_len < 1 || s->seq_len > vec::kRouteMaxSeqLen) return VECTOR_ERR_SHAPE;
  const int align = s->dtype == VECTOR_BF16 ? 8 : 4;      // elements per 16 bytes
  const int64_t strides[5] = {s->k_stride_head, s->k_stride_tok, s->v_stride_head, s->v_stride_tok, s->w_stride_head};
  for (int64_t st : strides)
    if (st < 0 || st % align) return VECTOR_ERR_SHAPE;
  if ((s->k_stride_tok && s->k_stride_tok < s->head_dim) || (s->v_stride_tok && s->v_stride_tok < s->head_dim)) return VECTOR_ERR_SHAPE;
  if (need_window) {
    if (s->window < 1 || s->window > s->seq_len) return VECTOR_ERR_SHAPE;
    if (s->pool_kernel < 1 || !(s->pool_kernel & 1)) return VECTOR_ERR_SHAPE;
    if (s->pool_mode != VECTOR_POOL_AVG && s->pool_mode != VECTOR_POOL_MAX) return VECTOR_ERR_SHAPE;
  }
  return VECTOR_OK;
}

// frequencies in radians per position (host) -> turns per position, by value for the kernels
int make_rope(const vector_rope* r, int head_dim, vec::RopeParams& out) {
  if (!r || !r->inv_freq || head_dim / 2 > vec::kMaxRotaryPairs) return VECTOR_ERR_ARG;
  if (r->pos_offset < 0 || r->pos_offset >= (1 << 24)) return VECTOR_ERR_ARG;
  const double two_pi = 6.283185307179586476925286766559;
  for (int i = 0; i < vec::kMaxRotaryPairs; ++i) out.turns_hi[i] = out.turns_lo[i] = 0.f;
  for (int i = 0; i < head_dim / 2; ++i) {
    if (!(r->inv_freq[i] == r->inv_freq[i])) return VECTOR_ERR_ARG;
    const double t = r->inv_freq[i] / two_pi;
    out.turns_hi[i] = (float)t;
    out.turns_lo[i] = (float)(t - (double)out.turns_hi[i]);
  }
  out.positions = r->positions;
  out.pos_offset = r->pos_offset;
  out.interleaved = r->interleaved != 0;
  return VECTOR_OK;
}

int check_ws(const void* ws, size_t have, size_t need) {
  if (need == 0) return VECTOR_OK;
  if (!ws || (reinterpret_cast<uintptr_t>(ws) & 255u) || have < need) return VECTOR_ERR_WORKSPACE;
  return VECTOR_OK;
}

}  // namespace

extern "C" {

int vector_budget_counts_frac(int32_t n, double f_retain, double f_approx, int32_t* n_pool, int32_t* n_approx) {
  if (!n_pool || !n_approx || n < 0) return VECTOR_ERR_ARG;
  if (!(f_retain >= 0.0) || !(f_approx >= 0.0) || f_retain + f_approx > 1.0 + 1e-12) return VECTOR_ERR_ARG;
  // the fractions are decimal ratios that binary doubles only approximate (1 - 0.9 - 0.05 is a hair
  // under 0.05): a product within 1e-9 of an integer is that integer
  const int32_t n_r = (int32_t)floor(f_retain * (double)n + 1e-9);
  const int32_t n_a = (int32_t)floor(f_approx * (double)n + 1e-9);
  *n_pool = n_r + n_a;
  *n_approx = n_a;
  return VECTOR_OK;
}

int vector_budget_counts(int32_t n, double p_c, double p_a, int32_t* n_pool, int32_t* n_approx) {
  if (!(p_c >= 0.0 && p_c <= 1.0) || !(p_a >= 0.0) || p_a > p_c + 1e-12 || 1.0 - p_c - p_a < -1e-12) return VECTOR_ERR_ARG;
  double f_retain = 1.0 - p_c - p_a;
  if (f_retain < 0.0) f_retain = 0.0;
  return vector_budget_counts_frac(n, f_retain, 2.0 * p_a, n_pool, n_approx);
}

double vector_pa_deploy(double p_c, double eps) {
  const double a = p_c / 2.0, b = (1.0 - p_c - eps) / 2.0;
  return a < b ? a : b;
}

size_t vector_workspace_bytes(const vector_shape* s, int32_t n_pool, int32_t n_approx, int32_t batch) {
  if (check_shape(s, true) != VECTOR_OK || n_pool < 0 || n_approx < 0 || n_approx > n_pool || batch < 1) return 0;
  size_t need = vec::score_workspace_bytes(*s);
  const size_t r = vec::route_workspace_bytes(s->n_kv_heads, s->seq_len, n_pool);
  if (r > need) need = r;
  // decode: the retained segment may grow by appended tokens up to seq_len rows
  const size_t d = vec::decode_workspace_bytes(batch, s->n_q_heads, s->n_kv_heads, s->head_dim, s->seq_len, n_approx);
  if (d > need) need = d;
  return need + 256;
}

const char* vector_strerror(int code) {
  switch (code) {
    case VECTOR_OK: return "ok";
    case VECTOR_ERR_ARG: return "invalid argument";
    case VECTOR_ERR_SHAPE: return "unsupported shape";
    case VECTOR_ERR_WORKSPACE: return "workspace too small or misaligned";
    case VECTOR_ERR_DTYPE: return "unknown element type";
    case VECTOR_ERR_HIP: return "HIP runtime error";
    default: return "unknown error";
  }
}

int vector_score(const vector_shape* s, const void* q_win, const void* k, float* score, void* ws, size_t ws_bytes,
                 void* stream) {
  int rc = check_shape(s, true);
  if (rc) return rc;
  if (!q_win || !k || !score || !aligned16(q_win) || !aligned16(k)) return VECTOR_ERR_ARG;
  if ((rc = check_ws(ws, ws_bytes, vec::score_workspace_bytes(*s)))) return rc;
  return vec::launch_score_residual(*s, q_win, k, nullptr, nullptr, score, nullptr, ws, (hipStream_t)stream);
}

int vector_residual(const vector_shape* s, const void* k, const void* v, const void* W, float* eps, void* ws,
                    size_t ws_bytes, void* stream) {
  (void)ws; (void)ws_bytes;
  int rc = check_shape(s, false);
  if (rc) return rc;
  if (!k || !v || !W || !eps || !aligned16(k) || !aligned16(v) || !aligned16(W)) return VECTOR_ERR_ARG;
  vector_shape t = *s;
  if (t.window < 1 || t.window > t.seq_len) t.window = 1;     // unused by the residual
  return vec::launch_score_residual(t, nullptr, k, v, W, nullptr, eps, nullptr, (hipStream_t)stream);
}

size_t vector_score_key_diversity_workspace_bytes(const vector_shape* s) {
  if (check_shape(s, false) != VECTOR_OK) return 0;
  return vec::diversity_workspace_bytes(*s);
}

int vector_score_key_diversity(const vector_shape* s, const void* k, float* score, void* ws, size_t ws_bytes, void* stream) {
  int rc = check_shape(s, false);
  if (rc) return rc;
  if (!k || !score || !aligned16(k)) return VECTOR_ERR_ARG;
  if ((rc = check_ws(ws, ws_bytes, vec::diversity_workspace_bytes(*s)))) return rc;
  return vec::launch_key_diversity(*s, k, score, ws, (hipStream_t)stream);
}

size_t vector_compress_workspace_bytes(const vector_shape* s, int32_t n_pool, int32_t n_approx) {
  if (check_shape(s, true) != VECTOR_OK || n_pool < 0 || n_approx < 0 || n_approx > n_pool) return 0;
  return vec::score_workspace_bytes(*s) + vec::route_workspace_bytes(s->n_kv_heads, s->seq_len, n_pool) + 256;
}

static int check_lse(const vector_shape* s, const vec::QueryLse* lse) {
  if (!lse->lse || (reinterpret_cast<uintptr_t>(lse->lse) & 3u)) return VECTOR_ERR_ARG;
  if (lse->stride_head != 0 && lse->stride_head < s->window) return VECTOR_ERR_ARG;
  return VECTOR_OK;
}

// vector_compress; with `stack`, several sequences of one shape as one problem (s holds the stacked head counts)
static int compress_impl(const vector_shape* s, const void* q_win, const void* k, const void* v, const void* W, int32_t n_pool,
                         int32_t n_approx, float* score, float* eps, uint8_t* tier, int32_t* idx_retain, int32_t* idx_approx,
                         void* k_ret, void* v_ret, void* k_apx, int32_t cap_retain, void* ws, size_t ws_bytes, void* stream,
                         const vec::SeqStack* stack, const vec::QueryLse* lse = nullptr, const vec::RopeParams* rope = nullptr) {
  int rc = check_shape(s, true);
  if (rc) return rc;
  if (lse && (rc = check_lse(s, lse))) return rc;
  const int n_retain = n_pool - n_approx;
  if (n_approx < 0 || n_pool < n_approx || n_pool > s->seq_len || cap_retain < n_retain) return VECTOR_ERR_ARG;
  if (!q_win || !k || !v || !W || !score || !eps || !tier) return VECTOR_ERR_ARG;
  if (!aligned16(q_win) || !aligned16(k) || !aligned16(v) || !aligned16(W)) return VECTOR_ERR_ARG;
  if (n_retain > 0 && (!idx_retain || !k_ret || !v_ret || !aligned16(k_ret) || !aligned16(v_ret))) return VECTOR_ERR_ARG;
  if (n_approx > 0 && (!idx_approx || !k_apx || !aligned16(k_apx))) return VECTOR_ERR_ARG;
  const size_t score_ws = vec::score_workspace_bytes(*s);
  if ((rc = check_ws(ws, ws_bytes, vector_compress_workspace_bytes(s, n_pool, n_approx)))) return rc;
  hipStream_t st = (hipStream_t)stream;
  void* route_ws = reinterpret_cast<unsigned char*>(ws) + (score_ws + 255) / 256 * 256;
  // the scorer's pooling launch also builds the routing's buckets of score keys
  void* buckets = n_pool > 0 ? route_ws : nullptr;
  if ((rc = vec::launch_score_residual(*s, q_win, k, v, W, score, eps, ws, st, rope, buckets, stack, lse))) return rc;
  if ((rc = vec::launch_route(s->n_kv_heads, s->seq_len, score, eps, n_pool, n_approx, tier, idx_retain, idx_approx, route_ws,
                              buckets != nullptr, st)))
    return rc;
  return vec::launch_compact(*s, k, v, idx_retain, idx_approx, n_retain, n_approx, k_ret, v_ret, k_apx, cap_retain, st, stack);
}

int vector_compress(const vector_shape* s, const void* q_win, const void* k, const void* v, const void* W, int32_t n_pool,
                    int32_t n_approx, float* score, float* eps, uint8_t* tier, int32_t* idx_retain, int32_t* idx_approx,
                    void* k_ret, void* v_ret, void* k_apx, int32_t cap_retain, void* ws, size_t ws_bytes, void* stream) {
  return compress_impl(s, q_win, k, v, W, n_pool, n_approx, score, eps, tier, idx_retain, idx_approx, k_ret, v_ret, k_apx, cap_retain,
                       ws, ws_bytes, stream, nullptr);
}

int vector_compress_lse(const vector_shape* s, const void* q_win, const void* k, const void* v, const void* W, const float* lse,
                        int64_t lse_stride_head, int32_t n_pool, int32_t n_approx, float* score, float* eps, uint8_t* tier,
                        int32_t* idx_retain, int32_t* idx_approx, void* k_ret, void* v_ret, void* k_apx, int32_t cap_retain,
                        void* ws, size_t ws_bytes, void* stream) {
  const vec::QueryLse ql = {lse, lse_stride_head};
  return compress_impl(s, q_win, k, v, W, n_pool, n_approx, score, eps, tier, idx_retain, idx_approx, k_ret, v_ret, k_apx, cap_retain,
                       ws, ws_bytes, stream, nullptr, &ql);
}

namespace {

// sequence b of a batch as a one-sequence problem: its shape (explicit strides, so that a packed
// ragged [Hkv, T, d] keeps its head stride) and where its blocks start
struct BatchItem {
  vector_shape shape;
  int64_t tok0, ret0, apx0, cap0;     // running sums of seq_len, n_retain, n_approx, cap_retain
};

int check_batch(const vector_shape* s, const vector_batch* bt) {
  if (!s || !bt) return VECTOR_ERR_ARG;
  if (bt->batch < 1 || !bt->seq_len || !bt->n_pool || !bt->n_approx || !bt->cap_retain) return VECTOR_ERR_ARG;
  int64_t total = 0;
  for (int b = 0; b < bt->batch; ++b) {
    vector_shape t = *s;
    t.seq_len = bt->seq_len[b];
    const int rc = check_shape(&t, true);
    if (rc) return rc;
    const int n_pool = bt->n_pool[b], n_approx = bt->n_approx[b];
    if (n_approx < 0 || n_pool < n_approx || n_pool > t.seq_len || bt->cap_retain[b] < n_pool - n_approx) return VECTOR_ERR_ARG;
    total += t.seq_len;
  }
  if (total > ((int64_t)1 << 40)) return VECTOR_ERR_SHAPE;
  return VECTOR_OK;
}

// Sequences b0, b0 + 1, ... with the same length, counts and capacity are handled as one problem
// with their heads stacked: the launches then fill the chip instead of running once per sequence.
int run_length(const vector_shape* s, const vector_batch* bt, int b0) {
  const int max_run = 65535 / s->n_q_heads;              // stacked head counts stay within the grid limits
  int r = 1;
  while (b0 + r < bt->batch && r < max_run && bt->seq_len[b0 + r] == bt->seq_len[b0] && bt->n_pool[b0 + r] == bt->n_pool[b0] &&
         bt->n_approx[b0 + r] == bt->n_approx[b0] && bt->cap_retain[b0 + r] == bt->cap_retain[b0])
    ++r;
  return r;
}

BatchItem batch_item(const vector_shape* s, const vector_batch* bt, int b, int64_t total_tokens, const BatchItem* prev) {
  BatchItem it;
  it.shape = *s;
  it.shape.seq_len = bt->seq_len[b];
  if (!it.shape.k_stride_tok) it.shape.k_stride_tok = s->head_dim;
  if (!it.shape.k_stride_head) it.shape.k_stride_head = total_tokens * it.shape.k_stride_tok;
  if (!it.shape.v_stride_tok) it.shape.v_stride_tok = s->head_dim;
  if (!it.shape.v_stride_head) it.shape.v_stride_head = total_tokens * it.shape.v_stride_tok;
  it.tok0 = prev ? prev->tok0 + bt->seq_len[b - 1] : 0;
  it.ret0 = prev ? prev->ret0 + (bt->n_pool[b - 1] - bt->n_approx[b - 1]) : 0;
  it.apx0 = prev ? prev->apx0 + bt->n_approx[b - 1] : 0;
  it.cap0 = prev ? prev->cap0 + bt->cap_retain[b - 1] : 0;
  return it;
}

}  // namespace

namespace {
// How the sequences from b0 on are taken together: a run of equal sequences (stacked heads), or a
// group of sequences of different lengths (one set of launches over their parameter tables), or
// one sequence on its own.
enum { PART_SINGLE = 0, PART_STACK, PART_RAGGED };
struct BatchPart { int kind, count; };

BatchPart next_part(const vector_shape* s, const vector_batch* bt, int b0, bool ragged_ok) {
  const int run = run_length(s, bt, b0);
  if (run > 1) return {PART_STACK, run};
  if (!ragged_ok || bt->n_pool[b0] < 1) return {PART_SINGLE, 1};
  const int max_count = std::min(vec::kMaxRaggedSeqs, 65535 / s->n_q_heads);
  int c = 1;
  while (b0 + c < bt->batch && c < max_count && bt->n_pool[b0 + c] >= 1 && run_length(s, bt, b0 + c) == 1) ++c;
  return {c > 1 ? PART_RAGGED : PART_SINGLE, c};
}

size_t seq_workspace_bytes(const vector_shape* s, const vector_batch* bt, int b) {
  vector_shape t = *s;
  t.seq_len = bt->seq_len[b];
  return (vector_compress_workspace_bytes(&t, bt->n_pool[b], bt->n_approx[b]) + 255) / 256 * 256;
}
}  // namespace

size_t vector_compress_batch_workspace_bytes(const vector_shape* s, const vector_batch* bt) {
  if (check_batch(s, bt) != VECTOR_OK) return 0;
  const bool ragged_ok = vec::score_heads_in_one_group(*s);
  size_t need = 0;
  for (int b = 0; b < bt->batch;) {
    const BatchPart part = next_part(s, bt, b, ragged_ok);
    size_t one = 0;
    if (part.kind == PART_RAGGED) {
      one = (vec::ragged_table_bytes(part.count) + 255) / 256 * 256;
      for (int i = 0; i < part.count; ++i) one += seq_workspace_bytes(s, bt, b + i);
    } else {
      vector_shape t = *s;
      t.seq_len = bt->seq_len[b];
      t.n_kv_heads *= part.count;
      t.n_q_heads *= part.count;
      one = vector_compress_workspace_bytes(&t, bt->n_pool[b], bt->n_approx[b]);
    }
    if (one > need) need = one;
    b += part.count;
  }
  return need;
}

// rope: null, or the rotary parameters with `positions` still the batch's array (ragged along the
// token axis like k), of which every part gets its piece
static int compress_batch_impl(const vector_shape* s, const vector_batch* bt, const void* q_win, const void* k, const void* v,
                               const void* W, float* score, float* eps, uint8_t* tier, int32_t* idx_retain, int32_t* idx_approx,
                               void* k_ret, void* v_ret, void* k_apx, void* ws, size_t ws_bytes, void* stream,
                               const vec::RopeParams* rope, const vec::QueryLse* lse = nullptr) {
  int rc = check_batch(s, bt);
  if (rc) return rc;
  if (lse && (rc = check_lse(s, lse))) return rc;
  // lse: [batch, Hq, stride_head] floats, sequence after sequence
  const int64_t lse_sh = lse ? (lse->stride_head ? lse->stride_head : s->window) : 0;
  const int64_t lse_seq = lse_sh * s->n_q_heads;
  if (!q_win || !k || !v || !W || !score || !eps || !tier) return VECTOR_ERR_ARG;
  if (!aligned16(q_win) || !aligned16(k) || !aligned16(v) || !aligned16(W)) return VECTOR_ERR_ARG;
  int64_t total = 0, total_ret = 0, total_apx = 0;
  for (int b = 0; b < bt->batch; ++b) {
    total += bt->seq_len[b];
    total_ret += bt->n_pool[b] - bt->n_approx[b];
    total_apx += bt->n_approx[b];
  }
  if (total_ret > 0 && (!idx_retain || !k_ret || !v_ret || !aligned16(k_ret) || !aligned16(v_ret))) return VECTOR_ERR_ARG;
  if (total_apx > 0 && (!idx_approx || !k_apx || !aligned16(k_apx))) return VECTOR_ERR_ARG;
  if ((rc = check_ws(ws, ws_bytes, vector_compress_batch_workspace_bytes(s, bt)))) return rc;
  // One part after the other on the stream (a run of equal sequences with its heads stacked, a group
  // of unequal ones over parameter tables, or a single sequence): the launches follow each other
  // without a host wait, and the workspace is reused in stream order.
  const size_t esz = s->dtype == VECTOR_BF16 ? 2 : 4;
  const int64_t H = s->n_kv_heads, d = s->head_dim;
  const bool ragged_ok = vec::score_heads_in_one_group(*s);
  hipStream_t st = (hipStream_t)stream;
  BatchItem it{}, prev{};
  for (int b = 0; b < bt->batch;) {
    const BatchPart part = next_part(s, bt, b, ragged_ok);
    if (part.kind == PART_RAGGED) {
      vec::RaggedSeq seqs[vec::kMaxRaggedSeqs];
      unsigned char* w8 = reinterpret_cast<unsigned char*>(ws);
      void* tables = w8;
      w8 += (vec::ragged_table_bytes(part.count) + 255) / 256 * 256;
      int64_t seqs_tok0 = 0;
      for (int i = 0; i < part.count; ++i) {
        const int bi = b + i;
        it = batch_item(s, bt, bi, total, bi ? &prev : nullptr);
        prev = it;
        if (i == 0) seqs_tok0 = it.tok0;
        vec::RaggedSeq& q = seqs[i];
        q.shape = it.shape;
        q.q = reinterpret_cast<const unsigned char*>(q_win) + (size_t)bi * s->n_q_heads * s->window * d * esz;
        q.k = reinterpret_cast<const unsigned char*>(k) + (size_t)(it.tok0 * it.shape.k_stride_tok) * esz;
        q.v = reinterpret_cast<const unsigned char*>(v) + (size_t)(it.tok0 * it.shape.v_stride_tok) * esz;
        q.score = score + H * it.tok0; q.eps = eps + H * it.tok0; q.tier = tier + H * it.tok0;
        q.idx_retain = idx_retain ? idx_retain + H * it.ret0 : nullptr;
        q.idx_approx = idx_approx ? idx_approx + H * it.apx0 : nullptr;
        q.k_ret = k_ret ? reinterpret_cast<unsigned char*>(k_ret) + (size_t)(H * it.cap0 * d) * esz : nullptr;
        q.v_ret = v_ret ? reinterpret_cast<unsigned char*>(v_ret) + (size_t)(H * it.cap0 * d) * esz : nullptr;
        q.k_apx = k_apx ? reinterpret_cast<unsigned char*>(k_apx) + (size_t)(H * it.apx0 * d) * esz : nullptr;
        q.n_pool = bt->n_pool[bi]; q.n_approx = bt->n_approx[bi]; q.cap_retain = bt->cap_retain[bi];
        q.pos_base = it.tok0 - seqs_tok0;
        q.lse = lse ? lse->lse + bi * lse_seq : nullptr;
        q.lse_stride_head = lse_sh;
        q.score_ws = w8;
        q.route_ws = w8 + (vec::score_workspace_bytes(it.shape) + 255) / 256 * 256;
        w8 += seq_workspace_bytes(s, bt, bi);
      }
      vec::RopeParams rp_part;
      if (rope) {
        rp_part = *rope;
        if (rope->positions) rp_part.positions = rope->positions + seqs_tok0;
      }
      if ((rc = vec::launch_score_residual_ragged(*s, seqs, part.count, W, tables, st, rope ? &rp_part : nullptr))) return rc;
      unsigned char* route_tables = reinterpret_cast<unsigned char*>(tables) + vec::ragged_table_bytes(part.count) -
                                    vec::route_ragged_table_bytes(part.count);
      if ((rc = vec::launch_route_compact_ragged(*s, seqs, part.count, route_tables, st))) return rc;
      b += part.count;
      continue;
    }
    it = batch_item(s, bt, b, total, b ? &prev : nullptr);
    prev = it;
    for (int i = 1; i < part.count; ++i) prev = batch_item(s, bt, b + i, total, &prev);     // the running sums skip over the run
    vec::SeqStack stack;
    stack.heads_per_seq = s->n_kv_heads;
    stack.k_stride_seq = (int64_t)bt->seq_len[b] * it.shape.k_stride_tok;     // ragged token axis: the next sequence follows
    stack.v_stride_seq = (int64_t)bt->seq_len[b] * it.shape.v_stride_tok;
    it.shape.n_kv_heads *= part.count;
    it.shape.n_q_heads *= part.count;
    const unsigned char* kb = reinterpret_cast<const unsigned char*>(k) + (size_t)(it.tok0 * it.shape.k_stride_tok) * esz;
    const unsigned char* vb = reinterpret_cast<const unsigned char*>(v) + (size_t)(it.tok0 * it.shape.v_stride_tok) * esz;
    const unsigned char* qb = reinterpret_cast<const unsigned char*>(q_win) + (size_t)b * s->n_q_heads * s->window * d * esz;
    const int n_pool = bt->n_pool[b], n_approx = bt->n_approx[b];
    const vec::QueryLse lse_one = {lse ? lse->lse + b * lse_seq : nullptr, lse_sh};     // a run's sequences follow each other
    vec::RopeParams rp_one;
    if (rope) {
      rp_one = *rope;
      if (rope->positions) rp_one.positions = rope->positions + it.tok0;
    }
    rc = compress_impl(&it.shape, qb, kb, vb, W, n_pool, n_approx, score + H * it.tok0, eps + H * it.tok0, tier + H * it.tok0,
                         idx_retain ? idx_retain + H * it.ret0 : nullptr, idx_approx ? idx_approx + H * it.apx0 : nullptr,
                         k_ret ? reinterpret_cast<unsigned char*>(k_ret) + (size_t)(H * it.cap0 * d) * esz : nullptr,
                         v_ret ? reinterpret_cast<unsigned char*>(v_ret) + (size_t)(H * it.cap0 * d) * esz : nullptr,
                         k_apx ? reinterpret_cast<unsigned char*>(k_apx) + (size_t)(H * it.apx0 * d) * esz : nullptr,
                         bt->cap_retain[b], ws, ws_bytes, stream, part.count > 1 ? &stack : nullptr, lse ? &lse_one : nullptr,
                         rope ? &rp_one : nullptr);
    if (rc) return rc;
    b += part.count;
  }
  return VECTOR_OK;
}

int vector_compress_batch(const vector_shape* s, const vector_batch* bt, const void* q_win, const void* k, const void* v,
                          const void* W, float* score, float* eps, uint8_t* tier, int32_t* idx_retain, int32_t* idx_approx,
                          void* k_ret, void* v_ret, void* k_apx, void* ws, size_t ws_bytes, void* stream) {
  return compress_batch_impl(s, bt, q_win, k, v, W, score, eps, tier, idx_retain, idx_approx, k_ret, v_ret, k_apx, ws, ws_bytes, stream,
                             nullptr);
}

int vector_compress_batch_rope(const vector_shape* s, const vector_batch* bt, const vector_rope* rope, const void* q_win, const void* k,
                               const void* v, const void* W, float* score, float* eps, uint8_t* tier, int32_t* idx_retain,
                               int32_t* idx_approx, void* k_ret, void* v_ret, void* k_apx, void* ws, size_t ws_bytes, void* stream) {
  if (!s) return VECTOR_ERR_ARG;
  vec::RopeParams rp;
  const int rc = make_rope(rope, s->head_dim, rp);
  if (rc) return rc;
  return compress_batch_impl(s, bt, q_win, k, v, W, score, eps, tier, idx_retain, idx_approx, k_ret, v_ret, k_apx, ws, ws_bytes, stream, &rp);
}

size_t vector_calibrate_workspace_bytes(const vector_shape* s) {
  if (check_shape(s, false) != VECTOR_OK) return 0;
  return vec::calibrate_workspace_bytes(*s);
}

int vector_calibrate(const vector_shape* s, const void* k, const void* v, void* W, void* ws, size_t ws_bytes, void* stream) {
  int rc = check_shape(s, false);
  if (rc) return rc;
  if (!k || !v || !W || !aligned16(k) || !aligned16(v) || !aligned16(W)) return VECTOR_ERR_ARG;
  if (s->seq_len < s->head_dim) return VECTOR_ERR_ARG;          // fewer tokens than unknowns per column: singular
  if ((rc = check_ws(ws, ws_bytes, vec::calibrate_workspace_bytes(*s)))) return rc;
  return vec::launch_calibrate(*s, k, v, W, ws, (hipStream_t)stream);
}

size_t vector_distortion_workspace_bytes(const vector_shape* s) {
  if (check_shape(s, false) != VECTOR_OK) return 0;
  return vec::distortion_workspace_bytes(s->n_kv_heads, s->seq_len);
}

int vector_distortion(const vector_shape* s, const float* weights, const uint8_t* tier, const float* eps, const void* v,
                      double* out, void* ws, size_t ws_bytes, void* stream) {
  int rc = check_shape(s, false);
  if (rc) return rc;
  if (!weights || !tier || !eps || !v || !out || !aligned16(v)) return VECTOR_ERR_ARG;
  if ((rc = check_ws(ws, ws_bytes, vec::distortion_workspace_bytes(s->n_kv_heads, s->seq_len)))) return rc;
  return vec::launch_distortion(*s, weights, tier, eps, v, out, ws, (hipStream_t)stream);
}

size_t vector_r2_workspace_bytes(const vector_shape* s) {
  if (check_shape(s, false) != VECTOR_OK) return 0;
  return vec::r2_workspace_bytes(s->n_kv_heads, s->seq_len, s->head_dim);
}

int vector_r2(const vector_shape* s, const void* k, const void* v, const void* W, double* out, void* ws, size_t ws_bytes,
              void* stream) {
  int rc = check_shape(s, false);
  if (rc) return rc;
  if (!k || !v || !W || !out || !aligned16(k) || !aligned16(v) || !aligned16(W)) return VECTOR_ERR_ARG;
  if ((rc = check_ws(ws, ws_bytes, vec::r2_workspace_bytes(s->n_kv_heads, s->seq_len, s->head_dim)))) return rc;
  vector_shape t = *s;
  if (t.window < 1 || t.window > t.seq_len) t.window = 1;
  float* eps = reinterpret_cast<float*>(ws);
  rc = vec::launch_score_residual(t, nullptr, k, v, W, nullptr, eps, nullptr, (hipStream_t)stream);
  if (rc) return rc;
  unsigned char* part = reinterpret_cast<unsigned char*>(ws) + ((size_t)s->n_kv_heads * s->seq_len * sizeof(float) + 255) / 256 * 256;
  return vec::launch_r2(*s, eps, v, out, part, (hipStream_t)stream);
}

int vector_probe_residual_mfma(const vector_shape* s, const void* k, const void* v, const void* W, float* eps,
                               int32_t repeat, void* stream) {
  int rc = check_shape(s, false);
  if (rc) return rc;
  if (!k || !v || !W || !eps || !aligned16(k) || !aligned16(v) || !aligned16(W) || repeat < 1) return VECTOR_ERR_ARG;
  vector_shape t = *s;
  if (t.window < 1 || t.window > t.seq_len) t.window = 1;
  return vec::launch_residual_probe(t, k, v, W, eps, repeat, (hipStream_t)stream);
}

int vector_score_residual(const vector_shape* s, const void* q_win, const void* k, const void* v, const void* W,
                          float* score, float* eps, void* ws, size_t ws_bytes, void* stream) {
  int rc = check_shape(s, true);
  if (rc) return rc;
  if (!q_win || !k || !v || !W || !score || !eps) return VECTOR_ERR_ARG;
  if (!aligned16(q_win) || !aligned16(k) || !aligned16(v) || !aligned16(W)) return VECTOR_ERR_ARG;
  if ((rc = check_ws(ws, ws_bytes, vec::score_workspace_bytes(*s)))) return rc;
  return vec::launch_score_residual(*s, q_win, k, v, W, score, eps, ws, (hipStream_t)stream);
}

int vector_score_residual_lse(const vector_shape* s, const void* q_win, const void* k, const void* v, const void* W,
                              const float* lse, int64_t lse_stride_head, float* score, float* eps, void* ws, size_t ws_bytes,
                              void* stream) {
  int rc = check_shape(s, true);
  if (rc) return rc;
  const vec::QueryLse ql = {lse, lse_stride_head};
  if ((rc = check_lse(s, &ql))) return rc;
  if (!q_win || !k || !v || !W || !score || !eps) return VECTOR_ERR_ARG;
  if (!aligned16(q_win) || !aligned16(k) || !aligned16(v) || !aligned16(W)) return VECTOR_ERR_ARG;
  if ((rc = check_ws(ws, ws_bytes, vec::score_workspace_bytes(*s)))) return rc;
  return vec::launch_score_residual(*s, q_win, k, v, W, score, eps, ws, (hipStream_t)stream, nullptr, nullptr, nullptr, &ql);
}

int vector_route(int32_t n_kv_heads, int32_t seq_len, const float* score, const float* eps, int32_t n_pool,
                 int32_t n_approx, uint8_t* tier, int32_t* idx_retain, int32_t* idx_approx, void* ws, size_t ws_bytes,
                 void* stream) {
  if (n_kv_heads < 1 || n_kv_heads > 65535 || seq_len < 1 || seq_len > vec::kRouteMaxSeqLen) return VECTOR_ERR_SHAPE;
  if (n_approx < 0 || n_pool < n_approx || n_pool > seq_len) return VECTOR_ERR_ARG;
  if (!score || !eps || !tier) return VECTOR_ERR_ARG;
  if ((n_pool - n_approx > 0 && !idx_retain) || (n_approx > 0 && !idx_approx)) return VECTOR_ERR_ARG;
  int rc = check_ws(ws, ws_bytes, vec::route_workspace_bytes(n_kv_heads, seq_len, n_pool));
  if (rc) return rc;
  return vec::launch_route(n_kv_heads, seq_len, score, eps, n_pool, n_approx, tier, idx_retain, idx_approx, ws, false,
                           (hipStream_t)stream);
}

int vector_compact(const vector_shape* s, const void* k, const void* v, const int32_t* idx_retain,
                   const int32_t* idx_approx, int32_t n_retain, int32_t n_approx, void* k_ret, void* v_ret,
                   void* k_apx, int32_t cap_retain, void* stream) {
  int rc = check_shape(s, false);
  if (rc) return rc;
  if (n_retain < 0 || n_approx < 0 || cap_retain < n_retain || (int64_t)n_retain + n_approx > s->seq_len) return VECTOR_ERR_ARG;
  if (!k || !v || !aligned16(k) || !aligned16(v)) return VECTOR_ERR_ARG;
  if (n_retain > 0 && (!idx_retain || !k_ret || !v_ret || !aligned16(k_ret) || !aligned16(v_ret))) return VECTOR_ERR_ARG;
  if (n_approx > 0 && (!idx_approx || !k_apx || !aligned16(k_apx))) return VECTOR_ERR_ARG;
  return vec::launch_compact(*s, k, v, idx_retain, idx_approx, n_retain, n_approx, k_ret, v_ret, k_apx, cap_retain,
                             (hipStream_t)stream);
}

static int decode_checked(const vector_cache* c, const void* q, float scale, void* out, int32_t flags, void* ws,
                          size_t ws_bytes, void* stream, const vec::RopeParams* rope, const void* k_new = nullptr,
                          const void* v_new = nullptr, bool step = false) {
  if (!c || !q || !out) return VECTOR_ERR_ARG;
  if (step && (!k_new || !v_new || !aligned16(k_new) || !aligned16(v_new) || c->cap_retain < 1)) return VECTOR_ERR_ARG;
  if (c->dtype != VECTOR_F32 && c->dtype != VECTOR_BF16) return VECTOR_ERR_DTYPE;
  if (c->head_dim != 64 && c->head_dim != 128) return VECTOR_ERR_SHAPE;
  if (c->batch < 1 || c->batch > 65535 || c->n_kv_heads < 1 || c->n_kv_heads > 65535) return VECTOR_ERR_SHAPE;
  if (c->n_q_heads < c->n_kv_heads || c->n_q_heads % c->n_kv_heads) return VECTOR_ERR_SHAPE;
  const int G = c->n_q_heads / c->n_kv_heads;
  if (G > 8 && G != 10 && G != 12 && G != 16) return VECTOR_ERR_SHAPE;      // the group sizes the kernels are built for
  if (c->cap_retain < 0 || c->n_approx < 0 || (flags & ~(VECTOR_DECODE_LITERAL | VECTOR_DECODE_OUT_F32)) || !(scale == scale))
    return VECTOR_ERR_ARG;
  if ((flags & VECTOR_DECODE_LITERAL) && (rope || c->dtype != VECTOR_BF16)) return VECTOR_ERR_DTYPE;
  if (!c->len_retain) return VECTOR_ERR_ARG;
  const int n_seq_arrays = (c->cap_retain_seq != nullptr) + (c->n_approx_seq != nullptr) + (c->ret_row_start != nullptr) +
                           (c->apx_row_start != nullptr);
  if (n_seq_arrays != 0 && n_seq_arrays != 4) return VECTOR_ERR_ARG;
  if (c->ret_block_table) {
    const int rows = c->ret_block_rows;
    if (n_seq_arrays != 0 || rows < 16 || (rows & (rows - 1)) || c->ret_blocks_per_seq < 1) return VECTOR_ERR_ARG;
    if ((int64_t)c->cap_retain > (int64_t)c->ret_blocks_per_seq * rows) return VECTOR_ERR_ARG;
  }
  if (c->cap_retain > 0 && (!c->k_ret || !c->v_ret || !aligned16(c->k_ret) || !aligned16(c->v_ret))) return VECTOR_ERR_ARG;
  if (c->n_approx > 0 && (!c->k_apx || !c->W || !aligned16(c->k_apx) || !aligned16(c->W))) return VECTOR_ERR_ARG;
  if (!aligned16(q) || !aligned16(out)) return VECTOR_ERR_ARG;
  int rc = check_ws(ws, ws_bytes,
                    vec::decode_workspace_bytes(c->batch, c->n_q_heads, c->n_kv_heads, c->head_dim, c->cap_retain, c->n_approx));
  if (rc) return rc;
  return vec::launch_decode_attn(*c, q, scale, out, flags, ws, (hipStream_t)stream, rope, k_new, v_new);
}

int vector_decode_step(const vector_cache* c, const void* q, const void* k_new, const void* v_new, float scale, void* out,
                       int32_t flags, void* ws, size_t ws_bytes, void* stream) {
  return decode_checked(c, q, scale, out, flags, ws, ws_bytes, stream, nullptr, k_new, v_new, true);
}

int vector_decode_step_rope(const vector_cache* c, const vector_rope* rope, const void* q, const void* k_new, const void* v_new,
                            float scale, void* out, int32_t flags, void* ws, size_t ws_bytes, void* stream) {
  if (!c) return VECTOR_ERR_ARG;
  vec::RopeParams rp;
  int rc = make_rope(rope, c->head_dim, rp);
  if (rc) return rc;
  return decode_checked(c, q, scale, out, flags, ws, ws_bytes, stream, &rp, k_new, v_new, true);
}

int vector_decode_attn(const vector_cache* c, const void* q, float scale, void* out, int32_t flags, void* ws,
                       size_t ws_bytes, void* stream) {
  return decode_checked(c, q, scale, out, flags, ws, ws_bytes, stream, nullptr);
}

int vector_decode_attn_rope(const vector_cache* c, const vector_rope* rope, const void* q, float scale, void* out,
                            int32_t flags, void* ws, size_t ws_bytes, void* stream) {
  if (!c) return VECTOR_ERR_ARG;
  vec::RopeParams rp;
  int rc = make_rope(rope, c->head_dim, rp);
  if (rc) return rc;
  return decode_checked(c, q, scale, out, flags, ws, ws_bytes, stream, &rp);
}

int vector_residual_rope(const vector_shape* s, const void* k, const void* v, const void* W, const vector_rope* rope,
                         float* eps, void* ws, size_t ws_bytes, void* stream) {
  (void)ws; (void)ws_bytes;
  int rc = check_shape(s, false);
  if (rc) return rc;
  if (!k || !v || !W || !eps || !aligned16(k) || !aligned16(v) || !aligned16(W)) return VECTOR_ERR_ARG;
  vec::RopeParams rp;
  if ((rc = make_rope(rope, s->head_dim, rp))) return rc;
  vector_shape t = *s;
  if (t.window < 1 || t.window > t.seq_len) t.window = 1;     // unused by the residual
  return vec::launch_score_residual(t, nullptr, k, v, W, nullptr, eps, nullptr, (hipStream_t)stream, &rp);
}

int vector_score_residual_rope(const vector_shape* s, const void* q_win, const void* k, const void* v, const void* W,
                               const vector_rope* rope, float* score, float* eps, void* ws, size_t ws_bytes,
                               void* stream) {
  int rc = check_shape(s, true);
  if (rc) return rc;
  if (!q_win || !k || !v || !W || !score || !eps) return VECTOR_ERR_ARG;
  if (!aligned16(q_win) || !aligned16(k) || !aligned16(v) || !aligned16(W)) return VECTOR_ERR_ARG;
  vec::RopeParams rp;
  if ((rc = make_rope(rope, s->head_dim, rp))) return rc;
  if ((rc = check_ws(ws, ws_bytes, vec::score_workspace_bytes(*s)))) return rc;
  return vec::launch_score_residual(*s, q_win, k, v, W, score, eps, ws, (hipStream_t)stream, &rp);
}

int vector_compress_rope(const vector_shape* s, const vector_rope* rope, const void* q_win, const void* k, const void* v,
                         const void* W, int32_t n_pool, int32_t n_approx, float* score, float* eps, uint8_t* tier,
                         int32_t* idx_retain, int32_t* idx_approx, void* k_ret, void* v_ret, void* k_apx, int32_t cap_retain,
                         void* ws, size_t ws_bytes, void* stream) {
  if (!s) return VECTOR_ERR_ARG;
  vec::RopeParams rp;
  const int rc = make_rope(rope, s->head_dim, rp);
  if (rc) return rc;
  return compress_impl(s, q_win, k, v, W, n_pool, n_approx, score, eps, tier, idx_retain, idx_approx, k_ret, v_ret, k_apx, cap_retain,
                       ws, ws_bytes, stream, nullptr, nullptr, &rp);
}

// options -> the internal forms; rope parameters are built into `rp`
static int take_options(const vector_shape* s, const vector_compress_options* opt, vec::RopeParams& rp, const vec::RopeParams** rope,
                        vec::QueryLse& ql, const vec::QueryLse** lse) {
  *rope = nullptr;
  *lse = nullptr;
  if (!s) return VECTOR_ERR_ARG;
  if (!opt) return VECTOR_OK;
  if (opt->rope) {
    const int rc = make_rope(opt->rope, s->head_dim, rp);
    if (rc) return rc;
    *rope = &rp;
  }
  if (opt->lse) {
    ql.lse = opt->lse;
    ql.stride_head = opt->lse_stride_head;
    *lse = &ql;
  } else if (opt->lse_stride_head != 0) {
    return VECTOR_ERR_ARG;
  }
  return VECTOR_OK;
}

int vector_compress_ex(const vector_shape* s, const vector_compress_options* opt, const void* q_win, const void* k, const void* v,
                       const void* W, int32_t n_pool, int32_t n_approx, float* score, float* eps, uint8_t* tier,
                       int32_t* idx_retain, int32_t* idx_approx, void* k_ret, void* v_ret, void* k_apx, int32_t cap_retain,
                       void* ws, size_t ws_bytes, void* stream) {
  vec::RopeParams rp;
  vec::QueryLse ql;
  const vec::RopeParams* rope;
  const vec::QueryLse* lse;
  const int rc = take_options(s, opt, rp, &rope, ql, &lse);
  if (rc) return rc;
  return compress_impl(s, q_win, k, v, W, n_pool, n_approx, score, eps, tier, idx_retain, idx_approx, k_ret, v_ret, k_apx, cap_retain,
                       ws, ws_bytes, stream, nullptr, lse, rope);
}

int vector_compress_batch_ex(const vector_shape* s, const vector_batch* bt, const vector_compress_options* opt, const void* q_win,
                             const void* k, const void* v, const void* W, float* score, float* eps, uint8_t* tier,
                             int32_t* idx_retain, int32_t* idx_approx, void* k_ret, void* v_ret, void* k_apx, void* ws,
                             size_t ws_bytes, void* stream) {
  vec::RopeParams rp;
  vec::QueryLse ql;
  const vec::RopeParams* rope;
  const vec::QueryLse* lse;
  const int rc = take_options(s, opt, rp, &rope, ql, &lse);
  if (rc) return rc;
  return compress_batch_impl(s, bt, q_win, k, v, W, score, eps, tier, idx_retain, idx_approx, k_ret, v_ret, k_apx, ws, ws_bytes, stream,
                             rope, lse);
}

}  // extern "C"
