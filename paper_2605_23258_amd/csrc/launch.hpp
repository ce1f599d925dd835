// Host-side launch helpers shared by the kernel files.
#pragma once
#include <hip/hip_runtime.h>

#include "../../include/vector.h"

namespace vec {

constexpr size_t kMaxLdsBytes = 160 * 1024;   // LDS per workgroup on gfx950

#define VEC_HIP(expr)                                   \
  do {                                                  \
    hipError_t e_ = (expr);                             \
    if (e_ != hipSuccess) return VECTOR_ERR_HIP;        \
  } while (0)

// Dynamic LDS above the default limit has to be opted into per kernel.
inline hipError_t set_max_lds(const void* func, size_t bytes) {
  if (bytes <= 48 * 1024) return hipSuccess;
  return hipFuncSetAttribute(func, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
}

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// optional per-kernel event timing (timing.hip)
enum KernelId { K_SCORE_STATS = 0, K_STATS_COMBINE, K_MASS_RESIDUAL, K_POOL, K_ROUTE, K_GATHER, K_DECODE_SPLIT,
                K_DECODE_COMBINE, K_COUNT };
bool timing_enabled();
void timing_begin(int id, hipStream_t stream);
void timing_end(int id, hipStream_t stream);

#define VEC_LAUNCH(id, kernel, grid, block, lds, stream, ...)                    \
  do {                                                                           \
    const bool t_ = ::vec::timing_enabled();                                     \
    if (t_) ::vec::timing_begin(id, stream);                                     \
    hipLaunchKernelGGL(kernel, grid, block, lds, stream, __VA_ARGS__);           \
    if (t_) ::vec::timing_end(id, stream);                                       \
  } while (0)

// kernel-file entry points used by the C ABI layer
size_t score_workspace_bytes(const vector_shape& s);
struct RopeParams;
// Several sequences of one shape handled as one problem with batch * Hkv heads (the shape passed
// along says so: n_kv_heads and n_q_heads are the stacked counts).  Head hv of the launch is KV
// head hv % heads_per_seq of sequence hv / heads_per_seq: its keys and values lie
// k_stride_seq / v_stride_seq elements after the previous sequence's (the strides inside a
// sequence stay the shape's), and its W is that KV head's.  Every other array is indexed by hv
// as it is.
struct SeqStack { int heads_per_seq; int64_t k_stride_seq, v_stride_seq; };

// The log-sum-exp of the window queries' attention rows, when the caller already has it (the
// attention kernel of the prefill returns it): natural log, logits scaled by 1 / sqrt(d), causal.
// Row r of query head hq at lse[hq * stride_head + r] (stride_head 0: w).
struct QueryLse { const float* lse; int64_t stride_head; };

int launch_score_residual(const vector_shape& s, const void* q, const void* k, const void* v, const void* W,
                          float* score, float* eps, void* ws, hipStream_t stream, const RopeParams* rope = nullptr,
                          void* route_ws = nullptr, const SeqStack* stack = nullptr, const QueryLse* lse = nullptr);

// A batch of sequences of different lengths through one set of launches.  Every sequence is
// the one-sequence problem it would be alone (its own shape with explicit strides, pointers to
// its own blocks, its own workspace), and gets exactly the parameters that call would compute;
// the parameter blocks go to `tables` (device, ragged_table_bytes(count) bytes) and every
// workgroup picks its sequence's block (launch head hv: sequence hv / Hkv, head hv % Hkv).
constexpr int kMaxRaggedSeqs = 64;
struct RaggedSeq {
  vector_shape shape;
  const void *q, *k, *v;
  float *score, *eps;
  uint8_t* tier;
  int32_t *idx_retain, *idx_approx;
  void *k_ret, *v_ret, *k_apx;
  int n_pool, n_approx, cap_retain;
  void *score_ws, *route_ws;
  int64_t pos_base;          // post-RoPE keys with a position array: where the sequence's positions start in it
  const float* lse;          // the sequence's window rows' log-sum-exp, or null
  int64_t lse_stride_head;
};
struct PoolSeq { const float* mass; float* score; int seq_len, n_prefix; void* route_ws; int n_range; };
size_t ragged_table_bytes(int count);
// whether the G * w query rows of a KV head go through the two passes at once (a ragged launch needs that)
bool score_heads_in_one_group(const vector_shape& s);
size_t route_ragged_table_bytes(int count);
int launch_score_residual_ragged(const vector_shape& s, const RaggedSeq* seqs, int count, const void* W, void* tables,
                                 hipStream_t stream, const RopeParams* rope = nullptr);
int launch_pool_scores_ragged(const PoolSeq* seqs, int count, int n_kv_heads, int pool_kernel, int pool_mode, void* tables,
                              hipStream_t stream);
// tables: the part of the table area after the scorer's (ragged_table_bytes - route_ragged_table_bytes from its start)
int launch_route_compact_ragged(const vector_shape& s, const RaggedSeq* seqs, int count, void* tables, hipStream_t stream);
// host bytes -> device memory in stream order, as kernel arguments of small copy launches (no
// host buffer has to outlive the call, and the copies can be captured into a graph)
int upload_table(const void* host, size_t bytes, void* dev, hipStream_t stream);

int launch_residual_probe(const vector_shape& s, const void* k, const void* v, const void* W, float* eps, int repeat,
                          hipStream_t stream);

size_t calibrate_workspace_bytes(const vector_shape& s);
int launch_calibrate(const vector_shape& s, const void* k, const void* v, void* W, void* ws, hipStream_t stream);

size_t distortion_workspace_bytes(int n_kv_heads, int seq_len);
int launch_distortion(const vector_shape& s, const float* w, const uint8_t* tier, const float* eps, const void* v,
                      double* out, void* ws, hipStream_t stream);

size_t r2_workspace_bytes(int n_kv_heads, int seq_len, int head_dim);
int launch_r2(const vector_shape& s, const float* eps, const void* v, double* out, void* part_ws, hipStream_t stream);

size_t diversity_workspace_bytes(const vector_shape& s);
int launch_key_diversity(const vector_shape& s, const void* k, float* score, void* ws, hipStream_t stream);

constexpr int kRouteMaxSeqLen = 1 << 20;      // per-chunk digit tables carry 16-bit counts: at most 32 chunks of 32768 tokens
size_t route_workspace_bytes(int n_kv_heads, int seq_len, int n_pool);
// Where, inside a routing workspace, the scorer's second pass leaves statistics of the attention
// mass: per head n_range float4 (count, sum, sum of squares of log2 mass), one per workgroup of that
// launch (n_range <= route_mass_range_slots(seq_len)).
void* route_mass_range(void* route_ws, int n_kv_heads);
int route_mass_range_slots(int seq_len);
// average pooling of the attention mass into the score; with a routing workspace (route_ws, sized by
// route_workspace_bytes) also the routing's buckets of score keys (then launch_route is told so and
// skips its own bucket launch)
// n_range: records per head the scorer left at route_mass_range (0: none, the buckets go by the keys' top bits)
int launch_pool_scores(const float* mass, float* score, int n_kv_heads, int seq_len, int n_prefix, int pool_kernel, int pool_mode,
                       void* route_ws, int n_range, hipStream_t stream);
int launch_route(int n_kv_heads, int seq_len, const float* score, const float* eps, int n_pool, int n_approx,
                 uint8_t* tier, int32_t* idx_retain, int32_t* idx_approx, void* ws, bool have_buckets, hipStream_t stream);

int launch_compact(const vector_shape& s, const void* k, const void* v, const int32_t* idx_retain,
                   const int32_t* idx_approx, int n_retain, int n_approx, void* k_ret, void* v_ret, void* k_apx,
                   int cap_retain, hipStream_t stream, const SeqStack* stack = nullptr);

size_t decode_workspace_bytes(int batch, int n_q_heads, int n_kv_heads, int head_dim, int cap_retain, int n_approx);
int launch_decode_attn(const vector_cache& c, const void* q, float scale, void* out, int flags, void* ws,
                       hipStream_t stream, const RopeParams* rope = nullptr, const void* k_new = nullptr,
                       const void* v_new = nullptr);

}  // namespace vec
