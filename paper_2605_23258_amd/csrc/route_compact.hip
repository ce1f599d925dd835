// Three-way routing (Section 3.2, Steps 1 and 3) and compaction into the packed cache.
//
// Both selections of a head (the n_pool highest scores; inside that pool the n_approx lowest
// residuals) are radix selects on order-preserving 32-bit keys with digits of 11, 11 and 10 bits,
// spread over the whole chip and synchronised by kernel boundaries only:
//
//   route_hist_kernel    grid (chunk, head).  Histogram of the leading digit of a chunk's score
//                        keys -> one partial histogram per chunk (16-bit counts, plain stores).
//                        The POOL variant first forms the score itself, the average pooling of the
//                        attention mass (Step 1's base scorer), so the scorer's last kernel already
//                        hands the routing its first histogram.
//   route_pool_kernel    grid (chunk, head).  Every workgroup sums the partial histograms of its
//                        head, picks the leading digit, reads all score keys of the head once,
//                        keeps those with that digit in LDS and finishes the select on them (all
//                        workgroups of a head reach the same threshold).  It then makes the
//                        ordered pass over its own chunk: tiers, the pool list (token index and
//                        residual key, in token order) and the leading-digit histogram of the
//                        chunk's residual keys.
//   route_split_kernel   grid (slice, head).  The same select on the residual keys of the pool
//                        list, then the ordered pass over a slice of the list: ascending
//                        idx_approx / idx_retain, and the approximated tier.
//
// Every slot comes from an ordered prefix sum (ties go to the lower token index); atomics only
// feed LDS histograms and the unordered candidate list of a select, so the result does not depend
// on scheduling.  No workgroup waits for another inside a kernel.
//
// gather_rows_kernel: row gather k_ret / v_ret / k_apx by the index lists.
#include "common.hpp"
#include "launch.hpp"

#ifdef VEC_ROUTE_TRACE
__device__ long long g_route_trace[32];
#define VEC_TRACE(slot) do { if (blockIdx.x == 0 && blockIdx.y == 0 && threadIdx.x == 0) g_route_trace[slot] = wall_clock64(); } while (0)
extern "C" __attribute__((visibility("default"))) int vector_debug_route_trace(long long* host_out) {
  return hipMemcpyFromSymbol(host_out, HIP_SYMBOL(g_route_trace), sizeof(long long) * 32) == hipSuccess ? 0 : -5;
}
#else
#define VEC_TRACE(slot) do { } while (0)
#endif

namespace vec {

namespace {

constexpr int RT = 1024;          // threads per selecting workgroup
constexpr int RW = RT / kWave;    // waves
constexpr int EPT = 4;            // consecutive elements per thread and tile (one 16-byte load)
constexpr int kTile = RT * EPT;   // elements per tile of a selecting workgroup
constexpr int kBatch = 8;         // tiles whose loads are in flight together
constexpr int kBins = 2048;
constexpr int kCandCap = 12288;   // candidates (keys sharing the chosen leading digit) kept in LDS, a 16th per wave
constexpr int HT = 512;           // threads of the histogram kernel
constexpr int kHistTile = HT * EPT;
constexpr int kMinChunk = 2048;   // tokens per chunk: doubled until a head has at most kMaxChunks
constexpr int kMaxChunks = 32;

// Order-preserving map float -> u32 (larger float, larger key); -0 and +0 share a key.
__device__ __forceinline__ uint32_t float_key(float x) {
  uint32_t b = __float_as_uint(x + 0.0f);
  return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}

__device__ __forceinline__ int level_shift(int level) { return level == 0 ? 21 : (level == 1 ? 10 : 0); }
__device__ __forceinline__ uint32_t level_mask(int level) { return level == 2 ? 1023u : 2047u; }

// hist[digit] += 1 for every active lane.  Keys of neighbouring tokens often share their
// leading bits, so a plain LDS atomic would serialise up to 64 lanes on one bin: lanes that
// agree with a leader are counted with one ballot and added by the leader alone; after two
// rounds the stragglers (few, spread over bins) add themselves.
__device__ __forceinline__ void hist_add_aggregated(int* hist, uint32_t digit, bool active, int lane) {
  unsigned long long todo = __ballot(active);
#pragma unroll
  for (int round = 0; round < 2; ++round) {
    if (todo == 0) return;
    const int leader = __ffsll((long long)todo) - 1;
    const uint32_t d = __builtin_amdgcn_readlane(digit, leader);
    const bool match = active && digit == d;
    const unsigned long long m = __ballot(match);
    if (lane == leader) atomicAdd(&hist[d], __popcll(m));
    active = active && !match;
    todo &= ~m;
  }
  if (active) atomicAdd(&hist[digit], 1);
}

// hist[digit] += cnt (cnt in 0..7) for every lane, lanes that agree with a leader merged
// through ballots of the three bits of cnt.
__device__ __forceinline__ void hist_add_weighted(int* hist, uint32_t digit, int cnt, int lane) {
  unsigned long long todo = __ballot(cnt > 0);
#pragma unroll
  for (int round = 0; round < 2; ++round) {
    if (todo == 0) return;
    const int leader = __ffsll((long long)todo) - 1;
    const uint32_t d = __builtin_amdgcn_readlane(digit, leader);
    const bool match = cnt > 0 && digit == d;
    const unsigned long long b0 = __ballot(match && (cnt & 1)), b1 = __ballot(match && (cnt & 2)),
                             b2 = __ballot(match && (cnt & 4));
    if (lane == leader) atomicAdd(&hist[d], __popcll(b0) + 2 * __popcll(b1) + 4 * __popcll(b2));
    if (match) cnt = 0;
    todo &= ~(b0 | b1 | b2);
  }
  if (cnt > 0) atomicAdd(&hist[digit], cnt);
}

// Leading digits of a thread's EPT consecutive keys into an LDS histogram: the keys that agree
// with the thread's first valid one go in together, the others one by one.
__device__ __forceinline__ void hist_add_thread_keys(int* hist, const uint32_t (&key)[EPT], const bool (&ok)[EPT], int lane) {
  uint32_t dg[EPT];
#pragma unroll
  for (int j = 0; j < EPT; ++j) dg[j] = key[j] >> 21;
  int first = -1;
#pragma unroll
  for (int j = EPT - 1; j >= 0; --j)
    if (ok[j]) first = j;
  const uint32_t d0 = first >= 0 ? dg[first] : 0u;
  int cnt = 0;
#pragma unroll
  for (int j = 0; j < EPT; ++j) cnt += ok[j] && dg[j] == d0;
  hist_add_weighted(hist, d0, cnt, lane);
#pragma unroll
  for (int j = 0; j < EPT; ++j)
    if (ok[j] && dg[j] != d0) atomicAdd(&hist[dg[j]], 1);
}

// 16-bit partial histogram of a workgroup: two bins per 32-bit store
template <int NT> __device__ __forceinline__ void store_partial(uint16_t* out, const int* hist) {
  uint32_t* o32 = reinterpret_cast<uint32_t*>(out);
  for (int i = threadIdx.x; i < kBins / 2; i += NT) o32[i] = (uint32_t)hist[2 * i] | ((uint32_t)hist[2 * i + 1] << 16);
}

// ---------------------------------------------------------------------------
// leading-digit histogram of the score keys (and, POOL, the pooled score itself)
// ---------------------------------------------------------------------------
struct HistParams {
  const float* src;       // POOL: attention mass [H, n]; otherwise the scores [H, n]
  float* score;           // POOL: output [H, n]
  uint16_t* part;         // [H, C, kBins] or null (POOL only: pooling without a histogram)
  int n, n_prefix, kernel, chunk_tokens, n_chunks;
};

template <bool POOL>
__global__ __launch_bounds__(HT) void route_hist_kernel(HistParams p) {
  __shared__ int hist[kBins];
  const int h = blockIdx.y, chunk = blockIdx.x;
  const int lane = threadIdx.x & 63;
  const bool do_hist = p.part != nullptr;
  if (do_hist) {
    for (int i = threadIdx.x; i < kBins; i += HT) hist[i] = 0;
    __syncthreads();
  }
  const float* src = p.src + (size_t)h * p.n;
  const int begin = chunk * p.chunk_tokens, end = min(p.n, begin + p.chunk_tokens);
  const bool vec4 = (p.n & 3) == 0 && (reinterpret_cast<uintptr_t>(src) & 15u) == 0 &&
                    (!POOL || (reinterpret_cast<uintptr_t>(p.score) & 15u) == 0);
  for (int tile = begin; tile < end; tile += kHistTile) {        // uniform trip count: whole waves take part
    const int t0 = tile + (int)threadIdx.x * EPT;
    float s[EPT];
    bool ok[EPT];
#pragma unroll
    for (int j = 0; j < EPT; ++j) ok[j] = t0 + j < end;
    if (POOL) {
      const int half = p.kernel / 2;
#pragma unroll
      for (int j = 0; j < EPT; ++j) {
        const int t = t0 + j;
        float out = INFINITY;                                      // window columns
        if (ok[j] && t < p.n_prefix) {
          const int lo = max(0, t - half), hi = min(p.n_prefix - 1, t + half);
          float acc = 0.f;
          for (int i = lo; i <= hi; ++i) acc += src[i];
          out = acc / (float)p.kernel;
        }
        s[j] = out;
      }
      float* dst = p.score + (size_t)h * p.n;
      if (vec4 && ok[EPT - 1]) {
        *reinterpret_cast<float4*>(dst + t0) = make_float4(s[0], s[1], s[2], s[3]);
      } else {
#pragma unroll
        for (int j = 0; j < EPT; ++j)
          if (ok[j]) dst[t0 + j] = s[j];
      }
    } else {
      if (vec4 && ok[EPT - 1]) {
        const float4 x = *reinterpret_cast<const float4*>(src + t0);
        s[0] = x.x; s[1] = x.y; s[2] = x.z; s[3] = x.w;
      } else {
#pragma unroll
        for (int j = 0; j < EPT; ++j) s[j] = ok[j] ? src[t0 + j] : 0.f;
      }
    }
    if (do_hist) {
      uint32_t key[EPT];
#pragma unroll
      for (int j = 0; j < EPT; ++j) key[j] = float_key(s[j]);
      hist_add_thread_keys(hist, key, ok, lane);
    }
  }
  if (do_hist) {
    __syncthreads();
    store_partial<HT>(p.part + ((size_t)h * p.n_chunks + chunk) * kBins, hist);
  }
}

// ---------------------------------------------------------------------------
// prefix sums: inside a wave on the DPP network, across the waves through one LDS row that
// every thread reads whole (no chain of dependent LDS reads)
// ---------------------------------------------------------------------------
template <int CTRL, int ROW_MASK> __device__ __forceinline__ int dpp_take(int v) {   // 0 where no lane feeds this one
  return __builtin_amdgcn_update_dpp(0, v, CTRL, ROW_MASK, 0xf, false);
}
__device__ __forceinline__ int wave_incl_scan_dpp(int v) {
  v += dpp_take<0x111, 0xf>(v);      // row_shr:1 .. 8: inclusive scan inside each row of 16 lanes
  v += dpp_take<0x112, 0xf>(v);
  v += dpp_take<0x114, 0xf>(v);
  v += dpp_take<0x118, 0xf>(v);
  v += dpp_take<0x142, 0xa>(v);      // row_bcast:15 into rows 1 and 3
  v += dpp_take<0x143, 0xc>(v);      // row_bcast:31 into rows 2 and 3
  return v;
}
__device__ __forceinline__ int wave_total_of_scan(int incl) { return __builtin_amdgcn_readlane(incl, 63); }

// RW per-wave values -> their sum over the waves before `wave`, and over all waves
__device__ __forceinline__ void wave_row_sums(const int* row, int wave, int& before, int& total) {
  const int4* r4 = reinterpret_cast<const int4*>(row);
  before = 0;
  total = 0;
#pragma unroll
  for (int q = 0; q < RW / 4; ++q) {
    const int4 v = r4[q];
    const int x[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      total += x[u];
      before += (q * 4 + u < wave) ? x[u] : 0;
    }
  }
}

// ---------------------------------------------------------------------------
// radix select shared by the two selecting kernels
// ---------------------------------------------------------------------------
constexpr int kWaveCand = kCandCap / RW;     // each wave keeps its own candidates: no shared counter

enum { ROW_PICK0 = 0, ROW_PICK1, ROW_PICK2, ROW_GT, ROW_EQ, ROW_EMIT0, ROW_EMIT1, ROW_COUNT };

struct SelectShared {
  int hist[3][kBins];                    // digits of levels 1 and 2 of a select, and one for the caller; zeroed at the start
  __align__(16) int row[ROW_COUNT][RW];  // per-wave terms of the workgroup-wide sums, one row per use
  int pick[3][4];                        // per level: digit, #(digit above it), count of its bin
  int overflow;                          // a wave found more candidates than it can keep
};

__device__ __forceinline__ void select_shared_init(SelectShared& sh) {
  int* h = &sh.hist[0][0];
  for (int i = threadIdx.x; i < 3 * kBins; i += RT) h[i] = 0;
  if (threadIdx.x == 0) sh.overflow = 0;
}

// The digit d with #(digit > d) < remaining <= #(digit >= d), from per-thread counts of bins
// kBins-1-2t (c0) and kBins-2-2t (c1); every thread gets d, #(digit > d) and the count of bin d.
__device__ __forceinline__ void pick_digit(int c0, int c1, int remaining, SelectShared& sh, int level, int& digit, int& above_out,
                                           int& count) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int b_hi = kBins - 1 - 2 * (int)threadIdx.x;
  const int tot = c0 + c1;
  const int incl_w = wave_incl_scan_dpp(tot);
  if (lane == 63) sh.row[ROW_PICK0 + level][wave] = incl_w;
  __syncthreads();
  int before, total;
  wave_row_sums(sh.row[ROW_PICK0 + level], wave, before, total);
  int above = incl_w - tot + before;
  if (above < remaining && remaining <= above + tot) {
    int d = b_hi, cnt = c0;
    if (remaining > above + c0) { above += c0; d = b_hi - 1; cnt = c1; }
    sh.pick[level][0] = d;
    sh.pick[level][1] = above;
    sh.pick[level][2] = cnt;
  }
  __syncthreads();
  digit = sh.pick[level][0];
  above_out = sh.pick[level][1];
  count = sh.pick[level][2];
}

// The k-th largest (1 <= k <= m) of the m keys that load4 delivers four at a time, given the
// leading-digit histogram of those keys as n_parts partial histograms.  Returns the threshold key,
// the number of keys equal to it that belong to the k largest (`quota`, taken in index order by
// the caller), and how many keys at positions below `before` are greater than / equal to the
// threshold.  load4(i0, key, ok): keys of positions i0 .. i0+3 (i0 a multiple of 4), ok = inside.
// cand_key / cand_pos: LDS, kCandCap entries each.  select_shared_init must have run (no barrier
// needed in between: the first pick has two).
// One trip to memory for the histograms and the first kBatch tiles of keys together; after that
// the select runs out of registers and LDS.
template <typename Load4>
__device__ __forceinline__ void select_threshold(Load4 load4, int m, int k, const uint16_t* part, int n_parts, int before,
                                                 SelectShared& sh, uint32_t* cand_key, int32_t* cand_pos, uint32_t& thr,
                                                 int& quota, int& base_gt, int& base_eq, int trace_base = 0) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  (void)trace_base;
  VEC_TRACE(trace_base + 0);
  const int n_tiles = (m + kTile - 1) / kTile;
  // ---- leading digit, from the partial histograms: thread t owns bins 2047-2t and 2046-2t ----
  int c0 = 0, c1 = 0;
  uint32_t cur[kBatch][EPT];
  bool cur_ok[kBatch][EPT];
  auto load_batch = [&](int tb, uint32_t (&key)[kBatch][EPT], bool (&ok)[kBatch][EPT]) {
#pragma unroll
    for (int u = 0; u < kBatch; ++u) {
      if (tb + u < n_tiles) {
        load4((tb + u) * kTile + (int)threadIdx.x * EPT, key[u], ok[u]);
      } else {
#pragma unroll
        for (int j = 0; j < EPT; ++j) { key[u][j] = 0u; ok[u][j] = false; }
      }
    }
  };
  {
    const uint32_t* p32 = reinterpret_cast<const uint32_t*>(part) + (kBins / 2 - 1 - (int)threadIdx.x);
    uint32_t v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) v[u] = p32[(size_t)min(u, n_parts - 1) * (kBins / 2)];
    load_batch(0, cur, cur_ok);                  // in flight together with the histograms
#pragma unroll
    for (int u = 0; u < 8; ++u)
      if (u < n_parts) { c1 += (int)(v[u] & 0xffffu); c0 += (int)(v[u] >> 16); }
    for (int c = 8; c < n_parts; c += 8) {
#pragma unroll
      for (int u = 0; u < 8; ++u) v[u] = p32[(size_t)min(c + u, n_parts - 1) * (kBins / 2)];
#pragma unroll
      for (int u = 0; u < 8; ++u)
        if (c + u < n_parts) { c1 += (int)(v[u] & 0xffffu); c0 += (int)(v[u] >> 16); }
    }
  }
  VEC_TRACE(trace_base + 1);
  int d0, above0, m0;
  pick_digit(c0, c1, k, sh, 0, d0, above0, m0);
  int remaining = k - above0;
  VEC_TRACE(trace_base + 2);

  // ---- all keys once: candidates (leading digit d0) into this wave's list and into the
  //      histogram of the second digit; earlier keys above the digit counted ----
  int gt = 0, n_mine = 0;
  uint32_t* my_key = cand_key + wave * kWaveCand;
  int32_t* my_pos = cand_pos + wave * kWaveCand;
  auto scan_batch = [&](int tb, const uint32_t (&key)[kBatch][EPT], const bool (&ok)[kBatch][EPT]) {
#pragma unroll
    for (int u = 0; u < kBatch; ++u) {
      if (tb + u < n_tiles) {                    // uniform
        const int i0 = (tb + u) * kTile + (int)threadIdx.x * EPT;
#pragma unroll
        for (int j = 0; j < EPT; ++j) {
          const int dg = (int)(key[u][j] >> 21);
          gt += ok[u][j] && i0 + j < before && dg > d0;
          const bool is_c = ok[u][j] && dg == d0;
          const unsigned long long b = __ballot(is_c);
          if (b) {
            if (is_c) {
              const int pos = n_mine + __popcll(b & ((1ull << lane) - 1ull));
              if (pos < kWaveCand) { my_key[pos] = key[u][j]; my_pos[pos] = i0 + j; }
              atomicAdd(&sh.hist[0][(key[u][j] >> 10) & 2047u], 1);
            }
            n_mine += __popcll(b);
          }
        }
      }
    }
  };
  for (int tb = 0; tb < n_tiles; tb += kBatch) {
    uint32_t nxt[kBatch][EPT];
    bool nxt_ok[kBatch][EPT];
    const bool more = tb + kBatch < n_tiles;
    if (more) load_batch(tb + kBatch, nxt, nxt_ok);      // requested before this batch is worked on
    scan_batch(tb, cur, cur_ok);
    if (more) {
#pragma unroll
      for (int u = 0; u < kBatch; ++u)
#pragma unroll
        for (int j = 0; j < EPT; ++j) { cur[u][j] = nxt[u][j]; cur_ok[u][j] = nxt_ok[u][j]; }
    }
  }
  if (n_mine > kWaveCand && lane == 0) sh.overflow = 1;
  __syncthreads();
  VEC_TRACE(trace_base + 3);
  const bool use_list = sh.overflow == 0;
  const int n_list = min(n_mine, kWaveCand);

  // visit every key whose leading digit is d0 (each wave its own): f(key, position)
  auto for_each_candidate = [&](auto f) {
    if (use_list) {
      for (int i = lane; i < n_list; i += kWave) f(my_key[i], my_pos[i]);
    } else {
      for (int t = 0; t < n_tiles; ++t) {
        uint32_t key[EPT];
        bool ok[EPT];
        const int i0 = t * kTile + (int)threadIdx.x * EPT;
        load4(i0, key, ok);
#pragma unroll
        for (int j = 0; j < EPT; ++j)
          if (ok[j] && (int)(key[j] >> 21) == d0) f(key[j], i0 + j);
      }
    }
  };

  // ---- second digit: its histogram was filled during the scan ----
  const int b_hi = kBins - 1 - 2 * (int)threadIdx.x;
  int d1, above1, m1;
  pick_digit(sh.hist[0][b_hi], sh.hist[0][b_hi - 1], remaining, sh, 1, d1, above1, m1);
  remaining -= above1;
  const uint32_t prefix22 = (((uint32_t)d0) << 21) | (((uint32_t)d1) << 10);
  // ---- third digit ----
  for_each_candidate([&](uint32_t key, int) {
    if ((key >> 10) == (prefix22 >> 10)) atomicAdd(&sh.hist[1][key & 1023u], 1);
  });
  __syncthreads();
  int d2, above2, m2;
  pick_digit(sh.hist[1][b_hi], sh.hist[1][b_hi - 1], remaining, sh, 2, d2, above2, m2);
  remaining -= above2;
  thr = prefix22 | (uint32_t)d2;
  quota = remaining;
  VEC_TRACE(trace_base + 4);

  // ---- keys before `before`: above the threshold, equal to it ----
  int eq = 0;
  const uint32_t t_key = thr;
  for_each_candidate([&](uint32_t key, int pos) {
    if (pos < before) { gt += key > t_key; eq += key == t_key; }
  });
  gt = wave_total_of_scan(wave_incl_scan_dpp(gt));
  eq = wave_total_of_scan(wave_incl_scan_dpp(eq));
  if (lane == 0) { sh.row[ROW_GT][wave] = gt; sh.row[ROW_EQ][wave] = eq; }
  __syncthreads();
  int unused;
  wave_row_sums(sh.row[ROW_GT], RW, unused, base_gt);
  wave_row_sums(sh.row[ROW_EQ], RW, unused, base_eq);
  VEC_TRACE(trace_base + 5);
}

// Ordered pass over positions [begin, end) in tiles of kTile: a thread's EPT consecutive
// elements are classified by load_cls (2: above the threshold, 1: equal, 0: below or outside);
// emit(position, selected, rank among the selected) is called for every element inside.
// Equal elements are selected while fewer than `quota` earlier ones exist.  The two running
// counts of a thread travel through one scan packed as (greater << 16) | equal.
template <typename ClsFn, typename EmitFn>
__device__ __forceinline__ void ordered_emit(ClsFn load_cls, EmitFn emit, int begin, int end, int base_gt, int base_eq, int quota,
                                             SelectShared& sh) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  int carry_gt = base_gt, carry_eq = base_eq, buf = 0;
  for (int tile = begin; tile < end; tile += kTile) {
    const int i0 = tile + (int)threadIdx.x * EPT;
    int cls[EPT];
    load_cls(i0, cls);
    int packed = 0;
#pragma unroll
    for (int j = 0; j < EPT; ++j) packed += (cls[j] == 2 ? 0x10000 : 0) + (cls[j] == 1 ? 1 : 0);
    const int incl = wave_incl_scan_dpp(packed);
    if (lane == 63) sh.row[ROW_EMIT0 + buf][wave] = incl;
    __syncthreads();
    int pre, tile_tot;
    wave_row_sums(sh.row[ROW_EMIT0 + buf], wave, pre, tile_tot);
    pre += incl - packed;
    int pre_gt = carry_gt + (pre >> 16), pre_eq = carry_eq + (pre & 0xffff);
    carry_gt += tile_tot >> 16;
    carry_eq += tile_tot & 0xffff;
#pragma unroll
    for (int j = 0; j < EPT; ++j) {
      if (i0 + j < end) {
        const bool sel = cls[j] == 2 || (cls[j] == 1 && pre_eq < quota);
        emit(i0 + j, sel, pre_gt + min(pre_eq, quota));
        pre_gt += cls[j] == 2;
        pre_eq += cls[j] == 1;
      }
    }
    buf ^= 1;
  }
}

struct RouteParams {
  const float* score; const float* eps;
  int n, n_pool, n_approx, n_heads;
  int chunk_tokens, n_chunks;      // selection by score: tokens per workgroup
  int slice, n_slices;             // selection by residual: pool entries per workgroup
  int pool_stride;                 // entries between the pool lists of two heads (a multiple of 4)
  const uint16_t* part0;           // [H, C, kBins] leading digits of the score keys
  uint16_t* part1;                 // [H, C, kBins] leading digits of the residual keys of pool members
  uint8_t* tier; int32_t* idx_retain; int32_t* idx_approx;
  int32_t* pool_idx; uint32_t* pool_key;
};

// Step 1: the pool is the n_pool tokens of highest score
__global__ __launch_bounds__(RT) void route_pool_kernel(RouteParams p) {
  __shared__ SelectShared sh;
  extern __shared__ __align__(16) unsigned char dyn_lds[];
  uint32_t* cand_key = reinterpret_cast<uint32_t*>(dyn_lds);
  int32_t* cand_pos = reinterpret_cast<int32_t*>(dyn_lds) + kCandCap;
  const int h = blockIdx.y, chunk = blockIdx.x;
  const float* sc = p.score + (size_t)h * p.n;
  const float* ep = p.eps + (size_t)h * p.n;
  const int n = p.n;
  select_shared_init(sh);
  const bool vec4 = (n & 3) == 0 && ((reinterpret_cast<uintptr_t>(sc) | reinterpret_cast<uintptr_t>(ep)) & 15u) == 0;
  auto load_f4 = [&](const float* a, int i0, float (&x)[EPT]) {
    if (vec4 && i0 + EPT <= n) {
      const float4 v = *reinterpret_cast<const float4*>(a + i0);
      x[0] = v.x; x[1] = v.y; x[2] = v.z; x[3] = v.w;
    } else {
#pragma unroll
      for (int j = 0; j < EPT; ++j) x[j] = i0 + j < n ? a[i0 + j] : 0.f;
    }
  };
  auto load4 = [&](int i0, uint32_t (&key)[EPT], bool (&ok)[EPT]) {
    float x[EPT];
    load_f4(sc, i0, x);
#pragma unroll
    for (int j = 0; j < EPT; ++j) { ok[j] = i0 + j < n; key[j] = ok[j] ? float_key(x[j]) : 0u; }
  };
  const int begin = chunk * p.chunk_tokens, end = min(n, begin + p.chunk_tokens);
  // this thread's tokens of the chunk's first tile: requested now, used by the ordered pass
  const int first_i0 = begin + (int)threadIdx.x * EPT;
  float sc0[EPT], ep0[EPT];
  load_f4(sc, first_i0, sc0);
  load_f4(ep, first_i0, ep0);
  uint32_t thr;
  int quota, base_gt, base_eq;
  select_threshold(load4, n, p.n_pool, p.part0 + (size_t)h * p.n_chunks * kBins, p.n_chunks, begin, sh, cand_key, cand_pos, thr,
                   quota, base_gt, base_eq, 0);

  // ordered pass over the chunk: tiers, pool list, leading digits of the residual keys
  uint8_t* tr = p.tier + (size_t)h * n;
  int32_t* pidx = p.pool_idx + (size_t)h * p.pool_stride;
  uint32_t* pkey = p.pool_key + (size_t)h * p.pool_stride;
  uint32_t ekey[EPT];
  ordered_emit(
      [&](int i0, int (&cls)[EPT]) {
        float x[EPT], e[EPT];
        if (i0 == first_i0) {
#pragma unroll
          for (int j = 0; j < EPT; ++j) { x[j] = sc0[j]; e[j] = ep0[j]; }
        } else {
          load_f4(sc, i0, x);
          load_f4(ep, i0, e);
        }
#pragma unroll
        for (int j = 0; j < EPT; ++j) {
          const uint32_t key = float_key(x[j]);
          cls[j] = i0 + j < end ? (key > thr ? 2 : (key == thr ? 1 : 0)) : 0;
          ekey[j] = ~float_key(e[j]);               // smaller residual, larger key
        }
      },
      [&](int i, bool sel, int rank) {
        tr[i] = sel ? VECTOR_TIER_RETAIN : VECTOR_TIER_EVICT;
        if (sel && rank < p.n_pool) {                // rank < n_pool by construction; never write past the list
          const uint32_t ek = ekey[i & (EPT - 1)];   // tiles start at multiples of EPT
          pidx[rank] = i;
          pkey[rank] = ek;
          atomicAdd(&sh.hist[2][ek >> 21], 1);
        }
      },
      begin, end, base_gt, base_eq, quota, sh);
  VEC_TRACE(6);
  __syncthreads();
  store_partial<RT>(p.part1 + ((size_t)h * p.n_chunks + chunk) * kBins, sh.hist[2]);
  VEC_TRACE(7);
}

// Step 3: inside the pool, the n_approx tokens of lowest residual lose their value
__global__ __launch_bounds__(RT) void route_split_kernel(RouteParams p) {
  __shared__ SelectShared sh;
  extern __shared__ __align__(16) unsigned char dyn_lds[];
  uint32_t* cand_key = reinterpret_cast<uint32_t*>(dyn_lds);
  int32_t* cand_pos = reinterpret_cast<int32_t*>(dyn_lds) + kCandCap;
  const int h = blockIdx.y, slice = blockIdx.x;
  const int m = p.n_pool;
  const int32_t* pidx = p.pool_idx + (size_t)h * p.pool_stride;
  const uint32_t* pkey = p.pool_key + (size_t)h * p.pool_stride;
  uint8_t* tr = p.tier + (size_t)h * p.n;
  int32_t* ir = p.idx_retain + (size_t)h * (p.n_pool - p.n_approx);
  int32_t* ia = p.idx_approx + (size_t)h * p.n_approx;
  const int begin = slice * p.slice, end = min(m, begin + p.slice);
  if (p.n_approx == 0) {
    for (int i = begin + (int)threadIdx.x; i < end; i += RT) ir[i] = pidx[i];
    return;
  }
  select_shared_init(sh);
  auto load_u4 = [&](const uint32_t* a, int i0, uint32_t (&x)[EPT]) {
    if (i0 + EPT <= m) {                             // lists start at 16-byte boundaries
      const uint4 v = *reinterpret_cast<const uint4*>(a + i0);
      x[0] = v.x; x[1] = v.y; x[2] = v.z; x[3] = v.w;
    } else {
#pragma unroll
      for (int j = 0; j < EPT; ++j) x[j] = i0 + j < m ? a[i0 + j] : 0u;
    }
  };
  auto load4 = [&](int i0, uint32_t (&key)[EPT], bool (&ok)[EPT]) {
    load_u4(pkey, i0, key);
#pragma unroll
    for (int j = 0; j < EPT; ++j) ok[j] = i0 + j < m;
  };
  // this thread's entries of the slice's first tile: requested now, used by the ordered pass
  const int first_i0 = begin + (int)threadIdx.x * EPT;
  uint32_t key0[EPT], tok0[EPT];
  load_u4(pkey, first_i0, key0);
  load_u4(reinterpret_cast<const uint32_t*>(pidx), first_i0, tok0);
  uint32_t thr;
  int quota, base_gt, base_eq;
  select_threshold(load4, m, p.n_approx, p.part1 + (size_t)h * p.n_chunks * kBins, p.n_chunks, begin, sh, cand_key, cand_pos, thr,
                   quota, base_gt, base_eq, 16);
  uint32_t tok[EPT];
  ordered_emit(
      [&](int i0, int (&cls)[EPT]) {
        uint32_t key[EPT];
        if (i0 == first_i0) {
#pragma unroll
          for (int j = 0; j < EPT; ++j) { key[j] = key0[j]; tok[j] = tok0[j]; }
        } else {
          load_u4(pkey, i0, key);
          load_u4(reinterpret_cast<const uint32_t*>(pidx), i0, tok);
        }
#pragma unroll
        for (int j = 0; j < EPT; ++j) cls[j] = i0 + j < end ? (key[j] > thr ? 2 : (key[j] == thr ? 1 : 0)) : 0;
      },
      [&](int i, bool sel, int rank) {
        const int t = (int)tok[i & (EPT - 1)];
        if (sel) {
          if (rank < p.n_approx) {
            ia[rank] = t;
            tr[min(max(t, 0), p.n - 1)] = VECTOR_TIER_APPROX;
          }
        } else if (i - rank < p.n_pool - p.n_approx) {
          ir[i - rank] = t;
        }
      },
      begin, end, base_gt, base_eq, quota, sh);
  VEC_TRACE(16 + 6);
}

// nothing is kept: every token is evicted
__global__ __launch_bounds__(256) void route_evict_all_kernel(uint8_t* __restrict__ tier, size_t total) {
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < total) tier[i] = VECTOR_TIER_EVICT;
}

// ---------------------------------------------------------------------------
// compaction: one 16-byte piece per thread, P pieces per row
// ---------------------------------------------------------------------------
struct GatherParams {
  const unsigned char* k; const unsigned char* v;
  int64_t k_sh, k_st, v_sh, v_st;          // byte strides
  const int32_t* idx_retain; const int32_t* idx_approx;
  int n_retain, n_approx, cap_retain, row_bytes, n;
  unsigned char* k_ret; unsigned char* v_ret; unsigned char* k_apx;
};

__global__ __launch_bounds__(256) void gather_rows_kernel(GatherParams p) {
  const int h = blockIdx.y, seg = blockIdx.z;       // seg 0: k_ret, 1: v_ret, 2: k_apx
  const int pieces = p.row_bytes / 16;
  const int rows = (seg == 2) ? p.n_approx : p.n_retain;
  const int64_t gid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int row = (int)(gid / pieces), piece = (int)(gid - (int64_t)row * pieces);
  if (row >= rows) return;
  const int32_t* idx = (seg == 2) ? p.idx_approx + (size_t)h * p.n_approx : p.idx_retain + (size_t)h * p.n_retain;
  int tok = idx[row];
  tok = min(max(tok, 0), p.n - 1);                  // an index list is trusted, but never walk out of the tensor
  const unsigned char* src = (seg == 1) ? p.v + h * p.v_sh + (int64_t)tok * p.v_st : p.k + h * p.k_sh + (int64_t)tok * p.k_st;
  unsigned char* dst = (seg == 0) ? p.k_ret + ((size_t)h * p.cap_retain + row) * p.row_bytes
                     : (seg == 1) ? p.v_ret + ((size_t)h * p.cap_retain + row) * p.row_bytes
                                  : p.k_apx + ((size_t)h * p.n_approx + row) * p.row_bytes;
  *reinterpret_cast<uint4*>(dst + piece * 16) = *reinterpret_cast<const uint4*>(src + piece * 16);
}

}  // namespace

// ---------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------
int route_chunk_tokens(int seq_len) {
  int ch = kMinChunk;
  while ((seq_len + ch - 1) / ch > kMaxChunks) ch *= 2;
  return ch;
}

namespace {
struct RouteLayout {
  int chunk_tokens, n_chunks, pool_stride;
  size_t off_idx, off_key, off_part0, off_part1, total;
};
RouteLayout route_layout(int n_kv_heads, int seq_len, int n_pool) {
  RouteLayout L;
  L.chunk_tokens = route_chunk_tokens(seq_len);
  L.n_chunks = (seq_len + L.chunk_tokens - 1) / L.chunk_tokens;
  L.pool_stride = (n_pool + 3) / 4 * 4;
  size_t off = 0;
  L.off_part0 = off; off += align_up((size_t)n_kv_heads * L.n_chunks * kBins * sizeof(uint16_t), 256);
  L.off_part1 = off; off += align_up((size_t)n_kv_heads * L.n_chunks * kBins * sizeof(uint16_t), 256);
  L.off_idx = off;   off += align_up((size_t)n_kv_heads * L.pool_stride * sizeof(int32_t), 256);
  L.off_key = off;   off += align_up((size_t)n_kv_heads * L.pool_stride * sizeof(uint32_t), 256);
  L.total = off;
  return L;
}
}  // namespace

size_t route_workspace_bytes(int n_kv_heads, int seq_len, int n_pool) { return route_layout(n_kv_heads, seq_len, n_pool).total; }

uint16_t* route_score_hist(void* route_ws) { return reinterpret_cast<uint16_t*>(route_ws); }   // off_part0 == 0

int launch_pool_scores(const float* mass, float* score, int n_kv_heads, int seq_len, int n_prefix, int pool_kernel,
                       uint16_t* score_hist, hipStream_t stream) {
  HistParams hp;
  hp.src = mass; hp.score = score; hp.part = score_hist; hp.n = seq_len; hp.n_prefix = n_prefix; hp.kernel = pool_kernel;
  hp.chunk_tokens = route_chunk_tokens(seq_len);
  hp.n_chunks = (seq_len + hp.chunk_tokens - 1) / hp.chunk_tokens;
  VEC_LAUNCH(K_POOL, route_hist_kernel<true>, dim3(hp.n_chunks, n_kv_heads), dim3(HT), 0, stream, hp);
  VEC_HIP(hipGetLastError());
  return VECTOR_OK;
}

int launch_route(int n_kv_heads, int seq_len, const float* score, const float* eps, int n_pool, int n_approx,
                 uint8_t* tier, int32_t* idx_retain, int32_t* idx_approx, void* ws, bool have_score_hist, hipStream_t stream) {
  if (n_pool == 0) {
    const size_t total = (size_t)n_kv_heads * seq_len;
    VEC_LAUNCH(K_ROUTE, route_evict_all_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, stream, tier, total);
    VEC_HIP(hipGetLastError());
    return VECTOR_OK;
  }
  const RouteLayout L = route_layout(n_kv_heads, seq_len, n_pool);
  unsigned char* w8 = reinterpret_cast<unsigned char*>(ws);
  RouteParams p;
  p.score = score; p.eps = eps; p.n = seq_len; p.n_pool = n_pool; p.n_approx = n_approx; p.n_heads = n_kv_heads;
  p.chunk_tokens = L.chunk_tokens; p.n_chunks = L.n_chunks; p.pool_stride = L.pool_stride;
  p.slice = kTile;
  while ((n_pool + p.slice - 1) / p.slice > kMaxChunks) p.slice *= 2;
  p.n_slices = (n_pool + p.slice - 1) / p.slice;
  uint16_t* part0 = reinterpret_cast<uint16_t*>(w8 + L.off_part0);
  p.part0 = part0;
  p.part1 = reinterpret_cast<uint16_t*>(w8 + L.off_part1);
  p.pool_idx = reinterpret_cast<int32_t*>(w8 + L.off_idx);
  p.pool_key = reinterpret_cast<uint32_t*>(w8 + L.off_key);
  p.tier = tier; p.idx_retain = idx_retain; p.idx_approx = idx_approx;
  const size_t lds = (size_t)kCandCap * 8;
  VEC_HIP(set_max_lds(reinterpret_cast<const void*>(route_pool_kernel), lds));
  VEC_HIP(set_max_lds(reinterpret_cast<const void*>(route_split_kernel), lds));
  const bool t_ = timing_enabled();
  if (t_) timing_begin(K_ROUTE, stream);             // the launches count as one routing step
  if (!have_score_hist) {
    HistParams hp;
    hp.src = score; hp.score = nullptr; hp.part = part0; hp.n = seq_len; hp.n_prefix = seq_len; hp.kernel = 1;
    hp.chunk_tokens = L.chunk_tokens; hp.n_chunks = L.n_chunks;
    hipLaunchKernelGGL(route_hist_kernel<false>, dim3(L.n_chunks, n_kv_heads), dim3(HT), 0, stream, hp);
  }
  hipLaunchKernelGGL(route_pool_kernel, dim3(L.n_chunks, n_kv_heads), dim3(RT), lds, stream, p);
  hipLaunchKernelGGL(route_split_kernel, dim3(p.n_slices, n_kv_heads), dim3(RT), lds, stream, p);
  if (t_) timing_end(K_ROUTE, stream);
  VEC_HIP(hipGetLastError());
  return VECTOR_OK;
}

int launch_compact(const vector_shape& s, const void* k, const void* v, const int32_t* idx_retain,
                   const int32_t* idx_approx, int n_retain, int n_approx, void* k_ret, void* v_ret, void* k_apx,
                   int cap_retain, hipStream_t stream) {
  const int esz = (s.dtype == VECTOR_BF16) ? 2 : 4;
  GatherParams p;
  p.k = reinterpret_cast<const unsigned char*>(k);
  p.v = reinterpret_cast<const unsigned char*>(v);
  const int64_t k_st = s.k_stride_tok ? s.k_stride_tok : s.head_dim;
  const int64_t v_st = s.v_stride_tok ? s.v_stride_tok : s.head_dim;
  p.k_st = k_st * esz;
  p.v_st = v_st * esz;
  p.k_sh = (s.k_stride_head ? s.k_stride_head : (int64_t)s.seq_len * k_st) * esz;
  p.v_sh = (s.v_stride_head ? s.v_stride_head : (int64_t)s.seq_len * v_st) * esz;
  p.idx_retain = idx_retain; p.idx_approx = idx_approx;
  p.n_retain = n_retain; p.n_approx = n_approx; p.cap_retain = cap_retain;
  p.row_bytes = s.head_dim * esz; p.n = s.seq_len;
  p.k_ret = reinterpret_cast<unsigned char*>(k_ret);
  p.v_ret = reinterpret_cast<unsigned char*>(v_ret);
  p.k_apx = reinterpret_cast<unsigned char*>(k_apx);
  const int pieces = p.row_bytes / 16;
  const int max_rows = n_retain > n_approx ? n_retain : n_approx;
  if (max_rows == 0) return VECTOR_OK;
  const int64_t threads = (int64_t)max_rows * pieces;
  dim3 grid((unsigned)((threads + 255) / 256), s.n_kv_heads, 3);
  VEC_LAUNCH(K_GATHER, gather_rows_kernel, grid, dim3(256), 0, stream, p);
  VEC_HIP(hipGetLastError());
  return VECTOR_OK;
}

}  // namespace vec
