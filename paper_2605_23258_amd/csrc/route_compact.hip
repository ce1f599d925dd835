// Three-way routing (Section 3.2, Steps 1 and 3) and compaction into the packed cache.
//
// route_kernel: one workgroup per KV head.
//   1. radix select (11+11+10-bit digits, LDS histograms) of the n_pool-th largest
//      score key -> threshold key and the number of threshold ties to take;
//   2. ordered prefix-sum pass over the tokens: pool membership with ties taken in
//      ascending token index, pool list (token index, residual key) in token order;
//   3. radix select of the n_approx-th smallest residual inside the pool;
//   4. ordered pass over the pool list: ascending idx_approx / idx_retain, tiers.
// Slot assignment comes from ordered scans only; atomics are used for histograms
// alone, so the result does not depend on scheduling.
// Up to RT*KC tokens per head route_cached_kernel does the same out of registers; beyond
// that the selection by score is spread over the chip (route_wide_* kernels below).
//
// gather_rows_kernel: row gather k_ret / v_ret / k_apx by the index lists.
#include "common.hpp"
#include "launch.hpp"

namespace vec {

namespace {

constexpr int RT = 1024;          // threads per routing workgroup
constexpr int RW = RT / kWave;    // waves
constexpr int EPT = 4;            // consecutive elements per thread in the ordered passes
constexpr int KC = 32;            // keys a thread can keep in registers across the radix passes
constexpr int KB = 8;             // otherwise: keys loaded together so that their latencies overlap

// Order-preserving map float -> u32 (larger float, larger key); -0 and +0 share a key.
__device__ __forceinline__ uint32_t float_key(float x) {
  uint32_t b = __float_as_uint(x + 0.0f);
  return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}

constexpr int kBins = 2048;

struct RouteShared {
  int hist[kBins];
  int wave_sum[RW];
  int wave_tot[2][RW];
  uint32_t tile_wave[(KC / EPT) * RW];   // register-cached ordered pass: totals, then exclusive prefixes, by (tile, wave)
  int digit, above;
};

// hist[digit] += 1 for every active lane, for the leading digit.  Importance scores of
// neighbouring tokens share their leading bits, so a plain LDS atomic would serialise up to
// 64 lanes on one bin: lanes that agree with a leader are counted with one ballot and added
// by the leader alone; after two rounds the stragglers (few, spread over bins) add themselves.
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

// k-th largest key among keyf(0..m-1), 1 <= k <= m.  Returns the key value and how many
// elements equal to it belong to the k largest.  Three passes of LDS histograms.
template <typename KeyFn>
__device__ void radix_select_desc(KeyFn keyf, int m, int k, RouteShared& sh, uint32_t& thr, int& quota) {
  uint32_t prefix = 0, mask = 0;
  int remaining = k;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const bool cached = m <= RT * KC;                 // keys stay in registers across the passes
  uint32_t kreg[KC];
  if (cached) {
#pragma unroll
    for (int j = 0; j < KC; ++j) {
      const int i = j * RT + threadIdx.x;
      kreg[j] = (i < m) ? keyf(i) : 0u;
    }
  }
  int shift = 32;
#pragma unroll 1
  for (int pass = 0; pass < 3; ++pass) {
    const int bits = pass == 2 ? 10 : 11;           // digits of 11, 11 and 10 bits, most significant first
    const uint32_t dmask = (1u << bits) - 1u;
    shift -= bits;
    for (int i = threadIdx.x; i < kBins; i += RT) sh.hist[i] = 0;
    __syncthreads();
    auto add = [&](uint32_t key, bool in) {
      const uint32_t digit = (key >> shift) & dmask;
      const bool active = in && (key & mask) == prefix;
      if (pass == 0) hist_add_aggregated(sh.hist, digit, active, lane);
      else if (active) atomicAdd(&sh.hist[digit], 1);      // later digits are spread: few conflicts
    };
    if (cached) {
#pragma unroll
      for (int j = 0; j < KC; ++j)
        if (j * RT < m) add(kreg[j], j * RT + threadIdx.x < m);        // uniform guard: whole waves take part
    } else {
      for (int base = 0; base < m; base += RT * KB) {
        uint32_t key[KB];
#pragma unroll
        for (int j = 0; j < KB; ++j) {
          const int i = base + j * RT + threadIdx.x;
          key[j] = (i < m) ? keyf(i) : 0u;
        }
#pragma unroll
        for (int j = 0; j < KB; ++j) add(key[j], base + j * RT + threadIdx.x < m);
      }
    }
    __syncthreads();
    // Thread t owns bins 2047-2t and 2046-2t, so thread order walks the digits downwards.
    // Find the digit d with  #(digit > d) < remaining <= #(digit >= d).
    const int b_hi = kBins - 1 - 2 * threadIdx.x;
    const int c0 = sh.hist[b_hi], c1 = sh.hist[b_hi - 1];
    const int tot = c0 + c1;
    const int incl_w = wave_incl_scan_i(tot, lane);
    if (lane == 63) sh.wave_sum[wave] = incl_w;
    __syncthreads();
    int above = incl_w - tot;
    for (int wv = 0; wv < wave; ++wv) above += sh.wave_sum[wv];
    if (above < remaining && remaining <= above + tot) {
      int d = b_hi;
      if (remaining > above + c0) { above += c0; d = b_hi - 1; }
      sh.digit = d;
      sh.above = above;
    }
    __syncthreads();
    prefix |= ((uint32_t)sh.digit) << shift;
    mask |= dmask << shift;
    remaining -= sh.above;
  }
  thr = prefix;
  quota = remaining;
  __syncthreads();      // sh.digit / sh.above may be rewritten by the next select
}

// Ordered pass over m elements in index order.  classify(i) returns 2 for "strictly
// selected", 1 for "threshold tie", 0 otherwise; emit(i, selected, rank_selected) is
// called for every element with its rank among the selected ones.  Ties are selected
// while fewer than `quota` earlier ties exist.  One tile is RT*EPT elements; the two
// counts of a thread (each <= EPT) travel through one scan packed as (gt << 16) | eq.
template <typename ClassFn, typename EmitFn>
__device__ void ordered_select(ClassFn classify, EmitFn emit, int m, int quota, RouteShared& sh) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  int carry_gt = 0, carry_eq = 0, buf = 0;
  int cls[EPT], next_cls[EPT];
#pragma unroll
  for (int j = 0; j < EPT; ++j) {
    const int i = threadIdx.x * EPT + j;
    cls[j] = (i < m) ? classify(i) : 0;
  }
  for (int base = 0; base < m; base += RT * EPT) {
    const int i0 = base + threadIdx.x * EPT;
    // the next tile's keys are requested before this tile's scan and barrier
#pragma unroll
    for (int j = 0; j < EPT; ++j) {
      const int i = i0 + RT * EPT + j;
      next_cls[j] = (i < m) ? classify(i) : 0;
    }
    int packed = 0;
#pragma unroll
    for (int j = 0; j < EPT; ++j) packed += (cls[j] == 2 ? 0x10000 : 0) + (cls[j] == 1 ? 1 : 0);
    const int incl = wave_incl_scan_i(packed, lane);
    if (lane == 63) sh.wave_tot[buf][wave] = incl;
    __syncthreads();
    int pre = incl - packed, tile_tot = 0;
    for (int wv = 0; wv < RW; ++wv) {
      const int t = sh.wave_tot[buf][wv];
      if (wv < wave) pre += t;
      tile_tot += t;
    }
    int pre_gt = carry_gt + (pre >> 16), pre_eq = carry_eq + (pre & 0xffff);
    carry_gt += tile_tot >> 16;
    carry_eq += tile_tot & 0xffff;
#pragma unroll
    for (int j = 0; j < EPT; ++j) {
      if (i0 + j < m) {
        const bool sel = cls[j] == 2 || (cls[j] == 1 && pre_eq < quota);
        emit(i0 + j, sel, pre_gt + min(pre_eq, quota));
        pre_gt += cls[j] == 2;
        pre_eq += cls[j] == 1;
      }
    }
#pragma unroll
    for (int j = 0; j < EPT; ++j) cls[j] = next_cls[j];
    buf ^= 1;
  }
}

__global__ __launch_bounds__(RT) void route_kernel(const float* __restrict__ score, const float* __restrict__ eps,
                                                   int n, int n_pool, int n_approx, uint8_t* __restrict__ tier,
                                                   int32_t* __restrict__ idx_retain, int32_t* __restrict__ idx_approx,
                                                   int32_t* __restrict__ pool_idx, uint32_t* __restrict__ pool_key) {
  __shared__ RouteShared sh;
  const int h = blockIdx.x;
  const float* sc = score + (size_t)h * n;
  const float* ep = eps + (size_t)h * n;
  uint8_t* tr = tier + (size_t)h * n;
  int32_t* pidx = pool_idx + (size_t)h * n_pool;
  uint32_t* pkey = pool_key + (size_t)h * n_pool;
  int32_t* ir = idx_retain + (size_t)h * (n_pool - n_approx);
  int32_t* ia = idx_approx + (size_t)h * n_approx;

  if (n_pool == 0) {
    for (int i = threadIdx.x; i < n; i += RT) tr[i] = VECTOR_TIER_EVICT;
    return;
  }

  // Step 1: the pool is the n_pool tokens of highest score
  uint32_t thr;
  int quota;
  radix_select_desc([&](int i) { return float_key(sc[i]); }, n, n_pool, sh, thr, quota);

  ordered_select(
      [&](int i) { uint32_t key = float_key(sc[i]); return key > thr ? 2 : (key == thr ? 1 : 0); },
      [&](int i, bool sel, int rank) {
        tr[i] = sel ? VECTOR_TIER_RETAIN : VECTOR_TIER_EVICT;
        if (sel && rank < n_pool) pidx[rank] = i;     // rank < n_pool by construction; never write past the list
      },
      n, quota, sh);
  __threadfence();
  __syncthreads();

  // Step 3: inside the pool, the n_approx tokens of lowest residual lose their value
  if (n_approx == 0) {
    for (int i = threadIdx.x; i < n_pool; i += RT) ir[i] = pidx[i];
    return;
  }
  // residual keys of the pool members, gathered in batches; smaller residual, larger key
  for (int base = 0; base < n_pool; base += RT * KB) {
    int tok[KB];
#pragma unroll
    for (int j = 0; j < KB; ++j) {
      const int i = base + j * RT + threadIdx.x;
      tok[j] = (i < n_pool) ? pidx[i] : 0;
    }
    float e[KB];
#pragma unroll
    for (int j = 0; j < KB; ++j) e[j] = ep[min(max(tok[j], 0), n - 1)];
#pragma unroll
    for (int j = 0; j < KB; ++j) {
      const int i = base + j * RT + threadIdx.x;
      if (i < n_pool) pkey[i] = ~float_key(e[j]);
    }
  }
  __threadfence();
  __syncthreads();
  radix_select_desc([&](int i) { return pkey[i]; }, n_pool, n_approx, sh, thr, quota);
  ordered_select(
      [&](int i) { uint32_t key = pkey[i]; return key > thr ? 2 : (key == thr ? 1 : 0); },
      [&](int i, bool sel, int rank) {
        const int tok = pidx[i];
        if (sel) {
          if (rank < n_approx) {
            ia[rank] = tok;
            tr[tok] = VECTOR_TIER_APPROX;
          }
        } else if (i - rank < n_pool - n_approx) {
          ir[i - rank] = tok;
        }
      },
      n_pool, quota, sh);
}

// ---------------------------------------------------------------------------
// Routing with every key held in registers (seq_len <= RT * KC).  A thread owns EPT
// consecutive tokens in each tile of RT*EPT tokens; scores and residuals are read from
// memory once, all loads in flight together, and the radix passes and the ordered pass run
// out of registers.  The only other memory round trip is the pool list between the steps.
// ---------------------------------------------------------------------------
// hist[digit] += cnt (cnt in 0..EPT) for every lane, lanes that agree with a leader merged
// through ballots of the three bits of cnt; see hist_add_aggregated.
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

// k-th largest of the keys in key[0..KC) (slot s is valid iff valid(s)); see radix_select_desc.
template <typename ValidFn>
__device__ __forceinline__ void radix_select_regs(const uint32_t (&key)[KC], ValidFn valid, int n_tiles, int k, RouteShared& sh,
                                  uint32_t& thr, int& quota) {
  static_assert(EPT == 4, "the weighted histogram add packs counts of up to 4 into three ballots");
  uint32_t prefix = 0, mask = 0;
  int remaining = k;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  int shift = 32;
#pragma unroll 1
  for (int pass = 0; pass < 3; ++pass) {
    const int bits = pass == 2 ? 10 : 11;
    const uint32_t dmask = (1u << bits) - 1u;
    shift -= bits;
    for (int i = threadIdx.x; i < kBins; i += RT) sh.hist[i] = 0;
    __syncthreads();
    if (pass == 0) {
      // neighbouring tokens mostly share the leading digit: count the thread's tokens that
      // agree with its first valid one and add them in one go; the others go one by one
#pragma unroll
      for (int t = 0; t < KC / EPT; ++t) {
        if (t < n_tiles) {                    // uniform: whole waves take part
          uint32_t dg[EPT];
          bool ok[EPT];
#pragma unroll
          for (int j = 0; j < EPT; ++j) { dg[j] = (key[t * EPT + j] >> shift) & dmask; ok[j] = valid(t * EPT + j); }
          int cnt = 0;
#pragma unroll
          for (int j = 0; j < EPT; ++j) cnt += ok[j] && dg[j] == dg[0];
          if (!ok[0]) cnt = 0;
          hist_add_weighted(sh.hist, dg[0], cnt, lane);
#pragma unroll
          for (int j = 1; j < EPT; ++j)
            if (ok[j] && !(ok[0] && dg[j] == dg[0])) atomicAdd(&sh.hist[dg[j]], 1);
        }
      }
    } else {
#pragma unroll
      for (int s = 0; s < KC; ++s)
        if (s / EPT < n_tiles && valid(s) && (key[s] & mask) == prefix) atomicAdd(&sh.hist[(key[s] >> shift) & dmask], 1);
    }
    __syncthreads();
    const int b_hi = kBins - 1 - 2 * threadIdx.x;
    const int c0 = sh.hist[b_hi], c1 = sh.hist[b_hi - 1];
    const int tot = c0 + c1;
    const int incl_w = wave_incl_scan_i(tot, lane);
    if (lane == 63) sh.wave_sum[wave] = incl_w;
    __syncthreads();
    int above = incl_w - tot;
    for (int wv = 0; wv < wave; ++wv) above += sh.wave_sum[wv];
    if (above < remaining && remaining <= above + tot) {
      int d = b_hi;
      if (remaining > above + c0) { above += c0; d = b_hi - 1; }
      sh.digit = d;
      sh.above = above;
    }
    __syncthreads();
    prefix |= ((uint32_t)sh.digit) << shift;
    mask |= dmask << shift;
    remaining -= sh.above;
  }
  thr = prefix;
  quota = remaining;
  __syncthreads();
}

// Ordered pass over keys held in registers; see ordered_select.  emit(slot, selected, rank).
// All tiles are scanned together: every wave scans each of its tiles, one wave turns the
// (tile, wave) totals into exclusive prefixes, and the ranks follow with two barriers in all.
// Counts travel packed, "greater" in the high half-word and "equal" in the low one (each at
// most RT * KC = 32768, so neither half overflows).
template <typename ValidFn, typename EmitFn>
__device__ __forceinline__ void ordered_select_regs(const uint32_t (&key)[KC], ValidFn valid, int n_tiles, uint32_t thr, int quota,
                                    EmitFn emit, RouteShared& sh) {
  constexpr int NTL = KC / EPT;
  static_assert(NTL * RW == 2 * kWave, "one wave, two entries per lane, covers the (tile, wave) table");
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  auto cls_of = [&](int s) { return valid(s) ? (key[s] > thr ? 2 : (key[s] == thr ? 1 : 0)) : 0; };
  uint32_t before[NTL];                         // packed counts of this wave's earlier lanes, per tile
#pragma unroll
  for (int t = 0; t < NTL; ++t) {
    uint32_t packed = 0;
    if (t < n_tiles) {
#pragma unroll
      for (int j = 0; j < EPT; ++j) {
        const int c = cls_of(t * EPT + j);
        packed += (c == 2 ? 0x10000u : 0u) + (c == 1 ? 1u : 0u);
      }
    }
    const uint32_t incl = (uint32_t)wave_incl_scan_i((int)packed, lane);
    before[t] = incl - packed;
    if (lane == 63) sh.tile_wave[t * RW + wave] = incl;
  }
  __syncthreads();
  if (wave == 0) {
    const uint32_t x0 = sh.tile_wave[2 * lane], x1 = sh.tile_wave[2 * lane + 1];
    const uint32_t incl = (uint32_t)wave_incl_scan_i((int)(x0 + x1), lane);
    sh.tile_wave[2 * lane] = incl - x0 - x1;
    sh.tile_wave[2 * lane + 1] = incl - x1;
  }
  __syncthreads();
#pragma unroll
  for (int t = 0; t < NTL; ++t) {
    if (t < n_tiles) {
      const uint32_t pre = sh.tile_wave[t * RW + wave] + before[t];
      int pre_gt = (int)(pre >> 16), pre_eq = (int)(pre & 0xffffu);
#pragma unroll
      for (int j = 0; j < EPT; ++j) {
        const int s = t * EPT + j;
        if (valid(s)) {
          const int c = cls_of(s);
          const bool sel = c == 2 || (c == 1 && pre_eq < quota);
          emit(s, sel, pre_gt + min(pre_eq, quota));
          pre_gt += c == 2;
          pre_eq += c == 1;
        }
      }
    }
  }
  __syncthreads();                              // the table is free for the next call
}

// Step 3 on a pool list held in memory (token index and residual key per pool slot, in token
// order) with at most RT*KC entries: keys in registers, as above.
__device__ __forceinline__ void pool_stage_cached(uint32_t (&key)[KC], uint32_t* side_lds, RouteShared& sh, int n_pool, int n_approx,
                                  uint8_t* tr, int32_t* ir, int32_t* ia, const int32_t* pidx, const uint32_t* pkey) {
  auto token_of = [&](int s) { return (s / EPT) * RT * EPT + (int)threadIdx.x * EPT + (s % EPT); };
  uint32_t thr;
  int quota;
  // Step 3: inside the pool, the n_approx tokens of lowest residual lose their value
  if (n_approx == 0) {
    for (int i = threadIdx.x; i < n_pool; i += RT) ir[i] = pidx[i];
    return;
  }
  const int p_tiles = (n_pool + RT * EPT - 1) / (RT * EPT);
#pragma unroll
  for (int s = 0; s < KC; ++s) {
    const int i = token_of(s);
    const bool in = s / EPT < p_tiles && i < n_pool;
    key[s] = in ? pkey[i] : 0u;
    if (s / EPT < p_tiles) side_lds[s * RT + threadIdx.x] = in ? (uint32_t)pidx[i] : 0u;
  }
  radix_select_regs(key, [&](int s) { return token_of(s) < n_pool; }, p_tiles, n_approx, sh, thr, quota);
  ordered_select_regs(key, [&](int s) { return token_of(s) < n_pool; }, p_tiles, thr, quota,
      [&](int s, bool sel, int rank) {
        const int i = token_of(s);
        const int tok = (int)side_lds[s * RT + threadIdx.x];
        if (sel) {
          if (rank < n_approx) {
            ia[rank] = tok;
            tr[tok] = VECTOR_TIER_APPROX;
          }
        } else if (i - rank < n_pool - n_approx) {
          ir[i - rank] = tok;
        }
      }, sh);
}

__global__ __launch_bounds__(RT) void route_cached_kernel(const float* __restrict__ score, const float* __restrict__ eps,
                                                          int n, int n_pool, int n_approx, uint8_t* __restrict__ tier,
                                                          int32_t* __restrict__ idx_retain,
                                                          int32_t* __restrict__ idx_approx, int32_t* __restrict__ pool_idx,
                                                          uint32_t* __restrict__ pool_key) {
  __shared__ RouteShared sh;
  // second word of every slot (residual bits, then pool token index): [slot][thread], kept in
  // LDS as an extension of the register file (each thread only ever touches its own column)
  extern __shared__ uint32_t side_lds[];
  const int h = blockIdx.x;
  const float* sc = score + (size_t)h * n;
  const float* ep = eps + (size_t)h * n;
  uint8_t* tr = tier + (size_t)h * n;
  int32_t* pidx = pool_idx + (size_t)h * n_pool;
  uint32_t* pkey = pool_key + (size_t)h * n_pool;
  int32_t* ir = idx_retain + (size_t)h * (n_pool - n_approx);
  int32_t* ia = idx_approx + (size_t)h * n_approx;

  if (n_pool == 0) {
    for (int i = threadIdx.x; i < n; i += RT) tr[i] = VECTOR_TIER_EVICT;
    return;
  }
  // slot s of a thread = token (s / EPT) * RT * EPT + tid * EPT + s % EPT
  auto token_of = [&](int s) { return (s / EPT) * RT * EPT + (int)threadIdx.x * EPT + (s % EPT); };
  const int n_tiles = (n + RT * EPT - 1) / (RT * EPT);

  // Step 1: the pool is the n_pool tokens of highest score.  One round trip brings in every
  // score and residual this thread will need.
  uint32_t key[KC];
  static_assert(EPT == 4, "a thread's tokens of one tile are one 16-byte load");
  if ((n & 3) == 0 && ((reinterpret_cast<uintptr_t>(sc) | reinterpret_cast<uintptr_t>(ep)) & 15u) == 0) {
    float4 s4[KC / EPT], e4[KC / EPT];
#pragma unroll
    for (int t = 0; t < KC / EPT; ++t) {
      const int i = token_of(t * EPT);
      if (t < n_tiles && i < n) {               // n is a multiple of 4: all four tokens are inside
        s4[t] = *reinterpret_cast<const float4*>(sc + i);
        e4[t] = *reinterpret_cast<const float4*>(ep + i);
      }
    }
#pragma unroll
    for (int t = 0; t < KC / EPT; ++t) {
      const bool in = t < n_tiles && token_of(t * EPT) < n;
      const float sv[EPT] = {s4[t].x, s4[t].y, s4[t].z, s4[t].w}, ev[EPT] = {e4[t].x, e4[t].y, e4[t].z, e4[t].w};
#pragma unroll
      for (int j = 0; j < EPT; ++j) {
        key[t * EPT + j] = in ? float_key(sv[j]) : 0u;
        if (t < n_tiles) side_lds[(t * EPT + j) * RT + threadIdx.x] = in ? ~float_key(ev[j]) : 0u;
      }
    }
  } else {
#pragma unroll
    for (int s = 0; s < KC; ++s) {
      const int i = token_of(s);
      const bool in = s / EPT < n_tiles && i < n;
      key[s] = in ? float_key(sc[i]) : 0u;
      if (s / EPT < n_tiles) side_lds[s * RT + threadIdx.x] = in ? ~float_key(ep[i]) : 0u;   // smaller residual, larger key
    }
  }
  uint32_t thr;
  int quota;
  radix_select_regs(key, [&](int s) { return token_of(s) < n; }, n_tiles, n_pool, sh, thr, quota);
  ordered_select_regs(key, [&](int s) { return token_of(s) < n; }, n_tiles, thr, quota,
      [&](int s, bool sel, int rank) {
        const int i = token_of(s);
        tr[i] = sel ? VECTOR_TIER_RETAIN : VECTOR_TIER_EVICT;
        if (sel && rank < n_pool) {            // rank < n_pool by construction; never write past the list
          pidx[rank] = i;
          pkey[rank] = side_lds[s * RT + threadIdx.x];
        }
      }, sh);
  __threadfence();
  __syncthreads();

  pool_stage_cached(key, side_lds, sh, n_pool, n_approx, tr, ir, ia, pidx, pkey);
}

// ---------------------------------------------------------------------------
// Long sequences (n > RT*KC): the selection by score runs on the whole chip
// ---------------------------------------------------------------------------
// One workgroup per head cannot hold a long sequence in registers and would walk it from
// memory for every radix digit.  Here a head is cut into chunks of RT*WK tokens, one workgroup
// each, which keeps its keys in registers for one kernel:
//   route_wide_hist_kernel<L>, L = 0, 1, 2: histogram of digit L of the chunk's keys that
//       match the digits chosen so far -> one partial histogram per chunk (plain stores, no
//       atomics between workgroups).  For L >= 1 every workgroup first chooses digit L-1
//       itself from the partial histograms of the previous launch (all of them come to the
//       same answer; chunk 0 records it).  L = 2 also counts the chunk's keys above the
//       two-digit prefix.
//   route_wide_emit_kernel: chooses the last digit (threshold key and tie quota), gets the
//       number of selected tokens in earlier chunks from the partial histograms, and makes the
//       ordered pass over its chunk: tiers, and the pool list (token index, residual key) in
//       token order.
//   route_pool_kernel: the selection by residual inside the pool, one workgroup per head, on
//       the pool list (keys in registers when the pool has at most RT*KC entries).
constexpr int WK = 8;                           // consecutive tokens per thread
constexpr int kWideChunk = RT * WK;
constexpr int kWideMaxChunks = 64;

struct WideState { uint32_t prefix, mask; int remaining, pad; };

struct WideParams {
  const float* score; const float* eps;
  int n, n_pool, n_heads, n_chunks;
  uint32_t* hist_part;        // [3][H][C][kBins]
  int* gt_part;               // [H][C]: keys of the chunk above the two-digit prefix
  WideState* state;           // [2][H]: after digit 0, after digit 1
  uint8_t* tier; int32_t* pool_idx; uint32_t* pool_key;
};

__device__ __forceinline__ int wide_shift(int level) { return level == 0 ? 21 : (level == 1 ? 10 : 0); }
__device__ __forceinline__ uint32_t wide_dmask(int level) { return level == 2 ? 1023u : 2047u; }

// The digit d with #(digit > d) < remaining <= #(digit >= d), from per-thread counts of bins
// kBins-1-2t (c0) and kBins-2-2t (c1); every thread gets d and #(digit > d).
__device__ __forceinline__ void wide_pick(int c0, int c1, int remaining, RouteShared& sh, int& digit, int& above_out) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int b_hi = kBins - 1 - 2 * threadIdx.x;
  const int tot = c0 + c1;
  const int incl_w = wave_incl_scan_i(tot, lane);
  if (lane == 63) sh.wave_sum[wave] = incl_w;
  __syncthreads();
  int above = incl_w - tot;
  for (int wv = 0; wv < wave; ++wv) above += sh.wave_sum[wv];
  if (above < remaining && remaining <= above + tot) {
    int d = b_hi;
    if (remaining > above + c0) { above += c0; d = b_hi - 1; }
    sh.digit = d;
    sh.above = above;
  }
  __syncthreads();
  digit = sh.digit;
  above_out = sh.above;
  __syncthreads();                              // sh.digit / sh.above / wave_sum are free again
}

// this thread's WK keys of the chunk (0 and not valid beyond n)
__device__ __forceinline__ void wide_load_keys(const float* sc, int n, int base, uint32_t (&key)[WK], bool (&valid)[WK]) {
  if ((n & 3) == 0 && (reinterpret_cast<uintptr_t>(sc) & 15u) == 0) {
#pragma unroll
    for (int q = 0; q < WK / 4; ++q) {
      const int i = base + 4 * q;
      float4 x = make_float4(0.f, 0.f, 0.f, 0.f);
      if (i < n) x = *reinterpret_cast<const float4*>(sc + i);
      const float xv[4] = {x.x, x.y, x.z, x.w};
#pragma unroll
      for (int j = 0; j < 4; ++j) { valid[4 * q + j] = i < n; key[4 * q + j] = i < n ? float_key(xv[j]) : 0u; }
    }
  } else {
#pragma unroll
    for (int j = 0; j < WK; ++j) { valid[j] = base + j < n; key[j] = valid[j] ? float_key(sc[base + j]) : 0u; }
  }
}

// sum over the chunks of one bin pair of a level's partial histograms
__device__ __forceinline__ void wide_bin_sums(const uint32_t* hp, int n_chunks, int& c0, int& c1) {
  const int b_hi = kBins - 1 - 2 * threadIdx.x;
  c0 = 0; c1 = 0;
  for (int c = 0; c < n_chunks; ++c) {
    const uint2 v = *reinterpret_cast<const uint2*>(hp + (size_t)c * kBins + b_hi - 1);   // bins b_hi-1, b_hi
    c1 += (int)v.x;
    c0 += (int)v.y;
  }
}

template <int L>
__global__ __launch_bounds__(RT) void route_wide_hist_kernel(WideParams p) {
  __shared__ RouteShared sh;
  const int h = blockIdx.y, chunk = blockIdx.x;
  const int lane = threadIdx.x & 63;
  const size_t level_stride = (size_t)p.n_heads * p.n_chunks * kBins;
  uint32_t prefix = 0, mask = 0;
  int remaining = p.n_pool;
  if (L >= 1) {
    if (L == 2) { const WideState st = p.state[h]; prefix = st.prefix; mask = st.mask; remaining = st.remaining; }
    int c0, c1, digit, above;
    wide_bin_sums(p.hist_part + (size_t)(L - 1) * level_stride + (size_t)h * p.n_chunks * kBins, p.n_chunks, c0, c1);
    wide_pick(c0, c1, remaining, sh, digit, above);
    prefix |= ((uint32_t)digit) << wide_shift(L - 1);
    mask |= wide_dmask(L - 1) << wide_shift(L - 1);
    remaining -= above;
    if (chunk == 0 && threadIdx.x == 0) {
      WideState st; st.prefix = prefix; st.mask = mask; st.remaining = remaining; st.pad = 0;
      p.state[(size_t)(L - 1) * p.n_heads + h] = st;
    }
  }
  uint32_t key[WK];
  bool valid[WK];
  wide_load_keys(p.score + (size_t)h * p.n, p.n, chunk * kWideChunk + (int)threadIdx.x * WK, key, valid);
  for (int i = threadIdx.x; i < kBins; i += RT) sh.hist[i] = 0;
  __syncthreads();
  int gt = 0;
#pragma unroll
  for (int j = 0; j < WK; ++j) {
    const bool active = valid[j] && (key[j] & mask) == prefix;
    const uint32_t digit = (key[j] >> wide_shift(L)) & wide_dmask(L);
    if (L == 0) hist_add_aggregated(sh.hist, digit, active, lane);
    else if (active) atomicAdd(&sh.hist[digit], 1);
    if (L == 2) gt += valid[j] && (key[j] & mask) > prefix;
  }
  __syncthreads();
  uint32_t* out = p.hist_part + (size_t)L * level_stride + ((size_t)h * p.n_chunks + chunk) * kBins;
  for (int i = threadIdx.x; i < kBins; i += RT) out[i] = (uint32_t)sh.hist[i];
  if (L == 2) {
    gt = wave_sum_i(gt);
    if (lane == 0) sh.wave_sum[threadIdx.x >> 6] = gt;
    __syncthreads();
    if (threadIdx.x == 0) {
      int t = 0;
      for (int wv = 0; wv < RW; ++wv) t += sh.wave_sum[wv];
      p.gt_part[(size_t)h * p.n_chunks + chunk] = t;
    }
  }
}

__global__ __launch_bounds__(RT) void route_wide_emit_kernel(WideParams p) {
  __shared__ RouteShared sh;
  __shared__ int base_lds[2];
  const int h = blockIdx.y, chunk = blockIdx.x;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const size_t level_stride = (size_t)p.n_heads * p.n_chunks * kBins;
  const uint32_t* hp2 = p.hist_part + 2 * level_stride + (size_t)h * p.n_chunks * kBins;
  const WideState st = p.state[(size_t)p.n_heads + h];
  int c0, c1, d2, above2;
  wide_bin_sums(hp2, p.n_chunks, c0, c1);
  wide_pick(c0, c1, st.remaining, sh, d2, above2);
  const uint32_t thr = st.prefix | (uint32_t)d2;
  const int quota = st.remaining - above2;
  // selected tokens of earlier chunks: keys above the two-digit prefix, keys of the prefix with
  // a last digit above d2, and threshold ties
  {
    const int b_hi = kBins - 1 - 2 * threadIdx.x;
    int x = 0;
    for (int c = 0; c < chunk; ++c) {
      const uint2 v = *reinterpret_cast<const uint2*>(hp2 + (size_t)c * kBins + b_hi - 1);
      x += (b_hi > d2 ? (int)v.y : 0) + (b_hi - 1 > d2 ? (int)v.x : 0);
    }
    x = wave_sum_i(x);
    if (lane == 0) sh.wave_sum[wave] = x;
    __syncthreads();
    if (threadIdx.x == 0) {
      int gt = 0, eq = 0;
      for (int wv = 0; wv < RW; ++wv) gt += sh.wave_sum[wv];
      for (int c = 0; c < chunk; ++c) {
        gt += p.gt_part[(size_t)h * p.n_chunks + c];
        eq += (int)hp2[(size_t)c * kBins + d2];
      }
      base_lds[0] = gt;
      base_lds[1] = eq;
    }
    __syncthreads();
  }
  const int base_gt = base_lds[0], base_eq = base_lds[1];
  // ordered pass over the chunk
  const int t_base = chunk * kWideChunk + (int)threadIdx.x * WK;
  uint32_t key[WK];
  bool valid[WK];
  wide_load_keys(p.score + (size_t)h * p.n, p.n, t_base, key, valid);
  float ev[WK];
#pragma unroll
  for (int j = 0; j < WK; ++j) ev[j] = valid[j] ? p.eps[(size_t)h * p.n + t_base + j] : 0.f;
  uint32_t packed = 0;
#pragma unroll
  for (int j = 0; j < WK; ++j)
    packed += (valid[j] && key[j] > thr ? 0x10000u : 0u) + (valid[j] && key[j] == thr ? 1u : 0u);
  const uint32_t incl = (uint32_t)wave_incl_scan_i((int)packed, lane);
  if (lane == 63) sh.tile_wave[wave] = incl;
  __syncthreads();
  uint32_t pre = incl - packed;
  for (int wv = 0; wv < wave; ++wv) pre += sh.tile_wave[wv];
  int pre_gt = base_gt + (int)(pre >> 16), pre_eq = base_eq + (int)(pre & 0xffffu);
  uint8_t* tr = p.tier + (size_t)h * p.n;
  int32_t* pidx = p.pool_idx + (size_t)h * p.n_pool;
  uint32_t* pkey = p.pool_key + (size_t)h * p.n_pool;
#pragma unroll
  for (int j = 0; j < WK; ++j) {
    if (valid[j]) {
      const int c = key[j] > thr ? 2 : (key[j] == thr ? 1 : 0);
      const bool sel = c == 2 || (c == 1 && pre_eq < quota);
      const int rank = pre_gt + min(pre_eq, quota);
      tr[t_base + j] = sel ? VECTOR_TIER_RETAIN : VECTOR_TIER_EVICT;
      if (sel && rank < p.n_pool) {                // rank < n_pool by construction; never write past the list
        pidx[rank] = t_base + j;
        pkey[rank] = ~float_key(ev[j]);            // smaller residual, larger key
      }
      pre_gt += c == 2;
      pre_eq += c == 1;
    }
  }
}

// Step 3 alone, on a pool list written by route_wide_emit_kernel
__global__ __launch_bounds__(RT) void route_pool_kernel(int n, int n_pool, int n_approx, uint8_t* __restrict__ tier,
                                                        int32_t* __restrict__ idx_retain, int32_t* __restrict__ idx_approx,
                                                        const int32_t* __restrict__ pool_idx, const uint32_t* __restrict__ pool_key) {
  __shared__ RouteShared sh;
  extern __shared__ uint32_t side_lds[];
  const int h = blockIdx.x;
  uint8_t* tr = tier + (size_t)h * n;
  const int32_t* pidx = pool_idx + (size_t)h * n_pool;
  const uint32_t* pkey = pool_key + (size_t)h * n_pool;
  int32_t* ir = idx_retain + (size_t)h * (n_pool - n_approx);
  int32_t* ia = idx_approx + (size_t)h * n_approx;
  if (n_pool <= RT * KC) {
    uint32_t key[KC];
    pool_stage_cached(key, side_lds, sh, n_pool, n_approx, tr, ir, ia, pidx, pkey);
    return;
  }
  if (n_approx == 0) {
    for (int i = threadIdx.x; i < n_pool; i += RT) ir[i] = pidx[i];
    return;
  }
  uint32_t thr;
  int quota;
  radix_select_desc([&](int i) { return pkey[i]; }, n_pool, n_approx, sh, thr, quota);
  ordered_select(
      [&](int i) { uint32_t key = pkey[i]; return key > thr ? 2 : (key == thr ? 1 : 0); },
      [&](int i, bool sel, int rank) {
        const int tok = pidx[i];
        if (sel) {
          if (rank < n_approx) {
            ia[rank] = tok;
            tr[tok] = VECTOR_TIER_APPROX;
          }
        } else if (i - rank < n_pool - n_approx) {
          ir[i - rank] = tok;
        }
      },
      n_pool, quota, sh);
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

#ifndef VEC_WIDE_MIN_TOKENS
#define VEC_WIDE_MIN_TOKENS (RT * KC + 1)
#endif
static bool route_is_wide(int seq_len, int n_pool) {
  return seq_len >= VEC_WIDE_MIN_TOKENS && n_pool > 0 && (seq_len + kWideChunk - 1) / kWideChunk <= kWideMaxChunks;
}

size_t route_workspace_bytes(int n_kv_heads, int seq_len, int n_pool) {
  size_t b = align_up((size_t)n_kv_heads * n_pool * sizeof(int32_t), 256) + align_up((size_t)n_kv_heads * n_pool * sizeof(uint32_t), 256);
  if (route_is_wide(seq_len, n_pool > 0 ? n_pool : 1)) {
    const size_t C = (seq_len + kWideChunk - 1) / kWideChunk;
    b += align_up((size_t)3 * n_kv_heads * C * kBins * sizeof(uint32_t), 256) + align_up((size_t)n_kv_heads * C * sizeof(int), 256) +
         align_up((size_t)2 * n_kv_heads * sizeof(WideState), 256);
  }
  return b;
}

int launch_route(int n_kv_heads, int seq_len, const float* score, const float* eps, int n_pool, int n_approx,
                 uint8_t* tier, int32_t* idx_retain, int32_t* idx_approx, void* ws, hipStream_t stream) {
  unsigned char* w8 = reinterpret_cast<unsigned char*>(ws);
  int32_t* pool_idx = reinterpret_cast<int32_t*>(w8);
  w8 += align_up((size_t)n_kv_heads * n_pool * sizeof(int32_t), 256);
  uint32_t* pool_key = reinterpret_cast<uint32_t*>(w8);
  w8 += align_up((size_t)n_kv_heads * n_pool * sizeof(uint32_t), 256);
  if (seq_len <= RT * KC && !route_is_wide(seq_len, n_pool)) {
    const int n_tiles = (seq_len + RT * EPT - 1) / (RT * EPT);
    const size_t lds = (size_t)n_tiles * EPT * RT * sizeof(uint32_t);
    VEC_HIP(set_max_lds(reinterpret_cast<const void*>(route_cached_kernel), lds));
    VEC_LAUNCH(K_ROUTE, route_cached_kernel, dim3(n_kv_heads), dim3(RT), lds, stream, score, eps, seq_len, n_pool,
               n_approx, tier, idx_retain, idx_approx, pool_idx, pool_key);
  } else if (route_is_wide(seq_len, n_pool)) {
    WideParams p;
    p.score = score; p.eps = eps; p.n = seq_len; p.n_pool = n_pool; p.n_heads = n_kv_heads;
    p.n_chunks = (seq_len + kWideChunk - 1) / kWideChunk;
    p.hist_part = reinterpret_cast<uint32_t*>(w8);
    w8 += align_up((size_t)3 * n_kv_heads * p.n_chunks * kBins * sizeof(uint32_t), 256);
    p.gt_part = reinterpret_cast<int*>(w8);
    w8 += align_up((size_t)n_kv_heads * p.n_chunks * sizeof(int), 256);
    p.state = reinterpret_cast<WideState*>(w8);
    p.tier = tier; p.pool_idx = pool_idx; p.pool_key = pool_key;
    const dim3 grid(p.n_chunks, n_kv_heads);
    const bool t_ = timing_enabled();
    if (t_) timing_begin(K_ROUTE, stream);           // the five launches count as one routing step
    hipLaunchKernelGGL(route_wide_hist_kernel<0>, grid, dim3(RT), 0, stream, p);
    hipLaunchKernelGGL(route_wide_hist_kernel<1>, grid, dim3(RT), 0, stream, p);
    hipLaunchKernelGGL(route_wide_hist_kernel<2>, grid, dim3(RT), 0, stream, p);
    hipLaunchKernelGGL(route_wide_emit_kernel, grid, dim3(RT), 0, stream, p);
    const int p_tiles = (n_pool + RT * EPT - 1) / (RT * EPT);
    const size_t lds = n_pool <= RT * KC ? (size_t)p_tiles * EPT * RT * sizeof(uint32_t) : 0;
    VEC_HIP(set_max_lds(reinterpret_cast<const void*>(route_pool_kernel), lds));
    hipLaunchKernelGGL(route_pool_kernel, dim3(n_kv_heads), dim3(RT), lds, stream, seq_len, n_pool, n_approx, tier, idx_retain,
                       idx_approx, pool_idx, pool_key);
    if (t_) timing_end(K_ROUTE, stream);
  } else {
    VEC_LAUNCH(K_ROUTE, route_kernel, dim3(n_kv_heads), dim3(RT), 0, stream, score, eps, seq_len, n_pool, n_approx, tier,
               idx_retain, idx_approx, pool_idx, pool_key);
  }
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
