// Three-way routing (Section 3.2, Steps 1 and 3) and compaction into the packed cache.
//
// Both selections of a head (the n_pool highest scores; inside that pool the n_approx lowest
// residuals) are radix selects on order-preserving 32-bit keys with digits of 11, 11 and 10 bits,
// spread over the whole chip and synchronised by kernel boundaries only:
//
//   route_bucket_kernel  grid (chunk, head).  Counts the leading digit of a chunk's score keys and
//                        writes the chunk's (key, token) pairs grouped by that digit, highest digit
//                        first, next to the table D[b] = #keys of the chunk with digit >= b.  The
//                        POOL variant first forms the score itself, the average pooling of the
//                        attention mass (Step 1's base scorer), so the scorer's last kernel already
//                        hands the routing its buckets.
//   route_pool_kernel    grid (chunk, head).  Every workgroup sums the D tables of its head: the
//                        leading digit of the threshold is the bin where the sum crosses n_pool,
//                        and the keys that share it are one contiguous piece of every chunk's
//                        bucket list.  Those few keys go to LDS and the select finishes on them (all
//                        workgroups of a head reach the same threshold).  Then the ordered pass
//                        over the workgroup's own chunk: tiers, the pool list (token index and
//                        residual key, in token order) and the D table of the chunk's residual keys.
//   route_split_kernel   grid (slice, head).  The same select on the residual keys of the pool
//                        list (read whole: a pool is a fraction of the sequence), then the ordered
//                        pass over a slice of the list: ascending idx_approx / idx_retain, and the
//                        approximated tier.
//
// Every slot of an output comes from an ordered prefix sum (ties go to the lower token index);
// atomics only feed LDS histograms and the order inside a bucket, which no result depends on.
// No workgroup waits for another inside a kernel.
//
// gather_rows_kernel: row gather k_ret / v_ret / k_apx by the index lists.
#include <cstring>

#include "common.hpp"
#include "launch.hpp"

#ifdef VEC_ROUTE_TRACE      // tuning builds only: time stamps of workgroup (0, 0)
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

constexpr int kBins = 2048;
constexpr int kTableStride = kBins + 8;   // 16-bit entries of a D table: D[0 .. 2048] and padding to 16 bytes
constexpr int EPT = 4;                    // consecutive elements per thread and tile (one 16-byte load)
constexpr int BT = 512;                   // threads of the bucket kernel
constexpr int kBucketTile = BT * EPT;
constexpr int kStageTokens = 4096;        // a chunk's bucket list is put together in LDS up to this length
constexpr int ST = 256;                   // threads of a selecting workgroup: one wave per SIMD
constexpr int SW = ST / kWave;
constexpr int kTile = ST * EPT;           // elements per tile of a selecting workgroup
constexpr int kBatch = 8;                 // tiles whose loads are in flight together
constexpr int kCandCap = 12288;           // candidates (keys sharing the threshold's leading digit) kept in LDS
constexpr int kWaveCand = kCandCap / SW;  // each wave keeps its own: no shared counter
constexpr int kMinChunk = 2048;           // tokens per chunk: doubled until a head has at most kMaxChunks
constexpr int kMaxChunks = 32;

// Order-preserving map float -> u32 (larger float, larger key); -0 and +0 share a key.
__device__ __forceinline__ uint32_t float_key(float x) {
  uint32_t b = __float_as_uint(x + 0.0f);
  return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}

// Leading digit of a key: which of the 2048 buckets of the first radix level it falls in.  Plain:
// the key's top 11 bits, a quarter of an octave of scores per bucket.  When the scorer has told
// where the bulk of a head's scores lies, 2046 buckets of 2^shift keys each are laid over that
// range instead, so that scores which agree in their leading bits (a flat attention row: every
// score within a few per cent of 1/n) still spread over the buckets; bucket 0 takes every key below
// the range and bucket 2047 every key above it (attention sinks, the +inf of the window columns).
// Keys of one bucket between 1 and 2046 agree in all bits from `shift` up; the two end buckets
// (and they alone) may hold keys that differ anywhere.  Wherever a score falls the select stays
// exact: the range only decides how evenly the buckets fill.
struct DigitMap {
  uint32_t lowq;
  int shift;
  __device__ __forceinline__ bool plain() const { return shift == 21 && lowq == 0u; }
  __device__ __forceinline__ uint32_t digit(uint32_t key) const {
    // a saturating difference: written with max (a compare-and-select around `q - lowq` is folded away by
    // this compiler at -O3, which then lets the difference wrap)
    const uint32_t q = key >> shift;
    return min(max(q, lowq) - lowq, 2047u);
  }
  __device__ __forceinline__ bool shares_high_bits(int d) const { return plain() || (d > 0 && d < 2047); }
};
// 2046 buckets of 2^shift keys each over [klo, khi], shift as small as that allows
__device__ __forceinline__ DigitMap digit_map_for_keys(uint32_t klo, uint32_t khi) {
  DigitMap plain = {0u, 21};
  if (khi < klo) return plain;
  // (khi >> s) - (klo >> s) <= ((khi - klo) >> s) + 1: start where the difference has 11 bits left
  const uint32_t diff = khi - klo;
  int s = diff ? max(0, 21 - (int)__clz(diff)) : 0;
  if ((khi >> s) - (klo >> s) > 2045u) ++s;
  if (s >= 21) return plain;
  DigitMap m = {max(klo >> s, 1u) - 1u, s};
  return m;
}
// cnt, sum_l, sum_ll: over the head's prefix columns of positive attention mass m, their number and
// the sums of l = log2(m) - log_ref and of l * l.  The buckets cover the mean of log2(m) give or
// take four standard deviations (and a 64th of an octave, so that equal masses still get a
// range): at most a sixteenth of the columns lie outside, whatever their distribution, and a few
// columns far from the rest (attention sinks, the zero-padded edges of the pooling) move the range
// very little.
__device__ __forceinline__ DigitMap digit_map_for_stats(float cnt, float sum_l, float sum_ll, float log_ref) {
  DigitMap plain = {0u, 21};
  if (!(cnt >= 1.f)) return plain;
  // hardware reciprocal, square root and exponential: a rough range is all that is needed, and
  // every wave of the head gets the same bits from the same inputs
  const float inv = __builtin_amdgcn_rcpf(cnt);
  const float mu = sum_l * inv;
  const float sd = __builtin_amdgcn_sqrtf(fmaxf(sum_ll * inv - mu * mu, 0.f));
  const float mid = log_ref + mu, half = 4.f * sd + 0.015625f;
  if (!(mid - half > -120.f) || !(mid + half < 120.f)) return plain;        // also NaN
  return digit_map_for_keys(float_key(__builtin_amdgcn_exp2f(mid - half)), float_key(__builtin_amdgcn_exp2f(mid + half)));
}
// The same from a sample of the keys themselves, for scores of any sign that arrive without
// statistics (vector_route on its own): cnt keys k = key >> 12 with sum s1 and sum of squares s2.
// For positive floats the key is linear in the score inside an octave and counts octaves across
// them, so its mean and deviation bound the bulk the same way.
__device__ __forceinline__ DigitMap digit_map_for_sample(unsigned long long cnt, unsigned long long s1, unsigned long long s2) {
  DigitMap plain = {0u, 21};
  if (cnt < 32) return plain;
  const double inv = 1.0 / (double)cnt, mu = (double)s1 * inv;
  const double var = (double)s2 * inv - mu * mu;
  const double half = 4.0 * sqrt(var > 0.0 ? var : 0.0) + 32.0;             // 32 * 4096 keys: a 64th of an octave
  const double lo = (mu - half) * 4096.0, hi = (mu + half) * 4096.0;
  const uint32_t klo = lo > 0.0 ? (uint32_t)lo : 0u, khi = hi < 4294967295.0 ? (uint32_t)hi : 0xffffffffu;
  return digit_map_for_keys(klo, khi);
}

// hist[digit] += cnt (cnt in 0..7) for every lane.  Keys of neighbouring tokens often share their
// leading bits, so a plain LDS atomic would serialise up to 64 lanes on one bin: lanes that agree
// with a leader are merged through ballots of the three bits of cnt and added by the leader alone;
// after two rounds the stragglers (few, spread over bins) add themselves.
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
__device__ __forceinline__ void hist_add_thread_keys(int* hist, const uint32_t (&key)[EPT], const bool (&ok)[EPT], int lane,
                                                     const DigitMap& map) {
  uint32_t dg[EPT];
#pragma unroll
  for (int j = 0; j < EPT; ++j) dg[j] = map.digit(key[j]);
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

// NW per-wave values -> their sum over the waves before `wave`, and over all waves
template <int NW> __device__ __forceinline__ void wave_row_sums(const int* row, int wave, int& before, int& total) {
  before = 0;
  total = 0;
#pragma unroll
  for (int q = 0; q < NW; ++q) {
    const int x = row[q];
    total += x;
    before += (q < wave) ? x : 0;
  }
}

// Counts of a 2048-bin LDS histogram -> D[b] = #(digit >= b), written as a 16-bit table to
// global memory (D[2048] = 0 and the padding included); the histogram itself is turned into
// #(digit > b), the first slot of bin b when the keys are laid out highest digit first.
// NT threads, thread t owns the kBins / NT bins below and including kBins - 1 - t * kBins / NT.
// row: LDS, NT / 64 ints.  Ends with a barrier.
template <int NT>
__device__ __forceinline__ void counts_to_table(int* hist, uint16_t* table, int* row) {
  constexpr int BPT = kBins / NT, NW = NT / kWave;
  static_assert(BPT % 2 == 0, "pairs of bins are stored as one word");
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int hi = kBins - 1 - BPT * (int)threadIdx.x;
  int c[BPT], s[BPT], run = 0;
#pragma unroll
  for (int k = 0; k < BPT; ++k) { c[k] = hist[hi - k]; run += c[k]; s[k] = run; }
  const int incl = wave_incl_scan_dpp(run);
  if (lane == 63) row[wave] = incl;
  __syncthreads();
  int before, total;
  wave_row_sums<NW>(row, wave, before, total);
  before += incl - run;
  uint32_t* t32 = reinterpret_cast<uint32_t*>(table);
#pragma unroll
  for (int k = 0; k < BPT; k += 2) {          // bins hi-k (odd) and hi-k-1 (even) share a word
    const uint32_t d_hi = (uint32_t)(before + s[k]), d_lo = (uint32_t)(before + s[k + 1]);
    t32[(hi - k - 1) >> 1] = d_lo | (d_hi << 16);
    hist[hi - k] = before + s[k] - c[k];
    hist[hi - k - 1] = before + s[k + 1] - c[k + 1];
  }
  if (threadIdx.x < (kTableStride - kBins) / 2) t32[kBins / 2 + threadIdx.x] = 0u;
  __syncthreads();
}

// ---------------------------------------------------------------------------
// buckets of the score keys by leading digit (and, POOL, the pooled score itself)
// ---------------------------------------------------------------------------
struct BucketParams;
struct BucketParams {
  const float* src;       // POOL: attention mass [H, n]; otherwise the scores [H, n]
  float* score;           // POOL: output [H, n]
  uint16_t* table;        // [H, C, kTableStride] or null (POOL only: pooling alone)
  uint32_t* bkey;         // [H, n]: chunk c owns [c * chunk_tokens, ...), keys grouped by digit, highest first
  int32_t* bpos;          // [H, n]: the token each key belongs to
  int n, n_prefix, kernel, chunk_tokens, n_chunks;
  int take_max;           // POOL: the window's largest mass instead of its sum over the kernel size
  uint32_t* map;          // [H, 2] with the buckets: the digit map (lowq, shift) this launch chooses, for the selecting launch
  const float4* range;    // [H, n_range] (count, sum l, sum l * l) of the mass left by the scorer's workgroups, when n_range > 0
  int n_range;
  float log_ref;          // what the scorer subtracted from log2(mass)
  const BucketParams* seq_table;   // RAGGED launches: the sequences' parameter blocks, seq_hps heads each
  int seq_hps;
};

// RAGGED launches (several sequences of different lengths at once): launch head hv is head
// hv % seq_hps of sequence hv / seq_hps, whose parameter block replaces the launch's own
template <bool RAGGED, typename P>
__device__ __forceinline__ void take_sequence(P& p, int& h) {
  if constexpr (RAGGED) {
    const int seq = h / p.seq_hps;
    h -= seq * p.seq_hps;
    p = p.seq_table[seq];
  }
}

template <bool POOL, bool RAGGED = false>
__global__ __launch_bounds__(BT) void route_bucket_kernel(BucketParams p) {
  int h = blockIdx.y;
  take_sequence<RAGGED>(p, h);
  if (RAGGED && (int)blockIdx.x >= p.n_chunks) return;
  __shared__ int hist[kBins];
  __shared__ int row[BT / kWave];
  __shared__ uint32_t sample[BT / kWave][4];
  __shared__ __align__(16) uint32_t stage_key[kStageTokens];
  __shared__ __align__(16) int32_t stage_pos[kStageTokens];
  const int chunk = blockIdx.x;
  const int lane = threadIdx.x & 63;
  const bool do_buckets = p.table != nullptr;
  DigitMap map = {0u, 21};
  // every wave adds up the head's statistics itself (in one fixed order), so all workgroups of
  // the head cut the same buckets
  constexpr int kRangeRegs = 2;
  float4 range_x[kRangeRegs];
  if (do_buckets && p.n_range > 0) {
    const float4* r = p.range + (size_t)h * p.n_range;
#pragma unroll
    for (int u = 0; u < kRangeRegs; ++u) {
      const int i = u * kWave + lane;
      range_x[u] = i < p.n_range ? r[i] : make_float4(0.f, 0.f, 0.f, 0.f);
    }
  }
  const float* src = p.src + (size_t)h * p.n;
  const float* scores = POOL ? p.score + (size_t)h * p.n : src;
  const int begin = chunk * p.chunk_tokens, end = min(p.n, begin + p.chunk_tokens);
  // the thread's first four inputs are requested now and only touched (not used) after the map is
  // there: they travel while the statistics are turned into the map, and the first tile's loads
  // below find them in the cache
  float warm = 0.f;
  if (do_buckets && p.n_range > 0) warm = src[min(begin + (int)threadIdx.x * EPT, p.n - 1)];
  if (do_buckets) {
    for (int i = threadIdx.x; i < kBins; i += BT) hist[i] = 0;
    if (p.n_range > 0) {
      float cnt = 0.f, sl = 0.f, sll = 0.f;
#pragma unroll
      for (int u = 0; u < kRangeRegs; ++u) { cnt += range_x[u].x; sl += range_x[u].y; sll += range_x[u].z; }
      const float4* r = p.range + (size_t)h * p.n_range;
      for (int i = kRangeRegs * kWave + lane; i < p.n_range; i += kWave) {       // long sequences only
        const float4 x = r[i];
        cnt += x.x; sl += x.y; sll += x.z;
      }
      map = digit_map_for_stats(wave_sum_dpp(cnt), wave_sum_dpp(sl), wave_sum_dpp(sll), p.log_ref);
      asm volatile("" ::"v"(warm));
    }
    if (!POOL) {
      // no statistics came with the scores: four keys out of every 256, the same sample in every
      // workgroup of the head (integer sums: any order gives the same map)
      uint32_t c = 0, s1 = 0, s2lo = 0, s2hi = 0;
      const bool al = (((size_t)h * p.n) & 3) == 0 && (reinterpret_cast<uintptr_t>(p.src) & 15u) == 0;
      for (int i = (int)threadIdx.x * 256; i < p.n; i += BT * 256) {
        float x[4] = {INFINITY, INFINITY, INFINITY, INFINITY};
        if (al && i + 4 <= p.n) {
          const float4 v = *reinterpret_cast<const float4*>(src + i);
          x[0] = v.x; x[1] = v.y; x[2] = v.z; x[3] = v.w;
        } else {
#pragma unroll
          for (int j = 0; j < 4; ++j)
            if (i + j < p.n) x[j] = src[i + j];
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const uint32_t key = float_key(x[j]);
          if (key > 0x007fffffu && key < 0xff800000u) {                     // finite
            const unsigned long long k = key >> 12, kk = k * k;
            c += 1; s1 += (uint32_t)k; s2lo += (uint32_t)(kk & 0xfffffu); s2hi += (uint32_t)(kk >> 20);
          }
        }
      }
      const int wave = threadIdx.x >> 6;
      c = (uint32_t)wave_total_of_scan(wave_incl_scan_dpp((int)c));
      s1 = (uint32_t)wave_total_of_scan(wave_incl_scan_dpp((int)s1));
      s2lo = (uint32_t)wave_total_of_scan(wave_incl_scan_dpp((int)s2lo));
      s2hi = (uint32_t)wave_total_of_scan(wave_incl_scan_dpp((int)s2hi));
      if (lane == 0) { sample[wave][0] = c; sample[wave][1] = s1; sample[wave][2] = s2lo; sample[wave][3] = s2hi; }
      __syncthreads();
      unsigned long long tc = 0, t1 = 0, t2 = 0;
#pragma unroll
      for (int w = 0; w < BT / kWave; ++w) {
        tc += sample[w][0]; t1 += sample[w][1];
        t2 += (unsigned long long)sample[w][2] + ((unsigned long long)sample[w][3] << 20);
      }
      map = digit_map_for_sample(tc, t1, t2);
    }
    if (chunk == 0 && threadIdx.x == 0) { p.map[2 * h] = map.lowq; p.map[2 * h + 1] = (uint32_t)map.shift; }
    __syncthreads();
  }
  const bool vec4 = (p.n & 3) == 0 && ((reinterpret_cast<uintptr_t>(src) | reinterpret_cast<uintptr_t>(scores)) & 15u) == 0;
  auto load_scores = [&](int t0, float (&s)[EPT]) {
    if (vec4 && t0 + EPT <= end) {
      const float4 x = *reinterpret_cast<const float4*>(scores + t0);
      s[0] = x.x; s[1] = x.y; s[2] = x.z; s[3] = x.w;
    } else {
#pragma unroll
      for (int j = 0; j < EPT; ++j) s[j] = t0 + j < end ? scores[t0 + j] : 0.f;
    }
  };
  uint32_t key0[EPT];                            // the keys of the first tile stay in registers for the scatter
  for (int tile = begin; tile < end; tile += kBucketTile) {        // uniform trip count: whole waves take part
    const int t0 = tile + (int)threadIdx.x * EPT;
    float s[EPT];
    bool ok[EPT];
#pragma unroll
    for (int j = 0; j < EPT; ++j) ok[j] = t0 + j < end;
    if (POOL) {
      const int half = p.kernel / 2;
      if (vec4 && half <= EPT && t0 >= EPT && t0 + 2 * EPT <= p.n) {
        // the 12 mass values around the thread's four tokens in three loads; each window is
        // folded in ascending token order, like the general loop below (mass is never negative,
        // so the maximum may start from zero)
        float m[3 * EPT];
#pragma unroll
        for (int q = 0; q < 3; ++q) {
          const float4 x = *reinterpret_cast<const float4*>(src + t0 - EPT + q * EPT);
          m[q * EPT + 0] = x.x; m[q * EPT + 1] = x.y; m[q * EPT + 2] = x.z; m[q * EPT + 3] = x.w;
        }
#pragma unroll
        for (int j = 0; j < EPT; ++j) {
          const int t = t0 + j;
          float acc = 0.f;
#pragma unroll
          for (int d = -EPT; d <= EPT; ++d)
            if (d >= -half && d <= half && t + d < p.n_prefix) acc = p.take_max ? fmaxf(acc, m[EPT + j + d]) : acc + m[EPT + j + d];
          s[j] = (ok[j] && t < p.n_prefix) ? (p.take_max ? acc : acc / (float)p.kernel) : INFINITY;
        }
      } else {
#pragma unroll
        for (int j = 0; j < EPT; ++j) {
          const int t = t0 + j;
          float out = INFINITY;                                      // window columns
          if (ok[j] && t < p.n_prefix) {
            const int lo = max(0, t - half), hi = min(p.n_prefix - 1, t + half);
            float acc = 0.f;
            for (int i = lo; i <= hi; ++i) acc = p.take_max ? fmaxf(acc, src[i]) : acc + src[i];
            out = p.take_max ? acc : acc / (float)p.kernel;
          }
          s[j] = out;
        }
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
      load_scores(t0, s);
    }
    if (do_buckets) {
      uint32_t key[EPT];
#pragma unroll
      for (int j = 0; j < EPT; ++j) key[j] = float_key(s[j]);
      hist_add_thread_keys(hist, key, ok, lane, map);
      if (tile == begin) {
#pragma unroll
        for (int j = 0; j < EPT; ++j) key0[j] = key[j];
      }
    }
  }
  if (!do_buckets) return;
  __syncthreads();
  counts_to_table<BT>(hist, p.table + ((size_t)h * p.n_chunks + chunk) * kTableStride, row);
  // scatter: hist[b] is now the next free slot of bin b in the chunk's list
  // The slots of neighbouring tokens are far apart in the list (the finer the buckets, the farther),
  // so the list of a chunk that fits is put together in LDS and written out in order; longer
  // chunks scatter their entries straight to memory.
  uint32_t* bkey = p.bkey + (size_t)h * p.n + begin;
  int32_t* bpos = p.bpos + (size_t)h * p.n + begin;
  const bool staged = p.chunk_tokens <= kStageTokens;
  for (int tile = begin; tile < end; tile += kBucketTile) {
    const int t0 = tile + (int)threadIdx.x * EPT;
    uint32_t key[EPT];
    if (tile == begin) {
#pragma unroll
      for (int j = 0; j < EPT; ++j) key[j] = key0[j];
    } else {                                     // later tiles: the scores this thread stored (or read) above
      float s[EPT];
      load_scores(t0, s);
#pragma unroll
      for (int j = 0; j < EPT; ++j) key[j] = float_key(s[j]);
    }
#pragma unroll
    for (int j = 0; j < EPT; ++j) {
      if (t0 + j < end) {
        const int slot = atomicAdd(&hist[map.digit(key[j])], 1);
        if (slot < end - begin) {                                                // always true: counted above
          if (staged) { stage_key[slot] = key[j]; stage_pos[slot] = t0 + j; }
          else { bkey[slot] = key[j]; bpos[slot] = t0 + j; }
        }
      }
    }
  }
  if (staged) {                                  // the list leaves LDS in order: whole cache lines per wave
    __syncthreads();
    const int cnt = end - begin;
    if ((((size_t)h * p.n) & 3) == 0) {
      for (int i = (int)threadIdx.x * 4; i < cnt; i += BT * 4) {
        if (i + 4 <= cnt) {
          *reinterpret_cast<uint4*>(bkey + i) = *reinterpret_cast<const uint4*>(stage_key + i);
          *reinterpret_cast<int4*>(bpos + i) = *reinterpret_cast<const int4*>(stage_pos + i);
        } else {
          for (int j = i; j < cnt; ++j) { bkey[j] = stage_key[j]; bpos[j] = stage_pos[j]; }
        }
      }
    } else {
      for (int i = threadIdx.x; i < cnt; i += BT) { bkey[i] = stage_key[i]; bpos[i] = stage_pos[i]; }
    }
  }
}

// ---------------------------------------------------------------------------
// radix select shared by the two selecting kernels
// ---------------------------------------------------------------------------
enum { ROW_PICK1 = 0, ROW_PICK2, ROW_GT, ROW_EQ, ROW_EMIT0, ROW_EMIT1, ROW_TABLE, ROW_COUNT };

struct SelectShared {
  __align__(16) int hist[3][kBins];      // digits of levels 1 and 2 of a select, and one for the caller; zeroed at the start
  int row[ROW_COUNT][SW];                // per-wave terms of the workgroup-wide sums, one row per use
  int pick[3][4];                        // per level: digit, #(digit above it), count of its bin (and the first level's group of eight bins)
  int coarse[ST + 1];                    // first step of the leading digit: sums at every eighth bin
  int seg_first[kMaxChunks], seg_count[kMaxChunks], seg_start[kMaxChunks];   // per chunk: where the keys with the chosen
                                         // leading digit sit, how many, and how many in earlier chunks
  int overflow;                          // a wave found more candidates than it can keep
};

__device__ __forceinline__ void select_shared_init(SelectShared& sh) {
  int* h = &sh.hist[0][0];
  for (int i = threadIdx.x; i < 3 * kBins; i += ST) h[i] = 0;
  if (threadIdx.x == 0) sh.overflow = 0;
}

// Leading digit of the k-th largest key from the D tables of a head's chunks: summed over the
// chunks, S[b] = #(digit >= b) falls from the key count at b = 0 to 0 at b = 2048, and the digit is
// the one bin with S[b+1] < k <= S[b].  Two steps, because what this costs is load instructions:
// thread t first sums only the entry at the low end of its eight bins (b = 2040 - 8t) over the
// chunks; the entry above its bins is its neighbour's sum, and one thread finds k between the two.
// Then one wave reads that thread's eight entries of every chunk (one 16-byte load per chunk and
// lane) and sums them across lanes.  Every thread gets the digit, #(digit above it) and the count
// of its bin.  prefetch() is called once the first loads are out, so that the caller's own first
// loads travel with them.
template <typename Prefetch>
__device__ __forceinline__ void pick_leading_digit(const uint16_t* tables, int n_parts, int k, SelectShared& sh, Prefetch prefetch,
                                                   int& digit, int& above, int& count) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int lo = kBins - 8 - 8 * (int)threadIdx.x;
  int s_lo = 0;
  bool first = true;
  constexpr int kInFlight = 16;                 // chunks requested together: one trip to memory for up to 16 of them
  for (int c = 0; c < n_parts; c += kInFlight) {
    uint16_t e[kInFlight];
#pragma unroll
    for (int u = 0; u < kInFlight; ++u) e[u] = tables[(size_t)min(c + u, n_parts - 1) * kTableStride + lo];
    if (first) { prefetch(); first = false; }
#pragma unroll
    for (int u = 0; u < kInFlight; ++u)
      if (c + u < n_parts) s_lo += (int)e[u];
  }
  sh.coarse[threadIdx.x + 1] = s_lo;            // coarse[t + 1] = S[2040 - 8t]; coarse[0] = S[2048] = 0
  if (threadIdx.x == 0) { sh.coarse[0] = 0; sh.pick[0][3] = 0; }    // no bracket (k outside the counts): the second step still reads inside the tables
  __syncthreads();
  const int s_hi = sh.coarse[threadIdx.x];      // S at the bin above this thread's eight
  if (s_hi < k && k <= s_lo) { sh.pick[0][3] = lo; sh.pick[0][1] = s_hi; }
  __syncthreads();
  if (wave == 0) {
    const int at = sh.pick[0][3];
    int S[9];
#pragma unroll
    for (int j = 0; j < 8; ++j) S[j] = 0;
    for (int c = lane; c < n_parts; c += kWave) {
      const uint4 v = *reinterpret_cast<const uint4*>(tables + (size_t)c * kTableStride + at);
      const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
      for (int q = 0; q < 4; ++q) { S[2 * q] += (int)(w[q] & 0xffffu); S[2 * q + 1] += (int)(w[q] >> 16); }
    }
#pragma unroll
    for (int j = 0; j < 8; ++j)
#pragma unroll
      for (int o = 32; o > 0; o >>= 1) S[j] += __shfl_xor(S[j], o, kWave);
    S[8] = sh.pick[0][1];
    if (lane == 0) {
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        if (S[j + 1] < k && k <= S[j]) {
          sh.pick[0][0] = at + j;
          sh.pick[0][1] = S[j + 1];
          sh.pick[0][2] = S[j] - S[j + 1];
        }
      }
    }
  }
  __syncthreads();
  digit = sh.pick[0][0];
  above = sh.pick[0][1];
  count = sh.pick[0][2];
}

// The digit d with #(digit > d) < remaining <= #(digit >= d) of an LDS histogram of counts
// (thread t owns bins 2040-8t .. 2047-8t).  level 1 or 2: which row / result slot to use.
__device__ __forceinline__ void pick_digit(const int* hist, int remaining, SelectShared& sh, int level, int& digit, int& above_out) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int lo = kBins - 8 - 8 * (int)threadIdx.x;
  const int4 a = *reinterpret_cast<const int4*>(hist + lo), b = *reinterpret_cast<const int4*>(hist + lo + 4);
  const int c[8] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};      // bins lo .. lo+7
  int tot = 0;
#pragma unroll
  for (int j = 0; j < 8; ++j) tot += c[j];
  const int incl = wave_incl_scan_dpp(tot);
  if (lane == 63) sh.row[ROW_PICK1 + level - 1][wave] = incl;
  __syncthreads();
  int before, total;
  wave_row_sums<SW>(sh.row[ROW_PICK1 + level - 1], wave, before, total);
  int above = incl - tot + before;                                  // keys in bins above this thread's
  if (above < remaining && remaining <= above + tot) {
#pragma unroll
    for (int j = 7; j >= 0; --j) {
      if (above < remaining && remaining <= above + c[j]) { sh.pick[level][0] = lo + j; sh.pick[level][1] = above; }
      above += c[j];
    }
  }
  __syncthreads();
  digit = sh.pick[level][0];
  above_out = sh.pick[level][1];
}

// The candidates of a select (keys that share the threshold's leading digit), each wave its own
// list in LDS.  Entries are appended either by the lanes that found one (`append_found`, inside
// uniform control flow) or as a dense run (`append_run`).
struct CandidateList {
  uint32_t* key;
  int32_t* pos;
  int n;                // appended so far by this wave (uniform); may exceed kWaveCand: then the list is not used
  bool shared = false;  // one list for the whole workgroup (n entries) instead of one per wave
  __device__ __forceinline__ void append_found(bool found, uint32_t k, int p, int lane, int* hist1) {
    const unsigned long long b = __ballot(found);
    if (b) {
      if (found) {
        const int at = n + __popcll(b & ((1ull << lane) - 1ull));
        if (at < kWaveCand) { key[at] = k; pos[at] = p; }
        atomicAdd(&hist1[(k >> 10) & 2047u], 1);
      }
      n += __popcll(b);
    }
  }
  __device__ __forceinline__ void append_run(bool valid, int n_valid, uint32_t k, int p, int lane, int* hist1) {
    if (valid) {
      const int at = n + lane;
      if (at < kWaveCand) { key[at] = k; pos[at] = p; }
      atomicAdd(&hist1[(k >> 10) & 2047u], 1);
    }
    n += n_valid;
  }
};

// The bits of the threshold below its leading digit, found on the candidates, and how many
// candidates at positions below `before` are above / equal to the threshold.  The candidates agree
// in every bit from `low_bits` up (`prefix` holds those bits; low_bits = 32, prefix = 0 for a bucket
// whose keys may differ anywhere); the bits below are taken at most 11 at a time from the top, one
// LDS histogram per step.  The first step's histogram, of first_digit(key, low_bits), is sh.hist[0],
// filled by the caller while it collected the candidates.  each_global(f) visits every candidate
// from memory (used when a wave's list overflowed).  Called by all threads after the candidates
// are in; starts with the barrier that publishes them.
__device__ __forceinline__ uint32_t first_digit(uint32_t key, int low_bits) {
  const int w = min(11, low_bits);
  return (key >> (low_bits - w)) & ((1u << w) - 1u);
}
template <typename GlobalEach>
__device__ __forceinline__ void finish_select(const CandidateList& list, GlobalEach each_global, uint32_t prefix, int low_bits,
                                              int remaining, int before, int gt, SelectShared& sh, uint32_t& thr, int& quota,
                                              int& base_gt, int& base_eq) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  if (!list.shared && list.n > kWaveCand && lane == 0) sh.overflow = 1;
  __syncthreads();
  const bool use_list = sh.overflow == 0;
  auto for_each_candidate = [&](auto f) {
    if (use_list) {
      const int first = list.shared ? (int)threadIdx.x : lane, step = list.shared ? ST : kWave;
      for (int i = first; i < list.n; i += step) f(list.key[i], list.pos[i]);
    } else {
      each_global(f);
    }
  };
  for (int step = 0;; ++step) {
    int* hist = sh.hist[step & 1];
    int d, above;
    pick_digit(hist, remaining, sh, 1 + (step & 1), d, above);
    remaining -= above;
    const int w = min(11, low_bits);
    low_bits -= w;
    prefix |= (uint32_t)d << low_bits;
    if (low_bits == 0) break;
    if (low_bits > 11) {                         // a third step follows the next one, in this histogram again
      for (int i = threadIdx.x; i < kBins; i += ST) hist[i] = 0;
    }
    int* next = sh.hist[(step + 1) & 1];
    const uint32_t known = prefix >> low_bits;   // low_bits <= 21 here
    const int lb = low_bits;
    for_each_candidate([&](uint32_t key, int) {
      if ((key >> lb) == known) atomicAdd(&next[first_digit(key, lb)], 1);
    });
    __syncthreads();
  }
  thr = prefix;
  quota = remaining;
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
  wave_row_sums<SW>(sh.row[ROW_GT], SW, unused, base_gt);
  wave_row_sums<SW>(sh.row[ROW_EQ], SW, unused, base_eq);
}

// Ordered pass over positions [begin, end) in tiles of kTile: a thread's EPT consecutive
// elements are classified by load_cls (2: above the threshold, 1: equal, 0: below or outside);
// emit(position, selected, rank among the selected) is called for every element inside.
// Equal elements are selected while fewer than `quota` earlier ones exist.  The two running
// counts of a thread travel through one scan packed as (greater << 16) | equal (a tile has
// 1024 elements, so neither half overflows).
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
    wave_row_sums<SW>(sh.row[ROW_EMIT0 + buf], wave, pre, tile_tot);
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

struct RouteParams;
struct RouteParams {
  const float* score; const float* eps;
  int n, n_pool, n_approx, n_heads;
  int chunk_tokens, n_chunks;      // selection by score: tokens per workgroup
  int slice, n_slices;             // selection by residual: pool entries per workgroup
  int pool_stride;                 // entries between the pool lists of two heads (a multiple of 4)
  const uint16_t* table0;          // [H, C, kTableStride] leading digits of the score keys
  const uint32_t* bkey;            // [H, n] score keys grouped by leading digit, chunk by chunk
  const int32_t* bpos;
  uint16_t* table1;                // [H, C, kTableStride] leading digits of the residual keys of pool members
  uint8_t* tier; int32_t* idx_retain; int32_t* idx_approx;
  int32_t* pool_idx; uint32_t* pool_key;
  const uint32_t* map;             // [H, 2]: the digit map (lowq, shift) of the head's score buckets
  const RouteParams* seq_table;        // RAGGED launches: the sequences' parameter blocks, seq_hps heads each
  int seq_hps;
};

// Step 1: the pool is the n_pool tokens of highest score
template <bool RAGGED>
__global__ __launch_bounds__(ST) void route_pool_kernel(RouteParams p) {
  int h = blockIdx.y;
  take_sequence<RAGGED>(p, h);
  if (RAGGED && (int)blockIdx.x >= p.n_chunks) return;
  __shared__ SelectShared sh;
  extern __shared__ __align__(16) unsigned char dyn_lds[];
  const int chunk = blockIdx.x;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const float* sc = p.score + (size_t)h * p.n;
  const float* ep = p.eps + (size_t)h * p.n;
  const int n = p.n;
  VEC_TRACE(0);
  select_shared_init(sh);
  // how the bucket launch cut the keys into leading digits
  DigitMap map = {p.map[2 * h], min((int)p.map[2 * h + 1], 21)};
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
  const int begin = chunk * p.chunk_tokens, end = min(n, begin + p.chunk_tokens);
  // this thread's tokens of the chunk's first two tiles: requested with the tables, used by the ordered pass
  const int first_i0 = begin + (int)threadIdx.x * EPT;
  float sc0[2][EPT], ep0[2][EPT];
  int d0, above0, m0;
  const uint16_t* tables = p.table0 + (size_t)h * p.n_chunks * kTableStride;
  pick_leading_digit(tables, p.n_chunks, p.n_pool, sh,
                     [&]() {
#pragma unroll
                       for (int u = 0; u < 2; ++u) { load_f4(sc, first_i0 + u * kTile, sc0[u]); load_f4(ep, first_i0 + u * kTile, ep0[u]); }
                     },
                     d0, above0, m0);
  VEC_TRACE(1);
  // where every chunk keeps its keys of digit d0: after the D[d0+1] keys of higher digits
  if (wave == 0) {                               // n_chunks <= 32: one lane per chunk
    int hi = 0, cnt = 0;
    if (lane < p.n_chunks) {
      const uint16_t* t = tables + (size_t)lane * kTableStride;
      hi = t[d0 + 1];
      cnt = (int)t[d0] - hi;
    }
    const int incl = wave_incl_scan_dpp(cnt);
    if (lane < p.n_chunks) { sh.seg_first[lane] = hi; sh.seg_count[lane] = cnt; sh.seg_start[lane] = incl - cnt; }
  }
  __syncthreads();
  VEC_TRACE(2);
  // Candidates: a group of threads per chunk reads that chunk's piece, kBatch loads in flight per
  // thread; candidate number = pieces of earlier chunks + place in the piece, which is also its
  // slot in the one list the waves then share out.  Keys above the digit in earlier chunks are
  // all selected.
  uint32_t* cand_key = reinterpret_cast<uint32_t*>(dyn_lds);
  int32_t* cand_pos = reinterpret_cast<int32_t*>(dyn_lds) + kCandCap;
  const uint32_t* bkey = p.bkey + (size_t)h * n;
  const int32_t* bpos = p.bpos + (size_t)h * n;
  int gt = 0;
  for (int c = 0; c < p.n_chunks; ++c)
    if (c < chunk && threadIdx.x == 0) gt += sh.seg_first[c];
  int groups = 1;
  while (groups < p.n_chunks) groups *= 2;
  const int tpc = ST / groups;                   // threads per chunk (at least 8)
  const int my_c = (int)threadIdx.x / tpc, my_sub = (int)threadIdx.x % tpc;
  const bool fits = m0 <= kCandCap;
  // what the candidates already agree on: everything above the digit's 2^shift keys, or nothing
  const bool high_shared = map.shares_high_bits(d0);
  const int low_bits = high_shared ? map.shift : 32;
  const uint32_t prefix = high_shared ? ((uint32_t)d0 + map.lowq) << map.shift : 0u;
  // More candidates than LDS holds usually means a plateau: scores that are all the same number (the
  // zeros of attention rows that underflow, a constant fill).  One look at the keys tells; then the
  // threshold is that number, and which of the equal tokens get in follows from the counts alone.
  bool plateau = false;
  uint32_t plateau_key = 0u;
  if (!fits) {
    uint32_t kmin = 0xffffffffu, kmax = 0u;
    const int cnt = my_c < p.n_chunks ? sh.seg_count[my_c] : 0;
    const int src0 = my_c < p.n_chunks ? my_c * p.chunk_tokens + sh.seg_first[my_c] : 0;
    for (int i0 = 0; i0 < cnt; i0 += tpc * kBatch) {
      uint32_t ck[kBatch];
#pragma unroll
      for (int u = 0; u < kBatch; ++u) ck[u] = bkey[src0 + min(i0 + u * tpc + my_sub, cnt - 1)];
#pragma unroll
      for (int u = 0; u < kBatch; ++u) { kmin = min(kmin, ck[u]); kmax = max(kmax, ck[u]); }
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
      kmin = min(kmin, (uint32_t)__shfl_xor((int)kmin, o, kWave));
      kmax = max(kmax, (uint32_t)__shfl_xor((int)kmax, o, kWave));
    }
    if (lane == 0) { sh.row[ROW_GT][wave] = (int)kmin; sh.row[ROW_EQ][wave] = (int)kmax; }
    __syncthreads();
#pragma unroll
    for (int q = 0; q < SW; ++q) { kmin = min(kmin, (uint32_t)sh.row[ROW_GT][q]); kmax = max(kmax, (uint32_t)sh.row[ROW_EQ][q]); }
    plateau = kmin == kmax;
    plateau_key = kmin;
    __syncthreads();                               // the rows are used again below
  }
  if (!plateau) {
    const bool live = my_c < p.n_chunks;
    const int cnt = live ? sh.seg_count[my_c] : 0;
    const int src0 = live ? my_c * p.chunk_tokens + sh.seg_first[my_c] : 0;
    const int dst0 = live ? sh.seg_start[my_c] : 0;
    for (int i0 = 0; i0 < cnt; i0 += tpc * kBatch) {
      uint32_t ck[kBatch];
      int cp[kBatch];
#pragma unroll
      for (int u = 0; u < kBatch; ++u) {
        const int i = min(i0 + u * tpc + my_sub, cnt - 1);
        ck[u] = bkey[src0 + i];
        cp[u] = bpos[src0 + i];
      }
#pragma unroll
      for (int u = 0; u < kBatch; ++u) {
        const int i = i0 + u * tpc + my_sub;
        if (i < cnt) {
          if (fits) { cand_key[dst0 + i] = ck[u]; cand_pos[dst0 + i] = cp[u]; }
          atomicAdd(&sh.hist[0][first_digit(ck[u], low_bits)], 1);
        }
      }
    }
  }
  if (!fits && threadIdx.x == 0) sh.overflow = 1;
  CandidateList list;                            // every wave a share of the one list
  list.key = cand_key;
  list.pos = cand_pos;
  list.n = fits ? m0 : kWaveCand + 1;
  list.shared = true;
  VEC_TRACE(3);
  uint32_t thr;
  int quota, base_gt, base_eq;
  if (plateau) {                                   // uniform
    thr = plateau_key;
    quota = p.n_pool - above0;                     // equal keys still to take, lowest token index first
    base_gt = 0;
    for (int c = 0; c < chunk; ++c) base_gt += sh.seg_first[c];
    base_eq = sh.seg_start[chunk];                 // the equal keys of earlier chunks come first
  } else {
    finish_select(
        list,
        [&](auto f) {
          const int cnt = my_c < p.n_chunks ? sh.seg_count[my_c] : 0;
          const int src0 = my_c < p.n_chunks ? my_c * p.chunk_tokens + sh.seg_first[my_c] : 0;
          for (int i = my_sub; i < cnt; i += tpc) f(bkey[src0 + i], bpos[src0 + i]);
        },
        prefix, low_bits, p.n_pool - above0, begin, gt, sh, thr, quota, base_gt, base_eq);
  }
  VEC_TRACE(4);

  // ordered pass over the chunk: tiers, pool list, leading digits of the residual keys
  uint8_t* tr = p.tier + (size_t)h * n;
  int32_t* pidx = p.pool_idx + (size_t)h * p.pool_stride;
  uint32_t* pkey = p.pool_key + (size_t)h * p.pool_stride;
  uint32_t ekey[EPT];
  ordered_emit(
      [&](int i0, int (&cls)[EPT]) {
        float x[EPT], e[EPT];
        if (i0 == first_i0 || i0 == first_i0 + kTile) {
          const int u = i0 == first_i0 ? 0 : 1;
#pragma unroll
          for (int j = 0; j < EPT; ++j) { x[j] = sc0[u][j]; e[j] = ep0[u][j]; }
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
  VEC_TRACE(5);
  __syncthreads();
  counts_to_table<ST>(sh.hist[2], p.table1 + ((size_t)h * p.n_chunks + chunk) * kTableStride, sh.row[ROW_TABLE]);
  VEC_TRACE(6);
}

// Step 3: inside the pool, the n_approx tokens of lowest residual lose their value
template <bool RAGGED>
__global__ __launch_bounds__(ST) void route_split_kernel(RouteParams p) {
  int h = blockIdx.y;
  take_sequence<RAGGED>(p, h);
  if (RAGGED && (int)blockIdx.x >= p.n_slices) return;
  __shared__ SelectShared sh;
  extern __shared__ __align__(16) unsigned char dyn_lds[];
  const int slice = blockIdx.x;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int m = p.n_pool;
  const int32_t* pidx = p.pool_idx + (size_t)h * p.pool_stride;
  const uint32_t* pkey = p.pool_key + (size_t)h * p.pool_stride;
  uint8_t* tr = p.tier + (size_t)h * p.n;
  int32_t* ir = p.idx_retain + (size_t)h * (p.n_pool - p.n_approx);
  int32_t* ia = p.idx_approx + (size_t)h * p.n_approx;
  const int begin = slice * p.slice, end = min(m, begin + p.slice);
  if (p.n_approx == 0) {
    for (int i = begin + (int)threadIdx.x; i < end; i += ST) ir[i] = pidx[i];
    return;
  }
  VEC_TRACE(16);
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
  const int n_tiles = (m + kTile - 1) / kTile;
  uint32_t cur[kBatch][EPT];
  auto load_batch = [&](int tb, uint32_t (&key)[kBatch][EPT]) {
#pragma unroll
    for (int u = 0; u < kBatch; ++u) {
      if (tb + u < n_tiles) {
        load_u4(pkey, (tb + u) * kTile + (int)threadIdx.x * EPT, key[u]);
      } else {
#pragma unroll
        for (int j = 0; j < EPT; ++j) key[u][j] = 0u;
      }
    }
  };
  // this thread's entries of the slice's first tile: requested with the tables, used by the ordered pass
  const int first_i0 = begin + (int)threadIdx.x * EPT;
  uint32_t key0[EPT], tok0[EPT];
  int d0, above0, m0;
  pick_leading_digit(p.table1 + (size_t)h * p.n_chunks * kTableStride, p.n_chunks, p.n_approx, sh,
                     [&]() {
                       load_batch(0, cur);
                       load_u4(pkey, first_i0, key0);
                       load_u4(reinterpret_cast<const uint32_t*>(pidx), first_i0, tok0);
                     },
                     d0, above0, m0);
  VEC_TRACE(17);
  // all keys of the pool once: candidates into this wave's list, earlier keys above the digit counted
  CandidateList list;
  list.key = reinterpret_cast<uint32_t*>(dyn_lds) + wave * kWaveCand;
  list.pos = reinterpret_cast<int32_t*>(dyn_lds) + kCandCap + wave * kWaveCand;
  list.n = 0;
  list.shared = false;
  int gt = 0;
  for (int tb = 0; tb < n_tiles; tb += kBatch) {
    uint32_t nxt[kBatch][EPT];
    const bool more = tb + kBatch < n_tiles;
    if (more) load_batch(tb + kBatch, nxt);          // requested before this batch is worked on
#pragma unroll
    for (int u = 0; u < kBatch; ++u) {
      if (tb + u < n_tiles) {                        // uniform
        const int i0 = (tb + u) * kTile + (int)threadIdx.x * EPT;
#pragma unroll
        for (int j = 0; j < EPT; ++j) {
          const bool ok = i0 + j < m;
          const int dg = (int)(cur[u][j] >> 21);
          gt += ok && i0 + j < begin && dg > d0;
          list.append_found(ok && dg == d0, cur[u][j], i0 + j, lane, sh.hist[0]);
        }
      }
    }
    if (more) {
#pragma unroll
      for (int u = 0; u < kBatch; ++u)
#pragma unroll
        for (int j = 0; j < EPT; ++j) cur[u][j] = nxt[u][j];
    }
  }
  VEC_TRACE(18);
  uint32_t thr;
  int quota, base_gt, base_eq;
  finish_select(
      list,
      [&](auto f) {
        for (int t = 0; t < n_tiles; ++t) {
          uint32_t key[EPT];
          const int i0 = t * kTile + (int)threadIdx.x * EPT;
          load_u4(pkey, i0, key);
#pragma unroll
          for (int j = 0; j < EPT; ++j)
            if (i0 + j < m && (int)(key[j] >> 21) == d0) f(key[j], i0 + j);
        }
      },
      (uint32_t)d0 << 21, 21, p.n_approx - above0, begin, gt, sh, thr, quota, base_gt, base_eq);
  VEC_TRACE(19);
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
  VEC_TRACE(20);
}

// nothing is kept: every token is evicted
__global__ __launch_bounds__(256) void route_evict_all_kernel(uint8_t* __restrict__ tier, size_t total) {
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < total) tier[i] = VECTOR_TIER_EVICT;
}

// ---------------------------------------------------------------------------
// compaction: one 16-byte piece per thread, P pieces per row
// ---------------------------------------------------------------------------
struct GatherParams;
struct GatherParams {
  const unsigned char* k; const unsigned char* v;
  int64_t k_sh, k_st, v_sh, v_st;          // byte strides
  int hps;                                 // stacked sequences: KV heads per sequence (0: one sequence)
  int64_t k_sb, v_sb;                      // byte strides between sequences
  const int32_t* idx_retain; const int32_t* idx_approx;
  int n_retain, n_approx, cap_retain, row_bytes, n;
  unsigned char* k_ret; unsigned char* v_ret; unsigned char* k_apx;
  const GatherParams* seq_table;               // RAGGED launches: the sequences' parameter blocks, seq_hps heads each
  int seq_hps;
};

template <bool RAGGED>
__global__ __launch_bounds__(256) void gather_rows_kernel(GatherParams p) {
  int h = blockIdx.y;
  take_sequence<RAGGED>(p, h);
  const int seg = blockIdx.z;                       // seg 0: k_ret, 1: v_ret, 2: k_apx
  const int pieces = p.row_bytes / 16;
  const int rows = (seg == 2) ? p.n_approx : p.n_retain;
  const int64_t gid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int row = (int)(gid / pieces), piece = (int)(gid - (int64_t)row * pieces);
  if (row >= rows) return;
  const int32_t* idx = (seg == 2) ? p.idx_approx + (size_t)h * p.n_approx : p.idx_retain + (size_t)h * p.n_retain;
  int tok = idx[row];
  tok = min(max(tok, 0), p.n - 1);                  // an index list is trusted, but never walk out of the tensor
  const int64_t hs = p.hps ? h / p.hps : 0, hh = p.hps ? h % p.hps : h;      // sequence and KV head of the launch head
  const unsigned char* src = (seg == 1) ? p.v + hs * p.v_sb + hh * p.v_sh + (int64_t)tok * p.v_st
                                        : p.k + hs * p.k_sb + hh * p.k_sh + (int64_t)tok * p.k_st;
  unsigned char* dst = (seg == 0) ? p.k_ret + ((size_t)h * p.cap_retain + row) * p.row_bytes
                     : (seg == 1) ? p.v_ret + ((size_t)h * p.cap_retain + row) * p.row_bytes
                                  : p.k_apx + ((size_t)h * p.n_approx + row) * p.row_bytes;
  *reinterpret_cast<uint4*>(dst + piece * 16) = *reinterpret_cast<const uint4*>(src + piece * 16);
}

}  // namespace

// ---------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------
static int route_chunk_tokens(int seq_len) {
  int ch = kMinChunk;
  while ((seq_len + ch - 1) / ch > kMaxChunks) ch *= 2;
  return ch;
}

namespace {
struct RouteLayout {
  int chunk_tokens, n_chunks, pool_stride;
  size_t off_map, off_range, off_table0, off_table1, off_bkey, off_bpos, off_idx, off_key, total;
};
RouteLayout route_layout(int n_kv_heads, int seq_len, int n_pool) {
  RouteLayout L;
  L.chunk_tokens = route_chunk_tokens(seq_len);
  L.n_chunks = (seq_len + L.chunk_tokens - 1) / L.chunk_tokens;
  L.pool_stride = (n_pool + 3) / 4 * 4;
  const size_t tables = align_up((size_t)n_kv_heads * L.n_chunks * kTableStride * sizeof(uint16_t), 256);
  const size_t per_token = align_up((size_t)n_kv_heads * seq_len * sizeof(uint32_t), 256);
  const size_t per_pool = align_up((size_t)n_kv_heads * L.pool_stride * sizeof(uint32_t), 256);
  size_t off = 0;
  L.off_map = off;    off += align_up((size_t)n_kv_heads * 2 * sizeof(uint32_t), 256);
  L.off_range = off;  off += align_up((size_t)n_kv_heads * route_mass_range_slots(seq_len) * sizeof(float4), 256);
  L.off_table0 = off; off += tables;
  L.off_table1 = off; off += tables;
  L.off_bkey = off;   off += per_token;
  L.off_bpos = off;   off += per_token;
  L.off_idx = off;    off += per_pool;
  L.off_key = off;    off += per_pool;
  L.total = off;
  return L;
}

void fill_bucket_params(BucketParams& bp, const RouteLayout& L, void* route_ws) {
  unsigned char* w8 = reinterpret_cast<unsigned char*>(route_ws);
  bp.table = w8 ? reinterpret_cast<uint16_t*>(w8 + L.off_table0) : nullptr;
  bp.bkey = w8 ? reinterpret_cast<uint32_t*>(w8 + L.off_bkey) : nullptr;
  bp.bpos = w8 ? reinterpret_cast<int32_t*>(w8 + L.off_bpos) : nullptr;
  bp.map = w8 ? reinterpret_cast<uint32_t*>(w8 + L.off_map) : nullptr;
  bp.range = w8 ? reinterpret_cast<const float4*>(w8 + L.off_range) : nullptr;
  bp.n_range = 0;
  bp.log_ref = 0.f;
  bp.seq_table = nullptr;
  bp.seq_hps = 0;
  bp.chunk_tokens = L.chunk_tokens;
  bp.n_chunks = L.n_chunks;
}
}  // namespace

size_t route_workspace_bytes(int n_kv_heads, int seq_len, int n_pool) { return route_layout(n_kv_heads, seq_len, n_pool).total; }

// the scorer's second pass runs at least 512 tokens per workgroup
int route_mass_range_slots(int seq_len) { return (seq_len + 511) / 512; }
void* route_mass_range(void* route_ws, int n_kv_heads) {
  return reinterpret_cast<unsigned char*>(route_ws) + route_layout(n_kv_heads, 1, 0).off_range;
}

namespace {
BucketParams pool_bucket_params(const float* mass, float* score, int n_kv_heads, int seq_len, int n_prefix, int pool_kernel,
                                int pool_mode, void* route_ws, int n_range, RouteLayout& L) {
  L = route_layout(n_kv_heads, seq_len, 0);      // the bucket areas do not depend on the pool size
  BucketParams bp;
  bp.src = mass; bp.score = score; bp.n = seq_len; bp.n_prefix = n_prefix; bp.kernel = pool_kernel; bp.take_max = pool_mode == VECTOR_POOL_MAX;
  fill_bucket_params(bp, L, route_ws);
  bp.n_range = route_ws ? n_range : 0;
  bp.log_ref = -log2f((float)(n_prefix > 0 ? n_prefix : 1));     // as in the scorer's second pass
  return bp;
}

RouteParams route_params(int n_kv_heads, int seq_len, const float* score, const float* eps, int n_pool, int n_approx, uint8_t* tier,
                         int32_t* idx_retain, int32_t* idx_approx, void* ws, RouteLayout& L) {
  L = route_layout(n_kv_heads, seq_len, n_pool);
  unsigned char* w8 = reinterpret_cast<unsigned char*>(ws);
  RouteParams p;
  p.score = score; p.eps = eps; p.n = seq_len; p.n_pool = n_pool; p.n_approx = n_approx; p.n_heads = n_kv_heads;
  p.chunk_tokens = L.chunk_tokens; p.n_chunks = L.n_chunks; p.pool_stride = L.pool_stride;
  p.slice = kTile;
  while ((n_pool + p.slice - 1) / p.slice > kMaxChunks) p.slice *= 2;
  p.n_slices = (n_pool + p.slice - 1) / p.slice;
  p.map = reinterpret_cast<const uint32_t*>(w8 + L.off_map);
  p.table0 = reinterpret_cast<uint16_t*>(w8 + L.off_table0);
  p.table1 = reinterpret_cast<uint16_t*>(w8 + L.off_table1);
  p.bkey = reinterpret_cast<uint32_t*>(w8 + L.off_bkey);
  p.bpos = reinterpret_cast<int32_t*>(w8 + L.off_bpos);
  p.pool_idx = reinterpret_cast<int32_t*>(w8 + L.off_idx);
  p.pool_key = reinterpret_cast<uint32_t*>(w8 + L.off_key);
  p.tier = tier; p.idx_retain = idx_retain; p.idx_approx = idx_approx;
  p.seq_table = nullptr; p.seq_hps = 0;
  return p;
}

GatherParams gather_params(const vector_shape& s, const void* k, const void* v, const int32_t* idx_retain, const int32_t* idx_approx,
                           int n_retain, int n_approx, void* k_ret, void* v_ret, void* k_apx, int cap_retain, const SeqStack* stack) {
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
  p.hps = stack ? stack->heads_per_seq : 0;
  p.k_sb = stack ? stack->k_stride_seq * esz : 0;
  p.v_sb = stack ? stack->v_stride_seq * esz : 0;
  p.idx_retain = idx_retain; p.idx_approx = idx_approx;
  p.n_retain = n_retain; p.n_approx = n_approx; p.cap_retain = cap_retain;
  p.row_bytes = s.head_dim * esz; p.n = s.seq_len;
  p.k_ret = reinterpret_cast<unsigned char*>(k_ret);
  p.v_ret = reinterpret_cast<unsigned char*>(v_ret);
  p.k_apx = reinterpret_cast<unsigned char*>(k_apx);
  p.seq_table = nullptr; p.seq_hps = 0;
  return p;
}

unsigned gather_grid_x(const GatherParams& p) {
  const int pieces = p.row_bytes / 16;
  const int max_rows = p.n_retain > p.n_approx ? p.n_retain : p.n_approx;
  return (unsigned)(((int64_t)max_rows * pieces + 255) / 256);
}
constexpr size_t kSelectLds = (size_t)kCandCap * 8;
}  // namespace

int launch_pool_scores(const float* mass, float* score, int n_kv_heads, int seq_len, int n_prefix, int pool_kernel, int pool_mode,
                       void* route_ws, int n_range, hipStream_t stream) {
  if (n_range < 0 || n_range > route_mass_range_slots(seq_len)) return VECTOR_ERR_ARG;
  RouteLayout L;
  const BucketParams bp = pool_bucket_params(mass, score, n_kv_heads, seq_len, n_prefix, pool_kernel, pool_mode, route_ws, n_range, L);
  VEC_LAUNCH(K_POOL, route_bucket_kernel<true>, dim3(L.n_chunks, n_kv_heads), dim3(BT), 0, stream, bp);
  VEC_HIP(hipGetLastError());
  return VECTOR_OK;
}

int launch_route(int n_kv_heads, int seq_len, const float* score, const float* eps, int n_pool, int n_approx,
                 uint8_t* tier, int32_t* idx_retain, int32_t* idx_approx, void* ws, bool have_buckets, hipStream_t stream) {
  if (n_pool == 0) {
    const size_t total = (size_t)n_kv_heads * seq_len;
    VEC_LAUNCH(K_ROUTE, route_evict_all_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, stream, tier, total);
    VEC_HIP(hipGetLastError());
    return VECTOR_OK;
  }
  RouteLayout L;
  const RouteParams p = route_params(n_kv_heads, seq_len, score, eps, n_pool, n_approx, tier, idx_retain, idx_approx, ws, L);
  VEC_HIP(set_max_lds(reinterpret_cast<const void*>(route_pool_kernel<false>), kSelectLds));
  VEC_HIP(set_max_lds(reinterpret_cast<const void*>(route_split_kernel<false>), kSelectLds));
  const bool t_ = timing_enabled();
  if (t_) timing_begin(K_ROUTE, stream);             // the launches count as one routing step
  if (!have_buckets) {
    BucketParams bp;
    bp.src = score; bp.score = nullptr; bp.n = seq_len; bp.n_prefix = seq_len; bp.kernel = 1; bp.take_max = 0;
    fill_bucket_params(bp, L, ws);
    hipLaunchKernelGGL(route_bucket_kernel<false>, dim3(L.n_chunks, n_kv_heads), dim3(BT), 0, stream, bp);
  }
  hipLaunchKernelGGL(route_pool_kernel<false>, dim3(L.n_chunks, n_kv_heads), dim3(ST), kSelectLds, stream, p);
  hipLaunchKernelGGL(route_split_kernel<false>, dim3(p.n_slices, n_kv_heads), dim3(ST), kSelectLds, stream, p);
  if (t_) timing_end(K_ROUTE, stream);
  VEC_HIP(hipGetLastError());
  return VECTOR_OK;
}

int launch_compact(const vector_shape& s, const void* k, const void* v, const int32_t* idx_retain,
                   const int32_t* idx_approx, int n_retain, int n_approx, void* k_ret, void* v_ret, void* k_apx,
                   int cap_retain, hipStream_t stream, const SeqStack* stack) {
  const GatherParams p = gather_params(s, k, v, idx_retain, idx_approx, n_retain, n_approx, k_ret, v_ret, k_apx, cap_retain, stack);
  const unsigned gx = gather_grid_x(p);
  if (gx == 0) return VECTOR_OK;
  VEC_LAUNCH(K_GATHER, gather_rows_kernel<false>, dim3(gx, s.n_kv_heads, 3), dim3(256), 0, stream, p);
  VEC_HIP(hipGetLastError());
  return VECTOR_OK;
}

// ---------------------------------------------------------------------------
// several sequences of different lengths in one set of launches
// ---------------------------------------------------------------------------
size_t route_ragged_table_bytes(int count) {
  return align_up(sizeof(BucketParams) * count, 256) + align_up(sizeof(RouteParams) * count, 256) +
         align_up(sizeof(GatherParams) * count, 256);
}

int launch_pool_scores_ragged(const PoolSeq* seqs, int count, int n_kv_heads, int pool_kernel, int pool_mode, void* tables,
                              hipStream_t stream) {
  if (count < 1 || count > kMaxRaggedSeqs) return VECTOR_ERR_ARG;
  BucketParams host[kMaxRaggedSeqs];
  unsigned gx = 0;
  for (int b = 0; b < count; ++b) {
    if (!seqs[b].route_ws || seqs[b].n_range < 0 || seqs[b].n_range > route_mass_range_slots(seqs[b].seq_len)) return VECTOR_ERR_ARG;
    RouteLayout L;
    host[b] = pool_bucket_params(seqs[b].mass, seqs[b].score, n_kv_heads, seqs[b].seq_len, seqs[b].n_prefix, pool_kernel, pool_mode,
                                 seqs[b].route_ws, seqs[b].n_range, L);
    if ((unsigned)L.n_chunks > gx) gx = (unsigned)L.n_chunks;
  }
  const int rc = upload_table(host, sizeof(BucketParams) * count, tables, stream);
  if (rc != VECTOR_OK) return rc;
  BucketParams lp = host[0];
  lp.seq_table = reinterpret_cast<const BucketParams*>(tables);
  lp.seq_hps = n_kv_heads;
  auto kernel = route_bucket_kernel<true, true>;
  VEC_LAUNCH(K_POOL, kernel, dim3(gx, (unsigned)count * n_kv_heads), dim3(BT), 0, stream, lp);
  VEC_HIP(hipGetLastError());
  return VECTOR_OK;
}

int launch_route_compact_ragged(const vector_shape& s, const RaggedSeq* seqs, int count, void* tables, hipStream_t stream) {
  if (count < 1 || count > kMaxRaggedSeqs) return VECTOR_ERR_ARG;
  RouteParams rhost[kMaxRaggedSeqs];
  GatherParams ghost[kMaxRaggedSeqs];
  unsigned g_pool = 0, g_split = 0, g_gather = 0;
  for (int b = 0; b < count; ++b) {
    const RaggedSeq& q = seqs[b];
    if (q.n_pool < 1) return VECTOR_ERR_ARG;               // nothing kept: that sequence goes through launch_route on its own
    RouteLayout L;
    rhost[b] = route_params(s.n_kv_heads, q.shape.seq_len, q.score, q.eps, q.n_pool, q.n_approx, q.tier, q.idx_retain, q.idx_approx,
                            q.route_ws, L);
    ghost[b] = gather_params(q.shape, q.k, q.v, q.idx_retain, q.idx_approx, q.n_pool - q.n_approx, q.n_approx, q.k_ret, q.v_ret, q.k_apx,
                             q.cap_retain, nullptr);
    if ((unsigned)rhost[b].n_chunks > g_pool) g_pool = (unsigned)rhost[b].n_chunks;
    if ((unsigned)rhost[b].n_slices > g_split) g_split = (unsigned)rhost[b].n_slices;
    const unsigned gg = gather_grid_x(ghost[b]);
    if (gg > g_gather) g_gather = gg;
  }
  unsigned char* t8 = reinterpret_cast<unsigned char*>(tables) + align_up(sizeof(BucketParams) * count, 256);
  unsigned char* rt = t8;
  unsigned char* gt = t8 + align_up(sizeof(RouteParams) * count, 256);
  int rc = upload_table(rhost, sizeof(RouteParams) * count, rt, stream);
  if (rc == VECTOR_OK) rc = upload_table(ghost, sizeof(GatherParams) * count, gt, stream);
  if (rc != VECTOR_OK) return rc;
  RouteParams rp = rhost[0];
  rp.seq_table = reinterpret_cast<const RouteParams*>(rt);
  rp.seq_hps = s.n_kv_heads;
  GatherParams gp = ghost[0];
  gp.seq_table = reinterpret_cast<const GatherParams*>(gt);
  gp.seq_hps = s.n_kv_heads;
  const unsigned heads = (unsigned)count * s.n_kv_heads;
  VEC_HIP(set_max_lds(reinterpret_cast<const void*>(route_pool_kernel<true>), kSelectLds));
  VEC_HIP(set_max_lds(reinterpret_cast<const void*>(route_split_kernel<true>), kSelectLds));
  const bool t_ = timing_enabled();
  if (t_) timing_begin(K_ROUTE, stream);
  hipLaunchKernelGGL(route_pool_kernel<true>, dim3(g_pool, heads), dim3(ST), kSelectLds, stream, rp);
  hipLaunchKernelGGL(route_split_kernel<true>, dim3(g_split, heads), dim3(ST), kSelectLds, stream, rp);
  if (t_) timing_end(K_ROUTE, stream);
  VEC_HIP(hipGetLastError());
  if (g_gather > 0) {
    VEC_LAUNCH(K_GATHER, gather_rows_kernel<true>, dim3(g_gather, heads, 3), dim3(256), 0, stream, gp);
    VEC_HIP(hipGetLastError());
  }
  return VECTOR_OK;
}

// ---------------------------------------------------------------------------
// parameter tables: host bytes to device memory as the arguments of small copy launches
// ---------------------------------------------------------------------------
namespace {
constexpr int kBlobBytes = 3584;
struct Blob { uint4 w[kBlobBytes / 16]; };
__global__ __launch_bounds__(256) void table_copy_kernel(Blob blob, uint4* dst, int words) {
  for (int i = threadIdx.x; i < words; i += 256) dst[i] = blob.w[i];
}
}  // namespace

int upload_table(const void* host, size_t bytes, void* dev, hipStream_t stream) {
  if (!host || !dev || (reinterpret_cast<uintptr_t>(dev) & 15u)) return VECTOR_ERR_ARG;
  const unsigned char* src = reinterpret_cast<const unsigned char*>(host);
  unsigned char* dst = reinterpret_cast<unsigned char*>(dev);
  for (size_t off = 0; off < bytes; off += kBlobBytes) {
    const size_t part = bytes - off < (size_t)kBlobBytes ? bytes - off : (size_t)kBlobBytes;
    Blob blob;
    memset(&blob, 0, sizeof(blob));
    memcpy(&blob, src + off, part);
    hipLaunchKernelGGL(table_copy_kernel, dim3(1), dim3(256), 0, stream, blob, reinterpret_cast<uint4*>(dst + off), (int)((part + 15) / 16));
  }
  VEC_HIP(hipGetLastError());
  return VECTOR_OK;
}

}  // namespace vec
