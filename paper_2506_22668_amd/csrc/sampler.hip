// Coalition sampler: bit-packed mask rows, regression weights and sizes.
//
// Paper, "Distributed Subgraph Sampling": samples are rows of a k x n binary mask
// matrix, drawn non-uniformly by coalition size, every sample with its complement
// (only half of the rows need random numbers), sorted by size so that any range of
// pairs can be produced independently of the others.
//
// A row of size s is the set of the s columns with the smallest (key, column),
// where key(r, j) is word j%4 of Philox4x32-10 (Salmon et al., SC'11) under key =
// seed and counter = (j/4, r_lo, r_hi, tag). One workgroup builds one pair: it finds
// the s-th smallest (key, column) by a radix select over regenerated keys, then emits
// both rows with wave ballots. Usually two passes over the keys are enough: the first
// histograms the top 12 bits and, at the same time, keeps the keys whose top bits fall
// in a window around the expected position of the threshold (s/n of the key range,
// +- 3 standard deviations); if the threshold bin is inside the window the exact
// threshold comes from those kept keys. Otherwise two more passes refine it
// (next 12 bits by histogram, last 8 bits + column tie-break from a candidate list).
#include <math.h>
#include <stdlib.h>

#include "internal.h"

namespace {

constexpr int kThreads = 256;
constexpr int kBins = 4096;
constexpr int kCandMax = 2048;

__device__ __forceinline__ void philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                              uint32_t k0, uint32_t k1, uint32_t out[4]) {
  const uint32_t M0 = 0xD2511F53u, M1 = 0xCD9E8D57u;
#pragma unroll
  for (int r = 0; r < 10; ++r) {
    if (r > 0) {
      k0 += 0x9E3779B9u;
      k1 += 0xBB67AE85u;
    }
    // one 32 x 32 -> 64 multiply per product (as a high and a low multiply the generator ran 18 % slower)
    unsigned long long p0, p1;
    asm("v_mad_u64_u32 %0, vcc, %1, %2, 0" : "=v"(p0) : "v"(c0), "s"(M0) : "vcc");
    asm("v_mad_u64_u32 %0, vcc, %1, %2, 0" : "=v"(p1) : "v"(c2), "s"(M1) : "vcc");
    const uint32_t hi0 = (uint32_t)(p0 >> 32), lo0 = (uint32_t)p0, hi1 = (uint32_t)(p1 >> 32), lo1 = (uint32_t)p1;
    c0 = hi1 ^ c1 ^ k0;
    c1 = lo1;
    c2 = hi0 ^ c3 ^ k1;
    c3 = lo0;
  }
  out[0] = c0;
  out[1] = c1;
  out[2] = c2;
  out[3] = c3;
}

// Smallest bin whose inclusive prefix count reaches `want` (1-based rank); returns the bin and the
// count of elements in earlier bins. Whole block participates: every thread sums 16 bins, wave 0
// scans the 256 partial sums with shuffles, and one lane walks the at most 4 + 16 remaining entries.
__device__ void select_bin(const uint32_t* hist, uint32_t* part, uint32_t want, uint32_t* res) {
  const int t = threadIdx.x;
  constexpr int kPer = kBins / kThreads;  // 16
  uint32_t s = 0;
#pragma unroll
  for (int i = 0; i < kPer; ++i) s += hist[t * kPer + i];
  part[t] = s;
  __syncthreads();
  if (t < 64) {
    const uint32_t v0 = part[4 * t], v1 = part[4 * t + 1], v2 = part[4 * t + 2], v3 = part[4 * t + 3];
    const uint32_t v = v0 + v1 + v2 + v3;
    uint32_t incl = v;
    for (int o = 1; o < 64; o <<= 1) {
      const uint32_t up = __shfl_up(incl, o, 64);
      if (t >= o) incl += up;
    }
    const unsigned long long reach = __ballot(incl >= want);
    const int lane = reach ? __ffsll((long long)reach) - 1 : 63;  // the total always reaches `want`
    if (t == lane) {
      uint32_t cum = incl - v;
      int p = 4 * t;
      const uint32_t pv[4] = {v0, v1, v2, v3};
      int q = 0;
      while (q < 3 && cum + pv[q] < want) cum += pv[q++];
      p += q;
      int b = p * kPer;
      const int bend = b + kPer - 1;
      while (b < bend && cum + hist[b] < want) cum += hist[b++];
      res[0] = (uint32_t)b;
      res[1] = cum;
    }
  }
  __syncthreads();
}

struct SampleArgs {
  int64_t n, W, K, H;
  int64_t enum_upto;  // pairs of the size classes 1..enum_upto are the subsets in lexicographic order, not sampled
  int64_t pair_begin, pair_end;
  const int64_t* b;     // class boundaries [H+1]
  const float* wtab;    // [H+1]
  uint32_t seed_lo, seed_hi, tag;
  uint64_t* Z;
  float* w;
  int32_t* sz;
  int* error_flag;
  uint32_t window_cap;  // entries of the dynamic-LDS window list
  int32_t* retry;          // pairs the one-pass kernel hands to the multi-pass kernel (offsets from pair_begin), or null
  uint32_t* retry_count;
  // player lists of the sparse small members (one-pass kernel only; null: none). Pair r of a class s <= list_max
  // owns list[list_cum[s] + (r - b[s-1] - 1) * s ..][s]; list_offset[r] gets that offset once the list is complete
  uint32_t* list;
  const int64_t* list_cum;
  int64_t* list_offset;
  int64_t list_max;
};

__global__ __launch_bounds__(kThreads) void sample_pairs_kernel(SampleArgs a) {
  __shared__ uint32_t hist[kBins];
  __shared__ uint32_t part[kThreads];
  __shared__ uint32_t res[2];
  __shared__ unsigned long long cand[kCandMax];
  __shared__ uint32_t cand_count;
  __shared__ uint32_t window_count;
  __shared__ unsigned long long threshold;
  extern __shared__ unsigned long long window[];  // (key << 32 | column) of the keys near the expected threshold

  const int t = threadIdx.x;
  const int lane = t & 63, wave = t >> 6;
  const int64_t n = a.n, W = a.W;
  const int64_t nq = (n + 3) >> 2;
  const uint64_t tail_mask = (n & 63) ? ((1ull << (n & 63)) - 1ull) : ~0ull;

  const int64_t todo = a.retry ? (int64_t)*a.retry_count : a.pair_end - a.pair_begin;
  for (int64_t it = blockIdx.x; it < todo; it += gridDim.x) {
    const int64_t r = a.pair_begin + (a.retry ? (int64_t)a.retry[it] : it);
    uint64_t* row_small = a.Z + (2 * (r - a.pair_begin)) * W;
    uint64_t* row_big = row_small + W;
    if (r == 0) {  // (empty, full): the two constraint rows
      for (int64_t wd = t; wd < W; wd += kThreads) {
        row_small[wd] = 0ull;
        row_big[wd] = (wd == W - 1) ? tail_mask : ~0ull;
      }
      if (t == 0) {
        a.w[0] = 0.f;
        a.w[1] = 0.f;
        a.sz[0] = 0;
        a.sz[1] = (int32_t)n;
      }
      continue;
    }
    // size of the small member: s = min{s : b_s >= r}
    int64_t lo = 1, hi = a.H;
    while (lo < hi) {
      int64_t mid = (lo + hi) >> 1;
      if (a.b[mid] >= r) hi = mid; else lo = mid + 1;
    }
    const uint32_t s = (uint32_t)lo;
    if ((int64_t)s <= a.enum_upto) {
      // An enumerated class: pair r is the j-th s-subset of the players in lexicographic order, j = r - 1 - b_(s-1).
      // Unranking: with c = C(m, t) the number of subsets that continue with element x (m = n-1-x players after
      // x, t elements still to choose after it), skip x while j >= c. c follows x and t by exact integer updates:
      // C(m-1, t) = c (m-t) / m and C(m-1, t-1) = c t / m (c <= K, so the products stay below 2^63 for the sizes
      // the host admits).
      for (int64_t wd = t; wd < W; wd += kThreads) {
        row_small[wd] = 0ull;
        row_big[wd] = (wd == W - 1) ? tail_mask : ~0ull;
      }
      __syncthreads();
      if (t == 0) {
        int64_t j = r - 1 - a.b[s - 1];
        int64_t m = n - 1, tt = (int64_t)s - 1, x = 0;
        uint64_t c = 1;
        for (int64_t u = 1; u <= tt; ++u) c = c * (uint64_t)(m - tt + u) / (uint64_t)u;
        for (uint32_t i = 0; i < s; ++i) {
          while ((uint64_t)j >= c) {
            j -= (int64_t)c;
            c = c * (uint64_t)(m - tt) / (uint64_t)m;
            --m;
            ++x;
          }
          row_small[x >> 6] |= 1ull << (x & 63);
          row_big[x >> 6] &= ~(1ull << (x & 63));
          if (tt > 0) c = c * (uint64_t)tt / (uint64_t)m;
          --m;
          --tt;
          ++x;
        }
        const float wt = a.wtab[s];
        const int64_t o = 2 * (r - a.pair_begin);
        a.w[o] = wt;
        a.w[o + 1] = wt;
        a.sz[o] = (int32_t)s;
        a.sz[o + 1] = (int32_t)(n - s);
      }
      __syncthreads();
      continue;
    }
    const uint32_t r_lo = (uint32_t)r, r_hi = (uint32_t)((uint64_t)r >> 32);

    // window of top-12-bit bins around the expected position of the s-th smallest key
    uint32_t win_lo, win_hi;
    {
      const float fs = (float)s, fn = (float)n;
      const float sigma = sqrtf(fs * (fn - fs) / fn);  // of the number of keys below a fixed quantile
      const uint32_t pred = (uint32_t)(((uint64_t)s << 12) / (uint64_t)n);
      const uint32_t delta = 2u + (uint32_t)ceilf(3.0f * sigma * 4096.0f / fn);
      win_lo = pred > delta ? pred - delta : 0u;
      win_hi = pred + delta < (uint32_t)kBins - 1u ? pred + delta : (uint32_t)kBins - 1u;
    }
    // pass A: histogram of the top 12 key bits; keys in the window are kept
    for (int i = t; i < kBins; i += kThreads) hist[i] = 0;
    if (t == 0) {
      cand_count = 0;
      window_count = 0;
    }
    __syncthreads();
    for (int64_t q = t; q < nq; q += kThreads) {
      uint32_t key[4];
      philox4x32_10((uint32_t)q, r_lo, r_hi, a.tag, a.seed_lo, a.seed_hi, key);
      const int64_t j0 = q << 2;
#pragma unroll
      for (int i = 0; i < 4; ++i)
        if (j0 + i < n) {
          const uint32_t bin = key[i] >> 20;
          atomicAdd(&hist[bin], 1u);
          if (bin >= win_lo && bin <= win_hi) {
            const uint32_t pos = atomicAdd(&window_count, 1u);
            if (pos < a.window_cap) window[pos] = ((unsigned long long)key[i] << 32) | (uint32_t)(j0 + i);
          }
        }
    }
    __syncthreads();
    select_bin(hist, part, s, res);
    const uint32_t bin1 = res[0];
    const uint32_t want2 = s - res[1];
    uint32_t want3 = 0;
    const bool in_window = bin1 >= win_lo && bin1 <= win_hi && window_count <= a.window_cap;
    __syncthreads();
    bool have_candidates = false;
    if (in_window) {
      // the keys of the threshold bin are among the kept ones: move them to the candidate list
      const uint32_t wc = window_count;
      for (uint32_t i = t; i < wc; i += kThreads) {
        const unsigned long long c = window[i];
        if ((uint32_t)(c >> 52) == bin1) {
          const uint32_t pos = atomicAdd(&cand_count, 1u);
          if (pos < kCandMax) cand[pos] = c;
        }
      }
      __syncthreads();
      have_candidates = cand_count <= kCandMax;
      want3 = want2;  // 1-based rank inside the threshold bin
      __syncthreads();
      if (!have_candidates && t == 0) cand_count = 0;
      __syncthreads();
    }
    if (!have_candidates) {
      // pass B: next 12 bits among keys in bin1
      for (int i = t; i < kBins; i += kThreads) hist[i] = 0;
      __syncthreads();
      for (int64_t q = t; q < nq; q += kThreads) {
        uint32_t key[4];
        philox4x32_10((uint32_t)q, r_lo, r_hi, a.tag, a.seed_lo, a.seed_hi, key);
        const int64_t j0 = q << 2;
#pragma unroll
        for (int i = 0; i < 4; ++i)
          if (j0 + i < n && (key[i] >> 20) == bin1) atomicAdd(&hist[(key[i] >> 8) & 0xFFFu], 1u);
      }
      __syncthreads();
      select_bin(hist, part, want2, res);
      const uint32_t prefix24 = (bin1 << 12) | res[0];
      want3 = want2 - res[1];  // 1-based rank among the candidates
      __syncthreads();
      // pass C: list the keys sharing the 24-bit prefix, as (key, column) composites
      for (int64_t q = t; q < nq; q += kThreads) {
        uint32_t key[4];
        philox4x32_10((uint32_t)q, r_lo, r_hi, a.tag, a.seed_lo, a.seed_hi, key);
        const int64_t j0 = q << 2;
#pragma unroll
        for (int i = 0; i < 4; ++i)
          if (j0 + i < n && (key[i] >> 8) == prefix24) {
            uint32_t pos = atomicAdd(&cand_count, 1u);
            if (pos < kCandMax) cand[pos] = ((unsigned long long)key[i] << 32) | (uint32_t)(j0 + i);
          }
      }
      __syncthreads();
    }
    uint32_t nc = cand_count;
    if (nc > kCandMax) {  // never in practice (needs > 2048 of n keys in one 2^-24 slice)
      if (t == 0) atomicExch(a.error_flag, 1);
      nc = kCandMax;
    }
    for (uint32_t i = t; i < nc; i += kThreads) {
      const unsigned long long me = cand[i];
      uint32_t rank = 0;
      for (uint32_t o = 0; o < nc; ++o) rank += (cand[o] < me) ? 1u : 0u;
      if (rank == want3 - 1) threshold = me;
    }
    __syncthreads();
    const unsigned long long thr = threshold;

    // pass D: emit. Each wave covers 4 words (256 columns) per step: lane l owns
    // the quad of columns 4l..4l+3 of that span.
    for (int64_t span = wave; span * 4 < W; span += kThreads / 64) {
      const int64_t q = span * 64 + lane;
      uint32_t nib = 0;
      if (q < nq) {
        uint32_t key[4];
        philox4x32_10((uint32_t)q, r_lo, r_hi, a.tag, a.seed_lo, a.seed_hi, key);
        const int64_t j0 = q << 2;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const unsigned long long comp = ((unsigned long long)key[i] << 32) | (uint32_t)(j0 + i);
          if (j0 + i < n && comp <= thr) nib |= (1u << i);
        }
      }
      // OR the 16 nibbles of each 16-lane group into one 64-bit word
      const int pos = (lane & 15) * 4;
      uint32_t wlo = pos < 32 ? (nib << pos) : 0u;
      uint32_t whi = pos >= 32 ? (nib << (pos - 32)) : 0u;
#pragma unroll
      for (int m = 1; m < 16; m <<= 1) {
        wlo |= (uint32_t)__shfl_xor((int)wlo, m, 64);
        whi |= (uint32_t)__shfl_xor((int)whi, m, 64);
      }
      const int64_t wd = span * 4 + (lane >> 4);
      if ((lane & 15) == 0 && wd < W) {
        const uint64_t word = ((uint64_t)whi << 32) | wlo;
        row_small[wd] = word;
        row_big[wd] = ~word & ((wd == W - 1) ? tail_mask : ~0ull);
      }
    }
    if (t == 0) {
      const float wt = a.wtab[s];
      const int64_t o = 2 * (r - a.pair_begin);
      a.w[o] = wt;
      a.w[o + 1] = wt;
      a.sz[o] = (int32_t)s;
      a.sz[o + 1] = (int32_t)(n - s);
    }
    __syncthreads();
  }
}

// The common case in one pass over the keys. The s-th smallest of n uniform 32-bit keys lies within a few standard
// deviations of (s/n) 2^32; so while the keys are generated once, every column whose key falls below a window
// around that value gets its bit at once (a lane builds one 32-bit word of the row from eight generator calls and
// stores it), the few keys inside the window are listed, and the keys below the window are counted. The threshold
// is then the (s - below)-th smallest of the listed (key, column) pairs, found through a histogram of the window's
// sub-ranges and a rank count inside the threshold's sub-range, and the listed columns at or below it are added to
// the written row with atomics. Pairs whose threshold falls outside the window (about 0.3 %) or whose lists overflow,
// the two constraint rows and enumerated classes are left to the multi-pass kernel through the retry list.
// Same keys, same comparison, same masks.
constexpr int kWinBins = 1024;
constexpr int kFastCand = 1024;
constexpr int kFastThreads = 512;
constexpr uint32_t kFastWindow = 4096;   // listed keys at most (32 KB of LDS)

__global__ __launch_bounds__(kFastThreads) void sample_pairs_fast_kernel(SampleArgs a) {
  __shared__ uint32_t whist[kWinBins];
  __shared__ unsigned long long cand[kFastCand];
  __shared__ unsigned long long window[kFastWindow];
  __shared__ uint32_t cand_count, window_count, below_total, sel[2], list_count;
  __shared__ unsigned long long threshold;

  const int t = threadIdx.x;
  const int lane = t & 63;
  const int64_t n = a.n, W = a.W;
  const int64_t D = 2 * W;   // 32-bit words of a row
  uint32_t wcap = a.window_cap < kFastWindow ? a.window_cap : kFastWindow;

  for (int64_t r = a.pair_begin + blockIdx.x; r < a.pair_end; r += gridDim.x) {
    uint32_t* row_small = (uint32_t*)(a.Z + (2 * (r - a.pair_begin)) * W);
    uint32_t* row_big = row_small + D;
    int64_t lo = 1, hi = a.H;
    while (lo < hi) {
      int64_t mid = (lo + hi) >> 1;
      if (a.b[mid] >= r) hi = mid; else lo = mid + 1;
    }
    const uint32_t s = (uint32_t)lo;
    // window [k_lo, k_hi] of key values: expected position of the threshold +- (3 sigma + 8) ranks
    uint32_t k_lo, k_hi;
    {
      const double fs = (double)s, fn = (double)n;
      const double half = 3.0 * sqrt(fs * (fn - fs) / fn) + 8.0;
      const double scale = 4294967296.0 / fn;
      const double x_lo = (fs - half) * scale, x_hi = (fs + half) * scale;
      k_lo = x_lo <= 0.0 ? 0u : (uint32_t)x_lo;
      k_hi = x_hi >= 4294967295.0 ? 0xffffffffu : (uint32_t)x_hi;
    }
    const uint32_t width = k_hi - k_lo;                          // keys k with k - k_lo <= width are listed
    const int shift = width >= (uint32_t)kWinBins ? 32 - __builtin_clz(width) - 10 : 0;   // (width >> shift) < kWinBins
    bool give_up = r == 0 || (int64_t)s <= a.enum_upto;          // uniform over the workgroup
    // the small member also goes out as a list of its players (sparse rows only): every lane appends the columns
    // of the word it has just built, in whatever order the lanes arrive
    const bool listing = a.list != nullptr && (int64_t)s <= a.list_max;
    const int64_t list_off = listing ? a.list_cum[s] + (r - a.b[s - 1] - 1) * (int64_t)s : 0;
    uint32_t* const lst = a.list + list_off;
    if (!give_up) {
      const uint32_t r_lo = (uint32_t)r, r_hi = (uint32_t)((uint64_t)r >> 32);
      for (int i = t; i < kWinBins; i += kFastThreads) whist[i] = 0;
      if (t == 0) {
        cand_count = 0;
        window_count = 0;
        below_total = 0;
        list_count = 0;
      }
      __syncthreads();
      uint32_t below = 0;
      for (int64_t d = t; d < D; d += kFastThreads) {   // a wave writes 256 contiguous bytes per step
        const int64_t c0 = d << 5;
        const uint32_t valid = c0 + 32 <= n ? 0xffffffffu : (c0 < n ? (1u << (uint32_t)(n - c0)) - 1u : 0u);
        uint32_t word = 0;
        if (valid) {
#pragma unroll 2
          for (int i = 0; i < 8; ++i) {
            uint32_t key[4];
            philox4x32_10((uint32_t)(d * 8 + i), r_lo, r_hi, a.tag, a.seed_lo, a.seed_hi, key);
            // the common case without a branch per key: a key below the window shifts a one into the word (first column
            // ends up in the top bit: reversed once at the end); key - k_lo <= width (unsigned: a key below k_lo wraps
            // to more than width, because k_lo + width < 2^32) marks a key inside the window, and the four tests of a
            // generator call share one branch
            bool in_window = false;
#pragma unroll
            for (int c = 0; c < 4; ++c) {
              word = (word << 1) | (key[c] < k_lo ? 1u : 0u);
              in_window |= key[c] - k_lo <= width;
            }
            if (in_window) {
#pragma unroll
              for (int c = 0; c < 4; ++c) {
                const uint32_t off = key[c] - k_lo;
                const int64_t col = c0 + 4 * i + c;
                if (off <= width && col < n) {
                  atomicAdd(&whist[off >> shift], 1u);
                  const uint32_t pos = atomicAdd(&window_count, 1u);
                  if (pos < wcap) window[pos] = ((unsigned long long)key[c] << 32) | (uint32_t)col;
                }
              }
            }
          }
          word = __brev(word);
          word &= valid;
          below += __popc(word);
        }
        row_small[d] = word;
        row_big[d] = ~word & valid;
        if (listing && word) {   // a lane with columns reserves their places by itself
          uint32_t pos = atomicAdd(&list_count, (uint32_t)__popc(word)), bits = word;
          while (bits) {
            if (pos < s) lst[pos] = (uint32_t)c0 + (uint32_t)(__ffs((int)bits) - 1);   // (past s only when the pair is given up)
            ++pos;
            bits &= bits - 1;
          }
        }
      }
      for (int o = 32; o > 0; o >>= 1) below += __shfl_xor(below, o, 64);
      if (lane == 0) atomicAdd(&below_total, below);
      __syncthreads();   // (also: the row's words are written before any of them is patched below)
      const uint32_t wc = window_count;
      const int64_t want = (int64_t)s - (int64_t)below_total;   // 1-based rank of the threshold among the listed keys
      give_up = wc > wcap || want < 1 || want > (int64_t)wc;
      if (!give_up) {
        if (t < 64) {  // the sub-range that holds rank `want`: wave 0 scans 16 bins per lane, one lane walks its 16
          constexpr int kPer = kWinBins / 64;
          uint32_t v = 0;
#pragma unroll
          for (int i = 0; i < kPer; ++i) v += whist[t * kPer + i];
          uint32_t incl = v;
          for (int o = 1; o < 64; o <<= 1) {
            const uint32_t up = __shfl_up(incl, o, 64);
            if (t >= o) incl += up;
          }
          const unsigned long long reach = __ballot(incl >= (uint32_t)want);
          const int owner = reach ? __ffsll((long long)reach) - 1 : 63;   // the total always reaches `want`
          if (t == owner) {
            uint32_t cum = incl - v;
            int bsel = t * kPer;
            const int bend = bsel + kPer - 1;
            while (bsel < bend && cum + whist[bsel] < (uint32_t)want) cum += whist[bsel++];
            sel[0] = (uint32_t)bsel;
            sel[1] = (uint32_t)want - cum;   // 1-based rank inside that sub-range
          }
        }
        __syncthreads();
        const uint32_t bin1 = sel[0], want3 = sel[1];
        for (uint32_t i = t; i < wc; i += kFastThreads) {
          const unsigned long long c = window[i];
          if ((((uint32_t)(c >> 32) - k_lo) >> shift) == bin1) {
            const uint32_t pos = atomicAdd(&cand_count, 1u);
            if (pos < kFastCand) cand[pos] = c;
          }
        }
        __syncthreads();
        const uint32_t nc = cand_count;
        give_up = nc > kFastCand;
        if (!give_up) {
          for (uint32_t i = t; i < nc; i += kFastThreads) {
            const unsigned long long me = cand[i];
            uint32_t rank = 0;
            for (uint32_t o = 0; o < nc; ++o) rank += (cand[o] < me) ? 1u : 0u;
            if (rank == want3 - 1) threshold = me;
          }
          __syncthreads();
          const unsigned long long thr = threshold;
          for (uint32_t i = t; i < wc; i += kFastThreads) {
            const unsigned long long c = window[i];
            if (c <= thr) {
              const uint32_t col = (uint32_t)c;
              const uint32_t bit = 1u << (col & 31);
              atomicOr(&row_small[col >> 5], bit);
              atomicAnd(&row_big[col >> 5], ~bit);
              if (listing) {
                const uint32_t pos = atomicAdd(&list_count, 1u);
                if (pos < s) lst[pos] = col;
              }
            }
          }
          if (t == 0) {
            const float wt = a.wtab[s];
            const int64_t o = 2 * (r - a.pair_begin);
            a.w[o] = wt;
            a.w[o + 1] = wt;
            a.sz[o] = (int32_t)s;
            a.sz[o + 1] = (int32_t)(n - s);
            if (listing) a.list_offset[r - a.pair_begin] = list_off;   // below + listed keys up to the threshold = s entries
          }
        }
      }
    }
    if (give_up && t == 0) a.retry[atomicAdd(a.retry_count, 1u)] = (int32_t)(r - a.pair_begin);
    __syncthreads();
  }
}

// Enumeration (n <= 24): pair r = (bit pattern r, its complement).
__global__ void enumerate_pairs_kernel(SampleArgs a) {
  const int64_t r = a.pair_begin + (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (r >= a.pair_end) return;
  const uint64_t full = (1ull << a.n) - 1ull;
  const uint64_t small = (uint64_t)r, big = ~small & full;
  const int pc = __popcll(small);
  const int cls = pc < (int)a.n - pc ? pc : (int)a.n - pc;
  const int64_t o = 2 * (r - a.pair_begin);
  a.Z[o] = small;
  a.Z[o + 1] = big;
  const float wt = cls == 0 ? 0.f : a.wtab[cls];
  a.w[o] = wt;
  a.w[o + 1] = wt;
  a.sz[o] = pc;
  a.sz[o + 1] = (int)a.n - pc;
}

}  // namespace

size_t ds_sample_arena_bytes(const ds_plan& plan) {
  return 2 * ds_align((plan.H + 2) * sizeof(int64_t)) + ds_align((plan.H + 1) * sizeof(float)) + ds_align((size_t)(plan.k / 2 + 2) * 4) + 512;
}

// entries of the lists of the size classes 1..max_size: class s has b[s] - b[s-1] pairs of s players
int64_t ds_pair_list_entries(const ds_plan& plan, int64_t max_size) {
  int64_t total = 0;
  for (int64_t s = 1; s <= max_size && s <= plan.H; ++s) total += (plan.b[s] - plan.b[s - 1]) * s;
  return total;
}

bool ds_sampler_lists_possible(const ds_ctx* ctx, const ds_plan& plan) {
  return !plan.enumerate && plan.n >= 4096 && ctx->tuning.sampler_window != -1 && plan.k / 2 < 0x7fffffffLL;
}

int ds_sample_launch(ds_ctx* ctx, const ds_plan& plan, uint64_t seed, uint32_t tag, int64_t pair_begin,
                     int64_t pair_end, uint64_t* Z, float* w, int32_t* sz, const ds_pair_lists* lists) {
  if (lists && (pair_begin != 0 || !ds_sampler_lists_possible(ctx, plan)))
    return ds_fail(ctx, DS_EINTERNAL, "sampler: player lists are written only by the one-pass kernel from pair 0");
  if (pair_begin < 0 || pair_end > plan.k / 2 || pair_begin > pair_end)
    return ds_fail(ctx, DS_EINVAL, "pair range [%lld, %lld) outside [0, %lld)", (long long)pair_begin,
                   (long long)pair_end, (long long)(plan.k / 2));
  if (pair_begin == pair_end) return DS_OK;
  if (plan.enum_upto > 0 && (double)plan.K * (double)plan.n >= 4.0e18)
    return ds_fail(ctx, DS_EINVAL, "saturated size classes: the plan is too large for exact 64-bit unranking");
  const int64_t H = plan.H;
  int64_t* d_b = (int64_t*)ds_arena_alloc(ctx, (H + 1) * sizeof(int64_t));
  float* d_wtab = (float*)ds_arena_alloc(ctx, (H + 1) * sizeof(float));
  const int64_t lmax = lists ? (lists->max_size < H ? lists->max_size : H) : 0;
  int64_t* d_cum = lists ? (int64_t*)ds_arena_alloc(ctx, (lmax + 2) * sizeof(int64_t)) : nullptr;
  if (!d_b || !d_wtab || (lists && !d_cum)) return ds_fail(ctx, DS_EINTERNAL, "sampler: arena exhausted");
  // the plan tables go through pinned staging so that the upload is asynchronous
  const size_t need = ds_align((H + 1) * sizeof(int64_t)) + ds_align((H + 1) * sizeof(float)) + ds_align((lmax + 2) * sizeof(int64_t));
  if (ctx->stage_busy) {
    DS_HIP(ctx, hipEventSynchronize(ctx->stage_ev));
    ctx->stage_busy = false;
  }
  if (need > ctx->h_stage_bytes) {
    if (ctx->h_stage) (void)hipHostFree(ctx->h_stage);
    ctx->h_stage = nullptr;
    ctx->h_stage_bytes = 0;
    if (hipHostMalloc((void**)&ctx->h_stage, need, hipHostMallocDefault) != hipSuccess)
      return ds_fail(ctx, DS_ENOMEM, "sampler: cannot allocate %zu bytes of pinned staging", need);
    ctx->h_stage_bytes = need;
  }
  char* hb = ctx->h_stage;
  char* hw = ctx->h_stage + ds_align((H + 1) * sizeof(int64_t));
  memcpy(hb, plan.b.data(), (H + 1) * sizeof(int64_t));
  memcpy(hw, plan.wtab.data(), (H + 1) * sizeof(float));
  DS_HIP(ctx, hipMemcpyAsync(d_b, hb, (H + 1) * sizeof(int64_t), hipMemcpyHostToDevice, ctx->stream));
  DS_HIP(ctx, hipMemcpyAsync(d_wtab, hw, (H + 1) * sizeof(float), hipMemcpyHostToDevice, ctx->stream));
  if (lists) {   // entries before each listed class; every pair starts without a list
    int64_t* hc = (int64_t*)(hw + ds_align((H + 1) * sizeof(float)));
    hc[0] = 0;
    hc[1] = 0;
    for (int64_t s = 1; s <= lmax; ++s) hc[s + 1] = hc[s] + (plan.b[s] - plan.b[s - 1]) * s;
    if (hc[lmax + 1] > lists->total) return ds_fail(ctx, DS_EINTERNAL, "sampler: the player lists need %lld entries, %lld are reserved", (long long)hc[lmax + 1], (long long)lists->total);
    DS_HIP(ctx, hipMemcpyAsync(d_cum, hc, (lmax + 2) * sizeof(int64_t), hipMemcpyHostToDevice, ctx->stream));
    DS_HIP(ctx, hipMemsetAsync(lists->offset, 0xFF, (size_t)(pair_end - pair_begin) * sizeof(int64_t), ctx->stream));
  }
  DS_HIP(ctx, hipEventRecord(ctx->stage_ev, ctx->stream));
  ctx->stage_busy = true;
  int* d_err = (int*)(ctx->d_mail + DS_MAIL_SAMPLER);
  DS_HIP(ctx, hipMemsetAsync(d_err, 0, sizeof(int64_t), ctx->stream));
  SampleArgs a;
  a.n = plan.n;
  a.W = (plan.n + 63) / 64;
  a.K = plan.K;
  a.H = H;
  a.enum_upto = plan.enum_upto;
  a.pair_begin = pair_begin;
  a.pair_end = pair_end;
  a.b = d_b;
  a.wtab = d_wtab;
  a.seed_lo = (uint32_t)seed;
  a.seed_hi = (uint32_t)(seed >> 32);
  a.tag = tag;
  a.Z = Z;
  a.w = w;
  a.sz = sz;
  a.error_flag = d_err;
  a.list = lists ? lists->entries : nullptr;
  a.list_cum = d_cum;
  a.list_offset = lists ? lists->offset : nullptr;
  a.list_max = lmax;
  // window list capacity: bins within 3 sigma of the expected threshold position at the widest size (s = n/2)
  {
    const double nn = (double)plan.n, sigma = sqrt(nn / 4.0);
    const double bins = 2.0 * (2.0 + ceil(3.0 * sigma * 4096.0 / nn)) + 1.0;
    double cap = bins * nn / 4096.0 * 1.5 + 64.0;
    if (cap < 256.0) cap = 256.0;
    if (cap > 4096.0) cap = 4096.0;  // (32 KB of LDS; what overflows it takes more passes)
    a.window_cap = (uint32_t)cap;
    // test hook: a smaller list forces the four-pass route (the result must not change)
    const int32_t tw = ctx->tuning.sampler_window;
    if (tw == -1) a.window_cap = 0;
    else if (tw > 0 && (uint32_t)tw < a.window_cap) a.window_cap = (uint32_t)tw;
  }
  const int64_t pairs = pair_end - pair_begin;
  if (plan.enumerate) {
    const int threads = 256;
    const int64_t blocks = (pairs + threads - 1) / threads;
    hipLaunchKernelGGL(enumerate_pairs_kernel, dim3((unsigned)blocks), dim3(threads), 0, ctx->stream, a);
  } else {
    const int64_t blocks = pairs < (int64_t)ctx->num_cus * 64 ? pairs : (int64_t)ctx->num_cus * 64;
    a.retry = nullptr;
    a.retry_count = nullptr;
    if (a.window_cap > 0 && pairs < 0x7fffffffLL && plan.n >= 4096) {   // (a lane makes 32 columns: short rows leave the one-pass kernel idle)
      // one pass for the pairs whose threshold falls where it is expected, the multi-pass kernel for the rest
      a.retry = (int32_t*)ds_arena_alloc(ctx, (size_t)(pairs + 1) * 4);
      a.retry_count = (uint32_t*)ds_arena_alloc(ctx, 256);
      if (!a.retry || !a.retry_count) return ds_fail(ctx, DS_EINTERNAL, "sampler: arena exhausted");
      DS_HIP(ctx, hipMemsetAsync(a.retry_count, 0, 4, ctx->stream));
      const int64_t fblocks = pairs < (int64_t)ctx->num_cus * 32 ? pairs : (int64_t)ctx->num_cus * 32;
      hipLaunchKernelGGL(sample_pairs_fast_kernel, dim3((unsigned)fblocks), dim3(kFastThreads), 0, ctx->stream, a);
      const int64_t rblocks = blocks < (int64_t)ctx->num_cus * 4 ? blocks : (int64_t)ctx->num_cus * 4;
      if (a.window_cap > 4096) a.window_cap = 4096;   // (the multi-pass kernel holds more static LDS)
      hipLaunchKernelGGL(sample_pairs_kernel, dim3((unsigned)rblocks), dim3(kThreads), (size_t)a.window_cap * 8, ctx->stream, a);
    } else {
      if (a.window_cap > 4096) a.window_cap = 4096;
      hipLaunchKernelGGL(sample_pairs_kernel, dim3((unsigned)blocks), dim3(kThreads), (size_t)a.window_cap * 8, ctx->stream, a);
    }
  }
  DS_HIP(ctx, hipGetLastError());
  return DS_OK;
}

int ds_sample_check(ds_ctx* ctx) {
  DS_HIP(ctx, hipMemcpyAsync(ctx->h_mail + DS_MAIL_SAMPLER, ctx->d_mail + DS_MAIL_SAMPLER, sizeof(int64_t),
                             hipMemcpyDeviceToHost, ctx->stream));
  DS_HIP(ctx, hipStreamSynchronize(ctx->stream));
  if (ctx->h_mail[DS_MAIL_SAMPLER] != 0)
    return ds_fail(ctx, DS_EINTERNAL, "sampler: candidate list overflow (more than %d keys share a 24-bit prefix)", kCandMax);
  return DS_OK;
}
