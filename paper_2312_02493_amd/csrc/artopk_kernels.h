// Device code of the AR-Topk compressor for gfx950 (wave64).
//
// Kernels (in the order one step runs them):
//   k_fill_zero      clears the per-call scratch (histograms, scan flags, ...)
//   k_guess          (long flat vectors) samples g + residual and guesses a lower
//                    bound on the key of the k-th largest magnitude
//   k_pass_a         acc = g + residual in place, per-worker variance
//                    partials, and per-chunk 12-bit top-digit histograms of |acc|
//   k_pass_mark      the same pass behind k_guess: instead of histograms a bit
//                    mask of the keys reaching the guessed bound; its blocks
//                    stride over the tiles of the vector
//   k_hist0          the same histograms alone (stand-alone select, segments,
//                    after a guess that did not hold)
//   k_stats          variance partials alone (stand-alone variance)
//   k_leader         finishes the variances and takes the first argmax
//   k_pick0          (flat VAR: finishes the variances, takes the leader;) finds the
//                    threshold digit and every chunk's list offset
//   k_pick_mask      the same first step when the fused pass left a mask: accepts
//                    the guessed bound or asks for the histogram route
//   k_compact1       ordered compaction of the leader's survivors, one block
//                    per chunk, no inter-block dependency
//   k_mask_or_hist   the survivor list written from the mask instead; or, after
//                    a guess that did not hold, k_hist0's work in the same launch
//   k_compact        ordered compaction with a decoupled look-back scan: the
//                    rarely needed deeper array passes and the final pass over
//                    the survivor list
//   k_list_hist      digit histograms over the survivor list
//   k_level1 / k_level2 / k_final   the launches behind the first pick where
//                    alternatives exist: each does whichever of two jobs the state
//                    asks for (list histogram or array pass; final pass over the
//                    list or level-3 array pass writing the outputs), so that the
//                    rarely needed array passes cost no launches of their own
//   k_tile_starts    number of kept indices below every tile of a streaming pass
//   k_pass_rest      (leader known up front) EF add + gather + residual zeroing
//                    of all other workers in one streaming pass over the tiles
//   k_sum_update     (leader known up front) ordered sum over the workers' gathered
//                    rows and the dense update in one pass over the tiles
//   k_sum_rows       ordered sum over the workers' gathered rows
//   k_gather         vals / ordered sum / residual zeroing at the k indices
//   k_zero_at        residual zeroing alone
//   k_update_fill    dense update = zeros + k scattered sums, written once
//   k_update_tiles   the same for long, sparsely kept vectors: zeros streamed tile
//                    by tile, the sums stored behind them
//
// Keys are the 31 magnitude bits of the float32 (sign cleared), so integer
// order on keys is the order of |x|.  The radix digits are 12 + 12 + 7 bits.
//
// Chunks.  A vector range is cut into at most kMaxChunks contiguous chunks, each
// a whole number of 8192-element tiles.  The histogram pass stores, per chunk,
// the SUFFIX sums of its top-digit histogram: S[c][b] = number of keys of chunk
// c whose top digit is >= b.  Once the threshold digit b0 is known, S[c][b0] is
// exactly the number of survivors chunk c will emit, so an exclusive scan over
// the chunks gives every chunk its place in the survivor list and the big
// compaction pass needs no communication between blocks.
#pragma once

#include <hip/hip_runtime.h>

#include <type_traits>
#include <stdint.h>
#include <limits.h>

namespace artopk {

constexpr int kMaxW = 64;
constexpr int kHistBins = 4096;          // 12-bit digits (the last digit uses 128 of them)
constexpr int kHistReps = 16;            // partial copies of a whole-vector histogram (spreads the atomics)
// One slot of whole-vector scratch (32-bit words): the partial histogram copies, then the
// histogram of the threshold-guess sample, then its control words.
constexpr int kSlotGuessHist = kHistReps * kHistBins;
constexpr int kSlotCtrl = kSlotGuessHist + kHistBins;  // [0] blocks done, [1] guessed key bound, [2] a tile kept its marks to the mask,
                                                       // [3] top digit of the bound, [4] sample keys above that digit, [5] refine blocks done
constexpr int kSlotMcount = kSlotCtrl + 16;            // marked elements per chunk (kMaxChunks words)
constexpr int kSlotRefine = kSlotMcount + 1024;        // second-digit histogram of the guess sample (k_guess_refine)
constexpr int kSlotWords = kSlotRefine + kHistBins;
constexpr uint32_t kNoGuess = 0xffffffffu;             // no key reaches this bound
constexpr int kGuessRun = 16;                          // consecutive elements per sample run
constexpr uint32_t kKeyMask = 0x7fffffffu;
constexpr uint32_t kQuotaInf = 0x7fffffffu;

// digit l (0,1,2) of a key: shift and mask
__host__ __device__ constexpr int digit_shift(int level) { return level == 0 ? 19 : (level == 1 ? 7 : 0); }
__host__ __device__ constexpr uint32_t digit_mask(int level) { return level == 2 ? 0x7fu : 0xfffu; }

constexpr uint32_t kTileOverflow = 0xffffffffu;
constexpr int kStageMax = 6144;  // list entries a tile can hand on (48 KiB of on-chip memory)

struct TileBuf {
  uint2* buf;       // [slot][tile][cap] staged list entries, or nullptr
  uint32_t* cnt;    // [slot][tile] entries staged per tile, or kTileOverflow
  int64_t buf_stride;  // entries per slot
  int64_t cnt_stride;  // tiles per slot
  int32_t cap;         // entries per tile (<= kStageMax)
};

struct PtrTable {
  float* p[kMaxW];
};

// Device-resident selection state; one per select in flight.
struct SelState {
  uint32_t lo, hi;         // candidate keys: lo <= key <= hi
  uint32_t n_gt;           // keys > hi inside the element range
  uint32_t need;           // entries still to be taken from the candidates (>= 1)
  uint32_t cand;           // number of candidate keys
  uint32_t level;          // radix digits resolved so far (0..3)
  uint32_t compact_level;  // level at which the survivor list was written (0 = not yet)
  uint32_t list_count;     // entries in the survivor list
  uint32_t use_mask;       // the list is written from the survivor bit mask of the fused pass
  uint32_t need_full;      // the guessed bound did not work out: the top-digit histogram of every key is needed
  uint32_t list_lo;        // with use_mask: the list holds every key >= list_lo (<= lo)
  uint32_t pad[5];
};

// Bits of the sticky device-side error word.
constexpr uint32_t kErrPick = 1u;      // a histogram did not cover the wanted count
constexpr uint32_t kErrWait = 2u;      // a bounded look-back wait expired
constexpr uint32_t kErrSequence = 4u;  // a kernel found the state it needs missing
constexpr uint32_t kErrIndex = 8u;     // an index outside [0, N) reached gather / scatter

// Layout of one segment's zero-initialised scratch block (32-bit words).
constexpr int kSegState = 0;                       // SelState (16 words)
constexpr int kSegCounters = 16;                   // tile counters of the look-back passes (16 words)
constexpr int kSegHist1 = 32;                      // next-digit histogram, digit 1
constexpr int kSegHist2 = kSegHist1 + kHistBins;   // next-digit histogram, digit 2
constexpr int kSegHtop = kSegHist2 + kHistBins;    // top-digit histogram (when built by k_hist0)
constexpr int kSegWords = kSegHtop + kHistBins;
constexpr int kNumLookback = 4;                    // flag words per tile: array level 2, 3, list pass, spare

struct ChunkGeom {
  int64_t chunk0;       // first element of chunk 0 (a multiple of kTile, <= range start)
  int64_t chunk_elems;  // elements per chunk (a multiple of kTile)
  int32_t nchunks;
};

// One selection problem: the k largest magnitudes of x[e_lo, e_hi).
struct SegDesc {
  int64_t e_lo, e_hi;
  ChunkGeom geom;      // chunk layout of the range
  int64_t koff;        // first slot of this segment in idx_out (and in the leader's vals row)
  int64_t list_base;   // first entry of this segment's survivor list (a multiple of 4)
  int64_t flag_base;   // first look-back tile of this segment
  int32_t chunk_begin; // first chunk slot of this segment in S / chunk_off
  uint32_t k;          // entries wanted
  uint32_t cap;        // survivor-list capacity of this segment
  int32_t vec;         // which vector of the pointer table to select on; -1 = the leader's
};

// Everything the selection kernels need; blockIdx.y
// picks the segment.  With table == nullptr there is one segment, `one`.
struct SelParams {
  PtrTable tab;
  const int32_t* leader_dev;
  int64_t n;               // length of the vector
  const uint32_t* h_all;   // [workers][kSlotWords] whole-vector histograms from the fused pass, or nullptr
  const uint64_t* mask;    // [workers][mask_stride] survivor bit masks from the fused pass, or nullptr
  int64_t mask_stride;     // 64-bit words per worker
  TileBuf tiles;           // list entries the fused pass staged per tile (buf == nullptr: none)
  int32_t use_mcount;      // the slots' per-chunk counts of marked elements are valid
  int32_t from_list;       // k_pick0: the top-digit histogram covers the survivor list written from the mask
  int32_t after_mask;      // k_pick0 behind k_mask_or_hist: from_list if the mask was used, else the full pick
  int32_t only_if_need_full;  // this launch runs only for segments whose state says need_full
  uint32_t* zero_base;     // [segments][kSegWords]
  uint64_t* flags;         // [tiles][kNumLookback]
  uint32_t* S;             // [slot][kMaxChunks][4096] per-chunk suffix histograms
  uint32_t* chunk_off;     // [chunks]
  uint2* list;             // survivor lists
  int32_t* idx_out;
  float* vals_row;         // leader's row of gathered values, or nullptr
  float* zero_vec;         // the selected vector itself if its kept entries are to become +0.0 on the way, or nullptr
  uint32_t* err;
  const SegDesc* table;
  // per-chunk kernels of a segmented selection run one block per chunk of the whole layout:
  // entry b = (segment << 16) | chunk within the segment; nullptr: grid = (chunks, segments)
  const uint32_t* chunk_map;
  int32_t slot_by_leader;  // S slot = index of the selected vector (histograms of all workers exist) or 0
  int32_t pad;
  SegDesc one;
};

// The (segment, chunk) a block of a per-chunk kernel works on.
__device__ __forceinline__ void block_chunk(const SelParams& p, int& seg, int& c) {
  if (p.chunk_map != nullptr) {
    const uint32_t m = p.chunk_map[blockIdx.x];
    seg = (int)(m >> 16);
    c = (int)(m & 0xffffu);
  } else {
    seg = (int)blockIdx.y;
    c = (int)blockIdx.x;
  }
}

struct SegView {
  SegDesc d;
  const float* x;  // the vector this segment selects on
  SelState* st;
  uint32_t* counters;
  uint32_t* hist1;
  uint32_t* hist2;
  uint32_t* htop;       // top-digit histogram of the selected vector's range: htop_reps partial copies to add up
  int htop_reps;
  uint32_t* hseg;       // the segment's own top-digit histogram (single copy), what k_hist0 fills without h_all
  const uint32_t* ctrl;  // control words of the vector's slot (guessed bound), or nullptr
  const uint64_t* mask;  // survivor bit mask of the vector, or nullptr
  const uint2* tbuf;     // list entries the fused pass staged per tile of the vector, or nullptr
  const uint32_t* tcnt;  // their number per tile (kTileOverflow: none, use the mask)
  int32_t tcap;          // entries per tile in tbuf
  const uint32_t* mcount;  // marked elements per chunk of the vector, or nullptr
  uint64_t* flags;
  uint32_t* S;
  uint32_t* chunk_off;
  uint2* list;
  int32_t* idx_out;
  float* vals_row;
};

// ---------------------------------------------------------------------------
// small helpers
// ---------------------------------------------------------------------------
__device__ __forceinline__ uint32_t lane_id() { return threadIdx.x & 63u; }

__device__ __forceinline__ uint32_t popc_lt(uint64_t mask) {
  // number of set bits of `mask` in lanes below the calling lane
  return __builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0u));
}

__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_down(v, off, 64);
  return v;  // valid in lane 0
}

__device__ __forceinline__ uint64_t wave_allsum_u64(uint64_t v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) {
    uint32_t lo = __shfl_xor((uint32_t)v, off, 64);
    uint32_t hi = __shfl_xor((uint32_t)(v >> 32), off, 64);
    v += ((uint64_t)hi << 32) | lo;
  }
  return v;  // the total, in every lane
}

constexpr int kTile = 8192;       // chunk granularity (a quarter of a tile of the fused pass)
constexpr int kMaxChunks = 1024;  // chunks per vector range
static_assert(kSlotRefine == kSlotMcount + kMaxChunks, "one count per chunk");
constexpr int kPassTile = 32768;      // elements per block iteration of the streaming passes (1024 threads x 8 float4)
constexpr int kMaxPassBlocks = 4096;  // blocks per worker of a streaming pass that strides over tiles

typedef float v4f __attribute__((ext_vector_type(4)));

// ---------------------------------------------------------------------------
// Variance in one pass that no single element can spoil.  Every thread keeps, in
// float64, the count and the sums of (x - c) and (x - c)^2 of the values it sees,
// with a shift c of its own: the mean of the first four of them.  At the end of a
// block the threads re-base their sums (exactly: S' = S + n d, SS' = SS + d (2 S + n d),
// d = c - r) to the shift r of the block's first thread and add them up.  For any
// data, a block that sees m values has (mean - r)^2 <= (m / 4) variance of its
// values (Cauchy-Schwarz: r is the mean of four of them), so the cancellation of
// the shifted one-pass formula is bounded by the block's length and does not grow
// with an outlier or an offset.  The block's sums become (count n, mean, M2 = sum
// of squared deviations from its mean); the blocks' triples of one worker are
// combined the same way, with the mean of the worker's first block as the shift:
//     N = sum n_b, A = sum n_b (mean_b - r), B = sum (M2_b + n_b (mean_b - r)^2),
//     mean = r + A / N, M2 = B - A^2 / N.
// The order of every sum is fixed by the launch shape, so the result is reproducible.
// Partials layout: partials[w][0][b] = n_b, [w][1][b] = mean_b, [w][2][b] = M2_b.
// ---------------------------------------------------------------------------
struct VarAcc {
  double c = 0.0, s = 0.0, ss = 0.0;
  uint32_t cnt = 0u;
  // the shift is taken from the first group (or element) a thread sees: call seed before the
  // first add of every batch (it acts once)
  __device__ __forceinline__ void seed4(const v4f t) {
    if (cnt == 0u) c = (((double)t.x + (double)t.y) + ((double)t.z + (double)t.w)) * 0.25;
  }
  __device__ __forceinline__ void seed1(float x) {
    if (cnt == 0u) c = (double)x;
  }
  __device__ __forceinline__ void add4(const v4f t) {
    const double d0 = (double)t.x - c, d1 = (double)t.y - c, d2 = (double)t.z - c, d3 = (double)t.w - c;
    s += (d0 + d1) + (d2 + d3);
    ss = fma(d0, d0, ss);
    ss = fma(d1, d1, ss);
    ss = fma(d2, d2, ss);
    ss = fma(d3, d3, ss);
    cnt += 4u;
  }
  __device__ __forceinline__ void add1(float x) {
    const double d = (double)x - c;
    s += d;
    ss = fma(d, d, ss);
    cnt += 1u;
  }
};

__device__ __forceinline__ double wave_allsum(double v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
  return v;  // the total, in every lane (the same bits: every lane adds the same pairs)
}

// Adds up the threads' sums of a block of T threads (all of them call it) and thread 0 writes
// the block's (n, mean, M2) to partials[w][.][b] (nblk blocks per worker).  Thread 0 must be a
// thread that saw a value whenever any thread of the block did (it owns the block's first group).
template <int T>
__device__ __forceinline__ void block_moments(const VarAcc& acc, double* __restrict__ partials, int w, int nblk,
                                              int b) {
  constexpr int NW = T / 64;
  __shared__ double red[3 * NW + 1];
  const int tid = threadIdx.x;
  if (tid == 0) red[3 * NW] = acc.c;
  __syncthreads();
  const double r = red[3 * NW];
  const double n_t = (double)acc.cnt;
  const double d = acc.cnt != 0u ? acc.c - r : 0.0;
  const double s = wave_sum(acc.s + n_t * d), ss = wave_sum(acc.ss + d * (2.0 * acc.s + n_t * d)), n = wave_sum(n_t);
  if ((tid & 63) == 0) {
    red[tid >> 6] = s;
    red[NW + (tid >> 6)] = ss;
    red[2 * NW + (tid >> 6)] = n;
  }
  __syncthreads();
  if (tid == 0) {
    double S1 = 0.0, S2 = 0.0, N = 0.0;
#pragma unroll
    for (int i = 0; i < NW; ++i) {
      S1 += red[i];
      S2 += red[NW + i];
      N += red[2 * NW + i];
    }
    double mean = 0.0, m2 = 0.0;
    if (N > 0.0) {
      const double sm = S1 / N;
      mean = r + sm;
      m2 = S2 - S1 * sm;
      if (m2 < 0.0) m2 = 0.0;  // rounding only (NaN stays NaN)
    }
    double* __restrict__ out = partials + (size_t)w * 3 * nblk + b;
    out[0] = N;
    out[nblk] = mean;
    out[2 * (size_t)nblk] = m2;
  }
}

// Variance of worker w from its blocks' partials; the 64 lanes of one wave call it, every lane
// returns the variance (population: M2 / N).
__device__ __forceinline__ double wave_variance(const double* __restrict__ partials, int w, int nblk) {
  const int lane = threadIdx.x & 63;
  const double* __restrict__ pn = partials + (size_t)w * 3 * nblk;
  const double* __restrict__ pm = pn + nblk;
  const double* __restrict__ pq = pm + nblk;
  const double r = pm[0];
  double n = 0.0, a = 0.0, bq = 0.0;
  int b = lane;
  for (; b + 448 < nblk; b += 512) {  // eight blocks' triples in flight per lane
    double nb[8], mb[8], qb[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      nb[j] = pn[b + 64 * j];
      mb[j] = pm[b + 64 * j];
      qb[j] = pq[b + 64 * j];
    }
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const double d = mb[j] - r;
      n += nb[j];
      a += nb[j] * d;
      bq += qb[j] + nb[j] * d * d;
    }
  }
  for (; b < nblk; b += 64) {
    const double nb = pn[b], d = pm[b] - r;
    n += nb;
    a += nb * d;
    bq += pq[b] + nb * d * d;
  }
  n = wave_allsum(n);
  a = wave_allsum(a);
  bq = wave_allsum(bq);
  double v = 0.0;
  if (n > 0.0) v = (bq - a * (a / n)) / n;
  if (!(v > 0.0)) v = (v != v) ? v : 0.0;
  return v;
}

template <bool NT>
__device__ __forceinline__ v4f load4(const float* p) {
  return NT ? __builtin_nontemporal_load(reinterpret_cast<const v4f*>(p)) : *reinterpret_cast<const v4f*>(p);
}
template <bool NT>
__device__ __forceinline__ void store4(float* p, v4f v) {
  if (NT)
    __builtin_nontemporal_store(v, reinterpret_cast<v4f*>(p));
  else
    *reinterpret_cast<v4f*>(p) = v;
}

// Gradient element types: float32, or 16 bits widened exactly to float32 before use
// (bfloat16: the bits become the upper half of the float32; float16: hardware conversion).
constexpr int kGF32 = 0, kGBF16 = 1, kGF16 = 2;

template <int GT>
__device__ __forceinline__ float widen16(uint32_t h) {  // h: the 16 bits in the low half
  if (GT == kGBF16) return __uint_as_float(h << 16);
  return (float)__builtin_bit_cast(_Float16, (unsigned short)h);
}

// Four consecutive gradient elements starting at element index e (a multiple of 4).
template <bool NT, int GT>
__device__ __forceinline__ v4f load4g(const float* base, int64_t e) {
  if (GT == kGF32) return load4<NT>(base + e);
  typedef uint32_t v2u __attribute__((ext_vector_type(2)));
  const v2u* p = reinterpret_cast<const v2u*>(reinterpret_cast<const unsigned short*>(base) + e);
  const v2u r = NT ? __builtin_nontemporal_load(p) : *p;
  v4f v;
  v.x = widen16<GT>(r.x & 0xffffu);
  v.y = widen16<GT>(r.x >> 16);
  v.z = widen16<GT>(r.y & 0xffffu);
  v.w = widen16<GT>(r.y >> 16);
  return v;
}

template <int GT>
__device__ __forceinline__ float load1g(const float* base, int64_t e) {
  if (GT == kGF32) return base[e];
  return widen16<GT>(reinterpret_cast<const unsigned short*>(base)[e]);
}

// Block-wide inclusive scans of one word per thread: a shuffle scan inside each
// wave, then the wave totals through `wtot` (T/64 words of shared memory that no
// thread still reads on entry).  Two barriers; `wtot` is free again on return.
// The exclusive value is the result minus the thread's own word.
template <int T>
__device__ __forceinline__ uint32_t block_suffix_incl(uint32_t v, uint32_t* wtot, uint32_t* total = nullptr) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  uint32_t s = v;
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    const uint32_t x = __shfl_down(s, off, 64);
    if (lane + off < 64) s += x;
  }
  if (lane == 0) wtot[wave] = s;
  __syncthreads();
  uint32_t add = 0u, tot = 0u;
#pragma unroll
  for (int i = 0; i < T / 64; ++i) {
    const uint32_t x = wtot[i];
    tot += x;
    if (i > wave) add += x;
  }
  __syncthreads();
  if (total) *total = tot;
  return s + add;
}

template <int T>
__device__ __forceinline__ uint32_t block_prefix_incl(uint32_t v, uint32_t* wtot, uint32_t* total = nullptr) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  uint32_t s = v;
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    const uint32_t x = __shfl_up(s, off, 64);
    if (lane >= off) s += x;
  }
  if (lane == 63) wtot[wave] = s;
  __syncthreads();
  uint32_t add = 0u, tot = 0u;
#pragma unroll
  for (int i = 0; i < T / 64; ++i) {
    const uint32_t x = wtot[i];
    tot += x;
    if (i < wave) add += x;
  }
  __syncthreads();
  if (total) *total = tot;
  return s + add;
}

// Adds the 4096-bin LDS histogram `lh` of a T-thread block to total[0..4096)
// and writes its suffix sums to dst[0..4096).  `red` is T words of LDS.  All
// threads of the block must call it after their last histogram update.
template <int T>
__device__ __forceinline__ void flush_suffix_hist(uint32_t* lh, uint32_t* red, uint32_t* __restrict__ dst,
                                                  uint32_t* __restrict__ total) {
  constexpr int BPT = kHistBins / T;  // consecutive bins per thread (a multiple of 4)
  static_assert(BPT >= 4 && BPT % 4 == 0, "block size must divide 1024");
  const int t = threadIdx.x;
  __syncthreads();
  uint32_t v[BPT];
#pragma unroll
  for (int j = 0; j < BPT / 4; ++j) {
    const uint4 q = reinterpret_cast<const uint4*>(lh)[(BPT / 4) * t + j];
    v[4 * j + 0] = q.x;
    v[4 * j + 1] = q.y;
    v[4 * j + 2] = q.z;
    v[4 * j + 3] = q.w;
  }
  // the plain counts also go to the histogram of the whole range (few bins are occupied)
#pragma unroll
  for (int j = 0; j < BPT; ++j)
    if (v[j]) atomicAdd(&total[BPT * t + j], v[j]);
#pragma unroll
  for (int j = BPT - 2; j >= 0; --j) v[j] += v[j + 1];
  const uint32_t carry = block_suffix_incl<T>(v[0], red) - v[0];
#pragma unroll
  for (int j = 0; j < BPT / 4; ++j) {
    uint4 q;
    q.x = v[4 * j + 0] + carry;
    q.y = v[4 * j + 1] + carry;
    q.z = v[4 * j + 2] + carry;
    q.w = v[4 * j + 3] + carry;
    reinterpret_cast<uint4*>(dst)[(BPT / 4) * t + j] = q;
  }
}

// leader >= 0 overrides the device-resident leader (used by the block that has just computed it)
__device__ __forceinline__ SegView seg_view(const SelParams& p, int seg, int leader = -1) {
  SegView v;
  v.d = p.table ? p.table[seg] : p.one;
  uint32_t* zb = p.zero_base + (size_t)seg * kSegWords;
  v.st = reinterpret_cast<SelState*>(zb + kSegState);
  v.counters = zb + kSegCounters;
  v.hist1 = zb + kSegHist1;
  v.hist2 = zb + kSegHist2;
  v.flags = p.flags + (size_t)v.d.flag_base * kNumLookback;
  const int vec = v.d.vec >= 0 ? v.d.vec : (leader >= 0 ? leader : *p.leader_dev);
  v.x = p.tab.p[vec];
  const size_t slot = p.slot_by_leader ? (size_t)vec : 0;  // histogram slot: per vector, or the only one
  v.htop = p.h_all ? const_cast<uint32_t*>(p.h_all) + slot * kSlotWords : zb + kSegHtop;
  v.htop_reps = p.h_all ? kHistReps : 1;
  v.hseg = zb + kSegHtop;
  v.ctrl = p.h_all ? p.h_all + slot * kSlotWords + kSlotCtrl : nullptr;
  v.mask = p.mask ? p.mask + slot * (size_t)p.mask_stride : nullptr;
  v.tbuf = (p.mask && p.tiles.buf) ? p.tiles.buf + slot * (size_t)p.tiles.buf_stride : nullptr;
  v.tcnt = (p.mask && p.tiles.buf) ? p.tiles.cnt + slot * (size_t)p.tiles.cnt_stride : nullptr;
  v.tcap = p.tiles.cap;
  v.mcount = (p.h_all && p.use_mcount) ? p.h_all + slot * kSlotWords + kSlotMcount : nullptr;
  v.S = p.S + (slot * kMaxChunks + (size_t)v.d.chunk_begin) * kHistBins;
  v.chunk_off = p.chunk_off + v.d.chunk_begin;
  v.list = p.list + v.d.list_base;
  v.idx_out = p.idx_out + v.d.koff;
  v.vals_row = p.vals_row ? p.vals_row + v.d.koff : nullptr;
  return v;
}

// ---------------------------------------------------------------------------
// k_fill_zero : clears three word ranges (any may be empty); if leader_dev is
// given it also records a leader that the host already knows.
// ---------------------------------------------------------------------------
__global__ void __launch_bounds__(256)
k_fill_zero(uint32_t* __restrict__ p1, size_t words1, uint32_t* __restrict__ p2, size_t words2,
            uint32_t* __restrict__ p3, size_t words3, int32_t leader, int32_t* __restrict__ leader_dev, int32_t* __restrict__ leader_out) {
  if (leader_dev != nullptr && blockIdx.x == 0 && threadIdx.x == 0) {
    *leader_dev = leader;
    if (leader_out) *leader_out = leader;
  }
  const size_t stride = (size_t)gridDim.x * 256;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < words1; i += stride) p1[i] = 0u;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < words2; i += stride) p2[i] = 0u;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < words3; i += stride) p3[i] = 0u;
}

// ---------------------------------------------------------------------------
// k_pass_a : acc = g + residual (in place over residual), variance partials,
//            and the histograms the selection needs from this pass.
//   grid = (nchunks, W), block = T; block (c, w) owns chunk c of worker w.
//   HIST: 0 nothing for the selection, 1 only for worker `hist_worker` (slot 0),
//         2 for every worker (worker w in slot w): per-chunk top-digit suffix
//         histograms S[slot][c] and the whole-vector histogram of the slot.
//   STATS: 0 none, 1 variance partials of acc, 2 of the raw gradient g: the
//   block's (count, mean, sum of squared deviations) in float64 (see VarAcc).
//   NT: non-temporal loads of g and stores of acc.
// ---------------------------------------------------------------------------
constexpr int kPassAUnroll = 4;

template <int STATS, int HIST, bool NT, int GT, int T, int U>
__global__ void __launch_bounds__(T)
k_pass_a(PtrTable g, PtrTable res, int64_t n, ChunkGeom geom, int hist_worker, uint32_t* __restrict__ S,
         uint32_t* __restrict__ h_all, double* __restrict__ partials) {
  constexpr bool LH = HIST != 0;  // an LDS histogram is built
  __shared__ __attribute__((aligned(16))) uint32_t lh[LH ? kHistBins : 4];
  __shared__ uint32_t red_u[LH ? T : 1];

  // with a known leader its blocks (the only ones that work for the selection) are dispatched first
  const int w = (HIST == 1) ? (int)((blockIdx.y + (unsigned)hist_worker) % gridDim.y) : (int)blockIdx.y;
  const int c = blockIdx.x;
  const int nblk = gridDim.x;
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const float* __restrict__ gp = g.p[w];
  float* __restrict__ rp = res.p[w];
  const bool do_hist = (HIST == 2) || (HIST == 1 && w == hist_worker);
  const size_t slot = (HIST == 2) ? (size_t)w : 0;

  if (LH) {
    if (do_hist)
      for (int b = tid; b < kHistBins; b += T) lh[b] = 0u;
    __syncthreads();
  }

  const int64_t c_lo = geom.chunk0 + (int64_t)c * geom.chunk_elems;
  int64_t c_hi = c_lo + geom.chunk_elems;
  if (c_hi > n) c_hi = n;
  const int64_t q_hi = c_hi >> 2;  // whole float4 groups of this chunk

  VarAcc va;

  // One tile: U rows of T float4 groups; the wave's rows start at group qw (a multiple of 64).
  // FULL: every group of the wave's rows lies inside the chunk, so nothing is predicated.
  auto tile = [&](const int64_t qw, auto full_tag) {
    constexpr bool FULL = decltype(full_tag)::value;
    v4f a[U], b[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      // groups outside the chunk re-read its last group (unused): no branch between the loads,
      // so that all of them are in flight together
      const int64_t q = qw + lane + u * T;
      const int64_t ql = (FULL || q < q_hi) ? q : q_hi - 1;
      a[u] = load4g<NT, GT>(gp, 4 * ql);
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {  // (one array after the other: see k_pass_mark)
      const int64_t q = qw + lane + u * T;
      const int64_t ql = (FULL || q < q_hi) ? q : q_hi - 1;
      b[u] = load4<NT>(rp + 4 * ql);
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int64_t q = qw + lane + u * T;
      const bool valid = FULL || q < q_hi;
      if (valid) {
        v4f v;
        v.x = a[u].x + b[u].x;
        v.y = a[u].y + b[u].y;
        v.z = a[u].z + b[u].z;
        v.w = a[u].w + b[u].w;
        store4<NT>(rp + 4 * q, v);
        if (STATS) {  // of the raw gradient, or of the error-fed value
          if (u == 0) va.seed4(STATS == 2 ? a[u] : v);
          va.add4(STATS == 2 ? a[u] : v);
        }
        if (LH) {
          if (do_hist) {
            atomicAdd(&lh[(__float_as_uint(v.x) & kKeyMask) >> 19], 1u);
            atomicAdd(&lh[(__float_as_uint(v.y) & kKeyMask) >> 19], 1u);
            atomicAdd(&lh[(__float_as_uint(v.z) & kKeyMask) >> 19], 1u);
            atomicAdd(&lh[(__float_as_uint(v.w) & kKeyMask) >> 19], 1u);
          }
        }
      }
    }
  };

  // the loop runs on the wave's first group, so all 64 lanes stay together
  const int64_t qw0 = (c_lo >> 2) + __builtin_amdgcn_readfirstlane(tid - lane);
  int64_t qw = qw0;
  for (; qw + (int64_t)(U - 1) * T + 64 <= q_hi; qw += T * U) tile(qw, std::true_type{});
  if (qw < q_hi) tile(qw, std::false_type{});
  // scalar tail (n not a multiple of 4): the block that owns the last chunk
  if (c_hi == n) {
    const int64_t j = (n >> 2) * 4 + tid;
    if (j < n) {
      const float gj = load1g<GT>(gp, j);
      const float v = gj + rp[j];
      rp[j] = v;
      if (STATS) {
        va.seed1(STATS == 2 ? gj : v);
        va.add1(STATS == 2 ? gj : v);
      }
      if (LH) {
        if (do_hist) atomicAdd(&lh[(__float_as_uint(v) & kKeyMask) >> 19], 1u);
      }
    }
  }

  if (STATS) block_moments<T>(va, partials, w, nblk, c);
  if (LH) {
    if (do_hist) {
      // many blocks add to the same few hundred bins: spread them over kHistReps partial copies
      flush_suffix_hist<T>(lh, red_u, S + (slot * kMaxChunks + (size_t)c) * kHistBins,
                           h_all + slot * kSlotWords + (size_t)(c % kHistReps) * kHistBins);
    }
  }
}

// ---------------------------------------------------------------------------
// k_pass_mark : the fused pass of the route with a guessed threshold bound:
//   acc = g + residual (in place over residual), variance partials (STATS as in
//   k_pass_a), and, instead of histograms, one bit per element: elements whose
//   key reaches the guessed bound of the worker's slot are marked in the slot's
//   bit mask and counted per chunk of the selection's chunk layout.
//   grid = (gx, W'), block = T; block (b, y) works on worker y (slot y) and takes
//   the tiles b, b + gx, b + 2 gx, ... of T U float4 groups, so that at any time
//   the blocks in flight read and write one contiguous window of each array
//   (measured 4 to 10 % faster than one contiguous chunk per block).
//   Mask layout: for every row of 64 float4 groups four 64-bit words, word e,
//   bit l <=> element 4 (64 row + l) + e is marked; the words of a tile are
//   ordered so that each wave writes the 32 words of its 8 rows as one 256-byte
//   piece (mask_word() gives the place; 32-byte pieces per row cost the pass 4 %).
//   The n mod 4 elements behind the last whole group are counted (in the last
//   chunk) but have no mask bit.
//   Counts: every wave adds its tile's count to mcount[chunk of the tile] in the
//   slot (cleared beforehand); chunk_elems must be a whole number of tiles.
//   Variance partials: block b of worker y (see VarAcc).
//   PLAIN: no bound is read and nothing is counted: the error-feedback add and the
//   statistics in the same striding order, for a step whose selection builds its own
//   histograms afterwards (long segmented vectors).  The ballots and the mask words
//   (zero, but for Inf and NaN) stay: without them the same pass streamed slower on
//   8 x 1e9 elements, 16.6 against 16.1 ms.
//   STAGE: the marked elements of a tile are also handed on as list entries
//   (index, raw bits), in ascending element order: ranked inside the block (the
//   128 row counts of the tile are scanned by every wave), collected in on-chip
//   memory and stored as one contiguous piece to tiles.buf[tile][0 .. count), with
//   tiles.cnt[tile] = count.  A tile with more marks than tiles.cap entries stores
//   none and reports kTileOverflow; its marks are still in the mask.  Whoever
//   builds the survivor list then copies the pieces instead of fetching the marked
//   values one by one.  In a tile that hands its marks on, the marked elements are
//   stored to the residual as +0.0 straight away: nearly all of them will be kept,
//   and the others get their values back from the list once the threshold is known
//   (see from_pieces(); restore_pieces() does it for all of them if the guess does
//   not hold).
// ---------------------------------------------------------------------------
// Inclusive prefix sums over the 64 lanes of a wave.
__device__ __forceinline__ uint32_t wave_incl_scan(uint32_t v) {
  const int lane = threadIdx.x & 63;
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    const uint32_t x = __shfl_up(v, off, 64);
    if (lane >= off) v += x;
  }
  return v;
}

// First of the four mask words of row `row` (256 elements) of a vector: tiles of 128 rows, inside a
// tile row r belongs to wave r mod 16 as its (r / 16)-th row.
__device__ __forceinline__ int64_t mask_word(int64_t row) {
  return (row >> 7) * 512 + (row & 15) * 32 + ((row >> 4) & 7) * 4;
}

template <int STATS, bool NT, int GT, int T, int U, bool STAGE, bool PLAIN = false>
__global__ void __launch_bounds__(T)
k_pass_mark(PtrTable g, PtrTable res, int64_t n, int64_t chunk_elems, uint32_t* __restrict__ h_all,
            uint64_t* __restrict__ mask, int64_t mask_stride, double* __restrict__ partials, TileBuf tiles) {
  static_assert(!(PLAIN && STAGE), "nothing is marked in the plain form");
  __shared__ uint32_t wcnt[STAGE ? (T / 64) * U : 1];  // the tile's 128 row counts, row-major
  __shared__ uint2 stage[STAGE ? kStageMax : 1];
  const int w = blockIdx.y;
  const int bx = blockIdx.x;
  const int nblk = gridDim.x;
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const float* __restrict__ gp = g.p[w];
  float* __restrict__ rp = res.p[w];
  uint32_t* __restrict__ slot = h_all + (size_t)w * kSlotWords;
  uint32_t* __restrict__ mcount = slot + kSlotMcount;
  uint64_t* __restrict__ mrow = mask + (size_t)w * (size_t)mask_stride;

  // Marked <=> not (|acc| < bound): the same as key >= bound on the magnitude bits, NaNs included.
  const uint32_t gkey = PLAIN ? kNoGuess : slot[kSlotCtrl + 1];
  const float gf = gkey != kNoGuess ? __uint_as_float(gkey) : __builtin_inff();

  const int64_t q_hi = n >> 2;  // whole float4 groups of the vector
  constexpr int64_t TQ = (int64_t)T * U;  // groups per tile
  const int64_t ntiles = (q_hi + TQ - 1) / TQ;

  VarAcc va;
  const int wave_first = __builtin_amdgcn_readfirstlane(tid - lane);
  static_assert(T == 1024 && U == 8, "mask_word() is laid out for 16 waves x 8 rows");
  const int wave = wave_first >> 6;
  uint2* __restrict__ tbuf = STAGE ? tiles.buf + (size_t)w * (size_t)tiles.buf_stride : nullptr;
  uint32_t* __restrict__ tcnt = STAGE ? tiles.cnt + (size_t)w * (size_t)tiles.cnt_stride : nullptr;
  // STAGE: what a lane keeps of a tile until its marks are ranked
  uint32_t own = 0u;      // bit 4 u + e: element e of this lane's group in row u is marked
  uint32_t rows_cnt = 0u; // lane u < U: marks of the wave's row u
  uint32_t bits[STAGE ? U : 1][4];

  // One tile: U rows of T float4 groups; the wave's rows start at group qw (a multiple of 64).
  // FULL: every group of the tile lies inside the vector, so nothing is predicated.
  auto tile = [&](const int64_t qw, auto full_tag) {
    constexpr bool FULL = decltype(full_tag)::value;
    v4f a[U], b[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      // groups outside the vector re-read its last group (unused): no branch between the loads,
      // so that all of them are in flight together
      const int64_t q = qw + lane + u * T;
      const int64_t ql = (FULL || q < q_hi) ? q : q_hi - 1;
      a[u] = load4g<NT, GT>(gp, 4 * ql);
    }
    // The tile's gradient loads first, then its residual loads: issued alternately (g, r, g, r, ...)
    // the same pass took 16.04 instead of 15.72 ms on 8 x 1e9 elements (residual first: 15.77).
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int64_t q = qw + lane + u * T;
      const int64_t ql = (FULL || q < q_hi) ? q : q_hi - 1;
      b[u] = load4<NT>(rp + 4 * ql);
    }
    uint32_t marked = 0u;  // of this wave in this tile
    uint64_t mine = 0ull;  // lane 4 u + e keeps word e of the wave's row u
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int64_t q = qw + lane + u * T;
      const bool valid = FULL || q < q_hi;
      v4f v = {0.f, 0.f, 0.f, 0.f};
      if (valid) {
        v.x = a[u].x + b[u].x;
        v.y = a[u].y + b[u].y;
        v.z = a[u].z + b[u].z;
        v.w = a[u].w + b[u].w;
        if (!STAGE) store4<NT>(rp + 4 * q, v);  // (STAGE stores below, the marked elements as +0.0)
        if (STATS) {  // of the raw gradient, or of the error-fed value
          if (u == 0) va.seed4(STATS == 2 ? a[u] : v);
          va.add4(STATS == 2 ? a[u] : v);
        }
      }
      const uint64_t m0 = __ballot(valid && !(__builtin_fabsf(v.x) < gf));
      const uint64_t m1 = __ballot(valid && !(__builtin_fabsf(v.y) < gf));
      const uint64_t m2 = __ballot(valid && !(__builtin_fabsf(v.z) < gf));
      const uint64_t m3 = __ballot(valid && !(__builtin_fabsf(v.w) < gf));
      const uint32_t row_marked = (uint32_t)(__popcll(m0) + __popcll(m1) + __popcll(m2) + __popcll(m3));
      marked += row_marked;
      if (STAGE) {
        const uint32_t o = (uint32_t)((m0 >> lane) & 1ull) | (uint32_t)((m1 >> lane) & 1ull) << 1 |
                           (uint32_t)((m2 >> lane) & 1ull) << 2 | (uint32_t)((m3 >> lane) & 1ull) << 3;
        own |= o << (4 * u);
        rows_cnt = lane == u ? row_marked : rows_cnt;
        bits[STAGE ? u : 0][0] = __float_as_uint(v.x);
        bits[STAGE ? u : 0][1] = __float_as_uint(v.y);
        bits[STAGE ? u : 0][2] = __float_as_uint(v.z);
        bits[STAGE ? u : 0][3] = __float_as_uint(v.w);
        if (valid) {
          // The marked elements go out as +0.0: they are survivors, nearly all of which the
          // selection keeps; the list carries their values on, and its final pass puts back the
          // few that are not kept.  (A tile that turns out not to hand its marks on stores them
          // again, below.)
          v4f z;
          z.x = (o & 1u) ? 0.0f : v.x;
          z.y = (o & 2u) ? 0.0f : v.y;
          z.z = (o & 4u) ? 0.0f : v.z;
          z.w = (o & 8u) ? 0.0f : v.w;
          store4<NT>(rp + 4 * q, z);
        }
      }
      mine = lane == 4 * u + 0 ? m0 : mine;
      mine = lane == 4 * u + 1 ? m1 : mine;
      mine = lane == 4 * u + 2 ? m2 : mine;
      mine = lane == 4 * u + 3 ? m3 : mine;
    }
    // rows behind the vector's end get zero words: the mask holds whole tiles
    if (lane < 4 * U) mrow[mask_word(qw >> 6) + lane] = mine;
    return marked;
  };

  for (int64_t ti = bx; ti < ntiles; ti += nblk) {
    const int64_t qw = ti * TQ + wave_first;  // wave-uniform, so all 64 lanes stay together (the masks need that)
    if (STAGE) own = 0u;
    const uint32_t marked = (ti + 1) * TQ <= q_hi ? tile(qw, std::true_type{}) : tile(qw, std::false_type{});
    if (!PLAIN && lane == 0 && marked != 0u) atomicAdd(&mcount[(ti * TQ * 4) / chunk_elems], marked);
    if (STAGE) {
      // rank the tile's marks: element order is row-major, row = 16 u + wave, then lane, then e
      if (lane < U) wcnt[lane * (T / 64) + wave] = rows_cnt;
      __syncthreads();
      const uint32_t c0 = wcnt[lane], c1 = wcnt[64 + lane];  // (every wave scans the 128 counts itself)
      const uint32_t s0 = wave_incl_scan(c0), s1 = wave_incl_scan(c1);
      const uint32_t half = __shfl(s0, 63, 64);
      const uint32_t total = half + __shfl(s1, 63, 64);
      const bool fits = total <= (uint32_t)tiles.cap;
      if (!fits) {  // rare: the marks stay in the mask only, so their values go back into the vector
#pragma unroll
        for (int u = 0; u < U; ++u) {
          if (((own >> (4 * u)) & 0xfu) != 0u) {
            const int64_t q = qw + lane + u * T;
            v4f v;
            v.x = __uint_as_float(bits[STAGE ? u : 0][0]);
            v.y = __uint_as_float(bits[STAGE ? u : 0][1]);
            v.z = __uint_as_float(bits[STAGE ? u : 0][2]);
            v.w = __uint_as_float(bits[STAGE ? u : 0][3]);
            store4<NT>(rp + 4 * q, v);
          }
        }
        if (tid == 0) atomicOr(&slot[kSlotCtrl + 2], 1u);
      }
      if (fits && total != 0u) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
          const int r = u * (T / 64) + wave;  // this wave's row u among the tile's 128
          // marks in the rows before it
          const uint32_t before = r < 64 ? __shfl(s0 - c0, r, 64) : half + __shfl(s1 - c1, r - 64, 64);
          const uint64_t b0 = __ballot((own >> (4 * u + 0)) & 1u), b1 = __ballot((own >> (4 * u + 1)) & 1u);
          const uint64_t b2 = __ballot((own >> (4 * u + 2)) & 1u), b3 = __ballot((own >> (4 * u + 3)) & 1u);
          if (((own >> (4 * u)) & 0xfu) != 0u) {
            uint32_t pos = before + popc_lt(b0) + popc_lt(b1) + popc_lt(b2) + popc_lt(b3);
            const uint32_t j0 = (uint32_t)(4 * (qw + lane + u * T));
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              if ((own >> (4 * u + e)) & 1u) {
                stage[pos] = make_uint2(j0 + (uint32_t)e, bits[STAGE ? u : 0][e]);
                ++pos;
              }
            }
          }
        }
      }
      __syncthreads();
      if (fits) {
        uint2* __restrict__ dst = tbuf + (size_t)ti * (size_t)tiles.cap;
        for (uint32_t i = (uint32_t)tid; i < total; i += T) dst[i] = stage[i];
      }
      if (tid == 0) tcnt[ti] = fits ? total : kTileOverflow;
      // (the next tile writes wcnt before its first barrier and stage behind it: both are free by then)
    }
  }
  // scalar tail (n not a multiple of 4): the first block
  if (bx == 0) {
    const int64_t j = q_hi * 4 + tid;
    if (j < n) {
      const float gj = load1g<GT>(gp, j);
      const float v = gj + rp[j];
      rp[j] = v;
      if (STATS) {
        va.seed1(STATS == 2 ? gj : v);
        va.add1(STATS == 2 ? gj : v);
      }
      if (!PLAIN && !(__builtin_fabsf(v) < gf)) atomicAdd(&mcount[(n - 1) / chunk_elems], 1u);
    }
  }

  if (STATS) block_moments<T>(va, partials, w, nblk, bx);
}

// ---------------------------------------------------------------------------
// k_stats : statistics of read-only vectors in float64.  grid = (nblk, W).
//   SHIFT (variance): the block's (count, mean, sum of squared deviations), see VarAcc.
//   !SHIFT (sum of squares): the block's sum of x and of x^2 to partials[w][b][0..1].
// VEC reads float4 groups (rows must be 16-byte aligned).
// ---------------------------------------------------------------------------
template <bool SHIFT, bool VEC>
__global__ void __launch_bounds__(256)
k_stats(PtrTable x, int64_t n, double* __restrict__ partials) {
  __shared__ double red[3 * 4];
  const int w = blockIdx.y, bx = blockIdx.x, nblk = gridDim.x, tid = threadIdx.x;
  const float* __restrict__ xp = x.p[w];
  const int64_t n4 = VEC ? (n >> 2) : 0;
  VarAcc va;                 // SHIFT
  double s = 0.0, ss = 0.0;  // !SHIFT
  if (VEC) {
    const v4f* __restrict__ x4 = reinterpret_cast<const v4f*>(xp);
    const int64_t tile = 256 * kPassAUnroll;
    const int64_t ntile = (n4 + tile - 1) / tile;
    for (int64_t t = bx; t < ntile; t += nblk) {
      const int64_t q0 = t * tile + tid;
      v4f a[kPassAUnroll];
#pragma unroll
      for (int u = 0; u < kPassAUnroll; ++u) {
        const int64_t q = q0 + u * 256;
        if (q < n4) a[u] = x4[q];
      }
#pragma unroll
      for (int u = 0; u < kPassAUnroll; ++u) {
        const int64_t q = q0 + u * 256;
        if (q < n4) {
          if (SHIFT) {
            if (u == 0) va.seed4(a[u]);
            va.add4(a[u]);
          } else {
            const double d0 = (double)a[u].x, d1 = (double)a[u].y, d2 = (double)a[u].z, d3 = (double)a[u].w;
            s += (d0 + d1) + (d2 + d3);
            ss = fma(d0, d0, ss);
            ss = fma(d1, d1, ss);
            ss = fma(d2, d2, ss);
            ss = fma(d3, d3, ss);
          }
        }
      }
    }
  }
  // elements not covered by whole float4 groups (all of them when the row is not 16-byte aligned)
  for (int64_t j = n4 * 4 + (int64_t)bx * 256 + tid; j < n; j += (int64_t)nblk * 256) {
    if (SHIFT) {
      va.seed1(xp[j]);
      va.add1(xp[j]);
    } else {
      const double d = (double)xp[j];
      s += d;
      ss = fma(d, d, ss);
    }
  }
  if (SHIFT) {
    block_moments<256>(va, partials, w, nblk, bx);
  } else {
    s = wave_sum(s);
    ss = wave_sum(ss);
    if ((tid & 63) == 0) {
      red[tid >> 6] = s;
      red[4 + (tid >> 6)] = ss;
    }
    __syncthreads();
    if (tid == 0) {
      partials[((size_t)w * nblk + bx) * 2 + 0] = (red[0] + red[1]) + (red[2] + red[3]);
      partials[((size_t)w * nblk + bx) * 2 + 1] = (red[4] + red[5]) + (red[6] + red[7]);
    }
  }
}

// ---------------------------------------------------------------------------
// k_gain : one block.  gain_w = V_w / (V_w + R_w) with V_w, R_w the sums of
// squares (second partial of every block) of worker w's gathered values and of
// its residual after the step; the two have disjoint support, so V_w + R_w is
// the squared norm of the error-fed gradient.
// ---------------------------------------------------------------------------
__global__ void __launch_bounds__(1024)
k_gain(const double* __restrict__ part_vals, int nblk_vals, const double* __restrict__ part_res, int nblk_res,
       int w_count, double* __restrict__ gain_out) {
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  for (int w = wave; w < w_count; w += 16) {
    double v = 0.0, r = 0.0;
    for (int b = lane; b < nblk_vals; b += 64) v += part_vals[((size_t)w * nblk_vals + b) * 2 + 1];
    for (int b = lane; b < nblk_res; b += 64) r += part_res[((size_t)w * nblk_res + b) * 2 + 1];
    v = wave_sum(v);
    r = wave_sum(r);
    if (lane == 0) gain_out[w] = (v + r > 0.0) ? v / (v + r) : 0.0;
  }
}

// ---------------------------------------------------------------------------
// k_sqnorm : one block.  out[w] = sum of the second partials (sums of squares)
// of vector w; argmax = first w with the largest value (also stored as leader).
// ---------------------------------------------------------------------------
__global__ void __launch_bounds__(1024)
k_sqnorm(const double* __restrict__ part, int nblk, int w_count, double* __restrict__ scratch,
         double* __restrict__ out, int32_t* __restrict__ leader_dev, int32_t* __restrict__ argmax_out) {
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  for (int w = wave; w < w_count; w += 16) {
    double v = 0.0;
    for (int b = lane; b < nblk; b += 64) v += part[((size_t)w * nblk + b) * 2 + 1];
    v = wave_sum(v);
    if (lane == 0) {
      scratch[w] = v;
      if (out) out[w] = v;
    }
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    int best = 0;
    for (int w = 1; w < w_count; ++w)
      if (scratch[w] > scratch[best]) best = w;
    if (leader_dev) *leader_dev = best;
    if (argmax_out) *argmax_out = best;
  }
}

__global__ void __launch_bounds__(256)
k_copy_i32(const int32_t* __restrict__ src_rows, const int32_t* __restrict__ row_dev, int64_t k,
           int32_t* __restrict__ dst) {
  const int64_t m = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (m < k) dst[m] = src_rows[(size_t)(*row_dev) * (size_t)k + (size_t)m];
}

// ---------------------------------------------------------------------------
// k_apply_update : w[idx[m]] = w[idx[m]] - eta * sum[m] (one float32 multiply,
// one float32 subtract), the sparse form of the model update.
// ---------------------------------------------------------------------------
__global__ void __launch_bounds__(256)
k_apply_update(float* __restrict__ weights, int64_t n, const int32_t* __restrict__ idx,
               const float* __restrict__ sum, int64_t k, float eta, uint32_t* __restrict__ err) {
  const int64_t m = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (m >= k) return;
  const int64_t i = (int64_t)idx[m];
  if (i < 0 || i >= n) {
    atomicOr(err, kErrIndex);
    return;
  }
  const float step = eta * sum[m];
  weights[i] = weights[i] - step;
}

// ---------------------------------------------------------------------------
// k_leader : one block of 1024 threads.  Merges the per-block moments of every
// worker in a fixed order, var_w = M2 / n, leader = first argmax.
// ---------------------------------------------------------------------------
__global__ void __launch_bounds__(1024)
k_leader(const double* __restrict__ partials, int w_count, int nblk, int64_t n,
         double* __restrict__ var_scratch, double* __restrict__ var_out,
         int32_t* __restrict__ leader_dev, int32_t* __restrict__ leader_out) {
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  for (int w = wave; w < w_count; w += 16) {
    const double v = wave_variance(partials, w, nblk);
    if (lane == 0) {
      var_scratch[w] = v;
      if (var_out) var_out[w] = v;
    }
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    int best = 0;
    for (int w = 1; w < w_count; ++w)
      if (var_scratch[w] > var_scratch[best]) best = w;
    *leader_dev = best;
    if (leader_out) *leader_out = best;
  }
}

__global__ void k_set_leader(int32_t leader, int32_t* __restrict__ leader_dev, int32_t* __restrict__ leader_out) {
  if (threadIdx.x == 0 && blockIdx.x == 0) {
    *leader_dev = leader;
    if (leader_out) *leader_out = leader;
  }
}

// The round-robin leader from the iteration counter kept on the device (Alg. 1,
// STAR branch): leader = counter mod w, then the counter moves on by one.
__global__ void k_counter_leader(uint64_t* __restrict__ counter, int32_t w, int32_t* __restrict__ leader_dev,
                                 int32_t* __restrict__ leader_out) {
  if (threadIdx.x == 0 && blockIdx.x == 0) {
    const uint64_t c = *counter;
    const int32_t leader = (int32_t)(c % (uint64_t)w);
    *leader_dev = leader;
    if (leader_out) *leader_out = leader;
    *counter = c + 1u;
  }
}

__global__ void k_set_counter(uint64_t* __restrict__ counter, uint64_t value) {
  if (threadIdx.x == 0 && blockIdx.x == 0) *counter = value;
}

// ---------------------------------------------------------------------------
// k_guess : a lower bound on the key of the k-th largest |g + residual| of each
// vector, from a sample, before the fused pass runs.  grid = (blocks, vectors),
// block = 256; vector y uses slot y.  The sample is `runs` runs of kGuessRun
// consecutive elements, run r starting at (r stride) rounded down to a multiple
// of kGuessRun.  The last block to finish takes the top digit d of the sample's
// m_hi-th largest key and publishes d << 19 (kNoGuess if the sample is smaller
// than m_hi).  The bound is only a guess: whoever uses it checks that at least
// k keys of the whole vector reach it.
//   With sample_keys (vector 0 only: room for runs kGuessRun keys) every block
//   also stores its sample's keys there, for k_guess_refine.
// ---------------------------------------------------------------------------
template <int GT>
__global__ void __launch_bounds__(256)
k_guess(PtrTable g, PtrTable res, uint32_t* __restrict__ slots, int runs, int64_t stride, uint32_t m_hi,
        uint32_t* __restrict__ sample_keys) {
  __shared__ uint32_t lh[kHistBins];
  __shared__ uint32_t wsum[4];
  __shared__ int last_sh, hit_sh;
  __shared__ uint32_t hit_above_sh;
  const int tid = threadIdx.x;
  const int v = blockIdx.y;
  const float* __restrict__ gp = g.p[v];
  const float* __restrict__ rp = res.p[v];
  uint32_t* __restrict__ ghist = slots + (size_t)v * kSlotWords + kSlotGuessHist;
  uint32_t* __restrict__ ctrl = slots + (size_t)v * kSlotWords + kSlotCtrl;
  for (int b = tid; b < kHistBins; b += 256) lh[b] = 0u;
  __syncthreads();
  for (int r = blockIdx.x * 256 + tid; r < runs; r += gridDim.x * 256) {
    const int64_t e0 = ((int64_t)r * stride) & ~(int64_t)(kGuessRun - 1);
    v4f a[kGuessRun / 4], b[kGuessRun / 4];
#pragma unroll
    for (int i = 0; i < kGuessRun / 4; ++i) {
      a[i] = load4g<false, GT>(gp, e0 + 4 * i);
      b[i] = load4<false>(rp + e0 + 4 * i);
    }
#pragma unroll
    for (int i = 0; i < kGuessRun / 4; ++i) {
      uint4 kq;
      kq.x = __float_as_uint(a[i].x + b[i].x) & kKeyMask;
      kq.y = __float_as_uint(a[i].y + b[i].y) & kKeyMask;
      kq.z = __float_as_uint(a[i].z + b[i].z) & kKeyMask;
      kq.w = __float_as_uint(a[i].w + b[i].w) & kKeyMask;
      atomicAdd(&lh[kq.x >> 19], 1u);
      atomicAdd(&lh[kq.y >> 19], 1u);
      atomicAdd(&lh[kq.z >> 19], 1u);
      atomicAdd(&lh[kq.w >> 19], 1u);
      if (sample_keys != nullptr && v == 0) reinterpret_cast<uint4*>(sample_keys + (size_t)r * kGuessRun)[i] = kq;
    }
  }
  __syncthreads();
  for (int b = tid; b < kHistBins; b += 256) {
    const uint32_t c = lh[b];
    if (c) atomicAdd(&ghist[b], c);
  }
  __threadfence();
  __syncthreads();
  if (tid == 0) {
    last_sh = atomicAdd(&ctrl[0], 1u) == gridDim.x - 1 ? 1 : 0;
    hit_sh = -1;
  }
  __syncthreads();
  if (!last_sh) return;
  __threadfence();
  // the last block: suffix sums over the sample histogram, 16 consecutive bins per thread
  uint32_t h[16];
  uint32_t tot = 0u;
#pragma unroll
  for (int j = 0; j < 16; ++j) {
    h[j] = __hip_atomic_load(&ghist[16 * tid + j], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    tot += h[j];
  }
  // inclusive suffix sum of tot over the 64 lanes, then over the 4 waves
  uint32_t suf = tot;
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    const uint32_t x = __shfl_down(suf, off, 64);
    if ((tid & 63) + off < 64) suf += x;
  }
  if ((tid & 63) == 0) wsum[tid >> 6] = suf;
  __syncthreads();
  uint32_t above = suf - tot;  // bins of higher threads in this wave
  for (int i = (tid >> 6) + 1; i < 4; ++i) above += wsum[i];
#pragma unroll
  for (int j = 15; j >= 0; --j) {
    if (above < m_hi && above + h[j] >= m_hi) {  // one thread, one bin
      hit_sh = 16 * tid + j;
      hit_above_sh = above;
    }
    above += h[j];
  }
  __syncthreads();
  const int hit = hit_sh;
  // bounds above infinity's digit would not survive the floating-point comparison of the fused pass
  const uint32_t bound = hit >= 0 ? (uint32_t)(hit < 0xff0 ? hit : 0xff0) << 19 : kNoGuess;
  if (tid == 0) {
    ctrl[3] = (hit >= 0 && hit < 0xff0) ? (uint32_t)hit : kNoGuess;  // (what k_guess_refine may refine)
    ctrl[4] = hit_above_sh;
  }
  if (tid == 0) ctrl[1] = bound;
}

// ---------------------------------------------------------------------------
// k_guess_refine : refines the bound k_guess published for vector 0 by the next 12
// key bits: among the stored sample keys of the bound's top digit d it takes the
// second digit of the key that is m_hi-th largest in the whole sample.  A bound
// this fine admits about 1 % more keys than needed (plus the margin in m_hi)
// instead of up to 15 %.  grid = blocks of 256 threads striding over the nkeys
// sample keys; the last block to finish picks.
// ---------------------------------------------------------------------------
__global__ void __launch_bounds__(256)
k_guess_refine(uint32_t* __restrict__ slots, const uint32_t* __restrict__ sample_keys, int nkeys, uint32_t m_hi) {
  __shared__ uint32_t lh[kHistBins];
  __shared__ uint32_t wsum[4];
  __shared__ int last_sh, hit_sh;
  const int tid = threadIdx.x;
  uint32_t* __restrict__ ctrl = slots + kSlotCtrl;
  uint32_t* __restrict__ hist = slots + kSlotRefine;
  const uint32_t d0 = ctrl[3];
  if (d0 == kNoGuess) return;  // (the same in every block)
  for (int b = tid; b < kHistBins; b += 256) lh[b] = 0u;
  __syncthreads();
  const uint4* __restrict__ sk = reinterpret_cast<const uint4*>(sample_keys);
  for (int q = blockIdx.x * 256 + tid; q < nkeys / 4; q += gridDim.x * 256) {
    const uint4 kq = sk[q];
    if ((kq.x >> 19) == d0) atomicAdd(&lh[(kq.x >> 7) & 0xfffu], 1u);
    if ((kq.y >> 19) == d0) atomicAdd(&lh[(kq.y >> 7) & 0xfffu], 1u);
    if ((kq.z >> 19) == d0) atomicAdd(&lh[(kq.z >> 7) & 0xfffu], 1u);
    if ((kq.w >> 19) == d0) atomicAdd(&lh[(kq.w >> 7) & 0xfffu], 1u);
  }
  __syncthreads();
  for (int b = tid; b < kHistBins; b += 256) {
    const uint32_t c = lh[b];
    if (c) atomicAdd(&hist[b], c);
  }
  __threadfence();
  __syncthreads();
  if (tid == 0) {
    last_sh = atomicAdd(&ctrl[5], 1u) == gridDim.x - 1 ? 1 : 0;
    hit_sh = -1;
  }
  __syncthreads();
  if (!last_sh) return;
  __threadfence();
  uint32_t h[16];
  uint32_t tot = 0u;
#pragma unroll
  for (int j = 0; j < 16; ++j) {
    h[j] = __hip_atomic_load(&hist[16 * tid + j], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    tot += h[j];
  }
  uint32_t suf = tot;
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    const uint32_t x = __shfl_down(suf, off, 64);
    if ((tid & 63) + off < 64) suf += x;
  }
  if ((tid & 63) == 0) wsum[tid >> 6] = suf;
  __syncthreads();
  uint32_t above = ctrl[4] + suf - tot;  // sample keys of higher top digit, or of higher second digit
  for (int i = (tid >> 6) + 1; i < 4; ++i) above += wsum[i];
#pragma unroll
  for (int j = 15; j >= 0; --j) {
    if (above < m_hi && above + h[j] >= m_hi) hit_sh = 16 * tid + j;  // one thread, one bin
    above += h[j];
  }
  __syncthreads();
  if (tid == 0 && hit_sh >= 0) ctrl[1] = (d0 << 19) | ((uint32_t)hit_sh << 7);
}

// ---------------------------------------------------------------------------
// k_hist0 : per-chunk top-digit suffix histograms of |x[e_lo .. e_hi)| for the
// leader's vector.  grid = (max chunks of a segment, segments), block = T (1024:
// there are at most about a thousand blocks, so a block must keep many loads in flight).
// Whole aligned float4 groups are read where they lie inside the array, single
// elements at its ragged end; elements outside the chunk are masked out.
// ---------------------------------------------------------------------------
// The guess did not hold after a fused pass that handed marked elements on per tile and stored
// +0.0 in their place: the block that owns chunk c puts the values of its tiles' pieces back into
// the vector before anything reads it (chunks are whole tiles on this route, so this is local to
// the block; the caller's barrier and this fence order it before the block's own reads).
template <int T>
__device__ __forceinline__ void restore_pieces(const SelParams& p, const SegView& sv, int c) {
  const int64_t c_begin = sv.d.geom.chunk0 + (int64_t)c * sv.d.geom.chunk_elems;
  int64_t c_end = c_begin + sv.d.geom.chunk_elems;
  if (c_end > (p.n & ~(int64_t)3)) c_end = p.n & ~(int64_t)3;
  for (int64_t t = c_begin / kPassTile; t * kPassTile < c_end; ++t) {
    const uint32_t cnt = sv.tcnt[t];
    if (cnt == kTileOverflow) continue;
    const uint2* __restrict__ piece = sv.tbuf + (size_t)t * (size_t)sv.tcap;
    for (uint32_t e = threadIdx.x; e < cnt; e += T) {
      const uint2 ent = piece[e];
      if ((int64_t)ent.x < p.n) p.zero_vec[ent.x] = __uint_as_float(ent.y);
    }
  }
  __threadfence();
}

template <int T>
__device__ __forceinline__ void hist0_body(const SelParams& p) {
  __shared__ __attribute__((aligned(16))) uint32_t lh[kHistBins];
  __shared__ uint32_t red_u[T];
  int seg, c;
  block_chunk(p, seg, c);
  const SegView sv = seg_view(p, seg);
  if (c >= sv.d.geom.nchunks) return;
  if (p.only_if_need_full && sv.st->need_full == 0u) return;
  const int tid = threadIdx.x;
  const float* __restrict__ xp = sv.x;
  for (int b = tid; b < kHistBins; b += T) lh[b] = 0u;
  if (sv.tbuf != nullptr && p.zero_vec != nullptr) restore_pieces<T>(p, sv, c);
  __syncthreads();
  int64_t cs = sv.d.geom.chunk0 + (int64_t)c * sv.d.geom.chunk_elems;
  int64_t ce = cs + sv.d.geom.chunk_elems;
  if (cs < sv.d.e_lo) cs = sv.d.e_lo;
  if (ce > sv.d.e_hi) ce = sv.d.e_hi;
  const int64_t n_vec = p.n & ~(int64_t)3;
  const int64_t q_lo = cs >> 2;
  const int64_t q_hi = (ce + 3) >> 2;  // exclusive
  for (int64_t q0 = q_lo + tid; q0 < q_hi; q0 += T * 4) {
    uint4 v[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {  // whole groups inside the array are read as one vector
      const int64_t j = (q0 + u * T) << 2;
      v[u] = make_uint4(0u, 0u, 0u, 0u);
      if (q0 + u * T < q_hi) {
        if (j + 4 <= n_vec) {
          v[u] = *reinterpret_cast<const uint4*>(xp + j);
        } else {
          v[u].x = (j + 0 < p.n) ? __float_as_uint(xp[j + 0]) : 0u;
          v[u].y = (j + 1 < p.n) ? __float_as_uint(xp[j + 1]) : 0u;
          v[u].z = (j + 2 < p.n) ? __float_as_uint(xp[j + 2]) : 0u;
          v[u].w = (j + 3 < p.n) ? __float_as_uint(xp[j + 3]) : 0u;
        }
      }
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int64_t j = (q0 + u * T) << 2;
      if (q0 + u * T < q_hi) {
        const uint32_t kk[4] = {v[u].x, v[u].y, v[u].z, v[u].w};
#pragma unroll
        for (int e = 0; e < 4; ++e)
          if (j + e >= cs && j + e < ce) atomicAdd(&lh[(kk[e] & kKeyMask) >> 19], 1u);
      }
    }
  }
  flush_suffix_hist<T>(lh, red_u, sv.S + (size_t)c * kHistBins, sv.htop);
}

template <int T>
__global__ void __launch_bounds__(T)
k_hist0(SelParams p) {
  hist0_body<T>(p);
}

// ---------------------------------------------------------------------------
// Selection state machine.  k_pick0 writes the state after the top digit (level
// 1) and decides whether the level-1 survivors fit the list.  Nothing else
// writes the state: later kernels replay the remaining digit picks from the
// next-digit histograms in their prologue (derive_state), every block for
// itself -- the result is a pure function of hist1 / hist2, so all blocks agree
// and no extra launches are needed.
// ---------------------------------------------------------------------------
__device__ __forceinline__ bool fits_list(const SelState& st, uint32_t cap) {
  return (uint64_t)st.n_gt + (uint64_t)st.cand <= (uint64_t)cap;
}

// Narrows st (in shared memory) by digit `digit` (1 or 2) using the histogram of
// that digit over the current candidates.  All T threads of the block call it;
// `part` is T words of shared memory.
template <int T>
__device__ void block_pick(SelState& st, const uint32_t* __restrict__ hist, int digit, uint32_t* part,
                           uint32_t* __restrict__ err) {
  constexpr int BPT = kHistBins / T;
  const int t = threadIdx.x;
  const int nbins = (int)digit_mask(digit) + 1;
  uint32_t h[BPT];
  uint32_t tot = 0u;
#pragma unroll
  for (int j = 0; j < BPT; ++j) {
    const int b = BPT * t + j;
    h[j] = (b < nbins) ? hist[b] : 0u;
    tot += h[j];
  }
  __syncthreads();  // st is stable and `part` is free
  uint32_t total;
  uint32_t above = block_suffix_incl<T>(tot, part, &total) - tot;
  const uint32_t need = st.need;
  int hit = -1;
  uint32_t hit_above = 0u, hit_cnt = 0u;
#pragma unroll
  for (int j = BPT - 1; j >= 0; --j) {
    if (hit < 0 && above < need && need <= above + h[j]) {
      hit = BPT * t + j;
      hit_above = above;
      hit_cnt = h[j];
    }
    above += h[j];
  }
  __syncthreads();  // every thread has read st.need
  if (hit >= 0) {   // exactly one thread when the histogram holds >= need keys
    const int sh = digit_shift(digit);
    st.lo = st.lo | ((uint32_t)hit << sh);
    st.hi = st.lo | ((1u << sh) - 1u);
    st.n_gt += hit_above;
    st.need -= hit_above;
    st.cand = hit_cnt;
    st.level = (uint32_t)digit + 1u;
  }
  if (t == 0 && total < need) atomicOr(err, kErrPick);  // histogram does not cover `need`
  __syncthreads();
}

// State at `want_level` (2 or 3) in st (shared).  st.compact_level = the level
// whose pass writes the survivor list (1, 2 or 3), st.list_count its size.
template <int T>
__device__ void derive_state(const SegView& sv, SelState& st, int want_level, uint32_t* part,
                             uint32_t* __restrict__ err) {
  if (threadIdx.x == 0) st = *sv.st;  // level 1; compact_level = 1 if the level-1 survivors fit
  __syncthreads();
  block_pick<T>(st, sv.hist1, 1, part, err);
  if (threadIdx.x == 0 && st.compact_level == 0u) {
    if (fits_list(st, sv.d.cap)) {
      st.compact_level = 2u;
      st.list_count = st.n_gt + st.cand;
    } else {
      st.compact_level = 3u;
    }
  }
  __syncthreads();
  if (want_level >= 3) {
    block_pick<T>(st, sv.hist2, 2, part, err);
    if (threadIdx.x == 0 && st.compact_level == 3u) st.list_count = st.n_gt + (st.cand < st.need ? st.cand : st.need);
    __syncthreads();
  }
}

// ---------------------------------------------------------------------------
// k_pick0 : one block of 1024 threads per segment.  Optionally first finishes
// the per-worker variances and takes the leader (flat VAR step).  Then: suffix
// sums of the top-digit histogram, threshold digit b0 = the largest b with at
// least k keys at or above it, the level-1 state, and for every chunk of the
// segment the offset of its survivors (keys with top digit >= b0) in the list.
// ---------------------------------------------------------------------------
struct LeaderArgs {
  const double* partials;  // nullptr: the leader is already in leader_dev
  int w_count, nblk;
  int64_t n;
  double* var_scratch;
  double* var_out;
  int32_t* leader_dev;
  int32_t* leader_out;
};

// Finishes the per-worker variances from the fused pass' partials and takes the first
// worker of largest variance (same arithmetic as k_leader).  All 1024 threads of the
// block call it; returns the leader in thread 0 only.
__device__ int block_take_leader(const LeaderArgs& la) {
  const int t = threadIdx.x;
  const int wave = t >> 6, lane = t & 63;
  for (int w = wave; w < la.w_count; w += 16) {
    const double v = wave_variance(la.partials, w, la.nblk);
    if (lane == 0) {
      la.var_scratch[w] = v;
      if (la.var_out) la.var_out[w] = v;
    }
  }
  __threadfence_block();
  __syncthreads();
  int best = 0;
  if (t == 0) {
    for (int w = 1; w < la.w_count; ++w)
      if (la.var_scratch[w] > la.var_scratch[best]) best = w;
    *la.leader_dev = best;
    if (la.leader_out) *la.leader_out = best;
  }
  return best;
}

__global__ void __launch_bounds__(1024)
k_pick0(SelParams p, LeaderArgs la) {
  __shared__ uint32_t part[1024];
  __shared__ int b0_sh;
  __shared__ int lead_sh;
  const int t = threadIdx.x;
  if (t == 0) {
    b0_sh = -1;
    lead_sh = -1;
  }
  if (la.partials != nullptr) {
    const int best = block_take_leader(la);
    if (t == 0) lead_sh = best;
  }
  __syncthreads();
  const SegView sv = seg_view(p, blockIdx.y, lead_sh);
  if (p.only_if_need_full && sv.st->need_full == 0u) return;
  if (p.from_list && sv.st->use_mask == 0u) return;
  const SelState prev = *sv.st;  // from_list: says how long the list is
  bool from_list = p.from_list != 0;
  const uint32_t* __restrict__ htop = sv.htop;
  int htop_reps = sv.htop_reps;
  if (p.after_mask) {  // the list was written from the mask, or k_hist0's work has just been done instead
    if (prev.use_mask != 0u) {
      from_list = true;
    } else if (prev.need_full != 0u) {
      htop = sv.hseg;
      htop_reps = 1;
    } else {
      return;
    }
  }
  const uint32_t k = sv.d.k;
  const int nchunks = sv.d.geom.nchunks;

  // suffix sums of the top-digit histogram: sx[j] = keys with digit >= 4t+j
  uint32_t h[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) h[j] = 0u;
  if (htop_reps == kHistReps) {  // sixteen loads in flight together
    for (int r0 = 0; r0 < kHistReps; r0 += 16) {
      uint4 q[16];
#pragma unroll
      for (int r = 0; r < 16; ++r) q[r] = reinterpret_cast<const uint4*>(htop + (size_t)(r0 + r) * kHistBins)[t];
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        h[0] += q[r].x;
        h[1] += q[r].y;
        h[2] += q[r].z;
        h[3] += q[r].w;
      }
    }
  } else {
    const uint4 q = reinterpret_cast<const uint4*>(htop)[t];
    h[0] = q.x;
    h[1] = q.y;
    h[2] = q.z;
    h[3] = q.w;
  }
  const uint32_t hsum = h[0] + h[1] + h[2] + h[3];
  uint32_t sx[5];
  sx[4] = block_suffix_incl<1024>(hsum, part) - hsum;
#pragma unroll
  for (int j = 3; j >= 0; --j) sx[j] = sx[j + 1] + h[j];
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    if (sx[j] >= k && sx[j + 1] < k) {  // the suffix sums are non-increasing: one hit
      b0_sh = 4 * t + j;
      SelState st{};
      st.lo = (uint32_t)(4 * t + j) << 19;
      st.hi = st.lo | 0x7ffffu;
      st.n_gt = sx[j + 1];
      st.need = k - sx[j + 1];
      st.cand = sx[j] - sx[j + 1];
      st.level = 1u;
      if (from_list) {  // the list exists already and holds every key >= list_lo
        st.compact_level = 1u;
        st.use_mask = 1u;
        st.list_lo = prev.list_lo;
        st.list_count = prev.list_count;
      } else {
        st.compact_level = fits_list(st, sv.d.cap) ? 1u : 0u;
        st.list_count = st.compact_level ? st.n_gt + st.cand : 0u;
      }
      *sv.st = st;
    }
  }
  __syncthreads();
  const int b0 = b0_sh;
  if (b0 < 0) {
    if (t == 0) atomicOr(p.err, kErrPick);
    return;
  }
  if (from_list) return;
  // exclusive scan of the per-chunk survivor counts
  const uint32_t mine = (t < nchunks) ? sv.S[(size_t)t * kHistBins + b0] : 0u;
  const uint32_t upto = block_prefix_incl<1024>(mine, part);
  if (t < nchunks) sv.chunk_off[t] = upto - mine;
}

// ---------------------------------------------------------------------------
// k_pick_mask : first selection kernel after a fused pass that marked the keys
// reaching a guessed bound.  One block of 1024 threads (flat selections only).
// Optionally takes the leader first.  Adds up the per-chunk counts of marked
// elements; if the bound holds at least k and at most min(cap, k + n/8) keys, every
// marked element will become a list entry (chunk offsets are written, the state stays
// at level 0 with use_mask set); otherwise the state asks for the histogram of
// every key (need_full).
// ---------------------------------------------------------------------------
__global__ void __launch_bounds__(1024)
k_pick_mask(SelParams p, LeaderArgs la) {
  __shared__ uint32_t part[1024];
  __shared__ int lead_sh;
  const int t = threadIdx.x;
  if (t == 0) lead_sh = -1;
  if (la.partials != nullptr) {
    const int best = block_take_leader(la);
    if (t == 0) lead_sh = best;
  }
  __syncthreads();
  const SegView sv = seg_view(p, blockIdx.y, lead_sh);
  const uint32_t k = sv.d.k;
  const int nchunks = sv.d.geom.nchunks;
  const uint32_t gkey = sv.ctrl[1];
  const uint32_t mine = (t < nchunks) ? sv.mcount[t] : 0u;
  uint32_t total;
  const uint32_t upto = block_prefix_incl<1024>(mine, part, &total);
  // accepted if the bound holds at least k keys and not more than the list takes; a list far
  // longer than k (beyond k + n/8) is not worth fetching entry by entry either
  const uint64_t span = (uint64_t)(sv.d.e_hi - sv.d.e_lo);
  uint64_t limit = (uint64_t)k + (span >> 3);
  if (limit > sv.d.cap) limit = sv.d.cap;
  const bool ok = gkey != kNoGuess && total >= k && total <= limit;
  if (ok && t < nchunks) sv.chunk_off[t] = upto - mine;
  if (t == 0) {
    SelState st{};
    if (ok) {
      st.hi = kKeyMask;
      st.need = k;
      st.cand = total;
      st.compact_level = 1u;
      st.use_mask = 1u;
      st.list_lo = gkey;
      st.list_count = total;
    } else {
      st.need_full = 1u;
    }
    *sv.st = st;
  }
}

// ---------------------------------------------------------------------------
// k_compact1 : level-1 compaction of the leader's range, one block per chunk.
// Survivors (key >= st.lo, i.e. top digit >= b0) are written to the survivor
// list in ascending element order at chunk_off[c] + rank inside the chunk;
// candidates (top digit == b0) also feed the next-digit histogram hist1.
// If the list cannot hold n_gt + cand entries nothing is written and only the
// histogram is built.  block = WAVES waves; in a tile every lane owns 4 R
// consecutive elements (lane-contiguous loads run at the same bandwidth as
// row-coalesced ones here), so a survivor's rank is the lane's exclusive prefix
// plus its position among the lane's own survivors: five or six ballots per
// tile instead of one per element.
// ---------------------------------------------------------------------------
constexpr int kC1Waves = 4, kC1R = 4;  // (flat vectors on the histogram route take 8 waves)

template <int WAVES, int R>
__device__ __forceinline__ void compact1_body(const SelParams& p) {
  constexpr int T = 64 * WAVES;
  constexpr int E = 4 * R;             // consecutive elements one lane owns in a tile
  constexpr int WSPAN = 64 * E;        // consecutive elements one wave owns in a tile
  constexpr int TILE = WAVES * WSPAN;  // elements per block iteration
  static_assert(E <= 32, "one 32-bit mask per lane");
  __shared__ uint32_t lh[kHistBins];
  __shared__ uint32_t wtot[2][WAVES];

  int seg, c;
  block_chunk(p, seg, c);
  const SegView sv = seg_view(p, seg);
  if (c >= sv.d.geom.nchunks) return;
  const int tid = threadIdx.x;
  const int wave = tid >> 6;
  const uint32_t lane = lane_id();
  const int64_t n = p.n, e_lo = sv.d.e_lo, e_hi = sv.d.e_hi;
  const ChunkGeom geom = sv.d.geom;
  const uint32_t cap = sv.d.cap;
  uint2* __restrict__ list = sv.list;

  const SelState st = *sv.st;
  if (st.level != 1u || st.use_mask != 0u || *p.err) return;
  const bool write_out = st.compact_level == 1u;  // the level-1 survivors fit the list
  const bool zero_out = write_out && p.zero_vec != nullptr;
  const uint32_t klo = st.lo, khi = st.hi;
  const float* __restrict__ xp = sv.x;

  for (int b = tid; b < kHistBins; b += T) lh[b] = 0u;
  __syncthreads();

  const int64_t c_begin = geom.chunk0 + (int64_t)c * geom.chunk_elems;  // a multiple of kTile
  const int64_t c_end = c_begin + geom.chunk_elems;
  const int64_t cs = c_begin > e_lo ? c_begin : e_lo;  // elements of the range owned by this chunk
  const int64_t ce = c_end < e_hi ? c_end : e_hi;
  const int64_t n_vec = n & ~(int64_t)3;
  const int64_t lane_off = (int64_t)wave * WSPAN + (int64_t)lane * E;

  uint32_t run = write_out ? sv.chunk_off[c] : 0u;  // list position of the next survivor of this chunk
  int buf = 0;

  // raw bits of one tile; a tile that is wholly inside the array is read with R unconditional loads
  // (conditions around the loads make the compiler wait for each before issuing the next), in the
  // last tile groups are read element by element where needed, absent elements as 0
  auto load_tile = [&](int64_t tb, uint32_t (&out)[E]) {
    const int64_t j0 = tb + lane_off;
    if (tb + TILE <= n_vec) {
#pragma unroll
      for (int r = 0; r < R; ++r) {
        const uint4 v = *reinterpret_cast<const uint4*>(xp + j0 + 4 * r);
        out[4 * r + 0] = v.x;
        out[4 * r + 1] = v.y;
        out[4 * r + 2] = v.z;
        out[4 * r + 3] = v.w;
      }
    } else {
#pragma unroll
      for (int r = 0; r < R; ++r) {
        const int64_t j = j0 + 4 * r;
        uint4 v;
        if (j + 4 <= n_vec) {
          v = *reinterpret_cast<const uint4*>(xp + j);
        } else {
          v.x = (j + 0 < n) ? __float_as_uint(xp[j + 0]) : 0u;
          v.y = (j + 1 < n) ? __float_as_uint(xp[j + 1]) : 0u;
          v.z = (j + 2 < n) ? __float_as_uint(xp[j + 2]) : 0u;
          v.w = (j + 3 < n) ? __float_as_uint(xp[j + 3]) : 0u;
        }
        out[4 * r + 0] = v.x;
        out[4 * r + 1] = v.y;
        out[4 * r + 2] = v.z;
        out[4 * r + 3] = v.w;
      }
    }
  };

  // the next tile's loads are issued before this tile is worked on
  uint32_t raw[E], nxt[E];
  if (c_begin < ce) load_tile(c_begin, raw);
  for (int64_t tb = c_begin; tb < ce; tb += TILE) {
    const int64_t j0 = tb + lane_off;  // this lane's E consecutive elements start here
    const bool more = tb + TILE < ce;
    if (more) load_tile(tb + TILE, nxt);
    // every element of this tile belongs to the chunk and the range?
    const bool clean = (tb >= cs) && (tb + TILE <= ce);

    // survivors (key >= klo) among this lane's elements, one bit each
    uint32_t own = 0u;
#pragma unroll
    for (int e = 0; e < E; ++e) {
      bool ok = (raw[e] & kKeyMask) >= klo;
      if (!clean) ok = ok && (j0 + e >= cs) && (j0 + e < ce);
      own |= ok ? (1u << e) : 0u;
    }
    const uint32_t cnt = (uint32_t)__popc(own);
    // exclusive prefix of cnt over the lanes and the wave total, from the bit planes of cnt
    uint32_t before = 0u, wsum = 0u;
#pragma unroll
    for (int b = 0; (1 << b) <= E; ++b) {
      const uint64_t plane = __ballot((cnt >> b) & 1u);
      before += popc_lt(plane) << b;
      wsum += (uint32_t)__popcll(plane) << b;
    }

    uint32_t base = 0u;
    if (write_out) {
      if (lane == 0) wtot[buf][wave] = wsum;
      __syncthreads();
      base = run;
#pragma unroll
      for (int i = 0; i < WAVES; ++i) {
        const uint32_t wt = wtot[buf][i];
        if (i < wave) base += wt;
        run += wt;
      }
      buf ^= 1;
    }
    if (own != 0u) {  // few lanes get here
      uint32_t pos = base + before;
#pragma unroll
      for (int e = 0; e < E; ++e) {
        if ((own >> e) & 1u) {
          const uint32_t kk = raw[e] & kKeyMask;
          if (kk <= khi) atomicAdd(&lh[(kk >> 7) & 0xfffu], 1u);  // candidate: feeds the next digit
          // (index, raw bits): the sign travels with the survivor
          if (write_out && pos < cap) list[pos] = make_uint2((uint32_t)(j0 + e), raw[e]);
          ++pos;
        }
      }
      // Keys above the threshold digit are kept whatever the later digits say: if asked to, put
      // +0.0 there now, while the group is in registers (the list carries the values on).  Only
      // when the list is written here, because the deeper array passes would re-read the vector.
      if (zero_out) {
#pragma unroll
        for (int r = 0; r < R; ++r) {
          uint32_t z[4];
          uint32_t hit = 0u;
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const bool a = ((own >> (4 * r + e)) & 1u) && (raw[4 * r + e] & kKeyMask) > khi;
            z[e] = a ? 0u : raw[4 * r + e];
            hit |= a ? (1u << e) : 0u;
          }
          if (hit) {  // (rewriting the lane's whole 64 bytes instead was measured slower)
            const int64_t j = j0 + 4 * r;
            if (clean && j + 4 <= n_vec) {
              *reinterpret_cast<uint4*>(p.zero_vec + j) = make_uint4(z[0], z[1], z[2], z[3]);
            } else {  // at a chunk's edge a group may hold a neighbour's elements
#pragma unroll
              for (int e = 0; e < 4; ++e)
                if ((hit >> e) & 1u) p.zero_vec[j + e] = 0.0f;
            }
          }
        }
      }
    }
    if (more) {
#pragma unroll
      for (int e = 0; e < E; ++e) raw[e] = nxt[e];
    }
  }

  __syncthreads();
  for (int b = tid; b < kHistBins; b += T) {
    const uint32_t v = lh[b];
    if (v) atomicAdd(&sv.hist1[b], v);
  }
}

// ---------------------------------------------------------------------------
// compact_mask_body (first job of k_mask_or_hist) : writes the survivor list from the
// bit mask the fused pass left behind instead of re-reading the vector; one block of
// 1024 threads per chunk, runs only if the state says use_mask.  Every marked element (key >=
// list_lo) becomes a list entry, in ascending element order, starting at
// chunk_off[c]; only the marked elements' values are fetched.  The top digits
// of all entries are counted into the slot's partial whole-vector histograms
// (copy c mod kHistReps), from which k_pick0 then takes the threshold digit.
//   Per slab of 1024 mask rows (256 elements each), two steps.  First thread t
//   owns row t: a block scan of the rows' popcounts gives the row's list
//   offset, and the thread writes the indices of its marked elements into the
//   list entries.  Then the block walks the slab's entries with one entry per
//   thread, UB of them in flight, fetching the values to complete the entries.
// ---------------------------------------------------------------------------
template <int UB>
__device__ __forceinline__ void compact_mask_body(const SelParams& p) {
  constexpr int T = 1024, WAVES = 16;
  constexpr uint32_t STAGE = 4096;  // a slab with at most this many marks keeps their indices on chip
  __shared__ uint32_t wtot[WAVES];
  __shared__ uint32_t lh[kHistBins];
  __shared__ uint32_t sidx[STAGE];

  const SegView sv = seg_view(p, blockIdx.y);
  const int c = blockIdx.x;
  if (c >= sv.d.geom.nchunks) return;
  const SelState st = *sv.st;
  if (st.use_mask == 0u || sv.mask == nullptr || *p.err) return;
  const int tid = threadIdx.x;
  const int wave = tid >> 6;
  const uint32_t lane = lane_id();
  const int64_t n = p.n;
  const ChunkGeom geom = sv.d.geom;
  const uint32_t cap = sv.d.cap;
  const uint32_t list_lo = st.list_lo;
  const float* __restrict__ xp = sv.x;
  const uint64_t* __restrict__ mk = sv.mask;
  uint2* list = sv.list;

  for (int b = tid; b < kHistBins; b += T) lh[b] = 0u;
  __syncthreads();

  const int64_t c_begin = geom.chunk0 + (int64_t)c * geom.chunk_elems;  // a multiple of 256
  int64_t c_end = c_begin + geom.chunk_elems;
  if (c_end > n) c_end = n;
  const int64_t n_vec = n & ~(int64_t)3;                      // marked elements end here
  const int64_t v_end = c_end < n_vec ? c_end : n_vec;
  const int64_t row_lo = c_begin >> 8;
  const int64_t row_hi = (v_end + 255) >> 8;                  // exclusive

  uint32_t run = sv.chunk_off[c];  // list position of the next entry of this chunk
  // a row's four mask words; rows behind the chunk re-read its last row (unused), so that the
  // loads sit in no branch and the next slab's can be in flight while this slab is worked on
  auto load_row = [&](int64_t row, uint4& lo2, uint4& hi2) {
    const int64_t rr = row < row_hi ? row : row_hi - 1;
    lo2 = reinterpret_cast<const uint4*>(mk + mask_word(rr))[0];
    hi2 = reinterpret_cast<const uint4*>(mk + mask_word(rr))[1];
  };
  uint4 cur_lo = make_uint4(0u, 0u, 0u, 0u), cur_hi = cur_lo;
  if (row_lo < row_hi) load_row(row_lo + tid, cur_lo, cur_hi);
  for (int64_t slab = row_lo; slab < row_hi; slab += T) {
    const int64_t row = slab + tid;
    uint4 nxt_lo = cur_lo, nxt_hi = cur_hi;
    if (slab + T < row_hi) load_row(row + T, nxt_lo, nxt_hi);  // block-uniform condition
    uint64_t m[4] = {0ull, 0ull, 0ull, 0ull};
    if (row < row_hi) {
      m[0] = ((uint64_t)cur_lo.y << 32) | cur_lo.x;
      m[1] = ((uint64_t)cur_lo.w << 32) | cur_lo.z;
      m[2] = ((uint64_t)cur_hi.y << 32) | cur_hi.x;
      m[3] = ((uint64_t)cur_hi.w << 32) | cur_hi.z;
    }
    const uint32_t cnt = (uint32_t)(__popcll(m[0]) + __popcll(m[1]) + __popcll(m[2]) + __popcll(m[3]));
    // exclusive prefix of cnt (<= 256) over the lanes and the wave total, from the bit planes of cnt
    uint32_t before = 0u, wsum = 0u;
#pragma unroll
    for (int b = 0; b <= 8; ++b) {
      const uint64_t plane = __ballot((cnt >> b) & 1u);
      before += popc_lt(plane) << b;
      wsum += (uint32_t)__popcll(plane) << b;
    }
    if (lane == 0) wtot[wave] = wsum;
    __syncthreads();
    uint32_t pos = run + before, total = 0u;
#pragma unroll
    for (int i = 0; i < WAVES; ++i) {
      const uint32_t wt = wtot[i];
      if (i < wave) pos += wt;
      total += wt;
    }
    // the row's marked elements in ascending order: by group, then by position in the group;
    // their indices go to the on-chip stage if the slab's marks fit there, else into the list
    const bool staged = total <= STAGE;  // the same in every thread
    uint64_t any = m[0] | m[1] | m[2] | m[3];
    while (any) {
      const int g = __builtin_ctzll(any);
      const uint64_t bit = 1ull << g;
      any &= ~bit;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        if (m[e] & bit) {
          const uint32_t j = (uint32_t)(row * 256 + 4 * g + e);
          if (staged)
            sidx[pos - run] = j;
          else if (pos < cap)
            list[pos].x = j;
          ++pos;
        }
      }
    }
    __threadfence_block();  // the indices are written before any thread of the block reads them
    __syncthreads();
    for (uint32_t e0 = (uint32_t)tid; e0 < total; e0 += T * UB) {
      uint32_t j[UB], raw[UB];
      bool ok[UB];
#pragma unroll
      for (int u = 0; u < UB; ++u) {
        const uint32_t e = e0 + (uint32_t)u * T;
        ok[u] = e < total && run + e < cap;
        j[u] = !ok[u] ? 0u : staged ? sidx[e] : list[run + e].x;
      }
#pragma unroll
      for (int u = 0; u < UB; ++u) raw[u] = __float_as_uint(xp[j[u]]);
#pragma unroll
      for (int u = 0; u < UB; ++u) {
        if (ok[u]) {
          if (staged)
            list[run + e0 + (uint32_t)u * T] = make_uint2(j[u], raw[u]);  // the whole entry at once
          else
            list[run + e0 + (uint32_t)u * T].y = raw[u];
          atomicAdd(&lh[(raw[u] & kKeyMask) >> 19], 1u);
        }
      }
    }
    run += total;
    cur_lo = nxt_lo;  // (only here: the copy waits for the loads)
    cur_hi = nxt_hi;
  }
  // the elements behind the last whole group of four are not in the mask
  if (c_end == n && n_vec < n && tid == 0) {
    for (int64_t j = n_vec; j < n; ++j) {
      const uint32_t raw = __float_as_uint(xp[j]);
      const uint32_t kk = raw & kKeyMask;
      if (kk >= list_lo) {
        atomicAdd(&lh[kk >> 19], 1u);
        if (run < cap) list[run] = make_uint2((uint32_t)j, raw);
        ++run;
      }
    }
  }

  __syncthreads();
  uint32_t* __restrict__ htop = sv.htop + (size_t)(c % sv.htop_reps) * kHistBins;
  for (int b = tid; b < kHistBins; b += T) {
    const uint32_t v = lh[b];
    if (v) atomicAdd(&htop[b], v);
  }
}

// ---------------------------------------------------------------------------
// compact_tiles_body : the survivor list from what the fused pass staged per tile
// (k_pass_mark with STAGE): one block of 1024 threads per chunk copies the tiles'
// pieces, in tile order, to the list from chunk_off[c] on and counts the entries'
// top digits, as compact_mask_body does.  The chunk is walked in slabs of eight
// tiles; a slab with a tile that staged nothing (kTileOverflow: more marks than a
// piece holds) is built from the mask instead: one thread per mask row writes the
// row's marked indices, then the block fetches the values entry by entry.
// ---------------------------------------------------------------------------
__device__ __forceinline__ void compact_tiles_body(const SelParams& p) {
  constexpr int T = 1024, WAVES = 16, SLAB = 8;  // tiles per slab (1024 mask rows)
  __shared__ uint32_t wtot[WAVES];
  __shared__ uint32_t lh[kHistBins];
  __shared__ uint32_t tc[SLAB];

  const SegView sv = seg_view(p, blockIdx.y);
  const int c = blockIdx.x;
  if (c >= sv.d.geom.nchunks) return;
  const SelState st = *sv.st;
  if (st.use_mask == 0u || sv.mask == nullptr || *p.err) return;
  const int tid = threadIdx.x;
  const int wave = tid >> 6;
  const uint32_t lane = lane_id();
  const int64_t n = p.n;
  const ChunkGeom geom = sv.d.geom;
  const uint32_t cap = sv.d.cap;
  const uint32_t list_lo = st.list_lo;
  const float* __restrict__ xp = sv.x;
  const uint64_t* __restrict__ mk = sv.mask;
  uint2* list = sv.list;

  for (int b = tid; b < kHistBins; b += T) lh[b] = 0u;

  const int64_t c_begin = geom.chunk0 + (int64_t)c * geom.chunk_elems;  // a whole number of tiles
  int64_t c_end = c_begin + geom.chunk_elems;
  if (c_end > n) c_end = n;
  const int64_t n_vec = n & ~(int64_t)3;                      // marked elements end here
  const int64_t v_end = c_end < n_vec ? c_end : n_vec;
  const int64_t tile_lo = c_begin / kPassTile;
  const int64_t tile_hi = (v_end + kPassTile - 1) / kPassTile;  // exclusive
  const int64_t row_end = (v_end + 255) >> 8;                   // exclusive

  uint32_t run = sv.chunk_off[c];  // list position of the next entry of this chunk
  for (int64_t t0 = tile_lo; t0 < tile_hi; t0 += SLAB) {
    const int ntl = (int)(tile_hi - t0 < SLAB ? tile_hi - t0 : SLAB);
    __syncthreads();  // tc, wtot and the histogram's clearing
    if (tid < SLAB) tc[tid] = tid < ntl ? sv.tcnt[t0 + tid] : 0u;
    __syncthreads();
    uint32_t pre[SLAB + 1];
    bool staged = true;
    pre[0] = 0u;
#pragma unroll
    for (int i = 0; i < SLAB; ++i) {
      const uint32_t v = tc[i];
      staged = staged && v != kTileOverflow;
      pre[i + 1] = pre[i] + (v != kTileOverflow ? v : 0u);
    }
    if (staged) {  // the same in every thread
      const uint32_t total = pre[SLAB];
      for (uint32_t f0 = (uint32_t)tid; f0 < total; f0 += 4 * T) {  // four entries in flight per thread
        uint2 ent[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          const uint32_t f = f0 + (uint32_t)u * T < total ? f0 + (uint32_t)u * T : total - 1u;
          int i = 0;
#pragma unroll
          for (int q = 1; q < SLAB; ++q) i += f >= pre[q] ? 1 : 0;  // the tile this entry belongs to
          ent[u] = sv.tbuf[(size_t)(t0 + i) * (size_t)sv.tcap + (f - pre[i])];
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          const uint32_t f = f0 + (uint32_t)u * T;
          if (f < total) {
            if (run + f < cap) list[run + f] = ent[u];
            atomicAdd(&lh[(ent[u].y & kKeyMask) >> 19], 1u);
          }
        }
      }
      run += total;
      continue;
    }
    // from the mask: thread t owns row 128 t0 + t
    const int64_t row = t0 * (kPassTile / 256) + tid;
    uint64_t m[4] = {0ull, 0ull, 0ull, 0ull};
    if (row < row_end) {
      const uint4 lo2 = reinterpret_cast<const uint4*>(mk + mask_word(row))[0];
      const uint4 hi2 = reinterpret_cast<const uint4*>(mk + mask_word(row))[1];
      m[0] = ((uint64_t)lo2.y << 32) | lo2.x;
      m[1] = ((uint64_t)lo2.w << 32) | lo2.z;
      m[2] = ((uint64_t)hi2.y << 32) | hi2.x;
      m[3] = ((uint64_t)hi2.w << 32) | hi2.z;
    }
    const uint32_t cnt = (uint32_t)(__popcll(m[0]) + __popcll(m[1]) + __popcll(m[2]) + __popcll(m[3]));
    uint32_t before = 0u, wsum = 0u;
#pragma unroll
    for (int b = 0; b <= 8; ++b) {
      const uint64_t plane = __ballot((cnt >> b) & 1u);
      before += popc_lt(plane) << b;
      wsum += (uint32_t)__popcll(plane) << b;
    }
    if (lane == 0) wtot[wave] = wsum;
    __syncthreads();
    uint32_t pos = run + before, total = 0u;
#pragma unroll
    for (int i = 0; i < WAVES; ++i) {
      const uint32_t wt = wtot[i];
      if (i < wave) pos += wt;
      total += wt;
    }
    uint64_t any = m[0] | m[1] | m[2] | m[3];
    while (any) {
      const int g = __builtin_ctzll(any);
      const uint64_t bit = 1ull << g;
      any &= ~bit;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        if (m[e] & bit) {
          if (pos < cap) list[pos].x = (uint32_t)(row * 256 + 4 * g + e);
          ++pos;
        }
      }
    }
    __threadfence_block();  // the indices are written before any thread of the block reads them
    __syncthreads();
    for (uint32_t e0 = (uint32_t)tid; e0 < total; e0 += T) {
      if (run + e0 < cap) {
        const uint32_t raw = __float_as_uint(xp[list[run + e0].x]);
        list[run + e0].y = raw;
        atomicAdd(&lh[(raw & kKeyMask) >> 19], 1u);
      }
    }
    run += total;
  }
  // the elements behind the last whole group of four are not in the mask
  if (c_end == n && n_vec < n && tid == 0) {
    for (int64_t j = n_vec; j < n; ++j) {
      const uint32_t raw = __float_as_uint(xp[j]);
      const uint32_t kk = raw & kKeyMask;
      if (kk >= list_lo) {
        atomicAdd(&lh[kk >> 19], 1u);
        if (run < cap) list[run] = make_uint2((uint32_t)j, raw);
        ++run;
      }
    }
  }

  __syncthreads();
  uint32_t* __restrict__ htop = sv.htop + (size_t)(c % sv.htop_reps) * kHistBins;
  for (int b = tid; b < kHistBins; b += T) {
    const uint32_t v = lh[b];
    if (v) atomicAdd(&htop[b], v);
  }
}

// k_mask_or_hist : the kernel behind k_pick_mask.  Per segment it does whichever of the two
// jobs the state asks for: the list from the mask (use_mask), or, after a guess that did not
// hold, the per-chunk histograms of every key (need_full; p_full are the parameters of that
// route: own top-digit histogram, only_if_need_full set).  Both are one 1024-thread block per
// chunk, so they share a launch.
template <int UB>
__global__ void __launch_bounds__(1024)
k_mask_or_hist(SelParams p, SelParams p_full) {
  const SelState* st = seg_view(p, blockIdx.y).st;
  if (st->use_mask != 0u) {
    if (p.tiles.buf != nullptr)
      compact_tiles_body(p);
    else
      compact_mask_body<UB>(p);
  } else if (st->need_full != 0u) {
    hist0_body<1024>(p_full);
  }
}

// ---------------------------------------------------------------------------
// Decoupled look-back over tiles.  Each tile publishes a 64-bit word
//   [63:62] status (0 none, 1 tile aggregate, 2 inclusive prefix)
//   [61:31] count A (keys above the range)      [30:0] count B (keys inside)
// Counts never exceed 2^31-1 in total, so packed words add field-wise.
// Called by the 64 lanes of one wave; returns the exclusive prefix of `tile`.
// The wait on a predecessor is bounded; expiry sets *err and returns what was
// gathered so far (every wave still leaves the kernel).
// ---------------------------------------------------------------------------
constexpr uint64_t kFlagAgg = 1ull << 62;
constexpr uint64_t kFlagIncl = 2ull << 62;
constexpr uint64_t kFlagValMask = (1ull << 62) - 1ull;
constexpr int kSpinLimit = 1 << 20;

__device__ __forceinline__ uint64_t flag_load(const uint64_t* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void flag_store(uint64_t* p, uint64_t v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

__device__ uint64_t lookback_exclusive(uint64_t* __restrict__ flags, int flag_stride, int64_t tile,
                                       uint64_t agg, uint32_t* __restrict__ err) {
  const uint32_t lane = lane_id();
  if (tile == 0) {
    if (lane == 0) flag_store(&flags[0], kFlagIncl | agg);
    return 0ull;
  }
  if (lane == 0) flag_store(&flags[tile * flag_stride], kFlagAgg | agg);
  uint64_t excl = 0ull;     // wave-uniform running total
  int64_t base = tile - 1;  // lane L inspects tile base - L
  while (true) {
    const int64_t my = base - (int64_t)lane;
    uint64_t word = kFlagIncl;  // tiles before the first act as an inclusive prefix of zero
    if (my >= 0) {
      int spins = 0;
      word = flag_load(&flags[my * flag_stride]);
      while ((word >> 62) == 0ull) {
        if (++spins > kSpinLimit) {
          atomicOr(err, kErrWait);
          word = kFlagIncl;
          break;
        }
        __builtin_amdgcn_s_sleep(2);
        word = flag_load(&flags[my * flag_stride]);
      }
    }
    const uint64_t incl_mask = __ballot((word >> 62) == 2ull);
    uint64_t contrib = word & kFlagValMask;
    if (incl_mask != 0ull) {
      const int first = __ffsll((long long)incl_mask) - 1;  // nearest tile holding an inclusive prefix
      if ((int)lane > first) contrib = 0ull;
      excl += wave_allsum_u64(contrib);
      break;
    }
    excl += wave_allsum_u64(contrib);
    base -= 64;
  }
  if (lane == 0) flag_store(&flags[tile * flag_stride], kFlagIncl | ((excl + agg) & kFlagValMask));
  return excl;
}

// ---------------------------------------------------------------------------
// k_compact : ordered compaction with two classes.
//   class A: key > st.hi           class B: st.lo <= key <= st.hi
//   An element is kept if it is in A, or in B with fewer than `quota` B
//   elements before it; its output position is
//        (#A before it) + min(#B before it, quota)
//   which is ascending in element order.  quota = infinity below level 3.
//
//   SRC_ARRAY (LIST = false): elements are x[e_lo .. e_hi) of the selected
//     vector, kept entries go to the survivor list as (index, bits).  Level 2
//     runs when the level-1 survivors did not fit the list, level 3 when the
//     level-2 ones did not either; a pass writes the list only if it fits
//     (otherwise it only feeds the next digit histogram).
//   SRC_LIST (LIST = true): elements are the survivor list, kept entries'
//     indices go to idx_out[0 .. k) and, if vals_row is given, their values
//     (the list carries the raw float bits) to vals_row[0 .. k).  Requires
//     level 3.
//
//   block = 512 threads = 8 waves; a tile is 8 waves x 8 rows x 64 lanes x 4
//   consecutive elements, each wave owning a contiguous 2048-element piece.
// ---------------------------------------------------------------------------
constexpr int kCompactThreads = 512;
constexpr int kCompactRows = 8;
constexpr int kCompactTile = kCompactThreads * 4 * kCompactRows;  // 16384 elements
constexpr int kWaveSpan = 64 * 4 * kCompactRows;                  // 2048 elements

// The pass itself; st is the state derived for it (in shared memory, the same in every thread).
// DIRECT (array source, level 3): the kept entries go straight to idx_out / vals_row (and are put
// to +0.0 in zero_vec) instead of into the list, so no pass over the list has to follow.
template <bool LIST, bool DIRECT>
__device__ __forceinline__ void compact_body(const SelParams& p, const SegView& sv, const SelState& st, int level,
                                             int launch_id, uint32_t zero_below) {
  static_assert(!(LIST && DIRECT), "DIRECT is a form of the array pass");
  __shared__ uint32_t lh[(!LIST && !DIRECT) ? kHistBins : 4];
  __shared__ uint64_t wave_tot[8];
  __shared__ uint64_t tile_excl;
  __shared__ int64_t tile_sh;

  int64_t n = p.n, e_lo = sv.d.e_lo, e_hi = sv.d.e_hi;
  const uint32_t cap = sv.d.cap;
  uint32_t* __restrict__ hist_next = sv.hist2;
  uint64_t* __restrict__ flags = sv.flags + launch_id;
  constexpr int flag_stride = kNumLookback;
  uint32_t* __restrict__ tile_counter = sv.counters + launch_id;
  uint2* __restrict__ list = sv.list;
  int32_t* __restrict__ idx_out = sv.idx_out;
  float* __restrict__ vals_row = sv.vals_row;
  const uint32_t k_out = sv.d.k;
  uint32_t* __restrict__ err = p.err;

  const int tid = threadIdx.x;
  const int wave = tid >> 6;
  const uint32_t lane = lane_id();

  // With zeroing on the way: the level-1 pass zeroed the keys above its range if it wrote the
  // list (zero_below = the top of that range); the pass that writes idx_out zeroes the kept rest,
  // or all of them otherwise (zero_below = every key).
  float* __restrict__ zero_vec = (LIST || DIRECT) ? p.zero_vec : nullptr;
  bool write_out;
  bool do_hist;
  uint32_t quota;
  int64_t first_tile, ntiles;
  if (!LIST) {
    // level 2 runs whenever level 1 did not fit; level 3 only if level 2 did not fit either
    if (level == 3 && st.compact_level != 3u) return;
    quota = (level == 3) ? st.need : kQuotaInf;
    write_out = st.compact_level == (uint32_t)level;
    do_hist = level < 3 && !DIRECT;
    first_tile = e_lo / kCompactTile;
    ntiles = (e_hi + kCompactTile - 1) / kCompactTile - first_tile;
  } else {
    if (st.level != 3u) {
      if (tid == 0 && blockIdx.x == 0) atomicOr(err, kErrSequence);
      return;
    }
    quota = st.need;
    write_out = true;
    do_hist = false;
    e_lo = 0;
    e_hi = (int64_t)st.list_count;
    n = (int64_t)cap;  // list arrays are allocated with cap rounded up to a whole tile
    first_tile = 0;
    ntiles = (e_hi + kCompactTile - 1) / kCompactTile;
  }
  const uint32_t klo = st.lo, khi = st.hi;
  const int dshift = digit_shift(level < 3 ? level : 2);
  const uint32_t dmask = digit_mask(level < 3 ? level : 2);

  const float* __restrict__ xp = LIST ? nullptr : sv.x;

  if (do_hist) {
    for (int b = tid; b < kHistBins; b += kCompactThreads) lh[b] = 0u;
  }
  __syncthreads();

  while (true) {
    if (tid == 0) tile_sh = (int64_t)atomicAdd(tile_counter, 1u);
    __syncthreads();
    const int64_t trel = tile_sh;
    if (trel >= ntiles) break;
    const int64_t tbase = (first_tile + trel) * kCompactTile + (int64_t)wave * kWaveSpan;

    // ---- load keys (and list payloads) --------------------------------
    uint32_t key[kCompactRows][4];
    int32_t pay[LIST ? kCompactRows : 1][4];
    uint32_t valid = 0u;  // bit (r*4+e)
    const bool full = (tbase >= e_lo) && (tbase + kWaveSpan <= e_hi) && (tbase + kWaveSpan <= (n & ~(int64_t)3));
    if (full) {
#pragma unroll
      for (int r = 0; r < kCompactRows; ++r) {
        const int64_t j = tbase + (int64_t)r * 256 + (int64_t)lane * 4;
        uint4 v;
        if (!LIST) {
          v = *reinterpret_cast<const uint4*>(xp + j);
        } else {
          const uint4 e01 = reinterpret_cast<const uint4*>(list + j)[0];  // (idx, bits) x 2
          const uint4 e23 = reinterpret_cast<const uint4*>(list + j)[1];
          v = make_uint4(e01.y, e01.w, e23.y, e23.w);
          pay[LIST ? r : 0][0] = (int32_t)e01.x;
          pay[LIST ? r : 0][1] = (int32_t)e01.z;
          pay[LIST ? r : 0][2] = (int32_t)e23.x;
          pay[LIST ? r : 0][3] = (int32_t)e23.z;
        }
        key[r][0] = v.x;  // raw bits; comparisons mask the sign off
        key[r][1] = v.y;
        key[r][2] = v.z;
        key[r][3] = v.w;
      }
      valid = 0xffffffffu;
    } else {
#pragma unroll
      for (int r = 0; r < kCompactRows; ++r) {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const int64_t j = tbase + (int64_t)r * 256 + (int64_t)lane * 4 + e;
          key[r][e] = 0u;
          if (LIST) pay[LIST ? r : 0][e] = 0;
          if (j >= e_lo && j < e_hi) {
            valid |= 1u << (r * 4 + e);
            if (!LIST) {
              key[r][e] = __float_as_uint(xp[j]);
            } else {
              const uint2 ent = list[j];
              key[r][e] = ent.y;
              pay[LIST ? r : 0][e] = (int32_t)ent.x;
            }
          }
        }
      }
    }

    // ---- classify, count, feed the next-digit histogram ----------------
    uint32_t isA = 0u, isB = 0u;
    uint32_t cntA = 0u, cntB = 0u;  // wave totals (uniform)
#pragma unroll
    for (int r = 0; r < kCompactRows; ++r) {
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const bool ok = (valid >> (r * 4 + e)) & 1u;
        const uint32_t mk = key[r][e] & kKeyMask;
        const bool a = ok && mk > khi;
        const bool b = ok && mk >= klo && mk <= khi;
        if (a) isA |= 1u << (r * 4 + e);
        if (b) isB |= 1u << (r * 4 + e);
        cntA += (uint32_t)__popcll(__ballot(a));
        cntB += (uint32_t)__popcll(__ballot(b));
        if (do_hist && b) atomicAdd(&lh[(mk >> dshift) & dmask], 1u);
      }
    }

    if (write_out) {
      if (lane == 0) wave_tot[wave] = ((uint64_t)cntA << 31) | (uint64_t)cntB;
      __syncthreads();
      if (wave == 0) {
        uint64_t agg = 0ull;
#pragma unroll
        for (int i = 0; i < 8; ++i) agg += wave_tot[i];
        const uint64_t ex = lookback_exclusive(flags, flag_stride, trel, agg, err);
        if (lane == 0) tile_excl = ex;
      }
      __syncthreads();
      uint64_t mine = tile_excl;
      for (int i = 0; i < wave; ++i) mine += wave_tot[i];
      uint32_t runA = (uint32_t)(mine >> 31);
      uint32_t runB = (uint32_t)(mine & 0x7fffffffu);

      if ((cntA | cntB) != 0u) {
#pragma unroll
        for (int r = 0; r < kCompactRows; ++r) {
          uint64_t bA[4], bB[4];
          uint32_t rowA = 0u, rowB = 0u, ltA = 0u, ltB = 0u;
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            bA[e] = __ballot((isA >> (r * 4 + e)) & 1u);
            bB[e] = __ballot((isB >> (r * 4 + e)) & 1u);
            rowA += (uint32_t)__popcll(bA[e]);
            rowB += (uint32_t)__popcll(bB[e]);
          }
          if ((rowA | rowB) != 0u) {
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              ltA += popc_lt(bA[e]);
              ltB += popc_lt(bB[e]);
            }
            uint32_t befA = runA + ltA, befB = runB + ltB;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              const bool a = (isA >> (r * 4 + e)) & 1u;
              const bool b = (isB >> (r * 4 + e)) & 1u;
              if (a || (b && befB < quota)) {
                const uint32_t pos = befA + (befB < quota ? befB : quota);
                const int64_t j = tbase + (int64_t)r * 256 + (int64_t)lane * 4 + e;
                if (!LIST && DIRECT) {
                  if (pos < k_out) {
                    idx_out[pos] = (int32_t)j;
                    if (vals_row) vals_row[pos] = __uint_as_float(key[r][e]);
                    if (zero_vec && ((key[r][e] & kKeyMask) <= zero_below) && j < p.n) zero_vec[j] = 0.0f;
                  }
                } else if (!LIST) {
                  if (pos < cap) list[pos] = make_uint2((uint32_t)j, key[r][e]);
                } else {
                  if (pos < k_out) {
                    idx_out[pos] = pay[LIST ? r : 0][e];
                    if (vals_row) vals_row[pos] = __uint_as_float(key[r][e]);
                    // kept entries that nothing has put to +0.0 yet
                    if (zero_vec && ((key[r][e] & kKeyMask) <= zero_below)) {
                      const int32_t zi = pay[LIST ? r : 0][e];
                      if (zi >= 0 && (int64_t)zi < p.n) zero_vec[zi] = 0.0f;
                    }
                  }
                }
              }
              befA += a ? 1u : 0u;
              befB += b ? 1u : 0u;
            }
          }
          runA += rowA;
          runB += rowB;
        }
      }
    }
    __syncthreads();  // tile_sh / wave_tot / tile_excl reused by the next tile
  }

  if (do_hist) {
    __syncthreads();
    for (int b = tid; b < kHistBins; b += kCompactThreads) {
      const uint32_t v = lh[b];
      if (v) atomicAdd(&hist_next[b], v);
    }
  }
}

// The survivor list was copied from pieces staged by a fused pass that stored +0.0 in place of
// every element it handed on (k_pass_mark with STAGE).  The pass that counts the last digit over the
// list (list_hist_body, digit 2) knows the threshold key up to its last seven bits, [lo, hi]: it gives
// the handed-on elements with key <= hi their values back and puts +0.0 over the keys > hi that no
// piece handed on (a tile whose marks stayed in the mask, the n mod 4 last elements).  The final pass
// over the list then has the kept entries with key <= hi left to zero.
__device__ __forceinline__ bool from_pieces(const SelParams& p, const SegView& sv) {
  return p.zero_vec != nullptr && sv.tbuf != nullptr && sv.st->use_mask != 0u;
}

// Keys the level-1 pass has already put to +0.0 in zero_vec lie above this one (every key if it
// has not zeroed any).
__device__ __forceinline__ uint32_t zeroed_above(const SelState* stp) {
  return (stp->compact_level == 1u && stp->use_mask == 0u) ? stp->hi : kKeyMask;
}

template <bool LIST>
__global__ void __launch_bounds__(kCompactThreads)
k_compact(SelParams p, int level, int launch_id) {
  __shared__ SelState st;
  __shared__ uint32_t pick_part[kCompactThreads];
  const SegView sv = seg_view(p, blockIdx.y);
  const SelState* __restrict__ stp = sv.st;
  const uint32_t zero_below = zeroed_above(stp);
  // the level-1 survivors fitted the list: the deeper array passes have nothing to do
  if (!LIST && (stp->compact_level == 1u || *p.err)) return;
  if (LIST && *p.err) return;
  // tiles are handed out by a counter, so blocks beyond the number of list tiles are not needed
  if (LIST && stp->compact_level == 1u && (uint64_t)blockIdx.x * kCompactTile >= (uint64_t)stp->list_count) return;
  derive_state<kCompactThreads>(sv, st, LIST ? 3 : level, pick_part, p.err);
  compact_body<LIST, false>(p, sv, st, level, launch_id, (LIST && from_pieces(p, sv)) ? (st.hi | 0x7fu) : zero_below);
}

// ---------------------------------------------------------------------------
// k_final : the last selection kernel where the deeper array passes exist.  If a list
// was written (at level 1, from the mask, or by the level-2 pass) it is the final
// pass over the list; if not even the level-2 survivors fitted one (e.g. an all-equal
// vector) it is the level-3 pass over the array, which then writes the outputs itself.
// ---------------------------------------------------------------------------
__global__ void __launch_bounds__(kCompactThreads)
k_final(SelParams p) {
  __shared__ SelState st;
  __shared__ uint32_t pick_part[kCompactThreads];
  const SegView sv = seg_view(p, blockIdx.y);
  const SelState* __restrict__ stp = sv.st;
  const uint32_t zero_below = zeroed_above(stp);
  if (*p.err) return;
  if (stp->compact_level == 1u && (uint64_t)blockIdx.x * kCompactTile >= (uint64_t)stp->list_count) return;
  derive_state<kCompactThreads>(sv, st, 3, pick_part, p.err);
  if (st.compact_level == 3u)
    compact_body<false, true>(p, sv, st, 3, 1, zero_below);
  else
    compact_body<true, false>(p, sv, st, 3, 2, from_pieces(p, sv) ? (st.hi | 0x7fu) : zero_below);
}

// ---------------------------------------------------------------------------
// k_list_hist : histogram of digit `digit` (1 or 2) over the candidates in the
// survivor list; runs only when the list was written at level 1 or from the
// mask.  Digit 1 is needed only for a list written from the mask (k_compact1
// counts it on the way); for digit 2 the digit-1 pick is replayed from hist1 in
// the prologue.
// ---------------------------------------------------------------------------
template <int T>
__device__ __forceinline__ void list_hist_body(const SelParams& p, int digit) {
  constexpr int PER = 8192 / T;  // entries per thread and round
  __shared__ uint32_t lh[kHistBins];
  __shared__ SelState st;
  __shared__ uint32_t pick_part[T];
  const SegView sv = seg_view(p, blockIdx.y);
  if (sv.st->compact_level != 1u || *p.err) return;
  if (digit == 1 && sv.st->use_mask == 0u) return;
  const int tid = threadIdx.x;
  const uint32_t cnt = sv.st->list_count;
  // 8192 entries per block and round; no more blocks than that needs
  uint32_t nb = (cnt + 8191u) / 8192u;
  if (nb > gridDim.x) nb = gridDim.x;
  if (blockIdx.x >= nb) return;
  if (digit == 2) {
    derive_state<T>(sv, st, 2, pick_part, p.err);
  } else {
    if (tid == 0) st = *sv.st;
    __syncthreads();
  }
  const int nbins = (int)digit_mask(digit) + 1;
  for (int b = tid; b < nbins; b += T) lh[b] = 0u;
  __syncthreads();
  const uint32_t klo = st.lo, khi = st.hi;
  const int sh = digit_shift(digit);
  const uint32_t dm = digit_mask(digit);
  if (digit == 2 && from_pieces(p, sv)) {
    // the same count, and on the way the residual is put right around the threshold (see from_pieces)
    const bool all_pieces = sv.ctrl != nullptr && sv.ctrl[2] == 0u;  // no tile kept its marks to the mask
    const int64_t n_vec = p.n & ~(int64_t)3;
    for (uint64_t base = (uint64_t)blockIdx.x * 8192u; base < cnt; base += (uint64_t)nb * 8192u) {
      uint2 ent[PER];
#pragma unroll
      for (int i = 0; i < PER; ++i) {  // (no branch around the loads: behind the list they re-read its last entry)
        const uint64_t q = base + (uint64_t)i * T + tid;
        ent[i] = sv.list[q < cnt ? q : cnt - 1u];
      }
#pragma unroll
      for (int i = 0; i < PER; ++i) {
        const int64_t j = (int64_t)ent[i].x;
        if (base + (uint64_t)i * T + tid >= cnt || j >= p.n) continue;
        const uint32_t kk = ent[i].y & kKeyMask;
        if (kk >= klo && kk <= khi) atomicAdd(&lh[(kk >> sh) & dm], 1u);
        const bool handed_on = j < n_vec && (all_pieces || sv.tcnt[j / kPassTile] != kTileOverflow);
        if (handed_on) {
          if (kk <= khi) p.zero_vec[j] = __uint_as_float(ent[i].y);
        } else if (kk > khi) {
          p.zero_vec[j] = 0.0f;
        }
      }
    }
  } else {
    for (uint64_t base = (uint64_t)blockIdx.x * 8192u; base < cnt; base += (uint64_t)nb * 8192u) {
      uint32_t key[PER];
#pragma unroll
      for (int i = 0; i < PER; ++i) {  // (no branch around the loads: behind the list they re-read its last entry)
        const uint64_t q = base + (uint64_t)i * T + tid;
        key[i] = sv.list[q < cnt ? q : cnt - 1u].y & kKeyMask;
      }
#pragma unroll
      for (int i = 0; i < PER; ++i)
        if (base + (uint64_t)i * T + tid < cnt && key[i] >= klo && key[i] <= khi)
          atomicAdd(&lh[(key[i] >> sh) & dm], 1u);
    }
  }
  __syncthreads();
  uint32_t* __restrict__ dst = digit == 1 ? sv.hist1 : sv.hist2;
  for (int b = tid; b < nbins; b += T) {
    const uint32_t v = lh[b];
    if (v) atomicAdd(&dst[b], v);
  }
}

__global__ void __launch_bounds__(256)
k_list_hist(SelParams p, int digit) {
  list_hist_body<256>(p, digit);
}

template <int WAVES, int R>
__global__ void __launch_bounds__(64 * WAVES)
k_compact1(SelParams p) {
  compact1_body<WAVES, R>(p);
}

// ---------------------------------------------------------------------------
// k_level1 : the kernel behind the first pick on the guess route.  If the list was
// written from the mask it counts the second digit over the list's candidates; if the
// guess did not hold it is the level-1 compaction of the histogram route.
// ---------------------------------------------------------------------------
__global__ void __launch_bounds__(64 * kC1Waves)
k_level1(SelParams p) {
  if (seg_view(p, blockIdx.y).st->use_mask != 0u)
    list_hist_body<64 * kC1Waves>(p, 1);
  else
    compact1_body<kC1Waves, kC1R>(p);
}

// ---------------------------------------------------------------------------
// k_level2 : the kernel between the level-1 pass and k_final where the deeper array
// passes exist.  If a list was written at level 1 (or from the mask) it counts the
// last digit over the list's candidates; if the level-1 survivors did not fit one it
// is the level-2 pass over the array (which writes the list if its survivors fit, and
// counts the last digit on the way).
// ---------------------------------------------------------------------------
__global__ void __launch_bounds__(kCompactThreads)
k_level2(SelParams p) {
  const SegView sv = seg_view(p, blockIdx.y);
  if (*p.err) return;
  if (sv.st->compact_level == 1u) {
    list_hist_body<kCompactThreads>(p, 2);
  } else {
    __shared__ SelState st;
    __shared__ uint32_t pick_part[kCompactThreads];
    derive_state<kCompactThreads>(sv, st, 2, pick_part, p.err);
    compact_body<false, false>(p, sv, st, 2, 0, kKeyMask);
  }
}


// ---------------------------------------------------------------------------
// k_tile_starts : tile_start[t] = number of kept indices below t * kPassTile, for
// t = 0 .. ntiles (so tile_start[ntiles] = k), from the ascending index list.
// One thread per index: idx[p] owns the entries of the tiles that begin between
// idx[p-1] and idx[p], the last index also the rest; the 64 lanes of a wave fill
// each owner's entries together, so a long run of empty tiles costs its length / 64.
// ---------------------------------------------------------------------------
__global__ void __launch_bounds__(256)
k_tile_starts(const int32_t* __restrict__ idx, int64_t k, int32_t ntiles, int32_t* __restrict__ tile_start) {
  const int64_t p = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int lane = threadIdx.x & 63;
  int32_t t0 = 1, t1 = 0, t_last = -1;  // [t0, t1] = entries this index owns (empty by default)
  if (p < k) {
    const int64_t i = (int64_t)idx[p];
    const int64_t prev = p > 0 ? (int64_t)idx[p - 1] : -1;
    if (i >= 0 && i >= prev) {  // otherwise not an ascending index list: k_pass_rest reports what is left unset
      const int64_t t = i / kPassTile;
      t1 = (int32_t)(t < ntiles ? t : ntiles);
      t0 = prev < 0 ? 0 : (int32_t)(prev / kPassTile) + 1;
      if (p == k - 1) t_last = t1;
    }
  }
  uint64_t todo = __ballot(t0 <= t1);
  while (todo != 0ull) {
    const int src = __ffsll((unsigned long long)todo) - 1;
    todo &= todo - 1;
    const int32_t a = __shfl(t0, src, 64), b = __shfl(t1, src, 64);
    const int32_t v = (int32_t)(p - lane + src);
    for (int32_t t = a + lane; t <= b; t += 64) tile_start[t] = v;
  }
  const uint64_t fin = __ballot(t_last >= 0);
  if (fin != 0ull) {
    const int src = __ffsll((unsigned long long)fin) - 1;
    const int32_t a = __shfl(t_last, src, 64) + 1;
    for (int32_t t = a + lane; t <= ntiles; t += 64) tile_start[t] = (int32_t)k;
  }
}

// ---------------------------------------------------------------------------
// k_tile_starts_search : the same table when there are many more kept indices than
// tiles: one thread per entry t looks up the first position whose index is not
// below t * kPassTile (binary search in the ascending list; the upper levels of the
// search are shared by all threads and stay in the cache).  A list that does not
// ascend gives bounds that k_pass_rest / k_update_tiles reject or clip.
// ---------------------------------------------------------------------------
__global__ void __launch_bounds__(256)
k_tile_starts_search(const int32_t* __restrict__ idx, int64_t k, int32_t ntiles, int32_t* __restrict__ tile_start) {
  const int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (t > ntiles) return;
  const int64_t target = t * kPassTile;
  int64_t lo = 0, hi = k;  // the answer lies in [lo, hi]
  while (lo < hi) {
    const int64_t mid = (lo + hi) >> 1;
    if ((int64_t)idx[mid] < target) lo = mid + 1; else hi = mid;
  }
  tile_start[t] = (int32_t)lo;
}

// ---------------------------------------------------------------------------
// k_pass_rest : for every worker except the leader, in one streaming pass:
//   acc = g + residual; at the kept indices vals[w][m] = acc and the residual
//   becomes +0.0, elsewhere the residual becomes acc.
// Used when the leader is known before the step starts (its own pass and the
// selection have already run, so idx is final and k_tile_starts has run).
// grid = (gx, W-1), block = T; block (b, y) works on worker (leader + 1 + y) mod W
// and takes the tiles b, b + gx, ... of T U float4 groups (see k_pass_mark).  Per
// tile it marks the kept positions, idx[tile_start[t] .. tile_start[t+1]), in an
// LDS slot table while the tile's loads are in flight.
// ---------------------------------------------------------------------------
template <bool NT, int GT, int T, int U>
__global__ void __launch_bounds__(T)
k_pass_rest(PtrTable g, PtrTable res, int w_count, int leader, int64_t n, const int32_t* __restrict__ idx, int64_t k,
            float* __restrict__ vals, const int32_t* __restrict__ tile_start, uint32_t* __restrict__ err) {
  constexpr int TILE = T * 4 * U;  // elements per tile: T threads x U float4
  static_assert(TILE == kPassTile, "tile_start is laid out for this tile");
  static_assert(TILE <= 32768, "slot entries are 16-bit offsets from the tile's first index");
  __shared__ __attribute__((aligned(16))) int16_t slot[TILE];
  const int tid = threadIdx.x;
  const int w = (int)(((unsigned)leader + 1u + blockIdx.y) % (unsigned)w_count);
  const float* __restrict__ gp = g.p[w];
  float* __restrict__ rp = res.p[w];
  float* __restrict__ vrow = vals + (size_t)w * (size_t)k;
  uint2* s2 = reinterpret_cast<uint2*>(slot);  // four 16-bit slots: one float4 group

  const int64_t q_end = n >> 2;  // whole float4 groups end here
  const int64_t ntiles = q_end > 0 ? (n + TILE - 1) / TILE : 0;  // fewer than four elements: only the scalar tail
  // The counter that loads are waited on counts them in issue order, so whatever is needed early
  // is issued early: the bounds of the NEXT tile's indices one tile ahead, this tile's indices
  // before its big loads; the slot table is then filled while those are in flight.
  int64_t ti = blockIdx.x;
  int32_t m0 = 0, m1 = 0;
  if (ti < ntiles) {
    m0 = tile_start[ti];
    m1 = tile_start[ti + 1];
  }
  for (; ti < ntiles; ti += gridDim.x) {
    const int64_t ti_next = ti + gridDim.x;
    int32_t n0 = 0, n1 = 0;
    if (ti_next < ntiles) {
      n0 = tile_start[ti_next];
      n1 = tile_start[ti_next + 1];
    }
    int64_t m_base = (int64_t)m0, m_end = (int64_t)m1;
    if (m_base < 0 || m_end > k || m_end < m_base || m_end - m_base > TILE) {  // idx was not ascending
      if (tid == 0) atomicOr(err, kErrIndex);
      m_end = m_base = 0;
    }
    const int64_t lo = ti * TILE;
    // (no branch around the load: beyond the tile's indices it re-reads the last index, unused)
    const int64_t p0 = m_base + tid;
    const int32_t i0 = idx[p0 < m_end ? p0 : k - 1];
    const int64_t q0 = (lo >> 2) + tid;
    const bool full = lo + TILE <= 4 * q_end;
    v4f a[U], b[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      // groups behind the vector re-read its last group (unused): no branch between or around the
      // loads, or the compiler would wait for all of them before the first use of an index
      const int64_t q = q0 + u * T;
      const int64_t ql = (full || q < q_end) ? q : q_end - 1;
      a[u] = load4g<NT, GT>(gp, 4 * ql);
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {  // (one array after the other: see k_pass_mark)
      const int64_t q = q0 + u * T;
      const int64_t ql = (full || q < q_end) ? q : q_end - 1;
      b[u] = load4<NT>(rp + 4 * ql);
    }
    // slot[j] = (position in idx) - m_base for a kept element j of this tile, else -1
#pragma unroll
    for (int u = 0; u < U; ++u) s2[tid + u * T] = make_uint2(0xffffffffu, 0xffffffffu);
    __syncthreads();
    {
      const int64_t i = (int64_t)i0 - lo;
      if (p0 < m_end && i >= 0 && i < TILE) slot[i] = (int16_t)tid;
    }
    for (int64_t p = p0 + T; p < m_end; p += T) {  // dense tiles only (more than T kept of 32 T elements)
      const int64_t i = (int64_t)idx[p] - lo;
      if (i >= 0 && i < TILE) slot[i] = (int16_t)(p - m_base);
    }
    __syncthreads();
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int64_t q = q0 + u * T;
      if (full || q < q_end) {
        const uint2 sl = s2[tid + u * T];
        v4f v;
        v.x = a[u].x + b[u].x;
        v.y = a[u].y + b[u].y;
        v.z = a[u].z + b[u].z;
        v.w = a[u].w + b[u].w;
        if ((sl.x & sl.y) != 0xffffffffu) {  // some element of this group is kept
          const int s0 = (int16_t)(sl.x & 0xffffu), s1 = (int16_t)(sl.x >> 16);
          const int s2v = (int16_t)(sl.y & 0xffffu), s3 = (int16_t)(sl.y >> 16);
          if (s0 >= 0) { vrow[m_base + s0] = v.x; v.x = 0.0f; }
          if (s1 >= 0) { vrow[m_base + s1] = v.y; v.y = 0.0f; }
          if (s2v >= 0) { vrow[m_base + s2v] = v.z; v.z = 0.0f; }
          if (s3 >= 0) { vrow[m_base + s3] = v.w; v.w = 0.0f; }
        }
        store4<NT>(rp + 4 * q, v);
      }
    }
    __syncthreads();  // the slot table is rebuilt for the next tile
    m0 = n0;
    m1 = n1;
  }
  // scalar tail of the vector (n not a multiple of 4): the first block
  if (blockIdx.x == 0) {
    const int64_t j = (n >> 2) * 4 + tid;
    if (j < n) {
      float v = load1g<GT>(gp, j) + rp[j];
      int64_t lo = 0, hi = k;  // binary search for j among the indices
      while (lo < hi) {
        const int64_t mid = (lo + hi) >> 1;
        if ((int64_t)idx[mid] < j) lo = mid + 1; else hi = mid;
      }
      if (lo < k && (int64_t)idx[lo] == j) {
        vrow[lo] = v;
        v = 0.0f;
      }
      rp[j] = v;
    }
  }
}

// ---------------------------------------------------------------------------
// k_sum_rows : sum[m] = ((vals[0][m] + vals[1][m]) + ...) + vals[W-1][m], float32,
// in that order.
// ---------------------------------------------------------------------------
__global__ void __launch_bounds__(256)
k_sum_rows(const float* __restrict__ vals, int w_count, int64_t k, float* __restrict__ sum) {
  const int64_t m0 = (int64_t)blockIdx.x * 1024 + threadIdx.x;  // this thread: m0, m0+256, m0+512, m0+768
  float s[4] = {0.0f, 0.0f, 0.0f, 0.0f};
  for (int w0 = 0; w0 < w_count; w0 += 4) {  // sixteen independent loads in flight, then the ordered adds
    float v[4][4];
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int e = 0; e < 4; ++e)
        if (w0 + j < w_count && m0 + e * 256 < k) v[j][e] = vals[(size_t)(w0 + j) * (size_t)k + (size_t)(m0 + e * 256)];
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int e = 0; e < 4; ++e)
        if (w0 + j < w_count && m0 + e * 256 < k) s[e] = (w0 + j == 0) ? v[j][e] : (s[e] + v[j][e]);
  }
#pragma unroll
  for (int e = 0; e < 4; ++e)
    if (m0 + e * 256 < k) sum[m0 + e * 256] = s[e];
}

// ---------------------------------------------------------------------------
// k_gather : one thread per kept index m.  vals[w][m] = x_w[idx[m]], sum[m] is
// the float32 sum over w = 0, 1, ..., W-1 in that order; with ZERO the
// position is then overwritten by +0.0 in every worker.
// ---------------------------------------------------------------------------
template <bool ZERO>
__global__ void __launch_bounds__(256)
k_gather(PtrTable tab, int w_count, int64_t n, const int32_t* __restrict__ idx, int64_t k,
         float* __restrict__ vals, float* __restrict__ sum, uint32_t* __restrict__ err) {
  const int64_t m = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (m >= k) return;
  const int64_t i = (int64_t)idx[m];
  if (i < 0 || i >= n) {  // never touch memory through an index outside the vector
    atomicOr(err, kErrIndex);
    return;
  }
  float s = 0.0f;
  for (int w0 = 0; w0 < w_count; w0 += 8) {  // eight independent loads in flight, then the ordered adds
    float v[8];
#pragma unroll
    for (int j = 0; j < 8; ++j)
      if (w0 + j < w_count) v[j] = tab.p[w0 + j][i];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      if (w0 + j < w_count) {
        if (vals) vals[(size_t)(w0 + j) * (size_t)k + (size_t)m] = v[j];
        s = (w0 + j == 0) ? v[j] : (s + v[j]);
        if (ZERO) tab.p[w0 + j][i] = 0.0f;
      }
    }
  }
  if (sum) sum[m] = s;
}

__global__ void __launch_bounds__(256)
k_zero_at(PtrTable tab, int w_count, int64_t n, const int32_t* __restrict__ idx, int64_t k,
          uint32_t* __restrict__ err) {
  const int64_t m = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (m >= k) return;
  const int64_t i = (int64_t)idx[m];
  if (i < 0 || i >= n) {
    atomicOr(err, kErrIndex);
    return;
  }
  for (int w = 0; w < w_count; ++w) tab.p[w][i] = 0.0f;
}

// ---------------------------------------------------------------------------
// k_update_fill : update = zeros(N) with update[idx[m]] = sum[m], every output
// element written exactly once.  Block b owns a contiguous run of 8192-element
// chunks; it locates its first index with a 256-way search, then per chunk
// builds the chunk in LDS (BATCH x 256 index/sum pairs per round, fetched ahead
// of the buffer clear) and streams it out.
// ---------------------------------------------------------------------------
constexpr int kFillChunk = 8192;

// What a thread holds of the (index, sum) pairs ahead of the chunk being built.
template <int BATCH>
struct FillAhead {
  int64_t ib[BATCH];
  float sb[BATCH];
};

constexpr int64_t kFillNone = INT64_MAX;  // no index: beyond every chunk

template <int BATCH>
__device__ __forceinline__ void fill_fetch(FillAhead<BATCH>& a, const int32_t* __restrict__ idx,
                                           const float* __restrict__ sum, int64_t k, int64_t from) {
  const int tid = threadIdx.x;
#pragma unroll
  for (int j = 0; j < BATCH; ++j) {
    // (no branch around the loads: behind the list they re-read its last entry, unused)
    const int64_t p = from + tid + j * 256;
    const int64_t pc = p < k ? p : k - 1;
    const int32_t iv = idx[pc];
    const float sv = sum[pc];
    a.ib[j] = p < k ? (int64_t)iv : kFillNone;
    a.sb[j] = sv;
  }
}

// Builds and streams out the chunks [c_begin, c_end) of the update; m = number of indices below
// the first of them, whose first pairs `a` already holds.  The pairs a chunk starts with are
// fetched one chunk ahead, before the previous chunk is streamed out, so that their latency is
// not part of the chunk's own chain; behind the last chunk the fetch goes to m_after (the start
// of the block's next run) if that is not negative.  All 256 threads call it.
template <int BATCH>
__device__ __forceinline__ void fill_run(FillAhead<BATCH>& a, float* __restrict__ buf, float* __restrict__ update,
                                         int64_t n, const int32_t* __restrict__ idx, const float* __restrict__ sum,
                                         int64_t k, int64_t c_begin, int64_t c_end, int64_t m, int64_t m_after) {
  constexpr int kGroups = kFillChunk / 4 / 256;  // float4 groups per thread and chunk
  const int tid = threadIdx.x;
  for (int64_t c = c_begin; c < c_end; ++c) {
    const int64_t lo = c * kFillChunk;
    const int64_t hi = (lo + kFillChunk < n) ? lo + kFillChunk : n;
    const int64_t len = hi - lo;
    const int64_t len4 = len >> 2;
    float4* b4 = reinterpret_cast<float4*>(buf);
    for (int i = tid; i < kFillChunk / 4; i += 256) b4[i] = make_float4(0.f, 0.f, 0.f, 0.f);
    __syncthreads();
    while (true) {
      int cnt = 0;
#pragma unroll
      for (int j = 0; j < BATCH; ++j) {
        const bool in = a.ib[j] < hi;
        if (in && a.ib[j] >= lo) {  // ib >= lo always holds for ascending idx
          const int64_t off = a.ib[j] - lo;
          buf[off] = a.sb[j];
        }
        cnt += __syncthreads_count(in);
      }
      m += cnt;
      const bool chunk_done = cnt < BATCH * 256;
      // the next chunk's first pairs, or the rest of this chunk's
      fill_fetch<BATCH>(a, idx, sum, k, (chunk_done && c == c_end - 1 && m_after >= 0) ? m_after : m);
      if (chunk_done) break;
    }
    // (the count barrier above also orders the LDS writes before the reads)
    float* __restrict__ up = update + lo;
#pragma unroll
    for (int j = 0; j < kGroups; ++j) {
      const int64_t i = tid + j * 256;
      if (i < len4) {
        // (non-temporal: with ordinary stores the time of this fill depended on what earlier
        // kernels had left in the caches, 115 to 150 us on 138 M elements; so it is 115 throughout)
        const float4 t4 = b4[i];
        const v4f tv = {t4.x, t4.y, t4.z, t4.w};
        store4<true>(up + 4 * i, tv);
      }
    }
    for (int64_t i = len4 * 4 + tid; i < len; i += 256) up[i] = buf[i];  // ragged end of the vector
    __syncthreads();
  }
}

template <int BATCH>
__global__ void __launch_bounds__(256)
k_update_fill(float* __restrict__ update, int64_t n, const int32_t* __restrict__ idx,
              const float* __restrict__ sum, int64_t k) {
  __shared__ __attribute__((aligned(16))) float buf[kFillChunk];
  __shared__ int64_t s_lo, s_hi;
  const int tid = threadIdx.x;
  const int64_t nchunk = (n + kFillChunk - 1) / kFillChunk;
  const int64_t c_begin = nchunk * (int64_t)blockIdx.x / (int64_t)gridDim.x;
  const int64_t c_end = nchunk * ((int64_t)blockIdx.x + 1) / (int64_t)gridDim.x;
  if (c_begin >= c_end) return;

  // m = number of indices below the first element of this block's run
  const int64_t target = c_begin * kFillChunk;
  if (tid == 0) {
    s_lo = 0;
    s_hi = k;
  }
  __syncthreads();
  while (true) {
    const int64_t lo = s_lo, hi = s_hi;  // answer lies in [lo, hi]
    const int64_t span = hi - lo;
    if (span <= 0) break;
    const int64_t stepw = (span + 255) / 256;
    const int64_t p = lo + (int64_t)tid * stepw;  // probe positions lo, lo+stepw, ...
    const bool below = (p < hi) && ((int64_t)idx[p] < target);
    const int cnt = __syncthreads_count(below);
    // probes 0..cnt-1 are below the target: the answer is in (lo+(cnt-1)*stepw, lo+cnt*stepw]
    if (tid == 0) {
      if (cnt == 0) {
        s_hi = lo;
      } else {
        const int64_t nlo = lo + (int64_t)(cnt - 1) * stepw + 1;
        int64_t nhi = lo + (int64_t)cnt * stepw;
        if (nhi > hi) nhi = hi;
        s_lo = nlo;
        s_hi = nhi;
      }
    }
    __syncthreads();
  }
  const int64_t m = s_lo;
  FillAhead<BATCH> a;
  fill_fetch<BATCH>(a, idx, sum, k, m);
  fill_run<BATCH>(a, buf, update, n, idx, sum, k, c_begin, c_end, m, -1);
}

// The same with the blocks striding over the tiles of the streaming passes (kPassTile elements, four
// chunks), whose first indices k_tile_starts has left in tile_start: no search, and at any time the
// blocks in flight write one contiguous window of the update.
template <int BATCH>
__global__ void __launch_bounds__(256)
k_update_fill_tiled(float* __restrict__ update, int64_t n, const int32_t* __restrict__ idx,
                    const float* __restrict__ sum, int64_t k, const int32_t* __restrict__ tile_start) {
  __shared__ __attribute__((aligned(16))) float buf[kFillChunk];
  constexpr int64_t kPer = kPassTile / kFillChunk;  // chunks per tile
  const int64_t nchunk = (n + kFillChunk - 1) / kFillChunk;
  const int64_t ntiles = (n + kPassTile - 1) / kPassTile;
  // (a start outside [0, k] can only come from an index list that was not ascending)
  auto start_of = [&](int64_t t) {
    const int64_t v = (int64_t)tile_start[t];
    return v < 0 ? (int64_t)0 : (v > k ? k : v);
  };
  int64_t ti = blockIdx.x;
  if (ti >= ntiles) return;
  int64_t m = start_of(ti);
  FillAhead<BATCH> a;
  fill_fetch<BATCH>(a, idx, sum, k, m);
  for (; ti < ntiles; ti += gridDim.x) {
    const int64_t tn = ti + gridDim.x;
    const int64_t m_next = tn < ntiles ? start_of(tn) : k;
    const int64_t c_begin = ti * kPer;
    const int64_t c_end = c_begin + kPer < nchunk ? c_begin + kPer : nchunk;
    fill_run<BATCH>(a, buf, update, n, idx, sum, k, c_begin, c_end, m, m_next);
    m = m_next;
  }
}

// ---------------------------------------------------------------------------
// k_update_tiles : the same dense update for long vectors: zeros streamed out tile
// by tile (kPassTile elements, blocks striding over the tiles as in k_pass_mark), and
// behind a tile's zeros the same block stores sum[m] at the tile's kept indices,
// idx[tile_start[t] .. tile_start[t+1]) (k_tile_starts has run).  The barrier between
// the two orders them for the block's stores to one address; the lines are still in
// the cache when the second store arrives, so memory sees each line once.
// NTZ: the zeros go out as non-temporal stores (measured per step: better on 138 M
// elements, 1.335 against 1.354 ms, because the kernels that follow find less of this
// vector in the caches; worse on 1e9, 654 against 626 us for the kernel itself).
// ---------------------------------------------------------------------------
template <int T, int U, bool NTZ>
__global__ void __launch_bounds__(T)
k_update_tiles(float* __restrict__ update, int64_t n, const int32_t* __restrict__ idx, const float* __restrict__ sum,
               int64_t k, const int32_t* __restrict__ tile_start, uint32_t* __restrict__ err) {
  constexpr int TILE = T * 4 * U;
  static_assert(TILE == kPassTile, "tile_start is laid out for this tile");
  const int tid = threadIdx.x;
  const int64_t q_end = n >> 2;  // whole float4 groups
  const int64_t ntiles = (n + TILE - 1) / TILE;
  const v4f zero = {0.f, 0.f, 0.f, 0.f};
  int64_t ti = blockIdx.x;
  int32_t m0 = 0, m1 = 0;
  if (ti < ntiles) {
    m0 = tile_start[ti];
    m1 = tile_start[ti + 1];
  }
  for (; ti < ntiles; ti += gridDim.x) {
    const int64_t ti_next = ti + gridDim.x;
    int32_t n0 = 0, n1 = 0;
    if (ti_next < ntiles) {  // the next tile's bounds, one tile ahead
      n0 = tile_start[ti_next];
      n1 = tile_start[ti_next + 1];
    }
    int64_t m_base = (int64_t)m0, m_end = (int64_t)m1;
    if (m_base < 0 || m_end > k || m_end < m_base || m_end - m_base > TILE) {  // idx was not ascending
      if (tid == 0) atomicOr(err, kErrIndex);
      m_end = m_base = 0;
    }
    const int64_t lo = ti * TILE;
    // this tile's first T (index, sum) pairs, fetched while the zeros go out
    // (no branch around the loads: behind the tile's pairs they re-read the last pair, unused)
    const int64_t p0 = m_base + tid;
    const int64_t pc = p0 < m_end ? p0 : k - 1;
    const int32_t i0 = idx[pc];
    const float s0 = sum[pc];
    const int64_t q0 = (lo >> 2) + tid;
    if (lo + TILE <= 4 * q_end) {
#pragma unroll
      for (int u = 0; u < U; ++u) store4<NTZ>(update + 4 * (q0 + u * T), zero);
    } else {  // the last tile: whole groups, then the ragged end
#pragma unroll
      for (int u = 0; u < U; ++u)
        if (q0 + u * T < q_end) store4<NTZ>(update + 4 * (q0 + u * T), zero);
      const int64_t j = 4 * q_end + tid;
      if (j < n) update[j] = 0.0f;
    }
    __syncthreads();  // the block's zeros are ordered before its values
    if (p0 < m_end) {
      const int64_t i = (int64_t)i0 - lo;
      if (i >= 0 && i < TILE && lo + i < n) update[lo + i] = s0;
    }
    for (int64_t p = p0 + T; p < m_end; p += T) {  // dense tiles only
      const int64_t i = (int64_t)idx[p] - lo;
      if (i >= 0 && i < TILE && lo + i < n) update[lo + i] = sum[p];
    }
    m0 = n0;
    m1 = n1;
  }
}

// ---------------------------------------------------------------------------
// k_sum_update : the end of a step whose leader was known up front, behind the
// other workers' pass: sum[m] = ((vals[0][m] + vals[1][m]) + ...) + vals[W-1][m] in
// float32, in that order, and the dense update, zeros with sum[m] at idx[m], every
// element written once.  Blocks stride over the tiles as in k_pass_rest and mark a
// tile's kept positions, idx[tile_start[t] .. tile_start[t+1]), in the same 16-bit
// slot table; the thread that owns a kept position adds up the rows' entries and
// stores the sum on its way through the tile's float4 groups.
// ---------------------------------------------------------------------------
template <int T, int U>
__global__ void __launch_bounds__(T)
k_sum_update(const float* __restrict__ vals, int w_count, int64_t n, const int32_t* __restrict__ idx, int64_t k,
             const int32_t* __restrict__ tile_start, float* __restrict__ sum_out, float* __restrict__ update,
             uint32_t* __restrict__ err) {
  constexpr int TILE = T * 4 * U;
  static_assert(TILE == kPassTile, "tile_start is laid out for this tile");
  static_assert(TILE <= 32768, "slot entries are 16-bit offsets from the tile's first index");
  __shared__ __attribute__((aligned(16))) int16_t slot[TILE];
  const int tid = threadIdx.x;
  uint2* s2 = reinterpret_cast<uint2*>(slot);  // four 16-bit slots: one float4 group
  const int64_t q_end = n >> 2;  // whole float4 groups end here
  const int64_t ntiles = q_end > 0 ? (n + TILE - 1) / TILE : 0;

  // sum of the rows' entries at position m, in worker order
  auto ordered_sum = [&](int64_t m) {
    float sacc = vals[m];
    for (int w = 1; w < w_count; ++w) sacc = sacc + vals[(size_t)w * (size_t)k + (size_t)m];
    return sacc;
  };

  int64_t ti = blockIdx.x;
  int32_t m0 = 0, m1 = 0;
  if (ti < ntiles) {
    m0 = tile_start[ti];
    m1 = tile_start[ti + 1];
  }
  for (; ti < ntiles; ti += gridDim.x) {
    const int64_t ti_next = ti + gridDim.x;
    int32_t n0 = 0, n1 = 0;
    if (ti_next < ntiles) {  // the next tile's bounds, one tile ahead
      n0 = tile_start[ti_next];
      n1 = tile_start[ti_next + 1];
    }
    int64_t m_base = (int64_t)m0, m_end = (int64_t)m1;
    if (m_base < 0 || m_end > k || m_end < m_base || m_end - m_base > TILE) {  // idx was not ascending
      if (tid == 0) atomicOr(err, kErrIndex);
      m_end = m_base = 0;
    }
    const int64_t lo = ti * TILE;
    const int64_t p0 = m_base + tid;
    const int32_t i0 = idx[p0 < m_end ? p0 : k - 1];
    const int64_t q0 = (lo >> 2) + tid;
    const bool full = lo + TILE <= 4 * q_end;
#pragma unroll
    for (int u = 0; u < U; ++u) s2[tid + u * T] = make_uint2(0xffffffffu, 0xffffffffu);
    __syncthreads();
    {
      const int64_t i = (int64_t)i0 - lo;
      if (p0 < m_end && i >= 0 && i < TILE) slot[i] = (int16_t)tid;
    }
    for (int64_t p = p0 + T; p < m_end; p += T) {  // dense tiles only (more than T kept of 32 T elements)
      const int64_t i = (int64_t)idx[p] - lo;
      if (i >= 0 && i < TILE) slot[i] = (int16_t)(p - m_base);
    }
    __syncthreads();
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int64_t q = q0 + u * T;
      if (full || q < q_end) {
        const uint2 sl = s2[tid + u * T];
        v4f z = {0.f, 0.f, 0.f, 0.f};
        if ((sl.x & sl.y) != 0xffffffffu) {  // some element of this group is kept
          const int s0 = (int16_t)(sl.x & 0xffffu), s1 = (int16_t)(sl.x >> 16);
          const int s2v = (int16_t)(sl.y & 0xffffu), s3 = (int16_t)(sl.y >> 16);
          if (s0 >= 0) { z.x = ordered_sum(m_base + s0); sum_out[m_base + s0] = z.x; }
          if (s1 >= 0) { z.y = ordered_sum(m_base + s1); sum_out[m_base + s1] = z.y; }
          if (s2v >= 0) { z.z = ordered_sum(m_base + s2v); sum_out[m_base + s2v] = z.z; }
          if (s3 >= 0) { z.w = ordered_sum(m_base + s3); sum_out[m_base + s3] = z.w; }
        }
        store4<true>(update + 4 * q, z);
      }
    }
    __syncthreads();  // the slot table is rebuilt for the next tile
    m0 = n0;
    m1 = n1;
  }
  // the n mod 4 last elements: the first block
  if (blockIdx.x == 0) {
    const int64_t j = (n >> 2) * 4 + tid;
    if (j < n) {
      int64_t lo = 0, hi = k;  // binary search for j among the indices
      while (lo < hi) {
        const int64_t mid = (lo + hi) >> 1;
        if ((int64_t)idx[mid] < j) lo = mid + 1; else hi = mid;
      }
      float upd = 0.0f;
      if (lo < k && (int64_t)idx[lo] == j) {
        upd = ordered_sum(lo);
        sum_out[lo] = upd;
      }
      update[j] = upd;
    }
  }
}

}  // namespace artopk
