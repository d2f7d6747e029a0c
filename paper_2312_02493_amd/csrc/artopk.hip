// Host side of the AR-Topk compressor library: argument checks, scratch
// management and kernel sequencing behind the C ABI declared in artopk.h.
// No call synchronises the stream except artopk_status / artopk_get_profile /
// artopk_destroy; all decisions that depend on the data (leader, thresholds,
// tie quotas, list sizes) stay in device memory.

#include "artopk.h"

#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <new>
#include <vector>

#include "artopk_kernels.h"

using namespace artopk;

// Fixed scratch of artopk_variance_static (the entry point that allocates nothing): the per-block
// moments of up to kMaxW workers x kMaxChunks blocks, then kMaxW variances, then the argmax word.
// Every GPU the library runs on holds its own copy until the process ends.  In host code this name
// is only a handle for hipGetSymbolAddress; the kernels get the address that call returns.
constexpr size_t kStaticPartials = (size_t)kMaxW * kMaxChunks * 3;
constexpr size_t kStaticDoubles = kStaticPartials + kMaxW + 1;
static __device__ __align__(256) double scratch[kStaticDoubles];

namespace {

constexpr int kPassAThreads = 1024, kPassAU = 8;        // 128 KiB of each array per block iteration
constexpr int kPassRestThreads = 1024, kPassRestU = 8;

struct Scratch {
  // zeroed before every select: one kSegWords block per segment, then the look-back flags
  uint32_t* h_all = nullptr;      // [max_w][kSlotWords] whole-vector histograms of the fused pass, guess sample
  uint64_t* mask = nullptr;       // [max_w][mask_stride] survivor bit masks of the fused pass
  int64_t mask_stride = 0;        // 64-bit words per worker
  uint32_t* zero_base = nullptr;  // [max_seg][kSegWords]
  uint64_t* flags = nullptr;      // [max_tiles][kNumLookback], directly behind the blocks
  int64_t max_tiles = 0;
  // not zeroed
  uint32_t* S = nullptr;          // [max_w * kMaxChunks + max_seg][4096] per-chunk suffix histograms
  uint32_t* chunk_off = nullptr;  // [kMaxChunks + max_seg]
  double* partials = nullptr;     // [max_w][kMaxPassBlocks][3] per-block moments (or [2] sums)
  double* var_scratch = nullptr;  // [max_w]
  int32_t* leader_dev = nullptr;
  uint64_t* counter_dev = nullptr;  // iteration counter of ARTOPK_STAR_COUNTER steps
  uint32_t* err_dev = nullptr;
  uint2* list = nullptr;          // survivor lists: (index, raw float bits)
  int64_t list_entries = 0;       // allocated entries
  float* vals = nullptr;          // [max_w][max_k] gathered rows when the caller passes no vals_out
  int32_t* idx_rows = nullptr;    // [max_w][max_k] every worker's own Top-k (literal Alg. 1 leader rule)
  int32_t* tile_start = nullptr;  // [max_n / kPassTile + 2] kept indices below every tile of the streaming pass
  uint2* tilebuf = nullptr;       // list entries the fused pass stages per tile (guess route, one marking worker)
  int64_t tilebuf_entries = 0;
  uint32_t* tile_cnt = nullptr;   // [max_n / kPassTile + 1] entries staged per tile
  uint32_t* sample_keys = nullptr;  // [16384 kGuessRun] keys of one vector's guess sample
  SegDesc* table_dev = nullptr;   // [max_seg] segment descriptors
  uint32_t* chunk_map = nullptr;  // [kMaxChunks + max_seg] (segment << 16) | chunk, one entry per chunk of the layout
  uint32_t cap = 0;               // list capacity of a flat (one-segment) select
};

// A selection problem laid out for the kernels: one descriptor per segment and
// the launch bounds derived from them.
struct Plan {
  int32_t nseg = 1;
  std::vector<SegDesc> desc;
  bool use_table = false;   // descriptors live in the device table (nseg > 1)
  int32_t max_chunks = 1;   // largest chunk count of a segment
  int64_t max_tiles = 1;    // largest look-back tile count of a segment
  int64_t total_tiles = 1;
  int64_t max_cap = 1;      // largest list capacity of a segment
  int32_t total_chunks = 0; // chunks of all segments together (entries of the device chunk map), 0: no map
};

}  // namespace

struct artopk_ctx {
  int device = 0;
  int num_cu = 256;
  hipStream_t stream = nullptr;
  int32_t max_w = 0;
  int64_t max_n = 0, max_k = 0;
  int32_t max_seg = 0;
  bool pass_a_nt = true;   // non-temporal g loads / acc stores in pass A
  bool leader_first = true;  // STAR / FIXED: leader pass + select first, then one fused pass over the rest
  // vectors of at least this many elements get a sampled threshold guess before the fused pass, which
  // then counts and marks only the keys that reach it (the selection no longer re-reads the vector)
  int64_t guess_min_n = (int64_t)1 << 25;
  // vectors of at least this many elements get their dense update from k_update_tiles
  int64_t update_tiles_min_n = (int64_t)1 << 22;
  int stage_tiles = 1;  // guess route, one marking worker: the fused pass hands the marked elements on per tile
                        // (0 never, 1 for selections of one element in 256 or denser, 2 whenever a piece can hold a tile's share)
  void* slab = nullptr;
  Scratch s;
  // how the last step ran (artopk_select_info)
  int32_t last_guessed = 0, last_dom_workers = 0;
  int g_type = ARTOPK_G_F32;  // element type of the gradients of the step being enqueued
  // descriptors of the last segmented layout uploaded to table_dev
  std::vector<int64_t> cached_off, cached_k;
  int64_t cached_n = -1;
  Plan cached_plan;
  // stage events: a ring of the most recent calls, 5 marks per call
  // (0 start, 1 after pass A, 2 after select, 3 after gather, 4 after update)
  bool profile = false;
  int profile_level = 0;
  int lvl1_a = 0, lvl1_b = 1;  // the two marks level 1 records (they bracket the dominant kernel)
  static constexpr int kRing = 64;
  static constexpr int kMarks = 5;
  hipEvent_t ev[kRing][kMarks] = {};
  bool ev_valid[kRing][kMarks] = {};
  bool ev_created = false;
  long prof_calls = 0;  // calls recorded since profiling was switched on
  int cur = 0;          // ring slot of the call being recorded
  char err[512] = {0};
};
static_assert(sizeof(artopk_ctx::err) == 512, "fail() writes up to 512 bytes");

namespace {

// error text of calls that have no context (artopk_last_error(NULL) returns it)
thread_local char g_noctx_err[512] = {0};

int fail(artopk_ctx* c, int code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(c ? c->err : g_noctx_err, sizeof(g_noctx_err), fmt, ap);
  va_end(ap);
  return code;
}

#define HIP_TRY(ctx, expr)                                                                   \
  do {                                                                                       \
    hipError_t e_ = (expr);                                                                  \
    if (e_ != hipSuccess)                                                                    \
      return fail((ctx), ARTOPK_EHIP, "%s failed: %s (%s:%d)", #expr, hipGetErrorString(e_), \
                  __FILE__, __LINE__);                                                       \
  } while (0)

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

int check_ptr_table(artopk_ctx* c, const float* const* tab, int32_t w, const char* name, int align = 16) {
  if (!tab) return fail(c, ARTOPK_EINVAL, "%s is NULL", name);
  for (int i = 0; i < w; ++i) {
    if (!tab[i]) return fail(c, ARTOPK_EINVAL, "%s[%d] is NULL", name, i);
    if (reinterpret_cast<uintptr_t>(tab[i]) % (uintptr_t)align)
      return fail(c, ARTOPK_EINVAL, "%s[%d] is not %d-byte aligned", name, i, align);
  }
  return ARTOPK_OK;
}

int check_common(artopk_ctx* c, int32_t w, int64_t n, int64_t k) {
  if (!c) return ARTOPK_EINVAL;
  if (w < 1 || w > c->max_w) return fail(c, ARTOPK_EINVAL, "W=%d outside [1, %d]", w, c->max_w);
  if (n < 1 || n > c->max_n) return fail(c, ARTOPK_EINVAL, "N=%lld outside [1, %lld]", (long long)n, (long long)c->max_n);
  if (n >= (1ll << 31)) return fail(c, ARTOPK_EINVAL, "N must be below 2^31");
  if (k < 1 || k > n) return fail(c, ARTOPK_EINVAL, "k=%lld outside [1, N]", (long long)k);
  if (k > c->max_k) return fail(c, ARTOPK_EINVAL, "k=%lld above max_k=%lld", (long long)k, (long long)c->max_k);
  return ARTOPK_OK;
}

int check_segments(artopk_ctx* c, int64_t n, int32_t nseg, const int64_t* seg_off, const int64_t* seg_k,
                   int64_t k) {
  if (nseg < 1) return fail(c, ARTOPK_EINVAL, "nseg must be >= 1");
  if (nseg > c->max_seg) return fail(c, ARTOPK_EINVAL, "nseg=%d above max_segments=%d", nseg, c->max_seg);
  if ((seg_off == nullptr) != (seg_k == nullptr))
    return fail(c, ARTOPK_EINVAL, "seg_off and seg_k must both be given or both be NULL");
  if (!seg_off) {
    if (nseg != 1) return fail(c, ARTOPK_EINVAL, "nseg > 1 needs seg_off and seg_k");
    return ARTOPK_OK;
  }
  if (seg_off[0] != 0 || seg_off[nseg] != n) return fail(c, ARTOPK_EINVAL, "segments must cover [0, N)");
  int64_t ksum = 0;
  for (int s = 0; s < nseg; ++s) {
    const int64_t sz = seg_off[s + 1] - seg_off[s];
    if (sz < 1) return fail(c, ARTOPK_EINVAL, "segment %d is empty or descending", s);
    if (seg_k[s] < 1 || seg_k[s] > sz) return fail(c, ARTOPK_EINVAL, "seg_k[%d] outside [1, size]", s);
    ksum += seg_k[s];
  }
  if (ksum != k) return fail(c, ARTOPK_EINVAL, "sum of seg_k (%lld) differs from k (%lld)", (long long)ksum, (long long)k);
  return ARTOPK_OK;
}

// The buffers of one call as byte ranges.  Ranges that are only read may overlap each other
// (two workers may share a gradient buffer); a range that is written must not overlap any other.
class RangeSet {
 public:
  void add(const void* p, size_t bytes, bool written, const char* name, int index = -1) {
    if (!p || bytes == 0 || n_ >= kCap) return;
    const uintptr_t lo = reinterpret_cast<uintptr_t>(p);
    r_[n_++] = Range{lo, lo + bytes, written, name, index};
  }
  void add_table(const void* const* tab, int32_t w, size_t bytes, bool written, const char* name) {
    for (int i = 0; i < w; ++i) add(tab[i], bytes, written, name, i);
  }
  // ARTOPK_OK, or ARTOPK_EINVAL with the first offending pair in the context's error text
  int check(artopk_ctx* c) {
    std::sort(r_, r_ + n_, [](const Range& a, const Range& b) { return a.lo < b.lo; });
    int far_any = -1, far_written = -1;  // ranges seen so far that reach furthest: any, written ones
    for (int i = 0; i < n_; ++i) {
      const int other = r_[i].written ? far_any : far_written;
      if (other >= 0 && r_[i].lo < r_[other].hi) {
        char a[48], b[48];
        label(r_[other], a, sizeof(a));
        label(r_[i], b, sizeof(b));
        return fail(c, ARTOPK_EINVAL, "buffers %s and %s overlap", a, b);
      }
      if (far_any < 0 || r_[i].hi > r_[far_any].hi) far_any = i;
      if (r_[i].written && (far_written < 0 || r_[i].hi > r_[far_written].hi)) far_written = i;
    }
    return ARTOPK_OK;
  }

 private:
  struct Range {
    uintptr_t lo, hi;
    bool written;
    const char* name;
    int index;
  };
  static void label(const Range& r, char* out, size_t cap) {
    if (r.index >= 0)
      snprintf(out, cap, "%s[%d]", r.name, r.index);
    else
      snprintf(out, cap, "%s", r.name);
  }
  static constexpr int kCap = 2 * kMaxW + 8;
  Range r_[kCap];
  int n_ = 0;
};

PtrTable make_table(const float* const* tab, int32_t w) {
  PtrTable t;
  for (int i = 0; i < kMaxW; ++i) t.p[i] = (i < w) ? const_cast<float*>(tab[i]) : nullptr;
  return t;
}

// Chunk layout of the element range [e_lo, e_hi): at most max_chunks chunks of
// whole tiles, chunk 0 starting at the tile boundary at or below e_lo.
ChunkGeom make_geom(int64_t e_lo, int64_t e_hi, int64_t max_chunks = kMaxChunks, bool whole_pass_tiles = false) {
  ChunkGeom g;
  g.chunk0 = e_lo / kTile * kTile;
  const int64_t span = e_hi - g.chunk0;
  int64_t ce = (span + max_chunks - 1) / max_chunks;
  ce = (ce + kTile - 1) / kTile * kTile;
  if (ce < kTile) ce = kTile;
  // chunks longer than one tile of the fused pass are whole tiles of it, so that only the last
  // chunk of a vector has a ragged tile
  // (and always, if the pass strides over its tiles and counts per chunk)
  constexpr int64_t pass_tile = (int64_t)kPassAThreads * kPassAU * 4;
  static_assert(pass_tile == kPassTile, "the kernels' tile");
  if (ce > kTile || whole_pass_tiles) ce = (ce + pass_tile - 1) / pass_tile * pass_tile;
  g.chunk_elems = ce;
  g.nchunks = (int32_t)((span + ce - 1) / ce);
  if (g.nchunks < 1) g.nchunks = 1;
  return g;
}

// Blocks per worker of the stand-alone variance kernel.
int stats_blocks(int num_cu, int32_t w, int64_t n) {
  const int64_t n4 = n >> 2;
  const int64_t tile = 256 * kPassAUnroll;
  int64_t ntile = (n4 + tile - 1) / tile;
  if (ntile < 1) ntile = 1;
  int64_t want = ((int64_t)num_cu * 8 + w - 1) / w;
  if (want < 1) want = 1;
  int64_t nblk = ntile < want ? ntile : want;
  if (nblk > kMaxChunks) nblk = kMaxChunks;
  return (int)nblk;
}

// A stage boundary (level 2 only).
void prof_mark(artopk_ctx* c, int mark) {
  if (!c->profile || c->profile_level < 2) return;
  if (hipEventRecord(c->ev[c->cur][mark], c->stream) == hipSuccess) c->ev_valid[c->cur][mark] = true;
}

// Level 1: the two events directly around the launch of the step's dominant kernel, stored as the
// marks lvl1_a / lvl1_b so that they read as that kernel's stage.
void prof_dom(artopk_ctx* c, bool end) {
  if (!c->profile || c->profile_level != 1) return;
  const int mark = end ? c->lvl1_b : c->lvl1_a;
  if (hipEventRecord(c->ev[c->cur][mark], c->stream) == hipSuccess) c->ev_valid[c->cur][mark] = true;
}

// Starts the record of a new call in the next ring slot.
void prof_begin(artopk_ctx* c) {
  if (!c->profile) return;
  c->cur = (int)(c->prof_calls % artopk_ctx::kRing);
  c->prof_calls++;
  for (int i = 0; i < artopk_ctx::kMarks; ++i) c->ev_valid[c->cur][i] = false;
}

int64_t tiles_of_range(int64_t e_lo, int64_t e_hi) {
  return (e_hi + kCompactTile - 1) / kCompactTile - e_lo / kCompactTile;
}

int64_t seg_list_cap(int64_t n_s, int64_t k_s) {
  int64_t share = n_s / 8;
  if (share < 4096) share = 4096;
  int64_t cap = k_s + share;
  return cap < n_s ? cap : n_s;
}

// One segment covering the whole vector.
Plan flat_plan(const artopk_ctx* c, int64_t n, int64_t k, int32_t vec = -1, bool whole_pass_tiles = false) {
  Plan pl;
  pl.nseg = 1;
  SegDesc d{};
  d.e_lo = 0;
  d.e_hi = n;
  d.geom = make_geom(0, n, kMaxChunks, whole_pass_tiles);
  d.koff = 0;
  d.list_base = 0;
  d.flag_base = 0;
  d.chunk_begin = 0;
  d.k = (uint32_t)k;
  d.cap = c->s.cap < (uint64_t)n ? c->s.cap : (uint32_t)n;
  d.vec = vec;
  pl.desc.push_back(d);
  pl.max_chunks = d.geom.nchunks;
  pl.max_tiles = pl.total_tiles = tiles_of_range(0, n);
  pl.max_cap = d.cap;
  return pl;
}

// Descriptors for nseg > 1 segments; uploads them to the device table unless the
// same layout is already there.  Copies from pageable memory, so the host
// buffer may be reused as soon as the call returns.
int segmented_plan(artopk_ctx* c, int64_t n, int32_t nseg, const int64_t* seg_off, const int64_t* seg_k,
                   const Plan** out) {
  const bool same = c->cached_n == n && (int32_t)c->cached_k.size() == nseg &&
                    memcmp(c->cached_off.data(), seg_off, sizeof(int64_t) * (nseg + 1)) == 0 &&
                    memcmp(c->cached_k.data(), seg_k, sizeof(int64_t) * nseg) == 0;
  if (!same) {
    Plan pl;
    pl.nseg = nseg;
    pl.use_table = true;
    pl.max_chunks = 1;
    pl.max_tiles = 1;
    pl.total_tiles = 0;
    pl.max_cap = 1;
    int64_t koff = 0, list_base = 0, flag_base = 0;
    int32_t chunk_begin = 0;
    for (int sgi = 0; sgi < nseg; ++sgi) {
      SegDesc d{};
      d.e_lo = seg_off[sgi];
      d.e_hi = seg_off[sgi + 1];
      const int64_t ns = d.e_hi - d.e_lo;
      int64_t mc = (int64_t)((double)kMaxChunks * (double)ns / (double)n);
      if (mc < 1) mc = 1;
      d.geom = make_geom(d.e_lo, d.e_hi, mc);
      d.koff = koff;
      d.list_base = list_base;
      d.flag_base = flag_base;
      d.chunk_begin = chunk_begin;
      d.k = (uint32_t)seg_k[sgi];
      d.cap = (uint32_t)seg_list_cap(ns, seg_k[sgi]);
      d.vec = -1;
      koff += seg_k[sgi];
      list_base += ((int64_t)d.cap + 3) / 4 * 4;
      const int64_t tiles = tiles_of_range(d.e_lo, d.e_hi);
      flag_base += tiles;
      chunk_begin += d.geom.nchunks;
      if (d.geom.nchunks > pl.max_chunks) pl.max_chunks = d.geom.nchunks;
      if (tiles > pl.max_tiles) pl.max_tiles = tiles;
      if ((int64_t)d.cap > pl.max_cap) pl.max_cap = d.cap;
      pl.desc.push_back(d);
    }
    pl.total_tiles = flag_base;
    if (list_base > c->s.list_entries || flag_base > c->s.max_tiles || chunk_begin > kMaxChunks + c->max_seg)
      return fail(c, ARTOPK_EINVAL, "segment layout exceeds the scratch sized at artopk_create");
    HIP_TRY(c, hipMemcpyAsync(c->s.table_dev, pl.desc.data(), sizeof(SegDesc) * nseg, hipMemcpyHostToDevice,
                              c->stream));
    // one block per chunk of the layout for the per-chunk kernels (a (chunks, segments) grid of a layout
    // with one long and many short segments is mostly blocks that find nothing to do)
    std::vector<uint32_t> cmap;
    cmap.reserve((size_t)chunk_begin);
    for (int sgi = 0; sgi < nseg; ++sgi)
      for (int32_t ch = 0; ch < pl.desc[sgi].geom.nchunks; ++ch) cmap.push_back(((uint32_t)sgi << 16) | (uint32_t)ch);
    HIP_TRY(c, hipMemcpyAsync(c->s.chunk_map, cmap.data(), sizeof(uint32_t) * cmap.size(), hipMemcpyHostToDevice,
                              c->stream));
    pl.total_chunks = chunk_begin;
    c->cached_plan = pl;
    c->cached_n = n;
    c->cached_off.assign(seg_off, seg_off + nseg + 1);
    c->cached_k.assign(seg_k, seg_k + nseg);
  }
  *out = &c->cached_plan;
  return ARTOPK_OK;
}

SelParams make_params(const artopk_ctx* c, const Plan& pl, const PtrTable& tab, int64_t n, int32_t* idx_out,
                      float* vals_row, int slot_by_leader, bool hist_from_pass) {
  const Scratch& s = c->s;
  SelParams p;
  p.tab = tab;
  p.leader_dev = s.leader_dev;
  p.n = n;
  p.h_all = hist_from_pass ? s.h_all : nullptr;
  p.mask = nullptr;
  p.mask_stride = s.mask_stride;
  p.tiles = TileBuf{nullptr, nullptr, 0, 0, 0};
  p.use_mcount = 0;
  p.from_list = 0;
  p.after_mask = 0;
  p.only_if_need_full = 0;
  p.zero_base = s.zero_base;
  p.flags = s.flags;
  p.S = s.S;
  p.chunk_off = s.chunk_off;
  p.list = s.list;
  p.idx_out = idx_out;
  p.vals_row = vals_row;
  p.zero_vec = nullptr;
  p.err = s.err_dev;
  p.table = pl.use_table ? s.table_dev : nullptr;
  p.chunk_map = (pl.use_table && pl.total_chunks > 0) ? s.chunk_map : nullptr;
  p.slot_by_leader = slot_by_leader;
  p.one = pl.desc[0];
  return p;
}

// Clears the per-segment scratch blocks and the look-back flags of a plan, and the
// whole-vector histograms of the first hist_slots slots a fused pass is about to fill.
// leader >= 0 also records a host-known leader (and copies it to leader_out).
int enqueue_clear(artopk_ctx* c, const Plan& pl, int hist_slots, int32_t leader = -1,
                  int32_t* leader_out = nullptr) {
  Scratch& s = c->s;
  const size_t words1 = (size_t)pl.nseg * kSegWords;
  const size_t words2 = (size_t)pl.total_tiles * kNumLookback * 2;
  const size_t words3 = (size_t)hist_slots * kSlotWords;
  const size_t total = words1 + words2 + words3;
  int blocks = (int)((total + 256 * 8 - 1) / (256 * 8));
  if (blocks < 1) blocks = 1;
  if (blocks > c->num_cu * 4) blocks = c->num_cu * 4;
  hipLaunchKernelGGL(k_fill_zero, dim3(blocks), dim3(256), 0, c->stream, s.zero_base, words1,
                     reinterpret_cast<uint32_t*>(s.flags), words2, s.h_all, words3, leader,
                     leader >= 0 ? s.leader_dev : nullptr, leader_out);
  HIP_TRY(c, hipGetLastError());
  return ARTOPK_OK;
}

// Launches the fused pass over grid.y workers with the wanted options.
template <int STATS, int HIST, int GT>
void launch_pass_a_g(artopk_ctx* c, dim3 grid, const PtrTable& g, const PtrTable& r, int64_t n, const ChunkGeom& geom,
                     int hist_worker) {
  Scratch& s = c->s;
  if (c->pass_a_nt)
    hipLaunchKernelGGL((k_pass_a<STATS, HIST, true, GT, kPassAThreads, kPassAU>), grid, dim3(kPassAThreads), 0,
                       c->stream, g, r, n, geom, hist_worker, s.S, s.h_all, s.partials);
  else
    hipLaunchKernelGGL((k_pass_a<STATS, HIST, false, GT, kPassAThreads, kPassAU>), grid, dim3(kPassAThreads), 0,
                       c->stream, g, r, n, geom, hist_worker, s.S, s.h_all, s.partials);
}

template <int STATS, int HIST>
void launch_pass_a_t(artopk_ctx* c, dim3 grid, const PtrTable& g, const PtrTable& r, int64_t n, const ChunkGeom& geom,
                     int hist_worker) {
  if (c->g_type == ARTOPK_G_BF16)
    launch_pass_a_g<STATS, HIST, kGBF16>(c, grid, g, r, n, geom, hist_worker);
  else if (c->g_type == ARTOPK_G_F16)
    launch_pass_a_g<STATS, HIST, kGF16>(c, grid, g, r, n, geom, hist_worker);
  else
    launch_pass_a_g<STATS, HIST, kGF32>(c, grid, g, r, n, geom, hist_worker);
}

void launch_pass_a(artopk_ctx* c, int stats, int hist, dim3 grid, const PtrTable& g, const PtrTable& r, int64_t n,
                   const ChunkGeom& geom, int hist_worker) {
#define PASS_A_CASE(S_, H_) \
  if (stats == S_ && hist == H_) return launch_pass_a_t<S_, H_>(c, grid, g, r, n, geom, hist_worker)
  PASS_A_CASE(0, 0);
  PASS_A_CASE(0, 1);
  PASS_A_CASE(0, 2);
  PASS_A_CASE(1, 0);
  PASS_A_CASE(1, 2);
  PASS_A_CASE(2, 0);
  PASS_A_CASE(2, 2);
#undef PASS_A_CASE
}

// Blocks per worker of a streaming pass that strides over the tiles of n elements.
int pass_blocks(int64_t n) {
  const int64_t ntiles = (n + kPassTile - 1) / kPassTile;
  return (int)(ntiles < kMaxPassBlocks ? ntiles : kMaxPassBlocks);
}

// The other workers' pass does best with fewer, longer-lived blocks (measured on 138 M x 3: 0.84 ms
// with 512 per worker against 0.85 - 0.87 with 1024 - 2048; no difference on 1e9 x 7), the marking
// pass with many (1e9 x 8: 16.35 ms with 4096 per worker, 16.55 with 2048).
int rest_blocks(int64_t n) {
  const int64_t ntiles = (n + kPassTile - 1) / kPassTile;
  return (int)(ntiles < 512 ? ntiles : 512);
}

// What the fused pass stages per tile for one marking worker (slot 0), or nothing.
TileBuf tile_buf(const artopk_ctx* c, int32_t tile_cap) {
  if (tile_cap <= 0) return TileBuf{nullptr, nullptr, 0, 0, 0};
  return TileBuf{c->s.tilebuf, c->s.tile_cnt, 0, 0, tile_cap};
}

// The fused pass of the guess route over the first nw workers of the tables (worker y in slot y).
// tile_cap > 0 (one worker, no statistics): the pass also stages the marked elements per tile.
template <int STATS, int GT, bool STAGE>
void launch_pass_mark_g(artopk_ctx* c, int nw, const PtrTable& g, const PtrTable& r, int64_t n, int64_t chunk_elems,
                        int32_t tile_cap) {
  Scratch& s = c->s;
  const dim3 grid(pass_blocks(n), nw);
  const TileBuf tb = tile_buf(c, STAGE ? tile_cap : 0);
  if (c->pass_a_nt)
    hipLaunchKernelGGL((k_pass_mark<STATS, true, GT, kPassAThreads, kPassAU, STAGE>), grid, dim3(kPassAThreads), 0,
                       c->stream, g, r, n, chunk_elems, s.h_all, s.mask, s.mask_stride, s.partials, tb);
  else
    hipLaunchKernelGGL((k_pass_mark<STATS, false, GT, kPassAThreads, kPassAU, STAGE>), grid, dim3(kPassAThreads), 0,
                       c->stream, g, r, n, chunk_elems, s.h_all, s.mask, s.mask_stride, s.partials, tb);
}

template <int STATS, bool STAGE>
void launch_pass_mark_t(artopk_ctx* c, int nw, const PtrTable& g, const PtrTable& r, int64_t n, int64_t chunk_elems,
                        int32_t tile_cap) {
  if (c->g_type == ARTOPK_G_BF16)
    launch_pass_mark_g<STATS, kGBF16, STAGE>(c, nw, g, r, n, chunk_elems, tile_cap);
  else if (c->g_type == ARTOPK_G_F16)
    launch_pass_mark_g<STATS, kGF16, STAGE>(c, nw, g, r, n, chunk_elems, tile_cap);
  else
    launch_pass_mark_g<STATS, kGF32, STAGE>(c, nw, g, r, n, chunk_elems, tile_cap);
}

void launch_pass_mark(artopk_ctx* c, int stats, int nw, const PtrTable& g, const PtrTable& r, int64_t n,
                      int64_t chunk_elems, int32_t tile_cap = 0) {
  if (stats == 0 && tile_cap > 0 && nw == 1) return launch_pass_mark_t<0, true>(c, nw, g, r, n, chunk_elems, tile_cap);
  if (stats == 0) return launch_pass_mark_t<0, false>(c, nw, g, r, n, chunk_elems, 0);
  if (stats == 1) return launch_pass_mark_t<1, false>(c, nw, g, r, n, chunk_elems, 0);
  return launch_pass_mark_t<2, false>(c, nw, g, r, n, chunk_elems, 0);
}

// The striding pass without a bound: error-feedback add and statistics of all w workers (per-block
// moments of pass_blocks(n) blocks per worker in partials).
template <int STATS, int GT>
void launch_pass_plain_g(artopk_ctx* c, int nw, const PtrTable& g, const PtrTable& r, int64_t n) {
  Scratch& s = c->s;
  const dim3 grid(pass_blocks(n), nw);
  const TileBuf tb = tile_buf(c, 0);
  if (c->pass_a_nt)
    hipLaunchKernelGGL((k_pass_mark<STATS, true, GT, kPassAThreads, kPassAU, false, true>), grid, dim3(kPassAThreads), 0,
                       c->stream, g, r, n, (int64_t)kPassTile, s.h_all, s.mask, s.mask_stride, s.partials, tb);
  else
    hipLaunchKernelGGL((k_pass_mark<STATS, false, GT, kPassAThreads, kPassAU, false, true>), grid, dim3(kPassAThreads), 0,
                       c->stream, g, r, n, (int64_t)kPassTile, s.h_all, s.mask, s.mask_stride, s.partials, tb);
}

template <int STATS>
void launch_pass_plain_t(artopk_ctx* c, int nw, const PtrTable& g, const PtrTable& r, int64_t n) {
  if (c->g_type == ARTOPK_G_BF16)
    launch_pass_plain_g<STATS, kGBF16>(c, nw, g, r, n);
  else if (c->g_type == ARTOPK_G_F16)
    launch_pass_plain_g<STATS, kGF16>(c, nw, g, r, n);
  else
    launch_pass_plain_g<STATS, kGF32>(c, nw, g, r, n);
}

void launch_pass_plain(artopk_ctx* c, int stats, int nw, const PtrTable& g, const PtrTable& r, int64_t n) {
  if (stats == 0) return launch_pass_plain_t<0>(c, nw, g, r, n);
  if (stats == 1) return launch_pass_plain_t<1>(c, nw, g, r, n);
  return launch_pass_plain_t<2>(c, nw, g, r, n);
}

template <int GT>
void launch_pass_rest_g(artopk_ctx* c, dim3 grid, const PtrTable& g, const PtrTable& r, int w, int leader, int64_t n,
                        const int32_t* idx, int64_t k, float* vals) {
  Scratch& s = c->s;
  if (c->pass_a_nt)
    hipLaunchKernelGGL((k_pass_rest<true, GT, kPassRestThreads, kPassRestU>), grid, dim3(kPassRestThreads), 0, c->stream,
                       g, r, w, leader, n, idx, k, vals, s.tile_start, s.err_dev);
  else
    hipLaunchKernelGGL((k_pass_rest<false, GT, kPassRestThreads, kPassRestU>), grid, dim3(kPassRestThreads), 0, c->stream,
                       g, r, w, leader, n, idx, k, vals, s.tile_start, s.err_dev);
}

// The number of kept indices below every tile of the streaming passes.
void enqueue_tile_starts(artopk_ctx* c, const int32_t* idx, int64_t n, int64_t k) {
  const int32_t ntiles = (int32_t)((n + kPassTile - 1) / kPassTile);
  // many kept indices per tile: a search per tile boundary beats a thread per index
  // (138 M elements, one in ten kept: 20 us with a thread per index)
  if (k > (int64_t)1024 * ntiles)
    hipLaunchKernelGGL(k_tile_starts_search, dim3((unsigned)(ntiles / 256 + 1)), dim3(256), 0, c->stream, idx, k,
                       ntiles, c->s.tile_start);
  else
    hipLaunchKernelGGL(k_tile_starts, dim3((unsigned)((k + 255) / 256)), dim3(256), 0, c->stream, idx, k, ntiles,
                       c->s.tile_start);
}

// The other workers' streaming pass (leader known, idx final), striding over the tiles;
// k_tile_starts must have run on idx.
void launch_pass_rest(artopk_ctx* c, const PtrTable& g, const PtrTable& r, int w, int leader, int64_t n,
                      const int32_t* idx, int64_t k, float* vals) {
  const dim3 grid(rest_blocks(n), w - 1);
  if (c->g_type == ARTOPK_G_BF16)
    launch_pass_rest_g<kGBF16>(c, grid, g, r, w, leader, n, idx, k, vals);
  else if (c->g_type == ARTOPK_G_F16)
    launch_pass_rest_g<kGF16>(c, grid, g, r, w, leader, n, idx, k, vals);
  else
    launch_pass_rest_g<kGF32>(c, grid, g, r, w, leader, n, idx, k, vals);
}

// Whether a flat step on n elements keeping k uses the sampled threshold guess.
struct GuessPlan {
  bool on = false;
  int runs = 0;
  int64_t stride = 0;
  uint32_t m_hi = 0;
  int32_t tile_cap = 0;  // > 0: one marking worker, whose fused pass stages up to this many list entries per tile
};

// marking = number of workers whose fused pass will mark (1: a leader known up front).
GuessPlan plan_guess(const artopk_ctx* c, int64_t n, int64_t k, int marking) {
  GuessPlan gp;
  if (c->s.mask == nullptr || n < c->guess_min_n) return gp;
  // A selection of more than one element in 32 is not worth fetching entry by entry from the mask.
  // With one marking worker its fused pass hands the marked elements on per tile instead (measured on
  // 138 M elements: one in ten kept 1.73 ms a step against 1.92 on the histogram route, one in a
  // hundred 1.40 against 1.43 with the mask alone, one in a thousand 1.365 against 1.347: a tile has
  // to hand on a hundred elements or so for the pieces to pay for what they cost the pass, so
  // sparser selections keep the mask alone unless the option asks for pieces everywhere).  Entries a
  // tile is expected to hand on: the keys reaching the guessed bound are at most about 1.2 k (the
  // bound is the lower edge of a top-digit bin, or with pieces of a second-digit bin), spread over
  // the tiles; room for 1.3 k's share plus six standard deviations of a tile's count.  Selections
  // too dense for a piece take the histogram route.
  const bool dense = k * 32 > n;
  const bool worth_pieces = k * 256 >= n;  // 128 kept elements per tile or more
  const double per_tile = 1.3 * (double)k * (double)kPassTile / (double)n;
  const int64_t want = ((int64_t)std::ceil(per_tile + 6.0 * std::sqrt(per_tile) + 32.0) + 63) / 64 * 64;
  const int64_t ntiles = (n + kPassTile - 1) / kPassTile;
  if ((c->stage_tiles == 2 || (c->stage_tiles == 1 && worth_pieces)) && marking == 1 && want <= kStageMax &&
      ntiles * want <= c->s.tilebuf_entries)
    gp.tile_cap = (int32_t)want;
  if (gp.tile_cap == 0 && dense) return gp;
  int64_t runs = n / (4 * kGuessRun);  // at most a quarter of the vector
  if (runs > 16384) runs = 16384;
  if (runs < 256) return gp;
  gp.runs = (int)runs;
  gp.stride = n / runs;
  // keys of the sample expected above the true threshold, plus six standard deviations and a few
  const double expect = (double)k * (double)(runs * kGuessRun) / (double)n;
  gp.m_hi = (uint32_t)std::ceil(expect + 6.0 * std::sqrt(expect) + 8.0);
  gp.on = (int64_t)gp.m_hi <= runs * kGuessRun;
  return gp;
}

// Samples the first nvec vectors of (g + residual) into slots 0 .. nvec-1 (cleared beforehand).
void enqueue_guess(artopk_ctx* c, const GuessPlan& gp, const PtrTable& g, const PtrTable& res, int nvec) {
  // one vector whose marked elements are handed on per tile: a finer bound keeps the list (and the
  // number of values to give back afterwards) close to k
  uint32_t* sample = (nvec == 1 && gp.tile_cap > 0) ? c->s.sample_keys : nullptr;
  // about 128 blocks over all vectors (measured: 8 vectors take 70 us with 64 blocks each, 32 us
  // with 16; one vector 15 us with 64 blocks, 19 us with 16)
  int gblocks = 128 / nvec;
  if (gblocks > 64) gblocks = 64;
  if (gblocks < 8) gblocks = 8;
  if (c->g_type == ARTOPK_G_BF16)
    hipLaunchKernelGGL(k_guess<kGBF16>, dim3(gblocks, nvec), dim3(256), 0, c->stream, g, res, c->s.h_all, gp.runs,
                       gp.stride, gp.m_hi, sample);
  else if (c->g_type == ARTOPK_G_F16)
    hipLaunchKernelGGL(k_guess<kGF16>, dim3(gblocks, nvec), dim3(256), 0, c->stream, g, res, c->s.h_all, gp.runs,
                       gp.stride, gp.m_hi, sample);
  else
    hipLaunchKernelGGL(k_guess<kGF32>, dim3(gblocks, nvec), dim3(256), 0, c->stream, g, res, c->s.h_all, gp.runs,
                       gp.stride, gp.m_hi, sample);
  if (sample != nullptr)
    hipLaunchKernelGGL(k_guess_refine, dim3(64), dim3(256), 0, c->stream, c->s.h_all, sample, gp.runs * kGuessRun,
                       gp.m_hi);
}

// Top-k of every segment of the plan on the vector tab.p[*leader_dev]; the
// scratch must have been cleared.  If hist_ready the per-chunk suffix
// histograms are already in S (flat plans only: pass A built them, in slot
// *leader_dev if slot_by_leader, else in slot 0).  vals_row, if given, receives
// the leader's values at the selected indices.
int enqueue_select(artopk_ctx* c, const Plan& pl, const PtrTable& tab, int64_t n, int32_t* idx_out,
                   bool hist_ready, int slot_by_leader, float* vals_row = nullptr,
                   const LeaderArgs* leader_args = nullptr, bool guessed = false, float* zero_vec = nullptr,
                   int32_t tile_cap = 0) {
  hipStream_t st = c->stream;
  const unsigned nseg = (unsigned)pl.nseg;
  SelParams p = make_params(c, pl, tab, n, idx_out, vals_row, hist_ready ? slot_by_leader : 0, hist_ready);
  p.zero_vec = zero_vec;
  LeaderArgs la{};
  if (leader_args) la = *leader_args;
  // the per-chunk kernels: one block per chunk of a segmented layout, else a (chunks, segments) grid
  const dim3 chunk_grid = p.chunk_map ? dim3((unsigned)pl.total_chunks, 1) : dim3(pl.max_chunks, nseg);

  if (guessed && hist_ready) {
    // The fused pass marked and counted the keys reaching a guessed bound.  If the bound works out
    // the list is written from the mask and the threshold digit taken from the list; otherwise the
    // state says need_full, and the same two launches build the histogram of every key and pick
    // from that, after which the selection goes on as without a guess.
    p.mask = c->s.mask;
    p.tiles = tile_buf(c, tile_cap);
    p.use_mcount = 1;
    hipLaunchKernelGGL(k_pick_mask, dim3(1, nseg), dim3(1024), 0, st, p, la);
    SelParams pf = p;
    pf.h_all = nullptr;
    pf.only_if_need_full = 1;
    hipLaunchKernelGGL((k_mask_or_hist<4>), dim3(pl.max_chunks, nseg), dim3(1024), 0, st, p, pf);
    SelParams pa = p;
    pa.after_mask = 1;
    hipLaunchKernelGGL(k_pick0, dim3(1, nseg), dim3(1024), 0, st, pa, LeaderArgs{});
  } else {
    if (!hist_ready) hipLaunchKernelGGL(k_hist0<1024>, chunk_grid, dim3(1024), 0, st, p);
    hipLaunchKernelGGL(k_pick0, dim3(1, nseg), dim3(1024), 0, st, p, la);
  }

  // The remaining kernels take tiles from a counter (or stride over the list), so any grid works:
  // about two blocks per compute unit over all segments together.
  const int64_t per_seg = ((int64_t)c->num_cu * 2 + nseg - 1) / nseg;
  // deeper array passes: they run only for segments whose level-1 survivors did not fit the list,
  // which cannot happen if the list takes the whole range
  const bool always_fits = nseg == 1 && (int64_t)pl.desc[0].cap >= pl.desc[0].e_hi - pl.desc[0].e_lo;
  int cblocks = (int)(pl.max_tiles < per_seg ? pl.max_tiles : per_seg);
  if (cblocks < 1) cblocks = 1;

  int64_t lblocks = (pl.max_cap + 256 * 16 - 1) / (256 * 16);
  if (lblocks > per_seg * 2) lblocks = per_seg * 2;
  if (lblocks < 1) lblocks = 1;
  // level 1: ordered compaction of the array (4 waves, 16 consecutive elements per lane: best of the
  // shapes measured on the 138 M and 1 G workloads); on the guess route the same launch counts
  // the second digit over a list that was written from the mask
  const bool long_list = nseg == 1 && (int64_t)pl.desc[0].k * 32 > n;
  if (guessed && hist_ready && long_list) {
    // a list of many millions of entries written from the staged pieces: the lean list kernel
    // counts its second digit; the array pass stands by for a guess that did not hold
    hipLaunchKernelGGL(k_list_hist, dim3((unsigned)lblocks, nseg), dim3(256), 0, st, p, 1);
    hipLaunchKernelGGL((k_compact1<kC1Waves, kC1R>), dim3(pl.max_chunks, nseg), dim3(64 * kC1Waves), 0, st, p);
  } else if (guessed && hist_ready) {
    const int64_t b1 = lblocks > pl.max_chunks ? lblocks : pl.max_chunks;
    hipLaunchKernelGGL(k_level1, dim3((unsigned)b1, nseg), dim3(64 * kC1Waves), 0, st, p);
  } else {
    // (8 waves a block: 21.6 against 27.6 us with 4 on 11.7 M elements, 35 against 38 us on 25.6 M in 54 segments)
    hipLaunchKernelGGL((k_compact1<8, kC1R>), chunk_grid, dim3(512), 0, st, p);
  }
  // A list of many millions of entries (one element in 32 kept, or more) is counted faster by the
  // lean kernel of its own (99 vs 66 us on 15 M entries: the merged one carries the array pass'
  // registers), which is worth the launch of an array pass that has nothing to do.
  if (always_fits) {
    hipLaunchKernelGGL(k_list_hist, dim3((unsigned)lblocks, nseg), dim3(256), 0, st, p, 2);
  } else if (long_list) {
    hipLaunchKernelGGL(k_compact<false>, dim3(cblocks, nseg), dim3(kCompactThreads), 0, st, p, 2, 0);
    hipLaunchKernelGGL(k_list_hist, dim3((unsigned)lblocks, nseg), dim3(256), 0, st, p, 2);
  } else {  // the same launch is the level-2 array pass where the level-1 survivors did not fit the list
    const int64_t b2 = lblocks > cblocks ? lblocks : cblocks;
    hipLaunchKernelGGL(k_level2, dim3((unsigned)b2, nseg), dim3(kCompactThreads), 0, st, p);
  }
  int64_t ltiles = (pl.max_cap + kCompactTile - 1) / kCompactTile;
  int fblocks = (int)(ltiles < per_seg ? ltiles : per_seg);
  if (fblocks < 1) fblocks = 1;
  if (always_fits) {
    hipLaunchKernelGGL(k_compact<true>, dim3(fblocks, nseg), dim3(kCompactThreads), 0, st, p, 3, 2);
  } else {  // the same launch is the level-3 array pass where no list could be written
    if (fblocks < cblocks) fblocks = cblocks;
    hipLaunchKernelGGL(k_final, dim3(fblocks, nseg), dim3(kCompactThreads), 0, st, p);
  }
  HIP_TRY(c, hipGetLastError());
  return ARTOPK_OK;
}

int enqueue_gather(artopk_ctx* c, const PtrTable& tab, int32_t w, int64_t n, const int32_t* idx, int64_t k,
                   float* vals, float* sum, bool zero) {
  const int blocks = (int)((k + 255) / 256);
  if (zero)
    hipLaunchKernelGGL(k_gather<true>, dim3(blocks), dim3(256), 0, c->stream, tab, (int)w, n, idx, k, vals, sum,
                       c->s.err_dev);
  else
    hipLaunchKernelGGL(k_gather<false>, dim3(blocks), dim3(256), 0, c->stream, tab, (int)w, n, idx, k, vals, sum,
                       c->s.err_dev);
  HIP_TRY(c, hipGetLastError());
  return ARTOPK_OK;
}

// tiles_ready: k_tile_starts has already run on this idx.
int enqueue_update_fill(artopk_ctx* c, float* update, int64_t n, const int32_t* idx, const float* sum,
                        int64_t k, bool tiles_ready = false) {
  // long vectors with few kept entries: zeros streamed tile by tile, values stored behind them
  // (measured on 138 M elements: faster at k = N / 1000, even at N / 100, 40 % slower at N / 10)
  if (n >= c->update_tiles_min_n && k * 128 <= n) {
    if (!tiles_ready) enqueue_tile_starts(c, idx, n, k);
    if (n < ((int64_t)1 << 28))  // (which kind of store the zeros take: measured, see the kernel)
      hipLaunchKernelGGL((k_update_tiles<kPassRestThreads, kPassRestU, true>), dim3(pass_blocks(n)),
                         dim3(kPassRestThreads), 0, c->stream, update, n, idx, sum, k, c->s.tile_start, c->s.err_dev);
    else
      hipLaunchKernelGGL((k_update_tiles<kPassRestThreads, kPassRestU, false>), dim3(pass_blocks(n)),
                         dim3(kPassRestThreads), 0, c->stream, update, n, idx, sum, k, c->s.tile_start, c->s.err_dev);
    HIP_TRY(c, hipGetLastError());
    return ARTOPK_OK;
  }
  const int64_t nchunk = (n + kFillChunk - 1) / kFillChunk;
  int blocks = (int)(nchunk < (int64_t)c->num_cu * 4 ? nchunk : (int64_t)c->num_cu * 4);
  if (blocks < 1) blocks = 1;
  // kept entries expected per 8192-element chunk decide how many are fetched per round
  const double per_chunk = (double)k / (double)n * kFillChunk;
  if (tiles_ready && n >= c->update_tiles_min_n) {
    // the tiles' first indices are there already: blocks stride over the tiles
    const int64_t ntiles = (n + kPassTile - 1) / kPassTile;
    const int tb = (int)(ntiles < (int64_t)c->num_cu * 4 ? ntiles : (int64_t)c->num_cu * 4);
    if (per_chunk <= 160.0)
      hipLaunchKernelGGL((k_update_fill_tiled<1>), dim3(tb), dim3(256), 0, c->stream, update, n, idx, sum, k, c->s.tile_start);
    else if (per_chunk <= 400.0)
      hipLaunchKernelGGL((k_update_fill_tiled<2>), dim3(tb), dim3(256), 0, c->stream, update, n, idx, sum, k, c->s.tile_start);
    else
      hipLaunchKernelGGL((k_update_fill_tiled<4>), dim3(tb), dim3(256), 0, c->stream, update, n, idx, sum, k, c->s.tile_start);
    HIP_TRY(c, hipGetLastError());
    return ARTOPK_OK;
  }
  if (per_chunk <= 160.0) {
    hipLaunchKernelGGL((k_update_fill<1>), dim3(blocks), dim3(256), 0, c->stream, update, n, idx, sum, k);
  } else if (per_chunk <= 400.0) {
    hipLaunchKernelGGL((k_update_fill<2>), dim3(blocks), dim3(256), 0, c->stream, update, n, idx, sum, k);
  } else {
    hipLaunchKernelGGL((k_update_fill<4>), dim3(blocks), dim3(256), 0, c->stream, update, n, idx, sum, k);
  }
  HIP_TRY(c, hipGetLastError());
  return ARTOPK_OK;
}


// Every worker's own Top-k (indices ascending, values) and the squared norm of its k values;
// argmax (first maximum) goes to leader_dev and, if given, argmax_out.  With hist_ready the
// per-chunk histograms of all workers are already in S (pass A with histograms for every worker).
int enqueue_topk_workers(artopk_ctx* c, const PtrTable& tab, int32_t w, int64_t n, int64_t k, int32_t* idx_rows,
                         float* val_rows, double* sqnorm_out, int32_t* argmax_out, bool hist_ready,
                         bool guessed = false) {
  Scratch& s = c->s;
  for (int32_t r = 0; r < w; ++r) {
    const Plan pl = flat_plan(c, n, k, r, guessed);
    int rc = enqueue_clear(c, pl, 0);
    if (rc) return rc;
    if ((rc = enqueue_select(c, pl, tab, n, idx_rows + (size_t)r * (size_t)k, hist_ready, 1,
                             val_rows + (size_t)r * (size_t)k, nullptr, guessed)))
      return rc;
  }
  PtrTable vtab;
  for (int i = 0; i < kMaxW; ++i) vtab.p[i] = (i < w) ? val_rows + (size_t)i * (size_t)k : nullptr;
  int nblk = (int)((k + 256 * 16 - 1) / (256 * 16));
  if (nblk < 1) nblk = 1;
  if (nblk > kMaxChunks) nblk = kMaxChunks;
  hipLaunchKernelGGL((k_stats<false, false>), dim3(nblk, w), dim3(256), 0, c->stream, vtab, k, s.partials);
  hipLaunchKernelGGL(k_sqnorm, dim3(1), dim3(1024), 0, c->stream, s.partials, nblk, (int)w, s.var_scratch,
                     sqnorm_out, s.leader_dev, argmax_out);
  HIP_TRY(c, hipGetLastError());
  return ARTOPK_OK;
}

}  // namespace

namespace {

// Where everything lies in the one allocation of a context.
struct Layout {
  uint32_t cap = 0;
  int64_t list_entries = 0, max_tiles = 0, mask_stride = 0, tilebuf_entries = 0;
  size_t o_hall = 0, o_mask = 0, o_zero = 0, o_S = 0, o_coff = 0, o_part = 0, o_var = 0, o_leader = 0, o_err = 0, o_counter = 0, o_list = 0, o_vals = 0, o_rows = 0, o_table = 0, o_cmap = 0, o_tstart = 0, o_tbuf = 0, o_tcnt = 0, o_sample = 0;
  size_t total = 0;
};

bool valid_limits(int32_t max_w, int64_t max_n, int64_t max_k, int32_t max_segments) {
  return !(max_w < 1 || max_w > ARTOPK_MAX_WORKERS || max_n < 1 || max_n >= (1ll << 31) || max_k < 1 ||
           max_k > max_n || max_segments < 1 || max_segments > 65535);
}

Layout scratch_layout(int32_t max_w, int64_t max_n, int64_t max_k, int32_t max_segments) {
  Layout L;
  // list capacity: every key above the range (< k of them) plus a generous share of candidates
  // (vectors of up to 4 Mi elements fit the list whole: their selection never needs the deeper
  // array passes, which are then not even launched)
  int64_t cand_share = max_n / 8;
  if (cand_share < ((int64_t)1 << 22)) cand_share = (int64_t)1 << 22;
  int64_t cap = max_k + cand_share;
  if (cap > max_n) cap = max_n;
  L.cap = (uint32_t)cap;
  // segmented layouts add per-segment rounding: n_s/8 may be raised to 4096 and bases are aligned
  L.list_entries = (int64_t)align_up((size_t)cap + (size_t)max_segments * 4100, kCompactTile) + kCompactTile;
  // a range [lo, hi) touches at most ceil(len / tile) + 1 look-back tiles
  L.max_tiles = (max_n + kCompactTile - 1) / kCompactTile + 2 * (int64_t)max_segments + 1;

  size_t off = 0;
  auto take = [&](size_t bytes) {
    size_t o = off;
    off = align_up(off + bytes, 256);
    return o;
  };
  // zeroed region: one block per segment, then the look-back flags
  L.o_hall = take((size_t)max_w * kSlotWords * sizeof(uint32_t));
  // one bit per element and worker, in rows of 256 elements (whole tiles of the fused pass)
  L.mask_stride = (max_n + kPassTile - 1) / kPassTile * (kPassTile / 64);
  L.o_mask = take((size_t)max_w * (size_t)L.mask_stride * sizeof(uint64_t));
  L.o_zero = take((size_t)max_segments * kSegWords * sizeof(uint32_t) +
                             (size_t)L.max_tiles * kNumLookback * sizeof(uint64_t));
  L.o_S = take(((size_t)max_w * kMaxChunks + (size_t)max_segments) * kHistBins * sizeof(uint32_t));
  L.o_coff = take(((size_t)kMaxChunks + (size_t)max_segments) * sizeof(uint32_t));
  L.o_part = take((size_t)max_w * kMaxPassBlocks * 3 * sizeof(double));
  L.o_var = take((size_t)max_w * sizeof(double));
  L.o_leader = take(sizeof(int32_t));
  L.o_err = take(sizeof(uint32_t));
  L.o_counter = take(sizeof(uint64_t));
  L.o_list = take((size_t)L.list_entries * sizeof(uint2));
  L.o_vals = take((size_t)max_w * (size_t)max_k * sizeof(float));
  L.o_rows = take((size_t)max_w * (size_t)max_k * sizeof(int32_t));
  L.o_table = take((size_t)max_segments * sizeof(SegDesc));
  L.o_cmap = take(((size_t)kMaxChunks + (size_t)max_segments) * sizeof(uint32_t));
  L.o_tstart = take((size_t)(max_n / kPassTile + 2) * sizeof(int32_t));
  // pieces of the survivor list staged per tile by the fused pass: room for kStageMax entries in
  // every tile of the longest vector (1.5 bytes per element)
  const int64_t max_tiles_pass = (max_n + kPassTile - 1) / kPassTile;
  L.tilebuf_entries = max_tiles_pass * (int64_t)kStageMax;
  L.o_tbuf = take((size_t)L.tilebuf_entries * sizeof(uint2));
  L.o_tcnt = take((size_t)(max_tiles_pass + 1) * sizeof(uint32_t));
  L.o_sample = take((size_t)16384 * kGuessRun * sizeof(uint32_t));
  L.total = off;
  return L;
}

}  // namespace

extern "C" {

int32_t artopk_version(void) { return 200; }  // 0.2.0: options, counted round-robin leader, allocation-free variance

const char* artopk_last_error(const artopk_ctx* ctx) { return ctx ? ctx->err : g_noctx_err; }

int artopk_create(artopk_ctx** out, int32_t max_w, int64_t max_n, int64_t max_k, int32_t max_segments,
                  void* hip_stream) {
  if (!out) return ARTOPK_EINVAL;
  if (!valid_limits(max_w, max_n, max_k, max_segments)) return ARTOPK_EINVAL;
  artopk_ctx* c = new (std::nothrow) artopk_ctx();
  if (!c) return ARTOPK_ENOMEM;
  c->stream = reinterpret_cast<hipStream_t>(hip_stream);
  c->max_w = max_w;
  c->max_n = max_n;
  c->max_k = max_k;
  c->max_seg = max_segments;
  hipError_t e = hipGetDevice(&c->device);
  int cus = 0;
  if (e == hipSuccess) e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, c->device);
  if (e != hipSuccess) {
    delete c;
    return ARTOPK_EHIP;
  }
  c->num_cu = cus > 0 ? cus : 256;

  Scratch& s = c->s;
  const Layout L = scratch_layout(max_w, max_n, max_k, max_segments);
  s.cap = L.cap;
  s.list_entries = L.list_entries;
  s.max_tiles = L.max_tiles;
  s.mask_stride = L.mask_stride;
  s.tilebuf_entries = L.tilebuf_entries;
  const size_t total = L.total;

  e = hipMalloc(&c->slab, total);
  if (e != hipSuccess) {
    delete c;
    return ARTOPK_ENOMEM;
  }
  char* base = static_cast<char*>(c->slab);
  s.h_all = reinterpret_cast<uint32_t*>(base + L.o_hall);
  s.mask = reinterpret_cast<uint64_t*>(base + L.o_mask);
  s.zero_base = reinterpret_cast<uint32_t*>(base + L.o_zero);
  // kSegWords is even, so the flags stay 8-byte aligned
  s.flags = reinterpret_cast<uint64_t*>(s.zero_base + (size_t)max_segments * kSegWords);
  s.S = reinterpret_cast<uint32_t*>(base + L.o_S);
  s.chunk_off = reinterpret_cast<uint32_t*>(base + L.o_coff);
  s.partials = reinterpret_cast<double*>(base + L.o_part);
  s.var_scratch = reinterpret_cast<double*>(base + L.o_var);
  s.leader_dev = reinterpret_cast<int32_t*>(base + L.o_leader);
  s.err_dev = reinterpret_cast<uint32_t*>(base + L.o_err);
  s.counter_dev = reinterpret_cast<uint64_t*>(base + L.o_counter);
  s.list = reinterpret_cast<uint2*>(base + L.o_list);
  s.vals = reinterpret_cast<float*>(base + L.o_vals);
  s.idx_rows = reinterpret_cast<int32_t*>(base + L.o_rows);
  s.table_dev = reinterpret_cast<SegDesc*>(base + L.o_table);
  s.chunk_map = reinterpret_cast<uint32_t*>(base + L.o_cmap);
  s.tile_start = reinterpret_cast<int32_t*>(base + L.o_tstart);
  s.tilebuf = reinterpret_cast<uint2*>(base + L.o_tbuf);
  s.tile_cnt = reinterpret_cast<uint32_t*>(base + L.o_tcnt);
  s.sample_keys = reinterpret_cast<uint32_t*>(base + L.o_sample);

  // leader, error word and step counter start at zero (stream-ordered before any later call)
  hipLaunchKernelGGL(k_fill_zero, dim3(1), dim3(256), 0, c->stream,
                     reinterpret_cast<uint32_t*>(s.leader_dev), (size_t)1, s.err_dev, (size_t)1,
                     reinterpret_cast<uint32_t*>(s.counter_dev), (size_t)2, 0, (int32_t*)nullptr,
                     (int32_t*)nullptr);
  if (hipGetLastError() != hipSuccess) {
    (void)hipFree(c->slab);
    delete c;
    return ARTOPK_EHIP;
  }
  *out = c;
  return ARTOPK_OK;
}

int64_t artopk_scratch_bytes(int32_t max_w, int64_t max_n, int64_t max_k, int32_t max_segments) {
  if (!valid_limits(max_w, max_n, max_k, max_segments)) return -1;
  return (int64_t)scratch_layout(max_w, max_n, max_k, max_segments).total;
}

int artopk_destroy(artopk_ctx* ctx) {
  if (!ctx) return ARTOPK_EINVAL;
  if (ctx->ev_created)
    for (int r = 0; r < artopk_ctx::kRing; ++r)
      for (int i = 0; i < artopk_ctx::kMarks; ++i)
        if (ctx->ev[r][i]) (void)hipEventDestroy(ctx->ev[r][i]);
  if (ctx->slab) (void)hipFree(ctx->slab);
  delete ctx;
  return ARTOPK_OK;
}

int artopk_status(artopk_ctx* ctx) {
  if (!ctx) return ARTOPK_EINVAL;
  HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));
  uint32_t err = 0;
  HIP_TRY(ctx, hipMemcpy(&err, ctx->s.err_dev, sizeof(err), hipMemcpyDeviceToHost));
  if (err) {
    uint32_t zero = 0;
    HIP_TRY(ctx, hipMemcpy(ctx->s.err_dev, &zero, sizeof(zero), hipMemcpyHostToDevice));
    return fail(ctx, ARTOPK_ESTATE, "device error word 0x%x (1 = histogram/count mismatch, 2 = scan wait expired, 4 = kernel sequence, 8 = index out of range)", err);
  }
  return ARTOPK_OK;
}

int artopk_set_profile(artopk_ctx* ctx, int32_t enable) {
  if (!ctx) return ARTOPK_EINVAL;
  if (enable && !ctx->ev_created) {
    for (int r = 0; r < artopk_ctx::kRing; ++r)
      for (int i = 0; i < artopk_ctx::kMarks; ++i) HIP_TRY(ctx, hipEventCreate(&ctx->ev[r][i]));
    ctx->ev_created = true;
  }
  ctx->profile = enable != 0;
  ctx->profile_level = enable;
  ctx->prof_calls = 0;
  for (int r = 0; r < artopk_ctx::kRing; ++r)
    for (int i = 0; i < artopk_ctx::kMarks; ++i) ctx->ev_valid[r][i] = false;
  return ARTOPK_OK;
}

int artopk_set_option(artopk_ctx* ctx, int32_t key, int64_t value) {
  if (!ctx) return ARTOPK_EINVAL;
  switch (key) {
    case ARTOPK_OPT_GUESS_MIN_N:
      if (value < 1 || value > (1ll << 31)) return fail(ctx, ARTOPK_EINVAL, "ARTOPK_OPT_GUESS_MIN_N outside [1, 2^31]");
      ctx->guess_min_n = value;
      return ARTOPK_OK;
    case ARTOPK_OPT_UPDATE_TILES_MIN_N:
      if (value < 1 || value > (1ll << 31))
        return fail(ctx, ARTOPK_EINVAL, "ARTOPK_OPT_UPDATE_TILES_MIN_N outside [1, 2^31]");
      ctx->update_tiles_min_n = value;
      return ARTOPK_OK;
    case ARTOPK_OPT_LEADER_FIRST:
      if (value != 0 && value != 1) return fail(ctx, ARTOPK_EINVAL, "ARTOPK_OPT_LEADER_FIRST takes 0 or 1");
      ctx->leader_first = value != 0;
      return ARTOPK_OK;
    case ARTOPK_OPT_NONTEMPORAL:
      if (value != 0 && value != 1) return fail(ctx, ARTOPK_EINVAL, "ARTOPK_OPT_NONTEMPORAL takes 0 or 1");
      ctx->pass_a_nt = value != 0;
      return ARTOPK_OK;
    case ARTOPK_OPT_STAGE_TILES:
      if (value < 0 || value > 2) return fail(ctx, ARTOPK_EINVAL, "ARTOPK_OPT_STAGE_TILES takes 0, 1 or 2");
      ctx->stage_tiles = (int)value;
      return ARTOPK_OK;
    default:
      return fail(ctx, ARTOPK_EINVAL, "unknown option %d", key);
  }
}

int artopk_get_option(const artopk_ctx* ctx, int32_t key, int64_t* value_out) {
  if (!ctx || !value_out) return ARTOPK_EINVAL;
  switch (key) {
    case ARTOPK_OPT_GUESS_MIN_N: *value_out = ctx->guess_min_n; return ARTOPK_OK;
    case ARTOPK_OPT_UPDATE_TILES_MIN_N: *value_out = ctx->update_tiles_min_n; return ARTOPK_OK;
    case ARTOPK_OPT_LEADER_FIRST: *value_out = ctx->leader_first ? 1 : 0; return ARTOPK_OK;
    case ARTOPK_OPT_NONTEMPORAL: *value_out = ctx->pass_a_nt ? 1 : 0; return ARTOPK_OK;
    case ARTOPK_OPT_STAGE_TILES: *value_out = ctx->stage_tiles; return ARTOPK_OK;
    default: return ARTOPK_EINVAL;
  }
}

// Reads back the selection state of segment 0 as the last step left it.
int artopk_select_info(artopk_ctx* ctx, int32_t* info_out, int32_t count) {
  if (!ctx || !info_out || count < 0) return ARTOPK_EINVAL;
  HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));
  SelState st{};
  HIP_TRY(ctx, hipMemcpy(&st, ctx->s.zero_base + kSegState, sizeof(st), hipMemcpyDeviceToHost));
  const int32_t v[5] = {ctx->last_guessed, ctx->last_guessed ? (int32_t)st.use_mask : 0, (int32_t)st.list_count,
                        (int32_t)st.compact_level, ctx->last_dom_workers};
  for (int i = 0; i < count && i < 5; ++i) info_out[i] = v[i];
  return ARTOPK_OK;
}

// Averages every stage over the calls recorded since profiling was enabled
// (at most the kRing most recent ones).
int artopk_get_profile(artopk_ctx* ctx, float* ms_out, int32_t count) {
  if (!ctx || !ms_out || count < 0) return ARTOPK_EINVAL;
  if (!ctx->ev_created) return fail(ctx, ARTOPK_EINVAL, "profiling was never enabled");
  HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));
  double acc[ARTOPK_PROF_COUNT] = {0, 0, 0, 0, 0};
  int cnt[ARTOPK_PROF_COUNT] = {0, 0, 0, 0, 0};
  for (int r = 0; r < artopk_ctx::kRing; ++r) {
    const bool* v = ctx->ev_valid[r];
    for (int i = 0; i < 4; ++i) {
      if (v[i] && v[i + 1]) {
        float ms = 0.f;
        HIP_TRY(ctx, hipEventElapsedTime(&ms, ctx->ev[r][i], ctx->ev[r][i + 1]));
        acc[i] += ms;
        cnt[i]++;
      }
    }
    int last = -1;
    for (int i = 4; i >= 1; --i)
      if (v[i]) {
        last = i;
        break;
      }
    if (v[0] && last > 0) {
      float ms = 0.f;
      HIP_TRY(ctx, hipEventElapsedTime(&ms, ctx->ev[r][0], ctx->ev[r][last]));
      acc[ARTOPK_PROF_TOTAL] += ms;
      cnt[ARTOPK_PROF_TOTAL]++;
    }
  }
  for (int i = 0; i < count && i < ARTOPK_PROF_COUNT; ++i) ms_out[i] = cnt[i] ? (float)(acc[i] / cnt[i]) : 0.f;
  return ARTOPK_OK;
}

int artopk_variance(artopk_ctx* ctx, const float* const* x, int32_t w, int64_t n, double* var_out,
                    int32_t* argmax_out) {
  int rc = check_common(ctx, w, n, 1);
  if (rc) return rc;
  if ((rc = check_ptr_table(ctx, x, w, "x"))) return rc;
  if (!var_out) return fail(ctx, ARTOPK_EINVAL, "var_out is NULL");
  {
    RangeSet rs;
    rs.add_table(reinterpret_cast<const void* const*>(x), w, (size_t)n * 4, false, "x");
    rs.add(var_out, (size_t)w * 8, true, "var_out");
    rs.add(argmax_out, 4, true, "argmax_out");
    if ((rc = rs.check(ctx))) return rc;
  }
  const PtrTable tab = make_table(x, w);
  const int nblk = stats_blocks(ctx->num_cu, w, n);
  Scratch& s = ctx->s;
  hipLaunchKernelGGL((k_stats<true, true>), dim3(nblk, w), dim3(256), 0, ctx->stream, tab, n, s.partials);
  hipLaunchKernelGGL(k_leader, dim3(1), dim3(1024), 0, ctx->stream, s.partials, (int)w, nblk, n, s.var_scratch,
                     var_out, s.leader_dev, argmax_out);
  HIP_TRY(ctx, hipGetLastError());
  return ARTOPK_OK;
}

namespace {

// Per-device address of the fixed scratch and the device's compute-unit count, looked up the
// first time artopk_variance_static runs with that device current.
struct StaticDevice {
  bool ready = false;
  double* ptr = nullptr;
  int num_cu = 0;
};
constexpr int kMaxDevices = 64;
StaticDevice g_static_dev[kMaxDevices];
std::mutex g_static_mu;

int static_device(const StaticDevice** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return fail(nullptr, ARTOPK_EHIP, "hipGetDevice failed: %s", hipGetErrorString(e));
  if (dev < 0 || dev >= kMaxDevices) return fail(nullptr, ARTOPK_EINVAL, "device %d outside [0, %d)", dev, kMaxDevices);
  std::lock_guard<std::mutex> lock(g_static_mu);
  StaticDevice& sd = g_static_dev[dev];
  if (!sd.ready) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess || p == nullptr)
      return fail(nullptr, ARTOPK_EHIP, "hipGetSymbolAddress(scratch) failed on device %d: %s", dev,
                  hipGetErrorString(e));
    int cus = 0;
    e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
    if (e != hipSuccess) return fail(nullptr, ARTOPK_EHIP, "hipDeviceGetAttribute failed: %s", hipGetErrorString(e));
    sd.ptr = static_cast<double*>(p);
    sd.num_cu = cus > 0 ? cus : 256;
    sd.ready = true;
  }
  *out = &sd;
  return ARTOPK_OK;
}

}  // namespace

int artopk_variance_static(const float* const* x, int32_t w, int64_t n, double* var_out, int32_t* argmax_out,
                           void* hip_stream) {
  if (w < 1 || w > ARTOPK_MAX_WORKERS)
    return fail(nullptr, ARTOPK_EINVAL, "W=%d outside [1, %d] (the fixed scratch holds %d workers)", w,
                ARTOPK_MAX_WORKERS, ARTOPK_MAX_WORKERS);
  if (n < 1 || n >= (1ll << 31)) return fail(nullptr, ARTOPK_EINVAL, "N=%lld outside [1, 2^31)", (long long)n);
  int rc = check_ptr_table(nullptr, x, w, "x");
  if (rc) return rc;
  if (!var_out) return fail(nullptr, ARTOPK_EINVAL, "var_out is NULL");
  {
    RangeSet rs;
    rs.add_table(reinterpret_cast<const void* const*>(x), w, (size_t)n * 4, false, "x");
    rs.add(var_out, (size_t)w * 8, true, "var_out");
    rs.add(argmax_out, 4, true, "argmax_out");
    if ((rc = rs.check(nullptr))) return rc;
  }
  const StaticDevice* sd = nullptr;
  if ((rc = static_device(&sd))) return rc;
  hipStream_t st = reinterpret_cast<hipStream_t>(hip_stream);
  const PtrTable tab = make_table(x, w);
  const int nblk = stats_blocks(sd->num_cu, w, n);  // <= kMaxChunks, so w * nblk * 3 <= kStaticPartials
  double* partials = sd->ptr;
  double* var_scratch = sd->ptr + kStaticPartials;
  int32_t* leader_word = reinterpret_cast<int32_t*>(sd->ptr + kStaticPartials + kMaxW);
  // every word of the scratch that is read is written first by these two launches: nothing to clear
  hipLaunchKernelGGL((k_stats<true, true>), dim3(nblk, w), dim3(256), 0, st, tab, n, partials);
  hipLaunchKernelGGL(k_leader, dim3(1), dim3(1024), 0, st, partials, (int)w, nblk, n, var_scratch, var_out,
                     leader_word, argmax_out);
  const hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(nullptr, ARTOPK_EHIP, "kernel launch failed: %s", hipGetErrorString(e));
  return ARTOPK_OK;
}

int artopk_select_topk(artopk_ctx* ctx, const float* acc, int64_t n, int32_t nseg, const int64_t* seg_off,
                       const int64_t* seg_k, int64_t k, int32_t* idx_out) {
  int rc = check_common(ctx, 1, n, k);
  if (rc) return rc;
  if (!acc || !aligned16(acc)) return fail(ctx, ARTOPK_EINVAL, "acc is NULL or not 16-byte aligned");
  if (!idx_out) return fail(ctx, ARTOPK_EINVAL, "idx_out is NULL");
  if ((rc = check_segments(ctx, n, nseg, seg_off, seg_k, k))) return rc;
  {
    RangeSet rs;
    rs.add(acc, (size_t)n * 4, false, "acc");
    rs.add(idx_out, (size_t)k * 4, true, "idx_out");
    if ((rc = rs.check(ctx))) return rc;
  }
  const float* one[1] = {acc};
  const PtrTable tab = make_table(one, 1);
  prof_begin(ctx);
  prof_mark(ctx, 1);
  Plan flat;
  const Plan* pl = &flat;
  if (seg_off && nseg > 1) {
    if ((rc = segmented_plan(ctx, n, nseg, seg_off, seg_k, &pl))) return rc;
  } else {
    flat = flat_plan(ctx, n, k);
  }
  if ((rc = enqueue_clear(ctx, *pl, 0, 0, nullptr))) return rc;  // the single vector is "leader 0"
  rc = enqueue_select(ctx, *pl, tab, n, idx_out, false, 0);
  prof_mark(ctx, 2);
  return rc;
}

int artopk_gather_sum(artopk_ctx* ctx, const float* const* acc, int32_t w, int64_t n, const int32_t* idx,
                      int64_t k, float* vals_out, float* sum_out) {
  int rc = check_common(ctx, w, n, k);
  if (rc) return rc;
  if ((rc = check_ptr_table(ctx, acc, w, "acc"))) return rc;
  if (!idx || !sum_out) return fail(ctx, ARTOPK_EINVAL, "idx or sum_out is NULL");
  {
    RangeSet rs;
    rs.add_table(reinterpret_cast<const void* const*>(acc), w, (size_t)n * 4, false, "acc");
    rs.add(idx, (size_t)k * 4, false, "idx");
    rs.add(vals_out, (size_t)w * (size_t)k * 4, true, "vals_out");
    rs.add(sum_out, (size_t)k * 4, true, "sum_out");
    if ((rc = rs.check(ctx))) return rc;
  }
  const PtrTable tab = make_table(acc, w);
  return enqueue_gather(ctx, tab, w, n, idx, k, vals_out, sum_out, false);
}

int artopk_scatter_residual(artopk_ctx* ctx, float* const* residual, int32_t w, int64_t n, const int32_t* idx,
                            int64_t k, const float* sum, float* update) {
  int rc = check_common(ctx, w, n, k);
  if (rc) return rc;
  if ((rc = check_ptr_table(ctx, residual, w, "residual"))) return rc;
  if (!idx || !sum || !update) return fail(ctx, ARTOPK_EINVAL, "idx, sum or update is NULL");
  if (!aligned16(update)) return fail(ctx, ARTOPK_EINVAL, "update is not 16-byte aligned");
  {
    RangeSet rs;
    rs.add_table(reinterpret_cast<const void* const*>(residual), w, (size_t)n * 4, true, "residual");
    rs.add(idx, (size_t)k * 4, false, "idx");
    rs.add(sum, (size_t)k * 4, false, "sum");
    rs.add(update, (size_t)n * 4, true, "update");
    if ((rc = rs.check(ctx))) return rc;
  }
  const PtrTable tab = make_table(residual, w);
  const int blocks = (int)((k + 255) / 256);
  hipLaunchKernelGGL(k_zero_at, dim3(blocks), dim3(256), 0, ctx->stream, tab, (int)w, n, idx, k, ctx->s.err_dev);
  HIP_TRY(ctx, hipGetLastError());
  return enqueue_update_fill(ctx, update, n, idx, sum, k);
}

int artopk_topk_workers(artopk_ctx* ctx, const float* const* acc, int32_t w, int64_t n, int64_t k,
                        int32_t* idx_out, float* vals_out, double* sqnorm_out, int32_t* argmax_out) {
  int rc = check_common(ctx, w, n, k);
  if (rc) return rc;
  if ((rc = check_ptr_table(ctx, acc, w, "acc"))) return rc;
  if (!idx_out) return fail(ctx, ARTOPK_EINVAL, "idx_out is NULL");
  {
    RangeSet rs;
    rs.add_table(reinterpret_cast<const void* const*>(acc), w, (size_t)n * 4, false, "acc");
    rs.add(idx_out, (size_t)w * (size_t)k * 4, true, "idx_out");
    rs.add(vals_out, (size_t)w * (size_t)k * 4, true, "vals_out");
    rs.add(sqnorm_out, (size_t)w * 8, true, "sqnorm_out");
    rs.add(argmax_out, 4, true, "argmax_out");
    if ((rc = rs.check(ctx))) return rc;
  }
  const PtrTable tab = make_table(acc, w);
  return enqueue_topk_workers(ctx, tab, w, n, k, idx_out, vals_out ? vals_out : ctx->s.vals, sqnorm_out,
                              argmax_out, false);
}

int artopk_compression_gain(artopk_ctx* ctx, const float* const* residual, int32_t w, int64_t n,
                            const float* vals, int64_t k, double* gain_out) {
  int rc = check_common(ctx, w, n, k);
  if (rc) return rc;
  if ((rc = check_ptr_table(ctx, residual, w, "residual"))) return rc;
  if (!vals || !gain_out) return fail(ctx, ARTOPK_EINVAL, "vals or gain_out is NULL");
  {
    RangeSet rs;
    rs.add_table(reinterpret_cast<const void* const*>(residual), w, (size_t)n * 4, false, "residual");
    rs.add(vals, (size_t)w * (size_t)k * 4, false, "vals");
    rs.add(gain_out, (size_t)w * 8, true, "gain_out");
    if ((rc = rs.check(ctx))) return rc;
  }
  Scratch& s = ctx->s;
  const PtrTable rtab = make_table(residual, w);
  PtrTable vtab;
  for (int i = 0; i < kMaxW; ++i) vtab.p[i] = (i < w) ? const_cast<float*>(vals) + (size_t)i * (size_t)k : nullptr;
  const int nblk_res = stats_blocks(ctx->num_cu, w, n);
  int nblk_vals = (int)((k + 256 * 16 - 1) / (256 * 16));
  if (nblk_vals < 1) nblk_vals = 1;
  if (nblk_vals > kMaxChunks / 2) nblk_vals = kMaxChunks / 2;
  // the two partial arrays share the variance scratch: residual partials first
  double* part_res = s.partials;
  double* part_vals = s.partials + (size_t)ctx->max_w * (kMaxChunks / 2) * 2;
  const int nblk_res_c = nblk_res > kMaxChunks / 2 ? kMaxChunks / 2 : nblk_res;
  hipLaunchKernelGGL((k_stats<false, true>), dim3(nblk_res_c, w), dim3(256), 0, ctx->stream, rtab, n, part_res);
  hipLaunchKernelGGL((k_stats<false, false>), dim3(nblk_vals, w), dim3(256), 0, ctx->stream, vtab, k, part_vals);
  hipLaunchKernelGGL(k_gain, dim3(1), dim3(1024), 0, ctx->stream, part_vals, nblk_vals, part_res, nblk_res_c, (int)w,
                     gain_out);
  HIP_TRY(ctx, hipGetLastError());
  return ARTOPK_OK;
}

int artopk_apply_update(artopk_ctx* ctx, float* weights, int64_t n, const int32_t* idx, const float* sum,
                        int64_t k, float eta) {
  int rc = check_common(ctx, 1, n, k);
  if (rc) return rc;
  if (!weights || !idx || !sum) return fail(ctx, ARTOPK_EINVAL, "weights, idx or sum is NULL");
  {
    RangeSet rs;
    rs.add(weights, (size_t)n * 4, true, "weights");
    rs.add(idx, (size_t)k * 4, false, "idx");
    rs.add(sum, (size_t)k * 4, false, "sum");
    if ((rc = rs.check(ctx))) return rc;
  }
  const int blocks = (int)((k + 255) / 256);
  hipLaunchKernelGGL(k_apply_update, dim3(blocks), dim3(256), 0, ctx->stream, weights, n, idx, sum, k, eta,
                     ctx->s.err_dev);
  HIP_TRY(ctx, hipGetLastError());
  return ARTOPK_OK;
}

namespace {

// One step; the g rows hold elements of type g_type (float32 rows are passed as they are, 16-bit
// rows behind the same pointer type).
int step_impl(artopk_ctx* ctx, const float* const* g, int32_t g_type, float* const* residual, int32_t w, int64_t n,
              int32_t nseg, const int64_t* seg_off, const int64_t* seg_k, int64_t k, int32_t mode,
              uint64_t step, int32_t fixed_leader, int32_t* leader_out, double* var_out, int32_t* idx_out,
              float* vals_out, float* sum_out, float* update_out) {
  int rc = check_common(ctx, w, n, k);
  if (rc) return rc;
  if (g_type != ARTOPK_G_F32 && g_type != ARTOPK_G_BF16 && g_type != ARTOPK_G_F16)
    return fail(ctx, ARTOPK_EINVAL, "unknown gradient element type %d", g_type);
  ctx->g_type = g_type;
  if ((rc = check_ptr_table(ctx, g, w, "g", g_type == ARTOPK_G_F32 ? 16 : 8))) return rc;
  if ((rc = check_ptr_table(ctx, residual, w, "residual"))) return rc;
  if (!idx_out || !sum_out) return fail(ctx, ARTOPK_EINVAL, "idx_out or sum_out is NULL");
  if (update_out && !aligned16(update_out)) return fail(ctx, ARTOPK_EINVAL, "update_out is not 16-byte aligned");
  if ((rc = check_segments(ctx, n, nseg, seg_off, seg_k, k))) return rc;
  {
    RangeSet rs;
    rs.add_table(reinterpret_cast<const void* const*>(g), w, (size_t)n * (g_type == ARTOPK_G_F32 ? 4 : 2), false, "g");
    rs.add_table(reinterpret_cast<const void* const*>(residual), w, (size_t)n * 4, true, "residual");
    rs.add(leader_out, 4, true, "leader_out");
    rs.add(var_out, (size_t)w * 8, true, "var_out");
    rs.add(idx_out, (size_t)k * 4, true, "idx_out");
    rs.add(vals_out, (size_t)w * (size_t)k * 4, true, "vals_out");
    rs.add(sum_out, (size_t)k * 4, true, "sum_out");
    rs.add(update_out, (size_t)n * 4, true, "update_out");
    if ((rc = rs.check(ctx))) return rc;
  }
  int leader_host = -1;
  if (mode == ARTOPK_STAR) {
    leader_host = (int)(step % (uint64_t)w);
  } else if (mode == ARTOPK_FIXED) {
    if (fixed_leader < 0 || fixed_leader >= w) return fail(ctx, ARTOPK_EINVAL, "fixed_leader outside [0, W)");
    leader_host = fixed_leader;
  } else if (mode == ARTOPK_VAR_TOPK) {
    if (seg_off != nullptr && nseg > 1)
      return fail(ctx, ARTOPK_EINVAL, "ARTOPK_VAR_TOPK is defined for the unsegmented selection only");
  } else if (mode != ARTOPK_VAR && mode != ARTOPK_VAR_G && mode != ARTOPK_STAR_COUNTER) {
    return fail(ctx, ARTOPK_EINVAL, "unknown mode %d", mode);
  }
  // the leader is found on the device, from statistics of the pass or from the counter
  const bool device_leader = mode == ARTOPK_VAR || mode == ARTOPK_VAR_G || mode == ARTOPK_STAR_COUNTER;

  Scratch& s = ctx->s;
  hipStream_t st = ctx->stream;
  const PtrTable gt = make_table(g, w);
  const PtrTable rt = make_table(residual, w);
  const bool segmented = seg_off != nullptr && nseg > 1;
  // a flat selection on a long vector samples a threshold guess first; its chunks are then whole
  // tiles of the fused pass, which strides over the tiles and counts per chunk
  const bool leader_first = (mode == ARTOPK_STAR || mode == ARTOPK_FIXED) && ctx->leader_first;
  const GuessPlan gp = segmented ? GuessPlan{} : plan_guess(ctx, n, k, leader_first ? 1 : (int)w);
  Plan flat;
  const Plan* pl = &flat;
  if (segmented) {
    if ((rc = segmented_plan(ctx, n, nseg, seg_off, seg_k, &pl))) return rc;
  } else {
    flat = flat_plan(ctx, n, k, -1, gp.on);
  }
  // pass A always works on whole-vector chunks; for a flat select they are the select's chunks too
  const ChunkGeom geom = make_geom(0, n, kMaxChunks, gp.on);
  const dim3 grid(geom.nchunks, w);

  // a long segmented vector: the fused pass strides over the tiles as on the guess route (the
  // selection builds the segments' histograms from the leader's vector afterwards either way)
  const bool seg_stride = segmented && n >= ctx->guess_min_n;

  ctx->last_guessed = 0;
  ctx->last_dom_workers = w;
  if (mode == ARTOPK_VAR_TOPK) {
    // Literal Alg. 1: Top-k on every worker, leader = largest squared norm of its own k values,
    // then the leader's indices are the shared ones.
    prof_begin(ctx);
    prof_mark(ctx, 0);
    if ((rc = enqueue_clear(ctx, *pl, (int)w))) return rc;
    // every worker selects on its own vector: on long vectors every worker gets a guessed bound and
    // leaves a mask, as under the variance rule
    ctx->last_guessed = gp.on ? 1 : 0;
    ctx->lvl1_a = 0;
    ctx->lvl1_b = 1;
    if (gp.on) enqueue_guess(ctx, gp, gt, rt, (int)w);
    prof_dom(ctx, false);
    if (gp.on) {
      launch_pass_mark(ctx, 0, (int)w, gt, rt, n, geom.chunk_elems);
    } else {
      launch_pass_a(ctx, 0, 2, grid, gt, rt, n, geom, -1);
    }
    prof_dom(ctx, true);
    prof_mark(ctx, 1);
    if ((rc = enqueue_topk_workers(ctx, rt, w, n, k, s.idx_rows, s.vals, var_out, leader_out, true, gp.on))) return rc;
    hipLaunchKernelGGL(k_copy_i32, dim3((int)((k + 255) / 256)), dim3(256), 0, st, s.idx_rows, s.leader_dev, k,
                       idx_out);
    prof_mark(ctx, 2);
    if ((rc = enqueue_gather(ctx, rt, w, n, idx_out, k, vals_out, sum_out, true))) return rc;
    prof_mark(ctx, 3);
    if (update_out && (rc = enqueue_update_fill(ctx, update_out, n, idx_out, sum_out, k))) return rc;
    prof_mark(ctx, 4);
    return ARTOPK_OK;
  }

  if (leader_first) {
    // The leader is known up front: run its pass and the selection first, then
    // stream over the other workers once, gathering and zeroing on the way.
    const int L = leader_host;
    ctx->lvl1_a = 2;
    ctx->lvl1_b = 3;
    float* vals = vals_out ? vals_out : s.vals;
    const float* g1[1] = {g[L]};
    const float* r1[1] = {residual[L]};
    const PtrTable g1t = make_table(g1, 1), r1t = make_table(r1, 1);
    prof_begin(ctx);
    prof_mark(ctx, 0);
    if ((rc = enqueue_clear(ctx, *pl, segmented ? 0 : 1, L, leader_out))) return rc;
    ctx->last_guessed = gp.on ? 1 : 0;
    ctx->last_dom_workers = w > 1 ? w - 1 : 1;
    if (gp.on) {
      enqueue_guess(ctx, gp, g1t, r1t, 1);
      launch_pass_mark(ctx, 0, 1, g1t, r1t, n, geom.chunk_elems, gp.tile_cap);
    } else if (seg_stride) {
      launch_pass_plain(ctx, 0, 1, g1t, r1t, n);
    } else {  // (segments build their histograms on the leader's vector afterwards)
      launch_pass_a(ctx, 0, segmented ? 0 : 1, dim3(geom.nchunks, 1), g1t, r1t, n, geom, segmented ? -1 : 0);
    }
    prof_mark(ctx, 1);
    // The leader's residual is zeroed inside the selection: its kernels have the kept values in
    // registers (level-1 compaction) or write the kept indices anyway (final list pass).
    if ((rc = enqueue_select(ctx, *pl, rt, n, idx_out, !segmented, 0, vals + (size_t)L * (size_t)k, nullptr, gp.on,
                             residual[L], gp.tile_cap)))
      return rc;
    prof_mark(ctx, 2);
    const int rest = (int)w - 1;
    enqueue_tile_starts(ctx, idx_out, n, k);
    prof_dom(ctx, false);
    if (rest > 0) {
      launch_pass_rest(ctx, gt, rt, (int)w, L, n, idx_out, k, vals);
    }
    prof_dom(ctx, true);
    prof_mark(ctx, 3);
    if (update_out && k * 128 <= n) {
      // few kept entries: the ordered sums and the dense update in one pass over the tiles, whose bounds
      // in idx are there already (138 M elements, one in a thousand kept: 96 us against 104 + 4; one in a
      // hundred: 133 against 116 + 5, the owner threads' loads of the rows' entries take over)
      hipLaunchKernelGGL((k_sum_update<kPassRestThreads, kPassRestU>), dim3(pass_blocks(n)), dim3(kPassRestThreads),
                         0, st, vals, (int)w, n, idx_out, k, s.tile_start, sum_out, update_out, s.err_dev);
      HIP_TRY(ctx, hipGetLastError());
    } else {
      hipLaunchKernelGGL(k_sum_rows, dim3((int)((k + 1023) / 1024)), dim3(256), 0, st, vals, (int)w, k, sum_out);
      HIP_TRY(ctx, hipGetLastError());
      if (update_out && (rc = enqueue_update_fill(ctx, update_out, n, idx_out, sum_out, k, true))) return rc;
    }
    prof_mark(ctx, 4);
    return ARTOPK_OK;
  }

  ctx->lvl1_a = 0;
  ctx->lvl1_b = 1;
  prof_begin(ctx);
  prof_mark(ctx, 0);
  // the flat select reuses the histograms pass A builds; segments build their own afterwards
  if ((rc = enqueue_clear(ctx, *pl, segmented ? 0 : (device_leader ? (int)w : 1)))) return rc;
  int slot_by_leader = 0;
  LeaderArgs leader_args{};
  const bool marking = gp.on && device_leader;
  if (mode == ARTOPK_STAR_COUNTER) {
    // every worker's pass prepares the selection, as under the variance rules, and the selection
    // kernels read the leader word that the counter kernel leaves
    hipLaunchKernelGGL(k_counter_leader, dim3(1), dim3(64), 0, st, s.counter_dev, (int32_t)w, s.leader_dev, leader_out);
    HIP_TRY(ctx, hipGetLastError());
    ctx->last_guessed = marking ? 1 : 0;
    if (marking) enqueue_guess(ctx, gp, gt, rt, (int)w);
    prof_dom(ctx, false);
    if (seg_stride) {
      launch_pass_plain(ctx, 0, (int)w, gt, rt, n);
    } else if (segmented) {
      launch_pass_a(ctx, 0, 0, grid, gt, rt, n, geom, -1);
    } else if (marking) {
      launch_pass_mark(ctx, 0, (int)w, gt, rt, n, geom.chunk_elems);
      slot_by_leader = 1;
    } else {
      launch_pass_a(ctx, 0, 2, grid, gt, rt, n, geom, -1);
      slot_by_leader = 1;
    }
    prof_dom(ctx, true);
    prof_mark(ctx, 1);
  } else if (mode == ARTOPK_VAR || mode == ARTOPK_VAR_G) {
    const int stats = mode == ARTOPK_VAR_G ? 2 : 1;  // variance of the raw gradient, or of g + residual
    if (segmented) {
      prof_dom(ctx, false);
      if (seg_stride)
        launch_pass_plain(ctx, stats, (int)w, gt, rt, n);
      else
        launch_pass_a(ctx, stats, 0, grid, gt, rt, n, geom, -1);
    } else {
      ctx->last_guessed = gp.on ? 1 : 0;
      if (gp.on) enqueue_guess(ctx, gp, gt, rt, (int)w);
      prof_dom(ctx, false);
      if (gp.on) {
        launch_pass_mark(ctx, stats, (int)w, gt, rt, n, geom.chunk_elems);
      } else {
        launch_pass_a(ctx, stats, 2, grid, gt, rt, n, geom, -1);
      }
      slot_by_leader = 1;
    }
    prof_dom(ctx, true);
    prof_mark(ctx, 1);
    if (segmented) {  // the segment histograms are built on the leader's vector, so it is needed now
      hipLaunchKernelGGL(k_leader, dim3(1), dim3(1024), 0, st, s.partials, (int)w,
                         seg_stride ? pass_blocks(n) : (int)geom.nchunks, n, s.var_scratch, var_out, s.leader_dev,
                         leader_out);
    } else {          // otherwise the selection's first kernel takes the leader itself
      leader_args.partials = s.partials;
      leader_args.w_count = (int)w;
      leader_args.nblk = marking ? pass_blocks(n) : (int)geom.nchunks;
      leader_args.n = n;
      leader_args.var_scratch = s.var_scratch;
      leader_args.var_out = var_out;
      leader_args.leader_dev = s.leader_dev;
      leader_args.leader_out = leader_out;
    }
  } else {
    prof_dom(ctx, false);
    if (seg_stride)
      launch_pass_plain(ctx, 0, (int)w, gt, rt, n);
    else
      launch_pass_a(ctx, 0, segmented ? 0 : 1, grid, gt, rt, n, geom, leader_host);
    prof_dom(ctx, true);
    prof_mark(ctx, 1);
    hipLaunchKernelGGL(k_set_leader, dim3(1), dim3(64), 0, st, (int32_t)leader_host, s.leader_dev, leader_out);
  }
  HIP_TRY(ctx, hipGetLastError());

  rc = enqueue_select(ctx, *pl, rt, n, idx_out, !segmented, slot_by_leader, nullptr,
                      leader_args.partials ? &leader_args : nullptr, marking);
  if (rc) return rc;
  prof_mark(ctx, 2);
  if ((rc = enqueue_gather(ctx, rt, w, n, idx_out, k, vals_out, sum_out, true))) return rc;
  prof_mark(ctx, 3);
  if (update_out && (rc = enqueue_update_fill(ctx, update_out, n, idx_out, sum_out, k))) return rc;
  prof_mark(ctx, 4);
  return ARTOPK_OK;
}

}  // namespace

int artopk_set_step_counter(artopk_ctx* ctx, uint64_t value) {
  if (!ctx) return fail(nullptr, ARTOPK_EINVAL, "artopk_set_step_counter: ctx is NULL");
  hipLaunchKernelGGL(k_set_counter, dim3(1), dim3(64), 0, ctx->stream, ctx->s.counter_dev, value);
  HIP_TRY(ctx, hipGetLastError());
  return ARTOPK_OK;
}

int artopk_step(artopk_ctx* ctx, const float* const* g, float* const* residual, int32_t w, int64_t n,
                int32_t nseg, const int64_t* seg_off, const int64_t* seg_k, int64_t k, int32_t mode,
                uint64_t step, int32_t fixed_leader, int32_t* leader_out, double* var_out, int32_t* idx_out,
                float* vals_out, float* sum_out, float* update_out) {
  return step_impl(ctx, g, ARTOPK_G_F32, residual, w, n, nseg, seg_off, seg_k, k, mode, step, fixed_leader,
                   leader_out, var_out, idx_out, vals_out, sum_out, update_out);
}

int artopk_step_g16(artopk_ctx* ctx, const void* const* g, int32_t g_type, float* const* residual, int32_t w,
                    int64_t n, int32_t nseg, const int64_t* seg_off, const int64_t* seg_k, int64_t k,
                    int32_t mode, uint64_t step, int32_t fixed_leader, int32_t* leader_out, double* var_out,
                    int32_t* idx_out, float* vals_out, float* sum_out, float* update_out) {
  if (ctx && g_type != ARTOPK_G_BF16 && g_type != ARTOPK_G_F16)
    return fail(ctx, ARTOPK_EINVAL, "artopk_step_g16 takes ARTOPK_G_BF16 or ARTOPK_G_F16 gradients");
  return step_impl(ctx, reinterpret_cast<const float* const*>(g), g_type, residual, w, n, nseg, seg_off, seg_k, k,
                   mode, step, fixed_leader, leader_out, var_out, idx_out, vals_out, sum_out, update_out);
}

}  // extern "C"
