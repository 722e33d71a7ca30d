// Host side of libbsgd: argument checks, workspace carving and kernel
// launches for the entry points declared in bsgd.h.  Every entry point only
// enqueues work on the caller's stream.
#include "bsgd_kernels.hpp"

#include "../../include/bsgd.h"
#include "../../include/bsgd_debug.h"

#include <algorithm>
#include <atomic>
#include <cmath>
#include <mutex>
#include <utility>
#include <vector>

using namespace bsgd;

namespace {

// ---------------------------------------------------------------------------
// workspace layout (all offsets multiples of 256 bytes)
//   [0,256)            WsHeader
//   [256,1280)         sel_idx int32[256]
//   then               Segment table[2T+1], starts uint32[2T+2]  (tensors and the gaps between them)
//   clipped steps:     partials double[max_chunks], gbar float[span rounded up]
// ---------------------------------------------------------------------------
constexpr size_t kAlign = 256;
inline size_t round_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

struct WsLayout {
  size_t sel_off, table_off, starts_off, rowscale_off, rowpart_off, partials_off, gbar_off, total;
  long long max_chunks;
};

bool clip_on(const bsgd_hyper* h) { return h && h->clip_norm > 0.0f && std::isfinite(h->clip_norm); }
bool worker_clip_on(const bsgd_hyper* h) {
  return h && h->worker_clip_norm > 0.0f && std::isfinite(h->worker_clip_norm);
}

// ---------------------------------------------------------------------------
// kernel variants (launch shapes)
// ---------------------------------------------------------------------------
using StepKernel = const void*;                      // k_step / k_row_sumsq instantiations: (StepParams, TableArg<multi>)

struct Variant {
  int BS, V, U, NT;
  StepKernel rows[3][2][2];  // [mode][multi][ema]   gradient from the kept rows, fused update
  StepKernel reduce[2];      // [multi]              clipped step, pass 1: mean + sum of squares
  StepKernel rowsq[2];       // [multi]              per-worker clipping: per-row sums of squares
  StepKernel apply[3][2][2]; // [mode][multi][ema]   clipped step, pass 2: gradient from the stored mean
  // the same first passes doing the selection themselves (the first launch of a step; null for the plain-load shape)
  StepKernel rows_sel[3][2][2];
  StepKernel reduce_sel[2];
};

template <int BS, int V, int U, int NT>
Variant make_variant() {
  using R = Shape<BS, V, U, NT != 0>;                // row loop shape
  using A = Shape<BS, V, 1, NT != 0>;                // pass 2 of a clipped step reads one stored row
  Variant v{};
  v.BS = BS; v.V = V; v.U = U; v.NT = NT;
#define BSGD_FILL(dst, MODE, SH, ROWS)                                                      \
  dst[0][0] = reinterpret_cast<StepKernel>(&k_step<MODE, SH, false, ROWS, false>);          \
  dst[0][1] = reinterpret_cast<StepKernel>(&k_step<MODE, SH, false, ROWS, true>);           \
  dst[1][0] = reinterpret_cast<StepKernel>(&k_step<MODE, SH, true, ROWS, false>);           \
  dst[1][1] = reinterpret_cast<StepKernel>(&k_step<MODE, SH, true, ROWS, true>);
  BSGD_FILL(v.rows[kSgd], kSgd, R, true)
  BSGD_FILL(v.rows[kMomentum], kMomentum, R, true)
  BSGD_FILL(v.rows[kRmspropMom], kRmspropMom, R, true)
  BSGD_FILL(v.apply[kSgd], kSgd, A, false)
  BSGD_FILL(v.apply[kMomentum], kMomentum, A, false)
  BSGD_FILL(v.apply[kRmspropMom], kRmspropMom, A, false)
#undef BSGD_FILL
  v.reduce[0] = reinterpret_cast<StepKernel>(&k_step<kClipReduce, R, false, true, false>);
  v.reduce[1] = reinterpret_cast<StepKernel>(&k_step<kClipReduce, R, true, true, false>);
  v.rowsq[0] = reinterpret_cast<StepKernel>(&k_row_sumsq<R, false>);
  v.rowsq[1] = reinterpret_cast<StepKernel>(&k_row_sumsq<R, true>);
  if constexpr (NT != 0) {
#define BSGD_FILL_SEL(dst, MODE)                                                               \
  dst[0][0] = reinterpret_cast<StepKernel>(&k_step<MODE, R, false, true, false, true>);        \
  dst[0][1] = reinterpret_cast<StepKernel>(&k_step<MODE, R, false, true, true, true>);         \
  dst[1][0] = reinterpret_cast<StepKernel>(&k_step<MODE, R, true, true, false, true>);         \
  dst[1][1] = reinterpret_cast<StepKernel>(&k_step<MODE, R, true, true, true, true>);
    BSGD_FILL_SEL(v.rows_sel[kSgd], kSgd)
    BSGD_FILL_SEL(v.rows_sel[kMomentum], kMomentum)
    BSGD_FILL_SEL(v.rows_sel[kRmspropMom], kRmspropMom)
#undef BSGD_FILL_SEL
    v.reduce_sel[0] = reinterpret_cast<StepKernel>(&k_step<kClipReduce, R, false, true, false, true>);
    v.reduce_sel[1] = reinterpret_cast<StepKernel>(&k_step<kClipReduce, R, true, true, false, true>);
  }
  return v;
}

// Ordered widest chunk first (the automatic choice walks it in order).
const Variant kVariants[] = {make_variant<256, 8, 2, 1>(), make_variant<256, 4, 2, 1>(), make_variant<256, 1, 8, 1>(),
                             make_variant<256, 8, 2, 0>()};
constexpr int kNumVariants = sizeof(kVariants) / sizeof(kVariants[0]);

// Smallest chunk (in elements) over the compiled shapes: bounds the number of
// workgroups, hence the size of the per-block partial-sum array.
long long min_chunk_elems() {
  long long m = 1LL << 40;
  for (const Variant& v : kVariants) {
    const long long e = 4LL * v.BS * v.V;
    if (e < m) m = e;
  }
  return m;
}

WsLayout layout(long long span, int T, bool clip, bool worker_clip) {
  WsLayout L{};
  const size_t max_segments = 2 * (size_t)T + 1;      // every tensor may be followed by a gap
  L.sel_off = kAlign;
  L.table_off = L.sel_off + round_up(sizeof(int) * kMaxWorkers, kAlign);
  L.starts_off = L.table_off + round_up(sizeof(Segment) * max_segments, kAlign);
  L.rowscale_off = L.starts_off + round_up(sizeof(unsigned) * (max_segments + 1), kAlign);
  L.rowpart_off = L.rowscale_off + round_up(sizeof(float) * kMaxWorkers, kAlign);
  L.max_chunks = span / min_chunk_elems() + 2;
  L.partials_off = L.rowpart_off;
  if (worker_clip) L.partials_off += round_up(sizeof(double) * (size_t)L.max_chunks * kMaxWorkers, kAlign);
  L.gbar_off = L.partials_off;
  L.total = L.partials_off;
  if (clip) {
    L.gbar_off = L.partials_off + round_up(sizeof(double) * (size_t)L.max_chunks, kAlign);
    L.total = L.gbar_off + round_up(sizeof(float) * ((size_t)span + 4), kAlign);
  }
  return L;
}

constexpr int kApplyRoundsPerLaunch = 8;
std::atomic<int> g_variant{-1};                      // -1: choose by problem size
thread_local int t_last_launches = 0;                // reduce/update launches of this thread's last call
thread_local int t_last_fused = 0;                   // 1: that call's selection ran inside its reduce/update launch
std::atomic<int> g_fuse_select{1};                   // 0: never fuse (testing aid)

// Automatic choice: the table is ordered widest chunk first; take the first
// shape that still yields enough workgroups to fill every CU several times.
int compute_units() {
  static const int cus = [] {
    int dev = 0, n = 0;
    if (hipGetDevice(&dev) != hipSuccess) return 256;
    if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) return 256;
    return n;
  }();
  return cus;
}

// Workgroups of `fn` a CU can hold at once (cached per kernel).
int workgroups_per_cu(StepKernel fn, int block) {
  struct Entry { StepKernel fn; int n; };
  static std::mutex mu;
  static std::vector<Entry> cache;
  std::lock_guard<std::mutex> lock(mu);
  for (const Entry& e : cache)
    if (e.fn == fn) return e.n;
  int per_cu = 0;
  if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, fn, block, 0) != hipSuccess || per_cu < 1) per_cu = 1;
  cache.push_back(Entry{fn, per_cu});
  return per_cu;
}

// `kernel_of` names the kernel of a shape that does the call's main pass.
template <class KernelOf>
const Variant& pick_variant(long long total_groups, KernelOf&& kernel_of) {
  const int forced = g_variant.load(std::memory_order_relaxed);
  if (forced >= 0) return kVariants[forced];
  const long long cus = compute_units();
  // Candidates: shapes whose chunks give nearly every CU two workgroups.
  // Among them the widest chunk streams best when its launches are full, but
  // a step is cut into launches of one round each, and a problem that is,
  // say, 3.1 rounds wide runs 4 launches at 78 % filling.  Measured (P = 2 M
  // .. 26 M, N = 50): bandwidth falls by 0.47 % per percent of unfilled
  // launch, and a chunk half as wide costs 2.5 % when both are full; so the
  // score is base - 0.47 * (1 - filling), and half-width chunks win where
  // they fill the launches 5 points better (e.g. P = 9 M: +5.6 %, 14 M: +3 %,
  // 2 M: +18 % over the narrow shape).  A problem that is resident all at
  // once (one launch) is filled as evenly as its workgroups spread over the CUs.
  const Variant* best = nullptr;
  double best_score = -1.0;
  int considered = 0;
  for (const Variant& v : kVariants) {
    if (!v.NT) continue;                               // plain-load shapes are for comparison only
    const long long chunks = (total_groups + (long long)v.BS * v.V - 1) / ((long long)v.BS * v.V);
    if (v.V < 4) {                                     // narrow shapes are for small problems only
      if (best == nullptr && chunks >= 4 * cus) best = &v;
      if (best != nullptr) break;
      continue;
    }
    const long long per_round = (512 / v.BS > 0 ? 512 / v.BS : 1) * cus;   // one round: 8 wavefronts per CU
    const double base = 1.0 - 0.025 * considered;      // each halving of the chunk width
    ++considered;
    if (4 * chunks < 7 * cus) continue;
    const long long resident = (long long)workgroups_per_cu(kernel_of(v), v.BS) * cus;   // what one launch can hold at once
    double filling;
    if (chunks <= resident) {
      filling = (double)chunks / (double)(cus * ((chunks + cus - 1) / cus));
    } else {
      const long long launches = (chunks + per_round - 1) / per_round;
      filling = (double)chunks / (double)(launches * per_round);
    }
    const double score = base - 0.47 * (1.0 - filling);
    if (score > best_score) { best_score = score; best = &v; }
  }
  if (best != nullptr) return *best;
  int narrowest = 0;
  for (int i = 1; i < kNumVariants; ++i)
    if ((long long)kVariants[i].BS * kVariants[i].V < (long long)kVariants[narrowest].BS * kVariants[narrowest].V) narrowest = i;
  return kVariants[narrowest];
}

// How many workgroups of `fn` one launch should hold: as many as are resident
// on the chip at once (capped at 8 wavefronts per CU, which is enough to
// saturate HBM).  A launch of exactly one such "round" starts every workgroup
// at the first kept row at the same moment, so the whole chip walks the rows
// together and DRAM sees a few long sequential streams; a longer launch lets
// workgroups drift apart and costs up to 15 % of bandwidth on long rows.
long long round_size(StepKernel fn, int block, size_t lds) {
  struct Entry { StepKernel fn; size_t lds; long long n; };
  static std::mutex mu;
  static std::vector<Entry> cache;
  std::lock_guard<std::mutex> lock(mu);
  for (const Entry& e : cache)
    if (e.fn == fn && e.lds == lds) return e.n;
  int per_cu = 0;
  if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, fn, block, lds) != hipSuccess || per_cu < 1)
    per_cu = 1;
  const int cap = (8 * 64) / block > 0 ? (8 * 64) / block : 1;
  if (per_cu > cap) per_cu = cap;
  const long long n = (long long)per_cu * compute_units();
  cache.push_back(Entry{fn, lds, n});
  return n;
}

// What a call will run on: the tensors as sorted, non-overlapping segments of
// the gradient row (gaps made explicit), built and checked on the host.
struct Plan {
  long long span = 0;                 // largest grad_offset + numel
  long long col_lo = 0, col_hi = 0;   // columns covered: [col_lo, col_hi)
  int S = 0;                          // segments (S == 1: `single` is used, the vectors stay empty)
  Segment single{};
  bool ema = false;                   // every tensor carries a moving average
  std::vector<Segment> segs;
  std::vector<unsigned> starts;       // S + 1 entries
};


// A run of consecutive chunks of which each (but for a few) holds columns of
// some tensor.  A call whose tensors leave wide gaps in the row (a
// partial-range update: only some layers' gradients are in) is enqueued run
// by run, so the gaps cost neither workgroups nor row reads.
struct Run { long long first, count; };

// Gaps narrower than this many chunks stay inside a run (their chunks are
// launched and stand down on the device before reading any row): a launch
// boundary costs more than a few idle workgroups.
constexpr long long kMergeGapChunks = 64;

std::vector<Run> chunk_runs(const Plan& plan, long long base, long long chunk_cols, long long total_chunks) {
  std::vector<Run> runs;
  if (plan.S <= 1) {
    runs.push_back(Run{0, total_chunks});
    return runs;
  }
  for (int j = 0; j < plan.S; ++j) {
    if (plan.segs[j].theta == nullptr) continue;       // a gap
    const long long c_first = ((long long)plan.starts[j] - base) / chunk_cols;
    const long long c_last = ((long long)plan.starts[j + 1] - 1 - base) / chunk_cols;
    if (!runs.empty() && c_first <= runs.back().first + runs.back().count + kMergeGapChunks) {
      const long long end = runs.back().first + runs.back().count;
      if (c_last + 1 > end) runs.back().count = c_last + 1 - runs.back().first;
    } else {
      runs.push_back(Run{c_first, c_last - c_first + 1});
    }
  }
  return runs;
}

// The segment table of a multi-tensor call during one enqueue_update: where
// the workspace copy lives and whether this call has written it yet.
struct TableCtx {
  const Plan* plan;
  Segment* d_table;
  unsigned* d_starts;
  bool uploaded;
};

// kernel arguments are limited to 4 KiB: StepParams and the embedded table must fit together
static_assert((sizeof(StepParams) + alignof(EmbeddedTable) - 1) / alignof(EmbeddedTable) * alignof(EmbeddedTable) +
                      sizeof(EmbeddedTable) <= 4096,
              "StepParams + EmbeddedTable exceed the kernel-argument buffer");
std::atomic<int> g_table_mode{0};                    // 0: by size; 1: always through the workspace

// Writes the whole table into the workspace (kernel launches that carry the
// descriptors as arguments; no host-to-device copy).
int upload_table(TableCtx& tc, hipStream_t stream) {
  const Plan& plan = *tc.plan;
  for (int first = 0; first < plan.S; first += kUploadBatch) {
    UploadArgs a{};
    a.first = first;
    a.count = (plan.S - first < kUploadBatch) ? (plan.S - first) : kUploadBatch;
    for (int i = 0; i < a.count; ++i) {
      a.seg[i] = plan.segs[first + i];
      a.start[i] = plan.starts[first + i];
    }
    a.is_last = (first + a.count == plan.S);
    a.end_col = plan.starts[plan.S];
    hipLaunchKernelGGL(k_upload_table, dim3(1), dim3(kUploadBatch), 0, stream, a, tc.d_table, tc.d_starts, plan.S);
    if (hipGetLastError() != hipSuccess) return BSGD_ERR_HIP;
  }
  tc.uploaded = true;
  return BSGD_OK;
}

// Segments [j0, j1] that the columns [lo, hi) fall into (lo < hi, both inside the covered range).
void segment_window(const Plan& plan, long long lo, long long hi, int* j0, int* j1) {
  const std::vector<unsigned>& st = plan.starts;      // S + 1 ascending entries
  *j0 = (int)(std::upper_bound(st.begin(), st.begin() + plan.S, (unsigned)lo) - st.begin()) - 1;
  *j1 = (int)(std::upper_bound(st.begin(), st.begin() + plan.S, (unsigned)(hi - 1)) - st.begin()) - 1;
}

// A pass goes out as ONE launch when it is small (under 2.5 rounds of chunks, or everything resident at once:
// launch boundaries then cost more than they bring), or when a round of it moves so little that a boundary costs
// more than letting workgroups drift (few kept rows, narrow chunks).  Measured with RMSProp-mom: wide chunks at
// P = 25 M, N = 8 (235 MB per round): one launch +1 %, N = 16 (369 MB): rounds +1..7 %; narrow chunks at
// P = 1.3-1.8 M (47-117 MB per round): one launch +4..8 % (N = 50), +25 % (N = 16).  Cutting a pass of 1.1-2
// rounds into two or three launches was measured too: -1.3..+0.5 % (P = 4.5-8 M, N = 50), so it stays whole.
constexpr double kLightRoundBytes = 250e6;

bool one_launch(StepKernel fn, int block, size_t lds, long long chunks, double bytes_per_chunk) {
  const long long round = round_size(fn, block, lds);
  const long long resident = (long long)workgroups_per_cu(fn, block) * compute_units();
  return chunks <= resident || 2 * chunks < 5 * round || bytes_per_chunk * (double)round < kLightRoundBytes;
}

// Enqueue the work on `chunks` chunks of `chunk_cols` columns, one chunk per
// workgroup, as a sequence of near-equal launches of at most
// `rounds_per_launch` rounds of workgroups each.  With several tensors
// (tc != null) every launch carries the segments its columns fall into as an
// argument; only when some launch would need more than fit there, the whole
// table goes through the workspace instead (written once per call).
// The chunks are first_chunk .. first_chunk+chunks-1 of the call's column
// space; their slots in the per-chunk partial-sum arrays start at first_slot.
// bytes_per_chunk: what the pass reads and writes per chunk (decides between one launch and rounds); 0 with
// rounds_per_launch > 1 for a pass that has its own launch length.
// first_fn: when set, the kernel of the first launch (the variant of fn that does the step's selection itself).
int launch(StepKernel fn, int block, long long first_chunk, long long first_slot, long long chunks,
           long long chunk_cols, hipStream_t stream, StepParams& p, TableCtx* tc, double bytes_per_chunk,
           int rounds_per_launch = 1, StepKernel first_fn = nullptr) {
  if (chunks <= 0) return BSGD_OK;
  if (first_chunk + chunks > 0x7fffffffLL || first_slot + chunks > 0x7fffffffLL || fn == nullptr) return BSGD_ERR_ARG;
  const bool multi = tc != nullptr;
  // near-equal launches of one resident round (times rounds_per_launch) each; the round depends on the dynamic LDS
  auto launch_size = [&](size_t lds) {
    long long round = rounds_per_launch * round_size(fn, block, lds);
    if (rounds_per_launch == 1 ? one_launch(fn, block, lds, chunks, bytes_per_chunk) : 2 * chunks < 5 * round)
      round = chunks;
    const long long launches = (chunks + round - 1) / round;
    return (chunks + launches - 1) / launches;
  };
  // columns a launch covers, clipped to the columns that belong to tensors
  auto span_of = [&](long long first, long long n, long long* lo, long long* hi) {
    *lo = p.base + (first_chunk + first) * chunk_cols;
    *hi = p.base + (first_chunk + first + n) * chunk_cols;
    if (*lo < p.col_lo) *lo = p.col_lo;
    if (*hi > p.col_hi) *hi = p.col_hi;
  };
  long long per = 0;
  bool embed = multi && g_table_mode.load(std::memory_order_relaxed) == 0;
  if (embed) {
    per = launch_size(sizeof(unsigned) * (kEmbedSegments + 1));
    for (long long first = 0; first < chunks && embed; first += per) {
      long long lo, hi;
      span_of(first, chunks - first < per ? chunks - first : per, &lo, &hi);
      int j0, j1;
      segment_window(*tc->plan, lo, hi, &j0, &j1);
      if (j1 - j0 + 1 > kEmbedSegments) embed = false;
    }
  }
  if (!embed) per = launch_size(multi ? sizeof(unsigned) * ((size_t)tc->plan->S + 1) : 0);
  if (multi && !embed && !tc->uploaded) {
    const int rc = upload_table(*tc, stream);
    if (rc != BSGD_OK) return rc;
  }

  EmbeddedTable et;                                   // filled per launch when the table travels as an argument
  NoTable none{};
  for (long long first = 0; first < chunks; first += per) {
    const long long n = chunks - first < per ? chunks - first : per;
    ++t_last_launches;
    p.chunk_base = (int)(first_chunk + first);
    p.slot_base = (int)(first_slot + first);
    size_t lds = 0;
    void* second = &none;
    if (multi) {
      if (embed) {
        long long lo, hi;
        span_of(first, n, &lo, &hi);
        int j0, j1;
        segment_window(*tc->plan, lo, hi, &j0, &j1);
        const int count = j1 - j0 + 1;
        for (int i = 0; i < count; ++i) {
          et.seg[i] = tc->plan->segs[j0 + i];
          et.start[i] = tc->plan->starts[j0 + i];
        }
        et.start[count] = tc->plan->starts[j1 + 1];
        p.table = nullptr;
        p.starts = nullptr;
        p.S = count;
      } else {
        p.table = tc->d_table;
        p.starts = tc->d_starts;
        p.S = tc->plan->S;
      }
      lds = sizeof(unsigned) * ((size_t)p.S + 1);
      second = &et;
    }
    void* args[] = {&p, second};
    hipError_t e = hipLaunchKernel(first == 0 && first_fn != nullptr ? first_fn : fn, dim3((unsigned)n), dim3(block),
                                   args, lds, stream);
    if (e != hipSuccess) return BSGD_ERR_HIP;
  }
  return BSGD_OK;
}

bool check_select_args(const float* arrival_t, int N, int b) {
  return arrival_t != nullptr && N >= 1 && b >= 0 && (long long)N + b <= BSGD_MAX_WORKERS;
}

}  // namespace

extern "C" {

static int enqueue_select(const float* arrival_t, int32_t N, int32_t b, const bsgd_select_opts* opts,
                          int32_t* sel_idx, int32_t* n_kept, int32_t* n_grad, float* t_step, int32_t* status,
                          hipStream_t stream) {
  SelectOpts o{nullptr, 0, INFINITY, 0, nullptr, (int*)n_grad};
  if (opts != nullptr) {
    if (opts->n_min < 0 || opts->n_min > N + b || opts->deadline != opts->deadline) return BSGD_ERR_ARG;
    o = SelectOpts{opts->tags, opts->step_tag, opts->deadline, opts->n_min, opts->row_count, (int*)n_grad};
  }
  const int W = N + b;
  void (*fn)(const float*, int, int, SelectOpts, int*, int*, float*, int*) =
      W <= 64 ? k_select<1, true> : W <= 128 ? k_select<2, false> : W <= 192 ? k_select<3, false> : k_select<4, false>;
  hipLaunchKernelGGL(fn, dim3(1), dim3(64), 0, stream, arrival_t, (int)N, W, o, (int*)sel_idx, (int*)n_kept, t_step,
                     (int*)status);
  return hipGetLastError() == hipSuccess ? BSGD_OK : BSGD_ERR_HIP;
}

static int enqueue_select_job(int32_t N, const SelectJob& j, hipStream_t stream) {
  const int W = j.W;
  void (*fn)(const float*, int, int, SelectOpts, int*, int*, float*, int*) =
      W <= 64 ? k_select<1, true> : W <= 128 ? k_select<2, false> : W <= 192 ? k_select<3, false> : k_select<4, false>;
  hipLaunchKernelGGL(fn, dim3(1), dim3(64), 0, stream, j.arrival_t, (int)N, W, j.opts, j.sel_idx, j.n_kept, j.t_step,
                     j.status);
  return hipGetLastError() == hipSuccess ? BSGD_OK : BSGD_ERR_HIP;
}

int bsgd_select_first_n(const float* arrival_t, int32_t N, int32_t b, int32_t* sel_idx, float* t_step,
                        int32_t* status, void* stream) {
  if (!check_select_args(arrival_t, N, b) || sel_idx == nullptr || status == nullptr) return BSGD_ERR_ARG;
  return enqueue_select(arrival_t, N, b, nullptr, sel_idx, nullptr, nullptr, t_step, status, (hipStream_t)stream);
}

int bsgd_select_ex(const float* arrival_t, int32_t N, int32_t b, const bsgd_select_opts* opts, int32_t* sel_idx,
                   int32_t* n_kept, float* t_step, int32_t* status, void* stream) {
  if (!check_select_args(arrival_t, N, b) || sel_idx == nullptr || status == nullptr || opts == nullptr)
    return BSGD_ERR_ARG;
  if (opts->n_min > 0 && n_kept == nullptr) return BSGD_ERR_ARG;   // the count is the only way to know how many
  if (opts->row_count != nullptr) return BSGD_ERR_ARG;             // the divisor lives in a step's workspace
  return enqueue_select(arrival_t, N, b, opts, sel_idx, n_kept, nullptr, t_step, status, (hipStream_t)stream);
}

size_t bsgd_workspace_bytes(int64_t span, int32_t N, int32_t b, int32_t T, const bsgd_hyper* hyper) {
  if (span < 0 || N < 1 || b < 0 || (long long)N + b > BSGD_MAX_WORKERS || T < 1 || T > BSGD_MAX_TENSORS ||
      hyper == nullptr)
    return 0;
  return layout(span, T, clip_on(hyper), worker_clip_on(hyper)).total;
}

// Host-only validation shared by bsgd_reduce_update and bsgd_step: nothing is
// enqueued unless this passes.
static int make_plan(const float* grads, int64_t ld, int32_t N, const bsgd_tensor* tensors, int32_t T,
                     const bsgd_hyper* hyper, const void* workspace, size_t workspace_bytes, Plan* plan,
                     int too_small_code = BSGD_ERR_ARG) {
  if (grads == nullptr || tensors == nullptr || hyper == nullptr || workspace == nullptr) return BSGD_ERR_ARG;
  if (N < 1 || N > BSGD_MAX_WORKERS || T < 1 || T > BSGD_MAX_TENSORS || ld < 0) return BSGD_ERR_ARG;
  if (hyper->opt < BSGD_SGD || hyper->opt > BSGD_RMSPROP_MOM) return BSGD_ERR_ARG;
  if ((reinterpret_cast<uintptr_t>(workspace) & (kAlign - 1)) != 0) return BSGD_ERR_ARG;
  // Row loads are aligned 16-byte accesses: the gradient base must be 16-byte
  // aligned and the row stride a multiple of 4 elements.
  if ((reinterpret_cast<uintptr_t>(grads) & 15) != 0 || (ld & 3) != 0) return BSGD_ERR_ARG;
  const int mode = hyper->opt;
  long long span = 0;
  int live = 0, last_live = -1, with_ema = 0;
  for (int j = 0; j < T; ++j) {
    const bsgd_tensor& t = tensors[j];
    if (t.numel < 0 || t.grad_offset < 0) return BSGD_ERR_ARG;
    if (t.numel == 0) continue;
    if (t.theta == nullptr || (reinterpret_cast<uintptr_t>(t.theta) & 3)) return BSGD_ERR_ARG;
    if (mode >= BSGD_MOMENTUM && (t.s0 == nullptr || (reinterpret_cast<uintptr_t>(t.s0) & 3))) return BSGD_ERR_ARG;
    if (mode == BSGD_RMSPROP_MOM && (t.s1 == nullptr || (reinterpret_cast<uintptr_t>(t.s1) & 3))) return BSGD_ERR_ARG;
    if (t.grad_offset > ld - t.numel) return BSGD_ERR_ARG;
    if (t.ema != nullptr) {
      if (reinterpret_cast<uintptr_t>(t.ema) & 3) return BSGD_ERR_ARG;
      ++with_ema;
    }
    if (t.grad_offset + t.numel > span) span = t.grad_offset + t.numel;
    ++live;
    last_live = j;
  }
  if (with_ema != 0 && with_ema != live) return BSGD_ERR_ARG;   // all tensors or none
  if (with_ema != 0 && !(hyper->ema_decay >= 0.0f && hyper->ema_decay <= 1.0f)) return BSGD_ERR_ARG;
  plan->ema = with_ema != 0;
  if (span >= 0xFFFFFFF0LL) return BSGD_ERR_ARG;       // segment starts are kept as 32-bit columns
  const WsLayout L = layout(span, T, clip_on(hyper), worker_clip_on(hyper));
  if (workspace_bytes < L.total) return too_small_code;
  plan->span = span;
  plan->S = 0;
  if (live == 0) return BSGD_OK;                       // nothing to update
  if (live == 1) {
    const bsgd_tensor& t = tensors[last_live];
    plan->S = 1;
    plan->single = Segment{t.theta, t.s0, t.s1, t.ema};
    plan->col_lo = t.grad_offset;
    plan->col_hi = t.grad_offset + t.numel;
    return BSGD_OK;
  }
  // sort by position in the row, refuse overlap, make gaps explicit
  std::vector<int> order;
  order.reserve(live);
  for (int j = 0; j < T; ++j)
    if (tensors[j].numel > 0) order.push_back(j);
  std::sort(order.begin(), order.end(),
            [&](int a, int b) { return tensors[a].grad_offset < tensors[b].grad_offset; });
  plan->segs.reserve(2 * (size_t)live);
  plan->starts.reserve(2 * (size_t)live + 1);
  long long at = tensors[order[0]].grad_offset;
  plan->col_lo = at;
  for (int idx : order) {
    const bsgd_tensor& t = tensors[idx];
    if (t.grad_offset < at) return BSGD_ERR_ARG;       // two tensors claim the same gradient columns
    if (t.grad_offset > at) {                          // a gap
      plan->segs.push_back(Segment{nullptr, nullptr, nullptr, nullptr});
      plan->starts.push_back((unsigned)at);
    }
    plan->segs.push_back(Segment{t.theta, t.s0, t.s1, t.ema});
    plan->starts.push_back((unsigned)t.grad_offset);
    at = t.grad_offset + t.numel;
  }
  plan->col_hi = at;
  plan->starts.push_back((unsigned)at);
  plan->S = (int)plan->segs.size();
  return BSGD_OK;
}

// N: kept rows when the host knows the count (n_dev null); otherwise the count is read from n_dev on the device and
// row_cap is the most it can be (N+b in the time-out mode).  Everything sized per kept row uses row_cap.
static int enqueue_select_job(int32_t N, const SelectJob& j, hipStream_t stream);

// job: the selection this update belongs to, not yet enqueued (null: sel_idx is ready, or will be by stream order).
// A step that goes out as one launch of the narrow shape does the selection inside that launch; otherwise
// k_select is enqueued first.
static int enqueue_update(const float* grads, int64_t ld, const int32_t* sel_idx, const int32_t* status, int32_t N,
                          int32_t row_cap, const int32_t* n_dev, const int32_t* div_dev, int32_t T,
                          const bsgd_hyper* hyper, void* workspace, const Plan& plan, hipStream_t stream,
                          const SelectJob* job = nullptr) {
  t_last_launches = 0;
  t_last_fused = 0;
  if (plan.S == 0) return job != nullptr ? enqueue_select_job(N, *job, stream) : (int)BSGD_OK;
  const int mode = hyper->opt;
  const bool clip = clip_on(hyper);
  const bool wclip = worker_clip_on(hyper);
  const WsLayout L = layout(plan.span, T, clip, wclip);
  char* ws = static_cast<char*>(workspace);

  StepParams p{};
  p.grads = grads;
  p.ld = ld;
  p.sel_idx = sel_idx;
  p.status = status;
  p.N = N;
  p.inv_n = 1.0f / (float)N;
  p.n_dev = n_dev;
  p.div_dev = div_dev;
  p.row_scale = wclip ? reinterpret_cast<const float*>(ws + L.rowscale_off) : nullptr;
  p.row_partials = reinterpret_cast<double*>(ws + L.rowpart_off);
  p.n_stride = row_cap;                                // rows per chunk in row_partials: as many as can be kept
  p.worker_clip = hyper->worker_clip_norm;
  p.lr = hyper->lr;
  p.mu = hyper->momentum;
  p.rho = hyper->decay;
  p.one_minus_rho = (float)(1.0 - (double)hyper->decay);
  p.eps = hyper->eps;
  p.alpha = hyper->ema_decay;
  p.one_minus_alpha = (float)(1.0 - (double)hyper->ema_decay);
  p.gbar = reinterpret_cast<float*>(ws + L.gbar_off);
  p.partials = reinterpret_cast<double*>(ws + L.partials_off);
  p.header = reinterpret_cast<const WsHeader*>(ws);
  p.table = reinterpret_cast<const Segment*>(ws + L.table_off);
  p.starts = reinterpret_cast<const unsigned*>(ws + L.starts_off);
  p.S = plan.S;
  p.single = plan.single;
  p.col_lo = plan.col_lo;
  p.col_hi = plan.col_hi;
  p.base = plan.col_lo & ~3LL;

  const long long cols = ((plan.col_hi + 3) & ~3LL) - p.base;   // columns the chunks must cover
  const bool multi = plan.S > 1;
  const int ema = plan.ema ? 1 : 0;
  // the shape is chosen for the columns that belong to tensors: wide gaps are neither launched nor read
  long long covered = plan.col_hi - plan.col_lo;
  for (int j = 0; j < (multi ? plan.S : 0); ++j)
    if (plan.segs[j].theta == nullptr) covered -= (long long)plan.starts[j + 1] - (long long)plan.starts[j];
  const Variant& var = pick_variant((covered + 3) / 4, [&](const Variant& v) {
    return clip ? v.reduce[multi ? 1 : 0] : v.rows[mode][multi ? 1 : 0][ema];
  });
  const long long chunk_cols = 4LL * var.BS * var.V;
  const long long total_chunks = (cols + chunk_cols - 1) / chunk_cols;
  if (total_chunks > L.max_chunks || total_chunks > 0x7fffffffLL) return BSGD_ERR_ARG;   // cannot happen

  TableCtx table{&plan, reinterpret_cast<Segment*>(ws + L.table_off), reinterpret_cast<unsigned*>(ws + L.starts_off), false};
  TableCtx* tc = multi ? &table : nullptr;

  // bytes a chunk of each pass moves: kept rows plus theta/state streams
  const int state_streams = 2 * (1 + mode + ema);      // read and written: theta, s0, s1, moving average
  const double col_bytes = 4.0 * (double)chunk_cols;
  const double rows_pass_bytes = col_bytes * (row_cap + (clip ? 1 : state_streams));
  const double rowsq_pass_bytes = col_bytes * row_cap;
  // only chunks that hold columns of some tensor are launched; the per-chunk partial sums are indexed by launch order
  const std::vector<Run> runs = chunk_runs(plan, p.base, chunk_cols, total_chunks);
  long long slots = 0;
  for (const Run& r : runs) slots += r.count;
  // The selection inside the step's first launch: at most 64 workers, no per-worker clip (its norm pass needs
  // the kept rows first).  Every workgroup of that launch ranks the arrival times for itself; its first one
  // publishes the kept rows and the status, which the step's later launches read like k_select's.
  const StepKernel first_pass = clip ? var.reduce[multi ? 1 : 0] : var.rows[mode][multi ? 1 : 0][ema];
  const StepKernel first_pass_sel = clip ? var.reduce_sel[multi ? 1 : 0] : var.rows_sel[mode][multi ? 1 : 0][ema];
  const bool fuse = job != nullptr && first_pass_sel != nullptr && job->W <= 64 && !wclip &&
                    g_fuse_select.load(std::memory_order_relaxed) != 0;
  if (job != nullptr && !fuse) {
    const int rc = enqueue_select_job(N, *job, stream);
    if (rc != BSGD_OK) return rc;
  }
  if (fuse) {
    p.job = *job;
    t_last_fused = 1;
  }
  auto launch_runs = [&](StepKernel fn, double bytes_per_chunk, int rounds, StepKernel first_fn = nullptr) {
    long long slot = 0;
    for (const Run& r : runs) {
      const int rc = launch(fn, var.BS, r.first, slot, r.count, chunk_cols, stream, p, tc, bytes_per_chunk, rounds,
                            slot == 0 ? first_fn : nullptr);
      if (rc != BSGD_OK) return rc;
      slot += r.count;
    }
    return (int)BSGD_OK;
  };
  if (wclip) {
    // per-worker clipping: every kept row's norm first (one more pass over the kept rows), then its scale
    int rc = launch_runs(var.rowsq[multi ? 1 : 0], rowsq_pass_bytes, 1);
    if (rc != BSGD_OK) return rc;
    hipLaunchKernelGGL(k_row_scales, dim3((unsigned)row_cap), dim3(kRowScaleBlock), 0, stream,
                       (const double*)p.row_partials, (int)slots, (int)row_cap, (int)N, (const int*)n_dev,
                       hyper->worker_clip_norm, (const int*)status, reinterpret_cast<float*>(ws + L.rowscale_off));
    if (hipGetLastError() != hipSuccess) return BSGD_ERR_HIP;
  }
  if (!clip) return launch_runs(first_pass, rows_pass_bytes, 1, fuse ? first_pass_sel : nullptr);

  int rc = launch_runs(first_pass, rows_pass_bytes, 1, fuse ? first_pass_sel : nullptr);
  if (rc != BSGD_OK) return rc;
  hipLaunchKernelGGL(k_finalize_norm, dim3(1), dim3(kFinalizeBlock), 0, stream, (const double*)p.partials,
                     (int)slots, hyper->clip_norm, (const int*)status, reinterpret_cast<WsHeader*>(ws));
  if (hipGetLastError() != hipSuccess) return BSGD_ERR_HIP;
  // the second pass has no row loop to keep in step: longer launches, fewer ramp-ups and tails
  return launch_runs(var.apply[mode][multi ? 1 : 0][ema], 0.0, kApplyRoundsPerLaunch);
}

int bsgd_reduce_update(const float* grads, int64_t ld, const int32_t* sel_idx, const int32_t* status, int32_t N,
                       const bsgd_tensor* tensors, int32_t T, const bsgd_hyper* hyper, void* workspace,
                       size_t workspace_bytes, void* stream) {
  if (sel_idx == nullptr) return BSGD_ERR_ARG;
  Plan plan;
  int rc = make_plan(grads, ld, N, tensors, T, hyper, workspace, workspace_bytes, &plan);
  if (rc != BSGD_OK) return rc;
  return enqueue_update(grads, ld, sel_idx, status, N, N, nullptr, nullptr, T, hyper, workspace, plan,
                        (hipStream_t)stream);
}

// status_out / t_step_out: where the selection writes the status word and the waiting time, and where the later
// kernels read the status from; null: the workspace header.
static int step_common(const float* grads, int64_t ld, const float* arrival_t, int32_t N, int32_t b,
                       const bsgd_select_opts* opts, const bsgd_tensor* tensors, int32_t T, const bsgd_hyper* hyper,
                       void* workspace, size_t workspace_bytes, void* stream, int32_t* status_out = nullptr,
                       float* t_step_out = nullptr, int too_small_code = BSGD_ERR_ARG) {
  if (!check_select_args(arrival_t, N, b)) return BSGD_ERR_ARG;
  if (opts != nullptr && (opts->n_min < 0 || opts->n_min > N + b || opts->deadline != opts->deadline)) return BSGD_ERR_ARG;
  const bool counted = opts != nullptr && opts->row_count != nullptr;
  if (counted && hyper != nullptr && worker_clip_on(hyper)) return BSGD_ERR_ARG;   // a sum of gradients has no single worker's norm
  Plan plan;
  // in deadline mode up to N+b rows may be kept
  const bool all_in_time = opts != nullptr && opts->n_min > 0;
  int rc = make_plan(grads, ld, all_in_time ? N + b : N, tensors, T, hyper, workspace, workspace_bytes, &plan,
                     too_small_code);
  if (rc != BSGD_OK) return rc;
  char* ws = static_cast<char*>(workspace);
  WsHeader* hdr = reinterpret_cast<WsHeader*>(ws);
  int* sel = reinterpret_cast<int*>(ws + kAlign);
  int32_t* status = status_out != nullptr ? status_out : &hdr->status;
  float* t_step = status_out != nullptr ? t_step_out : &hdr->t_step;
  SelectJob job{};
  job.arrival_t = arrival_t;
  job.W = N + b;
  job.opts = SelectOpts{nullptr, 0, INFINITY, 0, nullptr, &hdr->n_grad};
  if (opts != nullptr)
    job.opts = SelectOpts{opts->tags, opts->step_tag, opts->deadline, opts->n_min, opts->row_count, &hdr->n_grad};
  job.sel_idx = sel;
  job.n_kept = &hdr->n_kept;
  job.t_step = t_step;
  job.status = status;
  return enqueue_update(grads, ld, sel, status, N, all_in_time ? N + b : N, all_in_time ? &hdr->n_kept : nullptr,
                        counted ? &hdr->n_grad : nullptr, T, hyper, workspace, plan, (hipStream_t)stream, &job);
}

int bsgd_step(const float* grads, int64_t ld, const float* arrival_t, int32_t N, int32_t b,
              const bsgd_tensor* tensors, int32_t T, const bsgd_hyper* hyper, void* workspace,
              size_t workspace_bytes, void* stream) {
  return step_common(grads, ld, arrival_t, N, b, nullptr, tensors, T, hyper, workspace, workspace_bytes, stream);
}

int bsgd_step_ex(const float* grads, int64_t ld, const float* arrival_t, int32_t N, int32_t b,
                 const bsgd_select_opts* opts, const bsgd_tensor* tensors, int32_t T, const bsgd_hyper* hyper,
                 void* workspace, size_t workspace_bytes, void* stream) {
  if (opts == nullptr) return BSGD_ERR_ARG;
  return step_common(grads, ld, arrival_t, N, b, opts, tensors, T, hyper, workspace, workspace_bytes, stream);
}

// ---------------------------------------------------------------------------
// bsgd_step for callers that cannot hand over (or allocate) a workspace: the
// step's scratch lives in a device array that is part of this library's code
// object.  Each GPU holds its own copy at its own address from the moment the
// library's device code is loaded there until the process ends.
// ---------------------------------------------------------------------------
static __device__ __attribute__((used)) __align__(256) unsigned char scratch[BSGD_STATIC_SCRATCH_BYTES];

// In host code the name `scratch` is only a handle for the runtime's symbol
// table; the array's device address is asked for once per device, with that
// device current, and kept.
constexpr int kMaxDevices = 64;
static int static_scratch(void** out) {
  static std::mutex mu;
  static void* ptr_of_device[kMaxDevices] = {};
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return BSGD_ERR_HIP;
  std::lock_guard<std::mutex> lock(mu);
  if (ptr_of_device[dev] == nullptr) {
    void* ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || ptr == nullptr) return BSGD_ERR_HIP;
    if ((reinterpret_cast<uintptr_t>(ptr) & (kAlign - 1)) != 0) return BSGD_ERR_HIP;
    ptr_of_device[dev] = ptr;
  }
  *out = ptr_of_device[dev];
  return BSGD_OK;
}

int bsgd_step_noalloc(const float* grads, int64_t ld, const float* arrival_t, int32_t N, int32_t b,
                      const bsgd_tensor* tensors, int32_t T, const bsgd_hyper* hyper, int32_t* status, float* t_step,
                      void* stream) {
  if (status == nullptr) return BSGD_ERR_ARG;
  void* ws = nullptr;
  const int rc = static_scratch(&ws);
  if (rc != BSGD_OK) return rc;
  // Nothing in the array has to start at zero: every word a kernel of the step reads (status, kept rows, table,
  // partial sums, stored mean) is written earlier in the same step, so what the last call left behind is never seen.
  return step_common(grads, ld, arrival_t, N, b, nullptr, tensors, T, hyper, ws, (size_t)BSGD_STATIC_SCRATCH_BYTES,
                     stream, status, t_step, BSGD_ERR_SCRATCH);
}

int bsgd_last_status(const void* workspace, void* stream, int32_t* status_out, float* t_step_out) {
  if (workspace == nullptr) return BSGD_ERR_ARG;
  if (hipStreamSynchronize((hipStream_t)stream) != hipSuccess) return BSGD_ERR_HIP;
  WsHeader h;
  if (hipMemcpy(&h, workspace, sizeof(h), hipMemcpyDeviceToHost) != hipSuccess) return BSGD_ERR_HIP;
  if (status_out) *status_out = h.status;
  if (t_step_out) *t_step_out = h.t_step;
  return BSGD_OK;
}

int bsgd_last_kept_count(const void* workspace, void* stream, int32_t* n_kept_out) {
  if (workspace == nullptr || n_kept_out == nullptr) return BSGD_ERR_ARG;
  if (hipStreamSynchronize((hipStream_t)stream) != hipSuccess) return BSGD_ERR_HIP;
  WsHeader h;
  if (hipMemcpy(&h, workspace, sizeof(h), hipMemcpyDeviceToHost) != hipSuccess) return BSGD_ERR_HIP;
  *n_kept_out = h.n_kept;
  return BSGD_OK;
}

int bsgd_last_gradient_count(const void* workspace, void* stream, int32_t* n_gradients_out) {
  if (workspace == nullptr || n_gradients_out == nullptr) return BSGD_ERR_ARG;
  if (hipStreamSynchronize((hipStream_t)stream) != hipSuccess) return BSGD_ERR_HIP;
  WsHeader h;
  if (hipMemcpy(&h, workspace, sizeof(h), hipMemcpyDeviceToHost) != hipSuccess) return BSGD_ERR_HIP;
  *n_gradients_out = h.n_grad;
  return BSGD_OK;
}

int bsgd_last_selection(const void* workspace, void* stream, int32_t N, int32_t* sel_idx_out) {
  if (workspace == nullptr || sel_idx_out == nullptr || N < 1 || N > BSGD_MAX_WORKERS) return BSGD_ERR_ARG;
  if (hipStreamSynchronize((hipStream_t)stream) != hipSuccess) return BSGD_ERR_HIP;
  if (hipMemcpy(sel_idx_out, static_cast<const char*>(workspace) + kAlign, sizeof(int) * (size_t)N,
                hipMemcpyDeviceToHost) != hipSuccess)
    return BSGD_ERR_HIP;
  return BSGD_OK;
}

int bsgd_last_clip(const void* workspace, void* stream, double* norm_out, float* scale_out) {
  if (workspace == nullptr) return BSGD_ERR_ARG;
  if (hipStreamSynchronize((hipStream_t)stream) != hipSuccess) return BSGD_ERR_HIP;
  WsHeader h;
  if (hipMemcpy(&h, workspace, sizeof(h), hipMemcpyDeviceToHost) != hipSuccess) return BSGD_ERR_HIP;
  if (norm_out) *norm_out = h.norm;
  if (scale_out) *scale_out = h.clip_scale;
  return BSGD_OK;
}

int bsgd_set_tuning(int32_t block, int32_t vec, int32_t unroll, int32_t nontemporal) {
  if (block < 0 && vec < 0 && unroll < 0 && nontemporal < 0) {
    g_variant.store(-1, std::memory_order_relaxed);    // back to the automatic choice
    return BSGD_OK;
  }
  const int cur_i = g_variant.load(std::memory_order_relaxed);
  const Variant& cur = kVariants[cur_i < 0 ? 0 : cur_i];
  const int BS = block < 0 ? cur.BS : block, V = vec < 0 ? cur.V : vec, U = unroll < 0 ? cur.U : unroll;
  const int NT = nontemporal < 0 ? cur.NT : nontemporal;
  for (int i = 0; i < kNumVariants; ++i) {
    const Variant& v = kVariants[i];
    if (v.BS == BS && v.V == V && v.U == U && v.NT == NT) {
      g_variant.store(i, std::memory_order_relaxed);
      return BSGD_OK;
    }
  }
  return BSGD_ERR_ARG;
}

int bsgd_debug_chunk_runs(const bsgd_tensor* tensors, int32_t T, int64_t chunk_cols, int64_t* first, int64_t* count,
                          int32_t capacity, int32_t* n_runs) {
  if (tensors == nullptr || first == nullptr || count == nullptr || n_runs == nullptr || capacity < 1 ||
      chunk_cols < 4 || (chunk_cols & 3) != 0)
    return BSGD_ERR_ARG;
  // host arithmetic only: the pointers below are never dereferenced
  bsgd_hyper hy{};
  hy.opt = BSGD_SGD;
  Plan plan;
  const int rc = make_plan(reinterpret_cast<const float*>(uintptr_t(16)), (int64_t)0x7ffffffffffffffcLL, 1, tensors, T, &hy,
                           reinterpret_cast<const void*>(uintptr_t(256)), ~(size_t)0, &plan);
  if (rc != BSGD_OK) return rc;
  *n_runs = 0;
  if (plan.S == 0) return BSGD_OK;
  const long long base = plan.col_lo & ~3LL;
  const long long cols = ((plan.col_hi + 3) & ~3LL) - base;
  const std::vector<Run> runs = chunk_runs(plan, base, chunk_cols, (cols + chunk_cols - 1) / chunk_cols);
  if ((long long)runs.size() > capacity) return BSGD_ERR_ARG;
  for (size_t i = 0; i < runs.size(); ++i) {
    first[i] = runs[i].first;
    count[i] = runs[i].count;
  }
  *n_runs = (int32_t)runs.size();
  return BSGD_OK;
}

int bsgd_last_launch_count(void) { return t_last_launches; }

int bsgd_last_step_fused_selection(void) { return t_last_fused; }

int bsgd_set_fused_selection(int32_t on) {
  if (on != 0 && on != 1) return BSGD_ERR_ARG;
  g_fuse_select.store(on, std::memory_order_relaxed);
  return BSGD_OK;
}

int bsgd_set_table_mode(int32_t mode) {
  if (mode != 0 && mode != 1) return BSGD_ERR_ARG;
  g_table_mode.store(mode, std::memory_order_relaxed);
  return BSGD_OK;
}

int bsgd_num_shapes(void) { return kNumVariants; }

int bsgd_get_shape(int32_t i, int32_t* out4) {
  if (i < 0 || i >= kNumVariants || out4 == nullptr) return BSGD_ERR_ARG;
  const Variant& v = kVariants[i];
  out4[0] = v.BS; out4[1] = v.V; out4[2] = v.U; out4[3] = v.NT;
  return BSGD_OK;
}

int bsgd_calibration_copy(void* dst, const void* src, int64_t bytes, void* stream) {
  if (dst == nullptr || src == nullptr || bytes <= 0 || (bytes & 15) != 0) return BSGD_ERR_ARG;
  if ((reinterpret_cast<uintptr_t>(dst) & 15) != 0 || (reinterpret_cast<uintptr_t>(src) & 15) != 0) return BSGD_ERR_ARG;
  const long long n16 = bytes / 16;
  const long long grid = (n16 + 255) / 256;
  if (grid > 0x7fffffffLL) return BSGD_ERR_ARG;
  hipLaunchKernelGGL(k_calibration_copy, dim3((unsigned)grid), dim3(256), 0, (hipStream_t)stream,
                     static_cast<const f4*>(src), static_cast<f4*>(dst), n16);
  return hipGetLastError() == hipSuccess ? BSGD_OK : BSGD_ERR_HIP;
}

int bsgd_yardstick_streams(const void* const* read_ptrs, int32_t n_read, void* const* write_ptrs, int32_t n_write,
                           int64_t bytes, int32_t vec, void* stream) {
  if (n_read < 1 || n_read > kYardMaxStreams || n_write < 0 || n_write > kYardMaxStreams || read_ptrs == nullptr ||
      (n_write > 0 && write_ptrs == nullptr) || bytes <= 0 || (bytes & 15) != 0)
    return BSGD_ERR_ARG;
  YardArgs a{};
  for (int i = 0; i < n_read; ++i) {
    if (read_ptrs[i] == nullptr || (reinterpret_cast<uintptr_t>(read_ptrs[i]) & 15) != 0) return BSGD_ERR_ARG;
    a.rd[i] = static_cast<const f4*>(read_ptrs[i]);
  }
  for (int i = 0; i < n_write; ++i) {
    if (write_ptrs[i] == nullptr || (reinterpret_cast<uintptr_t>(write_ptrs[i]) & 15) != 0) return BSGD_ERR_ARG;
    a.wr[i] = static_cast<f4*>(write_ptrs[i]);
  }
  a.n_read = n_read;
  a.n_write = n_write;
  a.n16 = bytes / 16;
  // the mixes of the step's passes: read only; update of theta/ms/m; pass 2 of a clipped step; pre-combine; copy
  void (*fn)(YardArgs) = nullptr;
#define BSGD_YARD(R, W)                                                                           \
  if (n_read == R && n_write == W)                                                                \
    fn = vec == 1 ? k_yardstick<1, R, W> : vec == 2 ? k_yardstick<2, R, W>                        \
         : vec == 4 ? k_yardstick<4, R, W> : vec == 8 ? k_yardstick<8, R, W> : nullptr;
  BSGD_YARD(1, 0) BSGD_YARD(3, 3) BSGD_YARD(3, 2) BSGD_YARD(2, 2) BSGD_YARD(2, 1) BSGD_YARD(1, 1)
#undef BSGD_YARD
  if (fn == nullptr) return BSGD_ERR_ARG;               // a mix or width that is not compiled in
  const long long grid = (a.n16 + 256LL * vec - 1) / (256LL * vec);
  if (grid > 0x7fffffffLL) return BSGD_ERR_ARG;
  hipLaunchKernelGGL(fn, dim3((unsigned)grid), dim3(256), 0, (hipStream_t)stream, a);
  return hipGetLastError() == hipSuccess ? BSGD_OK : BSGD_ERR_HIP;
}

int bsgd_precombine(const float* grads, int64_t ld, int64_t cols, const float* arrival_t, const int32_t* group_size,
                    int32_t M, float* combined, int64_t ld_out, float* arrival_m, int32_t* row_count, void* stream) {
  if (grads == nullptr || arrival_t == nullptr || group_size == nullptr || combined == nullptr ||
      arrival_m == nullptr || row_count == nullptr)
    return BSGD_ERR_ARG;
  if (M < 1 || M > BSGD_MAX_WORKERS || cols < 1 || ld < cols || ld_out < cols || (ld & 3) != 0 || (ld_out & 3) != 0)
    return BSGD_ERR_ARG;
  if ((reinterpret_cast<uintptr_t>(grads) & 15) != 0 || (reinterpret_cast<uintptr_t>(combined) & 15) != 0)
    return BSGD_ERR_ARG;
  CombineParams p{};
  long long W = 0;
  for (int m = 0; m < M; ++m) {
    if (group_size[m] < 1 || W + group_size[m] > BSGD_MAX_WORKERS) return BSGD_ERR_ARG;
    p.first[m] = (unsigned char)W;
    W += group_size[m];
  }
  p.last = (int)W;
  // the output may not overlap the input
  const uintptr_t g0 = reinterpret_cast<uintptr_t>(grads), g1 = g0 + sizeof(float) * (size_t)W * (size_t)ld;
  const uintptr_t c0 = reinterpret_cast<uintptr_t>(combined), c1 = c0 + sizeof(float) * (size_t)M * (size_t)ld_out;
  if (c0 < g1 && g0 < c1) return BSGD_ERR_ARG;
  p.grads = grads;
  p.ld = ld;
  p.combined = combined;
  p.ld_out = ld_out;
  p.cols4 = (cols + 3) & ~3LL;
  p.M = M;
  // Narrow chunks (one 16-byte group per thread): with a third or more of the traffic written, many small
  // workgroups whose reads and writes interleave finely stream 10-15 % faster than wide ones (measured);
  // two rows per batch for machines of up to three workers, one row at a time for larger ones.
  using S2 = Shape<256, 1, 2, true>;
  using S1 = Shape<256, 1, 1, true>;
  const long long chunk_cols = 4LL * S2::BS * S2::V;
  const long long chunks = (p.cols4 + chunk_cols - 1) / chunk_cols;
  if (chunks > 0x7fffffffLL) return BSGD_ERR_ARG;
  hipStream_t st = (hipStream_t)stream;
  if (W <= 3LL * M)
    hipLaunchKernelGGL(k_precombine<S2>, dim3((unsigned)chunks, (unsigned)M), dim3(S2::BS), 0, st, p);
  else
    hipLaunchKernelGGL(k_precombine<S1>, dim3((unsigned)chunks, (unsigned)M), dim3(S1::BS), 0, st, p);
  if (hipGetLastError() != hipSuccess) return BSGD_ERR_HIP;
  hipLaunchKernelGGL(k_machine_arrival, dim3(1), dim3(64), 0, st, arrival_t, p, arrival_m, (int*)row_count);
  return hipGetLastError() == hipSuccess ? BSGD_OK : BSGD_ERR_HIP;
}

size_t bsgd_straggler_workspace_bytes(int32_t W, int64_t B) {
  if (W < 1 || W > BSGD_MAX_WORKERS || B < 1) return 0;
  const long long slabs = (B + kStragglerSlab - 1) / kStragglerSlab;
  return round_up(sizeof(double) * (size_t)slabs * (size_t)W, kAlign);
}

int bsgd_kth_arrival_times(const float* arrival_t, int32_t W, int64_t B, float* kth_time, double* mean_kth,
                           void* workspace, size_t workspace_bytes, void* stream) {
  if (arrival_t == nullptr || W < 1 || W > BSGD_MAX_WORKERS || B < 1) return BSGD_ERR_ARG;
  if (kth_time == nullptr && mean_kth == nullptr) return BSGD_ERR_ARG;
  const long long slabs = (B + kStragglerSlab - 1) / kStragglerSlab;
  if (slabs > 0x7fffffffLL) return BSGD_ERR_ARG;
  double* partial = nullptr;
  if (mean_kth != nullptr) {
    if (workspace == nullptr || (reinterpret_cast<uintptr_t>(workspace) & (kAlign - 1)) != 0 ||
        workspace_bytes < bsgd_straggler_workspace_bytes(W, B))
      return BSGD_ERR_ARG;
    partial = static_cast<double*>(workspace);
  }
  hipStream_t st = (hipStream_t)stream;
  void (*fn)(const float*, int, long long, float*, double*) =
      W <= 64 ? k_kth_times<1> : W <= 128 ? k_kth_times<2> : W <= 192 ? k_kth_times<3> : k_kth_times<4>;
  hipLaunchKernelGGL(fn, dim3((unsigned)slabs), dim3(kStragglerBlock), 0, st, arrival_t, (int)W, (long long)B,
                     kth_time, partial);
  if (hipGetLastError() != hipSuccess) return BSGD_ERR_HIP;
  if (mean_kth != nullptr) {
    hipLaunchKernelGGL(k_mean_kth, dim3((unsigned)W), dim3(kMeanBlock), 0, st, (const double*)partial, slabs, (int)W,
                       (long long)B, mean_kth);
    if (hipGetLastError() != hipSuccess) return BSGD_ERR_HIP;
  }
  return BSGD_OK;
}

int bsgd_time_to_converge(const double* mean_kth, int32_t W, const double* measured_N, const double* measured_iters,
                          int32_t n_measured, double* est, int32_t* best_N) {
  if (mean_kth == nullptr || est == nullptr || best_N == nullptr || W < 1 || n_measured < 0) return BSGD_ERR_ARG;
  if (n_measured > 0 && (measured_N == nullptr || measured_iters == nullptr)) return BSGD_ERR_ARG;
  std::vector<std::pair<double, double>> pts;
  for (int i = 0; i < n_measured; ++i) {
    if (measured_N[i] != measured_N[i] || measured_iters[i] != measured_iters[i]) return BSGD_ERR_ARG;
    pts.emplace_back(measured_N[i], measured_iters[i]);
  }
  std::sort(pts.begin(), pts.end());
  for (size_t i = 1; i < pts.size(); ++i)
    if (pts[i].first == pts[i - 1].first) return BSGD_ERR_ARG;   // two counts for one N
  const double nan = std::nan("");
  *best_N = 0;
  double best = INFINITY;
  size_t seg = 0;                                      // pts[seg] <= N <= pts[seg + 1]
  for (int N = 1; N <= W; ++N) {
    double iters = nan;
    if (!pts.empty() && N >= pts.front().first && N <= pts.back().first) {
      while (seg + 1 < pts.size() && pts[seg + 1].first < N) ++seg;
      if (pts.size() == 1 || pts[seg].first == N) {
        iters = pts[seg].second;
      } else {
        const double span = pts[seg + 1].first - pts[seg].first;
        iters = pts[seg].second + (pts[seg + 1].second - pts[seg].second) * ((N - pts[seg].first) / span);
      }
    }
    const double e = iters * mean_kth[N - 1];
    est[N - 1] = (iters == iters) ? e : nan;
    if (iters == iters && std::isfinite(e) && e <= best) {
      best = e;
      *best_N = N;
    }
  }
  return BSGD_OK;
}

const char* bsgd_strerror(int code) {
  switch (code) {
    case BSGD_OK: return "ok";
    case BSGD_ERR_ARG: return "invalid argument";
    case BSGD_ERR_TOO_FEW: return "fewer than N gradients arrived; parameters left untouched";
    case BSGD_ERR_HIP: return "HIP runtime call failed";
    case BSGD_ERR_SCRATCH: return "the step needs more scratch memory than the library's static buffer holds";
    default: return "unknown bsgd code";
  }
}

const char* bsgd_version(void) { return "bsgd 0.1 (gfx950)"; }

}  // extern "C"
