// Device code for the backup-worker Sync-SGD step on gfx950 (CDNA4).
//
// All of it is bandwidth- or latency-bound (no dense contraction, so no MFMA):
//   k_select         one wavefront ranks the N+b arrival times and writes the
//                    kept set (Algorithm 4, collect loop; tags and the
//                    time-out variant of Sec. 6 as options).
//   k_step           one streaming pass: gather-sum of the kept gradient rows
//                    in registers, mean, fused optimizer update and moving
//                    average (Algorithm 4, update lines; Sec. 3 "Sync-Opt").
//                    The same kernel, instantiated differently, is both
//                    halves of a step clipped by the global norm (Appendix
//                    A.3): rows -> stored mean + sums of squares, then stored
//                    mean x scale -> update; k_finalize_norm sits in between.
//   k_row_sumsq / k_row_scales   per-worker clipping (Appendix A.3 as printed).
//   k_precombine / k_machine_arrival   one message per machine (Sec. 6).
//   k_kth_times / k_mean_kth     time to collect k gradients (Sec. 3.1).
//   k_calibration_copy / k_yardstick   measurement aids: plain copies and
//                    plain streaming kernels with a chosen mix of streams.
// A step small enough to be one launch does its selection inside k_step
// (select_wave is shared by k_select and k_step<..., SELECT>).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>
#include <type_traits>

namespace bsgd {

typedef float f4 __attribute__((ext_vector_type(4)));
typedef f4 f4u __attribute__((aligned(4)));          // float4 that is only 4-byte aligned

// Launch shape of the reduce/update kernel.
//   BS   threads per workgroup
//   V    float4 columns per thread (a chunk is BS*V float4 groups wide);
//        thread t takes groups t, t+BS, ..., so each load instruction of a
//        wavefront covers 1 KiB of contiguous row
//   U    kept rows per batch of the row loop (see add_rows for the order of its loads and adds)
//   NT   gradient rows are loaded with the non-temporal (streaming) hint
template <int BS_, int V_, int U_, bool NT_>
struct Shape {
  static constexpr int BS = BS_, V = V_, U = U_;
  static constexpr bool NT = NT_;
  __device__ static __forceinline__ int group_of(int v) { return v * BS_ + (int)threadIdx.x; }
};

constexpr int kMaxWorkers = 256;

enum Mode : int { kSgd = 0, kMomentum = 1, kRmspropMom = 2, kClipReduce = 3 };

// One segment of the gradient row: a parameter tensor (theta != null) or a gap
// between tensors (theta == null).  Segments are sorted by their first column
// and tile [col_lo, col_hi) without overlap.
struct Segment {
  float* theta;
  float* s0;
  float* s1;
  float* ema;                // moving average of theta, or null
};

// Head of the workspace.
struct WsHeader {
  int status;          // BSGD_OK or BSGD_ERR_TOO_FEW
  float t_step;        // arrival time of the N-th kept gradient
  float clip_scale;    // min(1, c/||G||)
  int n_kept;          // how many rows (messages) the step kept
  double norm;         // ||G|| before clipping
  int n_grad;          // how many worker gradients those rows hold: the divisor of the mean
};


// ---------------------------------------------------------------------------
// Arrival-order selection
// ---------------------------------------------------------------------------

// Map an fp32 arrival time to a u32 whose unsigned order is the order of the
// times: -inf < ... < -0 = +0 < ... < +inf < NaN.
__device__ __forceinline__ unsigned ordered_time_bits(float t) {
  if (t != t) return 0xFFFFFFFFu;                     // NaN: never arrives, sorts last
  if (t == 0.0f) t = 0.0f;                            // -0 and +0 are the same instant
  unsigned u = __float_as_uint(t);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

constexpr unsigned kNeverArrives = 0xFF800000u;       // ordered bits of +inf; NaN is above

// Options of the selection (all wave-uniform).
struct SelectOpts {
  const int* tags;     // step tag carried by each message, or null
  int step_tag;        // messages with another tag are dropped (Algorithm 4's tag test)
  float deadline;      // messages arriving later are dropped; +inf: none
  int n_min;           // 0: keep the first N eligible; >= 1: keep every eligible one, at least n_min
  const int* row_count;  // worker gradients each row holds, or null (one each)
  int* n_grad;           // out: worker gradients held by the kept rows, or null
};

// One wavefront.  Worker w = lane + 64*r sits in slot r of its lane; its key
// is (ordered time << 32) | w, so keys are distinct and ties in time go to
// the lower worker index.  A message that is not eligible (wrong tag, past
// the deadline, +inf or NaN time) gets the "never arrives" time.  Each key
// counts how many keys are smaller; the kept set is rank < K, where K = N, or
// the number of eligible messages in deadline mode.  Output is compacted in
// ascending worker order with ballots and prefix popcounts.
// R = slots per lane = ceil(W / 64).  DPP: the keys are passed round the
// wavefront with DPP wave rotates (no LDS, no barrier; used for W <= 64,
// where it takes the same 4.1 us inside a step as the LDS form); otherwise
// they are put in LDS and read back as broadcasts (faster from two slots per
// lane on: W = 106: 4.4 against 4.6 us, W = 256: 1.8 us less per launch).
constexpr int kFewWorkers = 24;                      // up to here the keys are broadcast one by one (see select_wave)

// What a wavefront knows once it has ranked the arrival times (all wave-uniform).
struct Selected {
  int status;                    // BSGD_OK, BSGD_ERR_TOO_FEW, or BSGD_ERR_ARG for a kept row that holds no gradient
  int n_kept;                    // rows kept (0 when too few)
  int n_grad;                    // worker gradients those rows hold
  unsigned long long mask;       // bit w: worker w is kept (workers 0..63; the whole set when W <= 64)
};

// The selection, run by one whole wavefront (any wavefront of a workgroup:
// `lane` is the lane index).  Outputs go through the pointers that are not
// null; the result is also returned, so a kernel can run it for itself.
template <int R, bool DPP>
__device__ __forceinline__ Selected select_wave(const float* __restrict__ arrival_t, int N, int W, SelectOpts o,
                                                int* __restrict__ sel_idx, int* __restrict__ n_kept,
                                                float* __restrict__ t_step, int* __restrict__ status) {
  __shared__ unsigned long long keys[DPP ? 1 : 64 * R];
  const int lane = threadIdx.x & 63;
  unsigned long long key[R];
  float tval[R];
  int eligible = 0;
#pragma unroll
  for (int r = 0; r < R; ++r) {
    const int w = lane + 64 * r;
    tval[r] = 0.0f;
    key[r] = ~0ull;                                   // padding slot: after every real key
    bool ok = false;
    if (w < W) {
      tval[r] = arrival_t[w];
      unsigned bits = ordered_time_bits(tval[r]);
      ok = bits < kNeverArrives && tval[r] <= o.deadline && (o.tags == nullptr || o.tags[w] == o.step_tag);
      if (!ok) bits = 0xFFFFFFFFu;
      key[r] = ((unsigned long long)bits << 32) | (unsigned)w;
    }
    if constexpr (!DPP) keys[w] = key[r];
    eligible += __popcll(__ballot(ok));
  }
  if constexpr (!DPP) __syncthreads();
  const int K = o.n_min > 0 ? eligible : N;            // how many are kept
  const bool too_few = o.n_min > 0 ? (eligible < o.n_min) : (eligible < N);

  // One wavefront: latency is all this kernel costs, so the broadcast reads
  // are unrolled to keep several in flight (back-to-back launches with
  // W = 106: 3.3 us each this way against 8.2 us one read at a time).
  int rank[R];
#pragma unroll
  for (int r = 0; r < R; ++r) rank[r] = 0;
  if (DPP && R == 1 && W <= kFewWorkers) {
    // A handful of workers: every real key is broadcast in turn (lane j's
    // key through a scalar register), W steps instead of 63.  The key's own
    // lane compares it with itself, which counts nothing.
    const int lo = (int)(unsigned)key[0], hi = (int)(unsigned)(key[0] >> 32);
    for (int j = 0; j < W; ++j) {
      const unsigned long long kj = ((unsigned long long)(unsigned)__builtin_amdgcn_readlane(hi, j) << 32) |
                                    (unsigned)__builtin_amdgcn_readlane(lo, j);
      rank[0] += (kj < key[0]) ? 1 : 0;
    }
  } else if constexpr (DPP) {
    // The keys travel round the wavefront one lane at a time (DPP wave rotate):
    // after 63 steps every lane has seen every other lane's keys.  Padding
    // slots hold the largest key and are never counted.
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
      for (int r2 = 0; r2 < R; ++r2)
        if (r2 != r) rank[r] += (key[r2] < key[r]) ? 1 : 0;      // the other slots of this lane
    unsigned lo[R], hi[R];
#pragma unroll
    for (int r = 0; r < R; ++r) { lo[r] = (unsigned)key[r]; hi[r] = (unsigned)(key[r] >> 32); }
#pragma unroll 7
    for (int s = 1; s < 64; ++s) {
#pragma unroll
      for (int r2 = 0; r2 < R; ++r2) {
        lo[r2] = (unsigned)__builtin_amdgcn_update_dpp(0, (int)lo[r2], 0x13C, 0xF, 0xF, false);   // wave_ror:1
        hi[r2] = (unsigned)__builtin_amdgcn_update_dpp(0, (int)hi[r2], 0x13C, 0xF, 0xF, false);
      }
#pragma unroll
      for (int r2 = 0; r2 < R; ++r2) {
        const unsigned long long kj = ((unsigned long long)hi[r2] << 32) | lo[r2];
#pragma unroll
        for (int r = 0; r < R; ++r) rank[r] += (kj < key[r]) ? 1 : 0;
      }
    }
  } else {
#pragma unroll 8
    for (int j = 0; j < W; ++j) {
      const unsigned long long kj = keys[j];            // same address in every lane: LDS broadcast
#pragma unroll
      for (int r = 0; r < R; ++r) rank[r] += (kj < key[r]) ? 1 : 0;
    }
  }

  int base = 0;
  unsigned long long first_mask = 0;
#pragma unroll
  for (int r = 0; r < R; ++r) {
    const int w = lane + 64 * r;
    const bool keep = (w < W) && (rank[r] < K);
    const unsigned long long mask = __ballot(keep);
    if (r == 0) first_mask = mask;
    const int pos = base + __builtin_amdgcn_mbcnt_hi((unsigned)(mask >> 32), __builtin_amdgcn_mbcnt_lo((unsigned)mask, 0u));
    if (keep && sel_idx) sel_idx[pos] = w;
    base += __popcll(mask);
    if ((w < W) && rank[r] == K - 1 && t_step) *t_step = tval[r];   // the last kept arrival: how long the step waited
  }
  // rows that already combine several workers' gradients: the mean divides by the gradients kept
  int held = 0, bad = 0;
#pragma unroll
  for (int r = 0; r < R; ++r) {
    const int w = lane + 64 * r;
    if ((w < W) && (rank[r] < K) && !too_few) {
      const int c = o.row_count != nullptr ? o.row_count[w] : 1;
      held += c;
      bad |= (c < 1) ? 1 : 0;
    }
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) {
    held += __shfl_xor(held, off, 64);
    bad |= __shfl_xor(bad, off, 64);
  }
  Selected out;
  out.status = too_few ? -2 : (bad ? -1 : 0);
  out.n_kept = too_few ? 0 : K;
  out.n_grad = held;
  out.mask = first_mask;
  if (lane == 0) {
    if (status) *status = out.status;
    if (n_kept) *n_kept = out.n_kept;
    if (o.n_grad) *o.n_grad = held;
  }
  return out;
}

template <int R, bool DPP>
__global__ __launch_bounds__(64) void k_select(const float* __restrict__ arrival_t, int N, int W, SelectOpts o,
                                                int* __restrict__ sel_idx, int* __restrict__ n_kept,
                                                float* __restrict__ t_step, int* __restrict__ status) {
  select_wave<R, DPP>(arrival_t, N, W, o, sel_idx, n_kept, t_step, status);
}

// The selection as part of a step's first launch (no launch of its own for
// k_select, which is a third of a small step and 4 us of a large one):
// every wavefront of that launch ranks the W <= 64 arrival times itself (DPP
// rotates or scalar broadcasts only: no LDS, no barrier, no other wavefront to
// wait for) and takes the kept rows from the resulting 64-bit mask; the first
// wavefront of the launch also publishes what k_select would have written,
// and the step's later launches (if any) read that.
struct SelectJob {
  const float* arrival_t;
  int W;
  SelectOpts opts;
  int* sel_idx;              // outputs, as k_select's
  int* n_kept;
  float* t_step;
  int* status;
};

struct StepParams {
  const float* grads;        // [(N+b) x ld]
  long long ld;
  const int* sel_idx;        // [N] ascending
  const int* status;         // may be null
  int N;
  float inv_n;
  const int* n_dev;          // when set: the number of kept rows is read from here (deadline mode)
  const int* div_dev;        // when set: the divisor of the mean is read from here (rows that hold several gradients)
  const float* row_scale;    // per kept row: its own clip scale (per-worker clipping), or null
  double* row_partials;      // [chunk][n_stride]: per chunk and kept row, sum of squares (per-worker clipping)
  int n_stride;              // rows per chunk in row_partials
  float worker_clip;         // c of the per-worker clip
  float lr, mu, rho, one_minus_rho, eps;
  float alpha, one_minus_alpha;   // decay of the moving average of theta
  // clipped steps
  float* gbar;               // mean gradient, laid out like one gradient row
  double* partials;          // one sum of squares per workgroup
  const WsHeader* header;    // clip_scale is read from here by k_apply
  // segments (tensors and gaps) in gradient-row column order
  Segment single;            // the one tensor when there is exactly one
  const Segment* table;      // [S] in the workspace; null: the launch carries its part of the table as its second argument
  const unsigned* starts;    // [S+1] first column of each segment, then the end of the last one
  int S;                     // segments in the table this launch sees
  long long col_lo, col_hi;  // columns covered by tensors: [col_lo, col_hi)
  long long base;            // col_lo rounded down to a multiple of 4: column of chunk 0
  int chunk_base;            // chunk id of workgroup 0 of this launch
  int slot_base;             // index of workgroup 0's slot in partials / row_partials (chunks that hold no tensor
                             // are not launched and have no slot)
  SelectJob job;             // kernels with SELECT: the selection is theirs to do (sel_idx, status, n_dev, div_dev unused)
};

// ---------------------------------------------------------------------------
// Tensor table
// ---------------------------------------------------------------------------
constexpr int kUploadBatch = 96;                     // 96 x 36 bytes of descriptors fit the 4 KiB argument buffer

struct UploadArgs {
  int first, count, is_last;
  unsigned end_col;
  Segment seg[kUploadBatch];
  unsigned start[kUploadBatch];
};

// Segment descriptors travel in the kernel-argument buffer, so the host array
// is consumed at launch time and no host-to-device copy has to be ordered.
__global__ __launch_bounds__(kUploadBatch) void k_upload_table(UploadArgs a, Segment* __restrict__ table,
                                                                 unsigned* __restrict__ starts, int S) {
  const int i = threadIdx.x;
  if (i < a.count) {
    table[a.first + i] = a.seg[i];
    starts[a.first + i] = a.start[i];
  }
  if (i == 0 && a.is_last) starts[S] = a.end_col;
}

// The part of the segment table one launch needs usually fits the
// kernel-argument buffer next to StepParams; then nothing is uploaded at all.
// It is the second argument of the multi-tensor kernels and is read in place,
// through the address of the argument buffer (never by name: naming it would
// make every lane copy it to private memory).
constexpr int kEmbedSegments = 88;                   // 88 x 32 + 89 x 4 = 3172 bytes; with StepParams under 4 KiB

struct EmbeddedTable {
  Segment seg[kEmbedSegments];                       // the segments the launch's columns fall into ...
  unsigned start[kEmbedSegments + 1];                // ... their first columns, then the end of the last one
};
struct NoTable { char unused; };
template <bool MULTI>
using TableArg = std::conditional_t<MULTI, EmbeddedTable, NoTable>;

// Where this launch's segment table is: in the workspace (p.table set), else
// in the argument buffer right after StepParams.
template <bool MULTI, class P>
__device__ __forceinline__ void locate_table(const P& p, const Segment*& table, const unsigned*& starts) {
  table = p.table;
  starts = p.starts;
  if constexpr (MULTI) {
    if (p.table == nullptr) {
      constexpr size_t at = (sizeof(P) + alignof(EmbeddedTable) - 1) / alignof(EmbeddedTable) * alignof(EmbeddedTable);
      const char* args = (const char*)__builtin_amdgcn_kernarg_segment_ptr();
      table = reinterpret_cast<const Segment*>(args + at + offsetof(EmbeddedTable, seg));
      starts = reinterpret_cast<const unsigned*>(args + at + offsetof(EmbeddedTable, start));
    }
  }
}

// ---------------------------------------------------------------------------
// Reduce + update
// ---------------------------------------------------------------------------
template <bool NT>
__device__ __forceinline__ f4 load_row_f4(const char* rowbase, unsigned byte_off) {
  const f4* p = reinterpret_cast<const f4*>(rowbase + (size_t)byte_off);
  if constexpr (NT) return __builtin_nontemporal_load(p);
  else return *p;
}

// Sum of the kept rows for V float4 columns per thread, rows taken in
// batches of B so that B*V 16-byte loads are in flight before the first add.
// Adds happen in ascending row order (fixed, run-to-run identical).
// acc += scale * r, spelled as one fused multiply-add per component.  With
// scale == 1 this is exactly acc + r, so the unscaled path keeps its bits.
__device__ __forceinline__ void fma4(f4& acc, float scale, const f4& r) {
  acc.x = fmaf(scale, r.x, acc.x);
  acc.y = fmaf(scale, r.y, acc.y);
  acc.z = fmaf(scale, r.z, acc.z);
  acc.w = fmaf(scale, r.w, acc.w);
}

// The order in which a batch's loads and adds are issued is fixed by hand
// (the scheduling barriers), because it decides the bandwidth: the first row
// of a batch goes out as one burst of V loads and is added as it arrives,
// the other rows follow two loads at a time, each pair added before the next
// is requested.  A thread then has V, then 2, loads in flight.  Issuing all
// B*V loads before the first add is 6 % slower on every workload (measured),
// steady pipelines of 2..8 loads per thread are 0..5 % slower; left to
// itself the compiler picks one or the other depending on the register
// pressure of the rest of the kernel.
// MASK: the kept rows are the set bits of `mask`, taken from the lowest up
// (the same ascending order as the list) and cleared as they are used.
template <int V, int B, bool NT, bool MASK>
__device__ __forceinline__ void add_rows(f4 (&acc)[V], const float* __restrict__ grads, long long ld,
                                         long long colbase, const int* __restrict__ sel_idx, unsigned long long& mask,
                                         const float* __restrict__ row_scale, int j, const unsigned (&toff)[V]) {
  const char* rowbase[B];
  float sc[B];
#pragma unroll
  for (int u = 0; u < B; ++u) {
    long long k;
    if constexpr (MASK) {
      k = __builtin_amdgcn_readfirstlane((int)__builtin_ctzll(mask));   // the mask is the same in every lane
      mask &= mask - 1;
    } else {
      k = sel_idx[j + u];
    }
    sc[u] = row_scale != nullptr ? row_scale[j + u] : 1.0f;   // per-worker clip scale (wave-uniform)
    rowbase[u] = reinterpret_cast<const char*>(grads + k * ld + colbase);
  }
  if constexpr (V >= 4 && V % 2 == 0) {
    {
      f4 r[V];
#pragma unroll
      for (int v = 0; v < V; ++v) r[v] = load_row_f4<NT>(rowbase[0], toff[v]);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int v = 0; v < V; ++v) fma4(acc[v], sc[0], r[v]);
      __builtin_amdgcn_sched_barrier(0);
    }
#pragma unroll
    for (int u = 1; u < B; ++u) {
#pragma unroll
      for (int v = 0; v < V; v += 2) {
        const f4 r0 = load_row_f4<NT>(rowbase[u], toff[v]);
        const f4 r1 = load_row_f4<NT>(rowbase[u], toff[v + 1]);
        __builtin_amdgcn_sched_barrier(0);
        fma4(acc[v], sc[u], r0);
        fma4(acc[v + 1], sc[u], r1);
        __builtin_amdgcn_sched_barrier(0);
      }
    }
  } else {
    // narrow shapes (small problems): all rows of the batch at once
    f4 r[B][V];
#pragma unroll
    for (int u = 0; u < B; ++u)
#pragma unroll
      for (int v = 0; v < V; ++v) r[u][v] = load_row_f4<NT>(rowbase[u], toff[v]);
#pragma unroll
    for (int u = 0; u < B; ++u)
#pragma unroll
      for (int v = 0; v < V; ++v) fma4(acc[v], sc[u], r[u][v]);
  }
}

// All kept rows, in batches of U (then 8, 4, 2, 1 for what is left).
template <int V, int U, bool NT, bool MASK = false>
__device__ __forceinline__ void sum_rows(f4 (&acc)[V], const float* __restrict__ grads, long long ld,
                                         long long colbase, const int* __restrict__ sel_idx, unsigned long long mask,
                                         const float* __restrict__ row_scale, int N, const unsigned (&toff)[V]) {
  int j = 0;
  for (; j + U <= N; j += U) add_rows<V, U, NT, MASK>(acc, grads, ld, colbase, sel_idx, mask, row_scale, j, toff);
  if constexpr (U > 8) { if ((N - j) & 8) { add_rows<V, 8, NT, MASK>(acc, grads, ld, colbase, sel_idx, mask, row_scale, j, toff); j += 8; } }
  if constexpr (U > 4) { if ((N - j) & 4) { add_rows<V, 4, NT, MASK>(acc, grads, ld, colbase, sel_idx, mask, row_scale, j, toff); j += 4; } }
  if constexpr (U > 2) { if ((N - j) & 2) { add_rows<V, 2, NT, MASK>(acc, grads, ld, colbase, sel_idx, mask, row_scale, j, toff); j += 2; } }
  if constexpr (U > 1) { if ((N - j) & 1) { add_rows<V, 1, NT, MASK>(acc, grads, ld, colbase, sel_idx, mask, row_scale, j, toff); j += 1; } }
}

// The library is compiled with floating-point contraction off and spells its
// fused multiply-adds out, so an element gets the same bits whichever path
// (vector or edge) and launch shape handles it.
template <int MODE>
__device__ __forceinline__ void update_elem(float g, float& th, float& a, float& b, const StepParams& p) {
  if constexpr (MODE == kSgd) {
    th = fmaf(-p.lr, g, th);
  } else if constexpr (MODE == kMomentum) {
    a = fmaf(p.mu, a, g);
    th = fmaf(-p.lr, a, th);
  } else if constexpr (MODE == kRmspropMom) {
    a = fmaf(p.rho, a, p.one_minus_rho * (g * g));
    b = fmaf(p.mu, b, (p.lr * g) / sqrtf(a + p.eps));
    th = th - b;
  }
}

// Last line of Algorithm 4: thetabar <- alpha thetabar + (1-alpha) theta(t),
// with theta(t) the value before this step's update.
__device__ __forceinline__ float ema_elem(float e, float th_before, const StepParams& p) {
  return fmaf(p.alpha, e, p.one_minus_alpha * th_before);
}
__device__ __forceinline__ void ema_vec(f4& e, const f4& th_before, const StepParams& p) {
#pragma unroll
  for (int q = 0; q < 4; ++q) e[q] = ema_elem(e[q], th_before[q], p);
}

template <int MODE>
__device__ __forceinline__ void update_vec(const f4& g, f4& th, f4& a, f4& b, const StepParams& p) {
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    float t = th[q], x = 0.f, y = 0.f;
    if constexpr (MODE >= kMomentum) x = a[q];
    if constexpr (MODE == kRmspropMom) y = b[q];
    update_elem<MODE>(g[q], t, x, y, p);
    th[q] = t;
    if constexpr (MODE >= kMomentum) a[q] = x;
    if constexpr (MODE == kRmspropMom) b[q] = y;
  }
}

__device__ __forceinline__ float wave_sum(float x) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) x += __shfl_xor(x, off, 64);
  return x;
}

// Sum over the workgroup in a fixed order; the result is valid in thread 0.
template <int BS>
__device__ __forceinline__ double block_sum(float x, float* lds) {
  x = wave_sum(x);
  const int wave = threadIdx.x >> 6;
  if ((threadIdx.x & 63) == 0) lds[wave] = x;
  __syncthreads();
  double s = 0.0;
  if (threadIdx.x == 0) {
#pragma unroll
    for (int w = 0; w < BS / 64; ++w) s += (double)lds[w];
  }
  return s;
}

// theta/state float4 at a byte address that is only known to be 4-byte
// aligned.  They are read once and written once per step, so with NT they
// are streamed like the gradient rows (measured: +2..4 % of bandwidth).
//
// The addresses are typed global-memory pointers all the way.  A pointer
// that came out of an integer, or was read from a table in memory, is
// "generic" to the compiler and is accessed with the generic instructions
// and a 64-bit address register pair per access; a wave-uniform global
// pointer plus a 32-bit lane offset needs neither (26 vector registers fewer
// in the RMSProp-mom kernel when this was introduced).  Every theta/state pointer handed to the
// library is device memory, so the cast is safe.
typedef __attribute__((address_space(1))) char gbyte;
typedef __attribute__((address_space(1))) float gfloat;
typedef __attribute__((address_space(1))) f4u gf4u;
__device__ __forceinline__ gbyte* bytes_of(float* q) { return (gbyte*)reinterpret_cast<char*>(q); }

template <bool NT>
__device__ __forceinline__ f4 load_state(const gbyte* addr) {
  const gf4u* q = (const gf4u*)addr;
  if constexpr (NT) return __builtin_nontemporal_load(q);
  else return *q;
}
template <bool NT>
__device__ __forceinline__ void store_state(const f4& v, gbyte* addr) {
  gf4u* q = (gf4u*)addr;
  if constexpr (NT) __builtin_nontemporal_store(v, q);
  else *q = v;
}

// theta/state update of the groups V0..V0+VN-1 of one chunk against ONE piece
// (a tensor's column range, given relative to the chunk's first column):
// lanes whose group lies whole inside the piece fetch theta/state together,
// update, store; `done` collects which groups were handled.  Base addresses
// are wave-uniform, lanes add their byte offset.  With kClipReduce the groups
// only add to the sum of squares.
template <int MODE, bool EMA, class S, int V0, int VN, int V>
__device__ __forceinline__ void piece_update(const f4 (&g)[V], const unsigned (&toff)[V], const bool (&valid)[V],
                                             bool all, int lo_rel, int hi_rel, gbyte* pth, gbyte* ps0,
                                             gbyte* ps1, gbyte* pe, unsigned& done, float& sumsq,
                                             const StepParams& p) {
  bool in[VN];
#pragma unroll
  for (int i = 0; i < VN; ++i) {
    const int rel = 4 * S::group_of(V0 + i);
    in[i] = all || (valid[V0 + i] && rel >= lo_rel && rel + 4 <= hi_rel);
    done |= in[i] ? (1u << (V0 + i)) : 0u;
  }
  if constexpr (MODE == kClipReduce) {
#pragma unroll
    for (int i = 0; i < VN; ++i) {
      if (in[i]) {
        const f4 x = g[V0 + i];
        sumsq = fmaf(x.x, x.x, sumsq);
        sumsq = fmaf(x.y, x.y, sumsq);
        sumsq = fmaf(x.z, x.z, sumsq);
        sumsq = fmaf(x.w, x.w, sumsq);
      }
    }
  } else {
    f4 th[VN], a[VN], b[VN], e[VN];
#pragma unroll
    for (int i = 0; i < VN; ++i) {
      if (in[i]) {
        th[i] = load_state<S::NT>(pth + toff[V0 + i]);
        if constexpr (MODE >= kMomentum) a[i] = load_state<S::NT>(ps0 + toff[V0 + i]);
        if constexpr (MODE == kRmspropMom) b[i] = load_state<S::NT>(ps1 + toff[V0 + i]);
        if constexpr (EMA) e[i] = load_state<S::NT>(pe + toff[V0 + i]);
      }
    }
#pragma unroll
    for (int i = 0; i < VN; ++i) {
      if (in[i]) {
        if constexpr (EMA) {
          ema_vec(e[i], th[i], p);
          store_state<S::NT>(e[i], pe + toff[V0 + i]);
        }
        update_vec<MODE>(g[V0 + i], th[i], a[i], b[i], p);
        store_state<S::NT>(th[i], pth + toff[V0 + i]);
        if constexpr (MODE >= kMomentum) store_state<S::NT>(a[i], ps0 + toff[V0 + i]);
        if constexpr (MODE == kRmspropMom) store_state<S::NT>(b[i], ps1 + toff[V0 + i]);
      }
    }
  }
}

// Which segment holds column x: the last j with starts[j] <= x.  Requires
// starts[0] <= x < starts[S].
__device__ __forceinline__ int find_segment(const unsigned* starts, int S, unsigned x) {
  int lo = 0, hi = S;                                 // invariant: starts[lo] <= x < starts[hi]
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (starts[mid] <= x) lo = mid; else hi = mid;
  }
  return lo;
}

// SRC_ROWS: the gradient comes from summing the kept rows (MODE 0..2 updates
// directly; MODE kClipReduce stores the mean and a per-chunk sum of squares).
// !SRC_ROWS: the gradient is the stored mean times the clip scale (MODE 0..2).
//
// Work is cut in the column space of a gradient row, not per tensor: chunk c
// covers the BS*V float4 groups starting at column base + c*4*BS*V.  Every
// chunk is full width whatever the tensor sizes are, row loads are always
// aligned 16-byte groups, and small tensors share chunks.  theta/state are
// found through the sorted segment table: a chunk lying inside one tensor
// (nearly all of them) takes the uniform path with wave-uniform pointers and
// float4 accesses (4-byte aligned only, since a tensor may start anywhere in
// the row); a chunk holding a tensor boundary looks segments up per lane.
// SELECT (with SRC_ROWS): the launch is a step's first and does the selection itself, see SelectJob.
template <int MODE, class S, bool MULTI, bool SRC_ROWS, bool EMA, bool SELECT = false>
__global__ __launch_bounds__(S::BS) void k_step(StepParams p, TableArg<MULTI>) {
  static_assert(!SELECT || SRC_ROWS, "only a pass over the gradient rows can do the selection");
  constexpr int BS = S::BS, V = S::V, U = S::U;
  constexpr bool NT = S::NT;
  constexpr long long CH = 4LL * BS * V;               // columns per chunk
  extern __shared__ unsigned starts_lds[];             // MULTI: starts[S+1]
  __shared__ float red_lds[BS / 64];

  int n_rows;
  float inv_n;
  unsigned long long row_mask = 0;
  if constexpr (SELECT) {
    const bool publish = blockIdx.x == 0 && threadIdx.x < 64;   // one wavefront of the launch writes the outputs
    SelectOpts o = p.job.opts;
    if (!publish) o.n_grad = nullptr;
    const Selected sel = select_wave<1, true>(p.job.arrival_t, p.N, p.job.W, o, publish ? p.job.sel_idx : nullptr,
                                              publish ? p.job.n_kept : nullptr, publish ? p.job.t_step : nullptr,
                                              publish ? p.job.status : nullptr);
    if (sel.status != 0) return;                      // too few arrivals: touch nothing
    row_mask = sel.mask;
    n_rows = sel.n_kept;
    inv_n = o.row_count != nullptr ? 1.0f / (float)sel.n_grad : (o.n_min > 0 ? 1.0f / (float)n_rows : p.inv_n);
  } else {
    if (p.status != nullptr && *p.status != 0) return;  // too few arrivals: touch nothing
    n_rows = p.n_dev != nullptr ? *p.n_dev : p.N;
    inv_n = p.div_dev != nullptr ? 1.0f / (float)*p.div_dev : (p.n_dev != nullptr ? 1.0f / (float)n_rows : p.inv_n);
  }

  const Segment* table;
  const unsigned* starts;
  locate_table<MULTI>(p, table, starts);
  if constexpr (MULTI) {
    for (int i = threadIdx.x; i <= p.S; i += BS) starts_lds[i] = starts[i];
    __syncthreads();
  }
  const long long span_end4 = (p.col_hi + 3) & ~3LL;   // rows are readable up to here (<= ld)

  {
    const int chunk_id = (int)blockIdx.x + p.chunk_base;   // one chunk per workgroup
    const long long c0 = p.base + (long long)chunk_id * CH;   // first column of the chunk, multiple of 4

    // the segment holding the chunk's first column (clamped into the covered range)
    Segment seg;
    long long seg_start, seg_end;
    int j0 = 0;
    if constexpr (MULTI) {
      const long long x = c0 < p.col_lo ? p.col_lo : c0;
      j0 = __builtin_amdgcn_readfirstlane(find_segment(starts_lds, p.S, (unsigned)x));
      seg_start = (long long)(unsigned)__builtin_amdgcn_readfirstlane((int)starts_lds[j0]);
      seg_end = (long long)(unsigned)__builtin_amdgcn_readfirstlane((int)starts_lds[j0 + 1]);
      seg = table[j0];
    } else {
      seg_start = p.col_lo;
      seg_end = p.col_hi;
      seg = p.single;
    }
    const bool uniform = (c0 >= seg_start) && (c0 + CH <= seg_end) && (seg.theta != nullptr);

    // A chunk that lies wholly in a gap between tensors (a partial-range update
    // names only some layers) has nothing to do: no row of it is read.  Gaps
    // and tensors alternate in the table, so the chunk holds a tensor unless
    // its first piece is a gap and also its last one.
    if constexpr (MULTI) {
      if (seg.theta == nullptr) {
        long long last = c0 + CH - 1;
        if (last >= p.col_hi) last = p.col_hi - 1;
        if (last < p.col_lo) last = p.col_lo;
        if (__builtin_amdgcn_readfirstlane(find_segment(starts_lds, p.S, (unsigned)last)) == j0) {
          if constexpr (MODE == kClipReduce) {
            if (threadIdx.x == 0) p.partials[(int)blockIdx.x + p.slot_base] = 0.0;
          }
          return;
        }
      }
    }

    float scale = 1.0f;
    if constexpr (!SRC_ROWS) scale = p.header->clip_scale;
    float sumsq = 0.0f;

    // Lanes whose group starts past the readable end of the row (only in the
    // last chunk) re-read the chunk's first group and take no further part.
    unsigned toff[V];
    bool valid[V];
#pragma unroll
    for (int v = 0; v < V; ++v) {
      const int g = S::group_of(v);
      valid[v] = uniform || (c0 + 4LL * g < span_end4);
      toff[v] = valid[v] ? (unsigned)g * 16u : 0u;
    }

    f4 g[V];
    if constexpr (SRC_ROWS) {
#pragma unroll
      for (int v = 0; v < V; ++v) g[v] = f4{0.f, 0.f, 0.f, 0.f};
      sum_rows<V, U, NT, SELECT>(g, p.grads, p.ld, c0, p.sel_idx, row_mask, p.row_scale, n_rows, toff);
#pragma unroll
      for (int v = 0; v < V; ++v) g[v] *= inv_n;
    } else {
#pragma unroll
      for (int v = 0; v < V; ++v)
        g[v] = load_state<NT>(bytes_of(p.gbar + c0) + toff[v]) * scale;
    }

    // The segments ("pieces") the chunk's covered columns fall into: j0..j1.
    int j1 = j0;
    if constexpr (MULTI) {
      if (!uniform) {
        long long last = c0 + CH - 1;
        if (last >= p.col_hi) last = p.col_hi - 1;
        if (last < p.col_lo) last = p.col_lo;
        j1 = __builtin_amdgcn_readfirstlane(find_segment(starts_lds, p.S, (unsigned)last));
      }
    }

    if constexpr (MODE == kClipReduce) {
      // the stored mean is laid out like a row: whole groups, gaps included
#pragma unroll
      for (int v = 0; v < V; ++v)
        if (valid[v]) store_state<NT>(g[v], bytes_of(p.gbar + c0) + toff[v]);
    }

    unsigned done = 0;                                 // bit v: group v was handled as a whole by some piece
    if (uniform) {
      // ---- the chunk lies inside one tensor (almost always): every lane, all groups at once ---
      const long long e_bytes = (c0 - seg_start) * 4;
      piece_update<MODE, EMA, S, 0, V>(g, toff, valid, true, 0, 0, bytes_of(seg.theta) + e_bytes, bytes_of(seg.s0) + e_bytes,
                                       bytes_of(seg.s1) + e_bytes, bytes_of(seg.ema) + e_bytes, done, sumsq, p);
    } else {
      // ---- the chunk holds tensor boundaries, gaps or the end of the row -------------------
      // Every group lies in at most one piece, so the pieces' loads can share
      // one set of registers (different lanes): first all pieces fetch
      // theta/state for the lanes they own, then everything is updated once,
      // then all pieces store.  Groups go in two halves to bound registers.
      auto piece = [&](int pj, Segment& sg, int& lo_rel, int& hi_rel, long long& e_bytes) {
        sg = seg;
        long long lo = seg_start, hi = seg_end;
        if constexpr (MULTI) {
          if (pj != j0) {
            sg = table[pj];
            lo = (long long)(unsigned)__builtin_amdgcn_readfirstlane((int)starts_lds[pj]);
            hi = (long long)(unsigned)__builtin_amdgcn_readfirstlane((int)starts_lds[pj + 1]);
          }
        }
        // the piece in columns relative to the chunk's first one (fits 32 bits once clamped)
        const long long lo_c = lo - c0, hi_c = hi - c0;
        lo_rel = lo_c < -8 ? -8 : (int)lo_c;
        hi_rel = hi_c > CH + 8 ? (int)(CH + 8) : (int)hi_c;
        e_bytes = (c0 - lo) * 4;                     // byte offset of the piece's (virtual) element at column c0
      };
      constexpr int H = V;                             // groups per pass of the piece loops
#pragma unroll
      for (int v0 = 0; v0 < V; v0 += H) {
        f4 th[H], a[H], b[H], e[H];
        if constexpr (MODE != kClipReduce) {
#pragma unroll 1
          for (int pj = j0; pj <= j1; ++pj) {
            Segment sg; int lo_rel, hi_rel; long long e_bytes;
            piece(pj, sg, lo_rel, hi_rel, e_bytes);
            if (sg.theta == nullptr) continue;         // a gap
#pragma unroll
            for (int i = 0; i < H; ++i) {
              const int rel = 4 * S::group_of(v0 + i);
              if (valid[v0 + i] && rel >= lo_rel && rel + 4 <= hi_rel) {
                th[i] = *(const gf4u*)(bytes_of(sg.theta) + (e_bytes + (long long)toff[v0 + i]));
                if constexpr (MODE >= kMomentum) a[i] = *(const gf4u*)(bytes_of(sg.s0) + (e_bytes + (long long)toff[v0 + i]));
                if constexpr (MODE == kRmspropMom) b[i] = *(const gf4u*)(bytes_of(sg.s1) + (e_bytes + (long long)toff[v0 + i]));
                if constexpr (EMA) e[i] = *(const gf4u*)(bytes_of(sg.ema) + (e_bytes + (long long)toff[v0 + i]));
              }
            }
          }
#pragma unroll
          for (int i = 0; i < H; ++i) {                // lanes that own nothing: not stored
            if constexpr (EMA) ema_vec(e[i], th[i], p);
            update_vec<MODE>(g[v0 + i], th[i], a[i], b[i], p);
          }
        }
#pragma unroll 1
        for (int pj = j0; pj <= j1; ++pj) {
          Segment sg; int lo_rel, hi_rel; long long e_bytes;
          piece(pj, sg, lo_rel, hi_rel, e_bytes);
          if (sg.theta == nullptr) continue;           // a gap
#pragma unroll
          for (int i = 0; i < H; ++i) {
            const int rel = 4 * S::group_of(v0 + i);
            if (valid[v0 + i] && rel >= lo_rel && rel + 4 <= hi_rel) {
              done |= 1u << (v0 + i);
              if constexpr (MODE == kClipReduce) {
                const f4 x = g[v0 + i];
                sumsq = fmaf(x.x, x.x, sumsq);
                sumsq = fmaf(x.y, x.y, sumsq);
                sumsq = fmaf(x.z, x.z, sumsq);
                sumsq = fmaf(x.w, x.w, sumsq);
              } else {
                *(gf4u*)(bytes_of(sg.theta) + (e_bytes + (long long)toff[v0 + i])) = th[i];
                if constexpr (MODE >= kMomentum) *(gf4u*)(bytes_of(sg.s0) + (e_bytes + (long long)toff[v0 + i])) = a[i];
                if constexpr (MODE == kRmspropMom) *(gf4u*)(bytes_of(sg.s1) + (e_bytes + (long long)toff[v0 + i])) = b[i];
                if constexpr (EMA) *(gf4u*)(bytes_of(sg.ema) + (e_bytes + (long long)toff[v0 + i])) = e[i];
              }
            }
          }
        }
      }
      // Groups cut by a piece boundary (or lying in a gap), one per boundary
      // that is not a multiple of 4: element by element, but with the four
      // elements' look-ups, loads and stores each issued together.
#pragma unroll
      for (int v = 0; v < V; ++v) {
        const long long gcol = c0 + 4LL * S::group_of(v);
        if (((done >> v) & 1u) || !valid[v] || gcol + 4 <= p.col_lo || gcol >= p.col_hi) continue;
        bool ok[4];
        int jq[4];
        long long first_col[4];
        int j = j0;
        long long s_start = seg_start, s_end = seg_end;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const long long col = gcol + q;
          ok[q] = col >= p.col_lo && col < p.col_hi;
          if constexpr (MULTI) {
            if (ok[q]) {
              while (col >= s_end) {                   // walk the start columns on from the chunk's first piece
                ++j;
                s_start = s_end;
                s_end = starts_lds[j + 1];
              }
            }
          }
          jq[q] = j;
          first_col[q] = s_start;
        }
        Segment sq[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          sq[q] = seg;
          if constexpr (MULTI) {
            if (ok[q]) sq[q] = table[jq[q]];
          }
          ok[q] = ok[q] && sq[q].theta != nullptr;     // else: a gap
        }
        if constexpr (MODE == kClipReduce) {
#pragma unroll
          for (int q = 0; q < 4; ++q)
            if (ok[q]) sumsq = fmaf(g[v][q], g[v][q], sumsq);
        } else {
          float t1[4], a1[4], b1[4], e1[4];
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            t1[q] = a1[q] = b1[q] = e1[q] = 0.f;
            if (ok[q]) {
              const long long e = gcol + q - first_col[q];
              t1[q] = sq[q].theta[e];
              if constexpr (MODE >= kMomentum) a1[q] = sq[q].s0[e];
              if constexpr (MODE == kRmspropMom) b1[q] = sq[q].s1[e];
              if constexpr (EMA) e1[q] = sq[q].ema[e];
            }
          }
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            if (ok[q]) {
              const long long e = gcol + q - first_col[q];
              if constexpr (EMA) sq[q].ema[e] = ema_elem(e1[q], t1[q], p);
              update_elem<MODE>(g[v][q], t1[q], a1[q], b1[q], p);
              sq[q].theta[e] = t1[q];
              if constexpr (MODE >= kMomentum) sq[q].s0[e] = a1[q];
              if constexpr (MODE == kRmspropMom) sq[q].s1[e] = b1[q];
            }
          }
        }
      }
    }

    if constexpr (MODE == kClipReduce) {
      const double s = block_sum<BS>(sumsq, red_lds);
      if (threadIdx.x == 0) p.partials[(int)blockIdx.x + p.slot_base] = s;
    }
  }
}

// Per-worker clipping (Appendix A.3 as printed), pass A: for this chunk and
// every kept row, the sum of squares of the row's elements that belong to a
// tensor.  Same chunking and row order as k_step; rows are read U at a time.
// Output: row_partials[chunk][row] (fp64), reduced in a fixed order.
template <class S, bool MULTI>
__global__ __launch_bounds__(S::BS) void k_row_sumsq(StepParams p, TableArg<MULTI>) {
  constexpr int BS = S::BS, V = S::V, U = S::U;
  constexpr bool NT = S::NT;
  constexpr long long CH = 4LL * BS * V;
  constexpr int WAVES = BS / 64;
  extern __shared__ unsigned starts_lds[];             // MULTI: starts[S+1]
  __shared__ float wave_part[kMaxWorkers][WAVES];

  if (p.status != nullptr && *p.status != 0) return;
  const int n_rows = p.n_dev != nullptr ? *p.n_dev : p.N;
  const Segment* table;
  const unsigned* starts;
  locate_table<MULTI>(p, table, starts);
  if constexpr (MULTI) {
    for (int i = threadIdx.x; i <= p.S; i += BS) starts_lds[i] = starts[i];
    __syncthreads();
  }
  const long long span_end4 = (p.col_hi + 3) & ~3LL;
  const int chunk_id = (int)blockIdx.x + p.chunk_base;
  const long long c0 = p.base + (long long)chunk_id * CH;

  // which of a lane's elements belong to a tensor: 4 bits per group
  unsigned toff[V];
  unsigned member[V];
#pragma unroll
  for (int v = 0; v < V; ++v) {
    const long long gcol = c0 + 4LL * S::group_of(v);
    toff[v] = gcol < span_end4 ? (unsigned)S::group_of(v) * 16u : 0u;
    member[v] = 0;
  }
  {
    int j0 = 0, j1 = 0;
    if constexpr (MULTI) {
      long long first = c0 < p.col_lo ? p.col_lo : c0;
      long long last = c0 + CH - 1;
      if (last >= p.col_hi) last = p.col_hi - 1;
      if (last < first) last = first;
      j0 = __builtin_amdgcn_readfirstlane(find_segment(starts_lds, p.S, (unsigned)first));
      j1 = __builtin_amdgcn_readfirstlane(find_segment(starts_lds, p.S, (unsigned)last));
    }
#pragma unroll 1
    for (int pj = j0; pj <= j1; ++pj) {
      long long lo = p.col_lo, hi = p.col_hi;
      bool real = true;
      if constexpr (MULTI) {
        lo = (long long)(unsigned)__builtin_amdgcn_readfirstlane((int)starts_lds[pj]);
        hi = (long long)(unsigned)__builtin_amdgcn_readfirstlane((int)starts_lds[pj + 1]);
        real = table[pj].theta != nullptr;
      }
      if (!real) continue;
      const long long lo_c = lo - c0, hi_c = hi - c0;
      const int lo_rel = lo_c < -8 ? -8 : (int)lo_c;
      const int hi_rel = hi_c > CH + 8 ? (int)(CH + 8) : (int)hi_c;
#pragma unroll
      for (int v = 0; v < V; ++v) {
        const int rel = 4 * S::group_of(v);
#pragma unroll
        for (int q = 0; q < 4; ++q)
          if (rel + q >= lo_rel && rel + q < hi_rel) member[v] |= 1u << q;
      }
    }
  }

  const int slot = (int)blockIdx.x + p.slot_base;
  {
    // a chunk that holds no tensor column adds nothing to any norm: its rows are not read
    unsigned any = 0;
#pragma unroll
    for (int v = 0; v < V; ++v) any |= member[v];
    if (!__syncthreads_or((int)any)) {
      for (int row = threadIdx.x; row < n_rows; row += BS) p.row_partials[(long long)slot * p.n_stride + row] = 0.0;
      return;
    }
  }
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  for (int j = 0; j < n_rows; j += U) {
    f4 r[U][V];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int jj = j + u < n_rows ? j + u : n_rows - 1;        // a short last batch re-reads the last row
      const long long k = p.sel_idx[jj];
      const char* rowbase = reinterpret_cast<const char*>(p.grads + k * p.ld + c0);
#pragma unroll
      for (int v = 0; v < V; ++v) r[u][v] = load_row_f4<NT>(rowbase, toff[v]);
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      float sq = 0.f;
#pragma unroll
      for (int v = 0; v < V; ++v) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const float x = ((member[v] >> q) & 1u) ? r[u][v][q] : 0.f;
          sq = fmaf(x, x, sq);
        }
      }
      sq = wave_sum(sq);
      if (lane == 0 && j + u < n_rows) wave_part[j + u][wave] = sq;
    }
  }
  __syncthreads();
  for (int row = threadIdx.x; row < n_rows; row += BS) {
    double s = 0.0;
#pragma unroll
    for (int w = 0; w < WAVES; ++w) s += (double)wave_part[row][w];
    p.row_partials[(long long)slot * p.n_stride + row] = s;
  }
}

// Per-worker clipping, pass B: workgroup `row` adds its row's per-chunk sums
// in a fixed order (fp64) and writes scale = min(1, c/norm) for that row.
constexpr int kRowScaleBlock = 256;
__global__ __launch_bounds__(kRowScaleBlock) void k_row_scales(const double* __restrict__ row_partials, int chunks,
                                                                int n_stride, int N, const int* __restrict__ n_dev,
                                                                float c, const int* __restrict__ status,
                                                                float* __restrict__ row_scale) {
  __shared__ double red[kRowScaleBlock];
  if (status != nullptr && *status != 0) return;
  const int n_rows = n_dev != nullptr ? *n_dev : N;
  const int row = blockIdx.x;
  if (row >= n_rows) return;
  double s = 0.0;                                   // added in index order; a batch's loads go out together
  for (int i0 = threadIdx.x; i0 < chunks; i0 += 8 * kRowScaleBlock) {
    double x[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const int i = i0 + u * kRowScaleBlock;
      x[u] = i < chunks ? row_partials[(long long)i * n_stride + row] : 0.0;
    }
#pragma unroll
    for (int u = 0; u < 8; ++u) s += x[u];
  }
  red[threadIdx.x] = s;
  __syncthreads();
  for (int half = kRowScaleBlock / 2; half > 0; half >>= 1) {
    if (threadIdx.x < half) red[threadIdx.x] += red[threadIdx.x + half];
    __syncthreads();
  }
  if (threadIdx.x == 0) {
    const double nrm = sqrt(red[0]);
    row_scale[row] = (nrm <= (double)c) ? 1.0f : (float)((double)c / nrm);
  }
}

// One workgroup adds the per-block sums of squares in a fixed order (fp64),
// takes the root and writes norm and scale = min(1, c/norm) to the header.
constexpr int kFinalizeBlock = 1024;
__global__ __launch_bounds__(kFinalizeBlock) void k_finalize_norm(const double* __restrict__ partials, int n,
                                                                   float c, const int* __restrict__ status,
                                                                   WsHeader* __restrict__ header) {
  __shared__ double red[kFinalizeBlock];
  if (status != nullptr && *status != 0) return;
  // a thread's partials are added in index order; the loads of a batch go out together (one round trip per
  // 8 instead of one each: the kernel is nothing but latency)
  double s = 0.0;
  for (int i0 = threadIdx.x; i0 < n; i0 += 8 * kFinalizeBlock) {
    double x[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const int i = i0 + u * kFinalizeBlock;
      x[u] = i < n ? partials[i] : 0.0;
    }
#pragma unroll
    for (int u = 0; u < 8; ++u) s += x[u];
  }
  red[threadIdx.x] = s;
  __syncthreads();
  for (int half = kFinalizeBlock / 2; half > 0; half >>= 1) {
    if (threadIdx.x < half) red[threadIdx.x] += red[threadIdx.x + half];
    __syncthreads();
  }
  if (threadIdx.x == 0) {
    const double nrm = sqrt(red[0]);
    header->norm = nrm;
    header->clip_scale = (nrm <= (double)c) ? 1.0f : (float)((double)c / nrm);
  }
}

// ---------------------------------------------------------------------------
// Sec. 6: one message per machine (sum of the gradients of its workers)
// ---------------------------------------------------------------------------
struct CombineParams {
  const float* grads;        // [W x ld]
  long long ld;
  float* combined;           // [M x ld_out]
  long long ld_out;
  long long cols4;           // gradient length rounded up to a multiple of 4
  int M;
  unsigned char first[kMaxWorkers + 1];   // first row of each machine, then W (W <= 256 needs 9 bits: see last)
  int last;                  // W
};

// Workgroup (chunk, machine): adds the machine's rows over one chunk of
// columns, same chunking, row order and load shape as k_step's row loop.
template <class S>
__global__ __launch_bounds__(S::BS) void k_precombine(CombineParams p) {
  constexpr int BS = S::BS, V = S::V, U = S::U;
  constexpr bool NT = S::NT;
  constexpr long long CH = 4LL * BS * V;
  const int m = blockIdx.y;
  const long long c0 = (long long)blockIdx.x * CH;
  const int r0 = p.first[m];
  const int r1 = (m + 1 == p.M) ? p.last : (int)p.first[m + 1];
  unsigned toff[V];
  bool valid[V];
#pragma unroll
  for (int v = 0; v < V; ++v) {
    const int g = S::group_of(v);
    valid[v] = c0 + 4LL * g < p.cols4;
    toff[v] = valid[v] ? (unsigned)g * 16u : 0u;
  }
  f4 acc[V];
#pragma unroll
  for (int v = 0; v < V; ++v) acc[v] = f4{0.f, 0.f, 0.f, 0.f};
  for (int j = r0; j < r1; j += U) {
    f4 r[U][V];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      if (j + u < r1) {                               // wave-uniform: a machine's rows are the same for every lane
        const char* rowbase = reinterpret_cast<const char*>(p.grads + (long long)(j + u) * p.ld + c0);
#pragma unroll
        for (int v = 0; v < V; ++v) r[u][v] = load_row_f4<NT>(rowbase, toff[v]);
      }
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      if (j + u < r1) {
#pragma unroll
        for (int v = 0; v < V; ++v) acc[v] += r[u][v];
      }
    }
  }
  float* out = p.combined + (long long)m * p.ld_out + c0;
#pragma unroll
  for (int v = 0; v < V; ++v)
    if (valid[v]) store_state<NT>(acc[v], bytes_of(out) + toff[v]);
}

// One wavefront: machine m's message leaves with its last worker.
__global__ __launch_bounds__(64) void k_machine_arrival(const float* __restrict__ arrival_t, CombineParams p,
                                                         float* __restrict__ arrival_m, int* __restrict__ row_count) {
  for (int m = threadIdx.x; m < p.M; m += 64) {
    const int r0 = p.first[m];
    const int r1 = (m + 1 == p.M) ? p.last : (int)p.first[m + 1];
    float latest = -INFINITY;
    for (int w = r0; w < r1; ++w) {
      const float t = arrival_t[w];
      latest = (t != t) ? INFINITY : (t > latest ? t : latest);   // NaN: never finishes
      if (latest == INFINITY) break;
    }
    arrival_m[m] = latest;
    row_count[m] = r1 - r0;
  }
}

// ---------------------------------------------------------------------------
// Straggler analysis (Sec. 3.1): time to collect k gradients
// ---------------------------------------------------------------------------
constexpr int kStragglerBlock = 256;                 // 4 wavefronts; a wavefront takes whole iterations
constexpr int kStragglerWaves = kStragglerBlock / 64;
constexpr int kStragglerSlab = 64;                   // iterations per workgroup

// Each wavefront ranks one iteration's W arrival times the way k_select does
// (distinct 64-bit keys, every key counts the keys below it), writes the
// times in rank order and adds them, by rank, to its own fp64 sums in LDS.
// The workgroup's sums go to partial[workgroup][W] in a fixed order.
// R = slots per lane = ceil(W / 64).
template <int R>
__global__ __launch_bounds__(kStragglerBlock) void k_kth_times(const float* __restrict__ arrival_t, int W, long long B,
                                                                float* __restrict__ kth_time,
                                                                double* __restrict__ partial) {
  __shared__ unsigned long long keys[kStragglerWaves][64 * R];
  __shared__ double acc[kStragglerWaves][64 * R];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
  for (int r = 0; r < R; ++r) acc[wave][lane + 64 * r] = 0.0;
  const long long i0 = (long long)blockIdx.x * kStragglerSlab;

  for (int s = wave; s < kStragglerSlab; s += kStragglerWaves) {   // same trip count in every wavefront
    const long long i = i0 + s;
    const bool active = i < B;
    unsigned long long key[R];
    float tval[R];
#pragma unroll
    for (int r = 0; r < R; ++r) {
      const int w = lane + 64 * r;
      key[r] = ~0ull;                                 // padding: after every real key
      tval[r] = INFINITY;
      if (active && w < W) {
        const float t = arrival_t[i * W + w];
        const unsigned bits = ordered_time_bits(t);
        if (bits < kNeverArrives) tval[r] = t;        // else: never arrives, reported as +inf
        key[r] = ((unsigned long long)bits << 32) | (unsigned)w;
      }
      keys[wave][w] = key[r];
    }
    __syncthreads();
    int rank[R];
#pragma unroll
    for (int r = 0; r < R; ++r) rank[r] = 0;
    if (active) {
#pragma unroll 8
      for (int j = 0; j < W; ++j) {
        const unsigned long long kj = keys[wave][j];  // LDS broadcast
#pragma unroll
        for (int r = 0; r < R; ++r) rank[r] += (kj < key[r]) ? 1 : 0;
      }
#pragma unroll
      for (int r = 0; r < R; ++r) {
        if (lane + 64 * r < W) {                      // ranks of real keys are 0..W-1, each taken once
          if (kth_time != nullptr) kth_time[i * W + rank[r]] = tval[r];
          acc[wave][rank[r]] += (double)tval[r];
        }
      }
    }
    __syncthreads();
  }
  if (partial != nullptr) {
    for (int r = threadIdx.x; r < W; r += kStragglerBlock) {
      double sum = acc[0][r];
#pragma unroll
      for (int w = 1; w < kStragglerWaves; ++w) sum += acc[w][r];
      partial[(long long)blockIdx.x * W + r] = sum;
    }
  }
}

// Workgroup k adds column k of partial[slabs][W] in a fixed order and divides by B.
constexpr int kMeanBlock = 256;
__global__ __launch_bounds__(kMeanBlock) void k_mean_kth(const double* __restrict__ partial, long long slabs, int W,
                                                          long long B, double* __restrict__ mean_kth) {
  __shared__ double red[kMeanBlock];
  const int k = blockIdx.x;
  double sum = 0.0;
  for (long long g = threadIdx.x; g < slabs; g += kMeanBlock) sum += partial[g * W + k];
  red[threadIdx.x] = sum;
  __syncthreads();
  for (int half = kMeanBlock / 2; half > 0; half >>= 1) {
    if ((int)threadIdx.x < half) red[threadIdx.x] += red[threadIdx.x + half];
    __syncthreads();
  }
  if (threadIdx.x == 0) mean_kth[k] = red[0] / (double)B;
}

// Plain 16-byte-per-thread copy with a known byte count: the yardstick the
// profiler's HBM read/write counters are scaled against.
__global__ __launch_bounds__(256) void k_calibration_copy(const f4* __restrict__ src, f4* __restrict__ dst, long long n16) {
  const long long i = (long long)blockIdx.x * 256 + threadIdx.x;
  if (i < n16) dst[i] = src[i];
}

// Plain streaming kernel with a chosen mix of streams: reads n_read buffers,
// writes n_write buffers (a written buffer may be one of those read: in-place,
// like theta and state), V 16-byte groups per thread laid out like a k_step
// chunk, streaming hints on every access.  It does nothing else, so its
// bandwidth is what the memory system gives a kernel with that mix: the
// yardstick the step's passes are held against.
constexpr int kYardMaxStreams = 4;
struct YardArgs {
  const f4* rd[kYardMaxStreams];
  f4* wr[kYardMaxStreams];
  int n_read, n_write;
  long long n16;             // 16-byte groups per stream
};

template <int V, int R, int Wn>
__global__ __launch_bounds__(256) void k_yardstick(YardArgs a) {
  const long long base = (long long)blockIdx.x * (256LL * V) + threadIdx.x;
  f4 x[R][V];
#pragma unroll
  for (int s = 0; s < R; ++s)
#pragma unroll
    for (int v = 0; v < V; ++v) {
      const long long i = base + v * 256LL;
      x[s][v] = f4{0.f, 0.f, 0.f, 0.f};
      if (i < a.n16) x[s][v] = __builtin_nontemporal_load(a.rd[s] + i);
    }
  f4 y[V];
#pragma unroll
  for (int v = 0; v < V; ++v) {
    y[v] = x[0][v];
#pragma unroll
    for (int s = 1; s < R; ++s) y[v] = y[v] * 0.5f + x[s][v];
  }
  if constexpr (Wn == 0) {
    // read-only mix: the loads must stay alive, but nothing is written (finite inputs never add up to this pattern)
    float t = 0.f;
#pragma unroll
    for (int v = 0; v < V; ++v) t += y[v].x + y[v].y + y[v].z + y[v].w;
    if (__float_as_uint(t) == 0x7fc12345u && a.wr[0] != nullptr) a.wr[0][0] = y[0];
  }
#pragma unroll
  for (int s = 0; s < Wn; ++s)
#pragma unroll
    for (int v = 0; v < V; ++v) {
      const long long i = base + v * 256LL;
      if (i < a.n16) __builtin_nontemporal_store(y[v] + (float)s, a.wr[s] + i);
    }
}

}  // namespace bsgd
