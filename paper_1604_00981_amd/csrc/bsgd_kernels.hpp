// Device code for the backup-worker Sync-SGD step on gfx950 (CDNA4).
//
// Three pieces, all bandwidth- or latency-bound (no dense contraction, so no
// MFMA):
//   k_select         one wavefront ranks the N+b arrival times and writes the
//                    kept set (Algorithm 4, collect loop).
//   k_reduce_update  one streaming pass: gather-sum of the N kept gradient
//                    rows in registers, mean, fused optimizer update
//                    (Algorithm 4, update line; Sec. 3 "Sync-Opt").
//   k_finalize_norm / k_apply   the second half of a clipped step (global-norm
//                    clipping as in Appendix A.3): reduce the per-block sums
//                    of squares, then scale the stored mean and update.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace bsgd {

typedef float f4 __attribute__((ext_vector_type(4)));
typedef f4 f4u __attribute__((aligned(4)));          // float4 that is only 4-byte aligned

// Launch shape of the reduce/update kernel.
//   BS   threads per workgroup
//   V    float4 columns per thread (a chunk is BS*V float4 groups wide);
//        thread t takes groups t, t+BS, ..., so each load instruction of a
//        wavefront covers 1 KiB of contiguous row
//   U    kept rows loaded per batch before the first add
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
};

// Head of the workspace.
struct WsHeader {
  int status;          // BSGD_OK or BSGD_ERR_TOO_FEW
  float t_step;        // arrival time of the N-th kept gradient
  float clip_scale;    // min(1, c/||G||)
  int pad;
  double norm;         // ||G|| before clipping
};

struct StepParams {
  const float* grads;        // [(N+b) x ld]
  long long ld;
  const int* sel_idx;        // [N] ascending
  const int* status;         // may be null
  int N;
  float inv_n;
  float lr, mu, rho, one_minus_rho, eps;
  // clipped steps
  float* gbar;               // mean gradient, laid out like one gradient row
  double* partials;          // one sum of squares per workgroup
  const WsHeader* header;    // clip_scale is read from here by k_apply
  // segments (tensors and gaps) in gradient-row column order
  Segment single;            // the one tensor when there is exactly one
  const Segment* table;      // [S]
  const unsigned* starts;    // [S+1] first column of each segment, then col_hi
  int S;
  long long col_lo, col_hi;  // columns covered by tensors: [col_lo, col_hi)
  long long base;            // col_lo rounded down to a multiple of 4: column of chunk 0
  int chunk_base;            // chunk id of workgroup 0 of this launch
  int chunk_end;             // one past the last chunk this launch covers
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

// One wavefront.  Worker w = lane + 64*r sits in slot r of its lane; its key
// is (ordered time << 32) | w, so keys are distinct and ties in time go to
// the lower worker index.  Each key counts how many keys are smaller; the
// kept set is rank < N.  Output is compacted in ascending worker order with
// ballots and prefix popcounts.
__global__ __launch_bounds__(64) void k_select(const float* __restrict__ arrival_t, int N, int W,
                                                int* __restrict__ sel_idx, float* __restrict__ t_step,
                                                int* __restrict__ status) {
  __shared__ unsigned long long keys[kMaxWorkers];
  const int lane = threadIdx.x;
  constexpr int R = kMaxWorkers / 64;
  unsigned long long key[R];
  float tval[R];
#pragma unroll
  for (int r = 0; r < R; ++r) {
    const int w = lane + 64 * r;
    tval[r] = 0.0f;
    key[r] = ~0ull;                                   // padding slot: after every real key
    if (w < W) {
      tval[r] = arrival_t[w];
      key[r] = ((unsigned long long)ordered_time_bits(tval[r]) << 32) | (unsigned)w;
    }
    keys[w] = key[r];
  }
  __syncthreads();

  int rank[R];
#pragma unroll
  for (int r = 0; r < R; ++r) rank[r] = 0;
  for (int j = 0; j < W; ++j) {
    const unsigned long long kj = keys[j];            // same address in every lane: LDS broadcast
#pragma unroll
    for (int r = 0; r < R; ++r) rank[r] += (kj < key[r]) ? 1 : 0;
  }

  int base = 0;
#pragma unroll
  for (int r = 0; r < R; ++r) {
    const int w = lane + 64 * r;
    const bool keep = (w < W) && (rank[r] < N);
    const unsigned long long mask = __ballot(keep);
    const int pos = base + __builtin_amdgcn_mbcnt_hi((unsigned)(mask >> 32), __builtin_amdgcn_mbcnt_lo((unsigned)mask, 0u));
    if (keep) sel_idx[pos] = w;
    base += __popcll(mask);
    if ((w < W) && rank[r] == N - 1) {                // the N-th arrival decides the step
      const unsigned hi = (unsigned)(key[r] >> 32);
      if (t_step) *t_step = tval[r];
      *status = (hi >= kNeverArrives) ? -2 : 0;
    }
  }
}

// ---------------------------------------------------------------------------
// Tensor table
// ---------------------------------------------------------------------------
constexpr int kUploadBatch = 64;

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
template <int V, int B, bool NT>
__device__ __forceinline__ void add_rows(f4 (&acc)[V], const float* __restrict__ grads, long long ld,
                                         long long colbase, const int* __restrict__ sel_idx, int j,
                                         const unsigned (&toff)[V]) {
  f4 r[B][V];
#pragma unroll
  for (int u = 0; u < B; ++u) {
    const long long k = sel_idx[j + u];
    const char* rowbase = reinterpret_cast<const char*>(grads + k * ld + colbase);
#pragma unroll
    for (int v = 0; v < V; ++v) r[u][v] = load_row_f4<NT>(rowbase, toff[v]);
  }
#pragma unroll
  for (int u = 0; u < B; ++u)
#pragma unroll
    for (int v = 0; v < V; ++v) acc[v] += r[u][v];
}

// All kept rows, in batches of U (then 8, 4, 2, 1 for what is left).
template <int V, int U, bool NT>
__device__ __forceinline__ void sum_rows(f4 (&acc)[V], const float* __restrict__ grads, long long ld,
                                         long long colbase, const int* __restrict__ sel_idx, int N,
                                         const unsigned (&toff)[V]) {
  int j = 0;
  for (; j + U <= N; j += U) add_rows<V, U, NT>(acc, grads, ld, colbase, sel_idx, j, toff);
  if constexpr (U > 8) { if ((N - j) & 8) { add_rows<V, 8, NT>(acc, grads, ld, colbase, sel_idx, j, toff); j += 8; } }
  if constexpr (U > 4) { if ((N - j) & 4) { add_rows<V, 4, NT>(acc, grads, ld, colbase, sel_idx, j, toff); j += 4; } }
  if constexpr (U > 2) { if ((N - j) & 2) { add_rows<V, 2, NT>(acc, grads, ld, colbase, sel_idx, j, toff); j += 2; } }
  if constexpr (U > 1) { if ((N - j) & 1) { add_rows<V, 1, NT>(acc, grads, ld, colbase, sel_idx, j, toff); j += 1; } }
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
template <int MODE, class S, bool MULTI, bool SRC_ROWS>
__global__ __launch_bounds__(S::BS) void k_step(StepParams p) {
  constexpr int BS = S::BS, V = S::V, U = S::U;
  constexpr bool NT = S::NT;
  constexpr long long CH = 4LL * BS * V;               // columns per chunk
  extern __shared__ unsigned starts_lds[];             // MULTI: starts[S+1]
  __shared__ float red_lds[BS / 64];

  if (p.status != nullptr && *p.status != 0) return;  // too few arrivals: touch nothing

  if constexpr (MULTI) {
    for (int i = threadIdx.x; i <= p.S; i += BS) starts_lds[i] = p.starts[i];
    __syncthreads();
  }
  const long long span_end4 = (p.col_hi + 3) & ~3LL;   // rows are readable up to here (<= ld)

  for (int chunk_id = (int)blockIdx.x + p.chunk_base; chunk_id < p.chunk_end; chunk_id += (int)gridDim.x) {
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
      seg = p.table[j0];
    } else {
      seg_start = p.col_lo;
      seg_end = p.col_hi;
      seg = p.single;
    }
    const bool uniform = (c0 >= seg_start) && (c0 + CH <= seg_end) && (seg.theta != nullptr);

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
      sum_rows<V, U, NT>(g, p.grads, p.ld, c0, p.sel_idx, p.N, toff);
#pragma unroll
      for (int v = 0; v < V; ++v) g[v] *= p.inv_n;
    } else {
#pragma unroll
      for (int v = 0; v < V; ++v)
        g[v] = *reinterpret_cast<const f4*>(reinterpret_cast<const char*>(p.gbar + c0) + toff[v]) * scale;
    }

    if (uniform) {
      // ---- the whole chunk lies inside one tensor ------------------------------------
      const long long e_first = c0 - seg_start;        // element of the tensor at the chunk's first column
      if constexpr (MODE == kClipReduce) {
#pragma unroll
        for (int v = 0; v < V; ++v) {
          *reinterpret_cast<f4*>(reinterpret_cast<char*>(p.gbar + c0) + toff[v]) = g[v];
          sumsq = fmaf(g[v].x, g[v].x, sumsq);
          sumsq = fmaf(g[v].y, g[v].y, sumsq);
          sumsq = fmaf(g[v].z, g[v].z, sumsq);
          sumsq = fmaf(g[v].w, g[v].w, sumsq);
        }
      } else {
        // fetch theta/state for all groups first (independent loads in flight together)
        f4 th[V], a[V], b[V];
#pragma unroll
        for (int v = 0; v < V; ++v) {
          th[v] = *reinterpret_cast<const f4u*>(reinterpret_cast<const char*>(seg.theta + e_first) + toff[v]);
          if constexpr (MODE >= kMomentum) a[v] = *reinterpret_cast<const f4u*>(reinterpret_cast<const char*>(seg.s0 + e_first) + toff[v]);
          if constexpr (MODE == kRmspropMom) b[v] = *reinterpret_cast<const f4u*>(reinterpret_cast<const char*>(seg.s1 + e_first) + toff[v]);
        }
#pragma unroll
        for (int v = 0; v < V; ++v) {
          update_vec<MODE>(g[v], th[v], a[v], b[v], p);
          *reinterpret_cast<f4u*>(reinterpret_cast<char*>(seg.theta + e_first) + toff[v]) = th[v];
          if constexpr (MODE >= kMomentum) *reinterpret_cast<f4u*>(reinterpret_cast<char*>(seg.s0 + e_first) + toff[v]) = a[v];
          if constexpr (MODE == kRmspropMom) *reinterpret_cast<f4u*>(reinterpret_cast<char*>(seg.s1 + e_first) + toff[v]) = b[v];
        }
      }
    } else {
      // ---- the chunk holds a tensor boundary, a gap, or the end of the row ---------------
      // One group after the other (this path is rare; it favours few registers
      // over loads in flight).
#pragma unroll
      for (int v = 0; v < V; ++v) {
        const long long gcol = c0 + 4LL * S::group_of(v);
        if (gcol >= span_end4) continue;
        const f4 gv = g[v];
        if constexpr (MODE == kClipReduce) {
          // the stored mean is laid out like a row: whole groups, gaps included
          *reinterpret_cast<f4*>(p.gbar + gcol) = gv;
        }
        if (gcol + 4 <= p.col_lo || gcol >= p.col_hi) continue;
        // segment of the group's first covered column
        int j = 0;
        long long s_start = p.col_lo, s_end = p.col_hi;
        Segment sg = seg;
        if constexpr (MULTI) {
          const long long x = gcol < p.col_lo ? p.col_lo : gcol;
          j = find_segment(starts_lds, p.S, (unsigned)x);
          s_start = starts_lds[j];
          s_end = starts_lds[j + 1];
          sg = p.table[j];
        }
        if (gcol >= s_start && gcol + 4 <= s_end) {
          // whole group inside one segment
          if (sg.theta == nullptr) continue;           // a gap
          if constexpr (MODE == kClipReduce) {
            sumsq = fmaf(gv.x, gv.x, sumsq);
            sumsq = fmaf(gv.y, gv.y, sumsq);
            sumsq = fmaf(gv.z, gv.z, sumsq);
            sumsq = fmaf(gv.w, gv.w, sumsq);
          } else {
            const long long e = gcol - s_start;
            f4 th, a, b;
            th = *reinterpret_cast<const f4u*>(sg.theta + e);
            if constexpr (MODE >= kMomentum) a = *reinterpret_cast<const f4u*>(sg.s0 + e);
            if constexpr (MODE == kRmspropMom) b = *reinterpret_cast<const f4u*>(sg.s1 + e);
            update_vec<MODE>(gv, th, a, b, p);
            *reinterpret_cast<f4u*>(sg.theta + e) = th;
            if constexpr (MODE >= kMomentum) *reinterpret_cast<f4u*>(sg.s0 + e) = a;
            if constexpr (MODE == kRmspropMom) *reinterpret_cast<f4u*>(sg.s1 + e) = b;
          }
        } else {
          // the group is cut by a boundary: element by element
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            const long long col = gcol + q;
            if (col < p.col_lo || col >= p.col_hi) continue;
            if constexpr (MULTI) {
              while (col >= s_end) {                   // segments are non-empty: at most 3 steps per group
                ++j;
                s_start = s_end;
                s_end = starts_lds[j + 1];
                sg = p.table[j];
              }
            }
            if (sg.theta == nullptr) continue;         // a gap
            const float gq = gv[q];
            if constexpr (MODE == kClipReduce) {
              sumsq = fmaf(gq, gq, sumsq);
            } else {
              const long long e = col - s_start;
              float t1 = sg.theta[e], a1 = 0.f, b1 = 0.f;
              if constexpr (MODE >= kMomentum) a1 = sg.s0[e];
              if constexpr (MODE == kRmspropMom) b1 = sg.s1[e];
              update_elem<MODE>(gq, t1, a1, b1, p);
              sg.theta[e] = t1;
              if constexpr (MODE >= kMomentum) sg.s0[e] = a1;
              if constexpr (MODE == kRmspropMom) sg.s1[e] = b1;
            }
          }
        }
      }
    }

    if constexpr (MODE == kClipReduce) {
      const double s = block_sum<BS>(sumsq, red_lds);
      if (threadIdx.x == 0) p.partials[chunk_id] = s;
      __syncthreads();                                 // red_lds is reused by the next chunk
    }
  }  // chunk loop
}

// One workgroup adds the per-block sums of squares in a fixed order (fp64),
// takes the root and writes norm and scale = min(1, c/norm) to the header.
constexpr int kFinalizeBlock = 1024;
__global__ __launch_bounds__(kFinalizeBlock) void k_finalize_norm(const double* __restrict__ partials, int n,
                                                                   float c, const int* __restrict__ status,
                                                                   WsHeader* __restrict__ header) {
  __shared__ double red[kFinalizeBlock];
  if (status != nullptr && *status != 0) return;
  double s = 0.0;
  for (int i = threadIdx.x; i < n; i += kFinalizeBlock) s += partials[i];
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

// Plain 16-byte-per-thread copy with a known byte count: the yardstick the
// profiler's HBM read/write counters are scaled against.
__global__ __launch_bounds__(256) void k_calibration_copy(const f4* __restrict__ src, f4* __restrict__ dst, long long n16) {
  const long long i = (long long)blockIdx.x * 256 + threadIdx.x;
  if (i < n16) dst[i] = src[i];
}

}  // namespace bsgd
