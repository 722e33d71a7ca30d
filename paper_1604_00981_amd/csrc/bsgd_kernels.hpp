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
//   V    float4 columns per thread (a chunk is BS*V float4 groups wide)
//   U    kept rows loaded per batch before the first add
//   NT   gradient rows are loaded with the non-temporal (streaming) hint
//   MAP  0: thread t takes groups t, t+BS, ...   (workgroup-strided)
//        1: wave w takes V*64 consecutive groups (each wavefront reads one
//           contiguous V KiB piece of a row)
template <int BS_, int V_, int U_, bool NT_, int MAP_>
struct Shape {
  static constexpr int BS = BS_, V = V_, U = U_, MAP = MAP_;
  static constexpr bool NT = NT_;
  __device__ static __forceinline__ int group_of(int v) {
    if constexpr (MAP_ == 0) return v * BS_ + (int)threadIdx.x;
    else return (((int)threadIdx.x >> 6) * V_ + v) * 64 + ((int)threadIdx.x & 63);
  }
};
constexpr int kMaxWorkers = 256;

enum Mode : int { kSgd = 0, kMomentum = 1, kRmspropMom = 2, kClipReduce = 3 };

// What the host keeps per tensor on the device.
struct DevTensor {
  float* theta;
  float* s0;
  float* s1;
  long long grad_offset;
  long long numel;
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
  // tensors
  DevTensor single;          // used when there is exactly one tensor
  const DevTensor* table;    // [T]
  const int* chunk_begin;    // [T+1] first chunk of each tensor, then the total
  int T;
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
  int first, count, total_chunks, is_last;
  DevTensor t[kUploadBatch];
  int chunk_begin[kUploadBatch];
};

// Descriptors travel in the kernel-argument buffer, so the host array is
// consumed at launch time and no host-to-device copy has to be ordered.
__global__ __launch_bounds__(kUploadBatch) void k_upload_table(UploadArgs a, DevTensor* __restrict__ table,
                                                                 int* __restrict__ chunk_begin, int T) {
  const int i = threadIdx.x;
  if (i < a.count) {
    table[a.first + i] = a.t[i];
    chunk_begin[a.first + i] = a.chunk_begin[i];
  }
  if (i == 0 && a.is_last) chunk_begin[T] = a.total_chunks;
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

// The optimizer update of one element; g is the (mean, possibly clipped)
// aggregated gradient.
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

// Which tensor a chunk belongs to: the last j with chunk_begin[j] <= c.
__device__ __forceinline__ int find_tensor(const int* cb, int T, int c) {
  int lo = 0, hi = T;                                 // invariant: cb[lo] <= c < cb[hi]
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (cb[mid] <= c) lo = mid; else hi = mid;
  }
  return lo;
}

// SRC_ROWS: the gradient comes from summing the kept rows (MODE 0..2 updates
// directly; MODE kClipReduce stores the mean and a per-block sum of squares).
// !SRC_ROWS: the gradient is the stored mean times the clip scale (MODE 0..2).
//
// Work is cut into chunks of BS*V float4 groups.  Groups are aligned to the
// gradient row (not to theta): group g of a tensor covers elements
// [4g-h, 4g-h+4) with h = grad_offset mod 4, so row loads are 16-byte aligned
// whenever grads and ld are; theta/state accesses may then be only 4-byte
// aligned.  Chunks fully inside a tensor take the vector path with no
// per-lane tests; the first and last chunk of a tensor take the edge path.
template <int MODE, class S, bool MULTI, bool SRC_ROWS>
__global__ __launch_bounds__(S::BS) void k_step(StepParams p) {
  constexpr int BS = S::BS, V = S::V, U = S::U;
  constexpr bool NT = S::NT;
  extern __shared__ int cb_lds[];                      // MULTI: chunk_begin[T+1]
  __shared__ float red_lds[BS / 64];

  if (p.status != nullptr && *p.status != 0) return;  // too few arrivals: touch nothing

  DevTensor tz;
  int c = blockIdx.x;
  if constexpr (MULTI) {
    for (int i = threadIdx.x; i <= p.T; i += BS) cb_lds[i] = p.chunk_begin[i];
    __syncthreads();
    const int j = __builtin_amdgcn_readfirstlane(find_tensor(cb_lds, p.T, c));   // same in every lane
    c -= __builtin_amdgcn_readfirstlane(cb_lds[j]);
    tz = p.table[j];
  } else {
    tz = p.single;
  }

  const int h = (int)(tz.grad_offset & 3);
  const long long group0 = (long long)c * (BS * V);
  const long long e_first = 4 * group0 - h;            // first element this chunk covers (may be < 0)
  const long long colbase = tz.grad_offset + e_first;  // same thing inside a gradient row
  const bool interior = (e_first >= 0) && (e_first + 4LL * BS * V <= tz.numel);

  float scale = 1.0f;
  if constexpr (!SRC_ROWS) scale = p.header->clip_scale;

  float sumsq = 0.0f;

  if (interior) {
    unsigned toff[V];
#pragma unroll
    for (int v = 0; v < V; ++v) toff[v] = (unsigned)S::group_of(v) * 16u;

    // issue the parameter/state loads first so they overlap the row loop
    f4 th[V], a[V], b[V];
    if constexpr (MODE != kClipReduce) {
#pragma unroll
      for (int v = 0; v < V; ++v) {
        th[v] = *reinterpret_cast<const f4u*>(reinterpret_cast<const char*>(tz.theta + e_first) + toff[v]);
        if constexpr (MODE >= kMomentum) a[v] = *reinterpret_cast<const f4u*>(reinterpret_cast<const char*>(tz.s0 + e_first) + toff[v]);
        if constexpr (MODE == kRmspropMom) b[v] = *reinterpret_cast<const f4u*>(reinterpret_cast<const char*>(tz.s1 + e_first) + toff[v]);
      }
    }

    f4 g[V];
    if constexpr (SRC_ROWS) {
#pragma unroll
      for (int v = 0; v < V; ++v) g[v] = f4{0.f, 0.f, 0.f, 0.f};
      sum_rows<V, U, NT>(g, p.grads, p.ld, colbase, p.sel_idx, p.N, toff);
#pragma unroll
      for (int v = 0; v < V; ++v) g[v] *= p.inv_n;
    } else {
#pragma unroll
      for (int v = 0; v < V; ++v)
        g[v] = *reinterpret_cast<const f4*>(reinterpret_cast<const char*>(p.gbar + colbase) + toff[v]) * scale;
    }

    if constexpr (MODE == kClipReduce) {
#pragma unroll
      for (int v = 0; v < V; ++v) {
        *reinterpret_cast<f4*>(reinterpret_cast<char*>(p.gbar + colbase) + toff[v]) = g[v];
        sumsq = fmaf(g[v].x, g[v].x, sumsq);
        sumsq = fmaf(g[v].y, g[v].y, sumsq);
        sumsq = fmaf(g[v].z, g[v].z, sumsq);
        sumsq = fmaf(g[v].w, g[v].w, sumsq);
      }
    } else {
#pragma unroll
      for (int v = 0; v < V; ++v) {
        update_vec<MODE>(g[v], th[v], a[v], b[v], p);
        *reinterpret_cast<f4u*>(reinterpret_cast<char*>(tz.theta + e_first) + toff[v]) = th[v];
        if constexpr (MODE >= kMomentum) *reinterpret_cast<f4u*>(reinterpret_cast<char*>(tz.s0 + e_first) + toff[v]) = a[v];
        if constexpr (MODE == kRmspropMom) *reinterpret_cast<f4u*>(reinterpret_cast<char*>(tz.s1 + e_first) + toff[v]) = b[v];
      }
    }
  } else {
    // Edge chunk: per float4 group, a full group still uses one 16-byte load
    // per row; a group cut by the tensor's start or end goes element by element.
    for (int v = 0; v < V; ++v) {
      const long long e0 = e_first + 4LL * S::group_of(v);
      if (e0 + 4 <= 0 || e0 >= tz.numel) continue;
      const bool full = (e0 >= 0) && (e0 + 4 <= tz.numel);
      float gv[4] = {0.f, 0.f, 0.f, 0.f};
      bool ok[4];
#pragma unroll
      for (int q = 0; q < 4; ++q) ok[q] = (e0 + q >= 0) && (e0 + q < tz.numel);
      const long long col = tz.grad_offset + e0;
      if constexpr (SRC_ROWS) {
        if (full) {
          f4 acc[1] = {f4{0.f, 0.f, 0.f, 0.f}};
          const unsigned z[1] = {0u};
          sum_rows<1, U, NT>(acc, p.grads, p.ld, col, p.sel_idx, p.N, z);
          gv[0] = acc[0].x; gv[1] = acc[0].y; gv[2] = acc[0].z; gv[3] = acc[0].w;
        } else {
          for (int j = 0; j < p.N; ++j) {
            const float* row = p.grads + (long long)p.sel_idx[j] * p.ld + col;
#pragma unroll
            for (int q = 0; q < 4; ++q) if (ok[q]) gv[q] += row[q];
          }
        }
#pragma unroll
        for (int q = 0; q < 4; ++q) gv[q] *= p.inv_n;
      } else {
#pragma unroll
        for (int q = 0; q < 4; ++q) if (ok[q]) gv[q] = p.gbar[col + q] * scale;
      }
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        if (!ok[q]) continue;
        const long long e = e0 + q;
        if constexpr (MODE == kClipReduce) {
          p.gbar[col + q] = gv[q];
          sumsq = fmaf(gv[q], gv[q], sumsq);
        } else {
          float th = tz.theta[e], a = 0.f, b = 0.f;
          if constexpr (MODE >= kMomentum) a = tz.s0[e];
          if constexpr (MODE == kRmspropMom) b = tz.s1[e];
          update_elem<MODE>(gv[q], th, a, b, p);
          tz.theta[e] = th;
          if constexpr (MODE >= kMomentum) tz.s0[e] = a;
          if constexpr (MODE == kRmspropMom) tz.s1[e] = b;
        }
      }
    }
  }

  if constexpr (MODE == kClipReduce) {
    const double s = block_sum<BS>(sumsq, red_lds);
    if (threadIdx.x == 0) p.partials[blockIdx.x] = s;
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
