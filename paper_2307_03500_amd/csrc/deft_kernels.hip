// Device side of the DEFT selection path for gfx950 (MI355X): the per-layer norm pass
// (Sec. 4.2) and the segmented magnitude Top-k with ordered (index, value) compaction
// (Alg. 5, Sec. 4.4), which also serves the conventional Top-k over the whole vector (Sec. 1).
//
// Both are streaming passes bound by HBM bandwidth: 16-byte loads, 64-lane wavefront
// reductions/ballots, per-workgroup LDS histograms, no matrix instructions.
//
// Selection = exact radix select on the 31-bit key (bits & 0x7fffffff), digit levels of
// 11/10/10 bits.  The segment is read once in full and a second time where it can still hold
// selected entries; the rest works on a few hundred parked bytes per chunk:
//   hist0        pass 1: histogram of the top digit; largest top digit of every chunk
//   pass2        pass 2: skips chunks below the threshold's top-digit bucket; parks every key at
//                or above that bucket as {value bits, index}, in index order, in per-chunk slots;
//                histograms the bucket's keys on the second digit
//   slot_hist2   third digit level, from the slots
//   slot_count   per-chunk counts of keys > T and == T, from the slots
//   emit         ordered (index, value) write, from the slots
// A chunk whose slots overflowed is read from the segment again by the three slot kernels.
// The bucket search between levels runs inside the next kernel (short vectors) or as a
// one-workgroup-per-segment kernel (long vectors).
// Long vectors read a qualifying segment ONCE: a 1/128 sample places the threshold's top digit
// within four digits (sample_hist, bounds), the one full pass parks every key at or above the
// lowest of them and histograms the four digits on their top 21 bits (pass1_bounded), and an
// exact check of the counts (find_first) either yields the state after two digit levels or
// sends the segment down the two-read path above.  The sample decides how often a segment is
// read, never what is selected.
// An element is selected iff key > T, or key == T and fewer than r equal keys precede it in
// its segment.  Every pass walks the segments in fixed-size chunks; a chunk never spans two
// segments, so small layers simply own short chunks and large layers are split over many
// workgroups.
#include "deft.h"

#include <hip/hip_runtime.h>

#include <algorithm>
#include <atomic>
#include <chrono>
#include <cstring>
#include <mutex>
#include <vector>

namespace {

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / 64;
constexpr int64_t kMaxN = (int64_t(1) << 31) - 1;
constexpr uint32_t kMaxSlotCap = kThreads;  // unit of the slot capacities: a round of the slot kernels
// Workgroups of the long-vector first pass: at least the resident set (256 CUs x 3), so every
// slot is filled; latecomers find the counter exhausted and leave.
#ifndef DEFT_STREAM_GRID
#define DEFT_STREAM_GRID 1024
#endif
constexpr uint32_t kStreamGrid = DEFT_STREAM_GRID;
// Workgroups of the grid-stride third-level kernel of long vectors (measured on 1.42 GB: 24 / 17 /
// 15 / 12.8 / 13 us with 512 / 768 / 1024 / 1536 / 2048).
constexpr uint32_t kSlotWaveGrid = 2048;
constexpr uint32_t kOverflowGrid = 2048;  // workgroups of the launch that writes overflowed chunks

typedef float v4f __attribute__((ext_vector_type(4)));
typedef uint32_t v4u __attribute__((ext_vector_type(4)));

// ------------------------------------------------------------------------------------------
// reductions
// ------------------------------------------------------------------------------------------
__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_down(v, o, 64);
  return v;  // valid in lane 0
}

// Sum over the workgroup in a fixed order; result in every thread.
__device__ __forceinline__ double block_sum(double v, double* red) {
  v = wave_sum(v);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
  __syncthreads();
  return ((red[0] + red[1]) + red[2]) + red[3];
}

__device__ __forceinline__ uint32_t wave_sum_u32(uint32_t v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_down(v, o, 64);
  return v;
}

// ------------------------------------------------------------------------------------------
// norm pass (Sec. 4.2): sumsq[l] = sum over layer l of g^2, fp64
// ------------------------------------------------------------------------------------------
#ifndef DEFT_NORM_ITERS
#define DEFT_NORM_ITERS 4
#endif
constexpr int kNormIters = DEFT_NORM_ITERS;                // 16-byte loads per thread
constexpr int kNormChunk = kThreads * 4 * kNormIters;      // elements per workgroup

// Largest l in [0, L-1] with off[l] <= x (off[0] == 0 <= x).
__device__ __forceinline__ int layer_of(const int64_t* __restrict__ off, int L, int64_t x) {
  int lo = 0, hi = L;
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (off[mid] <= x) lo = mid; else hi = mid;
  }
  return lo;
}

// The vector is cut into fixed chunks of kNormChunk elements, whatever the layer layout, so
// every 16-byte load is aligned.  A chunk that lies inside one layer writes one partial
// (head).  A chunk holding layer boundaries writes the part of the layer it starts in (head),
// the part of the layer it ends in (tail) and finishes the layers that lie wholly inside it.
// Source of the values that are normed.  Plain: the vector itself.  Accumulating (Alg. 1, the
// step before the sparsifier): acc = e + eta * grad in fp32 -- product rounded, then sum
// rounded -- written back to `acc` on the way.
struct NormSrc {
  const float* g;                // plain: the vector; accumulating: the local error e
  const float* __restrict__ gr;  // accumulating: the fresh gradient
  float* acc;                    // accumulating: output (may alias g)
  float eta;
};

template <bool ACC>
__device__ __forceinline__ float norm_value(const NormSrc& src, int64_t i) {
  if (!ACC) return src.g[i];
  const float v = __fadd_rn(src.g[i], __fmul_rn(src.eta, src.gr[i]));
  src.acc[i] = v;
  return v;
}

template <bool ACC>
__device__ __forceinline__ void norm_one_chunk(
    const NormSrc& src, int64_t N, const int64_t* __restrict__ off, int L,
    double* __restrict__ head, double* __restrict__ tail, double* __restrict__ sumsq,
    int64_t chunk, double* red) {
  const int64_t cs = chunk * kNormChunk;
  const int64_t ce = min(N, cs + (int64_t)kNormChunk);
  const int lf = layer_of(off, L, cs);
  if (off[lf + 1] >= ce) {
    double a0 = 0.0, a1 = 0.0;
    if (ce - cs == kNormChunk) {
      // Streaming (non-temporal) loads: every byte is used once, so the lines should not
      // displace anything in L2.  Measured on 1.42 GB: 204 us against 222 us for plain loads
      // of the same launch shape (6.95 vs 6.37 TB/s).
      const v4f* __restrict__ p = reinterpret_cast<const v4f*>(src.g + cs);
      v4f v[kNormIters];
#pragma unroll
      for (int i = 0; i < kNormIters; ++i) v[i] = __builtin_nontemporal_load(&p[threadIdx.x + i * kThreads]);
      if (ACC) {
        const v4f* __restrict__ q = reinterpret_cast<const v4f*>(src.gr + cs);
        v4f w[kNormIters];
#pragma unroll
        for (int i = 0; i < kNormIters; ++i) w[i] = __builtin_nontemporal_load(&q[threadIdx.x + i * kThreads]);
        v4f* o = reinterpret_cast<v4f*>(src.acc + cs);
#pragma unroll
        for (int i = 0; i < kNormIters; ++i) {
          v[i].x = __fadd_rn(v[i].x, __fmul_rn(src.eta, w[i].x));
          v[i].y = __fadd_rn(v[i].y, __fmul_rn(src.eta, w[i].y));
          v[i].z = __fadd_rn(v[i].z, __fmul_rn(src.eta, w[i].z));
          v[i].w = __fadd_rn(v[i].w, __fmul_rn(src.eta, w[i].w));
          __builtin_nontemporal_store(v[i], &o[threadIdx.x + i * kThreads]);
        }
      }
#pragma unroll
      for (int i = 0; i < kNormIters; ++i) {
        const double x = v[i].x, y = v[i].y, z = v[i].z, w = v[i].w;
        a0 = fma(x, x, a0);
        a1 = fma(y, y, a1);
        a0 = fma(z, z, a0);
        a1 = fma(w, w, a1);
      }
#ifdef DEFT_PROBE_NORM_HIST
      // Measurement only: the top-digit histogram of every layer gathered by the norm pass itself
      // (per-workgroup LDS histogram, merged into the layer's with one atomic per occupied bin),
      // into scratch 64 MB behind the partial sums.  Not part of any result.
      {
        __shared__ uint32_t ph[2048];
        for (int b = threadIdx.x; b < 2048; b += kThreads) ph[b] = 0;
        __syncthreads();
#pragma unroll
        for (int i = 0; i < kNormIters; ++i) {
          atomicAdd(&ph[(__float_as_uint(v[i].x) & 0x7FFFFFFFu) >> 20], 1u);
          atomicAdd(&ph[(__float_as_uint(v[i].y) & 0x7FFFFFFFu) >> 20], 1u);
          atomicAdd(&ph[(__float_as_uint(v[i].z) & 0x7FFFFFFFu) >> 20], 1u);
          atomicAdd(&ph[(__float_as_uint(v[i].w) & 0x7FFFFFFFu) >> 20], 1u);
        }
        __syncthreads();
        uint32_t* gh = reinterpret_cast<uint32_t*>(head) + (16u << 20) + (size_t)lf * 2048;
        for (int b = threadIdx.x; b < 2048; b += kThreads) {
          const uint32_t c = ph[b];
          if (c) atomicAdd(&gh[b], c);
        }
      }
#endif
    } else {
      for (int64_t i = cs + threadIdx.x; i < ce; i += kThreads) {
        const double x = norm_value<ACC>(src, i);
        a0 = fma(x, x, a0);
      }
    }
    const double t = block_sum(a0 + a1, red);
    if (threadIdx.x == 0) { head[chunk] = t; tail[chunk] = 0.0; }
    return;
  }
  if (threadIdx.x == 0) tail[chunk] = 0.0;
  for (int l = lf; l < L; ++l) {
    const int64_t lo = off[l], hi = off[l + 1];
    if (l > lf && lo >= ce) break;
    const int64_t s = max(cs, lo), e = min(ce, hi);
    double a = 0.0;
    for (int64_t i = s + threadIdx.x; i < e; i += kThreads) {
      const double x = norm_value<ACC>(src, i);
      a = fma(x, x, a);
    }
    const double t = block_sum(a, red);
    if (threadIdx.x == 0) {
      if (l == lf) head[chunk] = t;
      else if (hi >= ce) tail[chunk] = t;
      else sumsq[l] = t;
    }
    if (hi >= ce) break;
  }
}

template <bool ACC>
__global__ __launch_bounds__(kThreads) void norm_chunks_kernel(
    NormSrc src, int64_t N, const int64_t* __restrict__ off, int L, double* __restrict__ head,
    double* __restrict__ tail, double* __restrict__ sumsq) {
  __shared__ double red[kWaves];
  norm_one_chunk<ACC>(src, N, off, L, head, tail, sumsq, blockIdx.x, red);
}

// Measurement aid: reads the vector once in the launch shape of the norm pass (fixed chunks of
// kNormChunk elements, kNormIters streaming 16-byte loads per thread) and does nothing else but
// fold the words together; the time of this kernel is the read rate the access pattern can reach
// on the machine at hand.  The fold is stored only if it hits one particular value, which keeps
// the loads alive without a store per workgroup.
__global__ __launch_bounds__(kThreads) void stream_probe_kernel(const float* __restrict__ g,
                                                                uint32_t* __restrict__ out) {
  const v4u* __restrict__ p = reinterpret_cast<const v4u*>(g + (int64_t)blockIdx.x * kNormChunk);
  v4u v[kNormIters];
#pragma unroll
  for (int i = 0; i < kNormIters; ++i) v[i] = __builtin_nontemporal_load(&p[threadIdx.x + i * kThreads]);
  uint32_t x = 0;
#pragma unroll
  for (int i = 0; i < kNormIters; ++i) x ^= v[i].x ^ v[i].y ^ v[i].z ^ v[i].w;
  if (x == 0x9E3779B9u) out[0] = x;
}

// vals[i] = acc[idx[i]]; acc[idx[i]] = 0   (Alg. 1, the steps after the index exchange)
__global__ __launch_bounds__(kThreads) void gather_zero_kernel(float* __restrict__ acc, int64_t N,
                                                               const int32_t* __restrict__ idx,
                                                               int64_t count,
                                                               float* __restrict__ vals) {
  const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
  if (i >= count) return;
  const int64_t j = idx[i];
  if (j < 0 || j >= N) { vals[i] = 0.0f; return; }
  vals[i] = acc[j];
  acc[j] = 0.0f;
}

// One workgroup per layer adds the partials of the chunks the layer touches, in chunk order
// per thread and a fixed order across threads.  1024 threads: the longest layer sets the time of
// this launch, which sits between the norm pass and the host's plan (a 51 M-element layer is
// 12 500 partials: 12 dependent rounds per thread instead of 49).
#ifndef DEFT_FINISH_THREADS
#define DEFT_FINISH_THREADS 1024
#endif
constexpr int kFinishThreads = DEFT_FINISH_THREADS;
__global__ __launch_bounds__(kFinishThreads) void norm_finish_kernel(
    const int64_t* __restrict__ off, int64_t N, const double* __restrict__ head,
    const double* __restrict__ tail, double* __restrict__ sumsq) {
  __shared__ double red[kFinishThreads / 64];
  const int l = blockIdx.x;
  const int64_t s = off[l], e = off[l + 1];
  if (e <= s || s < 0 || e > N) {
    if (threadIdx.x == 0) sumsq[l] = 0.0;
    return;
  }
  const int64_t b0 = s / kNormChunk, b1 = (e - 1) / kNormChunk;
  const bool first = (s == b0 * kNormChunk);
  if (b0 == b1) {
    if (threadIdx.x == 0) {
      if (first) sumsq[l] = head[b0];
      else if (e == min(N, (b0 + 1) * (int64_t)kNormChunk)) sumsq[l] = tail[b0];
      // otherwise the layer lies strictly inside chunk b0 and was finished there
    }
    return;
  }
  double a = 0.0;
  for (int64_t b = b0 + 1 + threadIdx.x; b <= b1; b += kFinishThreads) a += head[b];
  a = wave_sum(a);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = a;
  __syncthreads();
  if (threadIdx.x == 0) {
    double t = 0.0;
    for (int w = 0; w < kFinishThreads / 64; ++w) t += red[w];
    sumsq[l] = (first ? head[b0] : tail[b0]) + t;
  }
}

// ------------------------------------------------------------------------------------------
// selection
// ------------------------------------------------------------------------------------------
struct SegDesc {
  uint32_t start;       // first element of the segment in g
  uint32_t size;        // elements
  uint32_t k;           // entries to select, 1 <= k <= size
  uint32_t out_off;     // first output slot of the segment
  uint32_t chunk_base;  // first chunk id of the segment in the count/emit passes
  uint32_t hchunk_base; // first chunk id of the segment in the histogram passes (larger chunks)
  uint32_t sblock_base; // first workgroup of the segment in the sampling kernel (long vectors)
  uint32_t sampled;     // 0, or 1 + the number of the segment's bounded histogram: the segment is
                        // sampled ahead of its first pass (long vectors)
};

// How the first pass treats a segment of a long vector.
//   kModeFull:    top-digit histogram of every key, nothing parked (pass 2 parks).
//   kModeBounded: a sample of the segment has placed the threshold's top digit in
//                 b_lo .. b_lo + 3; the first pass parks every key whose top digit is at least
//                 b_lo and histograms the keys of those four digits on their top 21 bits (4096 bins
//                 of 2^10 keys), so that the segment is read once.  Checked exactly afterwards
//                 (find_first_kernel).
//   kModeFailed:  the check failed (the sample misled): the segment is read again as kModeFull.
constexpr uint32_t kModeFull = 0, kModeBounded = 1, kModeFailed = 2;
// The one-read pass is taken where it would park at most one key in kParkDiv, the slots' share
// of a chunk (beyond it most chunks would overflow their slots).  Conventional Top-k over 1.4 GB at
// d = 0.05 / 0.1 / 0.2: 459 / 572 / 818 us read once, 682 / 814 / 1064 us read twice.
#ifndef DEFT_PARK_DIV
#define DEFT_PARK_DIV 4
#endif
constexpr uint32_t kParkDiv = DEFT_PARK_DIV;
constexpr int kHiCopies = 16;
struct SegBound {
  uint32_t mode;
  uint32_t b_lo;
  uint32_t pad[2];
  // Counted by the first pass, in copies as for the histograms (workgroup b adds to
  // hi[b % kHiCopies]), two counts per word so that one atomic carries both: low half, the keys
  // above the four digits; high half, the parked keys whose low kBits2 bits are not all zero.
  unsigned long long hi[kHiCopies];
};
// Bits of the flag word the first bucket search leaves for the kernels behind it.
constexpr uint32_t kFlagPass2 = 2u;   // some segment needs the full first pass and pass 2
constexpr uint32_t kFlagLevel2 = 4u;  // some segment's threshold still lacks its last digit
constexpr uint32_t kFlagOverflow = 8u;  // some chunk parked more keys than it has slots
// Raised by whoever meets such a chunk, once per launch rather than once per chunk where chunks
// overflow in their thousands (dense selections): atomics on one word are served one by one.
__device__ __forceinline__ void raise_flag(uint32_t* flags, uint32_t bit) {
  if (!(__hip_atomic_load(flags, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) & bit)) atomicOr(flags, bit);
}

struct SegState {
  uint32_t prefix;  // key bits fixed so far (right-aligned)
  uint32_t k_rem;   // entries still to take inside the prefix bucket
  uint32_t T;       // threshold key once resolved
  uint32_t r;       // number of entries with key == T to take (lowest indices first)
  uint32_t done;    // threshold resolved
  uint32_t pad[3];
};

constexpr int kSegBatch = 120;
struct SegBatch {
  int32_t first;
  int32_t count;
  uint32_t total_chunks;  // written as the sentinel chunk_base of segment m by the last batch
  uint32_t total_hchunks;
  int32_t m;
  uint32_t total_sblocks;
  SegDesc d[kSegBatch];
};
static_assert(sizeof(SegBatch) <= 4000, "kernel argument block too large");

constexpr int kBits0 = 11, kBits1 = 10, kBits2 = 10;

// Run by one workgroup: stores a batch of segment descriptors (passed as kernel arguments) and
// their initial state; the last batch adds the sentinel descriptor that closes the chunk ranges.
__device__ __forceinline__ void store_segments(const SegBatch& b, SegDesc* __restrict__ seg,
                                               SegState* __restrict__ st,
                                               SegBound* __restrict__ bnd = nullptr) {
  for (int i = threadIdx.x; i < b.count; i += kThreads) {
    seg[b.first + i] = b.d[i];
    if (bnd) {
      SegBound z;
      z.mode = kModeFull; z.b_lo = 0; z.pad[0] = z.pad[1] = 0;
      for (int q = 0; q < kHiCopies; ++q) z.hi[q] = 0;
      bnd[b.first + i] = z;
    }
    SegState s;
    s.prefix = 0; s.k_rem = b.d[i].k; s.T = 0; s.r = 0; s.done = 0;
    s.pad[0] = s.pad[1] = s.pad[2] = 0;
    st[b.first + i] = s;
  }
  if (threadIdx.x == 0 && b.first + b.count == b.m) {
    SegDesc z; z.start = 0; z.size = 0; z.k = 0; z.out_off = 0; z.chunk_base = b.total_chunks;
    z.hchunk_base = b.total_hchunks; z.sblock_base = b.total_sblocks; z.sampled = 0;
    seg[b.m] = z;
  }
}

// Writes one batch of segment descriptors and their initial state; the first batch also
// clears the histograms.
__global__ __launch_bounds__(kThreads) void seg_setup_kernel(SegBatch b, SegDesc* __restrict__ seg,
                                                             SegState* __restrict__ st,
                                                             SegBound* __restrict__ bnd,
                                                             uint32_t* __restrict__ stats,
                                                             uint32_t* __restrict__ zero_from,
                                                             size_t zero_count) {
  if (b.first == 0 && blockIdx.x == 0 && threadIdx.x < DEFT_STAT_WORDS) stats[threadIdx.x] = 0;
  if (b.first == 0) {
    for (size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x; i < zero_count;
         i += (size_t)gridDim.x * kThreads)
      zero_from[i] = 0u;
  }
  if (blockIdx.x == 0) store_segments(b, seg, st, bnd);
}

// Clears the histogram area ahead of time (while the host still plans), for the selection that
// receives its descriptors with the first pass instead of through seg_setup_kernel.
__global__ __launch_bounds__(kThreads) void zero_words_kernel(uint32_t* __restrict__ p, size_t n) {
  for (size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x; i < n; i += (size_t)gridDim.x * kThreads)
    p[i] = 0u;
}

// Exclusive prefix over the wavefront of a per-lane count in [0, 7], by three ballots.
__device__ __forceinline__ uint32_t wave_excl_small(uint32_t cnt, uint32_t& total) {
  const unsigned long long b0 = __ballot(cnt & 1u), b1 = __ballot(cnt & 2u), b2 = __ballot(cnt & 4u);
  const int lane = threadIdx.x & 63;
  const unsigned long long below = (1ull << lane) - 1ull;
  total = (uint32_t)__popcll(b0) + 2u * (uint32_t)__popcll(b1) + 4u * (uint32_t)__popcll(b2);
  return (uint32_t)__popcll(b0 & below) + 2u * (uint32_t)__popcll(b1 & below) +
         4u * (uint32_t)__popcll(b2 & below);
}

// Segment that owns chunk c: largest j in [0, m-1] with seg[j].chunk_base <= c.
__device__ __forceinline__ int seg_of_chunk(const SegDesc* __restrict__ seg, int m, uint32_t c) {
  int lo = 0, hi = m;
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (seg[mid].chunk_base <= c) lo = mid; else hi = mid;
  }
  return lo;
}

__device__ __forceinline__ int seg_of_hchunk(const SegDesc* __restrict__ seg, int m, uint32_t c) {
  int lo = 0, hi = m;
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (seg[mid].hchunk_base <= c) lo = mid; else hi = mid;
  }
  return lo;
}

// A chunk of a segment [s, e): chunk boundaries sit at multiples of 4 elements counted from
// s rounded down to a multiple of 4, so 16-byte loads are aligned; elements outside [s, e) are
// masked.  Wave w of the workgroup owns the w-th quarter of the chunk and lane `lane` loads
// the 16-byte vector (i*64 + lane) of that quarter in step i, so index order inside a wave is
// (step, lane, component).
template <int ITERS>
struct Chunk {
  static constexpr int kElems = kThreads * 4 * ITERS;
  uint32_t key[ITERS][4];
  uint32_t raw[ITERS][4];
  uint32_t vbits[(ITERS + 7) / 8];  // a 4-bit mask of valid components per step, packed

  __device__ __forceinline__ uint32_t vmask(int i) const {
    return (vbits[i >> 3] >> ((i & 7) * 4)) & 0xFu;
  }
  int64_t base;           // absolute index of this thread's vector in step 0

  // Where the chunk sits and whether it lies wholly inside [s, e) (uniform over the workgroup).
  __device__ __forceinline__ bool place(int64_t s, int64_t e, uint32_t local_chunk) {
    const int64_t a = s & ~int64_t(3);
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int64_t cstart = a + (int64_t)local_chunk * kElems;
    base = cstart + ((int64_t)wave * ITERS * 64 + lane) * 4;
    return cstart >= s && cstart + kElems <= e;
  }

  // INTERIOR: all loads in flight together, issued in the order of the steps (the scheduler is
  // kept from reordering them) so that a kernel that walks the steps in order waits for one load
  // at a time instead of for the last one issued.
  template <bool INTERIOR>
  __device__ __forceinline__ void fetch(const float* __restrict__ g, int64_t s, int64_t e) {
    if (INTERIOR) {
      const v4u* __restrict__ p = reinterpret_cast<const v4u*>(g + base);
#pragma unroll
      for (int w = 0; w < (ITERS + 7) / 8; ++w) vbits[w] = 0xFFFFFFFFu;
#pragma unroll
      for (int i = 0; i < ITERS; ++i) {
        const v4u v = __builtin_nontemporal_load(&p[i * 64]);  // streamed: keep it out of L2's way
        raw[i][0] = v.x; raw[i][1] = v.y; raw[i][2] = v.z; raw[i][3] = v.w;
        __builtin_amdgcn_sched_barrier(0);
      }
    } else {
#pragma unroll
      for (int w = 0; w < (ITERS + 7) / 8; ++w) vbits[w] = 0u;
#pragma unroll
      for (int i = 0; i < ITERS; ++i) {
        const int64_t p = base + (int64_t)i * 256;
        if (p >= s && p + 4 <= e) {
          const uint4 v = *reinterpret_cast<const uint4*>(g + p);
          raw[i][0] = v.x; raw[i][1] = v.y; raw[i][2] = v.z; raw[i][3] = v.w;
          vbits[i >> 3] |= 0xFu << ((i & 7) * 4);
        } else {
#pragma unroll
          for (int c = 0; c < 4; ++c) {
            const int64_t q = p + c;
            raw[i][c] = 0;
            if (q >= s && q < e) {
              raw[i][c] = __float_as_uint(g[q]);
              vbits[i >> 3] |= 1u << ((i & 7) * 4 + c);
            }
          }
        }
      }
    }
#pragma unroll
    for (int i = 0; i < ITERS; ++i) {
#pragma unroll
      for (int c = 0; c < 4; ++c) key[i][c] = raw[i][c] & 0x7FFFFFFFu;
    }
  }

  __device__ __forceinline__ void load(const float* __restrict__ g, int64_t s, int64_t e,
                                       uint32_t local_chunk) {
    if (place(s, e, local_chunk)) fetch<true>(g, s, e);
    else fetch<false>(g, s, e);
  }
};

__host__ __device__ inline uint32_t chunks_of(uint32_t start, uint32_t size, uint32_t chunk_elems) {
  if (size == 0) return 0;
  const uint64_t a = start & ~3u;
  return (uint32_t)(((uint64_t)start + size - a + chunk_elems - 1) / chunk_elems);
}

// Histogram storage of one segment: level 0, 1, 2 one after the other, each level in several
// copies -- workgroup b merges into copy b % copies, the bucket search adds them up -- because
// device-scope atomics on one address serialise (about 22 ns each) and a merge sends one per
// workgroup and occupied bin: the tail of the kernels that build a histogram.  Measured on a
// 12 M-element share: first pass 15.0 -> 12.4 us with four copies of level 0; third-level kernel
// 6.7 -> 4.8 us with two copies of levels 1 and 2 (4.3 us with four, but the area to clear grows).
#ifndef DEFT_HIST0_COPIES
#define DEFT_HIST0_COPIES 4
#endif
#ifndef DEFT_HIST12_COPIES
#define DEFT_HIST12_COPIES 2
#endif
constexpr int kRep0 = DEFT_HIST0_COPIES;
constexpr int kRep12 = DEFT_HIST12_COPIES;
// Level 3 is not a fourth digit: it names the 4096-bin histogram that the first pass of a
// sampled long-vector segment builds over the four top digits around the threshold (12 bits of
// 2^10 keys each), which then stands for levels 0 and 1 together.  It has storage of its own, in
// kRepB copies (4, 8 and 16 copies: 219 / 223 / 225 us for the pass over 1.42 GB, within noise of
// each other; the search behind it reads them all: 4.8 / 6.1 / 8.6 us).
// A launch gives at most kMaxSampled segments such a histogram (it samples no more than that).
constexpr int kBitsB = 12;
#ifndef DEFT_BOUNDED_COPIES
#define DEFT_BOUNDED_COPIES 4
#endif
constexpr int kRepB = DEFT_BOUNDED_COPIES;
constexpr int kBoundedStride = (1 << kBitsB) * kRepB;
constexpr int kMaxSampled = 64;
__host__ __device__ constexpr int hist_copies(int level) {
  return level == 0 ? kRep0 : (level == 3 ? kRepB : kRep12);
}
constexpr int kHistStride = (1 << kBits0) * kRep0 + ((1 << kBits1) + (1 << kBits2)) * kRep12;
__host__ __device__ constexpr int hist_offset(int level) {
  return (level == 0 || level == 3) ? 0
                    : (level == 1 ? (1 << kBits0) * kRep0 : (1 << kBits0) * kRep0 + (1 << kBits1) * kRep12);
}

// Run by one whole workgroup: from the finished histogram of level LEVEL (its bins already
// loaded, each thread its own) and the state `s` before that level, locate the bucket holding
// the k_rem-th largest key of the current prefix and return the state after the level (in
// every thread).  If the bucket is taken
// entirely, or this was the last level, the threshold is resolved.
// Bins of a level's histogram owned by a thread of the bucket search: thread t owns the kPer
// bins just below kBins - t*kPer, i.e. threads walk the buckets from the largest keys down.
template <int LEVEL>
struct LevelBins {
  static constexpr int kBits = LEVEL == 0 ? kBits0 : (LEVEL == 1 ? kBits1 : (LEVEL == 2 ? kBits2 : kBitsB));
  static constexpr int kBins = 1 << kBits;
  static constexpr int kPer = kBins / kThreads;
  uint32_t v[kPer];
  __device__ __forceinline__ void load(const uint32_t* __restrict__ gh) {
    const int top = kBins - threadIdx.x * kPer;
#pragma unroll
    for (int q = 0; q < kPer; ++q) v[q] = gh[top - 1 - q];
    // the other copies of the level
#pragma unroll
    for (int c = 1; c < hist_copies(LEVEL); ++c) {
#pragma unroll
      for (int q = 0; q < kPer; ++q) v[q] += gh[c * kBins + top - 1 - q];
    }
  }
};

template <int LEVEL>
__device__ __forceinline__ SegState find_bucket(const LevelBins<LEVEL>& bins, SegState s,
                                                uint32_t* __restrict__ lds /* kWaves + 8 words */) {
  constexpr int kBits = LevelBins<LEVEL>::kBits;
  constexpr int kRemBits = LEVEL == 0 ? (kBits1 + kBits2) : ((LEVEL == 1 || LEVEL == 3) ? kBits2 : 0);
  constexpr int kBins = 1 << kBits;
  constexpr int kPer = kBins / kThreads;
  const int top = kBins - threadIdx.x * kPer;
  const uint32_t (&v)[kPer] = bins.v;
  uint32_t mine = 0;
#pragma unroll
  for (int q = 0; q < kPer; ++q) mine += v[q];
  // exclusive prefix of `mine` over threads (ascending thread = descending key)
  uint32_t inc = mine;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const uint32_t n = __shfl_up(inc, o, 64);
    if (lane >= o) inc += n;
  }
  __syncthreads();
  if (lane == 63) lds[wave] = inc;
  if (threadIdx.x == 0) {
    // result if no bucket qualifies (cannot happen while the histogram holds >= k_rem keys):
    // a threshold above every key, i.e. select nothing
    lds[kWaves + 0] = s.prefix; lds[kWaves + 1] = s.k_rem; lds[kWaves + 2] = 0x80000000u;
    lds[kWaves + 3] = 0u; lds[kWaves + 4] = 1u;
  }
  __syncthreads();
  uint32_t before = inc - mine;
  for (int w = 0; w < wave; ++w) before += lds[w];
  if (before < s.k_rem && s.k_rem <= before + mine) {
    uint32_t above = before;
#pragma unroll
    for (int q = 0; q < kPer; ++q) {
      if (above < s.k_rem && s.k_rem <= above + v[q]) {
        const uint32_t bin = (uint32_t)(top - 1 - q);
        SegState o = s;
        o.prefix = (s.prefix << kBits) | bin;
        o.k_rem = s.k_rem - above;
        if (kRemBits == 0) {
          o.T = o.prefix;
          o.r = o.k_rem;
          o.done = 1;
        } else if (v[q] == o.k_rem) {
          // the whole bucket is taken: every key >= its lowest key is selected
          o.T = o.prefix << kRemBits;
          o.r = 0xFFFFFFFFu;
          o.done = 1;
        }
        lds[kWaves + 0] = o.prefix; lds[kWaves + 1] = o.k_rem; lds[kWaves + 2] = o.T;
        lds[kWaves + 3] = o.r; lds[kWaves + 4] = o.done;
        break;
      }
      above += v[q];
    }
  }
  __syncthreads();
  SegState o = s;
  o.prefix = lds[kWaves + 0]; o.k_rem = lds[kWaves + 1]; o.T = lds[kWaves + 2];
  o.r = lds[kWaves + 3]; o.done = lds[kWaves + 4];
  return o;
}

// State hand-over between the passes.  st[v] (v = 0..3) is the state after v digit levels;
// each pass reads st[LEVEL], and -- when FUSED -- first derives st[LEVEL] itself from
// st[LEVEL-1] and the previous level's histogram (every workgroup repeats that small scan; the
// segment's first workgroup records it for the later passes).  When not FUSED a separate
// one-workgroup-per-segment kernel did it.  The fused form drops three dependent launches,
// which is what bounds short segments; long vectors keep the separate kernels because
// re-reading the histogram in every workgroup would add ~10 % traffic there.
template <int LEVEL_DONE, bool FUSED>
__device__ __forceinline__ SegState state_after(SegState* __restrict__ st, int m, int j,
                                                const uint32_t* __restrict__ hist, bool first_block,
                                                uint32_t* __restrict__ lds) {
  if (!FUSED || LEVEL_DONE == 0) return st[(size_t)LEVEL_DONE * m + j];
  constexpr int kPrev = LEVEL_DONE > 0 ? LEVEL_DONE - 1 : 0;
  // the bins are fetched before the previous state is known (they do not depend on it): one
  // memory round trip less on the critical path of every workgroup
  LevelBins<kPrev> bins;
  bins.load(hist + (size_t)j * kHistStride + hist_offset(kPrev));
  SegState s = st[(size_t)kPrev * m + j];
  if (!s.done) s = find_bucket<kPrev>(bins, s, lds);
  if (first_block && threadIdx.x == 0) st[(size_t)LEVEL_DONE * m + j] = s;
  return s;
}

// Pass 1 (the one full read of the segment): histogram of the top digit (11 bits) of every key.
template <int HITERS>
__device__ __forceinline__ void hist0_chunk(const float* __restrict__ g, const SegDesc& d, int j,
                                            uint32_t* __restrict__ hist, uint32_t* __restrict__ hmax) {
  constexpr int kBins = 1 << kBits0;
  constexpr int kShift = kBits1 + kBits2;
  __shared__ uint32_t lh[kBins];
  for (int b = threadIdx.x; b < kBins; b += kThreads) lh[b] = 0;
  __syncthreads();
  Chunk<HITERS> ch;
  // (the walk is written out once per form of the fetch, so that no control-flow join sits between
  // the loads and their first use: at a join the compiler waits for every load in flight)
  auto walk = [&]() __attribute__((always_inline)) {
#pragma unroll
  for (int i = 0; i < HITERS; ++i) {
    // Runs of equal keys (zero rows of an embedding, clipped or rounded gradients) would send
    // 64 lanes x 4 adds to one LDS address, which serialises.  If the whole wavefront holds one
    // digit in this step -- one ballot to find out -- a single lane adds 256; otherwise every
    // key adds itself.  (Aggregating partial matches per key was measured slower than plain
    // adds on Student-t data: 310 vs 270 us on 1.42 GB; this form costs one ballot per 4 keys.)
    const uint32_t d0 = ch.key[i][0] >> kShift;
    const uint32_t dl = (uint32_t)__builtin_amdgcn_readfirstlane((int)d0);
    const bool same = ch.vmask(i) == 0xF && d0 == dl && (ch.key[i][1] >> kShift) == dl &&
                      (ch.key[i][2] >> kShift) == dl && (ch.key[i][3] >> kShift) == dl;
    if (__ballot(!same) == 0ull) {
      if ((threadIdx.x & 63) == 0) atomicAdd(&lh[dl], 256u);
      continue;
    }
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      if ((ch.vmask(i) >> c) & 1u) atomicAdd(&lh[ch.key[i][c] >> kShift], 1u);
    }
  }
  };
  const int64_t seg_end = (int64_t)d.start + d.size;
  if (ch.place(d.start, seg_end, blockIdx.x - d.hchunk_base)) {
    ch.template fetch<true>(g, d.start, seg_end);
    walk();
  } else {
    ch.template fetch<false>(g, d.start, seg_end);
    walk();
  }
  __syncthreads();
  uint32_t* gh = hist + (size_t)j * kHistStride + hist_offset(0) + (blockIdx.x % kRep0) * kBins;
  int top_bin = 0;
  for (int b = threadIdx.x; b < kBins; b += kThreads) {
    const uint32_t v = lh[b];
    if (v) { atomicAdd(&gh[b], v); top_bin = b; }
  }
  // largest top digit present in the chunk (hmax starts at 0): pass 2 skips chunks that cannot
  // hold a candidate
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) top_bin = max(top_bin, __shfl_down(top_bin, o, 64));
  if ((threadIdx.x & 63) == 0 && top_bin > 0) atomicMax(&hmax[blockIdx.x], (uint32_t)top_bin);
}

template <int HITERS>
__global__ __launch_bounds__(kThreads) void hist0_kernel(const float* __restrict__ g,
                                                         const SegDesc* __restrict__ seg, int m,
                                                         uint32_t* __restrict__ hist,
                                                         uint32_t* __restrict__ hmax) {
  const int j = seg_of_hchunk(seg, m, blockIdx.x);
  const SegDesc d = seg[j];
  hist0_chunk<HITERS>(g, d, j, hist, hmax);
}

// The same pass with the segment descriptors arriving as kernel arguments (all of them: at most
// kSegBatch segments): workgroup 0 also stores them and the initial states for the later
// kernels, which saves the separate set-up launch in front of the dependent chain.  The
// histograms and chunk maxima must have been cleared before (zero_words_kernel).
template <int HITERS>
__global__ __launch_bounds__(kThreads) void hist0_inline_kernel(const float* __restrict__ g, SegBatch b,
                                                                SegDesc* __restrict__ seg,
                                                                SegState* __restrict__ st,
                                                                uint32_t* __restrict__ hist,
                                                                uint32_t* __restrict__ hmax) {
  int lo = 0, hi = b.count;
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (b.d[mid].hchunk_base <= blockIdx.x) lo = mid; else hi = mid;
  }
  const SegDesc d = b.d[lo];
  if (blockIdx.x == 0) store_segments(b, seg, st);
  hist0_chunk<HITERS>(g, d, lo, hist, hmax);
}

// ------------------------------------------------------------------------------------------
// Long vectors: a sample places the threshold ahead of the first pass
// ------------------------------------------------------------------------------------------
// One piece of kSamplePiece consecutive elements out of every block of kSampleBlock (1/128 of the
// segment), at a position inside the block that changes pseudo-randomly from block to block so
// that rows or columns of a matrix cannot line up with it.  A workgroup takes kSamplePiecesPerWg
// pieces (eight lanes per piece, one 16-byte load each, all loads in flight together) and
// histograms their keys on the top digit.
constexpr int kSampleBlock = 4096;
constexpr int kSamplePiece = 32;
constexpr int kSampleRows = 16;
constexpr int kSamplePiecesPerWg = (kThreads / 8) * kSampleRows;
constexpr int kSampleCopies = 2;  // copies of a segment's sample histogram
// A sampled count X of a class holding C of the segment's elements is near p*C with standard
// deviation at most sqrt(p*C) (p = sampled fraction).  The bounds below sit kSampleZ such
// deviations away from p*k; a sample that still misleads is caught by the exact check after the
// first pass, so this number trades speed, never results.  (Six rather than eight: a selection of
// 35 000 from 355 M elements, 277 sampled keys at or above the threshold, then fits its doubt
// into four digits and is read once, 280 instead of 361 us; the inputs built to mislead the
// sample are still the only ones that do.)
#ifndef DEFT_SAMPLE_Z
#define DEFT_SAMPLE_Z 6.0
#endif
constexpr double kSampleZ = DEFT_SAMPLE_Z;

__host__ __device__ inline uint32_t sample_pieces(uint32_t start, uint32_t size) {
  const uint64_t a = ((uint64_t)start + 3) & ~uint64_t(3);
  const uint64_t e = (uint64_t)start + size;
  return e > a ? (uint32_t)((e - a) / kSampleBlock) : 0u;
}

__device__ __forceinline__ int seg_of_sblock(const SegDesc* __restrict__ seg, int m, uint32_t c) {
  int lo = 0, hi = m;
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (seg[mid].sblock_base <= c) lo = mid; else hi = mid;
  }
  return lo;
}

// The sample histogram of a segment borrows the storage of its level-1 and level-2 histograms
// (kSampleCopies x 2048 words = their combined size); bounds_kernel clears it again.
static_assert(kSampleCopies * (1 << kBits0) == ((1 << kBits1) + (1 << kBits2)) * kRep12,
              "the sample histogram must fit the level-1/2 area exactly");

__global__ __launch_bounds__(kThreads) void sample_hist_kernel(const float* __restrict__ g,
                                                               const SegDesc* __restrict__ seg, int m,
                                                               uint32_t* __restrict__ hist) {
  constexpr int kBins = 1 << kBits0;
  constexpr int kShift = kBits1 + kBits2;
  __shared__ uint32_t lh[kBins];
  for (int b = threadIdx.x; b < kBins; b += kThreads) lh[b] = 0;
  const int j = seg_of_sblock(seg, m, blockIdx.x);
  const SegDesc d = seg[j];
  const uint32_t pieces = sample_pieces(d.start, d.size);
  const uint64_t a = ((uint64_t)d.start + 3) & ~uint64_t(3);
  const uint32_t first = (blockIdx.x - d.sblock_base) * kSamplePiecesPerWg + (threadIdx.x >> 3);
  v4u v[kSampleRows];
  uint32_t have = 0;
#pragma unroll
  for (int r = 0; r < kSampleRows; ++r) {
    const uint32_t q = first + r * (kThreads / 8);
    v[r] = v4u{0u, 0u, 0u, 0u};
    if (q < pieces) {
      const uint32_t off = ((q * 2654435761u) >> 25) & (kSampleBlock / kSamplePiece - 1);
      const uint64_t at = a + (uint64_t)q * kSampleBlock + off * kSamplePiece + (threadIdx.x & 7) * 4;
      v[r] = *reinterpret_cast<const v4u*>(g + at);
      have |= 1u << r;
    }
  }
  __syncthreads();
#pragma unroll
  for (int r = 0; r < kSampleRows; ++r) {
    if ((have >> r) & 1u) {
      atomicAdd(&lh[(v[r].x & 0x7FFFFFFFu) >> kShift], 1u);
      atomicAdd(&lh[(v[r].y & 0x7FFFFFFFu) >> kShift], 1u);
      atomicAdd(&lh[(v[r].z & 0x7FFFFFFFu) >> kShift], 1u);
      atomicAdd(&lh[(v[r].w & 0x7FFFFFFFu) >> kShift], 1u);
    }
  }
  __syncthreads();
  uint32_t* gh = hist + (size_t)j * kHistStride + hist_offset(1) + (blockIdx.x % kSampleCopies) * kBins;
  for (int b = threadIdx.x; b < kBins; b += kThreads) {
    const uint32_t c = lh[b];
    if (c) atomicAdd(&gh[b], c);
  }
}

// Largest bin b whose count of keys at or above it reaches `thr` (thr >= 1), given each thread's
// bins and the count above them; written to *out by the one thread that holds it, together with
// that count.  Nothing is written if the whole histogram holds fewer than thr keys.
__device__ __forceinline__ void crossing_bin(const LevelBins<0>& bins, uint32_t before, uint32_t thr,
                                             uint32_t* out) {
  constexpr int kPer = LevelBins<0>::kPer;
  const int top = LevelBins<0>::kBins - threadIdx.x * kPer;
  uint32_t above = before;
#pragma unroll
  for (int q = 0; q < kPer; ++q) {
    if (above < thr && thr <= above + bins.v[q]) { out[0] = (uint32_t)(top - 1 - q); out[1] = above + bins.v[q]; }
    above += bins.v[q];
  }
}

// One workgroup per segment: from the sample histogram, the top digit b_lo such that the
// threshold's top digit is one of b_lo .. b_lo + 3 beyond reasonable doubt -- or the decision to treat
// the segment in full (not sampled, too few samples to tell, the sample's doubt spanning more
// than four digits, or too many keys at or above b_lo to park).
__global__ __launch_bounds__(kThreads) void bounds_kernel(const SegDesc* __restrict__ seg,
                                                          uint32_t* __restrict__ hist,
                                                          SegBound* __restrict__ bnd,
                                                          uint32_t* __restrict__ flags) {
  __shared__ uint32_t wsum[kWaves];
  __shared__ uint32_t res[4];
  const int j = blockIdx.x;
  const SegDesc d = seg[j];
  if (!d.sampled) {  // bnd[j] already says kModeFull
    if (threadIdx.x == 0) atomicOr(flags, kFlagPass2);
    return;
  }
  uint32_t* gh = hist + (size_t)j * kHistStride + hist_offset(1);
  LevelBins<0> bins;
  {
    constexpr int kPer = LevelBins<0>::kPer;
    const int top = LevelBins<0>::kBins - threadIdx.x * kPer;
#pragma unroll
    for (int q = 0; q < kPer; ++q) {
      uint32_t c = 0;
#pragma unroll
      for (int r = 0; r < kSampleCopies; ++r) {
        c += gh[r * LevelBins<0>::kBins + top - 1 - q];
        gh[r * LevelBins<0>::kBins + top - 1 - q] = 0;  // hand the area back cleared
      }
      bins.v[q] = c;
    }
  }
  uint32_t mine = 0;
#pragma unroll
  for (int q = 0; q < LevelBins<0>::kPer; ++q) mine += bins.v[q];
  uint32_t inc = mine;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const uint32_t n = __shfl_up(inc, o, 64);
    if (lane >= o) inc += n;
  }
  if (lane == 63) wsum[wave] = inc;
  if (threadIdx.x == 0) { res[0] = 0; res[1] = 0; res[2] = 0xFFFFFFFFu; res[3] = 0; }
  __syncthreads();
  uint32_t before = inc - mine;
  for (int w = 0; w < wave; ++w) before += wsum[w];
  const uint32_t n_s = sample_pieces(d.start, d.size) * kSamplePiece;
  const double pk = (double)d.k * (double)n_s / (double)d.size;
  const double dev = kSampleZ * sqrt(pk) + 1.0;
  const uint32_t hi_thr = (uint32_t)ceil(pk + dev);
  const double lo_real = pk - dev;
  const uint32_t lo_thr = lo_real >= 0.0 ? (uint32_t)floor(lo_real) + 1u : 0u;
  // b_lo: keys at or above it number at least k beyond doubt.  b_hi: keys above it number fewer
  // than k beyond doubt.
  if (hi_thr <= n_s) crossing_bin(bins, before, hi_thr, &res[0]);
  if (lo_thr >= 1) crossing_bin(bins, before, lo_thr, &res[2]);
  __syncthreads();
  if (threadIdx.x == 0) {
    const uint32_t b_lo = res[0], at_or_above = res[1], b_hi = res[2];
    const bool ok = hi_thr <= n_s && lo_thr >= 1 && b_hi != 0xFFFFFFFFu && b_hi <= b_lo + 3 &&
                    (uint64_t)at_or_above * kParkDiv <= n_s;  // parks 1/kParkDiv of the segment at most
    bnd[j].mode = ok ? kModeBounded : kModeFull;
    bnd[j].b_lo = b_lo;
    if (!ok) atomicOr(flags, kFlagPass2);
  }
}

// Pass 1 for long vectors.  Merging a workgroup's histogram into the segment's costs one
// device-scope atomic per occupied bin; with one chunk per workgroup that merge took a quarter
// of the pass on a 1.4 GB vector (281 us; 211 us with the merge left out, 238 / 219 us when
// only every 4th / 20th workgroup merged).  Here a resident set of workgroups draws chunks from
// a counter (the next draw is issued before the current chunk is processed) and keeps
// accumulating in LDS; a workgroup merges when its next chunk belongs to another segment and
// when the chunks run out.  The counter only grows, so every workgroup leaves its loop.
//   kModeFull segments: histogram of the top digit of every key, largest top digit per chunk.
//   kModeBounded segments: keys whose top digit is at least b_lo are parked as in pass 2 (one
//     wavefront per count/emit chunk, index order) and, where the digit is one of b_lo .. b_lo + 3,
//     histogrammed on (key - (b_lo << 20)) >> 10, i.e. on their top 21 bits; keys above those four
//     digits are counted.  Nearly every step finds nothing to park: four compares and a ballot.
//   REDO launch: only the segments whose bound failed its check, treated as kModeFull; a no-op
//     (every workgroup leaves at once) unless the flag word says that some bound failed.
// Pass 1 for long vectors.  Merging a workgroup's histogram into the segment's costs one
// device-scope atomic per occupied bin; with one chunk per workgroup that merge took a quarter
// of the pass on a 1.4 GB vector (281 us; 211 us with the merge left out, 238 / 219 us when
// only every 4th / 20th workgroup merged).  Here a resident set of workgroups draws chunks from
// a counter (the next draw is issued before the current chunk is processed) and keeps
// accumulating in LDS; a workgroup merges when its next chunk belongs to another segment and
// when the chunks run out.  The counter only grows, so every workgroup leaves its loop.  The
// largest top digit of each chunk comes from the keys (the LDS histogram now spans chunks).
// With `bnd` (some segment of the launch was sampled) the pass covers only the segments that are
// not, or no longer, kModeBounded, and is a no-op unless the flag word says there are any.
template <int HITERS>
__global__ __launch_bounds__(kThreads) void hist0_stream_kernel(
    const float* __restrict__ g, const SegDesc* __restrict__ seg, int m, uint32_t hchunks,
    uint32_t* __restrict__ hist, uint32_t* __restrict__ hmax, uint32_t* __restrict__ next_chunk,
    const SegBound* __restrict__ bnd, const uint32_t* __restrict__ flags) {
  constexpr int kBins = 1 << kBits0;
  constexpr int kShift = kBits1 + kBits2;
  __shared__ uint32_t lh[kBins];
  __shared__ uint32_t draw[2];
  if (bnd && !(*flags & kFlagPass2)) return;
  for (int b = threadIdx.x; b < kBins; b += kThreads) lh[b] = 0;
  if (threadIdx.x == 0) draw[0] = atomicAdd(next_chunk, 1u);
  __syncthreads();
  uint32_t c = draw[0];
  int cur = -1, turn = 0;
  while (c < hchunks) {
    if (threadIdx.x == 0) draw[turn ^ 1] = atomicAdd(next_chunk, 1u);
    const int j = seg_of_hchunk(seg, m, c);
    if (bnd && bnd[j].mode == kModeBounded) {  // read once already, candidates parked
      __syncthreads();
      turn ^= 1;
      c = draw[turn];
      continue;
    }
    if (j != cur) {
      if (cur >= 0) {
        uint32_t* gh = hist + (size_t)cur * kHistStride + hist_offset(0) + (blockIdx.x % kRep0) * kBins;
        for (int b = threadIdx.x; b < kBins; b += kThreads) {
          const uint32_t v = lh[b];
          if (v) { atomicAdd(&gh[b], v); lh[b] = 0; }
        }
        __syncthreads();
      }
      cur = j;
    }
    const SegDesc d = seg[j];
    Chunk<HITERS> ch;
    ch.load(g, d.start, (int64_t)d.start + d.size, c - d.hchunk_base);
    uint32_t mx = 0;
#pragma unroll
    for (int i = 0; i < HITERS; ++i) {
      mx = max(mx, max(max(ch.key[i][0], ch.key[i][1]), max(ch.key[i][2], ch.key[i][3])));
      // a wavefront whose 256 keys of a step share one digit adds once (see hist0_kernel)
      const uint32_t d0 = ch.key[i][0] >> kShift;
      const uint32_t dl = (uint32_t)__builtin_amdgcn_readfirstlane((int)d0);
      const bool same = ch.vmask(i) == 0xF && d0 == dl && (ch.key[i][1] >> kShift) == dl &&
                        (ch.key[i][2] >> kShift) == dl && (ch.key[i][3] >> kShift) == dl;
      if (__ballot(!same) == 0ull) {
        if ((threadIdx.x & 63) == 0) atomicAdd(&lh[dl], 256u);
        continue;
      }
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        if ((ch.vmask(i) >> q) & 1u) atomicAdd(&lh[ch.key[i][q] >> kShift], 1u);
      }
    }
    int top_bin = (int)(mx >> kShift);  // masked elements carry key 0
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) top_bin = max(top_bin, __shfl_down(top_bin, o, 64));
    if ((threadIdx.x & 63) == 0 && top_bin > 0) atomicMax(&hmax[c], (uint32_t)top_bin);
    __syncthreads();  // the chunk is in the histogram and draw[turn ^ 1] is visible
    turn ^= 1;
    c = draw[turn];
  }
  if (cur < 0) return;
  uint32_t* gh = hist + (size_t)cur * kHistStride + hist_offset(0) + (blockIdx.x % kRep0) * kBins;
  for (int b = threadIdx.x; b < kBins; b += kThreads) {
    const uint32_t v = lh[b];
    if (v) atomicAdd(&gh[b], v);
  }
}

// The first pass over the kModeBounded segments of a long vector: one workgroup per histogram
// chunk, one wavefront per count/emit chunk.  Keys whose top digit is at least b_lo are parked as
// in pass 2 (index order) and, where the digit is one of b_lo .. b_lo + 3, histogrammed on
// (key - (b_lo << 20)) >> 10, i.e. on their top 21 bits; keys above those four digits are
// counted.  Nearly every step finds nothing to park: four compares and a ballot.
// A wavefront walks its 8192 elements in batches of kBatchVecs 16-byte vectors per lane, the next
// batch in flight while the current one is processed, in a loop that is kept rolled: the pass
// needs few registers (a chunk held whole, 32 vectors per lane, costs 256 and leaves one
// wavefront per SIMD: 310 us on 1.42 GB), so that many wavefronts per SIMD keep loads in flight.
#ifndef DEFT_PASS1_BATCH
#define DEFT_PASS1_BATCH 32
#endif
#ifndef DEFT_PASS1_DOUBLE
#define DEFT_PASS1_DOUBLE 0
#endif
constexpr int kBatchVecs = DEFT_PASS1_BATCH;
constexpr bool kBatchDouble = DEFT_PASS1_DOUBLE != 0;

struct VecBatch {
  v4u v[kBatchVecs];
  uint32_t valid[(kBatchVecs + 7) / 8];  // 4 bits per vector: which components lie inside the segment
  __device__ __forceinline__ uint32_t vmask(int i) const { return (valid[i >> 3] >> ((i & 7) * 4)) & 0xFu; }
};

// Loads vectors t0 .. t0 + kBatchVecs - 1 of this lane (vector t sits 256 * t elements behind
// `at`, the lane's first).  INTERIOR: the whole chunk lies inside [s, e).
template <bool INTERIOR>
__device__ __forceinline__ void load_batch(VecBatch& b, const float* __restrict__ g, int64_t at, int t0,
                                           int64_t s, int64_t e) {
  if (INTERIOR) {
    const v4u* __restrict__ p = reinterpret_cast<const v4u*>(g + at);
#pragma unroll
    for (int i = 0; i < kBatchVecs; ++i) b.v[i] = __builtin_nontemporal_load(&p[(t0 + i) * 64]);
    return;
  }
#pragma unroll
  for (int w = 0; w < (kBatchVecs + 7) / 8; ++w) b.valid[w] = 0;
#pragma unroll
  for (int i = 0; i < kBatchVecs; ++i) {
    const int64_t p = at + (int64_t)(t0 + i) * 256;
    uint32_t x[4] = {0u, 0u, 0u, 0u};
    if (p >= s && p + 4 <= e) {
      const uint4 w = *reinterpret_cast<const uint4*>(g + p);
      x[0] = w.x; x[1] = w.y; x[2] = w.z; x[3] = w.w;
      b.valid[i >> 3] |= 0xFu << ((i & 7) * 4);
    } else {
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        if (p + c >= s && p + c < e) {
          x[c] = __float_as_uint(g[p + c]);
          b.valid[i >> 3] |= 1u << ((i & 7) * 4 + c);
        }
      }
    }
    b.v[i] = v4u{x[0], x[1], x[2], x[3]};
  }
}

// The walk of one wavefront over its count/emit chunk.  The common step finds nothing to park
// (four compares and a ballot); the next most common finds at most one key per lane (one ballot
// places them); only a step in which some lane holds several takes the general three-ballot
// prefix.  Parked entries go to a staging array in LDS first and leave it when it is nearly full
// and at the end of the walk, 64 at a time: dense stores to the chunk's slots, and the histogram
// update with every lane busy instead of once per sparse step.  (A wavefront instruction
// occupies its SIMD for four cycles, which at full memory rate leaves about twenty of them per
// element on the whole chip.)
#ifndef DEFT_LONG_CAP_MULT
#define DEFT_LONG_CAP_MULT 8
#endif
#ifndef DEFT_STAGE_MULT
#define DEFT_STAGE_MULT 2
#endif
constexpr uint32_t kLongSlotCap = DEFT_LONG_CAP_MULT * kMaxSlotCap;  // the slot capacity of the long-vector shape
// ... and of the short one: a quarter of a chunk as well (with 256 slots the NCF-shaped
// conventional Top-k at d = 0.1 overflowed wherever it selects: 159 us, 143 us with 1024; the
// sparse sets do not notice).
#ifndef DEFT_SHORT_CAP_MULT
#define DEFT_SHORT_CAP_MULT 4
#endif
constexpr uint32_t kShortSlotCap = DEFT_SHORT_CAP_MULT * kMaxSlotCap;
// Entries a wavefront of the bounded first pass holds in LDS before it moves them to the slots: a
// step adds 256 at most, so the staging array is emptied whenever fewer than that are free.
constexpr uint32_t kStageCap = DEFT_STAGE_MULT * kMaxSlotCap;
static_assert(kStageCap >= 512, "a step of the walk may park 256 entries");
template <int HITERS, bool INTERIOR>
__device__ __forceinline__ uint32_t park_chunk(const float* __restrict__ g, int64_t at, int64_t s,
                                               int64_t e, uint32_t lo_key, uint32_t* __restrict__ lh,
                                               uint2* __restrict__ stage, uint2* __restrict__ my_slots,
                                               uint32_t cap) {
  constexpr int kBinsB = 1 << kBitsB;
  constexpr int kShift = kBits1 + kBits2;
  constexpr int kBatches = HITERS / kBatchVecs;
  const int lane = threadIdx.x & 63;
  const unsigned long long below = (1ull << lane) - 1ull;
  uint32_t filled = 0;   // entries parked so far
  uint32_t flushed = 0;  // of which have left the staging array
  uint32_t low_set = 0;
  auto bin_of = [&](uint32_t rawv) {
    const uint32_t rel = (rawv & 0x7FFFFFFFu) - lo_key;
    return rel < (4u << kShift) ? (rel >> kBits2) : (uint32_t)kBinsB;
  };
  auto one = [&](uint32_t rawv, uint32_t idx, uint32_t pos) { stage[pos - flushed] = make_uint2(rawv, idx); };
  // The staged entries (written and read by this wavefront only) leave for the slots, every lane
  // busy: dense stores, and the histogram update.  Entries beyond the slots are counted, not kept.
  auto flush = [&]() {
    for (uint32_t r = lane; r < filled - flushed; r += 64) {
      const uint2 en = stage[r];
      if (flushed + r < cap) my_slots[flushed + r] = en;
      atomicAdd(&lh[bin_of(en.x)], 1u);
      low_set += (en.x & ((1u << kBits2) - 1u)) ? 1u : 0u;
    }
    flushed = filled;
  };
  auto park = [&](const VecBatch& B, int t0) {
#pragma unroll
    for (int i = 0; i < kBatchVecs; ++i) {
      const uint32_t vm = INTERIOR ? 0xFu : B.vmask(i);
      const uint32_t raw[4] = {B.v[i].x, B.v[i].y, B.v[i].z, B.v[i].w};
      bool l[4];
#pragma unroll
      for (int q = 0; q < 4; ++q) l[q] = ((vm >> q) & 1u) && (raw[q] & 0x7FFFFFFFu) >= lo_key;
      const bool any = l[0] || l[1] || l[2] || l[3];
      const unsigned long long anyb = __ballot(any);
      if (anyb == 0ull) continue;
      if (filled - flushed > kStageCap - 256u) flush();  // room for whatever this step parks
      const uint32_t idx0 = (uint32_t)(at + (int64_t)(t0 + i) * 256);
      const uint32_t cnt = (uint32_t)l[0] + (uint32_t)l[1] + (uint32_t)l[2] + (uint32_t)l[3];
      if (__ballot(cnt > 1u) == 0ull) {
        // at most one key per lane: its slot is the number of lanes with a key below this one
        if (any) {
          const uint32_t comp = l[0] ? 0u : (l[1] ? 1u : (l[2] ? 2u : 3u));
          const uint32_t rawv = l[0] ? raw[0] : (l[1] ? raw[1] : (l[2] ? raw[2] : raw[3]));
          one(rawv, idx0 + comp, filled + (uint32_t)__popcll(anyb & below));
        }
        filled += (uint32_t)__popcll(anyb);
        continue;
      }
      uint32_t tot;
      uint32_t pos = filled + wave_excl_small(cnt, tot);
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        if (l[q]) {
          one(raw[q], idx0 + q, pos);
          ++pos;
        }
      }
      filled += tot;
    }
  };
  VecBatch bufA;
  load_batch<INTERIOR>(bufA, g, at, 0, s, e);
  __syncthreads();  // the workgroup's histogram is cleared
  if (kBatchDouble) {
    // two batches in turn: one being processed, the other in flight
    VecBatch bufB;
#pragma unroll 1
    for (int bt = 0; bt < kBatches; bt += 2) {
      load_batch<INTERIOR>(bufB, g, at, (bt + 1) * kBatchVecs, s, e);
      park(bufA, bt * kBatchVecs);
      if (bt + 2 < kBatches) load_batch<INTERIOR>(bufA, g, at, (bt + 2) * kBatchVecs, s, e);
      park(bufB, (bt + 1) * kBatchVecs);
    }
  } else {
#pragma unroll 1
    for (int bt = 0; bt < kBatches; ++bt) {
      if (bt) load_batch<INTERIOR>(bufA, g, at, bt * kBatchVecs, s, e);
      park(bufA, bt * kBatchVecs);
    }
  }
  flush();
  // how many parked keys have any of their low kBits2 bits set: if none has (gradients that
  // went through a 16-bit format), the 21 bits resolved by this pass are the whole key
  if (__ballot(low_set != 0) != 0ull) {
    low_set = wave_sum_u32(low_set);
    if (lane == 0) atomicAdd(&lh[kBinsB + 2], low_set);
  }
  return filled;
}

template <int HITERS>
__global__ __launch_bounds__(kThreads) void pass1_bounded_kernel(
    const float* __restrict__ g, const SegDesc* __restrict__ seg, int m, uint32_t* __restrict__ bhist,
    SegBound* __restrict__ bnd, uint32_t* __restrict__ live_cnt, uint2* __restrict__ slots,
    uint32_t cap) {
  constexpr int kBinsB = 1 << kBitsB;
  constexpr int kShift = kBits1 + kBits2;
  static_assert(HITERS % kBatchVecs == 0 && (!kBatchDouble || HITERS % (2 * kBatchVecs) == 0),
                "a wavefront's vectors split into whole batches (pairs of them when double-buffered)");
  constexpr int kElems = kThreads * 4 * HITERS;  // elements of a histogram chunk
  // kBinsB bins over the four digits, the count of the keys above them in [kBinsB], in
  // [kBinsB + 1] whether this workgroup has parked anything at all, in [kBinsB + 2] the number of
  // parked keys with a low bit set
  __shared__ uint32_t lh[kBinsB + 3];
  __shared__ uint2 stage[kWaves][kStageCap];
  const int j = seg_of_hchunk(seg, m, blockIdx.x);
  if (bnd[j].mode != kModeBounded) return;
  for (int b = threadIdx.x; b < kBinsB + 3; b += kThreads) lh[b] = 0;
  const SegDesc d = seg[j];
#ifdef DEFT_PROBE_NOPARK  // measurement only: nothing is ever parked (the check then fails: redone in full)
  const uint32_t lo_key = (bnd[j].b_lo << kShift) | 0x7FF00000u;
#else
  const uint32_t lo_key = bnd[j].b_lo << kShift;
#endif
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const uint32_t local = blockIdx.x - d.hchunk_base;
  const int64_t s = d.start, e = (int64_t)d.start + d.size;
  const int64_t cstart = (s & ~int64_t(3)) + (int64_t)local * kElems;
  // this lane's first vector: wave w owns the w-th quarter of the chunk
  const int64_t at = cstart + ((int64_t)wave * HITERS * 64 + lane) * 4;
  const uint32_t n_chunks = seg[j + 1].chunk_base - d.chunk_base;
  const uint32_t ec_local = local * 4 + wave;  // this wave's count/emit chunk
  uint2* my_slots = slots + (size_t)(d.chunk_base + ec_local) * cap;
  const uint32_t filled = (cstart >= s && cstart + kElems <= e)
                              ? park_chunk<HITERS, true>(g, at, s, e, lo_key, lh, stage[wave], my_slots, cap)
                              : park_chunk<HITERS, false>(g, at, s, e, lo_key, lh, stage[wave], my_slots, cap);
  if (lane == 0) {
    if (ec_local < n_chunks) live_cnt[d.chunk_base + ec_local] = filled;
    if (filled) lh[kBinsB + 1] = 1u;
  }
  __syncthreads();
  if (!lh[kBinsB + 1]) return;  // nothing parked (the common case in layers of small magnitude)
  uint32_t* gh = bhist + (size_t)(d.sampled - 1) * kBoundedStride + (blockIdx.x % kRepB) * kBinsB;
  for (int b = threadIdx.x; b < kBinsB; b += kThreads) {
    const uint32_t v = lh[b];
    if (v) atomicAdd(&gh[b], v);
  }
  if (threadIdx.x == 0 && (lh[kBinsB] | lh[kBinsB + 2]))
    atomicAdd(&bnd[j].hi[blockIdx.x % kHiCopies],
              (unsigned long long)lh[kBinsB] | ((unsigned long long)lh[kBinsB + 2] << 32));
}

// Pass 2 (the second, partial read).  The top digit b0 of the threshold is known.  Every key that can
// still be selected -- top digit above b0 (selected for sure) or equal to b0 ("candidates"; the
// two together are about as many as k) -- is parked with its index in a small per-chunk slot
// array, in index order; candidates are also histogrammed on their next digit.  The remaining
// digit level, the per-chunk counts AND the final ordered write are then worked out from the
// slots, without reading the segment again.  A chunk with more such keys than slots is marked
// by its count; the later kernels read that chunk from the segment instead (heavy ties, dense
// selections).  A workgroup handles one histogram chunk = 4 count/emit chunks, one per
// wavefront; a slot entry is {value bits, global index}.
template <int ITERS, bool FUSED>
__global__ __launch_bounds__(kThreads) void pass2_kernel(
    const float* __restrict__ g, const SegDesc* __restrict__ seg, SegState* __restrict__ st, int m,
    uint32_t* __restrict__ hist, const uint32_t* __restrict__ hmax, uint32_t* __restrict__ live_cnt,
    uint2* __restrict__ slots, uint32_t cap, const SegBound* __restrict__ bnd,
    const uint32_t* __restrict__ flags) {
  constexpr int HITERS = 4 * ITERS;
  constexpr int kBins = 1 << kBits1;
  __shared__ uint32_t lh[kBins];
  __shared__ uint32_t fl[kWaves + 8];
  // long vectors: nothing to do if the first pass has parked every segment's candidates itself
  if (!FUSED && bnd && !(*flags & kFlagPass2)) return;
  const int j = seg_of_hchunk(seg, m, blockIdx.x);
  if (!FUSED && bnd && bnd[j].mode == kModeBounded) return;
  const SegDesc d = seg[j];
  const uint32_t local = blockIdx.x - d.hchunk_base;
  const uint32_t my_max = hmax[blockIdx.x];  // fetched ahead of the bucket search
  const uint32_t n_chunks = seg[j + 1].chunk_base - d.chunk_base;
  const SegState s = state_after<1, FUSED>(st, m, j, hist, local == 0, fl);
  const uint32_t b0 = s.done ? (s.T >> (kBits1 + kBits2)) : s.prefix;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const uint32_t ec_local = local * 4 + wave;        // this wave's count/emit chunk
  const bool have_chunk = ec_local < n_chunks;
  if (my_max < b0) {
    // every key here lies below the threshold's bucket: nothing to park, no read
    if (lane == 0 && have_chunk) live_cnt[d.chunk_base + ec_local] = 0;
    return;
  }
  for (int b = threadIdx.x; b < kBins; b += kThreads) lh[b] = 0;
  __syncthreads();
  Chunk<HITERS> ch;
  uint2* my_slots = slots + (size_t)(d.chunk_base + ec_local) * cap;
  uint32_t filled = 0;
  // (written out once per form of the fetch: no join between the loads and their first use)
  auto walk = [&]() __attribute__((always_inline)) {
#pragma unroll
  for (int i = 0; i < HITERS; ++i) {
    uint32_t livem = 0;
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      const bool on = (ch.vmask(i) >> c) & 1u;
      livem |= (on && (ch.key[i][c] >> (kBits1 + kBits2)) >= b0) ? (1u << c) : 0u;
    }
    if (__ballot(livem != 0) == 0ull) continue;
    uint32_t tot;
    uint32_t pos = filled + wave_excl_small((uint32_t)__popc(livem), tot);
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      if ((livem >> c) & 1u) {
        const uint32_t key = ch.key[i][c];
        if (!s.done && (key >> (kBits1 + kBits2)) == b0) atomicAdd(&lh[(key >> kBits2) & (kBins - 1)], 1u);
        if (pos < cap) my_slots[pos] = make_uint2(ch.raw[i][c], (uint32_t)(ch.base + (int64_t)i * 256 + c));
        ++pos;
      }
    }
    filled += tot;
  }
  };
  const int64_t seg_end = (int64_t)d.start + d.size;
  if constexpr (FUSED) {
    if (ch.place(d.start, seg_end, local)) {
      ch.template fetch<true>(g, d.start, seg_end);
      walk();
    } else {
      ch.template fetch<false>(g, d.start, seg_end);
      walk();
    }
  } else {
    // (long vectors: twice the registers per chunk; the two copies of the walk cost the kernel a
    // third of its resident wavefronts, and other workgroups cover a wavefront's wait there)
    ch.load(g, d.start, seg_end, local);
    walk();
  }
  if (lane == 0 && have_chunk) live_cnt[d.chunk_base + ec_local] = filled;
  __syncthreads();
  if (s.done) return;
  uint32_t* gh = hist + (size_t)j * kHistStride + hist_offset(1) + (blockIdx.x % kRep12) * kBins;
  for (int b = threadIdx.x; b < kBins; b += kThreads) {
    const uint32_t v = lh[b];
    if (v) atomicAdd(&gh[b], v);
  }
}

// Last digit level, from the slots.  One workgroup per count/emit chunk, a thread per slot
// entry and round; a chunk whose candidates overflowed its slots is read from the segment instead.
template <int ITERS, bool FUSED>
__global__ __launch_bounds__(kThreads) void slot_hist2_kernel(
    const float* __restrict__ g, const SegDesc* __restrict__ seg, SegState* __restrict__ st, int m,
    uint32_t* __restrict__ hist, const uint32_t* __restrict__ live_cnt,
    const uint2* __restrict__ slots, uint32_t cap) {
  constexpr int kBins = 1 << kBits2;
  __shared__ uint32_t lh[kBins];
  __shared__ uint32_t fl[kWaves + 8];
  const int j = seg_of_chunk(seg, m, blockIdx.x);
  const SegDesc d = seg[j];
  const uint32_t local = blockIdx.x - d.chunk_base;
  const uint32_t n = live_cnt[blockIdx.x];
  // nothing parked here: no need for the state (the segment's first workgroup records it)
  if (n == 0 && (!FUSED || local != 0)) return;
  const SegState s = state_after<2, FUSED>(st, m, j, hist, local == 0, fl);
  if (s.done || n == 0) return;
  uint32_t* gh = hist + (size_t)j * kHistStride + hist_offset(2) + (blockIdx.x % kRep12) * kBins;
  if (n <= cap) {
    for (uint32_t r0 = 0; r0 < n; r0 += kThreads) {
      const bool on = r0 + threadIdx.x < n;
      const uint32_t e = on ? (slots[(size_t)blockIdx.x * cap + r0 + threadIdx.x].x & 0x7FFFFFFFu) : 0u;
      bool live = on && (e >> kBits2) == s.prefix;  // the threshold's first two digits
      const uint32_t digit = e & (kBins - 1);
      // equal digits are common (rounded gradients): one atomic per distinct digit and wave
      unsigned long long act = __ballot(live);
      while (act) {
        const int leader = __ffsll((long long)act) - 1;
        const uint32_t dl = (uint32_t)__builtin_amdgcn_readlane((int)digit, leader);
        const unsigned long long same = __ballot(live && digit == dl);
        if ((int)(threadIdx.x & 63) == leader) atomicAdd(&gh[dl], (uint32_t)__popcll(same));
        if (live && digit == dl) live = false;
        act &= ~same;
      }
    }
    return;
  }
  for (int b = threadIdx.x; b < kBins; b += kThreads) lh[b] = 0;
  __syncthreads();
  Chunk<ITERS> ch;
  ch.load(g, d.start, (int64_t)d.start + d.size, local);
#pragma unroll
  for (int i = 0; i < ITERS; ++i) {
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      const uint32_t key = ch.key[i][c];
      if (((ch.vmask(i) >> c) & 1u) && (key >> kBits2) == s.prefix) atomicAdd(&lh[key & (kBins - 1)], 1u);
    }
  }
  __syncthreads();
  for (int b = threadIdx.x; b < kBins; b += kThreads) {
    const uint32_t v = lh[b];
    if (v) atomicAdd(&gh[b], v);
  }
}

// One workgroup per segment: st[LEVEL+1] from st[LEVEL] and the level's histogram (the
// unfused form of the hand-over).
template <int LEVEL>
__global__ __launch_bounds__(kThreads) void find_kernel(SegState* __restrict__ st, int m,
                                                        const uint32_t* __restrict__ hist,
                                                        const SegBound* __restrict__ bnd,
                                                        uint32_t* __restrict__ flags) {
  __shared__ uint32_t fl[kWaves + 8];
  const int j = blockIdx.x;
  // a segment whose first pass covered two digit levels already has its state after level 1
  if (LEVEL <= 1 && bnd && bnd[j].mode == kModeBounded) return;
  SegState s = st[(size_t)LEVEL * m + j];
  LevelBins<LEVEL> bins;
  bins.load(hist + (size_t)j * kHistStride + hist_offset(LEVEL));
  if (!s.done) s = find_bucket<LEVEL>(bins, s, fl);
  if (threadIdx.x == 0) {
    st[(size_t)(LEVEL + 1) * m + j] = s;
    if (LEVEL == 1 && flags && !s.done) atomicOr(flags, kFlagLevel2);
  }
}

// The exact check behind the first pass over kModeBounded segments, one workgroup per segment:
// with c_hi keys above the four digits and c_mid keys inside them, the threshold lies inside iff
// c_hi < k <= c_hi + c_mid.  If so, the bucket search over the 4096-bin histogram gives the state
// after TWO digit levels (the full first pass, pass 2 and the searches of levels 0 and 1 then
// skip the segment).  If not -- the sample misled -- the segment is marked kModeFailed and the
// launches that follow treat it in full.
__global__ __launch_bounds__(kThreads) void find_first_kernel(SegState* __restrict__ st, int m,
                                                              const SegDesc* __restrict__ seg,
                                                              const uint32_t* __restrict__ bhist,
                                                              SegBound* __restrict__ bnd,
                                                              uint32_t* __restrict__ flags,
                                                              uint32_t* __restrict__ stats) {
  __shared__ uint32_t fl[kWaves + 8];
  __shared__ uint32_t wsum[kWaves];
  const int j = blockIdx.x;
  if (bnd[j].mode != kModeBounded) {
    if (threadIdx.x == 0) atomicAdd(&stats[DEFT_STAT_FULL], 1u);
    return;
  }
  const SegState s = st[j];
  LevelBins<3> bins;
  bins.load(bhist + (size_t)(seg[j].sampled - 1) * kBoundedStride);
  uint32_t mid = 0;
#pragma unroll
  for (int q = 0; q < LevelBins<3>::kPer; ++q) mid += bins.v[q];
  mid = wave_sum_u32(mid);
  if ((threadIdx.x & 63) == 0) wsum[threadIdx.x >> 6] = mid;
  __syncthreads();
  const uint32_t c_mid = wsum[0] + wsum[1] + wsum[2] + wsum[3];
  unsigned long long both = 0;
  for (int q = 0; q < kHiCopies; ++q) both += bnd[j].hi[q];
  const uint32_t c_hi = (uint32_t)both, low_set = (uint32_t)(both >> 32);
  const uint32_t k = s.k_rem;
  if (c_hi < k && (uint64_t)k <= (uint64_t)c_hi + c_mid) {
    SegState t = s;
    t.prefix = 0;
    t.k_rem = k - c_hi;
    t = find_bucket<3>(bins, t, fl);  // t.prefix: the bin, i.e. the key's top 21 bits less b_lo << 10
    SegState o = s;
    o.prefix = (bnd[j].b_lo << kBits1) + t.prefix;
    o.k_rem = t.k_rem;
    o.done = t.done;
    o.T = t.done ? (o.prefix << kBits2) : 0u;  // the whole bucket is taken
    o.r = t.done ? 0xFFFFFFFFu : 0u;
    if (!o.done && low_set == 0u) {
      // no parked key has any of its low bits set: the bucket holds one key value, which is the
      // threshold, and the last digit level has nothing left to find
      o.T = o.prefix << kBits2;
      o.r = o.k_rem;
      o.done = 1;
    }
    if (threadIdx.x == 0) {
      st[(size_t)m + j] = o;
      st[(size_t)2 * m + j] = o;
      atomicAdd(&stats[DEFT_STAT_BOUNDED], 1u);
      if (!o.done) atomicOr(flags, kFlagLevel2);
    }
  } else if (threadIdx.x == 0) {
    bnd[j].mode = kModeFailed;
    atomicOr(flags, kFlagPass2);
    atomicAdd(&stats[DEFT_STAT_REDONE], 1u);
  }
}

// Per count/emit chunk: how many keys exceed T and how many equal it -- from the slots of
// pass 2, or from the segment itself for a chunk that overflowed its slots.
template <int ITERS, bool FUSED>
__global__ __launch_bounds__(kThreads) void slot_count_kernel(
    const float* __restrict__ g, const SegDesc* __restrict__ seg, SegState* __restrict__ st, int m,
    const uint32_t* __restrict__ hist, const uint32_t* __restrict__ live_cnt,
    const uint2* __restrict__ slots, uint32_t cap, uint32_t* __restrict__ chunk_gt,
    uint32_t* __restrict__ chunk_eq, uint32_t* __restrict__ flags) {
  __shared__ uint32_t red[2 * kWaves];
  __shared__ uint32_t fl[kWaves + 8];
  const int j = seg_of_chunk(seg, m, blockIdx.x);
  const SegDesc d = seg[j];
  const uint32_t local = blockIdx.x - d.chunk_base;
  const uint32_t n = live_cnt[blockIdx.x];
  if (n == 0 && (!FUSED || local != 0)) {
    // nothing parked here: the counts are zero whatever the threshold is
    if (threadIdx.x == 0) { chunk_gt[blockIdx.x] = 0; chunk_eq[blockIdx.x] = 0; }
    return;
  }
  const uint32_t T = state_after<3, FUSED>(st, m, j, hist, local == 0, fl).T;
  uint32_t gt = 0, eq = 0;
  if (n <= cap) {
    for (uint32_t r = threadIdx.x; r < n; r += kThreads) {
      const uint32_t key = slots[(size_t)blockIdx.x * cap + r].x & 0x7FFFFFFFu;
      gt += key > T ? 1u : 0u;
      eq += key == T ? 1u : 0u;
    }
  } else {
    if (threadIdx.x == 0) raise_flag(flags, kFlagOverflow);  // the ordered write needs its second launch
    Chunk<ITERS> ch;
    ch.load(g, d.start, (int64_t)d.start + d.size, local);
#pragma unroll
    for (int i = 0; i < ITERS; ++i) {
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        const bool on = (ch.vmask(i) >> c) & 1u;
        gt += (on && ch.key[i][c] > T) ? 1u : 0u;
        eq += (on && ch.key[i][c] == T) ? 1u : 0u;
      }
    }
  }
  gt = wave_sum_u32(gt);
  eq = wave_sum_u32(eq);
  if ((threadIdx.x & 63) == 0) {
    red[threadIdx.x >> 6] = gt;
    red[kWaves + (threadIdx.x >> 6)] = eq;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    chunk_gt[blockIdx.x] = red[0] + red[1] + red[2] + red[3];
    chunk_eq[blockIdx.x] = red[kWaves] + red[kWaves + 1] + red[kWaves + 2] + red[kWaves + 3];
  }
}

// Wave-per-chunk forms of the two slot kernels for long vectors (states precomputed by the find
// kernels, so the four wavefronts of a workgroup may serve chunks of different segments): a
// quarter of the workgroups, and the trivial chunks cost a wavefront instead of a workgroup.
// Chunks that overflowed their slots are then handled by the whole workgroup, one at a time.
template <int ITERS>
__global__ __launch_bounds__(kThreads) void slot_hist2_wave_kernel(
    const float* __restrict__ g, const SegDesc* __restrict__ seg, const SegState* __restrict__ st,
    int m, uint32_t chunks, uint32_t* __restrict__ hist, const uint32_t* __restrict__ live_cnt,
    const uint2* __restrict__ slots, uint32_t cap, const uint32_t* __restrict__ flags) {
  // (a launch that sampled: nothing to do if every threshold is already resolved)
  if (flags && !(*flags & kFlagLevel2)) return;
  // The workgroups stride over groups of kWaves consecutive chunks and collect the digits in an
  // LDS histogram that is merged into the segment's when the segment changes and at the end:
  // rounded gradients put every candidate into the same few bins, and one device-scope atomic
  // per wavefront and chunk on those few addresses took 42 us on a 1.4 GB vector.  A group that
  // straddles two segments (rare) adds to the segments' histograms directly.
  constexpr int kBins = 1 << kBits2;
  __shared__ uint32_t acc[kBins];  // digits of segment `cur`, not yet merged
  __shared__ uint32_t lh[kBins];   // scratch of the overflow path
  __shared__ uint32_t ovf[kWaves];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  for (int b = threadIdx.x; b < kBins; b += kThreads) acc[b] = 0;
  __syncthreads();
  int cur = -1;
  const uint32_t groups = (chunks + kWaves - 1) / kWaves;
  for (uint32_t grp = blockIdx.x; grp < groups; grp += gridDim.x) {
    const uint32_t c0 = grp * kWaves;
    const int j0 = seg_of_chunk(seg, m, c0);
    const bool one_seg = seg_of_chunk(seg, m, min(c0 + kWaves - 1, chunks - 1)) == j0;
    if (one_seg && j0 != cur) {
      if (cur >= 0) {
        __syncthreads();
        uint32_t* gh = hist + (size_t)cur * kHistStride + hist_offset(2) + (blockIdx.x % kRep12) * kBins;
        for (int b = threadIdx.x; b < kBins; b += kThreads) {
          const uint32_t v = acc[b];
          if (v) { atomicAdd(&gh[b], v); acc[b] = 0; }
        }
        __syncthreads();
      }
      cur = j0;
    }
    const uint32_t c = c0 + wave;
    bool over = false;
    if (c < chunks) {
      const int j = one_seg ? j0 : seg_of_chunk(seg, m, c);
      const SegState s = st[(size_t)2 * m + j];
      const uint32_t n = live_cnt[c];
      if (!s.done && n > 0) {
        if (n > cap) {
          over = true;
        } else {
          uint32_t* dst = one_seg ? acc : hist + (size_t)j * kHistStride + hist_offset(2) + (blockIdx.x % kRep12) * kBins;
          for (uint32_t r0 = 0; r0 < n; r0 += 64) {
            const bool on = r0 + lane < n;
            const uint32_t e = on ? (slots[(size_t)c * cap + r0 + lane].x & 0x7FFFFFFFu) : 0u;
            bool live = on && (e >> kBits2) == s.prefix;
            const uint32_t digit = e & (kBins - 1);
            // equal digits are common: one atomic per distinct digit and wavefront
            unsigned long long act = __ballot(live);
            while (act) {
              const int leader = __ffsll((long long)act) - 1;
              const uint32_t dl = (uint32_t)__builtin_amdgcn_readlane((int)digit, leader);
              const unsigned long long same = __ballot(live && digit == dl);
              if (lane == leader) atomicAdd(&dst[dl], (uint32_t)__popcll(same));
              if (live && digit == dl) live = false;
              act &= ~same;
            }
          }
        }
      }
    }
    if (lane == 0) ovf[wave] = over ? 1u : 0u;
    __syncthreads();
    // chunks that overflowed their slots: the whole workgroup reads them from the segment
    for (int q = 0; q < kWaves; ++q) {
      if (!ovf[q]) continue;
      const uint32_t cq = c0 + q;
      const int j = seg_of_chunk(seg, m, cq);
      const SegDesc d = seg[j];
      const uint32_t prefix = st[(size_t)2 * m + j].prefix;
      __syncthreads();
      for (int b = threadIdx.x; b < kBins; b += kThreads) lh[b] = 0;
      __syncthreads();
      Chunk<ITERS> ch;
      ch.load(g, d.start, (int64_t)d.start + d.size, cq - d.chunk_base);
#pragma unroll
      for (int i = 0; i < ITERS; ++i) {
#pragma unroll
        for (int cc = 0; cc < 4; ++cc) {
          const uint32_t key = ch.key[i][cc];
          if (((ch.vmask(i) >> cc) & 1u) && (key >> kBits2) == prefix) atomicAdd(&lh[key & (kBins - 1)], 1u);
        }
      }
      __syncthreads();
      uint32_t* gh = hist + (size_t)j * kHistStride + hist_offset(2) + (blockIdx.x % kRep12) * kBins;
      for (int b = threadIdx.x; b < kBins; b += kThreads) {
        const uint32_t v = lh[b];
        if (v) atomicAdd(&gh[b], v);
      }
    }
    __syncthreads();  // ovf[] may be rewritten
  }
  if (cur < 0) return;
  __syncthreads();
  uint32_t* gh = hist + (size_t)cur * kHistStride + hist_offset(2) + (blockIdx.x % kRep12) * kBins;
  for (int b = threadIdx.x; b < kBins; b += kThreads) {
    const uint32_t v = acc[b];
    if (v) atomicAdd(&gh[b], v);
  }
}

template <int ITERS>
__global__ __launch_bounds__(kThreads) void slot_count_wave_kernel(
    const float* __restrict__ g, const SegDesc* __restrict__ seg, const SegState* __restrict__ st,
    int m, uint32_t chunks, const uint32_t* __restrict__ live_cnt,
    const uint2* __restrict__ slots, uint32_t cap, uint32_t* __restrict__ chunk_gt,
    uint32_t* __restrict__ chunk_eq, uint32_t* __restrict__ flags) {
  __shared__ uint32_t red[2 * kWaves];
  __shared__ uint32_t ovf[kWaves];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const uint32_t c = blockIdx.x * kWaves + wave;
  bool over = false;
  if (c < chunks) {
    const int j = seg_of_chunk(seg, m, c);
    const uint32_t T = st[(size_t)3 * m + j].T;
    const uint32_t n = live_cnt[c];
    if (n > cap) {
      over = true;
    } else {
      uint32_t gt = 0, eq = 0;
      for (uint32_t r0 = 0; r0 < n; r0 += 64) {
        if (r0 + lane < n) {
          const uint32_t key = slots[(size_t)c * cap + r0 + lane].x & 0x7FFFFFFFu;
          gt += key > T ? 1u : 0u;
          eq += key == T ? 1u : 0u;
        }
      }
      gt = wave_sum_u32(gt);
      eq = wave_sum_u32(eq);
      if (lane == 0) {
        chunk_gt[c] = gt;
        chunk_eq[c] = eq;
      }
    }
  }
  if (lane == 0) ovf[wave] = over ? 1u : 0u;
  __syncthreads();
  for (int q = 0; q < kWaves; ++q) {
    if (!ovf[q]) continue;
    const uint32_t cq = blockIdx.x * kWaves + q;
    const int j = seg_of_chunk(seg, m, cq);
    const SegDesc d = seg[j];
    const uint32_t T = st[(size_t)3 * m + j].T;
    if (threadIdx.x == 0) raise_flag(flags, kFlagOverflow);
    Chunk<ITERS> ch;
    ch.load(g, d.start, (int64_t)d.start + d.size, cq - d.chunk_base);
    uint32_t gt = 0, eq = 0;
#pragma unroll
    for (int i = 0; i < ITERS; ++i) {
#pragma unroll
      for (int cc = 0; cc < 4; ++cc) {
        const bool on = (ch.vmask(i) >> cc) & 1u;
        gt += (on && ch.key[i][cc] > T) ? 1u : 0u;
        eq += (on && ch.key[i][cc] == T) ? 1u : 0u;
      }
    }
    gt = wave_sum_u32(gt);
    eq = wave_sum_u32(eq);
    __syncthreads();
    if (lane == 0) { red[wave] = gt; red[kWaves + wave] = eq; }
    __syncthreads();
    if (threadIdx.x == 0) {
      chunk_gt[cq] = red[0] + red[1] + red[2] + red[3];
      chunk_eq[cq] = red[kWaves] + red[kWaves + 1] + red[kWaves + 2] + red[kWaves + 3];
    }
  }
}

// Exclusive prefix sums of the two per-chunk count arrays over ALL chunks of the launch
// (segment boundaries are ignored: a segment's own prefix is a difference of two entries).
// One workgroup per tile of kScanTile chunks writes tile-local prefixes and the tile totals; the
// wavefronts of emit_wave_kernel add up the totals of the tiles in front of their chunk.
constexpr int kScanPer = 8;
constexpr int kScanTile = kThreads * kScanPer;

__device__ __forceinline__ uint32_t block_excl_scan(uint32_t v, uint32_t* wsum, uint32_t& total) {
  uint32_t inc = v;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const uint32_t n = __shfl_up(inc, o, 64);
    if (lane >= o) inc += n;
  }
  __syncthreads();
  if (lane == 63) wsum[wave] = inc;
  __syncthreads();
  uint32_t before = inc - v;
  for (int w = 0; w < wave; ++w) before += wsum[w];
  total = wsum[0] + wsum[1] + wsum[2] + wsum[3];
  return before;
}

__global__ __launch_bounds__(kThreads) void scan_tiles_kernel(
    const uint32_t* __restrict__ chunk_gt, const uint32_t* __restrict__ chunk_eq, uint32_t chunks,
    uint32_t* __restrict__ pre_gt, uint32_t* __restrict__ pre_eq, uint32_t* __restrict__ tile_gt,
    uint32_t* __restrict__ tile_eq) {
  __shared__ uint32_t wsum[kWaves];
  const uint32_t base = blockIdx.x * kScanTile + threadIdx.x * kScanPer;
  uint32_t g[kScanPer], e[kScanPer], sg = 0, se = 0;
#pragma unroll
  for (int q = 0; q < kScanPer; ++q) {
    const bool on = base + q < chunks;
    g[q] = on ? chunk_gt[base + q] : 0u;
    e[q] = on ? chunk_eq[base + q] : 0u;
    sg += g[q];
    se += e[q];
  }
  uint32_t tg, te;
  uint32_t bg = block_excl_scan(sg, wsum, tg);
  uint32_t be = block_excl_scan(se, wsum, te);
#pragma unroll
  for (int q = 0; q < kScanPer; ++q) {
    if (base + q < chunks) { pre_gt[base + q] = bg; pre_eq[base + q] = be; }
    bg += g[q];
    be += e[q];
  }
  if (threadIdx.x == 0) { tile_gt[blockIdx.x] = tg; tile_eq[blockIdx.x] = te; }
}

// Ordered compaction of one chunk read from the segment itself (a chunk whose slots overflowed),
// by the whole workgroup.  ob: the chunk's first output position; eb: ties in the segment's
// earlier chunks; mode 0: none of the chunk's ties is taken, 1: all are, 2: the quota r ends
// inside this chunk and its ties are ranked in index order.
template <int ITERS>
__device__ __forceinline__ void emit_from_segment(
    const float* __restrict__ g, const SegDesc& d, uint32_t local_chunk, uint32_t T, uint32_t r,
    uint32_t eb, uint32_t ob, int mode, uint32_t lim, int32_t* __restrict__ idx_out,
    float* __restrict__ val_out, uint32_t (*wtot)[kWaves]) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  Chunk<ITERS> ch;
  ch.load(g, d.start, (int64_t)d.start + d.size, local_chunk);

  uint32_t sel[ITERS];  // 4-bit masks of selected components
  if (mode != 2) {
#pragma unroll
    for (int i = 0; i < ITERS; ++i) {
      sel[i] = 0;
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        const bool on = (ch.vmask(i) >> c) & 1u;
        const bool s = mode == 1 ? ch.key[i][c] >= T : ch.key[i][c] > T;
        sel[i] |= (on && s) ? (1u << c) : 0u;
      }
    }
  } else {
    // rank the ties of the chunk in index order: wave totals first, then in-wave prefixes
    uint32_t eqm[ITERS];
    uint32_t wave_eq = 0;
#pragma unroll
    for (int i = 0; i < ITERS; ++i) {
      eqm[i] = 0;
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        const bool on = (ch.vmask(i) >> c) & 1u;
        eqm[i] |= (on && ch.key[i][c] == T) ? (1u << c) : 0u;
      }
      wave_eq += (uint32_t)__popc(eqm[i]);
    }
    wave_eq = wave_sum_u32(wave_eq);
    if (lane == 0) wtot[1][wave] = wave_eq;
    __syncthreads();
    uint32_t rank = eb;
    for (int w = 0; w < wave; ++w) rank += wtot[1][w];
#pragma unroll
    for (int i = 0; i < ITERS; ++i) {
      uint32_t tot;
      uint32_t mine = rank + wave_excl_small((uint32_t)__popc(eqm[i]), tot);
      sel[i] = 0;
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        const bool on = (ch.vmask(i) >> c) & 1u;
        const bool is_eq = (eqm[i] >> c) & 1u;
        bool s = on && ch.key[i][c] > T;
        if (is_eq) { s = mine < r; ++mine; }
        sel[i] |= s ? (1u << c) : 0u;
      }
      rank += tot;
    }
  }

  uint32_t wave_sel = 0;
#pragma unroll
  for (int i = 0; i < ITERS; ++i) wave_sel += (uint32_t)__popc(sel[i]);
  wave_sel = wave_sum_u32(wave_sel);
  if (lane == 0) wtot[0][wave] = wave_sel;
  __syncthreads();
  uint32_t pos = ob;
  for (int w = 0; w < wave; ++w) pos += wtot[0][w];
  if (wtot[0][wave] == 0) return;
#pragma unroll
  for (int i = 0; i < ITERS; ++i) {
    if (__ballot(sel[i] != 0) == 0ull) continue;
    uint32_t tot;
    uint32_t mine = pos + wave_excl_small((uint32_t)__popc(sel[i]), tot);
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      if (((sel[i] >> c) & 1u) && mine < lim) {
        idx_out[mine] = (int32_t)(ch.base + (int64_t)i * 256 + c);
        val_out[mine] = __uint_as_float(ch.raw[i][c]);
        ++mine;
      }
    }
    pos += tot;
  }
}

// Ordered compaction of one chunk per workgroup (segments of at most 2048 chunks).  Ties
// are granted in index order until the quota r is used up, so a chunk's first output slot is
// out_off + (keys > T before it) + min(r, keys == T before it)  within its segment.  SCAN_HERE:
// the workgroup sums the counts of the preceding chunks of its segment itself -- cheaper than a
// scan launch when every segment is short; otherwise tile-local prefixes from scan_tiles_kernel
// plus the totals of the tiles in between.
struct WriteBase {
  SegDesc d;
  uint32_t T, r;      // threshold key, ties to take
  uint32_t cgt, ceq;  // the chunk's keys above / at the threshold
  uint32_t eb, ob;    // ties in the segment's earlier chunks; the chunk's first output position
  bool any;           // the chunk writes something
};

template <bool SCAN_HERE>
__device__ __forceinline__ WriteBase write_base(
    uint32_t c, const SegDesc* __restrict__ seg, const SegState* __restrict__ st, int m,
    const uint32_t* __restrict__ chunk_gt, const uint32_t* __restrict__ chunk_eq,
    const uint32_t* __restrict__ pre_gt, const uint32_t* __restrict__ pre_eq,
    const uint32_t* __restrict__ tile_gt, const uint32_t* __restrict__ tile_eq,
    uint32_t (*wtot)[kWaves]) {
  WriteBase w;
  const int j = seg_of_chunk(seg, m, c);
  w.d = seg[j];
  w.T = st[(size_t)3 * m + j].T;
  w.r = st[(size_t)3 * m + j].r;
  w.cgt = chunk_gt[c];
  w.ceq = chunk_eq[c];
  w.eb = 0;
  w.ob = 0;
  w.any = false;
  // a chunk that holds nothing to select is not read at all
  if (w.cgt == 0 && w.ceq == 0) return w;
  uint32_t sg = 0, se = 0;
  if (SCAN_HERE) {
    for (uint32_t i = w.d.chunk_base + threadIdx.x; i < c; i += kThreads) {
      sg += chunk_gt[i];
      se += chunk_eq[i];
    }
  } else {
    for (uint32_t t = w.d.chunk_base / kScanTile + threadIdx.x; t < c / kScanTile; t += kThreads) {
      sg += tile_gt[t];
      se += tile_eq[t];
    }
    if (threadIdx.x == 0) {
      sg += pre_gt[c] - pre_gt[w.d.chunk_base];
      se += pre_eq[c] - pre_eq[w.d.chunk_base];
    }
  }
  sg = wave_sum_u32(sg);
  se = wave_sum_u32(se);
  if ((threadIdx.x & 63) == 0) { wtot[0][threadIdx.x >> 6] = sg; wtot[1][threadIdx.x >> 6] = se; }
  __syncthreads();
  const uint32_t gt_before = wtot[0][0] + wtot[0][1] + wtot[0][2] + wtot[0][3];
  w.eb = wtot[1][0] + wtot[1][1] + wtot[1][2] + wtot[1][3];
  w.ob = w.d.out_off + gt_before + min(w.r, w.eb);
  __syncthreads();
  // (only ties here, and the quota used up before them: nothing to write)
  w.any = !(w.cgt == 0 && w.eb >= w.r);
  return w;
}

// The chunk's selectable keys come from its slots (parked in index order, one thread per
// entry).  A chunk that overflowed its slots is read from the segment again: here (OVERFLOW_HERE:
// short selections, where one more launch would cost more than the registers of that rare path),
// or by emit_overflow_kernel (long vectors: the path costs every workgroup of the kernel its
// registers and with them half the wavefronts a SIMD can hold).
template <int ITERS, bool SCAN_HERE, bool OVERFLOW_HERE>
__global__ __launch_bounds__(kThreads) void emit_kernel(
    const float* __restrict__ g, const SegDesc* __restrict__ seg, const SegState* __restrict__ st,
    int m, const uint32_t* __restrict__ chunk_gt, const uint32_t* __restrict__ chunk_eq,
    const uint32_t* __restrict__ pre_gt, const uint32_t* __restrict__ pre_eq,
    const uint32_t* __restrict__ tile_gt, const uint32_t* __restrict__ tile_eq,
    const uint32_t* __restrict__ live_cnt, const uint2* __restrict__ slots, uint32_t cap,
    int32_t* __restrict__ idx_out, float* __restrict__ val_out) {
  __shared__ uint32_t wtot[2][kWaves];
  const WriteBase w = write_base<SCAN_HERE>(blockIdx.x, seg, st, m, chunk_gt, chunk_eq, pre_gt, pre_eq,
                                            tile_gt, tile_eq, wtot);
  if (!w.any) return;
  const uint32_t T = w.T, r = w.r;
  const int mode = (w.eb >= r) ? 0 : ((r - w.eb >= w.ceq) ? 1 : 2);
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const uint32_t lim = w.d.out_off + w.d.k;  // a segment never writes past its own k slots
  const uint32_t n_live = live_cnt[blockIdx.x];
  if (n_live > cap) {
    if (OVERFLOW_HERE)
      emit_from_segment<ITERS>(g, w.d, blockIdx.x - w.d.chunk_base, T, r, w.eb, w.ob, mode, lim, idx_out,
                               val_out, wtot);
    return;
  }
  // entries in index order, kThreads at a time (one round unless the cap exceeds the workgroup)
  const unsigned long long below = (1ull << lane) - 1ull;
  uint32_t pos_base = w.ob, rank_base = w.eb;
  for (uint32_t r0 = 0; r0 < n_live; r0 += kThreads) {
    const bool on = r0 + threadIdx.x < n_live;
    const uint2 e = on ? slots[(size_t)blockIdx.x * cap + r0 + threadIdx.x] : make_uint2(0u, 0u);
    const uint32_t key = e.x & 0x7FFFFFFFu;
    const bool is_eq = on && key == T;
    bool take = on && key > T;
    if (mode == 1) {
      take = take || is_eq;
    } else if (mode == 2) {
      const unsigned long long eqb = __ballot(is_eq);
      if (lane == 0) wtot[1][wave] = (uint32_t)__popcll(eqb);
      __syncthreads();
      uint32_t rank = rank_base + (uint32_t)__popcll(eqb & below);
      for (int w2 = 0; w2 < wave; ++w2) rank += wtot[1][w2];
      take = take || (is_eq && rank < r);
      rank_base += wtot[1][0] + wtot[1][1] + wtot[1][2] + wtot[1][3];
    }
    const unsigned long long tb = __ballot(take);
    if (lane == 0) wtot[0][wave] = (uint32_t)__popcll(tb);
    __syncthreads();
    uint32_t pos = pos_base + (uint32_t)__popcll(tb & below);
    for (int w2 = 0; w2 < wave; ++w2) pos += wtot[0][w2];
    if (take && pos < lim) {
      idx_out[pos] = (int32_t)e.y;
      val_out[pos] = __uint_as_float(e.x);
    }
    pos_base += wtot[0][0] + wtot[0][1] + wtot[0][2] + wtot[0][3];
    __syncthreads();  // wtot is rewritten in the next round
  }
}

// The chunks that overflowed their slots (heavy ties, dense selections), written from the
// segment itself.  Launched behind every ordered write; a no-op unless the count kernel met such
// a chunk and raised kFlagOverflow.  A fixed set of workgroups strides over the chunks.
template <int ITERS, bool SCAN_HERE>
__global__ __launch_bounds__(kThreads) void emit_overflow_kernel(
    const float* __restrict__ g, const SegDesc* __restrict__ seg, const SegState* __restrict__ st,
    int m, uint32_t chunks, const uint32_t* __restrict__ chunk_gt,
    const uint32_t* __restrict__ chunk_eq, const uint32_t* __restrict__ pre_gt,
    const uint32_t* __restrict__ pre_eq, const uint32_t* __restrict__ tile_gt,
    const uint32_t* __restrict__ tile_eq, const uint32_t* __restrict__ live_cnt, uint32_t cap,
    const uint32_t* __restrict__ flags, int32_t* __restrict__ idx_out, float* __restrict__ val_out) {
  __shared__ uint32_t wtot[2][kWaves];
  if (!(*flags & kFlagOverflow)) return;
  for (uint32_t c = blockIdx.x; c < chunks; c += gridDim.x) {
    if (live_cnt[c] <= cap) continue;
    const WriteBase w = write_base<SCAN_HERE>(c, seg, st, m, chunk_gt, chunk_eq, pre_gt, pre_eq, tile_gt,
                                              tile_eq, wtot);
    if (w.any) {
      const int mode = (w.eb >= w.r) ? 0 : ((w.r - w.eb >= w.ceq) ? 1 : 2);
      emit_from_segment<ITERS>(g, w.d, c - w.d.chunk_base, w.T, w.r, w.eb, w.ob, mode,
                               w.d.out_off + w.d.k, idx_out, val_out, wtot);
    }
    __syncthreads();  // wtot is reused from one chunk to the next
  }
}

// The same for long vectors: one wavefront per chunk, so that the many chunks that hold nothing
// cost a wavefront's two loads instead of a workgroup (32 -> 17 us on a 1.4 GB vector, where
// three quarters of the chunks are empty); chunk prefixes come from scan_tiles_kernel
// (tile-local prefixes and tile totals; a segment's own prefix is a difference).  No barrier, no
// LDS: a wavefront leaves as soon as its chunk is done.  Chunks that overflowed their slots are
// left to emit_overflow_kernel.
__global__ __launch_bounds__(kThreads) void emit_wave_kernel(
    const SegDesc* __restrict__ seg, const SegState* __restrict__ st,
    int m, uint32_t chunks, const uint32_t* __restrict__ chunk_gt,
    const uint32_t* __restrict__ chunk_eq, const uint32_t* __restrict__ pre_gt,
    const uint32_t* __restrict__ pre_eq, const uint32_t* __restrict__ tile_gt,
    const uint32_t* __restrict__ tile_eq, const uint32_t* __restrict__ live_cnt,
    const uint2* __restrict__ slots, uint32_t cap, int32_t* __restrict__ idx_out,
    float* __restrict__ val_out) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const uint32_t c = blockIdx.x * kWaves + wave;
  if (c >= chunks) return;
  // everything that is indexed by the chunk alone is fetched at once, ahead of the chain
  // segment -> state -> prefixes -> slots (each link a round trip to memory)
  const uint32_t cgt = chunk_gt[c], ceq = chunk_eq[c];
  const uint32_t pg = pre_gt[c], pe = pre_eq[c], n = live_cnt[c];
  const uint2 first = (n != 0 && n <= cap && (uint32_t)lane < n) ? slots[(size_t)c * cap + lane]
                                                               : make_uint2(0u, 0u);
  if ((cgt == 0 && ceq == 0) || n > cap) return;
  const int j = seg_of_chunk(seg, m, c);
  const SegDesc d = seg[j];
  const uint32_t T = st[(size_t)3 * m + j].T, r = st[(size_t)3 * m + j].r;
  // prefix inside the segment: tile-local prefixes plus the totals of the tiles between the
  // segment's first chunk and this one (few: a tile spans 2048 chunks), summed by the lanes
  const uint32_t c0 = d.chunk_base;
  uint32_t sg = 0, se = 0;
  for (uint32_t t = c0 / kScanTile + lane; t < c / kScanTile; t += 64) {
    sg += tile_gt[t];
    se += tile_eq[t];
  }
  sg = (uint32_t)__builtin_amdgcn_readfirstlane((int)wave_sum_u32(sg));
  se = (uint32_t)__builtin_amdgcn_readfirstlane((int)wave_sum_u32(se));
  const uint32_t gt_before = sg + pg - pre_gt[c0];
  const uint32_t eb = se + pe - pre_eq[c0];
  const uint32_t ob = d.out_off + gt_before + min(r, eb);
  if (cgt == 0 && eb >= r) return;
  const int mode = (eb >= r) ? 0 : ((r - eb >= ceq) ? 1 : 2);
  const uint32_t lim = d.out_off + d.k;
  const unsigned long long below = (1ull << lane) - 1ull;
  uint32_t pos = ob, rank = eb;
  for (uint32_t r0 = 0; r0 < n; r0 += 64) {
    const bool on = r0 + lane < n;
    const uint2 e = r0 == 0 ? first : (on ? slots[(size_t)c * cap + r0 + lane] : make_uint2(0u, 0u));
    const uint32_t key = e.x & 0x7FFFFFFFu;
    const bool is_eq = on && key == T;
    bool take = on && key > T;
    if (mode == 1) {
      take = take || is_eq;
    } else if (mode == 2) {
      const unsigned long long eqb = __ballot(is_eq);
      take = take || (is_eq && rank + (uint32_t)__popcll(eqb & below) < r);
      rank += (uint32_t)__popcll(eqb);
    }
    const unsigned long long tb = __ballot(take);
    const uint32_t p = pos + (uint32_t)__popcll(tb & below);
    if (take && p < lim) {
      idx_out[p] = (int32_t)e.y;
      val_out[p] = __uint_as_float(e.x);
    }
    pos += (uint32_t)__popcll(tb);
  }
}

// ------------------------------------------------------------------------------------------
// host drivers
// ------------------------------------------------------------------------------------------
inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

#ifndef DEFT_SEL_ITERS_SMALL
#define DEFT_SEL_ITERS_SMALL 4
#endif
#ifndef DEFT_SEL_ITERS_LARGE
#define DEFT_SEL_ITERS_LARGE 8
#endif
// Unless the caller names a shape: selections from more than kLongVectorElems elements use the
// long-vector launch shape (larger chunks, separate bucket-search kernels, wave-per-chunk slot
// kernels); from kSampledVectorElems on they do if the one-read pass would cover at least half of
// them.  Measured: layer-wise shares of 44 M elements in 13 .. 144 segments, none sampled, 104 ..
// 128 us in the short shape against 116 .. 141 us in the long one (89 M: 199 .. 216 against
// 186 .. 208 us); one segment of 36 / 50 / 66 M elements, K = N/100, read once: 83 / 92 / 106 us
// against 108 / 134 / 168 us in the short shape.
constexpr int64_t kSampledVectorElems = int64_t(1) << 25;
constexpr int64_t kLongVectorElems = int64_t(1) << 26;
inline bool valid_shape(int32_t shape) {
  return shape >= DEFT_SHAPE_AUTO && shape <= DEFT_SHAPE_LONG_SAMPLED;
}
// Whether a segment of a long vector is sampled ahead of its first pass: it must be long enough
// for the sample (1/128 of it) to be cheap next to a second read, sparse enough for its
// candidates to fit the per-chunk slots on average, and k/128 large enough for the sample to
// place the threshold within four top digits.  DEFT_SHAPE_LONG_SAMPLED samples whatever can be sampled
// (the device side still turns down what its sample cannot place).
constexpr uint32_t kSampleMinElems = 1u << 22;
constexpr uint32_t kSampleMinK = 32768;  // 256 sampled keys at or above the threshold: fewer were turned down on every set tried
inline bool sample_segment(const SegDesc& d, int32_t shape) {
  if (shape == DEFT_SHAPE_LONG_PLAIN || sample_pieces(d.start, d.size) == 0) return false;
  if (shape == DEFT_SHAPE_LONG_SAMPLED) return true;
  return d.size >= kSampleMinElems && d.k >= kSampleMinK && (uint64_t)d.k * kParkDiv <= d.size;
}

struct SelectLayout {
  size_t stats, seg, st, bnd, hist, hmax, bhist, cgt, ceq, obase, ebase, tgt, teq, ccnt, slots, total;
};

// Slots per count/emit chunk.  Measured with caps sized to the average density (4x the
// expected picks, 32..256): the conventional Top-k then overflowed in most chunks that hold
// picks at all, because its picks sit in the few layers of large norm at many times the average
// density.  The slot arrays are written sparsely, so the largest cap costs address space only.
// Long vectors walk chunks twice as large with eight times the slots (a quarter of a chunk, 2 bytes
// of address space per element): at 512 slots the BERT-shaped conventional Top-k (K = N/100)
// overflowed in 840 .. 2000 of its 13365 chunks, each then read again from the segment by every
// kernel behind the first pass (178 us; 158 us with 1024 slots, 148 us with 2048).
inline uint32_t slot_cap_for(uint64_t /*total_k*/, uint64_t /*share*/, uint32_t chunk_elems) {
  return chunk_elems == kThreads * 4 * DEFT_SEL_ITERS_SMALL ? kShortSlotCap : kLongSlotCap;
}

SelectLayout select_layout(int64_t m, uint64_t chunks, uint32_t cap = std::max(kShortSlotCap, kLongSlotCap / 2)) {
  SelectLayout w;
  size_t o = 0;
  w.stats = o; o = 256;  // DEFT_STAT_ words, at the very start of the workspace
  w.seg = o;   o = align_up(o + sizeof(SegDesc) * (size_t)(m + 1), 256);
  w.st = o;    o = align_up(o + sizeof(SegState) * 4 * (size_t)m, 256);  // state after 0..3 levels
  w.bnd = o;   o = align_up(o + sizeof(SegBound) * (size_t)m, 256);
  w.hist = o;  o = o + sizeof(uint32_t) * kHistStride * (size_t)m;  // hmax follows: zeroed together
  // per-chunk maxima, then two chunk counters and the flag word of the long-vector first pass
  w.hmax = o;  o = o + sizeof(uint32_t) * (chunks / 4 + 2 * (size_t)m + 4);
  // the bounded histograms of the sampled segments follow directly: cleared in the same sweep
  w.bhist = o; o = align_up(o + sizeof(uint32_t) * kBoundedStride * (size_t)std::min<int64_t>(m, kMaxSampled), 256);
  w.cgt = o;   o = align_up(o + sizeof(uint32_t) * chunks, 256);
  w.ceq = o;   o = align_up(o + sizeof(uint32_t) * chunks, 256);
  w.obase = o; o = align_up(o + sizeof(uint32_t) * chunks, 256);
  w.ebase = o; o = align_up(o + sizeof(uint32_t) * chunks, 256);
  w.tgt = o;   o = align_up(o + sizeof(uint32_t) * (chunks / kScanTile + 1), 256);
  w.teq = o;   o = align_up(o + sizeof(uint32_t) * (chunks / kScanTile + 1), 256);
  w.ccnt = o;  o = align_up(o + sizeof(uint32_t) * chunks, 256);
  w.slots = o; o = align_up(o + sizeof(uint2) * chunks * cap, 256);
  w.total = o;
  return w;
}

// Upper bound on the chunk count of any set of m segments holding at most `elems` elements
// (the chunk size depends on the total, so the bound covers both regimes).
inline uint64_t max_chunks(int64_t elems, int64_t m) {
  // the smaller chunk size bounds both launch shapes
  return (uint64_t)(elems / (kThreads * 4 * DEFT_SEL_ITERS_SMALL) + 2 * m + 1);
}

#define HIP_TRY(x)                         \
  do {                                     \
    if ((x) != hipSuccess) return DEFT_EHIP; \
  } while (0)

// The two histogram passes walk chunks four times as large as the count/emit chunks: a
// histogram workgroup ends by merging up to 2048 bins into the segment's histogram with global
// atomics, a fixed cost that wants amortising; count/emit have no such tail and balance better
// with small chunks.  Each wavefront of a histogram workgroup covers one count/emit chunk.
template <int ITERS, bool FUSED>
int launch_select(const float* g, SegDesc* seg, SegState* st, int m, uint32_t chunks,
                  uint32_t hchunks, uint32_t* hist, uint32_t* cgt, uint32_t* ceq, uint32_t* obase,
                  uint32_t* ebase, uint32_t* tgt, uint32_t* teq, uint32_t* ccnt, uint32_t* hmax,
                  uint2* slots, SegBound* bnd, uint32_t* bhist, uint32_t sblocks, uint32_t* stats,
                  uint32_t cap, bool scan_in_emit, const SegBatch* inline_batch,
                  int32_t* idx_out, float* val_out, hipStream_t s) {
  if constexpr (FUSED) {
    if (inline_batch)
      hist0_inline_kernel<4 * ITERS><<<hchunks, kThreads, 0, s>>>(g, *inline_batch, seg, st, hist, hmax);
    else
      hist0_kernel<4 * ITERS><<<hchunks, kThreads, 0, s>>>(g, seg, m, hist, hmax);
  } else {
    // hmax[hchunks]: the chunk counter of the full first pass; hmax[hchunks + 2]: the flag word
    // (both zeroed with the histograms by seg_setup_kernel)
    uint32_t* flags = hmax + hchunks + 2;
    const unsigned grid1 = std::min<uint32_t>(hchunks, kStreamGrid);
    if (sblocks) {
      // sampled segments: placed by the sample, read once, checked; the four launches after
      // these are no-ops unless a segment was not sampled, turned down or refuted
      sample_hist_kernel<<<sblocks, kThreads, 0, s>>>(g, seg, m, hist);
      bounds_kernel<<<m, kThreads, 0, s>>>(seg, hist, bnd, flags);
      pass1_bounded_kernel<4 * ITERS><<<hchunks, kThreads, 0, s>>>(g, seg, m, bhist, bnd, ccnt, slots, cap);
      find_first_kernel<<<m, kThreads, 0, s>>>(st, m, seg, bhist, bnd, flags, stats);
    } else {
      bnd = nullptr;  // nothing sampled: every segment takes the full path, no checks needed
    }
    hist0_stream_kernel<4 * ITERS><<<grid1, kThreads, 0, s>>>(g, seg, m, hchunks, hist, hmax, hmax + hchunks,
                                                              bnd, flags);
    find_kernel<0><<<m, kThreads, 0, s>>>(st, m, hist, bnd, nullptr);
  }
  pass2_kernel<ITERS, FUSED><<<hchunks, kThreads, 0, s>>>(g, seg, st, m, hist, hmax, ccnt, slots, cap,
                                                         FUSED ? nullptr : bnd,
                                                         FUSED ? nullptr : hmax + hchunks + 2);
  if (!FUSED) find_kernel<1><<<m, kThreads, 0, s>>>(st, m, hist, bnd, bnd ? hmax + hchunks + 2 : nullptr);
  uint32_t* oflags = hmax + hchunks + 2;  // the flag word (cleared with the histograms)
  if (FUSED) {
    slot_hist2_kernel<ITERS, true><<<chunks, kThreads, 0, s>>>(g, seg, st, m, hist, ccnt, slots, cap);
    slot_count_kernel<ITERS, true><<<chunks, kThreads, 0, s>>>(g, seg, st, m, hist, ccnt, slots, cap,
                                                              cgt, ceq, oflags);
  } else {
    const uint32_t wblocks = (chunks + kWaves - 1) / kWaves;
    slot_hist2_wave_kernel<ITERS><<<std::min<uint32_t>(wblocks, kSlotWaveGrid), kThreads, 0, s>>>(
        g, seg, st, m, chunks, hist, ccnt, slots, cap, bnd ? hmax + hchunks + 2 : nullptr);
    find_kernel<2><<<m, kThreads, 0, s>>>(st, m, hist, bnd, nullptr);
    slot_count_wave_kernel<ITERS><<<wblocks, kThreads, 0, s>>>(g, seg, st, m, chunks, ccnt, slots,
                                                              cap, cgt, ceq, oflags);
  }
  // the ordered write from the slots, then (a no-op unless some chunk overflowed its slots) the
  // overflowed chunks from the segments
  const unsigned ogrid = std::min<uint32_t>(chunks, kOverflowGrid);
  if (scan_in_emit && FUSED) {
    emit_kernel<ITERS, true, true><<<chunks, kThreads, 0, s>>>(g, seg, st, m, cgt, ceq, obase, ebase, tgt,
                                                               teq, ccnt, slots, cap, idx_out, val_out);
  } else if (scan_in_emit) {
    emit_kernel<ITERS, true, false><<<chunks, kThreads, 0, s>>>(g, seg, st, m, cgt, ceq, obase, ebase, tgt,
                                                                teq, ccnt, slots, cap, idx_out, val_out);
    emit_overflow_kernel<ITERS, true><<<ogrid, kThreads, 0, s>>>(
        g, seg, st, m, chunks, cgt, ceq, obase, ebase, tgt, teq, ccnt, cap, oflags, idx_out, val_out);
  } else {
    const uint32_t tiles = (chunks + kScanTile - 1) / kScanTile;
    scan_tiles_kernel<<<tiles, kThreads, 0, s>>>(cgt, ceq, chunks, obase, ebase, tgt, teq);
    emit_wave_kernel<<<(chunks + kWaves - 1) / kWaves, kThreads, 0, s>>>(
        seg, st, m, chunks, cgt, ceq, obase, ebase, tgt, teq, ccnt, slots, cap, idx_out, val_out);
    emit_overflow_kernel<ITERS, false><<<ogrid, kThreads, 0, s>>>(
        g, seg, st, m, chunks, cgt, ceq, obase, ebase, tgt, teq, ccnt, cap, oflags, idx_out, val_out);
  }
  HIP_TRY(hipGetLastError());
  return DEFT_OK;
}

// A workspace layout fixed ahead of the plan (sized for m_cap segments and chunks_cap chunks)
// whose histogram area has already been cleared on the stream.
struct Precleared {
  int64_t m_cap;
  uint64_t chunks_cap;
};

// Words to clear for a layout: the histograms, the per-chunk maxima and the chunk counter.
// (The bounded histograms behind them belong to the long-vector shape, which clears its own.)
inline size_t clear_words(const SelectLayout& w) { return (w.bhist - w.hist) / sizeof(uint32_t); }

// Enqueue the selection of `m` validated, non-empty segments (k >= 1 each).  With `pre`, short
// selections of at most kSegBatch segments skip the set-up launch: the descriptors travel with
// the first pass.
int run_select(const float* g, const std::vector<SegDesc>& segs_in, int64_t share,
               int32_t* idx_out, float* val_out, void* ws, size_t ws_bytes, int32_t shape,
               hipStream_t s, const Precleared* pre = nullptr) {
  const int m = (int)segs_in.size();
  if (m == 0) return DEFT_OK;
  bool lng = shape >= DEFT_SHAPE_LONG;
  if (shape == DEFT_SHAPE_AUTO) {
    lng = share > kLongVectorElems;
    if (!lng && share > kSampledVectorElems) {
      uint64_t covered = 0;
      uint32_t n_cov = 0;
      for (const auto& d : segs_in)
        if (n_cov < kMaxSampled && sample_segment(d, shape)) { covered += d.size; ++n_cov; }
      lng = 2 * covered >= (uint64_t)share;
    }
  }
  const int iters = lng ? DEFT_SEL_ITERS_LARGE : DEFT_SEL_ITERS_SMALL;
  const bool small = !lng;
  const uint32_t ce = (uint32_t)kThreads * 4 * iters;
  const uint32_t hce = 4 * ce;
  std::vector<SegDesc> segs(segs_in);
  uint64_t chunks = 0, hchunks = 0, sblocks = 0, sampled_elems = 0;
  uint32_t n_sampled = 0;
  uint32_t longest = 0;  // chunks of the longest segment
  for (auto& d : segs) {
    d.chunk_base = (uint32_t)chunks;
    d.hchunk_base = (uint32_t)hchunks;
    d.sblock_base = (uint32_t)sblocks;
    d.sampled = 0;
    if (!small && n_sampled < kMaxSampled && sample_segment(d, shape)) {
      d.sampled = ++n_sampled;
      sblocks += (sample_pieces(d.start, d.size) + kSamplePiecesPerWg - 1) / kSamplePiecesPerWg;
      sampled_elems += d.size;
    }
    const uint32_t c = chunks_of(d.start, d.size, ce);
    longest = std::max(longest, c);
    chunks += c;
    hchunks += chunks_of(d.start, d.size, hce);
  }
  // Sampling adds four launches and a sweep of early-leaving workgroups over every chunk; it pays
  // when most of what is selected from is then read once.  (Layer-wise selection of one worker
  // of 4 on the GPT-2-medium-shaped set, where only a few of 80 segments qualify: 245 us without
  // any sampling, 270 us with.)
  if (shape != DEFT_SHAPE_LONG_SAMPLED && 2 * sampled_elems < (uint64_t)share) {
    for (auto& d : segs) d.sampled = 0;
    n_sampled = 0;
    sblocks = 0;
  }
  // every emit workgroup can afford to sum its segment's earlier chunk counts itself
  const bool scan_in_emit = longest <= 2048;
  if (chunks > max_chunks(share, m) || chunks >= (uint64_t(1) << 31)) return DEFT_EWS;
  uint64_t total_k = 0;
  for (const auto& d : segs) total_k += d.k;
  const uint32_t cap = slot_cap_for(total_k, (uint64_t)share, ce);
  const bool inline_segs = pre && small && m <= kSegBatch && m <= pre->m_cap && chunks <= pre->chunks_cap;
  const SelectLayout w = inline_segs ? select_layout(pre->m_cap, pre->chunks_cap, cap) : select_layout(m, chunks, cap);
  if (w.total > ws_bytes) return DEFT_EWS;
  char* base = static_cast<char*>(ws);
  SegDesc* seg = reinterpret_cast<SegDesc*>(base + w.seg);
  SegState* st = reinterpret_cast<SegState*>(base + w.st);
  SegBound* bnd = reinterpret_cast<SegBound*>(base + w.bnd);
  uint32_t* hist = reinterpret_cast<uint32_t*>(base + w.hist);
  SegBatch b;
  b.total_chunks = (uint32_t)chunks;
  b.total_hchunks = (uint32_t)hchunks;
  b.m = m;
  b.total_sblocks = (uint32_t)sblocks;
  if (inline_segs) {
    b.first = 0;
    b.count = m;
    std::memcpy(b.d, segs.data(), sizeof(SegDesc) * (size_t)m);
  } else {
    // histograms, the per-chunk maxima, and the two chunk counters and the flag word of the
    // long-vector first pass
    // (long vectors: also the bounded histograms of the sampled segments, which follow)
    const size_t nzero = small ? (size_t)kHistStride * m + hchunks + 3
                               : (w.bhist - w.hist) / sizeof(uint32_t) + (size_t)kBoundedStride * n_sampled;
    const unsigned setup_blocks = (unsigned)std::min<size_t>((nzero + 4 * kThreads - 1) / (4 * kThreads), 256);
    for (int first = 0; first < m; first += kSegBatch) {
      b.first = first;
      b.count = std::min(kSegBatch, m - first);
      std::memcpy(b.d, segs.data() + first, sizeof(SegDesc) * (size_t)b.count);
      seg_setup_kernel<<<first == 0 ? setup_blocks : 1, kThreads, 0, s>>>(
          b, seg, st, small ? nullptr : bnd, reinterpret_cast<uint32_t*>(base + w.stats), hist, nzero);
    }
  }
  uint32_t* cgt = reinterpret_cast<uint32_t*>(base + w.cgt);
  uint32_t* ceq = reinterpret_cast<uint32_t*>(base + w.ceq);
  uint32_t* ob = reinterpret_cast<uint32_t*>(base + w.obase);
  uint32_t* eb = reinterpret_cast<uint32_t*>(base + w.ebase);
  uint32_t* tg = reinterpret_cast<uint32_t*>(base + w.tgt);
  uint32_t* te = reinterpret_cast<uint32_t*>(base + w.teq);
  uint32_t* cc = reinterpret_cast<uint32_t*>(base + w.ccnt);
  uint32_t* hm = reinterpret_cast<uint32_t*>(base + w.hmax);
  uint2* sl = reinterpret_cast<uint2*>(base + w.slots);
  if (small)
    return launch_select<DEFT_SEL_ITERS_SMALL, true>(
        g, seg, st, m, (uint32_t)chunks, (uint32_t)hchunks, hist, cgt, ceq, ob, eb, tg, te, cc, hm, sl, nullptr,
        nullptr, 0, nullptr, cap, scan_in_emit, inline_segs ? &b : nullptr, idx_out, val_out, s);
  return launch_select<DEFT_SEL_ITERS_LARGE, false>(
      g, seg, st, m, (uint32_t)chunks, (uint32_t)hchunks, hist, cgt, ceq, ob, eb, tg, te, cc, hm, sl, bnd,
      reinterpret_cast<uint32_t*>(base + w.bhist), (uint32_t)sblocks,
      reinterpret_cast<uint32_t*>(base + w.stats), cap, scan_in_emit, nullptr, idx_out, val_out, s);
}

}  // namespace

// ------------------------------------------------------------------------------------------
// C ABI
// ------------------------------------------------------------------------------------------
extern "C" size_t deft_workspace_bytes(int op, int64_t elems, int32_t count) {
  if (elems < 0 || count < 0) return 0;
  switch (op) {
    case DEFT_OP_NORMS: {
      const size_t chunks = (size_t)((elems + kNormChunk - 1) / kNormChunk);
      return align_up(2 * sizeof(double) * std::max<size_t>(chunks, 1), 256);
    }
    case DEFT_OP_SELECT:
      return select_layout(std::max<int64_t>(count, 1), max_chunks(elems, count)).total;
    case DEFT_OP_TOPK_GLOBAL:
      return select_layout(1, max_chunks(elems, 1)).total;
    default:
      return 0;
  }
}

namespace {
// Enqueues the norm pass with its per-chunk partial sums in head[chunks], tail[chunks].
int launch_norms(const float* g, const float* grad, float eta, float* acc, int64_t N,
                 const int64_t* offsets_dev, int32_t L, double* sumsq_dev, double* head,
                 double* tail, hipStream_t s) {
  const unsigned chunks = (unsigned)((N + kNormChunk - 1) / kNormChunk);
  NormSrc src;
  src.g = g; src.gr = grad; src.acc = acc; src.eta = eta;
  if (acc)
    norm_chunks_kernel<true><<<chunks, kThreads, 0, s>>>(src, N, offsets_dev, L, head, tail, sumsq_dev);
  else
    norm_chunks_kernel<false><<<chunks, kThreads, 0, s>>>(src, N, offsets_dev, L, head, tail, sumsq_dev);
  norm_finish_kernel<<<L, kFinishThreads, 0, s>>>(offsets_dev, N, head, tail, sumsq_dev);
  HIP_TRY(hipGetLastError());
  return DEFT_OK;
}

int run_norms(const float* g, const float* grad, float eta, float* acc, int64_t N,
              const int64_t* offsets_dev, int32_t L, double* sumsq_dev, void* ws_dev,
              size_t ws_bytes, void* stream) {
  if (!g || !offsets_dev || !sumsq_dev || !ws_dev || L < 1 || N < 1) return DEFT_EINVAL;
  if (N > kMaxN) return DEFT_ERANGE;
  if ((reinterpret_cast<uintptr_t>(g) & 15u) || (reinterpret_cast<uintptr_t>(ws_dev) & 15u))
    return DEFT_EINVAL;
  if (ws_bytes < deft_workspace_bytes(DEFT_OP_NORMS, N, L)) return DEFT_EWS;
  const size_t chunks = (size_t)((N + kNormChunk - 1) / kNormChunk);
  double* head = static_cast<double*>(ws_dev);
  return launch_norms(g, grad, eta, acc, N, offsets_dev, L, sumsq_dev, head, head + chunks,
                      static_cast<hipStream_t>(stream));
}
}  // namespace

extern "C" int deft_layer_norms(const float* g_dev, int64_t N, const int64_t* offsets_dev,
                                int32_t L, double* sumsq_dev, void* ws_dev, size_t ws_bytes,
                                void* stream) {
  return run_norms(g_dev, nullptr, 0.0f, nullptr, N, offsets_dev, L, sumsq_dev, ws_dev, ws_bytes,
                   stream);
}

extern "C" int deft_accumulate_norms(const float* e_dev, const float* grad_dev, float eta,
                                     float* acc_dev, int64_t N, const int64_t* offsets_dev,
                                     int32_t L, double* sumsq_dev, void* ws_dev, size_t ws_bytes,
                                     void* stream) {
  if (!grad_dev || !acc_dev) return DEFT_EINVAL;
  if ((reinterpret_cast<uintptr_t>(grad_dev) & 15u) || (reinterpret_cast<uintptr_t>(acc_dev) & 15u))
    return DEFT_EINVAL;
  return run_norms(e_dev, grad_dev, eta, acc_dev, N, offsets_dev, L, sumsq_dev, ws_dev, ws_bytes,
                   stream);
}

extern "C" int deft_stream_read_probe(const float* g_dev, int64_t N, void* out_dev, void* stream) {
  if (!g_dev || !out_dev || N < kNormChunk) return DEFT_EINVAL;
  if (N > kMaxN) return DEFT_ERANGE;
  if (reinterpret_cast<uintptr_t>(g_dev) & 15u) return DEFT_EINVAL;
  stream_probe_kernel<<<(unsigned)(N / kNormChunk), kThreads, 0, static_cast<hipStream_t>(stream)>>>(
      g_dev, static_cast<uint32_t*>(out_dev));
  HIP_TRY(hipGetLastError());
  return DEFT_OK;
}

extern "C" int deft_gather_zero(float* acc_dev, int64_t N, const int32_t* idx_dev, int64_t count,
                                float* vals_out_dev, void* stream) {
  if (count < 0 || N < 1) return DEFT_EINVAL;
  if (N > kMaxN || count > kMaxN) return DEFT_ERANGE;
  if (count == 0) return DEFT_OK;
  if (!acc_dev || !idx_dev || !vals_out_dev) return DEFT_EINVAL;
  const unsigned blocks = (unsigned)((count + kThreads - 1) / kThreads);
  gather_zero_kernel<<<blocks, kThreads, 0, static_cast<hipStream_t>(stream)>>>(
      acc_dev, N, idx_dev, count, vals_out_dev);
  HIP_TRY(hipGetLastError());
  return DEFT_OK;
}

namespace {
int select_layers(const float* g_dev, int64_t N, const int64_t* offsets_host, const int64_t* k_host,
                  int32_t L, const int32_t* my_layers_host, int32_t my_count, int32_t* idx_out_dev,
                  float* val_out_dev, int64_t* seg_off_host, int64_t out_cap, void* ws_dev,
                  size_t ws_bytes, int32_t shape, void* stream, const Precleared* pre) {
  if (!g_dev || !offsets_host || !k_host || !seg_off_host || my_count < 0 || out_cap < 0 ||
      !valid_shape(shape))
    return DEFT_EINVAL;
  if (my_count > 0 && !my_layers_host) return DEFT_EINVAL;
  const int lay = deft_check_layout(offsets_host, L, N);
  if (lay != DEFT_OK) return lay;
  if (reinterpret_cast<uintptr_t>(g_dev) & 15u) return DEFT_EINVAL;
  std::vector<SegDesc> segs;
  segs.reserve(my_count);
  std::vector<int64_t> seg_off(my_count + 1, 0);
  int64_t share = 0, total_k = 0;
  for (int32_t j = 0; j < my_count; ++j) {
    const int32_t l = my_layers_host[j];
    if (l < 0 || l >= L) return DEFT_EINVAL;
    const int64_t size = offsets_host[l + 1] - offsets_host[l];
    const int64_t k = k_host[l];
    if (k < 0 || k > size) return DEFT_EINVAL;
    if (k > 0) {
      SegDesc d;
      d.start = (uint32_t)offsets_host[l];
      d.size = (uint32_t)size;
      d.k = (uint32_t)k;
      d.out_off = (uint32_t)total_k;
      d.chunk_base = 0;
      d.hchunk_base = 0;
      segs.push_back(d);
      share += size;
    }
    total_k += k;
    seg_off[j + 1] = total_k;
    if (total_k > kMaxN) return DEFT_ERANGE;
  }
  if (total_k > out_cap) return DEFT_ECAP;
  if (!segs.empty()) {
    if (!idx_out_dev || !val_out_dev || !ws_dev) return DEFT_EINVAL;
    if (reinterpret_cast<uintptr_t>(ws_dev) & 15u) return DEFT_EINVAL;
    if (share > kMaxN) return DEFT_ERANGE;  // a layer listed more than once
    if (ws_bytes < deft_workspace_bytes(DEFT_OP_SELECT, share, (int32_t)segs.size())) return DEFT_EWS;
  }
  const int rc = run_select(g_dev, segs, share, idx_out_dev, val_out_dev, ws_dev, ws_bytes, shape,
                            static_cast<hipStream_t>(stream), pre);
  if (rc != DEFT_OK) return rc;
  std::copy(seg_off.begin(), seg_off.end(), seg_off_host);
  return DEFT_OK;
}
}  // namespace

extern "C" int deft_select(const float* g_dev, int64_t N, const int64_t* offsets_host,
                           const int64_t* k_host, int32_t L, const int32_t* my_layers_host,
                           int32_t my_count, int32_t* idx_out_dev, float* val_out_dev,
                           int64_t* seg_off_host, int64_t out_cap, void* ws_dev, size_t ws_bytes,
                           int32_t launch_shape, void* stream) {
  return select_layers(g_dev, N, offsets_host, k_host, L, my_layers_host, my_count, idx_out_dev,
                       val_out_dev, seg_off_host, out_cap, ws_dev, ws_bytes, launch_shape, stream,
                       nullptr);
}

extern "C" int topk_global(const float* g_dev, int64_t N, int64_t K, int32_t* idx_out_dev,
                           float* val_out_dev, void* ws_dev, size_t ws_bytes, int32_t launch_shape,
                           void* stream) {
  if (!g_dev || N < 1 || K < 0 || K > N || !valid_shape(launch_shape)) return DEFT_EINVAL;
  if (N > kMaxN) return DEFT_ERANGE;
  if (reinterpret_cast<uintptr_t>(g_dev) & 15u) return DEFT_EINVAL;
  if (K == 0) return DEFT_OK;
  if (!idx_out_dev || !val_out_dev || !ws_dev) return DEFT_EINVAL;
  if (reinterpret_cast<uintptr_t>(ws_dev) & 15u) return DEFT_EINVAL;
  if (ws_bytes < deft_workspace_bytes(DEFT_OP_TOPK_GLOBAL, N, 1)) return DEFT_EWS;
  std::vector<SegDesc> segs(1);
  segs[0].start = 0;
  segs[0].size = (uint32_t)N;
  segs[0].k = (uint32_t)K;
  segs[0].out_off = 0;
  segs[0].chunk_base = 0;
  segs[0].hchunk_base = 0;
  return run_select(g_dev, segs, N, idx_out_dev, val_out_dev, ws_dev, ws_bytes, launch_shape,
                    static_cast<hipStream_t>(stream));
}

// Cyclic local Top-k (Sec. 1; Sec. 3.1): the worker whose turn it is selects the conventional
// Top-k of its own vector; the others select nothing.
extern "C" int deft_cltk_select(const float* g_dev, int64_t N, double d, int32_t n_workers,
                                int32_t rank, int64_t iteration, int32_t* idx_out_dev,
                                float* val_out_dev, int64_t out_cap, void* ws_dev, size_t ws_bytes,
                                int32_t launch_shape, void* stream, int64_t* count_out) {
  if (!count_out || rank < 0 || rank >= n_workers || out_cap < 0) return DEFT_EINVAL;
  int32_t leader = 0;
  int64_t K = 0;
  int rc = deft_cltk_leader(iteration, n_workers, &leader);
  if (rc == DEFT_OK) rc = deft_total_k(N, d, &K);
  if (rc != DEFT_OK) return rc;
  if (rank != leader) {
    *count_out = 0;
    return DEFT_OK;
  }
  if (K > out_cap) return DEFT_ECAP;
  rc = topk_global(g_dev, N, K, idx_out_dev, val_out_dev, ws_dev, ws_bytes, launch_shape, stream);
  if (rc == DEFT_OK) *count_out = K;
  return rc;
}

// ------------------------------------------------------------------------------------------
// The whole sparsifier call (Sec. 4: norms -> Alg. 3 -> Alg. 4 -> Alg. 5) behind one entry.
// ------------------------------------------------------------------------------------------
namespace {
// No sum of squares has this bit pattern: a NaN born from fp32 inputs keeps its low mantissa
// bits clear, and the default NaN is 0x7ff8000000000000.
constexpr uint64_t kSumUnset = ~uint64_t(0);

// How long deft_sparsify polls before it blocks, from the job: 0 = the default.
constexpr int64_t kDefaultSpinUs = 20000;
inline int64_t spin_limit_us(const deft_job& j) {
  return j.spin_us == 0 ? kDefaultSpinUs : (j.spin_us < 0 ? 0 : j.spin_us);
}

// Waits until the norm pass has overwritten every armed entry.  Polls the pinned array for at
// most `limit` microseconds, then blocks in hipStreamSynchronize.
int await_sums(const double* sumsq_pinned, int32_t L, hipStream_t s, int64_t limit) {
  const volatile uint64_t* w = reinterpret_cast<const volatile uint64_t*>(sumsq_pinned);
  int32_t cur = 0;
  if (limit > 0) {
    const auto t0 = std::chrono::steady_clock::now();
    uint32_t spins = 0;
    for (;;) {
      while (cur < L && w[cur] != kSumUnset) ++cur;
      if (cur == L) break;
      __builtin_ia32_pause();
      if ((++spins & 255u) == 0 &&
          std::chrono::duration_cast<std::chrono::microseconds>(std::chrono::steady_clock::now() - t0)
                  .count() > limit)
        break;
    }
  }
  if (cur < L) {
    HIP_TRY(hipStreamSynchronize(s));
    while (cur < L && w[cur] != kSumUnset) ++cur;
    if (cur < L) return DEFT_EHIP;
  }
  std::atomic_thread_fence(std::memory_order_acquire);
  return DEFT_OK;
}
}  // namespace

namespace {
// The whole call.  Plain: the vector `src` is normed and selected from.  Accumulating (grad and
// acc given): acc = src + eta * grad is formed by the norm pass and selected from.
int sparsify(const deft_job* job, const float* src, const float* grad, float eta, float* acc,
             int64_t iteration, void* stream, void* norms_done_event, int32_t* my_count_out,
             int64_t* k_r_out) {
  const float* g_dev = acc ? acc : src;  // what the selection reads
  if (!job || !src || !my_count_out || !k_r_out) return DEFT_EINVAL;
  if (acc && (!grad || (reinterpret_cast<uintptr_t>(grad) & 15u) ||
              (reinterpret_cast<uintptr_t>(src) & 15u)))
    return DEFT_EINVAL;
  const deft_job& j = *job;
  if (!j.offsets_host || !j.offsets_dev || !j.sizes_host || !j.sumsq_pinned || !j.norms_host ||
      !j.k_host || !j.owner_bin_host || !j.my_layers_host || !j.seg_off_host || !j.ws_dev)
    return DEFT_EINVAL;
  if (j.n_workers < 1 || j.rank < 0 || j.rank >= j.n_workers || iteration < 0 ||
      !(j.d > 0.0 && j.d <= 1.0) || j.out_cap < 0 || !valid_shape(j.launch_shape))
    return DEFT_EINVAL;
  int rc = deft_check_layout(j.offsets_host, j.L, j.N);
  if (rc != DEFT_OK) return rc;
  for (int32_t l = 0; l < j.L; ++l)
    if (j.sizes_host[l] != j.offsets_host[l + 1] - j.offsets_host[l] || j.sizes_host[l] < 1)
      return DEFT_EINVAL;
  if ((reinterpret_cast<uintptr_t>(g_dev) & 15u) || (reinterpret_cast<uintptr_t>(j.ws_dev) & 15u))
    return DEFT_EINVAL;
  if (j.ws_bytes < deft_workspace_bytes(DEFT_OP_SELECT, j.N, j.L) ||
      j.ws_bytes < deft_workspace_bytes(DEFT_OP_NORMS, j.N, j.L))
    return DEFT_EWS;
  if (!j.idx_out_dev || !j.val_out_dev) return DEFT_EINVAL;
  hipStream_t s = static_cast<hipStream_t>(stream);
  // Everything that can be refused without the data has been; from here on work is enqueued.

  volatile uint64_t* arm = reinterpret_cast<volatile uint64_t*>(j.sumsq_pinned);
  for (int32_t l = 0; l < j.L; ++l) arm[l] = kSumUnset;
  std::atomic_thread_fence(std::memory_order_seq_cst);
  rc = run_norms(src, grad, eta, acc, j.N, j.offsets_dev, j.L, j.sumsq_pinned, j.ws_dev, j.ws_bytes,
                 stream);
  if (rc != DEFT_OK) return rc;
  if (norms_done_event) HIP_TRY(hipEventRecord(static_cast<hipEvent_t>(norms_done_event), s));
  // While the host waits and plans, clear the histogram area of a layout that does not depend on
  // the plan (the norm pass's partial sums share the workspace: stream order keeps them safe).
  Precleared pre;
  pre.m_cap = j.L;
  pre.chunks_cap = max_chunks(j.N, j.L);
  {
    const SelectLayout w = select_layout(pre.m_cap, pre.chunks_cap);
    const size_t words = clear_words(w);
    const unsigned blocks = (unsigned)std::min<size_t>((words + 4 * kThreads - 1) / (4 * kThreads), 1024);
    zero_words_kernel<<<blocks, kThreads, 0, s>>>(
        reinterpret_cast<uint32_t*>(static_cast<char*>(j.ws_dev) + w.hist), words);
    HIP_TRY(hipGetLastError());
  }
  rc = await_sums(j.sumsq_pinned, j.L, s, spin_limit_us(j));
  if (rc != DEFT_OK) return rc;

  rc = deft_norms_from_sumsq(j.sumsq_pinned, j.L, j.norms_host);
  if (rc != DEFT_OK) return rc;
  rc = deft_alloc_k(j.norms_host, j.sizes_host, j.L, j.N, j.d, j.k_host);
  if (rc != DEFT_OK) return rc;
  int32_t cnt = 0;
  rc = deft_assign_layers(j.sizes_host, j.k_host, j.L, j.n_workers, iteration, j.rank,
                          j.owner_bin_host, j.my_layers_host, &cnt);
  if (rc != DEFT_OK) return rc;
  rc = select_layers(g_dev, j.N, j.offsets_host, j.k_host, j.L, j.my_layers_host, cnt, j.idx_out_dev,
                     j.val_out_dev, j.seg_off_host, j.out_cap, j.ws_dev, j.ws_bytes, j.launch_shape,
                     stream, &pre);
  if (rc != DEFT_OK) return rc;
  *my_count_out = cnt;
  *k_r_out = j.seg_off_host[cnt];
  return DEFT_OK;
}
}  // namespace

extern "C" int deft_sparsify(const deft_job* job, const float* g_dev, int64_t iteration,
                             void* stream, void* norms_done_event, int32_t* my_count_out,
                             int64_t* k_r_out) {
  return sparsify(job, g_dev, nullptr, 0.0f, nullptr, iteration, stream, norms_done_event,
                  my_count_out, k_r_out);
}

extern "C" int deft_accumulate_sparsify(const deft_job* job, const float* e_dev,
                                        const float* grad_dev, float eta, float* acc_dev,
                                        int64_t iteration, void* stream, void* norms_done_event,
                                        int32_t* my_count_out, int64_t* k_r_out) {
  if (!grad_dev || !acc_dev) return DEFT_EINVAL;
  return sparsify(job, e_dev, grad_dev, eta, acc_dev, iteration, stream, norms_done_event,
                  my_count_out, k_r_out);
}

// ------------------------------------------------------------------------------------------
// The norm pass for callers that cannot allocate or bring a workspace: its per-chunk partial
// sums live in a file-scope device array.
// ------------------------------------------------------------------------------------------
namespace {
constexpr int64_t kStaticNormMaxElems = DEFT_NOALLOC_MAX_ELEMS;
constexpr size_t kStaticNormChunks = (size_t)((kStaticNormMaxElems + kNormChunk - 1) / kNormChunk);
constexpr int kMaxDevices = 64;
}  // namespace

// head[kStaticNormChunks] followed by tail[kStaticNormChunks]: 4 MiB on every GPU the library
// runs on, held until the process ends.  In host code this name is only a handle for
// hipGetSymbolAddress; the device address it resolves to is what kernels and copies receive.
static __device__ __align__(256) double scratch[2 * kStaticNormChunks];

namespace {
std::mutex g_scratch_mutex;
double* g_scratch_ptr[kMaxDevices] = {};  // per device: each GPU holds its own copy of the array

// Device address of `scratch` on the current device, resolved once per device.
int static_scratch(double** out) {
  int dev = -1;
  HIP_TRY(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) return DEFT_EHIP;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    double* ptr = nullptr;
    HIP_TRY(hipGetSymbolAddress(reinterpret_cast<void**>(&ptr), HIP_SYMBOL(scratch)));
    if (!ptr) return DEFT_EHIP;
    g_scratch_ptr[dev] = ptr;
  }
  *out = g_scratch_ptr[dev];
  return DEFT_OK;
}
}  // namespace

extern "C" int deft_layer_norms_noalloc(const float* g_dev, int64_t N, const int64_t* offsets_dev,
                                        int32_t L, double* sumsq_dev, void* stream) {
  if (!g_dev || !offsets_dev || !sumsq_dev || L < 1 || N < 1) return DEFT_EINVAL;
  if (N > kMaxN) return DEFT_ERANGE;
  if (N > kStaticNormMaxElems) return DEFT_ELIMIT;
  if (reinterpret_cast<uintptr_t>(g_dev) & 15u) return DEFT_EINVAL;
  double* ptr = nullptr;
  const int rc = static_scratch(&ptr);
  if (rc != DEFT_OK) return rc;
  // Every chunk of this call writes its head and tail entry before norm_finish_kernel reads
  // them, so what an earlier call left in the array needs no clearing.
  return launch_norms(g_dev, nullptr, 0.0f, nullptr, N, offsets_dev, L, sumsq_dev, ptr,
                      ptr + kStaticNormChunks, static_cast<hipStream_t>(stream));
}
