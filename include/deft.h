/*
 * deft.h -- C ABI of the DEFT gradient-selection library for AMD MI355X (gfx950).
 *
 * The library covers the sparsifier of "DEFT: Exploiting Gradient Norm Difference between
 * Model Layers for Scalable Gradient Sparsification" (Yoon & Oh, ICPP 2023), Sec. 4:
 *   1) two-stage gradient vector partitioning            (Alg. 2, Sec. 4.1)   host
 *   2) per-layer gradient norm + local k assignment      (Alg. 3, Sec. 4.2)   device + host
 *   3) bin-packing layer allocation to workers           (Alg. 4, Sec. 4.3)   host
 *   4) layer-wise Top-k selection on the worker's layers (Alg. 5, Sec. 4.4)   device
 * and the conventional Top-k over the whole vector (Sec. 1, Sec. 3.1) as comparison path.
 *
 * Conventions
 *   - The gradient vector g is flat fp32 in device memory, N = n_g elements, N < 2^31, and
 *     its base address is 16-byte aligned.  Layer l is g[offsets[l] .. offsets[l+1]).
 *   - "_dev" pointers are device memory (or host memory the device can access, where
 *     noted); "_host" pointers and unmarked pointers of the host-only calls are ordinary
 *     host memory.  The caller owns every buffer.  The library allocates and frees no
 *     device memory and keeps no state between calls.
 *   - Device calls only enqueue work on `stream` (a hipStream_t passed as void*, NULL = the
 *     default stream).  They never synchronise (deft_sparsify alone waits on the host for
 *     its own norm pass); outputs are valid once the caller has
 *     synchronised the stream.  The workspace must stay untouched until then.  Host
 *     arrays passed to a device call are consumed before it returns.
 *     A device call launches kernels only (no allocation, no memset, no copy), so it may be
 *     recorded in a HIP graph; the graph then replays the plan (k, layer list) it was given.
 *   - Every call returns a status: DEFT_OK (0) or a negative code.  On DEFT_EINVAL,
 *     DEFT_ERANGE, DEFT_EWS and DEFT_ECAP nothing has been written or enqueued.
 *   - Magnitudes are compared through the integer key (bit pattern & 0x7fffffff): exact
 *     order of |g| for all non-NaN values, -0 equal to +0, NaN above infinity.  Among equal
 *     magnitudes the lower index is selected first.  Selected entries are reported in
 *     ascending index order with their original bit pattern.
 *   - Results are deterministic: the same inputs give the same bits.
 *   - The library reads no environment variable and has no settings of its own: what tunes a
 *     call travels in its arguments.  The selection calls take a launch shape: DEFT_SHAPE_AUTO
 *     picks by size (long-vector kernels above 2^26 selected-from elements, and above 2^25 where
 *     most of them lie in segments that can take the one-read pass); DEFT_SHAPE_SHORT and
 *     DEFT_SHAPE_LONG force one; _LONG_PLAIN and _LONG_SAMPLED also fix whether the long-vector
 *     kernels sample a segment ahead of their first pass (by default they do where it pays).
 *     The shape changes speed only, never results.
 */
#ifndef DEFT_H
#define DEFT_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define DEFT_OK 0
#define DEFT_EINVAL (-1) /* null pointer, bad count, bad density/rank, malformed offsets or k */
#define DEFT_ERANGE (-2) /* N >= 2^31: indices are 32-bit */
#define DEFT_EWS (-3)    /* workspace too small (see deft_workspace_bytes) */
#define DEFT_ECAP (-4)   /* output capacity too small */
#define DEFT_EHIP (-5)   /* HIP launch/runtime error */
#define DEFT_ELIMIT (-6) /* size beyond the built-in scratch of deft_layer_norms_noalloc */

#define DEFT_SHAPE_AUTO 0
#define DEFT_SHAPE_SHORT 1
#define DEFT_SHAPE_LONG 2
#define DEFT_SHAPE_LONG_PLAIN 3   /* long-vector kernels, no sampling ahead of the first pass */
#define DEFT_SHAPE_LONG_SAMPLED 4 /* long-vector kernels, every segment sampled if it can be */

/*
 * After a selection call that ran the long-vector kernels, the first DEFT_STAT_WORDS 32-bit words
 * of its workspace tell how the segments' first pass went (diagnostics; valid once the stream is
 * synchronised): how many segments had the threshold placed by a sample and were read once, how
 * many of those had to be redone in full because the exact check refuted the sample, and how many
 * were treated in full from the start (all three are zero after a call that sampled nothing).
 */
#define DEFT_STAT_BOUNDED 0
#define DEFT_STAT_REDONE 1
#define DEFT_STAT_FULL 2
#define DEFT_STAT_WORDS 4

#define DEFT_OP_NORMS 0
#define DEFT_OP_SELECT 1
#define DEFT_OP_TOPK_GLOBAL 2

/* Static, human-readable text for a status code. */
const char* deft_strerror(int status);

/*
 * Alg. 2 (Sec. 4.1): tensor sizes -> layer offsets.  A tensor holding more than n_g/n_workers
 * elements is cut into n_workers contiguous fractions whose sizes differ by at most one
 * (larger first); other tensors become one layer.  Empty tensors/fractions yield no layer.
 *   tensor_sizes[T]  in   sizes in model order (>= 0); n_g is their sum
 *   offsets[cap+1]   out  offsets[0] = 0 ... offsets[L] = n_g
 *   layer_tensor[cap] out (may be NULL) source tensor of each layer
 *   cap              in   capacity in layers; T * n_workers always suffices
 *   L_out            out  number of layers
 * Errors: DEFT_EINVAL (null, T < 0, n_workers < 1, negative size), DEFT_ECAP (cap too small),
 * DEFT_ERANGE (n_g >= 2^31).
 */
int deft_partition(const int64_t* tensor_sizes, int32_t T, int32_t n_workers, int64_t* offsets,
                   int32_t* layer_tensor, int32_t cap, int32_t* L_out);

/*
 * Host-side validation of a layer layout: offsets[0] == 0, non-decreasing, offsets[L] == N,
 * 1 <= L, 0 <= N < 2^31.  Returns DEFT_OK, DEFT_EINVAL or DEFT_ERANGE.
 */
int deft_check_layout(const int64_t* offsets_host, int32_t L, int64_t N);

/*
 * Sec. 4.2, first sentence of its second paragraph: the gradient norm of each layer.
 * Enqueues one streaming pass over g that writes sumsq[l] = sum of g_i^2 over layer l,
 * accumulated in fp64 (the square of an fp32 value is exact in fp64) with a fixed
 * reduction order.  The L2 norm is sqrt(sumsq[l]), taken by the caller.
 *   g_dev          in   N floats, device, 16-byte aligned
 *   offsets_dev    in   L+1 int64, device; must satisfy deft_check_layout (not re-checked on
 *                       the device: malformed offsets give meaningless sums, never an
 *                       out-of-range access)
 *   sumsq_dev      out  L doubles; device memory or pinned host memory mapped to the device
 *   ws_dev         scratch, deft_workspace_bytes(DEFT_OP_NORMS, N, L) bytes, 16-byte aligned
 * Errors: DEFT_EINVAL, DEFT_ERANGE, DEFT_EWS, DEFT_EHIP.
 */
int deft_layer_norms(const float* g_dev, int64_t N, const int64_t* offsets_dev, int32_t L,
                     double* sumsq_dev, void* ws_dev, size_t ws_bytes, void* stream);

/*
 * deft_layer_norms for callers that can neither allocate device memory nor bring a workspace:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * kernels, same results, same arguments minus the workspace: the per-chunk partial sums go to
 * an array built into the library's device image (4 MiB on every GPU the library runs on, held
 * until the process ends).  The call allocates and frees nothing.
 *   N  at most DEFT_NOALLOC_MAX_ELEMS (2^30 elements); beyond that DEFT_ELIMIT, nothing enqueued
 * The first call on a device looks up the array's address there (once per device; make that call
 * before a capture begins).  All calls on one GPU share that GPU's array: calls whose kernels
 * may overlap on one GPU (different streams, no ordering between them) race on it -- order them.
 * The array keeps the previous call's partial sums; every entry a call reads it has written
 * itself first, so nothing needs clearing.
 * Errors: DEFT_EINVAL, DEFT_ERANGE, DEFT_ELIMIT, DEFT_EHIP.
 */
#define DEFT_NOALLOC_MAX_ELEMS (1ll << 30)
int deft_layer_norms_noalloc(const float* g_dev, int64_t N, const int64_t* offsets_dev, int32_t L,
                             double* sumsq_dev, void* stream);

/*
 * First statement of Alg. 3 (k = n_g * d; density is defined in the footnote of Sec. 1):
 * K = floor(N * d + 0.5) in fp64, the number of entries the sparsifier selects in total.
 * Errors: DEFT_EINVAL (null, N < 1, d outside (0,1]), DEFT_ERANGE (N >= 2^31).
 */
int deft_total_k(int64_t N, double d, int64_t* K_out);

/*
 * norms[l] = sqrt(sumsq[l]) on the host (IEEE correctly-rounded square root): the step between
 * deft_layer_norms and deft_alloc_k.  In-place use (norms == sumsq) is allowed.
 * Errors: DEFT_EINVAL (null, L < 1, negative or NaN entry).
 */
int deft_norms_from_sumsq(const double* sumsq, int32_t L, double* norms);

/*
 * Alg. 3 (Sec. 4.2): local k of every layer.  k_remain starts at K = floor(N*d + 0.5).
 * Layers are served by descending norm (equal norms: lower position first); each receives
 * floor(k_remain * norm / norm_remain), at least 1 and at most its size, where norm_remain is
 * the sum of the norms of the layers not yet served.  All arithmetic is IEEE fp64 without
 * fused multiply-add.  The sum of k is K unless the lower/upper clamps bind on the tail.
 *   norms[L]  in   L2 norms (not squared), finite, >= 0
 *   sizes[L]  in   layer sizes, >= 1
 *   k_out[L]  out  1 <= k_out[l] <= sizes[l], by layer position
 * Errors: DEFT_EINVAL (null, L < 1, size < 1, negative or non-finite norm, d outside (0,1],
 * N < 1).
 */
int deft_alloc_k(const double* norms, const int64_t* sizes, int32_t L, int64_t N, double d,
                 int64_t* k_out);

/*
 * Alg. 4 (Sec. 4.3, Eq. 3): cost c_x = size_x * ln(k_x); the costliest unplaced layer (lowest
 * position among equals) goes to the lightest bin (lowest id among equals) until all are
 * placed.  The caller's bin is (iteration % n_workers + rank) % n_workers.  The broadcast of
 * the bins by the delegated worker is left to the caller (every caller can compute them).
 *   sizes[L], k[L]   in   sizes >= 1, 1 <= k <= size
 *   owner_bin[L]     out  bin id of each layer (the 4L-byte payload of Sec. 4.3)
 *   my_layers[L]     out  layers of the caller's bin in the order they were placed
 *   my_count         out  how many
 * Errors: DEFT_EINVAL (null, L < 1, n_workers < 1, rank outside [0,n), iteration < 0, bad k).
 */
int deft_assign_layers(const int64_t* sizes, const int64_t* k, int32_t L, int32_t n_workers,
                       int64_t iteration, int32_t rank, int32_t* owner_bin, int32_t* my_layers,
                       int32_t* my_count);

/*
 * Eq. 4-8: C_i for every bin, C(n) = max_i C_i, f(n), C_trivial(n) and f_trivial(n) for a
 * given assignment.  out5 = {C(n), f(n), C_trivial(n), f_trivial(n), n_g*ln(K)}.
 *   C_i[n_workers] out (may be NULL)
 * Errors: DEFT_EINVAL.
 */
int deft_cost_model(const int64_t* sizes, const int64_t* k, const int32_t* owner_bin, int32_t L,
                    int32_t n_workers, int64_t N, int64_t K, double* C_i, double* out5);

/*
 * Alg. 5 (Sec. 4.4): for each of the caller's layers, in the given order, the k_l entries of
 * largest magnitude; indices are global (layer start added).  Segment j of the output holds
 * layer my_layers[j]: entries seg_off[j] .. seg_off[j+1], ascending index, with the gathered
 * values (the (index, value) pairs Alg. 1 exchanges afterwards).
 *   g_dev              in   N floats, device, 16-byte aligned
 *   offsets_host[L+1]  in   host; must satisfy deft_check_layout (re-checked)
 *   k_host[L]          in   host; 0 <= k[l] <= size of layer l
 *   my_layers_host[my_count] in host; layer positions in [0, L); my_count >= 0
 *   idx_out_dev        out  out_cap int32, device
 *   val_out_dev        out  out_cap floats, device
 *   seg_off_host[my_count+1] out host, written before the call returns
 *   out_cap            in   capacity of idx/val in entries; must be >= sum of the k's
 *   ws_dev             scratch, deft_workspace_bytes(DEFT_OP_SELECT, share, my_count) bytes
 *                      where share >= total size of the caller's layers; 16-byte aligned
 *   launch_shape       in   one of the DEFT_SHAPE_ values
 * my_count == 0 is valid and enqueues nothing.
 * Errors: DEFT_EINVAL, DEFT_ERANGE, DEFT_EWS, DEFT_ECAP, DEFT_EHIP.
 */
int deft_select(const float* g_dev, int64_t N, const int64_t* offsets_host, const int64_t* k_host,
                int32_t L, const int32_t* my_layers_host, int32_t my_count, int32_t* idx_out_dev,
                float* val_out_dev, int64_t* seg_off_host, int64_t out_cap, void* ws_dev,
                size_t ws_bytes, int32_t launch_shape, void* stream);

/*
 * Conventional Top-k sparsifier (Sec. 1; the n = 1 case of Sec. 5.4): the K entries of largest
 * magnitude of the whole vector, ascending index, with values.  0 <= K <= N.
 *   ws_dev  scratch, deft_workspace_bytes(DEFT_OP_TOPK_GLOBAL, N, 1) bytes, 16-byte aligned
 * Errors: DEFT_EINVAL, DEFT_ERANGE, DEFT_EWS, DEFT_EHIP.
 */
int topk_global(const float* g_dev, int64_t N, int64_t K, int32_t* idx_out_dev,
                float* val_out_dev, void* ws_dev, size_t ws_bytes, int32_t launch_shape,
                void* stream);

/*
 * Cyclic local Top-k, the comparison scheme of Sec. 1 and Sec. 3.1: in iteration t the worker
 * t mod n_workers (deft_cltk_leader) selects the conventional Top-k of its own vector, with
 * K = deft_total_k(N, d), for everyone; the other workers select nothing.
 *   count_out  out  K on the leader (idx/val hold K entries once the stream is synchronised),
 *                   0 on every other rank (nothing enqueued, nothing written)
 *   out_cap    in   capacity of idx/val in entries; the leader needs out_cap >= K
 * Other arguments as topk_global.  Errors: those of topk_global; DEFT_EINVAL also for rank outside
 * [0, n_workers), n_workers < 1, iteration < 0, d outside (0,1]; DEFT_ECAP.
 */
int deft_cltk_leader(int64_t iteration, int32_t n_workers, int32_t* leader_out);
int deft_cltk_select(const float* g_dev, int64_t N, double d, int32_t n_workers, int32_t rank,
                     int64_t iteration, int32_t* idx_out_dev, float* val_out_dev, int64_t out_cap,
                     void* ws_dev, size_t ws_bytes, int32_t launch_shape, void* stream,
                     int64_t* count_out);

/*
 * Alg. 1, the step before the sparsifier, fused with the norm pass of Sec. 4.2:
 *   acc[i] = e[i] + eta * grad[i]   (fp32: product rounded, then sum rounded; no fused
 *                                    multiply-add)
 *   sumsq[l] = sum over layer l of acc[i]^2   (fp64, as deft_layer_norms)
 * in one pass (8 bytes read, 4 written per element instead of two passes).
 *   e_dev, grad_dev  in   N floats each, device, 16-byte aligned
 *   acc_dev          out  N floats, device, 16-byte aligned; may be the same buffer as e_dev
 *                         (in-place error feedback); must not overlap grad_dev otherwise
 *   offsets_dev, sumsq_dev, ws_dev, ws_bytes: as for deft_layer_norms (DEFT_OP_NORMS)
 * Errors: DEFT_EINVAL, DEFT_ERANGE, DEFT_EWS, DEFT_EHIP.
 */
int deft_accumulate_norms(const float* e_dev, const float* grad_dev, float eta, float* acc_dev,
                          int64_t N, const int64_t* offsets_dev, int32_t L, double* sumsq_dev,
                          void* ws_dev, size_t ws_bytes, void* stream);

/*
 * Alg. 1, the steps after the index exchange: vals[i] = acc[idx[i]], then acc[idx[i]] = +0, so
 * that acc becomes the next local error.  idx holds `count` distinct positions in [0, N)
 * (the selected indices of all workers are distinct because their layers are disjoint,
 * Sec. 4.3); entries outside [0, N) are skipped and their vals[i] set to 0.  Duplicate
 * entries give unspecified vals for the duplicates.
 *   acc_dev  in/out N floats, device;  idx_dev in, count int32, device;  vals_out_dev out
 * Errors: DEFT_EINVAL (null with count > 0, count < 0, N < 1), DEFT_ERANGE, DEFT_EHIP.
 */
int deft_gather_zero(float* acc_dev, int64_t N, const int32_t* idx_dev, int64_t count,
                     float* vals_out_dev, void* stream);

/*
 * Measurement aid, not a step of the method: one streaming read of the first N - N mod 4096
 * elements of g in the launch shape of deft_layer_norms and nothing else.  Its duration gives the
 * read rate this access pattern reaches on the machine at hand, the ceiling the passes of
 * deft_layer_norms and of the selection are measured against.
 *   out_dev  out  at least 4 bytes of device memory (hardly ever written)
 * Errors: DEFT_EINVAL (null, N < 4096, misaligned g), DEFT_ERANGE, DEFT_EHIP.
 */
int deft_stream_read_probe(const float* g_dev, int64_t N, void* out_dev, void* stream);

/*
 * One sparsifier call (Sec. 4, opening paragraph: norms -> local k -> layer allocation ->
 * layer-wise selection; the Sparsify() of Alg. 1) as a single entry point: the same work, in
 * the same order and with the same results, as
 *   deft_layer_norms -> wait for the sums -> deft_norms_from_sumsq -> deft_alloc_k ->
 *   deft_assign_layers -> deft_select.
 * Unlike the other device calls it BLOCKS the calling thread until the norm pass has
 * delivered its sums (the host plan needs them) and returns with the selection enqueued on
 * `stream`; idx/val are valid once the caller has synchronised the stream.  It waits by
 * reading job->sumsq_pinned (every entry is set to an impossible bit pattern before the norm
 * pass is enqueued and overwritten by it); after job->spin_us microseconds it falls back to
 * hipStreamSynchronize.  Not capturable in a HIP graph (it waits on the host).
 *
 * deft_job holds what stays the same from call to call; the caller fills it once.
 *   N, L, n_workers, rank, d     the job (d in (0,1], rank in [0, n_workers))
 *   launch_shape                 one of the DEFT_SHAPE_ values, as for deft_select
 *   spin_us                      how long to poll for the sums before blocking in the stream
 *                                synchronisation: 0 = default (20000), negative = do not poll
 *   offsets_host / offsets_dev   the same L+1 offsets in host and in device memory
 *   sizes_host[L]                layer sizes (offsets[l+1] - offsets[l])
 *   sumsq_pinned[L]              pinned host memory the device can write (hipHostMalloc);
 *                                holds the sums of squares after the call
 *   norms_host[L], k_host[L], owner_bin_host[L], my_layers_host[L], seg_off_host[L+1]
 *                                outputs of the plan, as for the step-wise calls
 *   idx_out_dev, val_out_dev, out_cap   outputs of deft_select
 *   ws_dev, ws_bytes             scratch, >= max(deft_workspace_bytes(DEFT_OP_NORMS, N, L),
 *                                deft_workspace_bytes(DEFT_OP_SELECT, N, L)); 16-byte aligned
 * Per call:
 *   g_dev              in   N floats, device, 16-byte aligned
 *   iteration          in   rotates the bin -> worker map (Alg. 4)
 *   norms_done_event   in   a hipEvent_t (as void*) recorded on `stream` right after the norm
 *                           pass, or NULL
 *   my_count_out       out  number of layers of the caller's bin
 *   k_r_out            out  number of selected entries (= seg_off_host[my_count])
 * Errors: those of the step-wise calls; DEFT_EHIP also if the sums never arrive.  Arguments
 * are checked before anything is written or enqueued, except DEFT_ECAP: the sum of the k's
 * depends on the data, so it is found after the norm pass; norms, k and the bins are then
 * valid and no selection has been enqueued.
 */
typedef struct deft_job {
  int64_t N;
  int32_t L;
  int32_t n_workers;
  int32_t rank;
  int32_t launch_shape;
  double d;
  const int64_t* offsets_host;
  const int64_t* offsets_dev;
  const int64_t* sizes_host;
  double* sumsq_pinned;
  double* norms_host;
  int64_t* k_host;
  int32_t* owner_bin_host;
  int32_t* my_layers_host;
  int64_t* seg_off_host;
  int32_t* idx_out_dev;
  float* val_out_dev;
  int64_t out_cap;
  void* ws_dev;
  size_t ws_bytes;
  int64_t spin_us;
} deft_job;

int deft_sparsify(const deft_job* job, const float* g_dev, int64_t iteration, void* stream,
                  void* norms_done_event, int32_t* my_count_out, int64_t* k_r_out);

/*
 * Alg. 1, the accumulation step and the sparsifier call that follows it, as a single entry
 * point: acc = e + eta * grad is formed by the norm pass (as deft_accumulate_norms: fp32,
 * product rounded, then sum rounded) and the selection then runs on acc, exactly as
 * deft_sparsify(job, acc_dev, ...) would after deft_accumulate_norms.
 *   e_dev, grad_dev  in   N floats each, device, 16-byte aligned
 *   acc_dev          out  N floats, device, 16-byte aligned; may be the same buffer as e_dev
 * Other arguments, blocking behaviour and errors: as deft_sparsify.
 */
int deft_accumulate_sparsify(const deft_job* job, const float* e_dev, const float* grad_dev,
                             float eta, float* acc_dev, int64_t iteration, void* stream,
                             void* norms_done_event, int32_t* my_count_out, int64_t* k_r_out);

/*
 * Upper bound on the scratch bytes of a device call.
 *   DEFT_OP_NORMS:        elems = N,            count = L
 *   DEFT_OP_SELECT:       elems = total size of the selected layers (N always suffices),
 *                         count = my_count
 *   DEFT_OP_TOPK_GLOBAL:  elems = N,            count ignored
 * Returns 0 for an unknown op or negative arguments.  Orders of magnitude: norms 16 bytes per
 * 4096 elements; selection about 2 bytes per element plus 48 KB per layer and 4 MB, nearly all
 * of it the per-chunk slot arrays, of which a few hundred bytes per chunk are touched.
 */
size_t deft_workspace_bytes(int op, int64_t elems, int32_t count);

#ifdef __cplusplus
}
#endif
#endif /* DEFT_H */
