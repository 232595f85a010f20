/* dct.h -- C ABI of libdct: the hard-thresholding hot path of Dynamic
 * Communication Thresholding (DCT) on one MI355X (gfx950).
 *
 * Everything a worker does to its own data before anything goes on the wire:
 *   DCT-DP (Algorithm 1): pick the magnitude threshold tau as the k-th largest
 *   |W_grad| every L iterations, and every iteration keep the entries with
 *   |W_grad| >= tau, emitted as (index, value) pairs;
 *   DCT-MP (Algorithm 2): per sample (row) keep the k largest |X_act|, and in the
 *   backward pass pass X_grad through the same mask.
 * The dct_ef_* calls are the same two DCT-DP steps with the error-feedback update
 * of Algorithm 1 fused in (the residual is added before, and refreshed after, the
 * compression).  The network transfer and the parameter server are not part of
 * this library.
 *
 * Conventions shared by every call
 *   - Pointers named d_* (and g, x, dy) are DEVICE pointers on the current HIP
 *     device; nothing is copied to or from the host.  Inputs are never modified.
 *   - The library allocates no device memory.  The caller owns every buffer,
 *     including workspaces (sizes from the *_workspace_bytes queries).
 *   - Every call only enqueues kernels on `hip_stream` (a hipStream_t passed as
 *     void*, NULL = the default stream) and returns without synchronising.
 *   - Return value: a dct_status.  Argument errors are detected on the host and
 *     nothing is enqueued.  No C++ type or exception crosses this boundary.
 *   - Magnitude order is the unsigned order of key(x) = bit pattern of x with the
 *     sign bit cleared (31 bits for fp32, 15 bits for bf16).  For non-NaN x this
 *     is the order of |x|; -0 and +0 are equal; denormals are ordered exactly;
 *     NaNs rank above infinity (deterministic, not meaningful).
 *   - Position i precedes j when key[i] > key[j], or the keys are equal and
 *     i < j: ties go to the lower index.
 *   - Indices are 0-based int32; survivors are emitted in ascending index order
 *     and values are copied bit for bit.
 */
#ifndef DCT_H_
#define DCT_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  DCT_OK = 0,
  DCT_ERR_INVALID = 1,   /* bad argument (null, zero size, k out of range, misaligned, ...) */
  DCT_ERR_WORKSPACE = 2, /* workspace pointer null, misaligned or too small                 */
  DCT_ERR_OVERFLOW = 3,  /* reported by the Python binding when count > capacity            */
  DCT_ERR_HIP = 4        /* a kernel launch failed                                          */
} dct_status;

typedef enum { DCT_F32 = 0, DCT_BF16 = 1 } dct_dtype;

typedef enum {
  DCT_GE_TAU = 0, /* the mask of Algorithm 1: keep every key >= tau_key (count varies)      */
  DCT_EXACT_K = 1 /* keep key > tau_key plus the tie_quota lowest-index entries with
                     key == tau_key: exactly k survivors on the vector tau was selected on  */
} dct_mode;

/* The threshold carried from a select iteration to the following reuse
 * iterations (Algorithm 1, the branch that keeps the previous iteration's tau).
 * Lives in DEVICE memory, 16 bytes, 16-byte aligned, caller-owned. */
typedef struct {
  uint32_t tau_key;   /* key of the k-th largest magnitude; always the key of an input element */
  uint32_t n_gt;      /* #{ i : key[i] >  tau_key }                                          */
  uint32_t n_eq;      /* #{ i : key[i] == tau_key }                                          */
  uint32_t tie_quota; /* k - n_gt, in [1, n_eq]                                              */
} dct_threshold;

/* Sentinel written to *d_count_out when dct_threshold_compact finds its
 * workspace uninitialised or refusing, or when one of its bounded waits runs out. */
#define DCT_COUNT_WORKSPACE_ERROR UINT64_MAX

/* tau_key of a threshold record whose selection gave up (see "Concurrency" at
 * dct_select_threshold); the other three words are 0.  No key has bit 31 set, so
 * a compaction with such a record keeps nothing. */
#define DCT_TAU_KEY_ERROR 0xFFFFFFFFu

/* ---------------------------------------------------------------- DCT-DP ---
 * Algorithm 1, threshold selection (the sort of the magnitudes and the pick of
 * the element at rank floor(N*eta)), computed exactly without sorting or copying
 * the gradient: a radix select over the key bits with LDS histograms.  The caller
 * passes the integer number of entries to keep, k; tau is the k-th largest key and
 * the mask keeps every key >= tau.  For a sparsity factor eta (the fraction that
 * is dropped: Sec. 2.2 says tau_i exceeds d*eta values of its row) with the
 * magnitudes sorted ascending and numbered from 0, the element at rank
 * floor(N*eta) is the (N - floor(N*eta))-th largest, so k = N - floor(N*eta).
 *
 *   g          device, n elements of `dt`, contiguous, aligned to the element size
 *   n          1 .. 2^31-1            k   1 .. n
 *   d_thr_out  device, receives the dct_threshold
 *   d_ws       device workspace, 256-byte aligned; contents on entry are irrelevant, it
 *              is scratch.  About 240 KB of counters, histograms and the key sample,
 *              plus, for n >= 2^22, a buffer for the keys that one pass over the vector
 *              finds between two bounds drawn from the sample.  How many those are
 *              depends on k / n: dct_select_threshold_workspace_bytes_for(dt, n, k) asks
 *              for twice the expected number (c4, 0.5 % kept of 2^28: 4 M keys, 16 MB);
 *              dct_select_threshold_workspace_bytes(dt, n) for what the worst k needs
 *              (n/16 keys: 6 % of the vector's bytes) and serves every k.  Any size from
 *              the first on is accepted and used; a buffer that proves too small costs
 *              time (the radix passes then read the vector), never exactness.
 *
 * Concurrency: the last kernel of the call runs all radix passes in one launch.
 * Between two passes up to 64 of its workgroups (one per compute unit, the first
 * of its grid) wait for each other at a grid barrier; after the last pass nobody
 * waits.  A device has room for the waiting workgroups of several selections at a
 * time (four streams at once are tested).  If other work keeps some of them off the
 * device for about a second, the waiting ones give up, every kernel still ends, and
 * the record reads {DCT_TAU_KEY_ERROR, 0, 0, 0}: select again.  The same holds for
 * dct_ef_select_threshold.
 */
size_t dct_select_threshold_workspace_bytes(int dt, uint64_t n);
size_t dct_select_threshold_workspace_bytes_for(int dt, uint64_t n, uint64_t k);
int dct_select_threshold(const void* g, int dt, uint64_t n, uint64_t k, dct_threshold* d_thr_out,
                         void* d_ws, size_t ws_bytes, void* hip_stream);

/* Algorithm 1, the mask of the entries with |W_grad| >= tau and the compressed
 * gradient, fused with an ordered stream compaction: one pass over g, survivors
 * written as idx[j] (ascending) and val[j] = g[idx[j]].
 *
 *   d_thr        device, threshold from dct_select_threshold (possibly of an
 *                earlier iteration: the reuse iterations of Algorithm 1)
 *   mode         DCT_GE_TAU or DCT_EXACT_K
 *   d_idx_out    device int32[capacity]     d_val_out  device dt[capacity]
 *   capacity     pairs the outputs can hold (may be 0).  If more entries survive,
 *                only the first `capacity` in index order are written and the TRUE
 *                count is still reported; nothing is written out of bounds.
 *   d_count_out  device uint64, receives the survivor count (8-byte aligned)
 *   d_ws         device workspace of dct_threshold_compact_workspace_bytes,
 *                256-byte aligned, that was initialised ONCE with
 *                dct_threshold_compact_workspace_init.  Each call leaves it
 *                initialised again, so it can be reused call after call on the same
 *                stream.  Two calls that share a workspace must not overlap.
 *
 * Concurrency.  One launch of one workgroup per compute unit.  When a workgroup has
 * streamed its share it publishes its count and waits for the counts of the
 * LOWER-numbered workgroups of the same launch, which the device started before it:
 * kernels on other streams can delay that wait but not block it.  Only a vector with
 * more than about four million survivors is cut into slices whose exchange involves
 * the whole grid; such a call wants all compute units free (e.g. a stream of its
 * own turn).  Every wait is bounded (dct_set_wait_limit).  If one runs out the call
 * still ends, *d_count_out = DCT_COUNT_WORKSPACE_ERROR, idx / val hold nothing
 * usable, g is untouched (compact again), and the workspace refuses further calls
 * with the same sentinel until it is initialised again.
 */
size_t dct_threshold_compact_workspace_bytes(int dt, uint64_t n);
int dct_threshold_compact_workspace_init(void* d_ws, size_t ws_bytes, void* hip_stream);
int dct_threshold_compact(const void* g, int dt, uint64_t n, const dct_threshold* d_thr, int mode,
                          int32_t* d_idx_out, void* d_val_out, uint64_t capacity, uint64_t* d_count_out,
                          void* d_ws, size_t ws_bytes, void* hip_stream);

/* dct_threshold_compact for callers that cannot allocate: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments,
 * results and errors as dct_threshold_compact, minus the workspace: the exchange
 * area (dct_threshold_compact_static_scratch_bytes() = about 49 KB, whatever n is)
 * is a static array in device memory that each GPU the library runs on holds until
 * the process ends.  The call allocates and frees nothing and needs no
 * initialisation call: it clears the array itself, with a small fill kernel ahead of
 * the compaction on `hip_stream` (two launches per call).  n beyond 2^31 - 1 is
 * DCT_ERR_INVALID as everywhere.  All calls on one GPU share that GPU's array: two
 * calls that overlap in time on one GPU (different streams, no ordering between
 * them) race and give undefined counts; order them.  The first call on a device
 * looks up the array's address (hipGetSymbolAddress); make it outside a graph capture.
 */
size_t dct_threshold_compact_static_scratch_bytes(void);
int dct_threshold_compact_static(const void* g, int dt, uint64_t n, const dct_threshold* d_thr, int mode,
                                 int32_t* d_idx_out, void* d_val_out, uint64_t capacity, uint64_t* d_count_out,
                                 void* hip_stream);

/* ------------------------------------------- DCT-DP with error feedback ---
 * Algorithm 1 keeps what compression drops: the residual is added to the gradient
 * before the selection and set to what the mask removed after it (Fig. 3).  These
 * two calls are dct_select_threshold and dct_threshold_compact applied to the
 * corrected gradient w = g + e, which is never materialised on its own.
 *
 *   dt     DCT_F32 only (anything else: DCT_ERR_INVALID).  w[i] = g[i] + e[i] is
 *          one IEEE-754 binary32 addition, round to nearest even, denormals kept.
 *          A NaN sum has an unspecified payload.
 *   e / e_in / e_out   device, n floats.  They must sit at the same offset within
 *          16 bytes as g (e.g. all 16-byte aligned), else DCT_ERR_INVALID.
 *
 * dct_ef_select_threshold: tau = k-th largest |g + e|; reads g and e, writes only
 * the threshold record.  Workspace as for dct_select_threshold.
 *
 * dct_ef_threshold_compact: survivors of w under `mode`, as (index, w[index])
 * pairs in ascending index order, and the new residual:
 *     e_out[i] = +0    if the pair (i, w[i]) was written to the outputs,
 *     e_out[i] = w[i]  otherwise (bit for bit).
 * An entry that passes the mask but finds no room (count > capacity) is therefore
 * kept in the residual, not lost.  e_out may be the same buffer as e_in (update in
 * place); otherwise the two must not overlap, and g must not overlap e_out.
 * Workspace, count and capacity as for dct_threshold_compact (same workspace).
 *
 * The residual is training state, so delivery is all or nothing.  The call is never
 * cut into slices (a workgroup waits for lower-numbered workgroups only), and one
 * workgroup decides for the whole launch whether every count has arrived.  If
 * *d_count_out reads DCT_COUNT_WORKSPACE_ERROR afterwards -- a wait ran out, or the
 * workspace was not initialised or had refused -- then NO pair was delivered and
 * e_out[i] = g[i] + e_in[i] for every i: the iteration has sent nothing and lost
 * nothing.  idx / val are unspecified.  Initialise the workspace again and go on.
 */
int dct_ef_select_threshold(const void* g, const void* e, int dt, uint64_t n, uint64_t k,
                            dct_threshold* d_thr_out, void* d_ws, size_t ws_bytes, void* hip_stream);
int dct_ef_threshold_compact(const void* g, const void* e_in, void* e_out, int dt, uint64_t n,
                             const dct_threshold* d_thr, int mode, int32_t* d_idx_out, void* d_val_out,
                             uint64_t capacity, uint64_t* d_count_out, void* d_ws, size_t ws_bytes,
                             void* hip_stream);

/* ---------------------------------------------------------------- DCT-MP ---
 * Algorithm 2, forward pass: for every row of X_act the k entries that come
 * first in the magnitude order (exactly k per row, ties to the lower column,
 * rows with fewer than k non-zeros are filled with their lowest-column zeros),
 * written in ascending column order.  This is the row's mask m_i as indices plus
 * the compressed row X_act,i . m_i.
 *
 *   x           device, B rows of D elements of `dt`, unit column stride,
 *               row_stride_elems >= D elements between rows
 *   k           1 .. D
 *   d_idx_out   device int32[B*k] (column indices)   d_val_out  device dt[B*k]
 *   d_tau_out   device dt[B] or NULL: tau_i = magnitude of the k-th entry of row i
 */
int dct_rowtopk_fwd(const void* x, int dt, uint32_t B, uint32_t D, uint64_t row_stride_elems, uint32_t k,
                    int32_t* d_idx_out, void* d_val_out, void* d_tau_out, void* hip_stream);

/* Algorithm 2, backward pass (the gradient passes through the mask of the forward pass):
 * dval[b, j] = dy[b, idx[b, j]].  No new selection takes place.  An index
 * outside [0, D) is not dereferenced; its output element is set to zero.
 */
int dct_rowtopk_bwd(const void* dy, int dt, uint32_t B, uint32_t D, uint64_t row_stride_elems, uint32_t k,
                    const int32_t* d_idx, void* d_dval_out, void* hip_stream);

/* ------------------------------------------- DCT-MP, the mask as a bitmap ---
 * Algorithm 2 sends the masked activations and the mask M.  These calls carry M literally,
 * as a bitmap, instead of k column indices: ceil(D/32) 32-bit words per row, bit
 * (c mod 32) of word (c div 32) set iff column c is kept, plus the k kept values in
 * ascending column order.  For bf16 and k = D/20 that is 2.25 bytes per kept entry
 * on the wire instead of 6.  The kept set is exactly that of dct_rowtopk_fwd.
 *
 *   dct_rowtopk_fwd_bitmask      x -> d_mask_out uint32[B * ceil(D/32)], d_val_out dt[B*k],
 *                                optional d_tau_out (as dct_rowtopk_fwd)
 *   dct_rowtopk_bwd_bitmask      dval[b, j] = dy[b, column of the j-th set bit of row b];
 *                                if a row's mask has fewer than k set bits the remaining
 *                                slots are zero, more than k: the first k count
 *   dct_rowtopk_scatter_bitmask  receiver side: out[b, 0..D) = zeros with val[b, j] at the
 *                                column of the j-th set bit (j < k); the padding between D
 *                                and the row stride is not touched
 */
int dct_rowtopk_fwd_bitmask(const void* x, int dt, uint32_t B, uint32_t D, uint64_t row_stride_elems, uint32_t k,
                            uint32_t* d_mask_out, void* d_val_out, void* d_tau_out, void* hip_stream);
int dct_rowtopk_bwd_bitmask(const void* dy, int dt, uint32_t B, uint32_t D, uint64_t row_stride_elems, uint32_t k,
                            const uint32_t* d_mask, void* d_dval_out, void* hip_stream);
int dct_rowtopk_scatter_bitmask(const uint32_t* d_mask, const void* d_val, int dt, uint32_t B, uint32_t D, uint32_t k,
                                void* d_out, uint64_t out_row_stride_elems, void* hip_stream);

/* --------------------------------------- DCT-MP, the mask as 16-bit indices ---
 * The same three operations with the mask of Algorithm 2 carried as uint16 column
 * indices (D <= 65536; a wider row returns DCT_ERR_INVALID): 4 bytes per kept bf16
 * entry on the wire instead of 6, and unlike the bitmap the cost does not grow as
 * the rows get sparser.  Kept set, order, values and tau are those of
 * dct_rowtopk_fwd; arguments as there except
 *   d_idx_out / d_idx   device uint16[B*k], 2-byte aligned
 * An index >= D is handled as in dct_rowtopk_bwd / dct_rowtopk_scatter.
 */
int dct_rowtopk_fwd_idx16(const void* x, int dt, uint32_t B, uint32_t D, uint64_t row_stride_elems, uint32_t k,
                          uint16_t* d_idx_out, void* d_val_out, void* d_tau_out, void* hip_stream);
int dct_rowtopk_bwd_idx16(const void* dy, int dt, uint32_t B, uint32_t D, uint64_t row_stride_elems, uint32_t k,
                          const uint16_t* d_idx, void* d_dval_out, void* hip_stream);
int dct_rowtopk_scatter_idx16(const uint16_t* d_idx, const void* d_val, int dt, uint32_t B, uint32_t D, uint32_t k,
                              void* d_out, uint64_t out_row_stride_elems, void* hip_stream);

/* ------------------------------------------------------ DCT-DP, many tensors ---
 * Layer-wise compression (Sec. 2.1: every layer's gradient is compressed on its
 * own, with its own threshold) for many tensors with a fixed number of launches:
 * a tensor of a million elements is about a microsecond of memory traffic, so one
 * call per layer is launch latency and nothing else.  The tensors are segments of
 * one address range, described by a table in HOST memory that is read during the
 * call only (it reaches the device as kernel arguments).
 *
 * Per segment s the results are exactly those of dct_select_threshold(g + offset,
 * n, k) and dct_threshold_compact(g + offset, n, thr[s], mode, idx + out_offset,
 * val + out_offset, capacity): indices are relative to the segment's first element.
 * Meant for tensors that sit in cache (the compaction reads each twice); a tensor of
 * hundreds of MB is better served by the single-tensor calls.
 *
 *   g           device base pointer, aligned to the element size
 *   h_segs      host, n_seg entries (1 .. 1024); n in 1 .. 2^31-1, k in 1 .. n
 *               (k is ignored by the compaction); the output ranges
 *               [out_offset, out_offset + capacity) must not overlap
 *   d_thr_out / d_thr   device, n_seg threshold records (16-byte aligned)
 *   d_count_out device uint64[n_seg]: the true survivor count of every segment
 *   d_ws        device, dct_batched_workspace_bytes(dt, h_segs, n_seg) bytes, 256-byte
 *               aligned, scratch (no initialisation needed); one workspace serves both
 *               calls, which must not overlap in time on it
 */
typedef struct {
  uint64_t offset;     /* first element of the tensor, in elements from g                   */
  uint64_t n;          /* elements                                                          */
  uint64_t k;          /* entries to keep (selection)                                       */
  uint64_t out_offset; /* first slot of this tensor's survivors in d_idx_out / d_val_out    */
  uint64_t capacity;   /* slots this tensor may fill (may be 0)                             */
} dct_segment;
size_t dct_batched_workspace_bytes(int dt, const dct_segment* h_segs, uint32_t n_seg);
int dct_select_threshold_batched(const void* g, int dt, const dct_segment* h_segs, uint32_t n_seg,
                                 dct_threshold* d_thr_out, void* d_ws, size_t ws_bytes, void* hip_stream);
int dct_threshold_compact_batched(const void* g, int dt, const dct_segment* h_segs, uint32_t n_seg,
                                  const dct_threshold* d_thr, int mode, int32_t* d_idx_out, void* d_val_out,
                                  uint64_t* d_count_out, void* d_ws, size_t ws_bytes, void* hip_stream);

/* ------------------------------------------------------------ receiver side ---
 * Decompression of the two message formats above (Sec. 2.1 counts compressing
 * and decompressing as the overhead of the method; in Algorithm 2 the next
 * worker consumes the masked activations; the parameter server sums sparse gradients).
 *
 * dct_scatter: (idx, val) pairs -> dense vector of n elements.
 *   d_idx, d_val  device, `capacity` pairs as written by dct_threshold_compact:
 *                 indices ascending and distinct.  An index outside [0, n) is
 *                 skipped.  (If the order is violated the result is unspecified;
 *                 nothing is written out of bounds.)
 *   d_count       device uint64 or NULL.  The number of pairs applied is
 *                 min(*d_count, capacity), read on the device (capacity if NULL;
 *                 0 if *d_count is DCT_COUNT_WORKSPACE_ERROR): the count written by
 *                 the compaction can be passed on without a host round trip.
 *   mode          DCT_SCATTER_ASSIGN: d_out = 0 everywhere, then d_out[idx[j]] = val[j]
 *                 (bit copies; every element of d_out is written exactly once when
 *                 d_out is 16-byte aligned).
 *                 DCT_SCATTER_ADD (DCT_F32 only): d_out[idx[j]] = d_out[idx[j]] + val[j],
 *                 one binary32 addition each; all other elements are left alone.
 *
 * dct_rowtopk_scatter: per-row lists of dct_rowtopk_fwd -> dense rows:
 *   d_out[b, 0..D) = 0, then d_out[b, idx[b, j]] = val[b, j]; elements between D and
 *   the row stride are not touched; a column outside [0, D) is skipped; columns of a
 *   row must be distinct.
 */
typedef enum { DCT_SCATTER_ASSIGN = 0, DCT_SCATTER_ADD = 1 } dct_scatter_mode;
int dct_scatter(const int32_t* d_idx, const void* d_val, const uint64_t* d_count, uint64_t capacity, int dt,
                void* d_out, uint64_t n, int mode, void* hip_stream);
int dct_rowtopk_scatter(const int32_t* d_idx, const void* d_val, int dt, uint32_t B, uint32_t D, uint32_t k,
                        void* d_out, uint64_t out_row_stride_elems, void* hip_stream);

/* ----------------------------------------------------------------- service ---
 * dct_status_string: a static string for a dct_status.
 *
 * dct_set_wait_limit: the number of polls after which a device-side wait of this
 * library gives up (the grid barriers of the selection, the count exchange of the
 * compaction).  Process-wide; 0 restores the default (2^20 polls, about a second).
 * Meant for tests of the give-up paths, which a tiny limit reaches while every
 * kernel still runs to its end; production code has no reason to call it.
 */
void dct_set_wait_limit(uint32_t polls);
const char* dct_status_string(int status);

#ifdef __cplusplus
}
#endif
#endif /* DCT_H_ */
