/*
 * fleet.h -- C ABI of the MI355X decode-step megakernel.
 *
 * One decode step of a Qwen3-style decoder stack (paper section 2.2: RMSNorm,
 * QKV projection, attention over the KV cache, output projection, RMSNorm +
 * gate/up projection, SiLU x multiply, down projection + residual; model shape
 * of section 5.2) runs as ONE persistent HIP kernel that walks a static task
 * graph (paper sections 3.1, 4.1, 4.2): wavefront-, CU-, chiplet- and
 * device-scoped tasks, per-XCD task queues, event counters with two-level
 * (XCD-local, then device) signalling.
 *
 * Conventions
 *   - every function that returns int returns 0 (FLEET_OK) or a negative fleet_err code;
 *     nothing throws or aborts (the closed-form helpers return -1 or 0.0 for a
 *     non-positive divisor).  fleet_strerror() names a code.
 *   - "device" pointers are HIP device memory of the current device, "host"
 *     pointers are ordinary host memory.  The library never takes ownership of
 *     a caller buffer.
 *   - bf16 tensors are raw 16-bit patterns; matrices are [out_features,
 *     in_features] row-major, in_features contiguous (paper section 4.3: the
 *     partition of chiplet k starts k*(N/8)*K elements after the base).
 *   - one step in flight per fleet_t; calls on one fleet_t are not thread-safe.
 */
#ifndef FLEET_H
#define FLEET_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct fleet fleet_t; /* opaque */

enum fleet_err {
  FLEET_OK = 0,
  FLEET_EINVAL = -1,   /* bad shape, null pointer, batch out of range, ...      */
  FLEET_ENOMEM = -2,   /* host or device allocation failed                       */
  FLEET_EHIP = -3,     /* a HIP call failed; see fleet_last_status().hip_error   */
  FLEET_ETIMEOUT = -4, /* a dependency wait ran out of time; the step aborted    */
  FLEET_ESMALL = -5,   /* output buffer too small; *len holds the needed size    */
  FLEET_EDEVICE = -6,  /* the device cannot hold the persistent grid             */
  FLEET_ETOOBIG = -7   /* fleet_decode_step_static: the step needs more working
                          memory than FLEET_STATIC_SCRATCH_BYTES                  */
};

/* Task scheduling (paper section 3.2 and Figure "tiling"). */
enum fleet_sched {
  FLEET_SCHED_COOPERATIVE = 0, /* N-split per XCD, M-major tile order inside (M-tile) */
  FLEET_SCHED_UNAWARE = 1,     /* 2-D tiles dealt to any worker, N-major               */
  FLEET_SCHED_MSPLIT = 2       /* the batch's m-tiles are split over the XCDs (section 3.2,
                                  "M-split"): with T m-tiles, n_xcd / T XCDs share one
                                  m-tile and split N among them; falls back to
                                  COOPERATIVE where T < 2 or T does not divide n_xcd   */
};

enum fleet_flags {
  FLEET_FLAG_TRACE = 1,        /* record per-task tickets and timestamps               */
  FLEET_FLAG_SINGLE_LEVEL = 2, /* every worker signals the device counter itself       */
  FLEET_FLAG_SEPARATE_NORM = 4,/* RMSNorm as CU-tasks also on the FMA path (default there:
                                  fused into the consuming GEMV); fleet_gemm: activations
                                  read from global memory instead of an LDS copy        */
  FLEET_FLAG_CHAINED = 8,      /* fleet_gemm: rep i+1 waits for rep i's event          */
  FLEET_FLAG_TIMING = 16,      /* record per-task timestamps only (no tickets: cheaper) */
  FLEET_FLAG_NO_SPLITK = 32,   /* MFMA GEMMs: never split K over workers (one k-slice)  */
  FLEET_FLAG_NO_STREAM = 64,   /* weight loads without the non-temporal (streaming)
                                  cache hint (section 3.2, cache-modifier flavours)     */
  FLEET_FLAG_NO_RESIDENT = 128,/* MFMA GEMMs: never hold a worker's whole weight share in
                                  registers across the dependency wait (small GEMMs then
                                  use split-K tiles)                                    */
  FLEET_FLAG_UNFUSED_SILU = 256,/* gate|up GEMM stores its fp32 sums; SiLU(gate) x up runs as
                                  a stage of CU-tasks of its own (section 3.2, operator
                                  fusion ablation)                                      */
  FLEET_FLAG_NT_STORES = 2048,  /* partial sums handed over inside one XCD (split-K GEMM tiles,
                                  split-KV attention) are stored with the non-temporal hint
                                  (section 3.2, cache-modifier flavours: nt stores on/off)  */
  FLEET_FLAG_PACKED_ONLY = 1024 /* every batch size runs the MFMA kernels on the library's
                                  packed weight copy: the caller may free wqkv, wo, wgu, wdown
                                  and lm_head once fleet_create has returned (one copy of
                                  the GEMM weights in device memory instead of two)     */
};

typedef struct {
  int32_t n_layers, hidden, n_q_heads, n_kv_heads, head_dim, ffn;
  int32_t vocab;      /* 0: no final norm / LM head                                     */
  int32_t max_batch;  /* 1..128 (max_batch * n_kv_heads <= 1024)                         */
  int32_t max_seq;    /* KV slots per sequence; positions[b] < max_seq                   */
  float rms_eps;      /* 1e-6                                                            */
  float rope_theta;   /* 1e6                                                             */
  int32_t sched_mode; /* enum fleet_sched                                                */
  int32_t tile_m;     /* GEMM tile height along the batch on the MFMA path: 16, 32, 64, or
                         0 = whole batch rounded up to 16 (reads each weight once).
                         Batches above 64 use 64-row tiles (0) or the given height.
                         Batch 1 runs FMA GEMV kernels, larger batches bf16 MFMA
                         kernels; the environment variable FLEET_FMA_MAX_BATCH (0..8),
                         read once by fleet_create (and by fleet_gemm and
                         fleet_graph_build per call), moves that switch                 */
  int32_t flags;      /* enum fleet_flags                                                */
} fleet_shape_t;

/* All device pointers, bf16, caller-owned, read-only, alive until fleet_destroy.
 * The per-layer members are HOST arrays of n_layers device pointers.
 * The FMA GEMV kernels (small batches) read these matrices in place.  When max_batch
 * reaches the MFMA kernels (see tile_m), fleet_create also makes a private repacked copy
 * of wqkv, wo, wgu, wdown and lm_head (same size again in device memory), which those
 * kernels read: a change the caller makes to these matrices after fleet_create is then
 * seen by small batches only. */
typedef struct {
  const void *embed;          /* [vocab, hidden] or NULL                                 */
  const void *const *ln1;     /* [hidden]                                                */
  const void *const *wqkv;    /* [(nq + 2 nkv) * head_dim, hidden], rows Q | K | V       */
  const void *const *q_norm;  /* [head_dim]                                              */
  const void *const *k_norm;  /* [head_dim]                                              */
  const void *const *wo;      /* [hidden, nq * head_dim]                                 */
  const void *const *ln2;     /* [hidden]                                                */
  const void *const *wgu;     /* [2 * ffn, hidden], rows gate | up                       */
  const void *const *wdown;   /* [hidden, ffn]                                           */
  const void *final_norm;     /* [hidden] or NULL                                        */
  const void *lm_head;        /* [vocab, hidden] or NULL                                 */
} fleet_weights_t;

typedef struct {
  int32_t code;        /* FLEET_OK, FLEET_ETIMEOUT, ...                                  */
  int32_t hip_error;   /* last hipError_t seen by the library                            */
  int32_t task;        /* task whose wait timed out, or -1                               */
  int32_t event;       /* event it waited for                                            */
  int32_t observed;    /* counter value seen                                             */
  int32_t needed;      /* counter value needed                                           */
  int32_t n_xcd;       /* XCDs found on the device                                       */
  int32_t workers[8];  /* workgroups that registered on each XCD in the last step        */
} fleet_status_t;

/*
 * fleet_create: validate the shape, probe the device (CU count, XCD count), repack the
 * GEMM weights into a private copy (max_batch on the MFMA path), build and upload the task
 * graph of every batch bucket (powers of two up to max_batch, and max_batch itself; with
 * vocab > 0 and embed also the graphs of fleet_decode_tokens), allocate the working memory
 * of one step, and build the RoPE table.  Paper section 4.3 (task registration at model
 * load).  *out is set on success; on failure everything allocated so far is freed.
 * Everything a step needs exists afterwards: the step calls allocate and copy nothing, and
 * a step of any batch <= max_batch runs the graph of the smallest bucket that holds it (the
 * tasks of the rows it does not have only follow their events; paper section 2.3: no
 * graph per batch size has to be captured on the way).
 * Device memory the library owns besides the packed copy: the descriptors of the graphs (a
 * few MB each), the activations of one step (a few MB), and, on the MFMA path, the partial
 * sums of split-K GEMM tiles: k-slices x padded batch x the widest split output, fp32, once
 * per XCD under the XCD-aware schedules (8 x 8 MB for the Qwen3-8B shape at batch 64).
 * Requirements: head_dim == 128, n_q_heads a multiple of n_kv_heads with ratio <= 4, vocab
 * a multiple of 16, hidden and ffn multiples of 32, at most 120 layers; every weight matrix smaller than 2 GiB
 * and max_seq * 256 < 2^31 (the kernels use 32-bit byte offsets inside a matrix and inside
 * one (sequence, kv head) stream of the cache).  Anything else: FLEET_EINVAL.
 */
int fleet_create(const fleet_shape_t *shape, const fleet_weights_t *weights, fleet_t **out);

/*
 * fleet_decode_step: one decode step for `batch` sequences, asynchronous on
 * `stream` (a hipStream_t; NULL = the default stream).  Paper section 2.2 for
 * what is computed, sections 4.1-4.2 for how it is executed.
 *   hidden_in  device bf16 [batch, hidden], or NULL to gather embed[tokens[b]]
 *   tokens     device int32 [batch] (used when hidden_in == NULL)
 *   k_cache, v_cache  device bf16 [n_layers][max_batch][n_kv][max_seq][head_dim];
 *              slot positions[b] of every layer is written, slots 0..positions[b]
 *              are read
 *   positions  device int32 [batch]: index of the new token (= valid slots before
 *              the step); not advanced by the library
 *   hidden_out device fp32 [batch, hidden]: residual stream after the last layer
 *   logits     device fp32 [batch, vocab], or NULL: the step then ends after the last
 *              layer and the final norm (no LM head)
 * hidden_in, the caches, hidden_out and logits must be 16-byte aligned (FLEET_EINVAL
 * otherwise): the kernels move them in 16-byte pieces.
 * The call launches two kernels on `stream` and does nothing else: no allocation, no
 * copy, no synchronisation (it can be captured into a HIP graph).
 * A dependency wait that times out aborts the step on the device; the next
 * fleet_last_status() reports FLEET_ETIMEOUT.
 * The result is a function of the inputs alone: every reduction has a fixed order, so
 * repeating the step on the same inputs gives the same bits (for a given batch size,
 * schedule and tile height).
 */
int fleet_decode_step(fleet_t *f, int32_t batch, const void *hidden_in, const int32_t *tokens,
                      void *k_cache, void *v_cache, const int32_t *positions,
                      float *hidden_out, float *logits, void *stream);

/*
 * fleet_decode_layers (test / measurement): layers [layer_begin, layer_end) on an
 * fp32 residual stream.  x_in, x_out device fp32 [batch, hidden] (may alias);
 * logits is written only when layer_end == n_layers and logits != NULL.  The
 * other arguments are as in fleet_decode_step.  Same per-layer computation and
 * the same task graph as the full step (paper section 2.2).
 */
int fleet_decode_layers(fleet_t *f, int32_t batch, int32_t layer_begin, int32_t layer_end,
                        const float *x_in, void *k_cache, void *v_cache,
                        const int32_t *positions, float *x_out, float *logits, void *stream);

/* fleet_destroy: free everything the library allocated.  NULL is accepted. */
int fleet_destroy(fleet_t *f);

/*
 * fleet_decode_step_static: fleet_decode_step for callers that cannot allocate device
 * memory and want none held per fleet_t for the step's working set (code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc).  The working memory of the
 * step -- activations, split-KV and split-K partial sums, dependency counters, status block
 * -- lives in a static device array of FLEET_STATIC_SCRATCH_BYTES that the library's code
 * object carries (every GPU the library runs on holds it until the process ends) instead
 * of the fleet's own allocation.  Arguments and results as fleet_decode_step; the results
 * are bit-identical to it.  A step whose working memory exceeds the array (large batches on
 * the MFMA path with split-K partial sums; the Qwen3-8B shape fits up to batch 16) is
 * refused with FLEET_ETOOBIG before anything is launched.  The call itself allocates
 * nothing, frees nothing and copies nothing from the host; counters and status are cleared
 * by a kernel at the start of every call.  All calls on one GPU share the array: calls
 * that overlap on one GPU (two streams, two fleets, two threads) race; calls on one stream
 * are safe.  fleet_last_status reports on the last step launched either way.
 */
#define FLEET_STATIC_SCRATCH_BYTES (32u << 20)
int fleet_decode_step_static(fleet_t *f, int32_t batch, const void *hidden_in, const int32_t *tokens,
                             void *k_cache, void *v_cache, const int32_t *positions,
                             float *hidden_out, float *logits, void *stream);

/*
 * fleet_decode_step_paged: fleet_decode_step over a paged KV cache.
 *   k_pool, v_pool  device bf16 [n_layers][n_pages][n_kv][page_size][head_dim]: a page holds
 *              page_size consecutive slots of one sequence, for every kv head of one layer
 *   page_table device int32 [batch][table_stride]: entry i of a sequence is the page that
 *              holds its slots i*page_size .. (the same page index in every layer)
 *   page_size  a power of two >= 64; positions[b] < table_stride * page_size and < max_seq
 * Everything else as in fleet_decode_step.  A page index outside [0, n_pages) or a position
 * beyond the table ends the step with FLEET_EINVAL in the status; nothing is read or
 * written through such an entry.
 */
int fleet_decode_step_paged(fleet_t *f, int32_t batch, const void *hidden_in, const int32_t *tokens,
                            void *k_pool, void *v_pool, const int32_t *page_table,
                            int32_t page_size, int32_t n_pages, int32_t table_stride,
                            const int32_t *positions, float *hidden_out, float *logits,
                            void *stream);

/*
 * fleet_decode_tokens: n_tokens greedy decode steps in ONE launch of the persistent kernel
 * (paper section 4.1: the kernel stays resident over the generated tokens; no return to the
 * host between steps).  Each step gathers embed[tokens[b]], runs the decoder stack and the LM
 * head as fleet_decode_step does, and a last stage of CU-tasks takes, per sequence, the index
 * of the largest logit (the lowest index among equal ones) as the next token.
 *   tokens     device int32 [batch], in/out: the input token of the first step; on return
 *              the last token generated
 *   positions  device int32 [batch], in/out: advanced by one per step (positions[b] +
 *              n_tokens <= max_seq, else the launch aborts with FLEET_EINVAL in the status)
 *   tokens_out device int32 [n_tokens, batch]: the token chosen in every step
 *   hidden_out device fp32 [batch, hidden], logits device fp32 [batch, vocab]: workspace
 *              and result of the last step
 * Needs embed, final_norm and lm_head.  Asynchronous on `stream`; fleet_last_status
 * reports a time-out or a bad position.  No trace is recorded for such a launch.
 */
int fleet_decode_tokens(fleet_t *f, int32_t batch, int32_t *tokens, void *k_cache, void *v_cache,
                        int32_t *positions, int32_t n_tokens, int32_t *tokens_out,
                        float *hidden_out, float *logits, void *stream);

/*
 * fleet_gemm (test / measurement): y = x . W^T as `reps` back-to-back device-tasks
 * of the persistent kernel, the GEMM of paper section 3.2 in isolation.
 *   x         device bf16 [B, K]
 *   w_copies  HOST array of n_copies device pointers, each bf16 [N, K]; rep i
 *             reads copy i % n_copies (rotating over more than the last-level
 *             cache keeps the timing HBM-bound)
 *   y         device fp32 [B, N]
 *   sched_mode, tile_m  as in fleet_shape_t
 *   elapsed_ms  HOST float or NULL: time of the one kernel launch that runs all
 *             reps, measured with HIP events on `stream`
 * K a multiple of 32, N of 16, N * K * 2 < 2^31, 1 <= B <= 128, 1 <= reps <= 1024.  Synchronous: returns after the
 * kernel has finished (it allocates and frees its own descriptors and, on the MFMA
 * path, packed copies of x and of every weight copy).  Repetitions are independent
 * of each other unless FLEET_FLAG_CHAINED is set; with a split-K plan a repetition
 * waits for the one before the previous (two sets of arrival counters).
 */
int fleet_gemm(int32_t B, int32_t K, int32_t N, const void *x, const void *const *w_copies,
               int32_t n_copies, float *y, int32_t sched_mode, int32_t tile_m, int32_t flags,
               int32_t reps, void *stream, float *elapsed_ms);

/*
 * fleet_graph_build (host only, no device needed): the task graph the library
 * would run for `batch` on a device with n_xcd chiplets, as int32 words:
 *   header[32], ops[n_ops][16], tasks[n_tasks][16], events[n_events][4],
 *   queue offsets[n_xcd + 1], queue entries[n_qent][4], layer marks[n_xcd][n_layers + 4],
 *   residual-ready events[n_layers + 1]
 * (word meanings documented in csrc/graph.hpp).  buf may be NULL to query the size; *len is
 * in/out in bytes.  Paper sections 3.1 (task scopes, events), 3.2 (partitioning,
 * traversal order), 4.3 (per-chiplet partition pointers).
 */
int fleet_graph_build(const fleet_shape_t *shape, int32_t batch, int32_t n_xcd,
                      int32_t n_workers, void *buf, size_t *len);

/* fleet_graph_dump: the same words for the graph `f` runs at `batch`: the graph of the
 * smallest batch bucket that holds `batch` (header word "batch" names the bucket). */
int fleet_graph_dump(fleet_t *f, int32_t batch, void *buf, size_t *len);

/*
 * fleet_trace_read (needs FLEET_FLAG_TRACE or FLEET_FLAG_TIMING): copy the last
 * step's execution records to host memory after synchronising the device.  Each
 * record is 8 int32 words: task, worker (workgroup id), xcd, time the task was
 * entered (before its wait), start ticket, end ticket (0 with FLEET_FLAG_TIMING),
 * start time (after the wait), end time; times in 100 MHz ticks relative to the
 * earliest start in the buffer.
 * Tickets come from one device-wide counter, so "end ticket of a predecessor <
 * start ticket of a successor" checks the dependency order (paper section 3.1).
 */
int fleet_trace_read(fleet_t *f, void *buf, size_t *len);

/* fleet_last_status: synchronise the device and report the last step's outcome. */
int fleet_last_status(fleet_t *f, fleet_status_t *out);

/*
 * fleet_device_probe: XCD id (hardware XCC_ID) of each of n_blocks workgroups of
 * a grid launched the way the persistent kernel is; xcd_of_block is a HOST array
 * of n_blocks int32.  Paper section 4.1 (workers discover their XCD).
 */
int fleet_device_probe(int32_t n_blocks, int32_t *xcd_of_block);

/*
 * fleet_copy (measurement): a plain streaming copy of `bytes` (a multiple of 16) from
 * src to dst, both device memory, on `stream`.  Its HBM traffic is known exactly
 * (bytes read + bytes written), which calibrates the hardware traffic counters the
 * roofline figures are checked against.
 */
int fleet_copy(void *dst, const void *src, size_t bytes, void *stream);

/*
 * Traffic accounting, closed forms (paper section 5.4, Table "weight sizes",
 * Eq. "l2-hit", Figure "roofline"): bytes are for bf16 weights.
 */
int64_t fleet_weight_bytes(int32_t K, int32_t N);                 /* K*N*2                */
int64_t fleet_weight_bytes_per_xcd(int32_t K, int32_t N, int32_t n_xcd);
int64_t fleet_l2_window_bytes(int32_t N, int32_t n_xcd, int32_t tile_n, int32_t tile_k);
double fleet_l2_hit_model(int32_t batch, int32_t tile_m, int32_t workers_per_xcd);
double fleet_effective_intensity(int32_t batch, double l2_hit);
/* algorithmic HBM bytes of one decode step: every weight once + K,V of every
 * attended slot + the new slot; positions is a HOST array of batch int32. */
int64_t fleet_step_bytes(const fleet_shape_t *shape, int32_t batch, const int32_t *positions);

const char *fleet_strerror(int code);

#ifdef __cplusplus
}
#endif
#endif /* FLEET_H */
