/*
 * qsac.h - C ABI of the MI355X (gfx950) QSAC decode step.
 *
 * One call to qsac_step() is one iteration of the loop of Algorithm 1
 * (Section 4 of the LiteCache paper, arXiv 2511.14510) for one attention layer,
 * for every (batch element, KV head) pair at once:
 *
 *   1. cache lookup: CosSim (Section 3.1) between each query head and its cached
 *      query label q_c, aggregated per KV head by Eq. (2) (Section 4.2), compared
 *      with the head's threshold tau; "at or above" reuses;
 *   2. on a miss: exact qkscores (Eq. (1)) of the head's query group against all
 *      N keys, S[n] = max over the group of q_g . k_n; the k best under (score
 *      descending, index ascending); a diff of that set against the tokens held
 *      by the head's cache slots; a fill of the missing rows only, from the K / V
 *      fill sources (HBM or host-mapped pinned memory); q_c <- q_t;
 *   3. softmax(q K_c^T / sqrt(d_k)) V_c over the k cached rows (Section 2.1).
 *
 * Every step runs in hand-written HIP kernels on the caller's streams.  All
 * buffers are caller-owned; the library allocates no device memory, never
 * synchronises inside qsac_step(), and keeps its own state (validity flags,
 * the sorted index set of each head, scratch) in the caller's workspace.
 *
 * Conventions: "e" is a 16-bit float (IEEE binary16 or bfloat16, chosen at
 * init).  P = batch * n_kv_heads pairs, pair p = b * n_kv_heads + h.
 * G = n_q_heads / n_kv_heads; query head g of pair p is b * n_q_heads + h*G + g.
 * D = head_dim = 128.  Tensors are dense, row-major, last index fastest.
 * "device-accessible" means HBM or host memory mapped into the device
 * (hipHostMalloc); every such pointer must be 16-byte aligned.
 *
 * Error behaviour: every function returns 0 (QSAC_OK) or a negative code; no
 * exceptions, no aborts.  Arguments are validated on the host before anything
 * is enqueued, so a call that fails validation (every code but QSAC_EHIP) has no
 * effect on the device or on the context.  QSAC_EHIP from qsac_step() means a HIP
 * call failed after part of the step may have been enqueued: the context then
 * refuses further steps with QSAC_ESTATE until qsac_reset() has invalidated the
 * caches, and its step counter does not count the failed step.
 */
#ifndef QSAC_H
#define QSAC_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum { QSAC_F16 = 0, QSAC_BF16 = 1 };

enum {
  QSAC_OK = 0,
  QSAC_EINVAL = -1,     /* a field has an unsupported value                     */
  QSAC_ENULL = -2,      /* a required pointer is NULL                           */
  QSAC_ERANGE = -3,     /* k, k_max, n_ctx (at most 2^20) or a head count is out of range */
  QSAC_EWORKSPACE = -4, /* workspace missing, misaligned or too small           */
  QSAC_EHIP = -5,       /* a HIP runtime call failed (see qsac_last_hip_error)  */
  QSAC_ESTATE = -6,     /* bad handle, k changed without qsac_reset, or a step failed with QSAC_EHIP */
  QSAC_EALIGN = -7,     /* a tensor pointer is not 16-byte aligned              */
  QSAC_ETIMEOUT = -8    /* push mode: a polling kernel gave up waiting for the host transfer threads */
};

enum {
  QSAC_MAX_GROUP = 8,      /* largest supported G                                */
  QSAC_MAX_KV_HEADS = 64,  /* largest supported n_kv_heads                       */
  QSAC_HEAD_DIM = 128
};

/* qsac_config.flags */
enum {
  QSAC_FLAG_DRY_RUN = 1,     /* validate only: the ctx never touches a device (for hosts without a GPU) */
  QSAC_FLAG_SERIAL = 2,      /* run everything on stream_main even when stream_side is given              */
  QSAC_FLAG_SCORE_VALU = 4,  /* score with packed dot-product ALU ops instead of the MFMA tile           */
  QSAC_FLAG_PROFILE = 8,     /* bracket every stage with timing events (single stream; see qsac_get_stage_ms) */
  QSAC_FLAG_FILL_KERNEL = 16,/* fill the missing rows with a kernel of its own (on stream_side if given, overlapped
                                with the attention of the heads that reused) instead of folding the fetch into the
                                attention kernel's row loads                                              */
  QSAC_FLAG_PUSH_FILL = 32,  /* push-mode transfer, the paper's own scheme (Section 5.2 GPU-centric synchronization,
                                Section 6.2 zero-copy transfer engine) as an alternative to the GPU pulling the rows:
                                the GPU publishes the compacted miss lists and a request flag (Flag1) in pinned host
                                memory, host transfer threads owned by the context copy the rows from the host K / V
                                store straight into the cache slots through the device's host-visible memory window
                                and set a completion flag (Flag2), and a polling kernel holds back the attention of
                                the heads that missed until it sees Flag2.  Both fill sources must then be host
                                memory and no head may be resident (QSAC_EINVAL otherwise).  The polling kernel's
                                wait is bounded (qsac_config.push_wait_us): if the flag does not arrive in time the
                                kernel records the fact and exits, the step's results are invalid, and the next call
                                on the context returns QSAC_ETIMEOUT until qsac_reset                         */
  QSAC_FLAG_PUSH_HOLD = 64,  /* test aid for push mode: the transfer threads ignore every request, so every polling
                                kernel runs into its bound                                                  */
  QSAC_FLAG_STAGGER = 128    /* staggered schedule (needs stream_side, batch >= 2 and batch * n_kv_heads <= 8192;
                                not with SERIAL, PROFILE, FILL_KERNEL or PUSH_FILL): after the gate, the batch runs
                                in a few slices of growing size, pipelined over the two streams: stream_main scores
                                and selects slice i + 1 and then attends to slice i, stream_side copies slice i's
                                missing rows into their slots as soon as its select is through, with a kernel that
                                keeps only as many reads in flight as the link needs.  The slices are independent
                                (Algorithm 1 is per head), so the results are those of the plain schedule up to the
                                summation order of the attention splits; what changes is that a slice is scored
                                (HBM) while the rows of the slice before it are fetched (PCIe, when the fill sources
                                are host memory): the overlap of transfer and computation, by a transfer engine of
                                its own, that Sections 5.2 and 6.2 of the paper are after.  The step still completes on
                                stream_main                                                                   */
};

typedef struct qsac_ctx qsac_ctx;

typedef struct {
  int32_t batch, n_q_heads, n_kv_heads, head_dim; /* head_dim must be 128; n_q_heads % n_kv_heads == 0 */
  int64_t n_ctx;                /* N, fixed for the life of the ctx; 1 <= N <= 2^20                      */
  int32_t k_max;                /* slot stride of the cache tensors; 1 <= k <= k_max <= N                */
  int32_t dtype;                /* QSAC_F16 | QSAC_BF16: type of q, K, V, prev_q and the slots           */
  const float *q_head_importance; /* HOST, [n_q_heads] weights s_j of Eq. (2), all > 0; NULL = all 1     */
  void *stream_main;            /* hipStream_t (NULL = default stream); borrowed                          */
  void *stream_side;            /* second hipStream_t or NULL; borrowed.  Given one, the attention of the heads that
                                   reused runs on it beside the select (with QSAC_FLAG_FILL_KERNEL: the fill kernel
                                   runs on it beside that attention).  The step still completes on stream_main. */
  void *workspace;              /* DEVICE, 256-byte aligned, >= qsac_workspace_bytes(); caller-owned       */
  size_t workspace_bytes;
  int32_t flags;
  /* Sink and recent tokens (Section 7.1: kept in the cache persistently): the first n_sink and the last
     n_recent of the N context tokens rank above every score, so every retrieved set contains them
     (k >= n_sink + n_recent).  0 = none. */
  int32_t n_sink, n_recent;
  /* Rows per KV head of the append-only buffer (Sections 6.1, 6.2), 0 = none; see qsac_step_args.K_app. */
  int32_t append_capacity;
  /* Push mode (QSAC_FLAG_PUSH_FILL) only: host transfer threads (0 = 4; at most 64) and the longest a polling
     kernel waits for them, in microseconds (0 = 2 000 000). */
  int32_t push_threads, push_wait_us;
} qsac_config;

/* Byte offsets of the library's arrays inside the workspace (for tests and tools that inspect them). */
typedef struct {
  size_t valid;      /* u32 [P]              1 once the head's cache has been filled                      */
  size_t set_sorted; /* i32 [P][k_max]       the head's cached index set, ascending                       */
  size_t keys;       /* u32 [P][n_pad]       order-preserving image of the fp32 scores of the last miss   */
  size_t hist;       /* u32 [P][3][2048]     radix histograms of the last miss                            */
  size_t bm_new;     /* u32 [P][words]       bitmap of the selected set                                   */
  size_t bm_eq;      /* u32 [P][words]       bitmap of keys equal to the k-th key                         */
  size_t bm_old;     /* u32 [P][words]       bitmap of the tokens cached before the step                  */
  size_t miss_count; /* i32 [P]              rows filled by the last step (0 on reuse)                    */
  size_t miss_slot;  /* i32 [P][k_max]       slots refilled, ascending                                    */
  size_t miss_tok;   /* i32 [P][k_max]       tokens fetched, ascending; pairs with miss_slot              */
  size_t part_ml;    /* f32 [P][G][splits][2]   running max (log2 domain) and sum of each attention split */
  size_t part_acc;   /* f32 [P][G][splits][128] unnormalised partial outputs                              */
  size_t stats;      /* u64 [8]              cumulative counters                                          */
  size_t importance; /* f64 [n_q_heads]      Eq. (2) weights                                              */
  size_t sel_r;      /* i32 [P][8]           per pair: keys equal to the k-th key that belong to the set, then the
                                             threshold bins found so far by the grid-wide select (last miss)      */
  size_t chunk_cnt;  /* i32 [P][n_pad/8192][2] set bits per 8192-key chunk of bm_new and bm_eq (long contexts)    */
  size_t fetch_tok;  /* i32 [P][k_max]       per slot: token whose rows the slot still has to receive, or -1      */
  size_t push;       /* u32 [4]              push mode: request sequence number, pairs published so far, polls
                                             that gave up                                                         */
  size_t total;      /* bytes needed                                                                      */
  int64_t n_pad;     /* N rounded up to the select chunk                                                  */
  int32_t words;     /* 32-bit words per bitmap                                                           */
  int32_t max_splits;/* attention splits provisioned per pair                                             */
} qsac_ws_layout;

/*
 * Per-step scalars kept in DEVICE memory, for a step that is captured once into a graph and replayed
 * (qsac_graph_capture): a replay cannot take new host values, so the kernels read these at run time and the
 * caller rewrites the block between replays (ordered on stream_main, e.g. by a small asynchronous copy).
 */
typedef struct {
  float tau[QSAC_MAX_KV_HEADS]; /* thresholds tau_i, one per KV head (entries past n_kv_heads are ignored)   */
  int32_t n_app;                /* valid rows of the append-only buffer; clamped to [0, qsac_step_args.n_app] */
  int32_t reserved[3];
} qsac_dev_params;

/*
 * Arguments of one step.  Everything is caller-owned and stays valid until
 * stream_main has run past the step.
 */
typedef struct {
  const void *q;        /* DEVICE e [B,Hq,D]        current queries q_t                                      */
  const void *K_dev;    /* DEVICE e [B,Hkv,N,D]     full K in HBM, read by the scoring pass                  */
  const void *K_src;    /* device-accessible e [B,Hkv,N,D]  fill source of K rows (may equal K_dev)          */
  const void *V_src;    /* device-accessible e [B,Hkv,N,D]  fill source of V rows                            */
  void *K_slots;        /* DEVICE e [B,Hkv,k_max,D] in/out  Replaceable Cache, K half (Section 3.3)          */
  void *V_slots;        /* DEVICE e [B,Hkv,k_max,D] in/out  Replaceable Cache, V half                        */
  int32_t *slot_idx;    /* DEVICE [B,Hkv,k_max]     in/out  token held by each slot                          */
  void *prev_q;         /* DEVICE e [B,Hq,D]        in/out  query label q_c; rewritten only on a miss         */
  const float *tau;     /* HOST [n_tau]             thresholds tau_i; n_tau is 1 (all heads) or n_kv_heads    */
  int32_t n_tau;
  int32_t k;            /* slots in use; constant between resets                                            */
  float *out;           /* DEVICE f32 [B,Hq,D]      attention output                                         */
  int32_t *topk_idx;    /* DEVICE [B,Hkv,k]         tokens in the head's cache after the step, ascending      */
  uint8_t *hit_mask;    /* DEVICE [B,Hkv,k]         1 where topk_idx[j] was cached before the step           */
  uint8_t *reuse_flags; /* DEVICE [B,Hkv]           1 where the gate reused the cached set                   */
  float *sim;           /* DEVICE f32 [B,Hq] or NULL  per-query-head CosSim                                   */
  /* Resident caching (Section 4.4): KV heads that are hard to reuse keep their full KV in HBM, so their
     misses never cross PCIe.  A head h with res_slot[h] >= 0 takes the K rows of its missing tokens from
     K_dev and the V rows from V_res[:, res_slot[h]]; the others use K_src / V_src.  Results do not depend
     on which heads are resident.  NULL res_slot = no resident heads. */
  const void *V_res;         /* DEVICE e [B,n_res,N,D] or NULL  full V of the resident KV heads          */
  const int8_t *res_slot;    /* HOST [n_kv_heads] or NULL       index in V_res, -1 = not resident         */
  int32_t n_res;             /* resident KV heads, 1 <= n_res <= n_kv_heads when res_slot is given       */
  /* Append-only buffer (Sections 6.1, 6.2): KV of the tokens generated during decoding, appended by the
     caller before the step.  The hybrid attention reads its n_app valid rows in place next to the k cached
     rows; they are not scored, selected or cached.  n_app = 0 = none. */
  const void *K_app;         /* DEVICE e [B,Hkv,append_capacity,D]                                        */
  const void *V_app;         /* DEVICE e [B,Hkv,append_capacity,D]                                        */
  int32_t n_app;             /* valid rows, 0 <= n_app <= append_capacity                                 */
  /* NULL, or per-step scalars in device memory.  Given one, the kernels take tau_i and the number of valid
     append-buffer rows from it when they run (tau / n_tau above are then ignored and may be NULL), and n_app
     above is the largest value the block will ever hold: it sizes the launch. */
  const qsac_dev_params *dev_params; /* DEVICE, 16-byte aligned */
} qsac_step_args;

/* Cumulative since init / reset, summed over pairs. */
typedef struct {
  uint64_t steps;        /* calls to qsac_step                          */
  uint64_t reuse_heads;  /* pairs that took the reuse branch            */
  uint64_t miss_heads;   /* pairs that took the miss branch             */
  uint64_t slot_hits;    /* rows of a fresh top-k that were cached      */
  uint64_t slot_misses;  /* rows filled from the fill sources (one row = a K row and a V row)     */
  uint64_t bytes_filled_host; /* bytes of those rows that came from host memory (over PCIe)        */
  uint64_t bytes_filled_dev;  /* bytes of those rows that came from HBM; host + dev = 512 * slot_misses */
  uint64_t resident_rows;/* of slot_misses, rows of resident heads (always from HBM)              */
  uint64_t guided_selects;/* misses whose top-k was taken from the candidates above a sampled bound */
  uint64_t reserved[1];
} qsac_stats;

/* Workspace size for a configuration (pure host function; 0 if the configuration is invalid). */
size_t qsac_workspace_bytes(const qsac_config *cfg);

/* Layout of the workspace (pure host function). */
int qsac_workspace_layout(const qsac_config *cfg, qsac_ws_layout *out);

/*
 * Creates a context and marks every head's cache invalid, so the first step of every
 * head is a miss that fills all k slots whatever tau is (Algorithm 1, line 1, assumes a
 * cache filled at step 0; this is that step).  Enqueues a clear of the workspace
 * bookkeeping on stream_main.  The ctx itself is host memory owned by the library.
 */
int qsac_init(const qsac_config *cfg, qsac_ctx **out);

/* Marks every head's cache invalid again and zeroes the counters (enqueued on stream_main). */
int qsac_reset(qsac_ctx *ctx);

/*
 * Enqueues one step (Algorithm 1, lines 3-18).  Results are valid once stream_main has run
 * past it.  The slot contents, slot_idx and prev_q need no initialisation before the first
 * step.  Inputs must be finite.
 */
int qsac_step(qsac_ctx *ctx, const qsac_step_args *args);

/* Synchronises stream_main and copies the counters to host_out. */
int qsac_get_stats(qsac_ctx *ctx, qsac_stats *host_out);

/* Releases the ctx (host memory and the two events it owns).  Does not touch caller buffers. */
int qsac_free(qsac_ctx *ctx);

const char *qsac_strerror(int code);

/*
 * One step as a replayable graph.  The paper runs the decode step from a captured graph because kernel
 * launches otherwise dominate short steps (Section 2.3), which is possible only while the step's launch
 * topology is static and no host decision sits inside it (Section 5.2, last paragraph): both hold here, the
 * gate's outcome is consumed on the device.  qsac_graph_capture() records the launches of one qsac_step(ctx,
 * args) on stream_main into a graph without running them; args->dev_params is required, since tau and the
 * append-buffer row count of a replay come from device memory.  Every pointer in args (q included: the caller
 * copies each new query into that buffer) and args->k are bound into the graph.  qsac_graph_launch() enqueues
 * one replay on stream_main and counts as one step; replays and plain qsac_step() calls on the same ctx may be
 * mixed.  Not available for contexts created with QSAC_FLAG_PROFILE or QSAC_FLAG_DRY_RUN (QSAC_ESTATE).
 * qsac_graph_free() releases the graph; the ctx must outlive it.
 */
typedef struct qsac_graph qsac_graph;
int qsac_graph_capture(qsac_ctx *ctx, const qsac_step_args *args, qsac_graph **out);
int qsac_graph_launch(qsac_graph *graph);
int qsac_graph_free(qsac_graph *graph);

/* hipError_t of the last failing HIP call on this thread (0 if none). */
int qsac_last_hip_error(void);

/*
 * qsac_step() for callers that cannot allocate device memory (code under graph capture, serving loops and
 * harnesses in which hipMalloc is forbidden) and therefore cannot bring a workspace: the library's state and
 * scratch of ONE layer live in a QSAC_STATIC_SCRATCH_BYTES array inside the library's device image, of which
 * every GPU the library runs on holds a copy until the process ends.  The call allocates nothing on the
 * device or the host, creates no events and copies nothing synchronously.
 *   cfg    as for qsac_init(); workspace / workspace_bytes are ignored, stream_side must be NULL, flags may
 *          hold QSAC_FLAG_SCORE_VALU and QSAC_FLAG_FILL_KERNEL only.  QSAC_EWORKSPACE if
 *          qsac_workspace_bytes(cfg) exceeds QSAC_STATIC_SCRATCH_BYTES.
 *   args   as for qsac_step(); inputs and outputs stay caller-owned.
 *   reset  non-zero: first mark every head's cache invalid and zero the counters (as qsac_init / qsac_reset
 *          do).  Required on the first call on a GPU and whenever cfg differs from the previous call's
 *          (QSAC_ESTATE otherwise); the array keeps the previous call's contents.
 * The array is per GPU (the current device of the calling thread), and every call on that GPU shares it:
 * calls that overlap on one GPU, from several threads or streams, race.
 */
enum { QSAC_STATIC_SCRATCH_BYTES = 32 << 20 };
int qsac_step_static(const qsac_config *cfg, const qsac_step_args *args, int reset);

/*
 * Stage timing, for contexts created with QSAC_FLAG_PROFILE.  The stages of a step, in launch
 * order, are: 0 "gate" (qsac_gate_kernel), 1 "score" (qsac_score_mfma_kernel or
 * qsac_score_valu_kernel), 2 "select" (qsac_select_small_kernel for N <= 65536, else
 * qsac_refine_kernel<1>, <2>, qsac_mark_kernel, qsac_diff_kernel), 3 "fill" (qsac_fill_kernel),
 * 4 "attn" (qsac_attn_kernel), 5 "combine" (qsac_combine_kernel).  qsac_get_stage_ms() waits for the last profiled step and writes
 * the summed duration of each stage in milliseconds to ms_sum[qsac_num_stages()] and the number
 * of steps summed to *n_steps.  A duration is the time between the events recorded on
 * stream_main before the stage's first kernel and before the next stage's.  qsac_stage_name(i)
 * is the stage's label, NULL past the end.
 */
int qsac_num_stages(void);
const char *qsac_stage_name(int i);
int qsac_get_stage_ms(qsac_ctx *ctx, double *ms_sum, uint64_t *n_steps);

/*
 * Adaptive per-head thresholds, Section 4.3, Eq. (3)-(5) (pure host function, fp64 inside):
 *   theta* = arccos(eta);  theta_i = lambda_i theta* + (1 - lambda_i) pi;  tau_i = cos(theta_i);  lambda_i = s_i^p
 * importance[n] are head importance scores s_i in [0, 1] (one per KV head when the result feeds
 * qsac_step_args.tau), eta in [-1, 1] the upper bound of the thresholds, p > 0 (the paper uses eta = 0.8,
 * p = 3).  tau_out[n] receives the thresholds.  QSAC_EINVAL for values outside those ranges.
 */
int qsac_adaptive_thresholds(const float *importance, int32_t n, float eta, float p, float *tau_out);

/*
 * Reuse difficulty of Section 4.4 (pure host function): D_i = tau_i - (avg_sim_i - eps), where avg_sim_i is
 * the head's profiled average cosine similarity of adjacent queries and eps > 0 a tolerance margin.  The
 * heads with the largest D_i are the candidates for resident caching.
 */
int qsac_reuse_difficulty(const float *tau, const float *avg_sim, int32_t n, float eps, float *d_out);

#ifdef __cplusplus
}
#endif
#endif /* QSAC_H */
