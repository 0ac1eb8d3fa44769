/*
 * mk.h -- C ABI of the MI355X decode-step megakernel library (libmk.so).
 *
 * The library runs one batch-1..16 LLM decode step (RMSNorm -> QKV projection
 * + RoPE -> GQA attention over the KV cache -> O projection + residual ->
 * SwiGLU MLP -> final norm + LM head) as ONE persistent kernel launch whose
 * execution order is fixed offline.  This mirrors the two phases of the paper
 * (Sec. 3): Phase I, offline synthesis -- the decoder and LM head are parsed
 * into a dependency DAG, candidates are pruned by the on-chip memory budget
 * (Sec. 4.1.1, Eq. 1-2), simulated, and the chosen trace is serialised
 * (Sec. 4.2.2, Steps 1-4); Phase II, online execution of the serialised trace
 * with no run-time scheduling decisions (Sec. 4.2.2, "execution-path
 * solidification").  The host engine keeps owning KV-cache allocation
 * (Sec. 4.3.1); the library owns the decode step, and can fill the cache from
 * a prompt with that same step (mk_fill_cache), not with a prefill of its own.
 *
 * Conventions
 *   - Every function returns 0 (MK_OK) or a negative MK_E* code; no C++
 *     exception crosses the boundary.  mk_last_error() returns a thread-local
 *     text for the last failure on the calling thread.
 *   - "dev" pointers are device (HBM) addresses on the device the schedule was
 *     bound to; "host" pointers are ordinary host memory.  Streams are passed
 *     as void* (a hipStream_t; NULL = the default stream).
 *   - A schedule handle is not thread-safe; decode steps on one handle must be
 *     stream-ordered.
 *   - bf16 means the upper 16 bits of an IEEE fp32, round-to-nearest-even.
 */
#ifndef MK_H_
#define MK_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    MK_OK = 0,
    MK_EINVAL = -1,      /* bad config, shape or argument                           */
    MK_ENOMEM = -2,      /* workspace too small / host allocation failed             */
    MK_EINFEASIBLE = -3, /* no candidate fits the LDS budget (Eq. 1-2)               */
    MK_ESCHED = -4,      /* the schedule failed verification                         */
    MK_EHIP = -5,        /* a HIP runtime call failed                                */
    MK_ETIMEOUT = -6,    /* a dependency wait inside the kernel hit its spin limit   */
    MK_ESTATE = -7       /* call order violated (e.g. decode before load_weights)    */
};

/* Fixed deployment configuration (paper abstract / Sec. 3: under a fixed
 * configuration the execution path is determined offline).  Model dimensions
 * follow the public Qwen2 / Qwen3 decoder family. */
typedef struct mk_config {
    int32_t n_layers, hidden, n_q_heads, n_kv_heads, head_dim, intermediate, vocab;
    int32_t qkv_bias;        /* 1: Q/K/V projections carry a bias                    */
    int32_t qk_norm;         /* 1: per-head RMSNorm on q and k before RoPE           */
    int32_t tie_embeddings;  /* 1: LM head shares the embedding matrix               */
    float rope_theta, rms_eps;
    int32_t max_batch;       /* 1..16                                                */
    int32_t max_context;     /* KV slots per sequence                                */
    int32_t n_workgroups;    /* persistent grid size; 0 = one per CU of device_id    */
    int32_t device_id;       /* only read when n_workgroups == 0 or at bind time     */
    int32_t use_mfma;        /* -1 auto (batch>1 -> MFMA), 0 VALU GEMV, 1 MFMA GEMV  */
    int32_t ring_kb;         /* LDS weight-page ring in KB (16..144, rounded down to 16): each wavefront streams its
                              * share of the workgroup's weights through its quarter of the ring, ahead of the
                              * consumer and across task boundaries; 0 = no ring (weights go straight to registers);
                              * -1 = auto (currently 0: the direct path measures faster); -2 = let the search pick   */
    int32_t split_qkv, split_o, split_gateup, split_down; /* K splits; 0 = search    */
    int32_t attn_chunks;     /* attention tasks per (sequence, KV head); 0 = search  */
    int32_t chunk_rows;      /* rows per 1 KB weight chunk for every matrix (2,4,8,16); 0 = search per matrix */
    int32_t rows_qkv, rows_o, rows_gateup, rows_down, rows_head; /* the same per matrix (overrides chunk_rows);
                              * 0 = chunk_rows / search (the LM head defaults to 16)                              */
    int32_t fuse_combine;    /* 1: no separate combine tasks -- every O-projection task combines the attention partials of
                              * the heads its K range covers in its own prologue (one dependency level less per layer);
                              * 0: combine tasks; -1: auto (currently 0)                                          */
    int32_t weight_bits;     /* 16 (or 0): bf16 matrices.  4: the seven decoder projections are W4A16 (Sec. 4.3.2):
                              * unsigned 4-bit codes q, two per byte along K (even k in the low nibble), and one bf16
                              * scale s per (row, group_size consecutive k): w = (q - 8) * s.  Embedding and LM head
                              * stay bf16.  max_batch 1: VALU form (codes dequantised in registers) unless use_mfma = 1;
                              * max_batch 2..8: matrix-core form (codes expanded to bf16 in registers, 16 rows per chunk).
                              * No page ring with W4.                                                              */
    int32_t group_size;      /* W4: 32, 64 or 128 (0 = 128); must divide hidden, n_q_heads*head_dim, intermediate  */
    uint32_t spin_limit;     /* dependency-wait poll limit; 0 = library default      */
    uint32_t flags;          /* MK_F_*                                               */
} mk_config;

enum {
    MK_F_TRACE = 1u,         /* record per-task clocks into the trace buffer          */
    MK_F_TIMING = 2u,        /* bracket each step's launch(es) with HIP events         */
    MK_F_NO_TABLE = 4u       /* mk_build_schedule: ignore the table of recorded profile-guided tilings */
};

typedef struct mk_schedule mk_schedule; /* opaque, library-owned host object */

/* Caller-owned DEVICE pointers, bf16, row-major [out][in].  Per-layer members
 * are HOST arrays of n_layers device pointers.  Bias / qk-norm arrays may be
 * NULL when the matching flag is 0; lm_head may be NULL when tied. */
typedef struct mk_weights {
    const void *embed;      /* [vocab][hidden]  */
    const void *lm_head;    /* [vocab][hidden]  */
    const void *final_norm; /* [hidden]         */
    const void *const *attn_norm, *const *wq, *const *wk, *const *wv;
    const void *const *bq, *const *bk, *const *bv, *const *q_norm, *const *k_norm;
    const void *const *wo, *const *mlp_norm, *const *w_gate, *const *w_up, *const *w_down;
    /* weight_bits == 4 only: bf16 scales [out][in / group_size] of the seven projections; the matrix
     * pointers above then address packed codes, uint8 [out][in / 2].  Ignored (may be NULL) otherwise. */
    const void *const *sq, *const *sk, *const *sv, *const *so, *const *s_gate, *const *s_up, *const *s_down;
} mk_weights;

typedef struct mk_stats {
    int32_t n_workgroups, threads_per_wg, n_tasks, n_counters, max_instr_per_wg;
    int32_t split_qkv, split_o, split_gateup, split_down, attn_chunks, use_mfma;
    int32_t lds_bytes, ring_pages, page_bytes, n_stage;  /* Eq. 1-2 outcome            */
    int64_t weight_bytes_per_step;   /* repacked weight bytes streamed by one step     */
    int64_t workspace_bytes;
    double sim_makespan_us;          /* cost-model prediction for one step             */
    double sim_duty_cycle;           /* sum of busy time / (workgroups * makespan)     */
    int32_t candidates_tried, candidates_pruned;
    int32_t rows_qkv, rows_o, rows_gateup, rows_down, rows_head;  /* rows per 1 KB weight chunk, per matrix */
    int32_t fuse_combine;
    int32_t from_table;              /* 1: the tiling is the profiled one recorded for this configuration */
    int32_t attention_mfma;          /* 1: the attention tasks run on the matrix cores */
} mk_stats;

/* Phase I (host only, touches no GPU unless n_workgroups == 0): build the
 * tile-task DAG of the decoder + LM head (Sec. 4.2.1 / Step 1-2), prune and
 * search the tiling space with the page-budget model and the pipeline
 * simulator (Step 3-4), verify, and emit the static per-workgroup instruction
 * lists.  *out is set only on success.
 *
 * Step 4 of the paper locks in the trace that offline PROFILING on the target
 * GPU scores best.  The profiling search (autotune.py, driving this same ABI on
 * the device) records its winner per deployment configuration in the text table
 * tuned_tilings.txt next to the library (another path: environment variable
 * MK_TUNED_TABLE, read here only).  When cfg fixes no tiling field (all split_*,
 * attn_chunks, chunk_rows, rows_* zero, fuse_combine <= 0, ring_kb <= 0, use_mfma
 * -1) and the table holds a line for (model dimensions, max_batch, n_workgroups,
 * weight_bits), that tiling is used (mk_stats.from_table = 1); otherwise, or with
 * MK_F_NO_TABLE, the cost model's own pick. */
int mk_build_schedule(const mk_config *cfg, mk_schedule **out);

/* Structural check of an emitted schedule against its DAG: every tile of every
 * operator appears exactly once; every counter's wait target equals its number
 * of signalling tasks; replaying the per-workgroup lists with blocking waits
 * terminates; every read-after-write, write-after-read and write-after-write
 * pair found by walking the tasks in topological (operator) order with a
 * last-writers table (Sec. 4.2.2 Step 2) is ordered by the emitted
 * waits/signals.  Returns MK_OK or MK_ESCHED (text in mk_last_error). */
int mk_schedule_verify(const mk_schedule *s);

/* Serialise / restore a schedule (the hand-over from offline synthesis to
 * online execution, Sec. 3).  dump: if buf is NULL only *bytes is written. */
int mk_schedule_dump(const mk_schedule *s, void *host_buf, size_t *bytes);
int mk_schedule_load(const void *host_buf, size_t bytes, mk_schedule **out);

int mk_get_stats(const mk_schedule *s, mk_stats *out);
int mk_get_config(const mk_schedule *s, mk_config *out);

/* Test / inspection hooks on the instruction lists (32 dwords per instruction). */
int mk_instr_count(const mk_schedule *s, int32_t wg);
int mk_instr_get(const mk_schedule *s, int32_t wg, int32_t idx, uint32_t *out32);
int mk_instr_set(mk_schedule *s, int32_t wg, int32_t idx, const uint32_t *in32);

/* Eq. 1 and Eq. 2 of Sec. 4.1.1 (integer floors). */
int64_t mk_pages_available(int64_t smem_max, int64_t n_stage, int64_t instr_buf, int64_t semaphores,
                           int64_t scratch, int64_t page_size);
int64_t mk_pipeline_stages(int64_t pages_total, int64_t pages_weight, int64_t pages_scale,
                           int64_t pages_act, int64_t pages_per_stage);

/* Device memory the caller must provide (repacked weights, activation and
 * partial-sum scratch, counters, instruction lists, RoPE table, trace). */
size_t mk_workspace_bytes(const mk_schedule *s);

/* Hand the library its workspace (dev pointer, 256-byte aligned, caller-owned,
 * must outlive the handle's use).  Uploads the instruction lists and the RoPE
 * table and zeroes the counters on `stream`.  Checks that the bound device
 * can keep n_workgroups workgroups co-resident for every kernel the handle may launch. */
int mk_bind_workspace(mk_schedule *s, void *dev_workspace, size_t bytes, void *stream);

/* Offline weight reorder (cf. Sec. 4.3.2 "weight reorder"): copy every matrix
 * into the workspace in the tile-major order the kernel streams (1 KB chunks of
 * R rows x 512/R consecutive k of bf16 -- 2048/R of 4-bit codes -- lane-major; R
 * is chosen per matrix by the schedule search; W4 scales go to a parallel array).  Asynchronous on `stream`; the caller's
 * buffers may be freed once the stream has been synchronised. */
int mk_load_weights(mk_schedule *s, const mk_weights *w, void *stream);

/* One decode step as ONE persistent kernel launch, asynchronous on `stream`.
 * For each sequence b < batch: embeds token_ids[b], appends its K/V at slot
 * positions[b] of kv_cache, attends over slots 0..positions[b], writes
 * logits_out[b][vocab] (fp32).
 *   token_ids, positions : dev int32 [batch]; 0 <= id < vocab, 0 <= pos < max_context
 *     (the kernel clamps out-of-range values and raises the error flag)
 *   kv_cache  : dev bf16 [n_layers][2][max_batch][n_kv_heads][max_context][head_dim]
 *   logits_out: dev fp32 [batch][vocab] */
int mk_decode_step(mk_schedule *s, const int32_t *token_ids, const int32_t *positions,
                   void *kv_cache, float *logits_out, int32_t batch, void *stream);

/* n_steps greedy decode steps as ONE persistent kernel launch (the kernel stays resident and walks
 * its instruction lists once per step; nothing returns to the host in between).  Step 0 decodes
 * token_ids at positions; step s > 0 decodes the arg-max token of step s-1 (first maximum, i.e. the
 * smallest row among equal logits) at positions + s.  Steps are ordered on the device by the
 * dependency counter of the arg-max tasks that close every step.
 *   tokens_out : dev int32 [n_steps][batch], the greedy token chosen by every step
 *   logits_out : dev fp32 [batch][vocab], holds the LAST step's logits when the launch ends
 *   positions[b] + n_steps - 1 must stay below max_context (otherwise clamped, error flag raised)
 * Other arguments as for mk_decode_step. */
int mk_decode_steps(mk_schedule *s, const int32_t *token_ids, const int32_t *positions, void *kv_cache,
                    float *logits_out, int32_t *tokens_out, int32_t batch, int32_t n_steps, void *stream);

/* Fills the cache from known tokens (a prompt) with the decode path itself: n_tokens decode steps as ONE persistent
 * launch, step s decoding token_ids[s][b] at positions[b] + s for every sequence b < batch, with no token feedback, no
 * LM head and no logits (the LM-head tasks only keep their place in the dependency chain).  Token by token this is
 * mathematically the batched causal prefill; it is NOT a GEMM prefill: every step streams the decoder weights once
 * (the paper leaves prefill to the host engine, Sec. 4.3; this call makes the library able to fill its own cache).
 *   token_ids : dev int32 [n_tokens][batch]
 *   positions : dev int32 [batch], position of the FIRST token of every sequence; positions[b] + n_tokens - 1 must
 *               stay below max_context (otherwise clamped, error flag raised)
 * Appends rows positions[b] .. positions[b] + n_tokens - 1 of K and V; asynchronous on `stream`. */
int mk_fill_cache(mk_schedule *s, const int32_t *token_ids, const int32_t *positions, void *kv_cache, int32_t batch,
                  int32_t n_tokens, void *stream);

/* Baseline with the same device task bodies and the same instruction lists,
 * but one kernel launch per DAG operator (stream order supplies the
 * dependencies).  Same arguments and results (bit-identical) as
 * mk_decode_step. */
int mk_decode_step_per_op(mk_schedule *s, const int32_t *token_ids, const int32_t *positions,
                          void *kv_cache, float *logits_out, int32_t batch, void *stream);

/* mk_decode_step for callers that cannot allocate device memory or let a library do so (code under
 * HIP graph capture, tight serving loops, harnesses that forbid it): the same single launch with the
 * same arguments and results, but the step's scratch (activations, partial sums, dependency counters,
 * error flags) lives in a device array built into the library, 16 MiB per GPU, held until the process
 * ends, instead of in the bound workspace.  The call makes no allocation of any kind; weights,
 * instruction lists and the RoPE table are still read from the workspace bound earlier.
 *   - MK_ENOMEM if the schedule's scratch (mk_get_stats: activations + counters) exceeds 16 MiB
 *     (every workload of the benchmark fits; the largest, the 1.7B shape at batch 16, needs 11.8 MB).
 *   - Every call on a GPU shares that GPU's one array: calls that overlap in time on the same GPU (two
 *     streams, two handles) race.  When the handle changes between calls the counters are re-zeroed on
 *     `stream` first.
 *   - The step number the dependency counters are compared with lives in the array too, and a one-workgroup
 *     kernel ahead of the step advances it: a call recorded into a HIP graph replays correctly (the recorded
 *     work is kernels only; tokens, positions and the cache are read through the pointers given at capture).
 *     mk_decode_step and mk_decode_steps pass that number as a kernel argument instead: a recorded call of
 *     theirs must not be replayed.
 *   - mk_check after such a step reports the flags of the static array. */
int mk_decode_step_static(mk_schedule *s, const int32_t *token_ids, const int32_t *positions,
                          void *kv_cache, float *logits_out, int32_t batch, void *stream);

/* Synchronises `stream` and reports the kernel's sticky error flag:
 * MK_OK, MK_ETIMEOUT (a wait hit spin_limit), MK_EINVAL (bad token/position) or
 * MK_ESCHED (the weight-page ring ran dry, i.e. corrupted instruction lists).
 * Clears the flag and re-arms the counters when an error was found. */
int mk_check(mk_schedule *s, void *stream);

/* Duration in milliseconds of the kernels launched by the most recent
 * mk_decode_step / mk_decode_step_per_op on this handle, measured with HIP
 * events recorded on the launch stream around the launch(es).  Synchronises
 * on the closing event. */
int mk_last_step_ms(mk_schedule *s, float *ms);

/* Streaming-read ceiling of the bound device, for the roofline report: a persistent grid of n_workgroups
 * workgroups reads the schedule's own repacked weight region (*bytes of it, a whole number of 1 KB chunks per
 * workgroup) with the load form of the weight stream (128-bit nontemporal loads, 16 in flight per lane) and
 * does nothing else; `reps` timed launches bracketed by HIP events on `stream`, after one untimed launch.
 * ms_out[reps] receives the durations.  Needs a bound workspace (the weights need not be loaded: the
 * kernel never looks at what it reads).  Synchronises `stream`. */
int mk_read_ceiling(mk_schedule *s, int32_t reps, float *ms_out, size_t *bytes, void *stream);

/* Change the run-time flags of a handle (only MK_F_TIMING may be toggled after
 * the schedule was built; MK_F_TRACE is fixed at build time because it sizes
 * the workspace). */
int mk_set_flags(mk_schedule *s, uint32_t flags);

/* Copy the per-task trace (MK_F_TRACE) to host: records of 8 x uint64, one per
 * (workgroup, instruction): {t_begin, t_dependencies_met, t_prologue_done, t_end, 4 task-internal marks}
 * in device wall-clock ticks (100 MHz).
 * *n_records in: capacity, out: records written. */
int mk_read_trace(mk_schedule *s, uint64_t *host_out, size_t *n_records, void *stream);

void mk_destroy(mk_schedule *s);
const char *mk_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* MK_H_ */
