/*
 * ps.h -- C ABI of the MI355X (gfx950) engine-step library.
 *
 * What is computed: one attention layer over the mixed batch that the SlideBatching local
 * scheduler forms each iteration (Alg. 1: prefill chunks of l_q tokens over a cached prefix
 * plus single-token decode requests of several priority classes), read through per-request
 * block lists from a paged KV cache, and the KV-block copies behind asynchronous offload and
 * budgeted, pipelined reload (Sec. 4.3; stream/event structure of Appendix B).
 *
 * Conventions for every function
 *   - returns PS_OK (0) or a negative ps_status; never throws, never aborts.
 *   - never blocks the host on the GPU unless its name says "wait" (exception: a call may
 *     wait for one of the library's own small staging buffers to become reusable).
 *   - ps_last_error() gives a thread-local text for the last failure on this thread.
 *   - pointers marked HOST are ordinary host memory, borrowed only for the duration of the
 *     call; DEVICE pointers are HIP device memory owned by the caller; PINNED pointers are
 *     page-locked host memory (hipHostMalloc) that the GPU can address directly.
 *   - bf16 values are 16-bit patterns (upper half of an IEEE binary32).
 *
 * KV cache layout (device, bf16), chosen so that both attention contractions read their
 * operands as contiguous 16-byte runs:
 *     cache[b][0][g][x/8][t][x%8]  K of block b, kv-head g, token slot t (0..15), dim x
 *                                  (groups of 8 dims; inside a group token-major)
 *     cache[b][1][g][x][t]         V of block b, kv-head g, dim x, token slot t   (dim-major)
 *   i.e. element offsets, with blk = block_tokens and d = head_dim:
 *     K: ((((b*2 + 0)*Hkv + g)*(d/8) + x/8)*blk + t)*8 + x%8
 *     V: (((b*2 + 1)*Hkv + g)*d + x)*blk + t
 *   One block is one contiguous run of 2*Hkv*blk*d*2 bytes (64 KiB at Hkv = 8); a swap moves
 *   whole runs, so the host copy of a block has the same internal layout.
 *   Token j of a request lives in block  block_ids[bt_start[r] + j / blk], slot j % blk.
 *   Slots past kv_len and blocks no table references may hold anything (NaN included); they
 *   never influence an output.
 */
#ifndef PS_H_
#define PS_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  PS_OK = 0,
  PS_EINVAL = -1, /* bad argument / inconsistent batch description            */
  PS_ENOMEM = -2, /* workspace too small, or a host allocation failed         */
  PS_EHIP = -3,   /* a HIP call failed; ps_last_error() holds its text        */
  PS_ESTATE = -4, /* unknown ticket; ps_step_next_layer without a batch to reuse */
  PS_EBUSY = -5   /* ticket still in flight (ps_ticket_query only)             */
} ps_status;

enum { PS_BF16 = 0, PS_F32 = 1 };

typedef struct ps_ctx ps_ctx;

/* Fixed per layer. */
typedef struct {
  int32_t n_q_heads;       /* Hq                                                          */
  int32_t n_kv_heads;      /* Hkv; Hq % Hkv == 0, group G = Hq/Hkv in 1..16               */
  int32_t head_dim;        /* must be 128                                                 */
  int32_t block_tokens;    /* must be 16                                                  */
  int32_t n_device_blocks; /* M: blocks in the device pool                                */
  int32_t n_host_blocks;   /* slots in the pinned host pool (0 if swaps are not used)     */
  float softmax_scale;     /* 0 => 1/sqrt(head_dim)                                       */
  int32_t out_dtype;       /* PS_BF16 (default) or PS_F32                                 */
  int32_t decode_chunk;    /* 0 (default): the decode tokens of a batch are cut into equally
                              long slots, one wave per slot and kv-head, all resident at once
                              (see decode_waves); N > 0, a multiple of 32 in [32, 65536]:
                              fixed split-K partitions of N KV tokens, one wave each, instead  */
  int32_t swap_workgroups; /* workgroups used by a swap kernel; 0 => library picks        */
  int32_t own_streams;     /* 0 (default): everything a step does is enqueued on the caller's
                              stream. 1: the context creates a copy stream of its own (default
                              priority) on which the batch description of step n+1 is uploaded
                              while the kernels of step n run. A process has few hardware
                              queues, and streams that share one run one after another, so
                              this is opt-in.                                                  */
  int32_t prefill_split_tiles; /* 0 (default): the library splits the KV range of long prefill
                              rows over several workgroups (partials merged like decode's) when
                              the launch would otherwise be unbalanced; N > 0: always split into
                              partitions of N 64-token KV tiles; -1: never split               */
  int32_t decode_waves;    /* waves of a decode launch when decode_chunk is 0 (each walks one
                              slot of one kv-head); 0 (default) => one per SIMD, i.e. four per
                              compute unit of the device; else in [1, 65536]                   */
  /* What the launch planner assumes of the machine when it prices the decode work against the
     prefill work of a mixed batch (which share of the compute units each gets) and a split of long
     prefill rows against its merge.  0 => the value measured on an MI355X, given in brackets;
     another part, clock or power limit wants its own (time two probe launches: a decode-only and a
     prefill-only batch with ps_set_profiling(ctx, 2)).                                            */
  float plan_stream_TBps;      /* rate at which decode waves on the whole chip stream the cache [6.3]  */
  float plan_tile_step_us;     /* one 64-token KV tile step of a prefill workgroup [1.78]              */
  float plan_merge_launch_steps; /* a merge launch, in tile steps [4.0]                                */
  float plan_merge_row_steps;  /* merging one split row of 32 heads, in tile steps [0.0047]            */
  float plan_decode_share;     /* fraction of the balanced decode share actually given to decode: the
                                  prefill workgroups inherit units that decode leaves early, never the
                                  other way round [0.95]                                               */
  int32_t plan_decode_knee_cus;/* compute units below which the decode work slows in proportion
                                  (above, HBM is the limit) [176]                                      */
  int32_t swap_dma_runs;   /* 0 (default): swap lists are moved by a kernel that reads or writes the
                              pinned host pool itself.  N > 0: a list whose host slots form at most N
                              runs of consecutive slots (in list order) and that fits the context's
                              staging buffer (1024 blocks) crosses the host link on the copy engines
                              instead: a kernel packs the listed device blocks into the staging
                              buffer (or unpacks them from it) and every run is one hipMemcpyAsync.
                              Measured on an MI355X with 512 blocks in 16 runs of 32: slower one way
                              (41 against 54 GB/s), faster when both directions run at once (36
                              against 32 GB/s each way), hence opt-in.  In [0, 65536]              */
  int32_t mixed_launch;    /* how the attention launch of a batch with both decode tokens and prefill
                              chunks is laid out.  1: the two kinds of work on disjoint compute units
                              (decode workgroups first, the prefill workgroups take the rest).  2: every
                              workgroup carries both (a prefill tile walk on eight waves, next to them two
                              waves that fetch the walk's tiles and two that walk decode slots; needs
                              decode_chunk and decode_waves 0, else as 1).  0 (default): the library picks:
                              2 when neither kind of work dwarfs the other (the prefill work priced at 0.65
                              to 8 times the decode work; at 1 or 1.6 to 8 times it when the prefill
                              workgroups' KV walks are short) and there is at least one prefill workgroup per compute
                              unit (measured 2 to 20 % faster on such launches, the same or slower
                              outside that range), else 1.                                            */
} ps_layer_cfg;

/* One mixed batch (the output of Alg. 1 as the attention layer sees it). HOST arrays. */
typedef struct {
  int32_t n_req;
  int32_t n_tokens;         /* == q_start[n_req]                                           */
  const int32_t* q_start;   /* [n_req+1] prefix sum of l_q; l_q == 1 is a decode token,
                               l_q > 1 a prefill chunk                                     */
  const int32_t* kv_len;    /* [n_req] cached length INCLUDING this step's l_q tokens      */
  const int32_t* bt_start;  /* [n_req+1] CSR offsets into block_ids;
                               bt_start[r+1]-bt_start[r] == ceil(kv_len[r]/block_tokens)   */
  const int32_t* block_ids; /* physical device block ids, logical order                   */
  const uint8_t* prio;      /* [n_req] priority class, may be NULL; carried, not used      */
} ps_batch;

/* GPU time of the phases of the last profiled ps_step, in milliseconds, in the order they run:
 * upload (only with own_streams: the wait for the copy stream; otherwise the upload shares the
 * append's launch and is counted there), append, attention (one launch for the decode and the
 * prefill work of the batch), merge (the split-K partials of decode tokens and prefill rows).
 * decode_ms and prefill_ms are filled in profiling mode 2 only, where the two kinds of work are
 * launched one after the other (each with the whole chip) and attention_ms is their sum. */
typedef struct {
  float upload_ms, append_ms, decode_ms, merge_ms, prefill_ms, total_ms, attention_ms;
  /* Shader clock, in MHz, at which the decode and the prefill workgroups of the attention launch ran: the
     median over the (first 2048) workgroups of each kind of their shader-clock ticks per tick of the
     constant 100 MHz counter; 0 if the step had none.  The chip lowers this clock under load (2400 at
     rest), and the matrix-pipe peak falls with it. */
  float decode_mhz, prefill_mhz;
} ps_step_times;

const char* ps_last_error(void);

/* Creates a context on the current HIP device. The context owns small pinned staging buffers,
 * events, with cfg.own_streams a copy stream, and two device copies of the batch description
 * (the arrays of ps_batch plus work lists, about 5 bytes per block-table entry; they grow, with
 * a hipMalloc inside ps_step, when a batch is larger than any before). PS_EINVAL on a bad cfg. */
int ps_create(const ps_layer_cfg* cfg, ps_ctx** out);
void ps_destroy(ps_ctx* ctx);

/* Device workspace (split-K partial results of the decode kernels) needed by ps_step for any
 * batch with n_req <= max_req, n_tokens <= max_tokens and at most max_table_entries block-table
 * entries.  (Engine-internal: the paper describes no attention kernel, Sec. 4.1 only says that decode
 * is memory-bound and prefill compute-bound; the same holds for ps_plan_decode, ps_plan_launch and the
 * profiling calls below.) */
int ps_workspace_bytes(const ps_ctx* ctx, int32_t max_req, int32_t max_tokens,
                       int64_t max_table_entries, size_t* out_bytes);

/* One mixed-batch attention layer (Sec. 4.1 describes the batch; the attention is causal
 * softmax attention: query token i of request r, at absolute position p+i with
 * p = kv_len - l_q, attends cached tokens 0..p+i of kv-head h/G, scale softmax_scale).
 *   q        DEVICE bf16 [n_tokens][Hq][d]
 *   k_new,
 *   v_new    DEVICE bf16 [n_tokens][Hkv][d], this step's new K/V rows, written into the cache
 *            at positions p..kv_len-1 of each request before attention; both NULL if the
 *            cache already holds them
 *   kv_cache DEVICE, layout above, n_device_blocks blocks
 *   out      DEVICE [n_tokens][Hq][d], bf16 or f32 per cfg.out_dtype
 *   workspace DEVICE, 256-byte aligned, at least ps_workspace_bytes(...) bytes; its contents
 *            are scratch and may be reused by the next call on the same stream (calls on
 *            different streams need different workspaces; the context's own two copies of the
 *            batch description are guarded by the library: a step that would overwrite a copy
 *            which a step on another stream may still read waits for that step first)
 *   hip_stream  hipStream_t (NULL = default stream); the step is ordered on it: it starts after
 *            the stream's earlier work and the stream's later work starts after it (with
 *            cfg.own_streams parts of it run on the context's streams in between)
 *   wait_ticket 0, or a ticket from ps_swap_in/ps_swap_out: the stream waits for that copy
 *            to complete before any kernel of this step runs (Appendix B: compute
 *            synchronises on the reload's event only just before it needs the blocks)
 * Validation is host-side, O(batch description): PS_EINVAL for NULL pointers, non-monotone
 * q_start / bt_start, l_q < 1, l_q > kv_len, wrong table length, block id outside [0, M),
 * k_new given without v_new; PS_ENOMEM if the workspace is too small. n_req == 0 is a
 * successful no-op. Nothing is enqueued if validation fails. */
int ps_step(ps_ctx* ctx, const ps_batch* batch, const void* q, const void* k_new,
            const void* v_new, void* kv_cache, void* out, void* workspace,
            size_t workspace_bytes, void* hip_stream, uint64_t wait_ticket);

/* The same batch on another layer's tensors (Sec. 4.3 and Appendix B walk a forward pass layer by
 * layer: the batch, its block tables and the order of work are those of the pass, only q, the new
 * K/V rows, the cache and the output change from layer to layer). Reuses the work lists and the
 * device copy of the batch description made by the last successful ps_step on this context: no
 * validation of the batch, no planning, no upload -- only the kernels. Arguments as for ps_step;
 * k_new/v_new must be given exactly when that ps_step had them; the workspace needs the same size
 * as for that ps_step; the call must be ordered after that ps_step (same stream, or a stream
 * that waits for it). PS_ESTATE if there is no such ps_step (none yet, the last one failed, or it
 * had n_req == 0); other errors as for ps_step. */
int ps_step_next_layer(ps_ctx* ctx, const void* q, const void* k_new, const void* v_new,
                       void* kv_cache, void* out, void* workspace, size_t workspace_bytes,
                       void* hip_stream, uint64_t wait_ticket);

/* For callers that cannot allocate device memory: code under HIP graph capture, serving loops and harnesses
 * that forbid hipMalloc.  ps_step, with the split-K partials and the device copy of the batch description in a
 * fixed array of PS_STATIC_SCRATCH_BYTES that the library holds on every GPU it runs on until the process ends,
 * in place of the caller's workspace and of the context's growable buffers.  The call allocates nothing, on the
 * device or pinned: the staging it uses was allocated by ps_create.  Arguments and errors as for ps_step;
 * PS_ENOMEM if the batch needs more than the array holds (2 MiB of batch description, i.e. about 500 000
 * block-table entries; PS_STATIC_SCRATCH_BYTES - 4 MiB of partials, e.g. 840 partial rows of 64 heads); nothing
 * is enqueued then.  Every call on a GPU shares that GPU's array, whatever the context: the array keeps the last
 * call's contents (nothing in it has to start at zero: a step writes every entry it reads), and calls that
 * overlap on one GPU race -- keep them on one stream, or order the streams.  ps_step_next_layer does not follow
 * this call (PS_ESTATE). */
#define PS_STATIC_SCRATCH_BYTES (32u << 20)
int ps_step_static(ps_ctx* ctx, const ps_batch* batch, const void* q, const void* k_new, const void* v_new,
                   void* kv_cache, void* out, void* hip_stream, uint64_t wait_ticket);

/* Host only, no device needed: the decode work list ps_step builds for the decode requests (l_q == 1)
 * of `batch` when `waves` decode waves are available (ps_step itself uses four per compute unit for
 * a decode-only batch and a share of that next to prefill work). The list: the requests'
 * 32-token KV tiles, laid end to end in batch order, are cut into n_slots = min(waves / n_kv_heads,
 * tiles / 16) slots of equal length (to within one tile); each (slot, kv-head) is walked by one wave.
 * With cfg.decode_chunk > 0: fixed partitions of that many tokens, one per slot, longest first.
 *   cfg     only n_kv_heads, n_device_blocks and decode_chunk are read
 *   seg     HOST int32 [seg_cap][5], out: per segment, in launch order: request index, first token,
 *           one past the last token, slot index, partials index (-1: the request's only segment)
 *   n_seg, n_slots  out
 * PS_EINVAL as for ps_step's batch checks; PS_ENOMEM if seg_cap is too small (*n_seg is set). */
int ps_plan_decode(const ps_layer_cfg* cfg, const ps_batch* batch, int32_t waves, int32_t* seg,
                   int32_t seg_cap, int32_t* n_seg, int32_t* n_slots);

/* Host only, no device needed: how ps_step lays out the attention launch of `batch` on a device with n_cus
 * compute units (the decode work and the prefill work of a mixed batch share one launch; the decode
 * workgroups, one compute unit each, come first and the prefill workgroups take the rest and inherit the
 * decode units as those finish). For tests of that host logic.
 *   out6[0] decode waves     out6[1] decode slots (waves / Hkv)
 *   out6[2] decode workgroups; 0 for a mixed batch whose workgroups carry both kinds of work (cfg.mixed_launch):
 *           then every prefill workgroup also walks up to two of the decode slots
 *   out6[3] prefill workgroups     out6[4] KV tiles (64 tokens) per partition of split prefill rows, 0 = no row split
 *   out6[5] split-K partial slots the step uses
 * Errors as for ps_step's validation. */
int ps_plan_launch(const ps_layer_cfg* cfg, const ps_batch* batch, int32_t n_cus, int32_t* out6);

/* Diagnostic of the launch whose workgroups carry both kinds of work (cfg.mixed_launch).  Its waves hand K/V tiles
 * to one another through flags in LDS, and every wait for a flag is bounded: a wave that has waited about a tenth
 * of a second for one stops waiting (its outputs are then wrong) and counts itself here, so that a mistake in the
 * hand-over shows as a number and a failed comparison, never as a launch that does not end.  (Engine-internal, no
 * counterpart in the paper.)
 *   out   HOST: waves that gave up since the library was loaded, over all contexts of the current device; 0 unless
 *         the library is broken.  The call synchronises the device.
 * PS_EINVAL for a NULL argument, PS_EHIP if the counter cannot be read. */
int ps_mixed_launch_faults(uint32_t* out);

/* Per-phase GPU timing of ps_step with events on its stream (adds a few microseconds), and the shader
 * clock its attention workgroups ran at (clock counters read in the kernel).  The first call with a
 * non-zero mode allocates 128 KiB of device memory for those counters and creates the events; no step
 * allocates for them.  Every call restarts the series that ps_get_step_times averages.
 * mode 0: off; 1: the phases as they run; 2: the decode and the prefill work of the attention
 * phase in launches of their own, one after the other. PS_EINVAL for any other mode; PS_EHIP if the
 * allocation fails. */
int ps_set_profiling(ps_ctx* ctx, int mode);
/* Blocks until the last profiled step has finished, then fills *out with the mean over the profiled steps
 * enqueued since the previous call (the most recent 64 of them; events are kept per step, so many steps can
 * run back to back with no host synchronisation between them and be read once); the clocks are those of the
 * last step.  With no profiled step since the previous call, that call's figures again.  PS_ESTATE before the
 * first profiled step. */
int ps_get_step_times(ps_ctx* ctx, ps_step_times* out);

/* Asynchronous offload (Sec. 4.3): host_pool[host_slot_ids[k]] <- cache[dev_block_ids[k]] for
 * the first min(n, copy_budget) entries, in list order (copy_budget < 0: unlimited), enqueued
 * on side_stream. *n_done gets that count, *ticket a completion handle (0 if nothing moved).
 * The device blocks may be reused only after the ticket completes.
 *   dev_block_ids, host_slot_ids  HOST int32 [n]
 *   kv_cache DEVICE; host_pool PINNED, n_host_blocks slots of one block each
 * PS_EINVAL: id outside its pool, duplicate id within a list, NULL pointer with n > 0. */
int ps_swap_out(ps_ctx* ctx, const int32_t* dev_block_ids, const int32_t* host_slot_ids,
                int32_t n, int32_t copy_budget, const void* kv_cache, void* host_pool,
                void* side_stream, int32_t* n_done, uint64_t* ticket);

/* Pipelined reload (Sec. 4.3): cache[dev_block_ids[k]] <- host_pool[host_slot_ids[k]], same
 * rules as ps_swap_out; copy_budget is B_copy of the adaptive copy-budget control. Pass the
 * ticket to ps_step so that attention starts only after the blocks have landed. */
int ps_swap_in(ps_ctx* ctx, const int32_t* host_slot_ids, const int32_t* dev_block_ids,
               int32_t n, int32_t copy_budget, const void* host_pool, void* kv_cache,
               void* side_stream, int32_t* n_done, uint64_t* ticket);

/* A ticket is the completion event of one swap call (Appendix B: reloads signal one event per layer
 * chunk, which the compute stream waits on only just before it needs the blocks; offloads run on a
 * stream of their own outside the forward path and are polled).  Tickets count up from 1; the library
 * keeps the events of the last 64, an older ticket counts as complete (its event was waited for before
 * its slot was reused).  PS_ESTATE: 0, or a ticket that was never handed out. */
int ps_ticket_query(ps_ctx* ctx, uint64_t ticket); /* PS_OK done | PS_EBUSY in flight | PS_ESTATE */
int ps_ticket_wait(ps_ctx* ctx, uint64_t ticket);  /* host blocks until done                      */

/* ------------------------------------------------------------------------------------------
 * Host-only batch former: SlideBatching (Alg. 1) with the block management of Sec. 4.3.
 * All times are integer picoseconds; all arithmetic is exact (128-bit intermediates), so two
 * implementations of the same rules agree bit for bit. No GPU call is made by these functions.
 * ------------------------------------------------------------------------------------------ */
typedef struct ps_sched ps_sched;

typedef struct {
  int32_t n_classes;        /* priority classes 1..n_classes (1 = highest), at most 8        */
  int32_t block_tokens;     /* s_blk, 16                                                      */
  int64_t class_weight[8];  /* w_{p}: priority weight of class p at index p-1 (Sec. 2)        */
  int64_t w_first;          /* w_p of Eq. 3: weight of the first token                        */
  int64_t w_decode;         /* w_d of Eq. 3: weight of every later token                      */
  int64_t ttft_slo_ps;      /* deadline_{r,i} = TTFT_SLO + (i-1) TPOT_SLO (Eq. 3)             */
  int64_t tpot_slo_ps;
  int64_t a_p, b_p, c_p;    /* T~_p = a_p l_q^2 + b_p l_q l_kv + c_p l_q   (Eq. 5), ps        */
  int64_t a_d, b_d;         /* T~_d = a_d l_kv + b_d                       (Eq. 6), ps        */
  int64_t t_c;              /* constant per-batch overhead (Eq. 4), ps                        */
  int64_t eta_ps;           /* lower bound of the latency budget (Alg. 1 line 7); > t_c       */
  int64_t tau_ps;           /* starvation threshold (Sec. 4.2)                                */
  int64_t gamma_num, gamma_den; /* aggressiveness coefficient gamma as a fraction              */
  int64_t beta_num, beta_den;   /* partial-copy threshold beta > 1 as a fraction (Sec. 4.3)    */
  int64_t rho_num, rho_den;     /* a request that waited >= rho*tau is never an eviction victim */
  int64_t t_block_ps;       /* profiled copy time of one block (Sec. 4.3)                     */
  int32_t n_off_base;       /* offload threshold n_off of class 1; halves per class, floor 1  */
  int32_t order_policy;     /* PS_ORDER_SLIDEBATCHING (0): Alg. 1 line 13 with the starvation rule;
                               PS_ORDER_FCFS: arrival order only, the first-come-first-served arm
                               of the comparisons in Sec. 5 (everything else of the round as is)   */
} ps_sched_cfg;

enum { PS_ORDER_SLIDEBATCHING = 0, PS_ORDER_FCFS = 1 };

/* Result of one scheduling round. Every pointer refers to memory owned by the scheduler and
 * stays valid until the next call on the same ps_sched. `batch` can be handed to ps_step as is:
 * members in admission order, l_q tokens each, kv_len including them, their device block tables. */
typedef struct {
  ps_batch batch;
  const int64_t* req_ids;            /* [batch.n_req]                                        */
  int64_t t_budget_ps;               /* max(t_min, eta)                                      */
  int64_t phi_ps;                    /* load judgment phi(Q), Eq. 8                          */
  int64_t t_batch_ps;                /* T_pd(B), Eq. 7; 0 if nothing was admitted            */
  int64_t copy_budget;               /* B_copy                                               */
  int32_t n_order;                   /* sorted queue                                         */
  int32_t n_urgent;
  const int64_t* order;              /* [n_order] request ids in scheduling order            */
  const int64_t* urgent;             /* [n_urgent] ids classified URGENT, in that order      */
  int32_t n_swap_in, n_swap_out;
  const int32_t* swap_in_host_slots; /* reload list for ps_swap_in (already within budget)   */
  const int32_t* swap_in_dev_blocks;
  const int32_t* swap_out_dev_blocks;/* offload list for ps_swap_out                         */
  const int32_t* swap_out_host_slots;
  int32_t n_evicted, n_emitted;
  const int64_t* evicted;            /* requests whose device blocks were freed              */
  const int64_t* emitted_req;        /* tokens delivered at now + t_batch: request ...       */
  const int32_t* emitted_index;      /* ... and 1-based token index                          */
  int32_t n_finished, reserved;
  const int64_t* finished;           /* requests that delivered their last token             */
  int64_t round;                     /* 1-based count of ps_form_batch calls on this scheduler:
                                        names the offload list of this round towards
                                        ps_sched_offloads_done                                */
} ps_batch_out;

/* dev_free_order / host_free_order: the block ids of the two pools in the order they are to be
 * handed out (each pool is a LIFO stack; a request's blocks are returned in logical order).
 * PS_EINVAL: bad cfg (eta <= t_c, zero denominators, n_classes outside 1..8, duplicates). */
int ps_sched_create(const ps_sched_cfg* cfg, const int32_t* dev_free_order, int32_t n_dev,
                    const int32_t* host_free_order, int32_t n_host, ps_sched** out);
void ps_sched_destroy(ps_sched* s);
/* Adds a request to the queue. PS_EINVAL: duplicate id, prio outside 1..n_classes,
 * prompt_len < 1, out_len < 1. */
int ps_sched_add_request(ps_sched* s, int64_t rid, int64_t arrival_ps, int32_t prio,
                         int32_t prompt_len, int32_t out_len);
/* One round of Alg. 1 at time now_ps over the requests that have arrived: orders the queue,
 * computes the copy budget, admits requests (evicting from the tail under memory pressure),
 * and applies the round to the state (blocks, computed tokens, delivered tokens, offloads). */
int ps_form_batch(ps_sched* s, int64_t now_ps, ps_batch_out* out);
/* Completion report of the offload thread (Sec. 4.3, Asynchronous Offloading): every device-to-host
 * copy issued by rounds <= upto_round (ps_batch_out.round) has landed, e.g. because ps_ticket_query
 * says so of that round's ps_swap_out.  Copies on one stream complete in issue order, so a watermark
 * is enough.  Until a copy is reported its host slot does not count at an eviction: the victim's device
 * blocks are freed at once, the pending transfer is discarded (its host slot released) and the tokens
 * it would have covered are recomputed.  Rounds whose offload list is empty need no report.
 * PS_EINVAL: a round that has not been formed. */
int ps_sched_offloads_done(ps_sched* s, int64_t upto_round);
/* Queue and pool occupancy, for tests and monitoring. Any pointer may be NULL. */
int ps_sched_counts(const ps_sched* s, int32_t* n_queued, int32_t* n_dev_free, int32_t* n_host_free);

/* Eq. 3 for one request of class prio: *gain = sum over the n_times delivered tokens of w_r(i) where
 * token_times[i-1] (relative to the request's arrival) is strictly before deadline_{r,i} = TTFT_SLO +
 * (i-1) TPOT_SLO; w_r(1) = w_first * class weight, w_r(i>1) = w_decode * class weight.  *ideal_gain = the
 * gain of out_len tokens all on time (Ideal_Gain of Sec. 5.1); *slo_attained = 1 iff the first token is
 * strictly before TTFT_SLO and the mean gap of the later ones strictly below TPOT_SLO (Sec. 5.1, Metrics).
 * token_times HOST [n_times]; any output pointer may be NULL.  Only the weights and SLOs of cfg are read. */
int ps_tdg_score(const ps_sched_cfg* cfg, int32_t prio, int32_t out_len, const int64_t* token_times,
                 int32_t n_times, int64_t* gain, int64_t* ideal_gain, int32_t* slo_attained);

typedef struct {
  int64_t rid, arrival_ps;
  int32_t prio, prompt_len, out_len, reserved;
} ps_trace_req;

typedef struct {
  int64_t gain, ideal_gain; /* summed over the finished requests (TDG ratio = gain / ideal_gain)   */
  int32_t slo_attained, finished, steps, reserved;
  int64_t end_ps;           /* the clock when the run stopped                                      */
} ps_sim_result;

/* Single-instance serving run on a virtual clock (host only): the requests of `trace` join the queue at
 * their arrival, every round is one ps_form_batch, the clock advances by its T_pd(B) (Eq. 7; by eta when
 * nothing could be admitted, to the next arrival when the queue is empty), tokens are delivered when their
 * batch ends and scored with Eq. 3.  The offload thread of Sec. 4.3 runs on the same clock: the copies a
 * round issues start when its batch has been computed and the earlier copies are through, take t_block per
 * block, and are reported (ps_sched_offloads_done) at the first round that starts at or after their end.
 * Stops after max_steps rounds or when the trace is exhausted.
 *   trace        HOST [n_trace], any order, distinct ids
 *   token_times  HOST int64 [sum of out_len], may be NULL: delivery times relative to arrival, request i of
 *                `trace` at offset sum_{j<i} out_len[j]
 *   n_delivered  HOST int32 [n_trace], may be NULL: tokens delivered per request
 * Errors as for ps_sched_create / ps_sched_add_request. */
int ps_sched_simulate(const ps_sched_cfg* cfg, const int32_t* dev_free_order, int32_t n_dev,
                      const int32_t* host_free_order, int32_t n_host, const ps_trace_req* trace, int32_t n_trace,
                      int32_t max_steps, int64_t* token_times, int32_t* n_delivered, ps_sim_result* out);

#ifdef __cplusplus
}
#endif
#endif /* PS_H_ */
