/*
 * pascal_sched — host-side phase-aware scheduler that decides, per decode
 * iteration, which requests run on which instance and which KV blocks move,
 * and hands the result over in the layouts the pkv kernels take (pkv.h).
 *
 * C ABI, host memory only: no pointer here is device memory and no call
 * touches the GPU.  The caller executes the returned data-movement orders with
 * kv_blocks_offload / kv_blocks_reload / kv_blocks_move (or gather + scatter)
 * and runs the batch with kv_append + paged_decode_attn(_layers).
 *
 * Model (paper Section IV).  A cluster of instances, each with its own pool of
 * KV blocks.  A request is in its reasoning phase (prefill and reasoning
 * tokens) until the model emits the end-of-reasoning token, then in its
 * answering phase.  Per instance a high-priority queue holds reasoning
 * requests and a low-priority queue holds answering requests (Section IV-C);
 * inside a queue requests take turns round-robin with a token quantum; a
 * reasoning request whose KV cache exceeds `demote_tokens` moves to the
 * low-priority queue.  New requests are routed by Algorithm 1, requests that
 * finish reasoning by Algorithm 2 followed by the adaptive-migration rule
 * (Section IV-B).  Time is whatever the caller passes as `now` (seconds).
 *
 * Every function returns PASCAL_OK or a negative status; on error nothing
 * changed (the one exception: PASCAL_ERR_CAPACITY from pascal_plan or
 * pascal_commit means host memory ran out midway and the object can only be
 * destroyed).  A scheduler object must not be used from two threads at once.
 */
#ifndef PASCAL_SCHED_H_
#define PASCAL_SCHED_H_

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define PASCAL_OK 0
#define PASCAL_ERR_NULL (-1)     /* a required pointer is NULL                           */
#define PASCAL_ERR_ARG (-2)      /* a value is out of range                              */
#define PASCAL_ERR_STATE (-3)    /* plan without the previous commit, or the reverse     */
#define PASCAL_ERR_CAPACITY (-4) /* an output array is too small, or a prompt can never
                                    fit an instance                                      */

/* What the model produced for a request in one iteration. */
#define PASCAL_TOKEN 0
#define PASCAL_END_OF_REASONING 1 /* the marker that closes the reasoning phase          */
#define PASCAL_END_OF_SEQUENCE 2

/* Data-movement orders, to be executed in the order given. */
#define PASCAL_OP_OFFLOAD 1      /* preemption: blocks -> host store, then they are free */
#define PASCAL_OP_RELOAD 2       /* resumption: host store -> these new blocks           */
#define PASCAL_OP_PREFILL 3      /* first run: the prompt's KV goes into these blocks    */
#define PASCAL_OP_GROW 4         /* a block appended to a running request, no data moves */
#define PASCAL_OP_MIGRATE 5      /* phase transition: blocks on `instance` -> blocks on
                                    `other_instance`, then the former are free           */
#define PASCAL_OP_MIGRATE_HOST 6 /* the same, but the destination has no room: the image
                                    goes to its host store and is reloaded there later   */
#define PASCAL_OP_FREE 7         /* the request finished; informational                  */

#define PASCAL_REASONING 0
#define PASCAL_ANSWERING 1
#define PASCAL_QUEUED 0          /* admitted, never run: no KV yet                       */
#define PASCAL_RESIDENT 1        /* KV in the instance's GPU blocks                      */
#define PASCAL_OFFLOADED 2       /* KV in the instance's host store                      */
#define PASCAL_FINISHED 3

/* The two ablations of the paper's Section V-D: a request stays where it did its
 * reasoning; or Algorithm 2's choice is followed without the adaptive override. */
#define PASCAL_FLAG_NO_MIGRATION 1
#define PASCAL_FLAG_NOT_ADAPTIVE 2

typedef struct {
  int32_t num_instances;   /* >= 1 (the paper evaluates 8, Section V-A)                  */
  int32_t gpu_blocks;      /* KV blocks of one instance's pool                           */
  int32_t block_tokens;    /* tokens per block (16 for the pkv kernels)                  */
  int32_t quantum_tokens;  /* round-robin quantum of both queues (500, Section V-A)      */
  int32_t demote_tokens;   /* KV size beyond which a reasoning request is demoted (5000) */
  int32_t headroom_blocks; /* free blocks that count as "sufficient memory" in the
                              adaptive-migration rule                                    */
  int32_t max_batch;       /* most requests in one iteration's batch; 0 = no limit       */
  int32_t flags;           /* 0, or PASCAL_FLAG_* ored together                          */
  double target_tpot_s;    /* the reader's pace, seconds per answering token (0.1)       */
} pascal_config;

typedef struct {
  int32_t kind;            /* PASCAL_OP_*                                                */
  int32_t instance;        /* where `n_blocks` blocks live (the source of a migration)   */
  int32_t request;
  int32_t other_instance;  /* destination of a migration, else -1                        */
  int32_t first_block;     /* index into the flat block-id array fetched with the ops    */
  int32_t n_blocks;        /* ids [first_block, first_block + n_blocks) on `instance`,
                              in the order of the request's block table                  */
  int32_t n_other_blocks;  /* then this many ids on `other_instance` (PASCAL_OP_MIGRATE) */
  int32_t reserved;
} pascal_op;

typedef struct {
  int32_t instance, phase, state, level; /* level: 0 high-priority queue, 1 low          */
  int32_t prompt_tokens, kv_tokens;      /* kv_tokens: tokens whose K,V are cached       */
  int32_t reasoning_tokens, answering_tokens;
  int32_t n_blocks;                      /* GPU blocks held                              */
  int32_t preemptions, migrations, reserved;
  double arrival, finish;                /* finish < 0 while unfinished                  */
  double ttft;                           /* first answering token - arrival; < 0 before  */
  double qoe;                            /* Section II-C measure from TPOT alone, over the
                                            answering tokens so far, in (0, 1]           */
} pascal_request_info;

typedef struct pascal_sched pascal_sched;

int pascal_create(const pascal_config* config, pascal_sched** out);
void pascal_destroy(pascal_sched* s);

/* A new request enters its reasoning phase: Algorithm 1 picks the instance with
 * the smallest KV footprint (GPU + host store, prompts still waiting included)
 * among those whose answering requests keep up with their readers, or among all
 * when none does.  Request ids count up from 0. */
int pascal_submit(pascal_sched* s, int32_t prompt_tokens, double now, int32_t* request,
                  int32_t* instance);

/* Intra-instance scheduler, one iteration (Section IV-C): walks the
 * high-priority queue, then the low-priority queue, each in round-robin order,
 * and gives every request the blocks its KV cache needs after this iteration.
 * When blocks are short, resident requests further back are evicted, last
 * first, never one ahead; a request that cannot be made to fit waits.  The
 * counts of the batch and of the resulting orders come back; fetch the
 * contents with the three calls below.  pascal_commit must follow. */
int pascal_plan(pascal_sched* s, int32_t instance, int32_t* n_selected, int32_t* n_ops,
                int32_t* n_op_blocks);

/* The planned batch: request ids and context lengths after the iteration (a
 * first-run request attends over its prompt), in batch order. */
int pascal_plan_batch(const pascal_sched* s, int32_t instance, int32_t* requests,
                      int32_t* context_lens, int32_t capacity);

/* The batch's block tables, int32 [n_selected][max_blocks_per_seq] as
 * paged_decode_attn reads them; unused entries are set to `fill`. */
int pascal_plan_block_tables(const pascal_sched* s, int32_t instance, int32_t* block_tables,
                             int32_t max_blocks_per_seq, int32_t fill);

/* The orders of the latest pascal_plan or pascal_commit on this instance. */
int pascal_ops(const pascal_sched* s, int32_t instance, pascal_op* ops, int32_t op_capacity,
               int32_t* blocks, int32_t block_capacity);

/* The iteration's tokens, one PASCAL_TOKEN / _END_OF_REASONING / _END_OF_SEQUENCE
 * per batch entry: counters and quanta advance, a request that used up its
 * quantum goes to the back of its queue, finished requests release their
 * blocks, oversized reasoning requests are demoted, and a request that closed
 * its reasoning phase is placed by Algorithm 2 (fewest reasoning requests among
 * compliant instances; all instances and reasoning + fresh answering requests
 * when none complies) unless the adaptive rule keeps it where it is. */
int pascal_commit(pascal_sched* s, int32_t instance, double now, const int32_t* token_kinds,
                  int32_t n, int32_t* n_ops, int32_t* n_op_blocks);

/* The signals the two algorithms read for an instance: t (1 = every answering
 * request keeps up with its reader), m (KV blocks, GPU + host store + waiting
 * prompts), r (requests in the high-priority queue), a (answering requests
 * still in their first quantum), free GPU blocks.  Any output may be NULL. */
int pascal_instance_signals(const pascal_sched* s, int32_t instance, double now, int32_t* t,
                            int64_t* m, int32_t* r, int32_t* a, int32_t* free_blocks);

int pascal_request(const pascal_sched* s, int32_t request, pascal_request_info* out);

/* Token pacer (Section II-C): how many answering tokens the user has been shown by
 * `now`.  Tokens produced in a burst are held back and released one per
 * target_tpot_s, so a request that was ahead of its reader keeps streaming
 * while it is preempted: visible = number of k with d_k <= now, where
 * d_0 = g_0 and d_k = max(g_k, d_{k-1} + target_tpot_s) over the production
 * times g. */
int pascal_request_visible_tokens(const pascal_sched* s, int32_t request, double now,
                                  int32_t* visible);

/* The request's GPU blocks in table order; returns their number or a negative status. */
int pascal_request_blocks(const pascal_sched* s, int32_t request, int32_t* blocks,
                          int32_t capacity);

const char* pascal_status_string(int status);

#ifdef __cplusplus
}
#endif
#endif /* PASCAL_SCHED_H_ */
