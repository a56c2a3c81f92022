/*
 * libmdi -- one node's model partition for model-distributed LLM inference on
 * AMD MI355X (gfx950).
 *
 * The paper's problem statement (Sec. III-A): a node owns a contiguous chunk of
 * the decoder, receives the intermediate activations of sample n from the
 * previous node, runs them through its local layers using the n-th KV cache
 * (Sec. III-D, "rotating KV caches"), and hands the result to the next node.
 * A sample's first visit carries the whole prompt and builds the cache
 * (Alg. 1 / Alg. 2, "first iteration"); every later visit carries only the
 * newest token's activation (Sec. III-D).  The starter node additionally owns
 * the embedding and the output layers (final norm + vocabulary projection,
 * Sec. III-B), which hold no KV state (Sec. III-E).
 *
 * This header is the whole boundary: plain C, POD structs, raw pointers.
 * Unless a parameter says "host", every data pointer is a DEVICE pointer that
 * the caller allocated (the library allocates no device memory at all; its
 * working set lives in the caller-provided arena).  All compute calls enqueue
 * work on the partition's HIP stream and return without waiting; argument and
 * state errors are detected on the host before anything is enqueued.
 *
 * Thread-safety: calls on one partition must be serialised by the caller;
 * different partitions may be driven concurrently from different threads and
 * streams.
 *
 * Process-wide state.  Partitions share no data, with one exception that the
 * persistent decode launch forces: that launch (one kernel for a whole decode
 * step, used whenever the shape allows it, see decode_path) keeps one
 * workgroup per compute unit resident (two of half the size when it carries
 * several messages) and its workgroups wait for each other, so two such
 * launches must never be dispatched side by side, or each could hold a part
 * of the compute units and wait for the rest.  The library therefore keeps, per
 * HIP device, a mutex-guarded event that orders every persistent launch after
 * the previous one of any other partition on that device: decode steps of
 * different partitions run one after the other even when their streams differ
 * (first visits, output layers and the one-kernel-per-operation path are
 * ordinary launches and do overlap).  The launch also assumes that nothing
 * else occupies the compute units for good (another process's persistent
 * kernel, say).  Every wait inside it is bounded: if the workgroups cannot all
 * become resident, or an exchange never completes, the kernel gives up, the
 * step's outputs are invalid and mdi_partition_sync reports MDI_ERR_HIP; the
 * partition must then be destroyed (its exchange counters are no longer
 * consistent), other partitions are unaffected.  Two more things are kept per
 * process: the fixed scratch array of mdi_sample_topk_static (one copy per GPU,
 * see there), and a counter that numbers the launches of the output layers
 * (the number travels with the per-workgroup argmax candidates, so that a
 * candidate left behind by an earlier launch is never taken for a new one).
 *
 * Two tuning knobs are read from the environment when a partition is created:
 * MDI_GROUP_CTX = context length from which, in models whose query heads share
 * kv heads in even groups, the decode kernel lets two query heads take one pass
 * over the cache together (default 4096; below it every head takes its own).
 * Results are within the parity bar either way; the order of additions differs.
 * MDI_BATCH_GROUP = 1, 2 or 4 fixes the number of query heads per attention
 * work item of mdi_decode_batch (by default chosen per call from the number of
 * messages and the longest context); used by tests to reach every variant on
 * small shapes.
 */
#ifndef MDI_H
#define MDI_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define MDI_ABI_VERSION 1u
#define MDI_API __attribute__((visibility("default")))

typedef struct mdi_partition mdi_partition; /* opaque host object */

typedef enum {
  MDI_OK = 0,
  MDI_ERR_ARG = -1,   /* null pointer, index out of range, unsupported shape          */
  MDI_ERR_STATE = -2, /* decode before the first visit, prefill of a live sequence     */
  MDI_ERR_CTX = -3,   /* the call would grow a sequence beyond max_ctx                 */
  MDI_ERR_NOMEM = -4, /* arena too small, or the KV page pool is exhausted             */
  MDI_ERR_HIP = -5,   /* a HIP runtime call or kernel launch reported an error         */
  MDI_ERR_LIMIT = -6  /* mdi_sample_topk_static: vocabulary beyond its fixed scratch   */
} mdi_status;

enum { MDI_NORM_LAYERNORM = 0, MDI_NORM_RMSNORM = 1 };
enum { MDI_MLP_GELU_TANH = 0, MDI_MLP_GELU_ERF = 1, MDI_MLP_SWIGLU = 2 };
enum { MDI_POS_LEARNED = 0, MDI_POS_ROPE = 1 };
enum { MDI_F32 = 0, MDI_BF16 = 1 };
enum { MDI_HAS_EMBED = 1u, MDI_HAS_HEAD = 2u };

/*
 * Model and cache geometry.  Passed by pointer (host), copied at create.
 *
 * dtype selects the storage type of weight matrices, embeddings, KV cache
 * entries and of the activations crossing this boundary (acts_in / acts_out):
 * MDI_F32 = IEEE binary32, MDI_BF16 = bfloat16 bit patterns.  Norm gains,
 * norm biases and linear biases are always binary32.  Every accumulation
 * (dot products, norms, softmax) is binary32 in both modes.
 */
typedef struct mdi_config {
  uint32_t abi_version;    /* MDI_ABI_VERSION */
  uint32_t n_layer;        /* layers of the WHOLE model (layer_hi is checked against it) */
  uint32_t d_model;        /* embedding dimension; multiple of 8                        */
  uint32_t n_head;         /* query heads H; n_head * head_dim may differ from d_model  */
  uint32_t n_kv_head;      /* key/value heads K; H % K == 0 (grouped-query attention)    */
  uint32_t head_dim;       /* h; multiple of 8, at most 256                             */
  uint32_t d_ff;           /* MLP width F; multiple of 8                                */
  uint32_t vocab;          /* V                                                         */
  uint32_t max_ctx;        /* longest sequence (prompt + generated) a cache may hold     */
  uint32_t max_seqs;       /* number of samples in flight = number of KV caches          */
  uint32_t kv_page_tokens; /* tokens per KV page; 0 = 16; max_ctx * this < 2^32         */
  uint32_t kv_pages;       /* pages in the pool; 0 = max_seqs * ceil(max_ctx / page)     */
  uint32_t max_prefill;    /* longest first visit T; 0 = max_ctx (sizes prefill scratch) */
  uint32_t norm_kind;      /* MDI_NORM_*                                                */
  float norm_eps;
  uint32_t mlp_kind;       /* MDI_MLP_*                                                 */
  uint32_t pos_kind;       /* MDI_POS_*: learned absolute table added at embed, or RoPE  */
  float rope_base;         /* RoPE: angle of pair i at position p is p * base^(-2i/h),
                              pairing element i with element i + h/2 of each head        */
  uint32_t has_bias;       /* linear layers carry biases (GPT-2 family)                 */
  uint32_t tie_embed;      /* vocabulary projection shares the embedding matrix          */
  uint32_t dtype;          /* MDI_F32 | MDI_BF16                                        */
  uint32_t decode_path;    /* how a decode step is launched.  0 = automatic: one persistent kernel launch
                              when the shape allows it, else one kernel per operation; 1 = always one
                              kernel per operation; other values = 0                               */
} mdi_config;

/*
 * Source weights of one decoder layer, device pointers, `[out_features,
 * in_features]` row-major, contiguous, in cfg.dtype; vectors in binary32.
 * Pointers that do not apply (biases when has_bias == 0, ln*_b for RMSNorm,
 * w_gate for GELU MLPs) are NULL.  A NULL bias with has_bias == 1 means zero.
 * has_bias covers the attention projections and the GELU MLP; a SwiGLU MLP
 * carries no biases: b_up / b_down must be NULL there (MDI_ERR_ARG otherwise).
 */
typedef struct mdi_layer_weights {
  const void *ln1_g, *ln1_b; /* [d] pre-attention norm                                  */
  const void *wq, *wk, *wv;  /* [H*h, d], [K*h, d], [K*h, d]                            */
  const void *bq, *bk, *bv;  /* [H*h], [K*h], [K*h]                                     */
  const void *wo, *bo;       /* [d, H*h], [d]                                           */
  const void *ln2_g, *ln2_b; /* [d] pre-MLP norm                                        */
  const void *w_gate;        /* SwiGLU gate [F, d]                                      */
  const void *w_up, *b_up;   /* SwiGLU up / GELU first matrix [F, d], [F]               */
  const void *w_down, *b_down; /* [d, F], [d]                                           */
} mdi_layer_weights;

typedef struct mdi_weights {
  const void *wte;     /* [V, d] token embedding; needed with MDI_HAS_EMBED, and with
                          MDI_HAS_HEAD when tie_embed                                   */
  const void *wpe;     /* [max_ctx, d] learned positions; MDI_HAS_EMBED + MDI_POS_LEARNED */
  const void *lnf_g, *lnf_b; /* [d] final norm; MDI_HAS_HEAD                            */
  const void *lm_head; /* [V, d]; MDI_HAS_HEAD and not tie_embed                        */
  const mdi_layer_weights *layers; /* HOST array of layer_hi - layer_lo entries          */
} mdi_weights;

/*
 * Size in bytes of the device arena a partition needs: the node's model chunk
 * (Sec. III-B: the layers it was assigned, plus embedding / output layers on
 * the starter), one KV cache per sample in flight (Sec. III-D; the paper's
 * memory tables, Sec. IV-C, count exactly these per node), page tables and
 * scratch.  arena_bytes: host pointer, written on MDI_OK.
 */
MDI_API mdi_status mdi_partition_bytes(const mdi_config *cfg, uint32_t layer_lo, uint32_t layer_hi,
                               uint32_t flags, size_t *arena_bytes);

/*
 * Build the chunk of layers [layer_lo, layer_hi) (Sec. III-B).  flags:
 * MDI_HAS_EMBED = inputs are int32 token ids (starter's input portion);
 * MDI_HAS_HEAD = mdi_sample_greedy is available (starter's output portion).
 * layer_lo == layer_hi is legal only with MDI_HAS_HEAD and without
 * MDI_HAS_EMBED: an output portion without transformer blocks (Sec. III-E).
 *
 * The weights are copied, repacked, into `arena` (256-byte aligned device
 * memory of at least mdi_partition_bytes() bytes, owned by the caller and kept
 * alive until destroy); the copies are enqueued on `hip_stream`
 * (a hipStream_t; NULL = the default stream), so the sources may be freed once
 * that stream has drained.  *out receives the new handle.
 */
MDI_API mdi_status mdi_partition_create(const mdi_config *cfg, uint32_t layer_lo, uint32_t layer_hi,
                                const mdi_weights *weights, uint32_t flags, void *arena,
                                size_t arena_bytes, void *hip_stream, mdi_partition **out);

/*
 * First visit of sample seq_id (Alg. 1 round 0 / Alg. 2 "n-th KV cache is
 * None"): initialise its cache and forward all T prompt positions.
 * acts_in: int32[T] token ids with MDI_HAS_EMBED, else [T, d] in cfg.dtype.
 * acts_out: [T, d] in cfg.dtype, row-major.  acts_in and acts_out must not overlap.
 * Errors: MDI_ERR_STATE if the sequence is live, MDI_ERR_CTX if T > max_ctx,
 * MDI_ERR_ARG if T == 0, T > max_prefill or seq_id >= max_seqs,
 * MDI_ERR_NOMEM if the page pool cannot hold T more tokens.
 */
MDI_API mdi_status mdi_prefill(mdi_partition *part, uint32_t seq_id, const void *acts_in, uint32_t T,
                       void *acts_out);

/*
 * A first visit in several pieces: forward the next T prompt positions of
 * sample seq_id, which continue at its current cache length (0 for a fresh
 * sample: then this is mdi_prefill).  The positions attend to the cache and
 * to each other causally, so the pieces together compute what one
 * mdi_prefill of the whole prompt computes; a node can then let other
 * samples' messages in between the pieces of a long prompt instead of
 * stalling them for the whole first visit (the start-up transient of
 * Sec. IV-B grows with what a first visit costs).
 * Arguments and errors as mdi_prefill, except that a live sequence is not an
 * error; MDI_ERR_CTX if the cache length + T exceeds max_ctx.
 */
MDI_API mdi_status mdi_prefill_chunk(mdi_partition *part, uint32_t seq_id, const void *acts_in,
                             uint32_t T, void *acts_out);

/*
 * Later visit (Sec. III-D): forward only the newest position through the local
 * layers, reading and extending KV cache seq_id.  The position is implicit:
 * the partition counts each sequence's length, as the paper's message carries
 * only the sample id (Sec. III-E).
 * act_in: int32[1] token id with MDI_HAS_EMBED, else [d] in cfg.dtype.
 * act_out: [d] in cfg.dtype.
 * Errors: MDI_ERR_STATE before the first visit, MDI_ERR_CTX when the cache is
 * full, MDI_ERR_NOMEM when no page is free.
 */
MDI_API mdi_status mdi_decode_step(mdi_partition *part, uint32_t seq_id, const void *act_in,
                           void *act_out);

/*
 * Later visits of n different samples whose messages wait in the node's input
 * queue (Sec. III-A: arriving messages are queued and taken out in order;
 * Sec. III-C: several samples are in flight at once).  Every message is still
 * forwarded on its own, with its own pass over the layer weights, and each
 * sample's result is that of mdi_decode_step up to the order in which a row's
 * partial sums are added (a few units in the last place of the accumulation
 * type; for a given call pattern results are reproducible bit for bit).  On
 * the persistent decode path up to 8 messages share one launch: two sets of
 * workgroups share the compute units, each set alternates its messages inside
 * every phase, so that the exchange between workgroups that ends one message's
 * phase is covered by other messages' weight streaming.
 * seq_ids: host uint32[n], pairwise different.  acts_in / acts_out: host arrays
 * of n device pointers, each as act_in / act_out of mdi_decode_step.
 * Errors: as mdi_decode_step, checked for all n messages before the first is
 * taken (on such an error no sequence has advanced); MDI_ERR_ARG also when
 * n == 0 or a sample id occurs twice.
 */
MDI_API mdi_status mdi_decode_steps(mdi_partition *part, uint32_t n, const uint32_t *seq_ids,
                            const void *const *acts_in, void *const *acts_out);

/*
 * Later visits of n different samples whose messages wait in the input queue
 * (Sec. III-A, III-C), taken through the local layers TOGETHER: one pass over
 * the layer weights serves up to 16 messages (each weight is fetched once and
 * multiplied with all their vectors on the matrix cores), attention runs per
 * sample over each sample's own cache (Sec. III-D).  This goes beyond the
 * paper's one-message-at-a-time rule: the traffic of a pass is the weights
 * once plus every sample's cache, instead of the weights once per message.
 * More than 16 messages take several passes; a lone message is forwarded as
 * by mdi_decode_step.  Needs bf16 storage, the persistent decode path,
 * d_model, n_head * head_dim, d_ff multiples of 32 (d_model at most 4096);
 * other partitions forward the messages as mdi_decode_steps does
 * (mdi_partition_info(4) tells).  Vectors between the matrix products are
 * rounded to bf16 here (as in a first visit), so a sample's result agrees with
 * mdi_decode_step's within the bf16 parity bar, not to the last bits; for a
 * given call pattern results are reproducible bit for bit.
 * Arguments and errors: as mdi_decode_steps.
 */
MDI_API mdi_status mdi_decode_batch(mdi_partition *part, uint32_t n, const uint32_t *seq_ids,
                            const void *const *acts_in, void *const *acts_out);

/*
 * Output layers (Alg. 1 "process output layers ... get token", with greedy
 * argmax in place of sampling): final norm, vocabulary projection, argmax
 * (lowest index on exact ties).  Needs MDI_HAS_HEAD; touches no KV state.
 * act_in: [d] in cfg.dtype (the last block's output for the newest position).
 * token_out: int32[1].  logits_out: float[V] or NULL.
 */
MDI_API mdi_status mdi_sample_greedy(mdi_partition *part, uint32_t seq_id, const void *act_in,
                             int32_t *token_out, float *logits_out);

/*
 * Output layers with a draw from the output distribution (Alg. 1 samples the
 * pmf; the paper names no knobs, the usual temperature and top-k are taken):
 * final norm, vocabulary projection, then a token drawn from
 * softmax(logits / temperature) restricted to the top_k largest logits (ties:
 * the lower index ranks first) by inverting the cumulative distribution, in
 * rank order and binary32, at the uniform number u = (x >> 8) / 2^24, x the
 * first word of Philox-4x32-10 (Salmon et al., SC'11) for counter
 * (seq_id, step, 0, 0) and key (seed mod 2^32, seed / 2^32): the token is the
 * first candidate j with u * sum(w) < w_0 + ... + w_j, w_j = exp((l_j - l_max)
 * / temperature).  The same (seed, seq_id, step) always gives the same token.
 * temperature > 0; 1 <= top_k <= 64 (top_k = 1 is mdi_sample_greedy).
 * act_in, token_out, logits_out: as in mdi_sample_greedy.
 */
MDI_API mdi_status mdi_sample_topk(mdi_partition *part, uint32_t seq_id, const void *act_in,
                           float temperature, uint32_t top_k, uint64_t seed, uint32_t step,
                           int32_t *token_out, float *logits_out);

/*
 * mdi_sample_topk for callers that cannot allocate device memory or hand the
 * library any: code under HIP graph capture, tight serving loops, harnesses
 * that forbid allocation.  Same arguments, same result (token and logits are
 * bit-identical to mdi_sample_topk's; top_k = 1 gives the greedy token), but
 * the kernels' scratch - the [V] float logits the sampler works on, the
 * per-workgroup argmax candidates and the arrival counter - is not taken from
 * the partition's arena: it lives in a fixed array inside the library
 * (1 MiB + 24.25 KiB of device memory per GPU, held until the process ends).
 * The call allocates and frees nothing and records no memset (the counter is
 * cleared by a small fill kernel).  Limit: vocab <= 262144, else MDI_ERR_LIMIT.
 * All calls on one GPU share the array: calls that overlap on a GPU (different
 * streams, different partitions, different threads) race; the caller orders
 * them.  Other errors as mdi_sample_topk; MDI_ERR_STATE also when the
 * partition's device is not the current one on the array's first use.
 */
MDI_API mdi_status mdi_sample_topk_static(mdi_partition *part, uint32_t seq_id, const void *act_in,
                                  float temperature, uint32_t top_k, uint64_t seed, uint32_t step,
                                  int32_t *token_out, float *logits_out);

/*
 * Output layers for n samples whose last hidden states wait at the starter
 * together (Alg. 1 "process output layers ... get token", once per returning
 * sample; several samples are in flight, Sec. III-C): ONE pass over the
 * vocabulary matrix serves up to 16 samples (each row is fetched once and
 * multiplied with all their normalised activations on the matrix cores); more
 * than 16 take several passes.  top_k = 1: greedy argmax as mdi_sample_greedy
 * (temperature, seed, steps ignored; steps may be NULL); top_k > 1: the draw
 * of mdi_sample_topk per sample with counter (seq_ids[i], steps[i]).
 * seq_ids, acts_in, steps: HOST arrays of n; acts_in[i]: device, [d] in
 * cfg.dtype.  tokens_out: device int32[n].  logits_out: device float[n][V]
 * (row i = sample i) or NULL.  Needs bf16 storage, d_model a
 * multiple of 32 (at most 4608), activations aligned to 16 bytes and the
 * persistent decode path; otherwise, and for n = 1, the samples are served
 * one by one exactly as mdi_sample_greedy / mdi_sample_topk would
 * (mdi_partition_info(6) tells).  In the shared pass the normalised
 * activations are rounded to bf16, so logits agree with mdi_sample_greedy's
 * within the bf16 parity bar, not to the last bits; the token is the argmax of
 * (or the draw from) the logits this call returns.  Errors: as
 * mdi_sample_topk; n = 0 does nothing.
 */
MDI_API mdi_status mdi_sample_batch(mdi_partition *part, uint32_t n, const uint32_t *seq_ids,
                            const void *const *acts_in, float temperature, uint32_t top_k,
                            uint64_t seed, const uint32_t *steps, int32_t *tokens_out,
                            float *logits_out);

/*
 * Wait for everything enqueued on the partition's stream and report errors that
 * only the device can detect: MDI_ERR_HIP if the stream failed or if a
 * workgroup of a persistent decode kernel gave up waiting for the others (its
 * waits are bounded; the step's outputs are then invalid); MDI_ERR_ARG if a
 * token id outside [0, vocab) reached a kernel (token ids live in device
 * memory, so they are checked where they are read; such an id is read as
 * token 0 and the outputs that depend on it are meaningless).  The condition
 * stays set until the partition is destroyed.
 */
MDI_API mdi_status mdi_partition_sync(mdi_partition *part);

/*
 * Back to "the n-th KV cache is None" (Alg. 2): drop sample seq_id's cache, its
 * pages return to the pool, and its next message must be a first visit again.
 * The caller orders this after the work that still reads the cache (same stream
 * or a wait); nothing is enqueued.
 */
MDI_API mdi_status mdi_seq_reset(mdi_partition *part, uint32_t seq_id);

/*
 * Tokens currently cached for seq_id, i.e. the position the next message of
 * that sample takes (Sec. III-E: a message carries only the sample id, the node
 * keeps count); 0 = no cache yet (Alg. 2).  len: host pointer.
 */
MDI_API mdi_status mdi_seq_len(const mdi_partition *part, uint32_t seq_id, uint32_t *len);

/*
 * Bytes one decode step of this partition must move at context length ctx
 * (packed weights + KV read for ctx positions + KV write + activation in/out),
 * and the same for one mdi_sample_greedy call (ctx ignored when head != 0).
 * bytes: host pointer.
 */
MDI_API mdi_status mdi_step_bytes(const mdi_partition *part, uint32_t ctx, int head, uint64_t *bytes);

/*
 * Measurement aid for the bandwidth roofline: time one kind of decode kernel in
 * isolation with HIP events on the partition's stream.  One repetition launches
 * the kernel once for every local layer in turn (so consecutive launches stream
 * different weights and nothing is served from a cache), `reps` repetitions
 * are timed back to back, and the call waits for them.  which: 1 = attention
 * output projection, 2 = MLP up (+gate) projection, 3 = MLP down projection.
 * They read and write only the partition's scratch vectors (no KV state).
 * avg_us / bytes_per_launch: host pointers; mean duration of one launch in
 * microseconds and the matrix bytes one launch must read.
 */
MDI_API mdi_status mdi_time_kernel(mdi_partition *part, int which, uint32_t reps, float *avg_us,
                                   uint64_t *bytes_per_launch);

/*
 * Introspection.  what: 0 = decode path in use (2 = persistent single launch,
 * 1 = one kernel per operation), 1 = workgroups in one set of the persistent
 * launch (0 on the other path), 2 = its LDS bytes per workgroup (0 likewise),
 * 3 = arena bytes in use, 4 = messages one pass of mdi_decode_batch can take
 * (0: this partition forwards them one pass each), 5 = bytes of the local
 * layers' matrices (what one pass over the weights reads), 6 = samples one
 * pass of mdi_sample_batch can take (0: it serves them one by one).  value:
 * host pointer.
 */
MDI_API mdi_status mdi_partition_info(const mdi_partition *part, uint32_t what, uint64_t *value);

/*
 * Profiling aid for the persistent decode kernel: when trace is not NULL, every
 * following decode step records, per workgroup, layer and phase (QKV, attention,
 * output projection, MLP up, MLP down), up to eight 100 MHz timestamps: 0 phase
 * entered (first tiles issued), 1 barrier passed, 2 input vector staged, 3 first
 * wavefront done streaming, 4 all wavefronts done (GEMV phases), 5 results
 * stored, 6 stores acknowledged; slot 7 is unused.  trace: device buffer of
 * uint64 [2][workgroups][local layers][5][8] (mdi_partition_info gives the workgroup
 * count; a launch that carries several messages, see mdi_decode_steps, records the
 * first message of each of its two sets of workgroups, first and second half),
 * owned by the caller; NULL switches tracing off.
 */
MDI_API mdi_status mdi_partition_trace(mdi_partition *part, void *trace);

/*
 * The node leaves the ring (the starter's stop message of Sec. III-A ends a
 * secondary's loop, Alg. 2): frees the host object.  Nothing is enqueued and
 * nothing waited for: the caller drains the partition's stream first
 * (mdi_partition_sync) and keeps the arena, which stays its own.
 */
MDI_API void mdi_partition_destroy(mdi_partition *part);

MDI_API const char *mdi_strerror(mdi_status st);

#ifdef __cplusplus
}
#endif
#endif /* MDI_H */
