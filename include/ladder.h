/*
 * ladder.h -- C-ABI of the MI355X (gfx950) Ladder-Residual shard forward.
 *
 * One context = one tensor-parallel rank's shard (or n_real_shards emulated
 * ranks) of a stack of N Ladder-Residual Transformer layers, 2N modules
 * (odd m = attention of layer (m+1)/2, even m = SwiGLU MLP of layer m/2), on
 * ONE GPU.  The paper's blocking AllReduce is replaced by a local sum of the
 * rank partial sums (computed shards + caller-supplied synthetic partials of
 * the ranks that are not computed).  In the one-kernel-per-operation
 * schedules that sum runs on internal streams with HIP events playing the
 * role of the paper's AsyncAllReduce handles (Algorithm 1); in the fused
 * decode schedule it is the epilogue of the module's last projection and
 * the overlap Algorithm 1 obtains from the handles comes from putting the
 * independent work of neighbouring modules into one launch.  Nothing crosses
 * a GPU boundary.
 *
 * Conventions
 *   - row-vector convention y = x W; every matrix handed in is row-major
 *     [in_features][out_features].
 *   - all head counts and the SwiGLU intermediate size are PER-SHARD sizes.
 *   - "T" below = the storage dtype selected by ladder_config.dtype
 *     (LADDER_FP32: float, LADDER_BF16: bfloat16 bit pattern in uint16).
 *   - every pointer named "device" is a HIP device pointer of the current
 *     device; config / weight-descriptor structs are host memory.
 *   - calls are ordered on the stream given to ladder_init: the work runs on
 *     the context's own streams, which wait for that stream at entry and which
 *     that stream waits for before the call returns; calls return without
 *     synchronising; outputs are valid once the caller has synchronised the
 *     stream.
 *   - every entry point returns 0 or a negative LADDER_E_* code; nothing
 *     throws or aborts across the boundary; a failed call leaves the
 *     context's position unchanged.  ladder_last_error gives a text.
 *   - a context is not thread-safe.
 */
#ifndef LADDER_H_
#define LADDER_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct ladder_ctx ladder_ctx; /* opaque, owned by the library */

enum { LADDER_FP32 = 0, LADDER_BF16 = 1 };
enum { LADDER_WIRING_LADDER = 0, LADDER_WIRING_STANDARD = 1, LADDER_WIRING_PARALLEL = 2 };
enum { LADDER_PATH_AUTO = 0, LADDER_PATH_GENERIC = 1 };

enum {
  LADDER_OK = 0,
  LADDER_E_ARG = -1,      /* null pointer, non-positive size, unknown enum */
  LADDER_E_SHAPE = -2,    /* sizes that do not fit each other or the limits */
  LADDER_E_STATE = -3,    /* call order: decode before prefill / load_kv, layer not loaded */
  LADDER_E_OVERFLOW = -4, /* position + new tokens > max_seq */
  LADDER_E_HIP = -5       /* a HIP runtime call failed (text in ladder_last_error) */
};

typedef struct {
  int32_t n_layers;       /* N */
  int32_t hidden;         /* H, replicated on every rank; multiple of 8 */
  int32_t n_q_heads;      /* local query heads; multiple of n_kv_heads */
  int32_t n_kv_heads;     /* local KV heads */
  int32_t head_dim;       /* d, even, <= 256 */
  int32_t inter;          /* local SwiGLU intermediate size */
  int32_t tp_degree;      /* R */
  int32_t n_real_shards;  /* 1..R shards computed by this context; the other R - n_real_shards
                             ranks contribute synthetic partial sums (ladder_set_peer_partials) */
  int32_t max_batch;      /* largest B of any call */
  int32_t max_seq;        /* KV-cache capacity in positions per sequence */
  int32_t max_tokens;     /* largest T of a prefill call (workspaces hold max_batch*max_tokens rows) */
  int32_t dtype;          /* LADDER_FP32 | LADDER_BF16: storage type T of weights, inputs, KV cache, peers */
  int32_t wiring;         /* LADDER_WIRING_LADDER: module m reads x_{m-2} (Eq. 2);
                             LADDER_WIRING_STANDARD: module m reads x_{m-1} (Eq. 1);
                             LADDER_WIRING_PARALLEL: the parallel attention / MLP block that section "Faster
                             Inference with Ladder Residual" compares with: both modules of a layer read the
                             layer's input (attention x_{m-1}, MLP x_{m-2}); one reduce per layer where the
                             reduce is a step of its own (n_standard_layers must be 0) */
  int32_t n_standard_layers; /* hybrid: with wiring LADDER, the first n_standard_layers layers still use
                                the standard wiring (the paper's hybrid keeps ladder for the upper layers) */
  int32_t reduce_on_side_stream; /* 1: reduce + residual add overlap the next module on a side stream;
                                    0: everything in order on one stream (same results).  Like
                                    overlap_modules it applies to calls of at most 64 rows that do not take
                                    the fused decode schedule; larger calls (prefill) always run in order:
                                    their kernels fill the chip and measured slower when spread over streams */
  int32_t peer_pool;      /* number of distinct synthetic peer sets; module m uses set m % peer_pool */
  int32_t peer_rows;      /* rows of each synthetic peer tensor (>= rows of any call), 0 if no peers */
  int32_t kernel_path;    /* LADDER_PATH_AUTO: MFMA/streaming kernels when dtype and sizes allow;
                             LADDER_PATH_GENERIC: the plain kernels (any size, both dtypes) */
  int32_t overlap_modules; /* 1: attention modules and MLP modules run on two internal streams, so that
                              module m+1 (which under the ladder wiring needs only x_{m-1}) can execute
                              while module m still runs; 0: one compute stream.  Same results. */
  int32_t decode_graph;   /* 1: a decode step of the bf16 streaming path is captured once into a HIP graph
                             and replayed (the position lives in device memory and is advanced by the
                             graph itself); 0: eager launches.  Same results. */
  int32_t decode_fused;   /* 1 or 2: decode steps of the bf16 streaming path (batch <= 16, one computed shard,
                             max_seq <= 65536) use the fused launches: residual add, partial-sum reduce,
                             RMSNorm, rotary, cache append and SwiGLU are epilogues / prologues of the
                             projections.  1: the independent projections / attention of neighbouring modules
                             share one launch where the wiring leaves them independent (ladder: two launches per
                             layer; parallel block: three); 2: one job per launch whatever the wiring (five per
                             layer), which leaves every collective a whole module to hide behind;
                             3: the launch list of 1 as ONE launch per step (a "chained" step): persistent
                             workgroups run the list's blocks in turn, and a module starts when the modules whose
                             streams it reads (x_{m-2} and x_{m-1} of Algorithm 1) have raised their completion
                             flags, not when a launch has ended; same arithmetic in the same order, same bits.
                             It keeps one buffer per stream x_m and per layer (about 3.4 KB x hidden x n_layers
                             more workspace at 16 rows; ladder_workspace_bytes counts it);
                             0: one kernel per operation */
  int32_t reduce_delay_us; /* emulated all-reduce latency (Fig. 2 / Table 2 of the paper vary the interconnect), 0 .. 10000.
                              Fused decode schedules: the collective that completes x_m starts when the last
                              workgroup of module m's residual update ends (the workgroups leave the device's
                              wall-clock time) and lasts this many microseconds; the projections that read x_m
                              hold their workgroups back until then (a bounded wait on the clock, inside the
                              launch), while the other jobs run; the arithmetic is unchanged (same bits).
                              One kernel per operation: a timed wait of that length in
                              front of every partial-sum reduce, on the stream the reduce runs on.
                              (LADDER_WIRING_PARALLEL: one collective per layer.) */
  float rms_eps;          /* RMSNorm epsilon (inside the square root) */
  float rope_theta;       /* rotary base; pair (2j,2j+1) turns by pos * theta^(-2j/d) */
} ladder_config;

/* Device pointers to ONE shard of ONE layer (caller-owned; read only inside ladder_load_layer,
 * which copies / repacks them; they may be freed afterwards).  Section "Tensor Parallelism
 * Background": first matmuls are split along the output dimension, second along the input one. */
typedef struct {
  const void* attn_norm; /* T [H]            gain of AttentionNorm (Algorithm 1) */
  const void* wq;        /* T [H][nq*d]      this shard's query-head columns */
  const void* wk;        /* T [H][nkv*d] */
  const void* wv;        /* T [H][nkv*d] */
  const void* wo;        /* T [nq*d][H]      rows of the same query heads */
  const void* mlp_norm;  /* T [H]            gain of MLPNorm */
  const void* w_gate;    /* T [H][I] */
  const void* w_up;      /* T [H][I] */
  const void* w_down;    /* T [I][H] */
} ladder_layer_weights;

/* Creates a context for the block stack that Algorithm 1 / Eq. 2 define (N layers of an attention module and
 * an MLP module around one residual stream, section "Ladder Residual"; module shapes per "Llama-3's model
 * architecture", section "Setup"; this rank's shard per section "Tensor Parallelism Background"): validates
 * the configuration, allocates the repacked-weight store, the KV cache, workspaces, the internal streams and
 * events (the handles of Algorithm 1's AsyncAllReduce) on the current device.
 *   cfg        host pointer.
 *   hip_stream the caller's hipStream_t (NULL = the null stream); all work is ordered on it.
 *   out        receives the context.
 * Errors: LADDER_E_ARG, LADDER_E_SHAPE, LADDER_E_HIP (then *out is NULL). */
int ladder_init(const ladder_config* cfg, void* hip_stream, ladder_ctx** out);

/* Copies / repacks one shard of one layer into the context (enqueued on the caller's stream): the
 * weights of AttentionNorm, Attention, MLPNorm and MLP of Algorithm 1, split as section "Tensor Parallelism
 * Background" says.  layer in [0, N), shard in [0, n_real_shards).  Every (layer, shard) must be loaded
 * before the first forward call (else LADDER_E_STATE there).  The two gains are taken from shard 0's call
 * (they are replicated across ranks) and may be NULL for the other shards.  Repacking only re-orders: the
 * library keeps the weights' bits as given. */
int ladder_load_layer(ladder_ctx* ctx, int32_t layer, int32_t shard, const ladder_layer_weights* w);

/* The other ranks' terms of the AllReduce of Eq. 2 (x_m = AllReduce(h_m(x_{m-2})) + x_{m-1}) on one GPU:
 * synthetic partial sums of the ranks that are not computed: device T
 * [peer_pool][R - n_real_shards][peer_rows][H], caller-owned, NOT copied: it must stay valid and
 * unchanged while forward calls use it.  Row b*T + t of a set is added for token t of sequence b.
 * NULL switches the peers off.  A change takes effect at the next forward call (a captured decode step is
 * captured again).  LADDER_E_SHAPE if the configuration has no peers. */
int ladder_set_peer_partials(ladder_ctx* ctx, const void* peers);

/* The cache that the attention modules of Algorithm 1 read at decode (section "Setup": generation after a
 * prompt of 1024 tokens), without running the prompt: fills the KV cache of (layer, shard) with caller-made
 * content instead of a prefill:
 * k, v device T [B][nkv][S][d] (k already rotated).  Sets the context position to S once every
 * (layer, shard) has been given the same B and S.  LADDER_E_SHAPE / LADDER_E_OVERFLOW on misfit. */
int ladder_load_kv(ladder_ctx* ctx, int32_t layer, int32_t shard, const void* k, const void* v,
                   int32_t B, int32_t S);

/* Prefill: resets the position to 0 and runs modules 1..2N (Eq. 2 / Algorithm 1, or Eq. 1 per the
 * wiring) on T tokens of each of B sequences with causal attention, filling the KV cache; position
 * becomes T.
 *   x_in   device T   [B][T][H]  input embeddings x_0.
 *   x_out  device f32 [B][T][H]  x_2N = residual + last attention output + last MLP output.
 * Errors: LADDER_E_ARG, LADDER_E_SHAPE (B > max_batch, T > max_tokens, B*T > peer_rows),
 * LADDER_E_OVERFLOW (T > max_seq), LADDER_E_STATE (a layer is not loaded), LADDER_E_HIP. */
int ladder_prefill(ladder_ctx* ctx, const void* x_in, int32_t B, int32_t T, void* x_out);

/* One decode step = modules 1..2N of Eq. 2 / Algorithm 1 (or Eq. 1 per the wiring) on one new token per
 * sequence (section "Inference Implementation": token-by-token generation after the prefill): one new
 * embedding per sequence at the current position (the batch size is the one of the preceding prefill /
 * load_kv); appends to the cache; position += 1.
 *   x_in   device T   [B][H]
 *   x_out  device f32 [B][H]
 * Errors: LADDER_E_STATE (no prefill / load_kv yet), LADDER_E_OVERFLOW (cache full), others as above;
 * LADDER_E_HIP also when a kernel of an EARLIER step gave up its bounded in-launch wait (that step's output
 * is then invalid; the failing call itself does nothing and clears the condition). */
int ladder_decode_step(ladder_ctx* ctx, const void* x_in, void* x_out);

/* ---- pipeline stages (section "Compatibility with other Parallelism Techniques") ------------------
 *
 * A context whose layers are one pipeline stage of a deeper model: instead of embeddings it takes, and instead
 * of x_2N it leaves, the three tensors that Algorithm 1 passes from block to block, with every reduction they
 * depend on complete (at a stage boundary the asynchronous AllReduce has to be waited for):
 *   residual   the stream without the outputs of the last two modules,
 *   attn       the reduced output of the last attention module,
 *   mlp        the reduced output of the last MLP module.
 * The first block of the stage adds attn_in to the residual before its attention module and mlp_in before its
 * MLP module, as every later block does with its predecessor's outputs.  The first stage is given the
 * embeddings (as f32) in residual_in and NULL for attn_in and mlp_in (= zeros); the model's output x_2N is the
 * sum of the three tensors the last stage leaves.  The outputs are computed as differences of consecutive
 * streams (fp32: residual_out + attn_out reproduces the stream the stage held to within one rounding).
 * Otherwise as ladder_prefill / ladder_decode_step (cache, position, batch, errors).  The synthetic peer partial
 * sums of the stage's module m are set (m mod peer_pool) of THIS context.
 *   residual_in, attn_in, mlp_in      device f32 [B][T][H] ([B][H] for a decode step), 16-byte aligned, caller-owned
 *   residual_out, attn_out, mlp_out   device f32, same shape, distinct buffers; may be the input buffers
 * Decode steps are launched eagerly also in a context that replays ladder_decode_step from a captured graph.
 * Errors: LADDER_E_ARG (null residual_in / outputs, misaligned or coinciding outputs), LADDER_E_STATE also when
 * a layer of the context has the standard or the parallel wiring (the hand-over is the ladder wiring's). */
int ladder_prefill_stage(ladder_ctx* ctx, const float* residual_in, const float* attn_in, const float* mlp_in,
                         int32_t B, int32_t T, float* residual_out, float* attn_out, float* mlp_out);
int ladder_decode_step_stage(ladder_ctx* ctx, const float* residual_in, const float* attn_in, const float* mlp_in,
                             float* residual_out, float* attn_out, float* mlp_out);

/* Ends the block stack of ladder_init: releases everything the context owns (synchronises its streams
 * first).  NULL is a no-op. */
void ladder_free(ladder_ctx* ctx);

/* ---- generation head (Llama-3 architecture around the block stack; the paper's engine is a prefill
 *      followed by token-by-token decoding, sections "Inference Implementation" and "Setup") ------
 *
 * ladder_load_head copies the token-embedding table, and copies / repacks this rank's slice of the
 * output projection (split along the vocabulary, the rule of section "Tensor Parallelism Background"
 * for a first matmul):
 *   table       device T [vocab][H]
 *   final_norm  device T [H]             gain of the RMSNorm in front of the output projection
 *   w_lm        device T [H][vocab_local]
 * All three are caller-owned and may be freed afterwards.  Once per context (LADDER_E_STATE again).
 * Errors: LADDER_E_ARG, LADDER_E_SHAPE (sizes), LADDER_E_HIP. */
int ladder_load_head(ladder_ctx* ctx, const void* table, const void* final_norm, const void* w_lm, int32_t vocab,
                     int32_t vocab_local);

/* Token embedding: x_out[r][:] = table[tokens[r]][:].
 *   tokens  device int32 [rows]  (an id outside [0, vocab) reads row 0 or vocab - 1 instead, so that no
 *                                access leaves the table, and is REPORTED: once the kernel has run, the next
 *                                ladder_embed, ladder_prefill or ladder_decode_step of this context fails with
 *                                LADDER_E_ARG, does nothing else, and clears the condition)
 *   x_out   device T [rows][H]   rows <= max_batch * max_tokens; ready to be x_in of ladder_prefill
 *                                ([B][T][H], rows = B*T) or ladder_decode_step ([B][H]).
 * Enqueued on the caller's stream.  Errors: LADDER_E_ARG, LADDER_E_STATE (head not loaded), LADDER_E_SHAPE. */
int ladder_embed(ladder_ctx* ctx, const int32_t* tokens, int32_t rows, void* x_out);

/* Final RMSNorm + output projection + greedy sampling for one position per sequence:
 * logits = rmsnorm(x, final_norm) . w_lm, token = index of the largest logit of this rank's slice
 * (lowest index among equal maxima; the index is local to the slice).
 *   x           device f32 [rows][H]    rows of x_2N (rows <= max_batch)
 *   logits_out  device f32 [rows][vocab_local], or NULL
 *   tokens_out  device int32 [rows], or NULL (not both NULL)
 * Enqueued on the caller's stream.  Errors: LADDER_E_ARG, LADDER_E_STATE (head not loaded), LADDER_E_SHAPE. */
int ladder_head(ladder_ctx* ctx, const float* x, int32_t rows, float* logits_out, int32_t* tokens_out);

/* ladder_head for callers that cannot allocate (code under HIP graph capture, tight serving loops, harnesses
 * that forbid hipMalloc): the same final RMSNorm + output projection + greedy arg max, with the normed rows and
 * the logits -- which ladder_head keeps in buffers the context allocated -- in a fixed static device array
 * of the library instead (LADDER_HEAD_STATIC_MAX_ROWS x (LADDER_HEAD_STATIC_MAX_HIDDEN +
 * LADDER_HEAD_STATIC_MAX_VOCAB) x 4 bytes = 2.5 MiB per GPU, held until the process ends).  The call
 * allocates and frees nothing, on the host side of the runtime or the device.
 *   x           device f32 [rows][H]
 *   tokens_out  device int32 [rows]   (the same tokens as ladder_head gives)
 * Every call on a GPU shares that GPU's array (whatever the context): calls that overlap on one GPU --
 * different streams, or different host threads -- race; calls ordered on one stream do not.  Nothing in the
 * array has to start at zero: a call overwrites all it reads.
 * Errors: as ladder_head; LADDER_E_SHAPE also when rows, hidden or vocab_local exceed the limits below;
 * LADDER_E_STATE when the current device is not the context's. */
#define LADDER_HEAD_STATIC_MAX_ROWS 16
#define LADDER_HEAD_STATIC_MAX_HIDDEN 8192
#define LADDER_HEAD_STATIC_MAX_VOCAB 32768
int ladder_head_static(ladder_ctx* ctx, const float* x, int32_t rows, int32_t* tokens_out);

/* ---- helpers ---------------------------------------------------------------------------- */

/* Text of the last error of this context (or of the last failed ladder_init / sizing call when ctx is NULL).
 * The pointer stays valid until the next failing call.  (With LADDER_DEBUG set in the environment the library
 * also writes the host-side steps of graph capture and of the per-operation schedule to stderr.) */
const char* ladder_last_error(const ladder_ctx* ctx);

/* Where the context stands in the prefill-then-decode run (section "Setup"): current number of cached
 * positions per sequence and current batch size (0 before any prefill / load_kv).  LADDER_E_ARG on NULL. */
int ladder_position(const ladder_ctx* ctx, int32_t* pos, int32_t* batch);

/* Device bytes the context holds (weights store + KV cache + workspaces + generation head, if loaded). */
size_t ladder_device_bytes(const ladder_ctx* ctx);

/* Sizing before any allocation (host only, no GPU needed, callable before ladder_init): the device bytes that
 * ladder_init(cfg) allocates apart from the weight store -- KV cache, rotary tables, norm gains, residual
 * stream, partial-sum and activation buffers of Algorithm 1's modules -- and the bytes of the weight store
 * itself.  Their sum is ladder_device_bytes of a fresh context.  0 if the configuration is rejected (the
 * text is in ladder_last_error(NULL)). */
size_t ladder_workspace_bytes(const ladder_config* cfg);
size_t ladder_weight_bytes(const ladder_config* cfg);

/* Test hook for the in-launch waits of the fused decode schedules (decode_fused = 1: the output projection of a
 * layer waits, inside the launch, for that layer's attention workgroups; decode_fused = 3: every job of the
 * chained step waits for the jobs that produce what it reads; all such waits are bounded): max_polls polls instead
 * of 2^20, and target_bias added to the value a wait polls for.  With a bias no producer can reach, the waits give
 * up: the waiting workgroups store nothing, every kernel still ends normally, and the NEXT ladder_decode_step /
 * ladder_prefill returns LADDER_E_HIP (and puts the device's copy of the position back in step with the host's).
 * (1 << 20, 0) restores normal operation.  Errors: LADDER_E_ARG. */
int ladder_set_wait_limit(ladder_ctx* ctx, int32_t max_polls, int32_t target_bias);

/* Timeline of a chained decode step (decode_fused = 3), for measurement.  A chained step is one launch of
 * persistent workgroups ("slots") that run the blocks of the step's launch list in turn (the modules of
 * Algorithm 1 in their order, each starting when the streams it reads are complete), so events around the launch
 * say nothing about its parts.  With the timeline on, every slot records for every block the device wall-clock
 * time at which it took the block (and requested its first weight tiles), at which the block's inputs were
 * complete, and at which the block ended; ladder_timeline_read returns the records of the last step.  (Where a
 * launch of the list has more blocks than there are slots, the blocks beyond the slots are not dealt out beforehand
 * but taken, one at a time, by slots that have finished their own block of that launch; those are not recorded.)
 *   out / cap   caller's array (host) and its capacity; *n_out receives the number of records of the step (call
 *               with out = NULL to size the array); records beyond cap are not written.
 *   ticks_per_us  receives the rate of the clock the times are in (may be NULL).
 * Recording changes no result; it costs three stores per block.
 * Errors: LADDER_E_STATE if the context does not run chained steps, replays captured steps (decode_graph = 1), or
 * has recorded nothing yet; LADDER_E_ARG on NULL; LADDER_E_HIP if the recording buffer cannot be allocated. */
typedef struct ladder_timeline_rec {
  int32_t slot;          /* persistent workgroup */
  int32_t launch;        /* index of the block's launch in the step's launch list */
  int32_t kind;          /* LADDER_TL_* */
  int32_t tiles;         /* 16-column weight tiles of the block (projections; 0 for attention) */
  int64_t weight_bytes;  /* weight bytes the block streams */
  uint64_t t_take, t_ready, t_end;
} ladder_timeline_rec;
enum { LADDER_TL_ATTN = 0, LADDER_TL_QKV = 1, LADDER_TL_O = 2, LADDER_TL_GATE_UP = 3, LADDER_TL_DOWN = 4 };
int ladder_timeline_enable(ladder_ctx* ctx, int32_t on);
int ladder_timeline_read(ladder_ctx* ctx, ladder_timeline_rec* out, int64_t cap, int64_t* n_out, double* ticks_per_us);

/* Per-kernel timing for measurement.  With profiling on, every kernel launch is bracketed by HIP
 * events on the stream it is launched on; ladder_profile_read synchronises, folds the events
 * recorded since the last read into per-class totals and returns them.
 *   cls        one of LADDER_K_*;  launches / total_ms receive the totals (may be NULL).
 * Profiling changes no result; it slows the call (events between launches). */
enum {
  LADDER_K_REDUCE_NORM = 0, /* partial-sum reduce + residual add + RMSNorm (side stream) */
  LADDER_K_GEMV = 1,        /* decode weight-streaming skinny GEMM (all four projections) */
  LADDER_K_GEMM = 2,        /* prefill MFMA GEMM */
  LADDER_K_ROPE_APPEND = 3,
  LADDER_K_ATTN_DECODE = 4, /* split-KV decode attention + combine */
  LADDER_K_ATTN_PREFILL = 5,
  LADDER_K_GENERIC = 6,     /* plain kernels (fp32 / any-size path) */
  LADDER_K_OTHER = 7,
  LADDER_K_FUSED_DECODE = 8, /* fused decode launches (projection(s) and/or attention of one step) */
  LADDER_K_COUNT = 9
};
int ladder_profile_enable(ladder_ctx* ctx, int32_t on);
int ladder_profile_read(ladder_ctx* ctx, int32_t cls, int64_t* launches, double* total_ms);
int ladder_profile_reset(ladder_ctx* ctx);

/* Measurement helper: copies `bytes` bytes (a multiple of 16; both device pointers 16-byte aligned,
 * caller-owned, not overlapping) with a plain copy kernel on the caller's stream.  It reads and writes
 * exactly `bytes` bytes of HBM once, which is what hardware byte counters (rocprofv3 FETCH_SIZE /
 * WRITE_SIZE) are scaled by when the traffic of the other kernels is measured.
 * Errors: LADDER_E_ARG (NULL), LADDER_E_SHAPE (size / alignment), LADDER_E_HIP. */
int ladder_calibration_copy(ladder_ctx* ctx, void* dst, const void* src, size_t bytes);

#ifdef __cplusplus
}
#endif
#endif /* LADDER_H_ */
