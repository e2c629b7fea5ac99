// Host side of the C-ABI: configuration checks, memory plan, weight loading (repack into matrix-core
// tiles), and the schedules of the Ladder-Residual forward (Algorithm 1 / Eq. 2).
//
// All work runs on the context's own streams; the caller's stream is fenced in and out with events.
//
// Per-operation schedule (forward_body: prefill, fp32, several computed shards).  Module m (1..2N)
// writes its partial sums into parts[m%2].  "AsyncAllReduce(m)" = reduce_norm: it waits for the event
// recorded after module m, folds the partial sums (computed shards, split-K slots, synthetic peers)
// into the fp32 residual x in place (x_m = x_{m-1} + sum), and emits the RMS-normed input of the
// module(s) that read x_m: module m+2 with the ladder wiring, module m+1 with the standard wiring (the
// parallel attention / MLP block: both modules of a layer read the layer's input, lag_of()).
// The event recorded after it is the handle; module m+lag waits on it.  For calls of at most 64 rows
// the two module kinds may run on two streams (or the reduces on a side stream), so that with the
// ladder wiring reduce(m) overlaps module m+1; larger calls run in order on one stream, and with the
// packed weights and one computed shard their reduce is the epilogue of the module's last GEMM
// (fuse_residual).
//
// Fused decode schedule (build_fused_plan / fused_body: bf16, batch <= 16, one computed shard).  A
// decode step is a fixed list of launches of one kernel, each holding up to four independent jobs
// (under the ladder wiring the MLP projections of layer l and the attention side of layer l+1);
// reduce, residual add, RMSNorm, rotary and cache append are epilogues of the projections.
#include <math.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <array>
#include <string>
#include <algorithm>
#include <vector>

#include "../../include/ladder.h"
#include "common.h"
#include "decode_fused.h"

namespace {

std::string g_init_error;

// Scratch of ladder_head_static, the entry point for callers that cannot allocate: normed rows in the storage
// type, then the logits.  One copy per GPU, held until the process ends; its device address is looked up
// once per device (resolve_static_scratch), and host code only ever uses that looked-up pointer.
#define HEAD_STATIC_Y_BYTES ((size_t)LADDER_HEAD_STATIC_MAX_ROWS * LADDER_HEAD_STATIC_MAX_HIDDEN * 4)
#define HEAD_STATIC_LOGIT_BYTES ((size_t)LADDER_HEAD_STATIC_MAX_ROWS * LADDER_HEAD_STATIC_MAX_VOCAB * 4)
static __device__ __align__(256) unsigned char scratch[HEAD_STATIC_Y_BYTES + HEAD_STATIC_LOGIT_BYTES];
#define STATIC_SCRATCH_MAX_DEVICES 64
void* g_scratch_ptr[STATIC_SCRATCH_MAX_DEVICES] = {};

// device address of this GPU's copy of `scratch` (dev must be the current device); null + error on failure
hipError_t resolve_static_scratch(int dev, void** out) {
  *out = nullptr;
  if (dev < 0 || dev >= STATIC_SCRATCH_MAX_DEVICES) return hipErrorInvalidDevice;
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!p) return hipErrorInvalidSymbol;
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return hipSuccess;
}

struct ProfRec {
  int cls;
  hipEvent_t start, stop;
};

struct LayerStore {
  // generic path: raw copies, T [K][N]
  char *wq = nullptr, *wk = nullptr, *wv = nullptr, *wo = nullptr, *wg = nullptr, *wu = nullptr, *wd = nullptr;
  // streaming / MFMA path: packed tiles
  char *pqkv = nullptr, *po = nullptr, *pgu = nullptr, *pd = nullptr;
  char *cache_k = nullptr, *cache_v = nullptr;
  bool loaded = false;
  int kv_B = 0, kv_S = 0;
};

}  // namespace

struct ladder_ctx {
  ladder_config cfg;
  bool bf16 = false, fast = false;
  size_t esz = 4;
  int n_mod = 0, n_peers = 0, s_cap = 0, rows_cap = 0, nqkv = 0;
  // caller's stream (fences only) and the internal streams: s_attn runs the attention modules (and
  // everything else when nothing overlaps), s_mlp the MLP modules, side the reduces
  hipStream_t main = nullptr, s_attn = nullptr, s_mlp = nullptr, side = nullptr;
  hipEvent_t ev_mod[2] = {nullptr, nullptr}, ev_red[2] = {nullptr, nullptr};
  hipEvent_t ev_begin = nullptr, ev_end = nullptr, ev_fork = nullptr;
  int* pos_dev = nullptr;       // device copy of the position, read by the decode kernels
  char* emb_stage = nullptr;    // T [max_batch][H]: decode input staged for the captured graph
  hipGraphExec_t graph_exec = nullptr;
  int graph_batch = 0;
  bool graph_stale = false;     // the captured step no longer matches the context (peers changed)
  std::vector<void*> allocs;
  size_t dev_bytes = 0;
  size_t weight_bytes = 0;      // of dev_bytes: the weight store
  bool dry = false;             // sizing pass: the memory plan is walked, no HIP call is made
  std::vector<LayerStore> store;  // [layer * n_real + shard]
  std::vector<char*> gain_attn, gain_mlp;  // per layer, T [H]
  std::vector<char> gains_loaded;
  float *cos_tab = nullptr, *sin_tab = nullptr;
  const char* peers = nullptr;
  // workspaces
  float* x = nullptr;
  char* y[2] = {nullptr, nullptr};
  // wide calls of the packed-weight path: the residual update is the epilogue of a module's last GEMM, which
  // leaves un-normed bf16 rows in y[] and the rows' 1/rms in y_rs[]; y_scale[i] is y_rs[i] while y[i] holds
  // such rows and null while it holds normed ones
  float* ssq_part = nullptr;
  float* y_rs[2] = {nullptr, nullptr};
  const float* y_scale[2] = {nullptr, nullptr};
  float* parts[2] = {nullptr, nullptr};
  size_t parts_cap = 0;  // elements per parity buffer
  float* qkv = nullptr;
  size_t qkv_cap = 0;
  char *qbuf = nullptr, *obuf = nullptr, *act = nullptr;
  float* gu = nullptr;
  float *att_o = nullptr, *att_ml = nullptr;
  // fused decode path: ring of three residual buffers (x_m lives in ring[m % 3]), arrival tickets, and
  // the launch list of one step
  bool fused = false;
  // (chained step: no buffer is written twice within the one launch of a step, so the ring has a slot per stream,
  // ring_n = 2N + 1, and q and the SwiGLU output have a buffer per layer, n_fbuf = N; else ring_n = 3, n_fbuf = 1)
  int ring_n = 3, n_fbuf = 1;
  std::vector<float*> x_ring;
  // what the projections multiply: x_m times the gain of the reading module's RMSNorm, as a split bf16 matrix
  // [32][H] (decode_fused.h); slot [m % 3][reader & 1] (a stream has at most one odd = attention and one even =
  // MLP reader); and the rows' sums of squares per 16-column tile, [H/16][16]
  std::vector<std::array<bf16_t*, 2>> xop_ring;
  std::vector<float*> ssq_ring;
  StepItem* chain_surplus_dev = nullptr;   // chained step: the launches' surplus lists, FUSED_CLAIM_MAX items per launch
  unsigned* chain_claim_ctr = nullptr;     // their counters (a cache line each, in the range the embedding kernel clears)
  int chain_launch_cap = 0;
  float* ssq_first = nullptr;   // sums of squares of what module 1 reads when its lag is 2 (x_0, or a stage's x_{-1})
  std::vector<bf16_t*> f_q, f_act;   // split q, SwiGLU output: [32][width]
  std::vector<bf16_t*> f_o;          // attention output
  // chained step (decode_fused = 3): persistent workgroups, the step's launch list as per-slot item lists and
  // job tables in device memory, completion words of the producer projections
  bool chain = false;
  int chain_slots = 0, chain_items = 0, chain_lds = 0;
  size_t chain_items_cap = 0;         // items per slot the device array has room for
  int chain_gemv_cap = 0, chain_attn_cap = 0;
  StepItem* chain_items_dev = nullptr;
  GemvJob* chain_gemv_dev = nullptr;
  AttnJob* chain_attn_dev = nullptr;
  // timeline of a chained step (measurement): per slot and item the times of taking, readiness and end, and what
  // the host knows of the item
  struct ChainMeta { int launch, kind, tiles; long long weight_bytes; };
  std::vector<std::vector<ChainMeta>> chain_meta;   // [slot][item]
  unsigned long long* chain_tl_dev = nullptr;
  bool timeline_on = false;
  unsigned* sync_words = nullptr;     // completion words of the projections, [4 N] x FUSED_SYNC_WORDS, behind att_done in one allocation
  int n_zero_words = 0;               // words the embedding kernel clears at the start of a step
  unsigned* err_word = nullptr;   // host-visible word that a kernel raises when its bounded in-launch wait gives up
  unsigned* err_word_dev = nullptr;   // its device address
  int wait_spins = 1 << 20;       // polls of that wait (about a second); a test shortens it
  unsigned wait_bias = 0;         // added to the wait's target (0 in normal operation; a test makes it unreachable)
  unsigned* tk_att = nullptr;     // arrival tickets of split attention, [max_batch][nkv]
  std::vector<FusedArgs> fused_plan;
  // emulated collectives (reduce_delay_us) of the fused schedule: t_done[m] = wall-clock time at which the last
  // workgroup of the residual update that completes stream x_m ended (0 .. 2N)
  unsigned long long* t_done = nullptr;
  int fused_plan_batch = 0;
  int n_cu = 256;                 // compute units of the device (workgroup slots of a fused launch = 2 per CU)
  int wall_khz = 100000;          // rate of the device's wall clock (delay_kernel)
  unsigned* att_done = nullptr;   // fused decode: per layer, completion words (FUSED_SYNC_WORDS) of the attention job: how many (sequence, kv head) outputs are final
  // generation head (ladder_load_head)
  char* head_table = nullptr;     // T [vocab][H]
  char* head_gain = nullptr;      // T [H]
  char* head_w = nullptr;         // plain path: T [H][vocab_local]
  char* head_wp = nullptr;        // streaming path: packed tiles
  char* head_y = nullptr;         // T [max_batch][H] normed rows
  float* head_logits = nullptr;   // f32 [max_batch][vocab_local]
  int vocab = 0, vocab_local = 0;
  bool head_fast = false;
  const char* fused_plan_peers = nullptr;
  int device = 0;                 // the device the context lives on
  void* static_scratch = nullptr; // this device's copy of the file-scope scratch array (ladder_head_static)
  int pos = 0, batch = 0;
  std::string err;
  // profiling
  bool prof = false;
  std::vector<ProfRec> prof_pending;
  std::vector<hipEvent_t> prof_pool;
  long long prof_n[LADDER_K_COUNT] = {};
  double prof_ms[LADDER_K_COUNT] = {};
};

namespace {

// LADDER_DEBUG=1 in the environment: host-side progress lines on stderr
bool debug_on() {
  static const bool on = getenv("LADDER_DEBUG") != nullptr;
  return on;
}
#define DBG(...)                                   \
  do {                                             \
    if (debug_on()) {                              \
      fprintf(stderr, "[ladder] " __VA_ARGS__);    \
      fprintf(stderr, "\n");                       \
      fflush(stderr);                              \
    }                                              \
  } while (0)

int fail(ladder_ctx* c, int code, const std::string& msg) {
  if (c) c->err = msg;
  else g_init_error = msg;
  return code;
}

#define HIP_TRY(c, expr)                                                                        \
  do {                                                                                          \
    hipError_t e_ = (expr);                                                                     \
    if (e_ != hipSuccess)                                                                       \
      return fail((c), LADDER_E_HIP, std::string(#expr) + ": " + hipGetErrorString(e_));        \
  } while (0)

int dev_alloc(ladder_ctx* c, void** p, size_t bytes, bool zero) {
  *p = nullptr;
  if (bytes == 0) bytes = 16;
  if (c->dry) {   // sizing pass (ladder_workspace_bytes): nothing is allocated
    c->dev_bytes += bytes;
    return LADDER_OK;
  }
  HIP_TRY(c, hipMalloc(p, bytes));
  c->allocs.push_back(*p);
  c->dev_bytes += bytes;
  if (zero) HIP_TRY(c, hipMemsetAsync(*p, 0, bytes, c->main));
  return LADDER_OK;
}

// launch bracketed by profiling events when enabled
template <typename F>
hipError_t timed(ladder_ctx* c, int cls, hipStream_t s, F&& f) {
  if (!c->prof) return f();
  hipEvent_t e[2];
  for (int i = 0; i < 2; ++i) {
    if (!c->prof_pool.empty()) {
      e[i] = c->prof_pool.back();
      c->prof_pool.pop_back();
    } else {
      hipError_t r = hipEventCreate(&e[i]);
      if (r != hipSuccess) return r;
    }
  }
  hipError_t r = hipEventRecord(e[0], s);
  if (r != hipSuccess) return r;
  r = f();
  if (r != hipSuccess) return r;
  r = hipEventRecord(e[1], s);
  c->prof_pending.push_back({cls, e[0], e[1]});
  return r;
}

int lag_of(const ladder_ctx* c, int m) {  // module m reads x_{m - lag}
  if (c->cfg.wiring == LADDER_WIRING_STANDARD) return 1;
  if (c->cfg.wiring == LADDER_WIRING_PARALLEL) return (m & 1) ? 1 : 2;   // both modules of a layer read the layer's input
  return (m - 1) / 2 < c->cfg.n_standard_layers ? 1 : 2;
}


int check_config(const ladder_config* g, std::string& why) {
  if (g->n_layers <= 0 || g->hidden <= 0 || g->n_q_heads <= 0 || g->n_kv_heads <= 0 || g->head_dim <= 0 ||
      g->inter <= 0 || g->tp_degree <= 0 || g->n_real_shards <= 0 || g->max_batch <= 0 || g->max_seq <= 0 ||
      g->max_tokens <= 0) {
    why = "sizes must be positive";
    return LADDER_E_ARG;
  }
  if (g->dtype != LADDER_FP32 && g->dtype != LADDER_BF16) { why = "unknown dtype"; return LADDER_E_ARG; }
  if (g->wiring != LADDER_WIRING_LADDER && g->wiring != LADDER_WIRING_STANDARD && g->wiring != LADDER_WIRING_PARALLEL) { why = "unknown wiring"; return LADDER_E_ARG; }
  if (g->kernel_path != LADDER_PATH_AUTO && g->kernel_path != LADDER_PATH_GENERIC) { why = "unknown kernel_path"; return LADDER_E_ARG; }
  if (!(g->rms_eps > 0.f) || !(g->rope_theta > 0.f)) { why = "rms_eps and rope_theta must be positive"; return LADDER_E_ARG; }
  if (g->n_standard_layers < 0 || g->n_standard_layers > g->n_layers) { why = "n_standard_layers out of range"; return LADDER_E_SHAPE; }
  if (g->wiring == LADDER_WIRING_PARALLEL && g->n_standard_layers != 0) { why = "n_standard_layers must be 0 with the parallel wiring"; return LADDER_E_SHAPE; }
  if (g->hidden % 8) { why = "hidden must be a multiple of 8"; return LADDER_E_SHAPE; }
  if (g->n_q_heads % g->n_kv_heads) { why = "n_q_heads must be a multiple of n_kv_heads"; return LADDER_E_SHAPE; }
  if (g->head_dim % 2 || g->head_dim > 256) { why = "head_dim must be even and <= 256"; return LADDER_E_SHAPE; }
  if (g->n_real_shards > g->tp_degree) { why = "n_real_shards exceeds tp_degree"; return LADDER_E_SHAPE; }
  if (g->max_tokens > g->max_seq) { why = "max_tokens exceeds max_seq"; return LADDER_E_SHAPE; }
  if ((g->decode_graph != 0 && g->decode_graph != 1) || (g->overlap_modules != 0 && g->overlap_modules != 1)) { why = "decode_graph / overlap_modules must be 0 or 1"; return LADDER_E_ARG; }
  if (g->decode_fused < 0 || g->decode_fused > 3) { why = "decode_fused must be 0, 1, 2 or 3"; return LADDER_E_ARG; }
  if (g->reduce_delay_us < 0 || g->reduce_delay_us > 10000) { why = "reduce_delay_us must be in 0 .. 10000"; return LADDER_E_ARG; }
  if (g->peer_pool < 0 || g->peer_rows < 0) { why = "peer_pool / peer_rows negative"; return LADDER_E_ARG; }
  if (g->tp_degree > g->n_real_shards && g->peer_pool > 0 && g->peer_rows <= 0) { why = "peer_rows must be positive when peers are used"; return LADDER_E_SHAPE; }
  if ((long long)g->max_batch * g->max_tokens > (1ll << 24)) { why = "max_batch * max_tokens too large"; return LADDER_E_SHAPE; }
  return LADDER_OK;
}

bool fast_shapes_ok(const ladder_config* g) {
  const int gq = g->n_q_heads / g->n_kv_heads;
  return g->dtype == LADDER_BF16 && g->hidden % 32 == 0 && (g->n_q_heads * g->head_dim) % 32 == 0 &&
         g->inter % 32 == 0 && (g->head_dim == 64 || g->head_dim == 128) &&
         (gq == 1 || gq == 2 || gq == 4 || gq == 8) && g->max_seq <= 65536;
}

int collect_profile(ladder_ctx* c) {
  if (c->prof_pending.empty()) return LADDER_OK;
  HIP_TRY(c, hipStreamSynchronize(c->main));
  HIP_TRY(c, hipStreamSynchronize(c->s_attn));
  HIP_TRY(c, hipStreamSynchronize(c->s_mlp));
  HIP_TRY(c, hipStreamSynchronize(c->side));
  for (auto& r : c->prof_pending) {
    float ms = 0.f;
    HIP_TRY(c, hipEventElapsedTime(&ms, r.start, r.stop));
    c->prof_n[r.cls] += 1;
    c->prof_ms[r.cls] += ms;
    c->prof_pool.push_back(r.start);
    c->prof_pool.push_back(r.stop);
  }
  c->prof_pending.clear();
  return LADDER_OK;
}

// consumers of x_m: module m+1 if its lag is 1 (m == 0: module 1 always), module m+2 if its lag is 2
// (m == 0: module 2 always -- modules 1 and 2 both read x_0)
int consumers_of(const ladder_ctx* c, int m, int out[2]) {
  int nc = 0;
  if (m + 1 <= c->n_mod && (m == 0 || lag_of(c, m + 1) == 1)) out[nc++] = m + 1;
  if (m + 2 <= c->n_mod && ((m == 0 && lag_of(c, 2) == 2) || (m > 0 && lag_of(c, m + 2) == 2))) out[nc++] = m + 2;
  return nc;
}

// Wide calls (more than 64 rows) of the packed-weight path with one real shard: the residual update of module m
// (Algorithm 1: the module's reduced output joins the stream; the AllReduce as a sum over rank partial sums, Eq. 2) is the
// epilogue of the module's last GEMM instead of a kernel of its own, which saves a round trip of the fp32
// product through memory.  The epilogue leaves the new rows, times the reading module's gain, as bf16 for the
// modules that read x_m; their 1/rms (from the sums of squares the epilogue also leaves) scales the consumer's
// product instead (the factor commutes with the product).
int fuse_residual(ladder_ctx* c, GemmArgs& a, int m, float* x_copy, int cons[2]) {
  const ladder_config& g = c->cfg;
  a.epilogue = 3; a.x_res = c->x; a.x_copy = x_copy;
  if (c->peers && c->n_peers > 0) {
    const size_t set = (size_t)(m % g.peer_pool);
    a.peers = (const bf16_t*)(c->peers + set * c->n_peers * (size_t)g.peer_rows * g.hidden * c->esz);
    a.n_peers = c->n_peers; a.peer_stride = (size_t)g.peer_rows * g.hidden;
  }
  const int nc = consumers_of(c, m, cons);
  auto gain_of = [&](int cm) { return (const bf16_t*)((cm & 1) ? c->gain_attn[(cm - 1) / 2] : c->gain_mlp[(cm - 1) / 2]); };
  if (nc > 0) { a.xh_a = (bf16_t*)c->y[cons[0] & 1]; a.gain_a = gain_of(cons[0]); a.ssq_part = c->ssq_part; }
  if (nc > 1) { a.xh_b = (bf16_t*)c->y[cons[1] & 1]; a.gain_b = gain_of(cons[1]); }
  return nc;
}

int finish_residual(ladder_ctx* c, const GemmArgs& a, int rows, int nc, const int cons[2], hipStream_t s) {
  if (nc == 0) return LADDER_OK;
  const ladder_config& g = c->cfg;
  float* ra = c->y_rs[cons[0] & 1];
  float* rb = nc > 1 ? c->y_rs[cons[1] & 1] : nullptr;
  HIP_TRY(c, timed(c, LADDER_K_REDUCE_NORM, s, [&] { return launch_row_rms(c->ssq_part, gemm_ssq_parts(a), rows, g.hidden, g.rms_eps, ra, rb, s); }));
  c->y_scale[cons[0] & 1] = ra;
  if (nc > 1) c->y_scale[cons[1] & 1] = rb;
  return LADDER_OK;
}

// ---------------------------------------------------------------------------------------------
// one module's compute on the main stream; writes parts[m%2] and returns the number of slots written, or (fuse)
// updates the residual itself and returns -1 slots: then no reduce follows
// ---------------------------------------------------------------------------------------------
int run_module(ladder_ctx* c, int m, int B, int T, int pos0, hipStream_t s, int* n_slots, bool fuse, float* x_copy) {
  const ladder_config& g = c->cfg;
  const int rows = B * T, H = g.hidden, d = g.head_dim, nq = g.n_q_heads, nkv = g.n_kv_heads, I = g.inter;
  const int layer = (m - 1) / 2, par = m & 1;
  const bool is_attn = (m & 1) == 1;
  const char* yin = c->y[par];
  float* pout = c->parts[par];
  const size_t pstride = (size_t)rows * H;
  const bool skinny = rows <= 64;
  const bool dev_pos = c->fast && T == 1;  // decode kernels of the bf16 path read the position from device memory
  int slots = 0;
  for (int r = 0; r < g.n_real_shards; ++r) {
    LayerStore& L = c->store[(size_t)layer * g.n_real_shards + r];
    if (is_attn) {
      int qkv_slots = 1;
      if (!c->fast) {
        const int nqd = nq * d, nkd = nkv * d;
        HIP_TRY(c, timed(c, LADDER_K_GENERIC, s, [&] { return launch_gemm_generic(yin, L.wq, c->qkv, rows, nqd, H, c->nqkv, 0, c->bf16, s); }));
        HIP_TRY(c, timed(c, LADDER_K_GENERIC, s, [&] { return launch_gemm_generic(yin, L.wk, c->qkv, rows, nkd, H, c->nqkv, nqd, c->bf16, s); }));
        HIP_TRY(c, timed(c, LADDER_K_GENERIC, s, [&] { return launch_gemm_generic(yin, L.wv, c->qkv, rows, nkd, H, c->nqkv, nqd + nkd, c->bf16, s); }));
      } else if (skinny) {
        GemvArgs a{};
        a.x = (const bf16_t*)yin; a.ldx = H; a.wp = L.pqkv; a.M = rows; a.K = H; a.N = c->nqkv;
        a.ksplit = gemv_plan(rows, c->nqkv, H, true).ksplit;
        a.out = c->qkv; a.out_stride = (size_t)rows * c->nqkv; a.slot0 = 0; a.epilogue = 0;
        qkv_slots = a.ksplit;
        HIP_TRY(c, timed(c, LADDER_K_GEMV, s, [&] { return launch_gemv(a, s); }));
      } else {
        GemmArgs a{};
        a.x = (const bf16_t*)yin; a.ldx = H; a.wp = L.pqkv; a.M = rows; a.K = H; a.N = c->nqkv; a.row_scale = c->y_scale[par];
        if (!dev_pos) {
          // rotary embedding and cache append are the GEMM's epilogue (no fp32 q|k|v round trip through memory)
          a.epilogue = 2; a.q_out = (bf16_t*)c->qbuf; a.cache_k = (bf16_t*)L.cache_k; a.cache_v = (bf16_t*)L.cache_v;
          a.cos_tab = c->cos_tab; a.sin_tab = c->sin_tab; a.T = T; a.pos0 = pos0; a.nq = nq; a.nkv = nkv; a.d = d; a.max_seq = c->s_cap;
          qkv_slots = 0;
        } else {   // (a decode step of more than 64 sequences: the position lives in device memory)
          a.out = c->qkv; a.epilogue = 0;
        }
        HIP_TRY(c, timed(c, LADDER_K_GEMM, s, [&] { return launch_gemm_mfma(a, s); }));
      }
      RopeAppendArgs ra{};
      ra.qkv = c->qkv; ra.n_parts = qkv_slots; ra.part_stride = (size_t)rows * c->nqkv;
      ra.q_out = c->qbuf; ra.cache_k = L.cache_k; ra.cache_v = L.cache_v;
      ra.cos_tab = c->cos_tab; ra.sin_tab = c->sin_tab;
      ra.B = B; ra.T = T; ra.pos0 = pos0; ra.nq = nq; ra.nkv = nkv; ra.d = d; ra.max_seq = c->s_cap; ra.pos_dev = dev_pos ? c->pos_dev : nullptr;
      if (qkv_slots > 0) HIP_TRY(c, timed(c, LADDER_K_ROPE_APPEND, s, [&] { return launch_rope_append(ra, c->bf16, s); }));
      if (!c->fast) {
        AttnGenericArgs aa{c->qbuf, L.cache_k, L.cache_v, c->obuf, B, T, pos0, nq, nkv, d, c->s_cap};
        HIP_TRY(c, timed(c, LADDER_K_GENERIC, s, [&] { return launch_attn_generic(aa, c->bf16, s); }));
      } else if (T == 1) {
        AttnDecodeArgs aa{};
        aa.q = (const bf16_t*)c->qbuf; aa.cache_k = (const bf16_t*)L.cache_k; aa.cache_v = (const bf16_t*)L.cache_v;
        aa.part_o = c->att_o; aa.part_ml = c->att_ml; aa.o = (bf16_t*)c->obuf;
        aa.B = B; aa.nq = nq; aa.nkv = nkv; aa.d = d; aa.max_seq = c->s_cap; aa.n_pos = pos0 + 1;
        // launch shape fixed by the cache capacity (not the current position) so that a captured step
        // stays valid as the sequence grows; workgroups past the visible range exit at once
        int chunk = 32;
        for (int cand : {128, 64}) {
          if ((long long)B * nkv * ((g.max_seq + cand - 1) / cand) >= 256) { chunk = cand; break; }
        }
        while (chunk < 128 && (g.max_seq + chunk - 1) / chunk > 512) chunk *= 2;  // combine holds <= 512 chunk weights
        aa.chunk = chunk; aa.n_chunks = (g.max_seq + chunk - 1) / chunk; aa.pos_dev = c->pos_dev;
        HIP_TRY(c, timed(c, LADDER_K_ATTN_DECODE, s, [&] { return launch_attn_decode(aa, s); }));
      } else {
        AttnPrefillArgs aa{(const bf16_t*)c->qbuf, (const bf16_t*)L.cache_k, (const bf16_t*)L.cache_v,
                           (bf16_t*)c->obuf, B, T, pos0, nq, nkv, d, c->s_cap};
        HIP_TRY(c, timed(c, LADDER_K_ATTN_PREFILL, s, [&] { return launch_attn_prefill(aa, s); }));
      }
      const int nqd = nq * d;
      if (!c->fast) {
        HIP_TRY(c, timed(c, LADDER_K_GENERIC, s, [&] { return launch_gemm_generic(c->obuf, L.wo, pout + slots * pstride, rows, H, nqd, H, 0, c->bf16, s); }));
        slots += 1;
      } else if (skinny) {
        GemvArgs a{};
        a.x = (const bf16_t*)c->obuf; a.ldx = nqd; a.wp = L.po; a.M = rows; a.K = nqd; a.N = H;
        a.ksplit = gemv_plan(rows, H, nqd, true).ksplit;
        a.out = pout; a.out_stride = pstride; a.slot0 = slots; a.epilogue = 0;
        HIP_TRY(c, timed(c, LADDER_K_GEMV, s, [&] { return launch_gemv(a, s); }));
        slots += a.ksplit;
      } else {
        GemmArgs a{};
        a.x = (const bf16_t*)c->obuf; a.ldx = nqd; a.wp = L.po; a.M = rows; a.K = nqd; a.N = H; a.out = pout + slots * pstride; a.epilogue = 0;
        int cons[2], nc = 0;
        if (fuse) nc = fuse_residual(c, a, m, x_copy, cons);
        HIP_TRY(c, timed(c, LADDER_K_GEMM, s, [&] { return launch_gemm_mfma(a, s); }));
        if (fuse) { const int rc = finish_residual(c, a, rows, nc, cons, s); if (rc) return rc; }
        slots += 1;
      }
    } else {
      if (!c->fast) {
        HIP_TRY(c, timed(c, LADDER_K_GENERIC, s, [&] { return launch_gemm_generic(yin, L.wg, c->gu, rows, I, H, 2 * I, 0, c->bf16, s); }));
        HIP_TRY(c, timed(c, LADDER_K_GENERIC, s, [&] { return launch_gemm_generic(yin, L.wu, c->gu, rows, I, H, 2 * I, I, c->bf16, s); }));
        HIP_TRY(c, timed(c, LADDER_K_GENERIC, s, [&] { return launch_swiglu(c->gu, c->act, rows, I, c->bf16, s); }));
        HIP_TRY(c, timed(c, LADDER_K_GENERIC, s, [&] { return launch_gemm_generic(c->act, L.wd, pout + slots * pstride, rows, H, I, H, 0, c->bf16, s); }));
        slots += 1;
      } else if (skinny) {
        GemvArgs a{};
        a.x = (const bf16_t*)yin; a.ldx = H; a.wp = L.pgu; a.M = rows; a.K = H; a.N = 2 * I; a.ksplit = 1;
        a.act = (bf16_t*)c->act; a.epilogue = 1;
        HIP_TRY(c, timed(c, LADDER_K_GEMV, s, [&] { return launch_gemv(a, s); }));
        GemvArgs b{};
        b.x = (const bf16_t*)c->act; b.ldx = I; b.wp = L.pd; b.M = rows; b.K = I; b.N = H;
        b.ksplit = gemv_plan(rows, H, I, true).ksplit;
        b.out = pout; b.out_stride = pstride; b.slot0 = slots; b.epilogue = 0;
        HIP_TRY(c, timed(c, LADDER_K_GEMV, s, [&] { return launch_gemv(b, s); }));
        slots += b.ksplit;
      } else {
        GemmArgs a{};
        a.x = (const bf16_t*)yin; a.ldx = H; a.wp = L.pgu; a.M = rows; a.K = H; a.N = 2 * I; a.act = (bf16_t*)c->act; a.epilogue = 1;
        a.row_scale = c->y_scale[par];
        HIP_TRY(c, timed(c, LADDER_K_GEMM, s, [&] { return launch_gemm_mfma(a, s); }));
        GemmArgs b{};
        b.x = (const bf16_t*)c->act; b.ldx = I; b.wp = L.pd; b.M = rows; b.K = I; b.N = H; b.out = pout + slots * pstride; b.epilogue = 0;
        int cons[2], nc = 0;
        if (fuse) nc = fuse_residual(c, b, m, x_copy, cons);
        HIP_TRY(c, timed(c, LADDER_K_GEMM, s, [&] { return launch_gemm_mfma(b, s); }));
        if (fuse) { const int rc = finish_residual(c, b, rows, nc, cons, s); if (rc) return rc; }
        slots += 1;
      }
    }
  }
  *n_slots = fuse ? -1 : slots;
  return LADDER_OK;
}

// reduce(m): x += partial sums of module m (+ peers); emit the normed inputs of the modules that read x_m.
// m == 0: x = emb, emit inputs of the modules that read x_0.
// Timed wait standing in for the latency of a collective: one wavefront polls the constant-rate wall
// clock until `ticks` have passed.  Bounded: it also leaves after a fixed number of polls (each poll
// sleeps ~0.2 us, 2^20 polls ~ 0.2 s), so the kernel ends whatever the clock does.
__global__ __launch_bounds__(64) void delay_kernel(unsigned long long ticks) {
  const unsigned long long t0 = wall_clock64();
  for (int i = 0; i < (1 << 20); ++i) {
    if (wall_clock64() - t0 >= ticks) break;
    __builtin_amdgcn_s_sleep(8);
  }
}

// Same, until `ticks` after the time *t0 (left by an earlier kernel of the stream): the end of an emulated
// collective whose start another kernel has recorded.
__global__ __launch_bounds__(64) void wait_until_kernel(const unsigned long long* t0, unsigned long long ticks) {
  const unsigned long long t1 = *t0 + ticks;
  for (int i = 0; i < (1 << 20); ++i) {
    if (wall_clock64() >= t1) break;
    __builtin_amdgcn_s_sleep(8);
  }
}

// What a pipeline stage takes from the stage before it and hands to the next one (section "Compatibility with other
// Parallelism Techniques"): the stream without the last two module outputs, and those two outputs, fp32 [rows][H].
struct StageIo {
  const float *res, *att, *mlp;     // in (att, mlp: null = zeros)
  float *r_out, *a_out, *m_out;     // out
};

// r = x_{2N-2}, a = x_{2N-1} - x_{2N-2}, m = x_{2N} - x_{2N-1}, element by element (the inputs may be the outputs:
// every thread reads its element of all three before it writes)
__global__ __launch_bounds__(256) void stage_out_kernel(const float4* x2, const float4* x1, const float4* x0,
                                                        float4* r, float4* a, float4* m, size_t n4) {
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n4; i += (size_t)gridDim.x * 256) {
    const float4 v2 = x2[i], v1 = x1[i], v0 = x0[i];
    r[i] = v2;
    a[i] = make_float4(v1.x - v2.x, v1.y - v2.y, v1.z - v2.z, v1.w - v2.w);
    m[i] = make_float4(v0.x - v1.x, v0.y - v1.y, v0.z - v1.z, v0.w - v1.w);
  }
}
int launch_stage_out(ladder_ctx* c, const float* x2, const float* x1, const float* x0, const StageIo& st, int rows, hipStream_t s) {
  const size_t n4 = (size_t)rows * c->cfg.hidden / 4;   // (hidden is a multiple of 4: checked at init for every path)
  const unsigned grid = (unsigned)std::min<size_t>((n4 + 255) / 256, 4096);
  HIP_TRY(c, timed(c, LADDER_K_OTHER, s, [&] {
    hipLaunchKernelGGL(stage_out_kernel, dim3(grid), dim3(256), 0, s, (const float4*)x2, (const float4*)x1, (const float4*)x0,
                       (float4*)st.r_out, (float4*)st.a_out, (float4*)st.m_out, n4);
    return hipGetLastError();
  }));
  return LADDER_OK;
}

// the start of a stage that is handed three tensors: x_{-1} = res + att (module 1 reads it), x_0 = x_{-1} + mlp (the
// stream; module 2 reads it); ladder wiring in both modules
int run_stage_in(ladder_ctx* c, const StageIo& st, int rows, hipStream_t s) {
  const ladder_config& g = c->cfg;
  HIP_TRY(c, hipMemcpyAsync(c->x, st.res, (size_t)rows * g.hidden * 4, hipMemcpyDeviceToDevice, s));
  for (int cm = 1; cm <= 2; ++cm) {
    ReduceNormArgs a{};
    a.x = c->x; a.rows = rows; a.H = g.hidden; a.eps = g.rms_eps;
    a.parts = cm == 1 ? st.att : st.mlp; a.n_parts = a.parts ? 1 : 0; a.part_stride = (size_t)rows * g.hidden;
    a.out_a = c->y[cm & 1];
    a.gain_a = cm == 1 ? (const void*)c->gain_attn[0] : (const void*)c->gain_mlp[0];
    c->y_scale[cm & 1] = nullptr;   // normed rows
    HIP_TRY(c, timed(c, LADDER_K_REDUCE_NORM, s, [&] { return launch_reduce_norm(a, c->bf16, s); }));
  }
  return LADDER_OK;
}

int run_reduce(ladder_ctx* c, int m, int rows, int n_slots, const void* emb, float* x_out, hipStream_t s) {
  const ladder_config& g = c->cfg;
  ReduceNormArgs a{};
  a.x = c->x; a.emb = emb; a.rows = rows; a.H = g.hidden; a.eps = g.rms_eps;
  if (m > 0) {
    a.parts = c->parts[m & 1]; a.n_parts = n_slots; a.part_stride = (size_t)rows * g.hidden;
    if (c->peers && c->n_peers > 0) {
      const size_t set = (size_t)(m % g.peer_pool);
      a.peers = c->peers + set * c->n_peers * (size_t)g.peer_rows * g.hidden * c->esz;
      a.n_peers = c->n_peers; a.peer_stride = (size_t)g.peer_rows * g.hidden;
    }
  }
  int consumers[2];
  const int nc = consumers_of(c, m, consumers);
  for (int i = 0; i < nc; ++i) {
    const int cm = consumers[i], layer = (cm - 1) / 2;
    void* out = c->y[cm & 1];
    c->y_scale[cm & 1] = nullptr;   // normed rows
    const void* gain = (cm & 1) ? (const void*)c->gain_attn[layer] : (const void*)c->gain_mlp[layer];
    if (i == 0) { a.out_a = out; a.gain_a = gain; }
    else { a.out_b = out; a.gain_b = gain; }
  }
  a.x_out = x_out;
  // (the parallel block sums the partial sums of both modules of a layer before its one collective: the
  // attention module's reduce stands for the local addition, the MLP module's for the collective)
  const bool local_only = g.wiring == LADDER_WIRING_PARALLEL && (m & 1);
  if (m > 0 && g.reduce_delay_us > 0 && !local_only) {   // the emulated collective takes this long before its result is there
    const unsigned long long ticks = (unsigned long long)g.reduce_delay_us * (unsigned long long)c->wall_khz / 1000ull;
    HIP_TRY(c, timed(c, LADDER_K_OTHER, s, [&] {
      hipLaunchKernelGGL(delay_kernel, dim3(1), dim3(64), 0, s, ticks);
      return hipGetLastError();
    }));
  }
  HIP_TRY(c, timed(c, LADDER_K_REDUCE_NORM, s, [&] { return launch_reduce_norm(a, c->bf16, s); }));
  return LADDER_OK;
}

// the 2N modules and their reduces on the internal streams; does not touch the caller's stream.
// Stream plan:
//   overlap_modules: odd (attention) modules and their reduces on s_attn, even (MLP) modules and their
//     reduces on s_mlp.  Under the ladder wiring module m+1 needs only x_{m-1}, so it executes while
//     module m and reduce(m) still run on the other stream; reduce(m) waits for reduce(m-1) (the
//     residual is updated in place, in module order) through an event.
//   else reduce_on_side_stream: all modules on s_attn, all reduces on the side stream.
//   else (and for every call with more than 64 rows): everything in order on s_attn.
int forward_body(ladder_ctx* c, const void* x_in, int B, int T, int pos0, void* x_out, const StageIo* st = nullptr) {
  const int rows = B * T;
  // calls with more than 64 rows (prefill) run in order on one stream: each of their kernels fills the
  // chip, and the same work measured 4 % (reduce on the side stream) to 16 % (two module streams) slower
  // when spread over streams
  // (and so does a pipeline stage's call: its hand-over reads the stream between the last modules)
  const bool small = rows <= 64 && !st;
  const bool overlap = small && c->cfg.overlap_modules != 0;
  const bool side = small && !overlap && c->cfg.reduce_on_side_stream != 0;
  hipStream_t s0 = c->s_attn;
  auto module_stream = [&](int m) { return (overlap && (m & 1) == 0) ? c->s_mlp : s0; };
  auto reduce_stream = [&](int m) { return m == 0 ? s0 : (overlap ? module_stream(m) : (side ? c->side : s0)); };
  // (the skinny kernels have no such epilogue, several real shards would each add to the residual, and the
  // emulated collective latency wants the reduce as a step of its own)
  const bool fuse = c->fast && rows > 64 && c->cfg.n_real_shards == 1 && c->cfg.reduce_delay_us == 0;
  int rc = st ? run_stage_in(c, *st, rows, s0) : run_reduce(c, 0, rows, 0, x_in, c->n_mod == 0 ? (float*)x_out : nullptr, s0);
  if (rc) return rc;
  const size_t x_bytes = (size_t)rows * c->cfg.hidden * 4;
  if (overlap && c->n_mod >= 2) {  // fork: the MLP stream starts once x_0 and its normed copies exist
    HIP_TRY(c, hipEventRecord(c->ev_fork, s0));
    HIP_TRY(c, hipStreamWaitEvent(c->s_mlp, c->ev_fork, 0));
  }
  for (int m = 1; m <= c->n_mod; ++m) {
    DBG("module %d", m);
    hipStream_t sm = module_stream(m), rs = reduce_stream(m);
    const int src = m - lag_of(c, m);
    if (src >= 1 && reduce_stream(src) != sm) HIP_TRY(c, hipStreamWaitEvent(sm, c->ev_red[src & 1], 0));
    int n_slots = 0;
    // (a stage's hand-over: the stream as it is before the last attention module's output joins it ...)
    if (st && m == c->n_mod - 1) HIP_TRY(c, hipMemcpyAsync(st->r_out, c->x, x_bytes, hipMemcpyDeviceToDevice, s0));
    rc = run_module(c, m, B, T, pos0, sm, &n_slots, fuse, m == c->n_mod ? (float*)x_out : nullptr);
    if (rc) return rc;
    if (n_slots >= 0) {   // (else the module has updated the residual itself: wide calls run on one stream)
      if (rs != sm) {
        HIP_TRY(c, hipEventRecord(c->ev_mod[m & 1], sm));
        HIP_TRY(c, hipStreamWaitEvent(rs, c->ev_mod[m & 1], 0));
      }
      if (m >= 2 && reduce_stream(m - 1) != rs) HIP_TRY(c, hipStreamWaitEvent(rs, c->ev_red[(m - 1) & 1], 0));
      rc = run_reduce(c, m, rows, n_slots, nullptr, m == c->n_mod ? (float*)x_out : nullptr, rs);
      if (rc) return rc;
      if (overlap || side) HIP_TRY(c, hipEventRecord(c->ev_red[m & 1], rs));
    }
    // (... and after it has; the two outputs are the differences of consecutive streams)
    if (st && m == c->n_mod - 1) HIP_TRY(c, hipMemcpyAsync(st->a_out, c->x, x_bytes, hipMemcpyDeviceToDevice, s0));
    if (st && m == c->n_mod) {
      rc = launch_stage_out(c, st->r_out, st->a_out, c->x, *st, rows, s0);
      if (rc) return rc;
    }
  }
  // join: the last reduce is after every module and every earlier reduce
  if (c->n_mod >= 1 && reduce_stream(c->n_mod) != s0) HIP_TRY(c, hipStreamWaitEvent(s0, c->ev_red[c->n_mod & 1], 0));
  return LADDER_OK;
}

// plain grid-stride copy, 16 bytes per thread and pass: the known-size dispatch that HBM counters are scaled by
__global__ __launch_bounds__(256) void calibration_copy_kernel(const uint4* __restrict__ src, uint4* __restrict__ dst, size_t n16) {
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += (size_t)gridDim.x * 256) dst[i] = src[i];
}

__global__ void set_pos_kernel(int* p, int v) { *p = v; }
__global__ void inc_pos_kernel(int* p) { *p += 1; }

// ---------------------------------------------------------------------------------------------
// fused decode path: the launch list of one step (see decode_fused.hip)
// ---------------------------------------------------------------------------------------------
bool fused_usable(const ladder_ctx* c) {
  const ladder_config& g = c->cfg;
  return c->fast && g.decode_fused != 0 && g.n_real_shards == 1 && g.max_batch <= 16 && g.max_seq <= 65536 &&
         g.hidden % 32 == 0;
}

void build_fused_plan(ladder_ctx* c, int B) {
  const ladder_config& g = c->cfg;
  const int H = g.hidden, d = g.head_dim, nq = g.n_q_heads, nkv = g.n_kv_heads, I = g.inter, N = g.n_layers;
  const int nqd = nq * d;
  // attention: a (sequence, kv head) is cut into splits of positions (multiples of 64) that meet through
  // an arrival ticket when there is more than one.  A split of 256 positions is one 32-key block per
  // wavefront, i.e. one memory round trip; splits grow beyond that only when there would be more
  // attention workgroups than CUs.
  int n_splits = std::min((g.max_seq + 255) / 256, std::max(1, c->n_cu / (B * nkv)));
  n_splits = std::max(1, std::min(n_splits, (g.max_seq + 63) / 64));

  const int split_len = ((g.max_seq + n_splits - 1) / n_splits + 63) / 64 * 64;
  n_splits = (g.max_seq + split_len - 1) / split_len;
  auto layer = [&](int l) -> LayerStore& { return c->store[(size_t)(l - 1)]; };  // l = 1..N (one shard)
  auto R = [&](int m) { return (size_t)(m % c->ring_n); };            // ring slot of stream x_m
  auto F = [&](int l) { return (size_t)((l - 1) % c->n_fbuf); };      // q / SwiGLU buffer of layer l

  auto job_qkv = [&](int l, int src) {
    GemvJob j{};
    j.xb = c->xop_ring[R(src)][1]; j.ldx = H; j.normed = 1; j.eps = g.rms_eps; j.ssq = c->ssq_ring[R(src)];
    j.reads_stream = src;
    if (l == 1 && lag_of(c, 1) == 2) j.ssq = c->ssq_first;   // (x_{-1}: x_0 itself unless a pipeline stage hands over)
    j.wp = layer(l).pqkv; j.M = B; j.K = H; j.N = c->nqkv;
    j.n_groups = c->nqkv / 16; j.epi = EPI_QKV_ROPE;
    j.q_out = c->f_q[F(l)];
    j.cache_k = (bf16_t*)layer(l).cache_k; j.cache_v = (bf16_t*)layer(l).cache_v;
    j.cos_tab = c->cos_tab; j.sin_tab = c->sin_tab; j.pos_dev = c->pos_dev;
    j.nq = nq; j.nkv = nkv; j.d = d; j.max_seq = c->s_cap;
    // short K range: two tiles per workgroup (8B shape, batch 4: 2.90 -> 2.81 ms per step; 1.2B: 0.86 -> 0.83);
    // over hidden 8192 one tile is already 256 KiB and two were slower
    if (H <= 4096 && j.n_groups % 2 == 0) { j.tn = 2; j.n_groups /= 2; }
    return j;
  };
  // the job adds the output (and peers) of module m to ring slot at - 1 and leaves the sum in slot at (at = m
  // unless the two modules of a layer are added in the other order)
  auto residual = [&](GemvJob& j, int m, int at) {
    j.N = H; j.n_groups = H / 16; j.epi = EPI_RESIDUAL;
    j.x_old = c->x_ring[R(at - 1)]; j.x_new = c->x_ring[R(at)];
    // the modules that read what this job leaves in slot `at` (x_at; under the parallel wiring the odd slots hold
    // an intermediate sum that nobody reads): each gets its operand, the new rows times its norm's gain
    int cons[2];
    const int nc = consumers_of(c, at, cons);
    for (int i = 0; i < nc; ++i) {
      const int cm = cons[i], cl = (cm - 1) / 2;
      if (cm & 1) { j.xop_a = c->xop_ring[R(at)][1]; j.gain_a = (const bf16_t*)c->gain_attn[cl]; }
      else { j.xop_b = c->xop_ring[R(at)][0]; j.gain_b = (const bf16_t*)c->gain_mlp[cl]; }
    }
    if (nc > 0) j.ssq_new = c->ssq_ring[R(at)];
    // a collective ends every module (x_at is then complete); the parallel block has one per layer, after the
    // second of its two local additions (the odd slots hold the intermediate sum)
    if (g.wiring != LADDER_WIRING_PARALLEL || (at & 1) == 0) j.completes_stream = at;
    if (c->peers && c->n_peers > 0) {
      j.peers = (const bf16_t*)c->peers + (size_t)(m % g.peer_pool) * c->n_peers * (size_t)g.peer_rows * H;
      j.n_peers = c->n_peers; j.peer_stride = (size_t)g.peer_rows * H;
    }
  };
  auto job_o = [&](int l, int m, int at = -1) {
    GemvJob j{};
    j.xb = c->f_o[F(l)]; j.ldx = nqd; j.wp = layer(l).po; j.M = B; j.K = nqd; j.after_attention = 1;
    residual(j, m, at < 0 ? m : at);
    // its K range is short: two tiles per workgroup halve the number of (latency-bound) workgroups
    if (j.n_groups % 2 == 0) { j.tn = 2; j.n_groups /= 2; }
    return j;
  };
  auto job_gu = [&](int l, int src) {
    GemvJob j{};
    j.xb = c->xop_ring[R(src)][0]; j.ldx = H; j.normed = 1; j.eps = g.rms_eps; j.ssq = c->ssq_ring[R(src)];
    j.reads_stream = src;
    j.wp = layer(l).pgu; j.M = B; j.K = H; j.N = 2 * I;
    j.n_groups = 2 * I / 16; j.epi = EPI_SWIGLU; j.act = c->f_act[F(l)];
    // every workgroup reads the batch's rows of x over its whole K range (from L2): at 13 rows and more that
    // traffic is worth halving with two tiles per workgroup (70B shard, batch 14 / 16: 5.42 -> 5.09 / 5.80 -> 5.31
    // ms per step; batch 12 and less: slower; for QKV and down: slower at every batch)
    // (and when the K range is short, a tile of it is too little work for a workgroup: 1.2B shape 0.89 -> 0.86 ms)
    // (and when pairs of tiles fit the chip in one round, one workgroup per CU, instead of two rounds of single
    // tiles: 70B shard at R = 8, batch 4: 3.51 -> 3.41 ms)
    // (measured: batch 1 - 6 faster, 7 - 12 slower)
    if ((B >= 13 || H <= 2048 || (j.n_groups / 2 <= c->n_cu && B <= 6)) && j.n_groups % 2 == 0) { j.tn = 2; j.n_groups /= 2; }
    // (13 rows and more, and more pairs than the chip holds workgroups: four tiles per workgroup halve the operand
    // traffic once more.  Where the pairs fit, quadruples leave CUs without a workgroup: 70B R = 4 shard at batch 16,
    // 448 pairs against 224 quadruples: chained step 8.36 against 10.30 ms, separate launches 9.15 against 9.17; 8B
    // shape at batch 16, 896 pairs against 448 quadruples: 3.91 against 3.88 and 4.06 against 4.00)
    if (B >= 13 && j.tn == 2 && j.n_groups % 2 == 0 && j.n_groups > 2 * c->n_cu) { j.tn = 4; j.n_groups /= 2; }
    return j;
  };
  auto job_dn = [&](int l, int m, int at = -1) {
    GemvJob j{};
    j.xb = c->f_act[F(l)]; j.ldx = I; j.wp = layer(l).pd; j.M = B; j.K = I;
    residual(j, m, at < 0 ? m : at);
    return j;
  };
  auto job_att = [&](int l) {
    AttnJob a{};
    a.q = c->f_q[F(l)]; a.cache_k = (const bf16_t*)layer(l).cache_k; a.cache_v = (const bf16_t*)layer(l).cache_v;
    if (c->chain) a.done = c->att_done + (size_t)(l - 1) * FUSED_SYNC_WORDS;   // (every attention job of a chained step is a producer)
    a.part_o = c->att_o; a.part_ml = c->att_ml; a.o = c->f_o[F(l)]; a.tickets = c->tk_att;
    a.B = B; a.nq = nq; a.nkv = nkv; a.max_seq = c->s_cap; a.n_splits = n_splits; a.split_len = split_len;
    a.pos_dev = c->pos_dev;
    return a;
  };
  auto blocks_of = [&](const GemvJob& j) { return j.n_groups; };
  auto lds_of = [&](const GemvJob&) { return (int)fused_gemv_lds_bytes(); };
  // Jobs side by side in one launch, in dispatch order.  Workgroups are dispatched in block order and a
  // CU holds two of them: the job whose workgroups run longest (whole-K streams over hidden) goes first
  // so that each lands on a CU of its own, and the short ones fill the second slots.
  auto several = [&](std::initializer_list<GemvJob> jobs) {
    FusedArgs f{};
    int i = 0, total = 0;
    for (const GemvJob& j : jobs) {
      if (blocks_of(j) <= 0) continue;
      f.kind[i] = JOB_GEMV; f.g[i] = j; total += blocks_of(j); f.block_end[i] = total;
      f.lds_bytes = std::max(f.lds_bytes, lds_of(j));
      ++i;
    }
    f.n_jobs = i;
    for (; i < FUSED_MAX_JOBS; ++i) f.block_end[i] = total;   // unused job slots: no block index reaches them
    return f;
  };
  auto one = [&](const GemvJob& j) { return several({j}); };
  auto two = [&](const GemvJob& first, const GemvJob& second) { return several({first, second}); };
  auto att = [&](const AttnJob& aj, std::initializer_list<GemvJob> beside) {
    FusedArgs f{};
    f.kind[0] = JOB_ATTN; f.a = aj; f.block_end[0] = n_splits * nkv * B; f.n_jobs = 1;
    f.lds_bytes = (int)fused_attn_lds_bytes(d, nq / nkv);
    for (const GemvJob& j : beside) {
      const int i = f.n_jobs;
      f.kind[i] = JOB_GEMV; f.g[i] = j; f.block_end[i] = f.block_end[i - 1] + blocks_of(j);
      f.lds_bytes = std::max(f.lds_bytes, lds_of(j));
      f.n_jobs = i + 1;
    }
    for (int i = f.n_jobs; i < FUSED_MAX_JOBS; ++i) f.block_end[i] = f.block_end[f.n_jobs - 1];
    return f;
  };
  // { qkv , down }.  A launch is as long as its most loaded CU, and workgroups are handed to the CUs in block
  // order, one per CU and then a second one per CU in the same order.  So: pairs of down tiles first, as many
  // as there are CUs left beside QKV's (one long workgroup per CU), then the QKV workgroups, then the rest of
  // down as single tiles, which land in the second slots of the first CUs - those of the pairs, not those of
  // QKV's whole-K workgroups (70B shard: 176 pairs + 80 QKV + 160 single tiles; 3.41 -> 3.37 ms per step
  // against { QKV, 80 pairs, 352 single tiles }).  Taken when it lowers the weight bytes of the most loaded CU
  // (the 8B shape, whose down tiles are 459 KiB each, is faster the other way); else: QKV first, and as many
  // down workgroups with two tiles as it takes to make every workgroup resident from the start.
  auto qkv_down = [&](const GemvJob& qkv, const GemvJob& dn) {
    const int slots = 2 * c->n_cu;
    const int n_pairs = c->n_cu - blocks_of(qkv);
    // weight bytes of the most loaded CU under that placement (workgroups past the second round: ignored)
    auto worst_cu = [&](std::initializer_list<GemvJob> jobs) {
      std::vector<long long> load((size_t)c->n_cu, 0);
      int idx = 0;
      for (const GemvJob& j : jobs)
        for (int w = 0; w < blocks_of(j) && idx < slots; ++w, ++idx) load[(size_t)(idx % c->n_cu)] += (long long)std::max(1, j.tn) * j.K * 32;
      return *std::max_element(load.begin(), load.end());
    };
    const int over = blocks_of(qkv) + blocks_of(dn) - slots;
    GemvJob dbl_o = dn, sgl_o = dn;   // the plan that starts with QKV
    const bool mixed_o = over > 0 && 2 * over <= blocks_of(dn);
    if (mixed_o) {
      dbl_o.tn = 2; dbl_o.group0 = 0; dbl_o.n_groups = over;                      // tiles [0, 2 * over)
      sgl_o.group0 = 2 * over; sgl_o.n_groups = blocks_of(dn) - 2 * over;         // tiles [2 * over, end)
    }
    // Better still where it fits: ONE workgroup per CU, down in workgroups of three and two tiles beside QKV's
    // (two streaming workgroups that share a CU run below the rate of one: 70B shard 160 x 3 + 16 x 2 tiles + 80
    // QKV workgroups on 256 CUs: 3.39 -> 3.35 ms per step)
    const int n_dn = c->n_cu - blocks_of(qkv);
    if (dn.tn != 2 && blocks_of(dn) % 2 == 0 && n_dn > 0 && 2 * n_dn <= blocks_of(dn) && blocks_of(dn) <= 3 * n_dn) {
      const int a3 = (blocks_of(dn) - 2 * n_dn) & ~1;      // workgroups of three tiles (even, so that the pairs start on an even tile)
      const int b2 = (blocks_of(dn) - 3 * a3) / 2;         // workgroups of two tiles
      GemvJob tri = dn, dbl = dn;
      tri.tn = 3; tri.group0 = 0; tri.n_groups = a3;                 // tiles [0, 3 a3)
      dbl.tn = 2; dbl.group0 = 3 * a3 / 2; dbl.n_groups = b2;        // tiles [3 a3, end)
      if (a3 + b2 + blocks_of(qkv) <= c->n_cu + 1) return several({tri, qkv, dbl});
    }
    if (dn.tn != 2 && n_pairs > 0 && 2 * n_pairs <= blocks_of(dn) && c->n_cu + blocks_of(dn) - 2 * n_pairs <= slots) {
      GemvJob dbl = dn, sgl = dn;
      dbl.tn = 2; dbl.group0 = 0; dbl.n_groups = n_pairs;                    // tiles [0, 2 * n_pairs)
      sgl.group0 = 2 * n_pairs; sgl.n_groups = blocks_of(dn) - 2 * n_pairs;  // tiles [2 * n_pairs, end)
      const long long worst_new = worst_cu({dbl, qkv, sgl});
      const long long worst_old = mixed_o ? worst_cu({qkv, dbl_o, sgl_o}) : worst_cu({qkv, dn});
      if (worst_new < worst_old) return several({dbl, qkv, sgl});
    }
    if (!mixed_o) return two(qkv, dn);
    return several({qkv, dbl_o, sgl_o});
  };
  auto src_of = [&](int m) { const int s = m - lag_of(c, m); return s < 0 ? 0 : s; };

  std::vector<FusedArgs>& plan = c->fused_plan;
  plan.clear();
  const bool paired = g.decode_fused == 1 || g.decode_fused == 3;   // (2: one job per launch whatever the wiring)
  // layers with the standard wiring come first (all of them under LADDER_WIRING_STANDARD, the lower ones of a hybrid stack)
  const int n_std = g.wiring == LADDER_WIRING_STANDARD ? N : g.n_standard_layers;
  if (g.wiring != LADDER_WIRING_PARALLEL && paired) {
    // Standard layers: the chain of Eq. 1 leaves nothing to pair, one job per launch.  The last standard layer's down
    // projection shares its launch with the first ladder layer's QKV projection, which reads x_{2 n_std - 1}.
    for (int l = 1; l <= n_std; ++l) {
      plan.push_back(one(job_qkv(l, src_of(2 * l - 1))));
      plan.push_back(att(job_att(l), {}));
      plan.push_back(one(job_o(l, 2 * l - 1)));
      plan.push_back(one(job_gu(l, src_of(2 * l))));
      if (l == n_std && n_std < N) plan.push_back(qkv_down(job_qkv(n_std + 1, src_of(2 * n_std + 1)), job_dn(n_std, 2 * n_std)));
      else plan.push_back(one(job_dn(l, 2 * l)));
    }
    // Ladder layers.
    // Modules 1 and 2 both read x_0; then TWO launches per layer:
    //     { attention_l , gate/up_l , o_l }     { qkv_{l+1} , down_l }
    // Attention and gate/up, and the next layer's QKV and down, do not depend on each other under the
    // ladder wiring.  The attention workgroups are few and latency bound: beside the largest weight stream
    // they cost nothing.  o_l does depend on attention_l: its workgroups wait (asleep) on a per-layer arrival
    // counter that the attention workgroups raise once their device-coherent stores of the output have
    // completed, and read the attention output with device-coherent loads (no fence on either side).  A workgroup only ever waits for workgroups with lower block indices, which
    // were dispatched before it and wait for nothing, so the wait always ends (it is bounded all the same).
    // This is the one dependency between jobs of a launch (20 producers, 256 consumers): o_l streams beside gate/up instead of in a launch of its own at a third of the streaming
    // rate (4.03 -> 3.87 ms per step on the 70B shard).  An acquire fence in the consumers instead of
    // coherent loads made the step 5.1 ms (an agent-scope acquire empties the L2 under the weight streams);
    // o_l at the end of the launch instead of among the first workgroups 4.1 ms (it then runs after
    // gate/up, not beside it); cutting gate/up over two launches 4.1 - 4.6 ms.
    if (n_std == 0) plan.push_back(one(job_qkv(1, 0)));
    for (int l = n_std + 1; l <= N; ++l) {
      AttnJob aj = job_att(l);
      aj.done = c->att_done + (size_t)(l - 1) * FUSED_SYNC_WORDS;
      GemvJob o = job_o(l, 2 * l - 1);
      aj.done_flagged = 1;   // (a flag word per (sequence, kv head), polled by o_l's workgroups: no atomic at the attention job's end)
      o.wait_on = aj.done; o.wait_flags = (unsigned)(B * nkv); o.wait_bias = c->wait_bias; o.wait_spins = c->wait_spins; o.err_word = c->err_word_dev;
      // block order: attention, as many gate/up workgroups as leave every CU one long workgroup, o_l (resident
      // from the start, asleep until attention is done, then beside the rest of gate/up), the rest of gate/up
      GemvJob gu_a = job_gu(l, 2 * l - 2), gu_b = gu_a;
      // every workgroup of the launch should be resident from the start (two per CU): workgroups beyond that wait
      // for a slot, and the last in block order are long gate/up workgroups.  Where attention, gate/up and o_l
      // make more than that (large batches: attention has a workgroup per sequence and split), o_l takes four
      // tiles per workgroup, if its K range is long enough for that to pay (measured: 8B shape at batch 16
      // 4.06 -> 3.86 ms per step, 70B R = 4 shard at batch 16 8.89 -> 8.61; with the R = 8 shard's K range of
      // 1024, batch 8 and 16, it cost 1 - 2 %).
      if (n_splits * nkv * B + blocks_of(gu_a) + blocks_of(o) > 2 * c->n_cu && nqd >= 2048 && o.tn == 2 && o.n_groups % 2 == 0) { o.tn = 4; o.n_groups /= 2; }
      // Chained step: a slot ends every block with its stores' round trip and its count before it asks for the next
      // one, so where single gate/up tiles make more blocks than there are slots, pairs (same sums in the same order:
      // same bits).  8B shape at batch 1 / 4 / 8: 2.52 / 2.75 / 3.22 -> 2.46 / 2.64 / 3.02 ms per step; R = 8 shard at
      // batch 8 / 12: 4.24 / 5.83 -> 3.98 / 4.67; quadruples instead: slower than pairs, except the 8B shape at batch 8
      // (3.00).  With separate launches the hardware refills a slot at once and single tiles stay ahead at 7 - 12 rows.
      if (c->chain && std::max(1, gu_a.tn) == 1 && gu_a.n_groups % 2 == 0 &&
          n_splits * nkv * B + blocks_of(gu_a) + blocks_of(o) > c->chain_slots) {
        gu_a.tn = 2; gu_a.n_groups /= 2; gu_b = gu_a;
      }
      const int n_a = std::min(gu_a.n_groups / 2, c->n_cu / 2);   // (any position in the first half measured the same)
      gu_a.n_groups = n_a;
      gu_b.group0 = n_a; gu_b.n_groups -= n_a;
      if (n_a > 0) plan.push_back(att(aj, {gu_a, o, gu_b}));
      else plan.push_back(att(aj, {o, gu_b}));
      if (l < N) plan.push_back(qkv_down(job_qkv(l + 1, 2 * l - 1), job_dn(l, 2 * l)));
      else plan.push_back(one(job_dn(N, 2 * N)));
    }
  } else if (g.wiring == LADDER_WIRING_PARALLEL && paired) {
    // both modules of layer l read x_{2l-2}: THREE launches per layer,
    //     { gate/up_l , qkv_l }     { attention_l , down_l }     { o_l }
    // with the two outputs added in the order MLP, attention (the sum is the same up to rounding): down_l does
    // not wait for attention that way, and o_l, which does, is the short one.
    for (int l = 1; l <= N; ++l) {
      plan.push_back(two(job_gu(l, 2 * l - 2), job_qkv(l, 2 * l - 2)));
      plan.push_back(att(job_att(l), {job_dn(l, 2 * l, 2 * l - 1)}));
      plan.push_back(one(job_o(l, 2 * l - 1, 2 * l)));
    }
  } else {
    for (int l = 1; l <= N; ++l) {
      plan.push_back(one(job_qkv(l, src_of(2 * l - 1))));
      plan.push_back(att(job_att(l), {}));
      plan.push_back(one(job_o(l, 2 * l - 1)));
      plan.push_back(one(job_gu(l, src_of(2 * l))));
      plan.push_back(one(job_dn(l, 2 * l)));
    }
  }
  // Emulated collective latency (reduce_delay_us): the collective that completes stream x_m starts when the last
  // workgroup of module m's residual update ends (those workgroups leave the wall-clock time in t_done[m]) and
  // lasts the configured time; a projection that reads x_m holds its workgroups back until then (they have
  // requested their first weight tiles already), while the other jobs of its launch run.  The arithmetic stays
  // where it is (the other ranks' partial sums are local memory here): what is emulated is WHEN a reduced stream
  // may be read, so a schedule hides the latency exactly where it has independent work to run meanwhile.
  if (g.reduce_delay_us > 0) {
    const unsigned long long ticks = (unsigned long long)g.reduce_delay_us * (unsigned long long)c->wall_khz / 1000ull;
    for (FusedArgs& fa : plan)
      for (int k = 0; k < fa.n_jobs; ++k) {
        if (fa.kind[k] != JOB_GEMV) continue;
        GemvJob& j = fa.g[k];
        if (j.normed && j.reads_stream > 0) { j.t_ready = c->t_done + j.reads_stream; j.delay_ticks = ticks; }
        if (j.epi == EPI_RESIDUAL && j.completes_stream > 0) j.t_done = c->t_done + j.completes_stream;
      }
  }
  c->fused_plan_batch = B;
  c->fused_plan_peers = c->peers;
}

// Chained step: turns the launch list into the item lists and job tables of ONE persistent launch.
// Every buffer the jobs hand to each other is written once per step here, so "who produces what a job reads" is a
// lookup by address: the job waits for that producer's completion words (a projection's, or the attention job's),
// at which every producer workgroup counts itself.  Block b of launch p goes to slot b mod n_slots, the slots' lists in launch order: that keeps
// the placement the launch list was laid out for (the first n_cu blocks of a launch on a CU each).
// Must not run under stream capture (it allocates nothing, but copies the tables synchronously).
int build_chain(ladder_ctx* c, int B) {
  const ladder_config& g = c->cfg;
  (void)B;
  // The producers of a step: every projection (by its weights: the parts of one projection share them) and every
  // attention job.  words: its completion words; blocks: its workgroups (attention: those that write final outputs);
  // polls: the workgroups that wait for it.
  struct Producer { const void* key; unsigned* words; unsigned blocks, seen, polls; bool flagged; };
  std::vector<Producer> prod;
  auto producer_of = [&](const void* key) {
    for (size_t i = 0; i < prod.size(); ++i)
      if (prod[i].key == key) return (int)i;
    prod.push_back(Producer{key, nullptr, 0u, 0u, 0u, false});
    return (int)prod.size() - 1;
  };
  std::vector<std::pair<const void*, int>> ready;   // (buffer, the producer that completes it), latest last
  auto find_ready = [&](const void* buf) {
    if (buf)
      for (size_t i = ready.size(); i-- > 0;)
        if (ready[i].first == buf) return ready[i].second;
    return -1;
  };
  auto set_ready = [&](const void* buf, int p) {
    if (!buf) return;
    for (auto& e : ready)
      if (e.first == buf) { e.second = p; return; }
    ready.push_back({buf, p});
  };
  // pass 1: who waits for whom (dep[launch][job] = up to two producers), the producers' sizes
  std::vector<std::array<std::array<int, 2>, FUSED_MAX_JOBS>> dep(c->fused_plan.size());
  int n_attn = 0;
  for (size_t p = 0; p < c->fused_plan.size(); ++p) {
    const FusedArgs& fa = c->fused_plan[p];
    for (int k = 0; k < fa.n_jobs; ++k) {
      dep[p][(size_t)k] = {-1, -1};
      const int blocks = fa.block_end[k] - (k > 0 ? fa.block_end[k - 1] : 0);
      if (fa.kind[k] == JOB_ATTN) {
        const AttnJob& a = fa.a;
        if (!a.done) return fail(c, LADDER_E_ARG, "chained step: an attention job without completion words");
        dep[p][(size_t)k][0] = find_ready(a.q);
        const int me = producer_of(a.done);
        prod[(size_t)me].words = a.done;
        prod[(size_t)me].blocks = (unsigned)(a.B * a.nkv);
        set_ready(a.o, me);
        ++n_attn;
      } else {
        const GemvJob& j = fa.g[k];
        dep[p][(size_t)k][0] = find_ready(j.xb);
        if (j.epi == EPI_RESIDUAL) {
          const int d2 = find_ready(j.x_old);
          if (dep[p][(size_t)k][0] < 0) dep[p][(size_t)k][0] = d2;
          else if (d2 != dep[p][(size_t)k][0]) dep[p][(size_t)k][1] = d2;
        }
        prod[(size_t)producer_of(j.wp)].blocks += (unsigned)j.n_groups;
      }
      for (int d : dep[p][(size_t)k])
        if (d >= 0) prod[(size_t)d].polls += (unsigned)blocks;
    }
    // what this launch's projections write is complete when they are (registered after the launch's jobs have
    // looked up their own inputs: no job reads what a later block of its own launch writes)
    for (int k = 0; k < fa.n_jobs; ++k) {
      if (fa.kind[k] != JOB_GEMV) continue;
      const GemvJob& j = fa.g[k];
      const int me = producer_of(j.wp);
      if (j.epi == EPI_SWIGLU) set_ready(j.act, me);
      if (j.epi == EPI_RESIDUAL) { set_ready(j.x_new, me); set_ready(j.xop_a, me); set_ready(j.xop_b, me); }
      if (j.epi == EPI_QKV_ROPE) set_ready(j.q_out, me);
    }
  }
  if ((int)prod.size() - n_attn > 4 * g.n_layers) return fail(c, LADDER_E_ARG, "chained step: more projections than completion words");
  // completion words of the projections; a producer's workgroups raise a flag word each (no atomics at its end)
  // where the polls stay cheap: lines polled x workgroups polling them, per round, at most 512 (the attention
  // job's few outputs polled by an output projection; a QKV projection polled by the attention workgroups)
  {
    int n_proj = 0;
    for (Producer& pr : prod) {
      if (!pr.words) pr.words = c->sync_words + (size_t)(n_proj++) * FUSED_SYNC_WORDS;
      const unsigned lines = (pr.blocks + 31u) / 32u;
      // (measured at the 70B shard: limit 1300, which adds gate/up -> down: 3.23 -> 3.32 ms per step; 2100, which adds
      // the output projection: 3.42; everything flagged: 3.70; nothing flagged: 3.24)
      pr.flagged = pr.blocks <= 256u && lines * pr.polls <= 512u;
    }
  }
  // pass 2: the jobs' tables and the slots' item lists
  std::vector<GemvJob> gemv;
  std::vector<AttnJob> attn;
  std::vector<std::vector<StepItem>> slot((size_t)c->chain_slots);
  std::vector<StepItem> surplus(c->fused_plan.size() * FUSED_CLAIM_MAX);
  size_t n_surplus_lists = 0;   // launches up to the last one that has a list
  c->chain_meta.assign((size_t)c->chain_slots, {});
  int lds = 0;
  for (size_t p = 0; p < c->fused_plan.size(); ++p) {
    FusedArgs& fa = c->fused_plan[p];
    lds = std::max(lds, fa.lds_bytes);
    int job_index[FUSED_MAX_JOBS];
    for (int k = 0; k < fa.n_jobs; ++k) {
      const int d1 = dep[p][(size_t)k][0], d2 = dep[p][(size_t)k][1];
      if (fa.kind[k] == JOB_ATTN) {
        AttnJob& a = fa.a;
        a.wait_on = nullptr;
        if (d1 >= 0) { a.wait_on = prod[(size_t)d1].words; a.wait_flags = prod[(size_t)d1].flagged ? prod[(size_t)d1].blocks : 0u; }
        a.wait_bias = c->wait_bias; a.wait_spins = c->wait_spins; a.err_word = c->err_word_dev;
        a.done_flagged = prod[(size_t)producer_of(a.done)].flagged ? 1 : 0;
        job_index[k] = (int)attn.size();
        attn.push_back(a);
      } else {
        GemvJob& j = fa.g[k];
        Producer& me = prod[(size_t)producer_of(j.wp)];
        j.wait_on = nullptr; j.wait_on2 = nullptr; j.coherent_x = 0;
        if (d1 >= 0) { j.wait_on = prod[(size_t)d1].words; j.wait_flags = prod[(size_t)d1].flagged ? prod[(size_t)d1].blocks : 0u; }
        if (d2 >= 0) { j.wait_on2 = prod[(size_t)d2].words; j.wait_flags2 = prod[(size_t)d2].flagged ? prod[(size_t)d2].blocks : 0u; }
        j.wait_bias = c->wait_bias; j.wait_spins = c->wait_spins; j.err_word = c->err_word_dev;
        j.done_ctr = me.words;
        j.done_target = me.blocks;
        j.done_ord0 = me.seen;
        j.done_flagged = me.flagged ? 1 : 0;
        me.seen += (unsigned)j.n_groups;
        job_index[k] = (int)gemv.size();
        gemv.push_back(j);
      }
    }
    // Which slot runs which block: block b < n_slots on slot b.  Where a launch has more blocks than there are slots,
    // the hardware would hand the next block to the first workgroup slot that becomes free: the last FUSED_CLAIM_MAX
    // of the blocks beyond the slots form the launch's surplus list, from which the slots take blocks as they finish
    // (decode_fused.h); any blocks between the two go, in block order, to the slot with the least work of this launch
    // so far (a block's work: its weight bytes plus a fixed part; ties: the lowest slot).
    const int total = fa.block_end[fa.n_jobs - 1];
    std::vector<long long> load((size_t)c->chain_slots, 0);
    const int n_dyn = std::min(std::max(0, total - c->chain_slots), (int)FUSED_CLAIM_MAX);
    if (n_dyn > 0 && (int)p >= c->chain_launch_cap) return fail(c, LADDER_E_ARG, "chained step: more launches than surplus lists sized at init");
    for (int b = 0, k = 0; b < total; ++b) {
      while (b >= fa.block_end[k]) ++k;
      const int lb = b - (k > 0 ? fa.block_end[k - 1] : 0);
      // (an output projection of the same launch cannot start before the attention job has ended: a block queued
      // behind it would wait that long as well.  Headline shape at 32768 cached positions, 736 blocks per launch:
      // 7.39 -> 5.64 ms per step.  Pricing an attention block by the cache rows of its split instead of a constant
      // made the 8B shape at batch 16 13 % slower: 3.67 -> 4.15 ms.)
      const long long att_work = fa.kind[0] == JOB_ATTN ? (96 + 128) * 1024 : 0;
      const long long work = fa.kind[k] == JOB_ATTN ? att_work
                             : 96 * 1024 + (long long)std::max(1, fa.g[k].tn) * fa.g[k].K * 32 + (fa.g[k].after_attention ? att_work : 0);
      StepItem it{};
      const hipError_t e = fa.kind[k] == JOB_ATTN ? fused_chain_attn_item(attn[(size_t)job_index[k]], job_index[k], lb, &it)
                                                  : fused_chain_item(gemv[(size_t)job_index[k]], job_index[k], lb, &it);
      if (e != hipSuccess) return fail(c, LADDER_E_ARG, "chained step: a job of the launch list is outside what the kernel runs");
      if (b >= total - n_dyn) {
        surplus[p * FUSED_CLAIM_MAX + (size_t)(b - (total - n_dyn))] = it;
        continue;
      }
      const int sl = b < c->chain_slots ? b : (int)(std::min_element(load.begin(), load.end()) - load.begin());
      load[(size_t)sl] += work;
      slot[(size_t)sl].push_back(it);
      ladder_ctx::ChainMeta meta{(int)p, LADDER_TL_ATTN, 0, 0};
      if (fa.kind[k] == JOB_GEMV) {
        const GemvJob& j = fa.g[k];
        meta.kind = j.epi == EPI_QKV_ROPE ? LADDER_TL_QKV : j.epi == EPI_SWIGLU ? LADDER_TL_GATE_UP : j.after_attention ? LADDER_TL_O : LADDER_TL_DOWN;
        meta.tiles = std::max(1, j.tn);
        meta.weight_bytes = (long long)meta.tiles * j.K * 32;
      }
      c->chain_meta[(size_t)sl].push_back(meta);
    }
    if (n_dyn > 0) {
      StepItem it{};
      if (fused_chain_claim_item(c->chain_surplus_dev + p * FUSED_CLAIM_MAX, c->chain_claim_ctr + p * 32, n_dyn, &it) != hipSuccess)
        return fail(c, LADDER_E_ARG, "chained step: a surplus list is outside what the kernel runs");
      for (size_t w = 0; w < slot.size(); ++w) {
        slot[w].push_back(it);
        c->chain_meta[w].push_back(ladder_ctx::ChainMeta{(int)p, -1, 0, 0});   // (not a block: skipped by the timeline)
      }
      n_surplus_lists = p + 1;
    }
  }
  size_t n_items = 0;
  for (const auto& v : slot) n_items = std::max(n_items, v.size());
  n_items += 1;   // the end marker
  if (n_items > c->chain_items_cap || (int)gemv.size() > c->chain_gemv_cap || (int)attn.size() > c->chain_attn_cap)
    return fail(c, LADDER_E_ARG, "chained step: the launch list is longer than the tables sized at init");
  std::vector<StepItem> flat((size_t)c->chain_slots * n_items);   // (zero items: kind 0 ends a list)
  for (size_t w = 0; w < slot.size(); ++w) std::copy(slot[w].begin(), slot[w].end(), flat.begin() + w * n_items);
  HIP_TRY(c, hipStreamSynchronize(c->s_attn));   // (a step that reads the old tables may still be running)
  HIP_TRY(c, hipMemcpy(c->chain_items_dev, flat.data(), flat.size() * sizeof(StepItem), hipMemcpyHostToDevice));
  HIP_TRY(c, hipMemcpy(c->chain_gemv_dev, gemv.data(), gemv.size() * sizeof(GemvJob), hipMemcpyHostToDevice));
  if (!attn.empty()) HIP_TRY(c, hipMemcpy(c->chain_attn_dev, attn.data(), attn.size() * sizeof(AttnJob), hipMemcpyHostToDevice));
  if (n_surplus_lists) HIP_TRY(c, hipMemcpy(c->chain_surplus_dev, surplus.data(), n_surplus_lists * FUSED_CLAIM_MAX * sizeof(StepItem), hipMemcpyHostToDevice));
  c->chain_items = (int)n_items;
  c->chain_lds = lds;
  return LADDER_OK;
}

// the launch list (and, for a chained step, its tables on the device) for a step of B sequences: built at the
// first step and again after a change of the batch, the peers or the wait limits
int ensure_fused_plan(ladder_ctx* c, int B) {
  if (!c->fused_plan.empty() && c->fused_plan_batch == B && c->fused_plan_peers == c->peers) return LADDER_OK;
  build_fused_plan(c, B);
  if (c->chain) {
    // the last module's residual update delivers the result and advances the position itself (where an emulated
    // collective still has to end after the launch, both are left to the caller)
    if (c->cfg.reduce_delay_us == 0) {
      bool first = true;
      for (FusedArgs& fa : c->fused_plan)
        for (int k = 0; k < fa.n_jobs; ++k)
          if (fa.kind[k] == JOB_GEMV && fa.g[k].epi == EPI_RESIDUAL && fa.g[k].completes_stream == c->n_mod) {
            fa.g[k].x_copy = fa.g[k].x_new;   // (the kernel's x_out argument takes its place when there is one)
            fa.g[k].pos_inc = first ? c->pos_dev : nullptr;
            first = false;
          }
    }
    const int rc = build_chain(c, B);
    if (rc) { c->fused_plan.clear(); return rc; }
  }
  return LADDER_OK;
}

// one decode step on stream s: x_0 from `emb`, the launch list, x_2N left in ring[2N % 3]
// x_out (may be null): the caller's f32 [B][H], written by the last module's residual update itself; the same job
// advances the position in device memory.  (Where an emulated collective still has to end after the last launch,
// both are left to the caller of this function: the result must not appear before its collective is over.)
// *finished: bit 0 = the result is in x_out, bit 1 = the position has been advanced
enum { FUSED_DELIVERED = 1, FUSED_ADVANCED = 2 };
int fused_body(ladder_ctx* c, const void* emb, int B, hipStream_t s, float* x_out, int* finished, const StageIo* st = nullptr) {
  const ladder_config& g = c->cfg;
  {
    const int rc = ensure_fused_plan(c, B);
    if (rc) return rc;
  }
  *finished = 0;
  if (g.reduce_delay_us == 0 && !c->chain) {
    // the last launch's last residual job is the last module's (every launch list ends with it)
    FusedArgs& last = c->fused_plan.back();
    for (int k = last.n_jobs - 1; k >= 0; --k)
      if (last.kind[k] == JOB_GEMV && last.g[k].epi == EPI_RESIDUAL && last.g[k].completes_stream == c->n_mod) {
        bool reads_pos = false;
        for (int q = 0; q < last.n_jobs; ++q) reads_pos = reads_pos || last.kind[q] == JOB_ATTN || (last.kind[q] == JOB_GEMV && last.g[q].epi == EPI_QKV_ROPE);
        // (a residual job cut in parts: every part copies its rows, the first part advances the position)
        const bool fold = x_out != nullptr && !reads_pos;
        bool first = true;
        for (int q = 0; q < last.n_jobs; ++q)
          if (last.kind[q] == JOB_GEMV && last.g[q].epi == EPI_RESIDUAL && last.g[q].completes_stream == c->n_mod) {
            last.g[q].x_copy = fold ? x_out : nullptr;
            last.g[q].pos_inc = (fold && first) ? c->pos_dev : nullptr;
            first = false;
          }
        *finished = fold ? (FUSED_DELIVERED | FUSED_ADVANCED) : 0;
        break;
      }
  }
  auto events = [&](hipEvent_t (&e)[2]) -> hipError_t {
    e[0] = e[1] = nullptr;
    if (!c->prof) return hipSuccess;
    for (int i = 0; i < 2; ++i) {
      if (!c->prof_pool.empty()) {
        e[i] = c->prof_pool.back();
        c->prof_pool.pop_back();
      } else {
        hipError_t r = hipEventCreate(&e[i]);
        if (r != hipSuccess) return r;
      }
    }
    return hipSuccess;
  };
  hipEvent_t e[2];
  HIP_TRY(c, events(e));
  {
    // x_0 and the operands of the modules that read it (module 1, and module 2 where its lag is 2)
    EmbedArgs ea{};
    ea.emb = (const bf16_t*)emb; ea.x0 = c->x_ring[0]; ea.ssq = c->ssq_ring[0]; ea.rows = B; ea.H = g.hidden;
    if (st) { ea.emb = nullptr; ea.res = st->res; ea.att = st->att; ea.mlp = st->mlp; }
    if (lag_of(c, 1) == 2) ea.ssq_a = c->ssq_first;
    ea.zero_words = c->att_done; ea.n_zero = c->n_zero_words;
    int cons[2];
    const int nc = consumers_of(c, 0, cons);
    for (int i = 0; i < nc; ++i) {
      const int cm = cons[i], cl = (cm - 1) / 2;
      if (cm & 1) { ea.xop_a = c->xop_ring[0][1]; ea.gain_a = (const bf16_t*)c->gain_attn[cl]; }
      else { ea.xop_b = c->xop_ring[0][0]; ea.gain_b = (const bf16_t*)c->gain_mlp[cl]; }
    }
    HIP_TRY(c, launch_embed(ea, s, e[0], e[1]));
  }
  if (c->prof) c->prof_pending.push_back({LADDER_K_OTHER, e[0], e[1]});
  const int gq = g.n_q_heads / g.n_kv_heads;
  if (c->chain) {
    HIP_TRY(c, events(e));
    HIP_TRY(c, launch_fused_chain(c->chain_items_dev, c->chain_items, c->chain_gemv_dev, c->chain_attn_dev, x_out,
                                  c->timeline_on ? c->chain_tl_dev : nullptr, c->chain_slots, c->chain_lds, g.head_dim, gq,
                                  s, e[0], e[1]));
    if (c->prof) c->prof_pending.push_back({LADDER_K_FUSED_DECODE, e[0], e[1]});
    if (g.reduce_delay_us == 0) *finished = FUSED_ADVANCED | (x_out ? FUSED_DELIVERED : 0);
  } else {
    for (const FusedArgs& fa : c->fused_plan) {
      HIP_TRY(c, events(e));
      HIP_TRY(c, launch_fused_decode(fa, g.head_dim, gq, s, e[0], e[1]));
      if (c->prof) c->prof_pending.push_back({LADDER_K_FUSED_DECODE, e[0], e[1]});
    }
  }
  if (g.reduce_delay_us > 0) {   // x_2N is complete when the last module's emulated collective is
    const unsigned long long ticks = (unsigned long long)g.reduce_delay_us * (unsigned long long)c->wall_khz / 1000ull;
    HIP_TRY(c, timed(c, LADDER_K_OTHER, s, [&] {
      hipLaunchKernelGGL(wait_until_kernel, dim3(1), dim3(64), 0, s, (const unsigned long long*)(c->t_done + c->n_mod), ticks);
      return hipGetLastError();
    }));
  }
  if (st) {   // the last three streams of the step are still in their ring slots (the ring has at least three)
    auto X = [&](int m) { return c->x_ring[(size_t)(m % c->ring_n)]; };
    const int rc = launch_stage_out(c, X(c->n_mod - 2), X(c->n_mod - 1), X(c->n_mod), *st, B, s);
    if (rc) return rc;
  }
  return LADDER_OK;
}

int fence_in(ladder_ctx* c) {
  HIP_TRY(c, hipEventRecord(c->ev_begin, c->main));
  HIP_TRY(c, hipStreamWaitEvent(c->s_attn, c->ev_begin, 0));
  return LADDER_OK;
}
int fence_out(ladder_ctx* c) {
  HIP_TRY(c, hipEventRecord(c->ev_end, c->s_attn));
  HIP_TRY(c, hipStreamWaitEvent(c->main, c->ev_end, 0));
  return LADDER_OK;
}

int forward(ladder_ctx* c, const void* x_in, int B, int T, int pos0, void* x_out, const StageIo* st = nullptr) {
  int rc = fence_in(c);
  if (rc) return rc;
  rc = forward_body(c, x_in, B, T, pos0, x_out, st);
  if (rc) return rc;
  return fence_out(c);
}

// one decode step replayed from a captured graph: stage the input, launch, copy the result out
int decode_graph_step(ladder_ctx* c, const void* x_in, void* x_out) {
  const int B = c->batch, H = c->cfg.hidden;
  if (!c->graph_exec || c->graph_batch != B || c->graph_stale) {
    if (c->graph_exec) {
      HIP_TRY(c, hipStreamSynchronize(c->s_attn));   // (a replay may still be running)
      HIP_TRY(c, hipGraphExecDestroy(c->graph_exec));
      c->graph_exec = nullptr;
    }
    c->graph_stale = false;
    if (c->fused) {   // (the launch list is built outside the capture: a chained step copies tables to the device)
      const int rcp = ensure_fused_plan(c, B);
      if (rcp) return rcp;
    }
    hipGraph_t graph = nullptr;
    DBG("capture: begin (batch %d)", B);
    HIP_TRY(c, hipStreamBeginCapture(c->s_attn, hipStreamCaptureModeThreadLocal));
    int finished = 0;
    int rc = c->fused ? fused_body(c, c->emb_stage, B, c->s_attn, nullptr, &finished) : forward_body(c, c->emb_stage, B, 1, 0, nullptr);
    DBG("capture: body recorded rc=%d", rc);
    if (rc == LADDER_OK && !(finished & FUSED_ADVANCED)) {
      DBG("capture: inc_pos");
      hipLaunchKernelGGL(inc_pos_kernel, dim3(1), dim3(1), 0, c->s_attn, c->pos_dev);
      hipError_t e = hipGetLastError();
      if (e != hipSuccess) rc = fail(c, LADDER_E_HIP, std::string("inc_pos: ") + hipGetErrorString(e));
    }
    hipError_t ee = hipStreamEndCapture(c->s_attn, &graph);
    DBG("capture: end -> %s", hipGetErrorString(ee));
    if (rc) {
      if (graph) (void)hipGraphDestroy(graph);
      return rc;
    }
    if (ee != hipSuccess) return fail(c, LADDER_E_HIP, std::string("hipStreamEndCapture: ") + hipGetErrorString(ee));
    hipError_t ei = hipGraphInstantiate(&c->graph_exec, graph, nullptr, nullptr, 0);
    DBG("capture: instantiate -> %s", hipGetErrorString(ei));
    (void)hipGraphDestroy(graph);
    if (ei != hipSuccess) {
      c->graph_exec = nullptr;
      return fail(c, LADDER_E_HIP, std::string("hipGraphInstantiate: ") + hipGetErrorString(ei));
    }
    c->graph_batch = B;
  }
  int rc = fence_in(c);
  if (rc) return rc;
  HIP_TRY(c, hipMemcpyAsync(c->emb_stage, x_in, (size_t)B * H * c->esz, hipMemcpyDeviceToDevice, c->s_attn));
  DBG("graph launch");
  HIP_TRY(c, hipGraphLaunch(c->graph_exec, c->s_attn));
  DBG("graph launched");
  const float* result = c->fused ? c->x_ring[(size_t)(c->n_mod % c->ring_n)] : c->x;
  HIP_TRY(c, hipMemcpyAsync(x_out, result, (size_t)B * H * 4, hipMemcpyDeviceToDevice, c->s_attn));
  return fence_out(c);
}

// one decode step of the fused path, launched eagerly (st: a pipeline stage's step, which takes and leaves its
// three tensors instead of x_in / x_out)
int decode_fused_step(ladder_ctx* c, const void* x_in, void* x_out, const StageIo* st = nullptr) {
  const int B = c->batch, H = c->cfg.hidden;
  int rc = fence_in(c);
  if (rc) return rc;
  int finished = 0;
  rc = fused_body(c, x_in, B, c->s_attn, (float*)x_out, &finished, st);
  if (rc) return rc;
  // (what the last launch has not done itself)
  if (!st && !(finished & FUSED_DELIVERED))
    HIP_TRY(c, hipMemcpyAsync(x_out, c->x_ring[(size_t)(c->n_mod % c->ring_n)], (size_t)B * H * 4, hipMemcpyDeviceToDevice, c->s_attn));
  if (!(finished & FUSED_ADVANCED)) {
    hipLaunchKernelGGL(inc_pos_kernel, dim3(1), dim3(1), 0, c->s_attn, c->pos_dev);
    HIP_TRY(c, hipGetLastError());
  }
  return fence_out(c);
}

// A kernel of an earlier call has raised the error word (its bounded in-launch wait gave up, so that call's
// output is not valid): reported once, by the next forward call, which does nothing else.
int check_device_error(ladder_ctx* c) {
  volatile unsigned* w = c->err_word;
  if (w && w[0] != 0u) {
    w[0] = 0u;
    // (workgroups that gave up stored nothing; where the step's last job advances the position itself, that may
    // not have happened: the device's copy is put back in step with the host's count)
    hipLaunchKernelGGL(set_pos_kernel, dim3(1), dim3(1), 0, c->main, c->pos_dev, c->pos);
    (void)hipGetLastError();
    return fail(c, LADDER_E_HIP, "a kernel of an earlier decode step gave up a bounded in-launch wait (a job waiting for the job that produces its input): that step's output is invalid");
  }
  if (w && w[1] != 0u) {
    w[1] = 0u;
    return fail(c, LADDER_E_ARG, "an earlier ladder_embed was given a token id outside [0, vocab): the embeddings it wrote for that id are those of the nearest valid id");
  }
  return LADDER_OK;
}

int all_loaded(ladder_ctx* c) {
  for (auto& L : c->store)
    if (!L.loaded) return fail(c, LADDER_E_STATE, "a (layer, shard) has not been given to ladder_load_layer");
  for (char v : c->gains_loaded)
    if (!v) return fail(c, LADDER_E_STATE, "norm gains missing: shard 0 of a layer has not been loaded");
  return LADDER_OK;
}

}  // namespace

// =================================================================================================
extern "C" {

// ladder_init, or (dry) the same walk through the memory plan without a single HIP call: then *out receives a
// context that owns nothing but its byte counts
static int init_impl(const ladder_config* cfg, void* hip_stream, ladder_ctx** out, bool dry) {
  if (out) *out = nullptr;
  if (!cfg || !out) return fail(nullptr, LADDER_E_ARG, "null argument");
  std::string why;
  int rc = check_config(cfg, why);
  if (rc) return fail(nullptr, rc, why);
  ladder_ctx* c = new ladder_ctx();
  c->dry = dry;
  c->cfg = *cfg;
  const ladder_config& g = c->cfg;
  c->bf16 = g.dtype == LADDER_BF16;
  c->esz = c->bf16 ? 2 : 4;
  c->fast = g.kernel_path == LADDER_PATH_AUTO && fast_shapes_ok(cfg);
  c->n_mod = 2 * g.n_layers;
  c->n_peers = (g.peer_pool > 0) ? g.tp_degree - g.n_real_shards : 0;
  c->s_cap = (g.max_seq + 127) / 128 * 128;
  c->rows_cap = g.max_batch * g.max_tokens;
  c->nqkv = (g.n_q_heads + 2 * g.n_kv_heads) * g.head_dim;
  c->main = (hipStream_t)hip_stream;

  auto bail = [&](int code) {
    std::string msg = c->err;
    if (c->dry) delete c;
    else ladder_free(c);
    g_init_error = msg;
    return code;
  };
#define INIT_TRY(expr)          \
  do {                          \
    int rc_ = (expr);           \
    if (rc_) return bail(rc_);  \
  } while (0)
#define INIT_HIP(expr)                                                                       \
  do {                                                                                       \
    if (c->dry) break;                                                                       \
    hipError_t e_ = (expr);                                                                  \
    if (e_ != hipSuccess) {                                                                  \
      c->err = std::string(#expr) + ": " + hipGetErrorString(e_);                            \
      return bail(LADDER_E_HIP);                                                             \
    }                                                                                        \
  } while (0)

  {
    int dev_id = 0, khz = 0;
    INIT_HIP(hipGetDevice(&dev_id));
    c->device = dev_id;
    if (!c->dry && hipDeviceGetAttribute(&khz, hipDeviceAttributeWallClockRate, dev_id) == hipSuccess && khz > 0) c->wall_khz = khz;
    INIT_HIP(resolve_static_scratch(dev_id, &c->static_scratch));
  }
  INIT_HIP(hipStreamCreateWithFlags(&c->s_attn, hipStreamNonBlocking));
  INIT_HIP(hipStreamCreateWithFlags(&c->s_mlp, hipStreamNonBlocking));
  INIT_HIP(hipStreamCreateWithFlags(&c->side, hipStreamNonBlocking));
  INIT_HIP(hipEventCreateWithFlags(&c->ev_begin, hipEventDisableTiming));
  INIT_HIP(hipEventCreateWithFlags(&c->ev_end, hipEventDisableTiming));
  INIT_HIP(hipEventCreateWithFlags(&c->ev_fork, hipEventDisableTiming));
  for (int i = 0; i < 2; ++i) {
    INIT_HIP(hipEventCreateWithFlags(&c->ev_mod[i], hipEventDisableTiming));
    INIT_HIP(hipEventCreateWithFlags(&c->ev_red[i], hipEventDisableTiming));
  }
  const int H = g.hidden, d = g.head_dim, nq = g.n_q_heads, nkv = g.n_kv_heads, I = g.inter;
  const size_t esz = c->esz;
  c->store.resize((size_t)g.n_layers * g.n_real_shards);
  c->gain_attn.resize(g.n_layers);
  c->gain_mlp.resize(g.n_layers);
  c->gains_loaded.assign(g.n_layers, 0);

  // weights: one allocation for the whole model
  size_t per_shard;
  if (c->fast) {
    per_shard = packed_tiles_bytes(H, c->nqkv) + packed_tiles_bytes(nq * d, H) + packed_tiles_bytes(H, 2 * I) +
                packed_tiles_bytes(I, H);
  } else {
    per_shard = ((size_t)H * c->nqkv + (size_t)nq * d * H + 3 * (size_t)H * I) * esz;
    per_shard = (per_shard + 255) / 256 * 256;
  }
  char* wbase = nullptr;
  INIT_TRY(dev_alloc(c, (void**)&wbase, per_shard * c->store.size(), false));
  c->weight_bytes = c->dev_bytes;
  char* gbase = nullptr;
  INIT_TRY(dev_alloc(c, (void**)&gbase, (size_t)g.n_layers * 2 * H * esz, false));
  // KV cache: K rows [B][nkv][s_cap][d]; V transposed [B][nkv][d][s_cap]; zero-filled so that no
  // kernel ever reads an uninitialised bit pattern
  const size_t kv_one = (size_t)g.max_batch * nkv * c->s_cap * d * esz;
  char* kvbase = nullptr;
  INIT_TRY(dev_alloc(c, (void**)&kvbase, kv_one * 2 * c->store.size(), true));
  for (size_t i = 0; i < c->store.size(); ++i) {
    LayerStore& L = c->store[i];
    char* p = wbase + per_shard * i;
    if (c->fast) {
      L.pqkv = p; p += packed_tiles_bytes(H, c->nqkv);
      L.po = p; p += packed_tiles_bytes(nq * d, H);
      L.pgu = p; p += packed_tiles_bytes(H, 2 * I);
      L.pd = p;
    } else {
      L.wq = p; p += (size_t)H * nq * d * esz;
      L.wk = p; p += (size_t)H * nkv * d * esz;
      L.wv = p; p += (size_t)H * nkv * d * esz;
      L.wo = p; p += (size_t)nq * d * H * esz;
      L.wg = p; p += (size_t)H * I * esz;
      L.wu = p; p += (size_t)H * I * esz;
      L.wd = p;
    }
    L.cache_k = kvbase + kv_one * 2 * i;
    L.cache_v = L.cache_k + kv_one;
  }
  for (int l = 0; l < g.n_layers; ++l) {
    c->gain_attn[l] = gbase + (size_t)(2 * l) * H * esz;
    c->gain_mlp[l] = gbase + (size_t)(2 * l + 1) * H * esz;
  }
  // rotary tables, made on the host in double precision
  {
    const int half = d / 2;
    std::vector<float> ct((size_t)c->s_cap * half), st((size_t)c->s_cap * half);
    for (int j = 0; j < half && !c->dry; ++j) {
      const double inv_freq = pow((double)g.rope_theta, -2.0 * j / (double)d);
      for (int p = 0; p < c->s_cap; ++p) {
        const double ang = (double)p * inv_freq;
        ct[(size_t)p * half + j] = (float)cos(ang);
        st[(size_t)p * half + j] = (float)sin(ang);
      }
    }
    INIT_TRY(dev_alloc(c, (void**)&c->cos_tab, ct.size() * 4, false));
    INIT_TRY(dev_alloc(c, (void**)&c->sin_tab, st.size() * 4, false));
    INIT_HIP(hipMemcpy(c->cos_tab, ct.data(), ct.size() * 4, hipMemcpyHostToDevice));
    INIT_HIP(hipMemcpy(c->sin_tab, st.data(), st.size() * 4, hipMemcpyHostToDevice));
  }
  // the words a kernel raises when something went wrong on the device (word 0: a bounded in-launch wait gave up;
  // word 1: ladder_embed met a token id outside the table): host memory that the device can write, so that the
  // host can look at them at the start of every call without synchronising anything
  INIT_HIP(hipHostMalloc((void**)&c->err_word, 64, hipHostMallocMapped));
  if (c->err_word) c->err_word[0] = c->err_word[1] = 0u;
  INIT_HIP(hipHostGetDevicePointer((void**)&c->err_word_dev, c->err_word, 0));
  // workspaces
  // rows x slots of the partial-sum buffers: a skinny call (rows <= 64) may use up to 8 split-K slots
  // per shard, a wide call uses one
  const size_t rows = (size_t)c->rows_cap;
  const size_t skinny_rows = rows < 64 ? rows : 64;
  const size_t row_slots = rows > 8 * skinny_rows ? rows : 8 * skinny_rows;
  INIT_TRY(dev_alloc(c, (void**)&c->x, rows * H * 4, false));
  INIT_TRY(dev_alloc(c, (void**)&c->pos_dev, 256, true));
  INIT_TRY(dev_alloc(c, (void**)&c->emb_stage, (size_t)g.max_batch * H * esz, false));
  for (int i = 0; i < 2; ++i) INIT_TRY(dev_alloc(c, (void**)&c->y[i], rows * H * esz, false));
  c->parts_cap = (size_t)g.n_real_shards * H * row_slots;
  for (int i = 0; i < 2; ++i) INIT_TRY(dev_alloc(c, (void**)&c->parts[i], c->parts_cap * 4, false));
  c->qkv_cap = (size_t)c->nqkv * row_slots;
  INIT_TRY(dev_alloc(c, (void**)&c->qkv, c->qkv_cap * 4, false));
  INIT_TRY(dev_alloc(c, (void**)&c->qbuf, rows * nq * d * esz, false));
  INIT_TRY(dev_alloc(c, (void**)&c->obuf, rows * nq * d * esz, false));
  INIT_TRY(dev_alloc(c, (void**)&c->act, rows * I * esz, false));
  if (!c->fast) INIT_TRY(dev_alloc(c, (void**)&c->gu, rows * 2 * I * 4, false));
  if (c->fast) {
    INIT_TRY(dev_alloc(c, (void**)&c->ssq_part, (size_t)((H + 63) / 64) * rows * 4, false));
    for (int i = 0; i < 2; ++i) INIT_TRY(dev_alloc(c, (void**)&c->y_rs[i], rows * 4, false));
    const size_t chunks = (size_t)(c->s_cap / 32);
    const size_t gq = nq / nkv;
    INIT_TRY(dev_alloc(c, (void**)&c->att_o, (size_t)g.max_batch * nkv * chunks * gq * d * 4, false));
    INIT_TRY(dev_alloc(c, (void**)&c->att_ml, (size_t)g.max_batch * nkv * chunks * gq * 2 * 4, false));
    c->fused = fused_usable(c);
    if (c->fused) {
      INIT_HIP(fused_decode_prepare(d, gq));
      int dev_id = 0, n_cu = 0;
      INIT_HIP(hipGetDevice(&dev_id));
      INIT_HIP(hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev_id));
      if (n_cu > 0) c->n_cu = n_cu;
      c->chain = g.decode_fused == 3;
      if (c->chain) {
        // persistent workgroups: as many as are resident together (a sizing pass assumes two per CU)
        c->chain_slots = c->dry ? 2 * c->n_cu : fused_chain_slots(d, (int)gq, c->n_cu);
        // (the launch lists are laid out for two resident workgroups per CU; with one, a step takes half as long again)
        if (c->chain_slots < 2 * c->n_cu) {
          c->err = "the chained decode kernel does not fit this device with two workgroups per CU";
          return bail(LADDER_E_HIP);
        }
        c->ring_n = c->n_mod + 1;
        c->n_fbuf = g.n_layers;
      }
      c->x_ring.assign((size_t)c->ring_n, nullptr);
      c->xop_ring.assign((size_t)c->ring_n, std::array<bf16_t*, 2>{nullptr, nullptr});
      c->ssq_ring.assign((size_t)c->ring_n, nullptr);
      c->f_q.assign((size_t)c->n_fbuf, nullptr);
      c->f_act.assign((size_t)c->n_fbuf, nullptr);
      c->f_o.assign((size_t)c->n_fbuf, nullptr);
      // (a chained step sizes its buffers for the rows it can have, not for 16: it has one of each per stream)
      const size_t ring_rows = c->chain ? (size_t)g.max_batch : 16, ring_slots = c->chain ? (size_t)fused_slots(g.max_batch) : 32;
      for (int i = 0; i < c->ring_n; ++i) {
        INIT_TRY(dev_alloc(c, (void**)&c->x_ring[(size_t)i], ring_rows * H * 4, true));
        for (int k = 0; k < 2; ++k) INIT_TRY(dev_alloc(c, (void**)&c->xop_ring[(size_t)i][(size_t)k], ring_slots * H * 2, true));
        INIT_TRY(dev_alloc(c, (void**)&c->ssq_ring[(size_t)i], (size_t)(H / 16) * 16 * 4, true));
      }
      for (int i = 0; i < c->n_fbuf; ++i) {
        INIT_TRY(dev_alloc(c, (void**)&c->f_q[(size_t)i], (size_t)32 * nq * d * 2, true));
        INIT_TRY(dev_alloc(c, (void**)&c->f_act[(size_t)i], ring_slots * I * 2, true));
        INIT_TRY(dev_alloc(c, (void**)&c->f_o[(size_t)i], (size_t)32 * nq * d * 2, true));
      }
      INIT_TRY(dev_alloc(c, (void**)&c->ssq_first, (size_t)(H / 16) * 16 * 4, true));
      INIT_TRY(dev_alloc(c, (void**)&c->t_done, (size_t)(c->n_mod + 1) * 8, true));
      // arrival counters of the attention jobs (a cache line each) and, for a chained step, the completion words of
      // its projections behind them: one range, cleared by the embedding kernel at the start of every step
      c->chain_launch_cap = c->chain ? 5 * g.n_layers + 1 : 0;
      c->n_zero_words = g.n_layers * FUSED_SYNC_WORDS * (c->chain ? 5 : 1) + c->chain_launch_cap * 32;
      INIT_TRY(dev_alloc(c, (void**)&c->att_done, (size_t)c->n_zero_words * 4, true));
      c->sync_words = c->att_done + (size_t)g.n_layers * FUSED_SYNC_WORDS;
      c->chain_claim_ctr = c->att_done + (size_t)g.n_layers * FUSED_SYNC_WORDS * 5;   // (behind the projections' words)
      if (c->chain) {
        // tables of the persistent launch, sized for the longest launch list a batch can have: at most 5 N + 1
        // launches, whose blocks (all projections' tiles and the attention workgroups) are dealt out over the slots
        const size_t blocks_max = (size_t)(c->nqkv + 2 * H + 2 * I) / 16 + (size_t)std::max(c->n_cu, g.max_batch * nkv);
        c->chain_items_cap = (size_t)(5 * g.n_layers + 1) * (1 + (blocks_max + (size_t)c->chain_slots - 1) / (size_t)c->chain_slots) + 1;
        c->chain_gemv_cap = 8 * g.n_layers + 8;
        c->chain_attn_cap = g.n_layers;
        INIT_TRY(dev_alloc(c, (void**)&c->chain_items_dev, (size_t)c->chain_slots * c->chain_items_cap * sizeof(StepItem), false));
        INIT_TRY(dev_alloc(c, (void**)&c->chain_gemv_dev, (size_t)c->chain_gemv_cap * sizeof(GemvJob), false));
        INIT_TRY(dev_alloc(c, (void**)&c->chain_attn_dev, (size_t)c->chain_attn_cap * sizeof(AttnJob), false));
        INIT_TRY(dev_alloc(c, (void**)&c->chain_surplus_dev, (size_t)c->chain_launch_cap * FUSED_CLAIM_MAX * sizeof(StepItem), false));
      }
      // arrival tickets start at zero and are put back to zero by the last arrival of every launch
      INIT_TRY(dev_alloc(c, (void**)&c->tk_att, (size_t)g.max_batch * nkv * 4, true));
    }
  }
#undef INIT_TRY
#undef INIT_HIP
  *out = c;
  return LADDER_OK;
}

int ladder_init(const ladder_config* cfg, void* hip_stream, ladder_ctx** out) { return init_impl(cfg, hip_stream, out, false); }

size_t ladder_workspace_bytes(const ladder_config* cfg) {
  ladder_ctx* c = nullptr;
  if (init_impl(cfg, nullptr, &c, true) != LADDER_OK || !c) return 0;
  const size_t bytes = c->dev_bytes - c->weight_bytes;
  delete c;
  return bytes;
}

size_t ladder_weight_bytes(const ladder_config* cfg) {
  ladder_ctx* c = nullptr;
  if (init_impl(cfg, nullptr, &c, true) != LADDER_OK || !c) return 0;
  const size_t bytes = c->weight_bytes;
  delete c;
  return bytes;
}

int ladder_set_wait_limit(ladder_ctx* c, int32_t max_polls, int32_t target_bias) {
  if (!c) return LADDER_E_ARG;
  if (max_polls < 1 || max_polls > (1 << 24) || target_bias < 0) return fail(c, LADDER_E_ARG, "max_polls must be in 1 .. 2^24, target_bias >= 0");
  c->wait_spins = max_polls;
  c->wait_bias = (unsigned)target_bias;
  c->fused_plan.clear();     // the launch list carries both: it is built again at the next step
  c->graph_stale = true;
  return LADDER_OK;
}

int ladder_load_layer(ladder_ctx* c, int32_t layer, int32_t shard, const ladder_layer_weights* w) {
  if (!c) return LADDER_E_ARG;
  if (!w || !w->wq || !w->wk || !w->wv || !w->wo || !w->w_gate || !w->w_up || !w->w_down)
    return fail(c, LADDER_E_ARG, "null weight pointer");
  const ladder_config& g = c->cfg;
  if (layer < 0 || layer >= g.n_layers || shard < 0 || shard >= g.n_real_shards)
    return fail(c, LADDER_E_SHAPE, "layer / shard out of range");
  if (shard == 0 && (!w->attn_norm || !w->mlp_norm)) return fail(c, LADDER_E_ARG, "null gain pointer");
  const int H = g.hidden, d = g.head_dim, nq = g.n_q_heads, nkv = g.n_kv_heads, I = g.inter;
  const size_t esz = c->esz;
  LayerStore& L = c->store[(size_t)layer * g.n_real_shards + shard];
  hipStream_t s = c->main;
  if (shard == 0) {
    HIP_TRY(c, hipMemcpyAsync(c->gain_attn[layer], w->attn_norm, H * esz, hipMemcpyDeviceToDevice, s));
    HIP_TRY(c, hipMemcpyAsync(c->gain_mlp[layer], w->mlp_norm, H * esz, hipMemcpyDeviceToDevice, s));
    c->gains_loaded[layer] = 1;
  }
  if (c->fast) {
    // a pure re-ordering: the packed tiles hold the stored bf16 values bit for bit
    HIP_TRY(c, launch_repack_tiles((const bf16_t*)w->wq, L.pqkv, H, nq * d, c->nqkv, 0, 0, s));
    HIP_TRY(c, launch_repack_tiles((const bf16_t*)w->wk, L.pqkv, H, nkv * d, c->nqkv, nq * d, 0, s));
    HIP_TRY(c, launch_repack_tiles((const bf16_t*)w->wv, L.pqkv, H, nkv * d, c->nqkv, (nq + nkv) * d, 0, s));
    HIP_TRY(c, launch_repack_tiles((const bf16_t*)w->wo, L.po, nq * d, H, H, 0, 0, s));
    HIP_TRY(c, launch_repack_tiles((const bf16_t*)w->w_gate, L.pgu, H, I, 2 * I, 0, 1, s));
    HIP_TRY(c, launch_repack_tiles((const bf16_t*)w->w_up, L.pgu, H, I, 2 * I, 0, 2, s));
    HIP_TRY(c, launch_repack_tiles((const bf16_t*)w->w_down, L.pd, I, H, H, 0, 0, s));
  } else {
    HIP_TRY(c, hipMemcpyAsync(L.wq, w->wq, (size_t)H * nq * d * esz, hipMemcpyDeviceToDevice, s));
    HIP_TRY(c, hipMemcpyAsync(L.wk, w->wk, (size_t)H * nkv * d * esz, hipMemcpyDeviceToDevice, s));
    HIP_TRY(c, hipMemcpyAsync(L.wv, w->wv, (size_t)H * nkv * d * esz, hipMemcpyDeviceToDevice, s));
    HIP_TRY(c, hipMemcpyAsync(L.wo, w->wo, (size_t)nq * d * H * esz, hipMemcpyDeviceToDevice, s));
    HIP_TRY(c, hipMemcpyAsync(L.wg, w->w_gate, (size_t)H * I * esz, hipMemcpyDeviceToDevice, s));
    HIP_TRY(c, hipMemcpyAsync(L.wu, w->w_up, (size_t)H * I * esz, hipMemcpyDeviceToDevice, s));
    HIP_TRY(c, hipMemcpyAsync(L.wd, w->w_down, (size_t)I * H * esz, hipMemcpyDeviceToDevice, s));
  }
  L.loaded = true;
  return LADDER_OK;
}

int ladder_set_peer_partials(ladder_ctx* c, const void* peers) {
  if (!c) return LADDER_E_ARG;
  if (peers && c->n_peers == 0) return fail(c, LADDER_E_SHAPE, "this configuration has no synthetic peers");
  // a captured decode step carries the peers' addresses in its kernel arguments: it is captured again at the
  // next step (decode_graph_step) when they change
  if ((const char*)peers != c->peers) c->graph_stale = true;
  c->peers = (const char*)peers;
  return LADDER_OK;
}

int ladder_load_kv(ladder_ctx* c, int32_t layer, int32_t shard, const void* k, const void* v, int32_t B, int32_t S) {
  if (!c) return LADDER_E_ARG;
  if (!k || !v) return fail(c, LADDER_E_ARG, "null k / v");
  const ladder_config& g = c->cfg;
  if (layer < 0 || layer >= g.n_layers || shard < 0 || shard >= g.n_real_shards)
    return fail(c, LADDER_E_SHAPE, "layer / shard out of range");
  if (B <= 0 || B > g.max_batch || S <= 0) return fail(c, LADDER_E_SHAPE, "B or S out of range");
  if (S > g.max_seq) return fail(c, LADDER_E_OVERFLOW, "S exceeds max_seq");
  LayerStore& L = c->store[(size_t)layer * g.n_real_shards + shard];
  HIP_TRY(c, launch_load_kv(k, v, L.cache_k, L.cache_v, B, g.n_kv_heads, S, g.head_dim, c->s_cap, c->bf16, c->main));
  L.kv_B = B;
  L.kv_S = S;
  bool all = true;
  for (auto& X : c->store) all = all && X.kv_B == B && X.kv_S == S;
  if (all) {
    c->pos = S;
    c->batch = B;
    hipLaunchKernelGGL(set_pos_kernel, dim3(1), dim3(1), 0, c->main, c->pos_dev, S);
    HIP_TRY(c, hipGetLastError());
  }
  return LADDER_OK;
}

int ladder_prefill(ladder_ctx* c, const void* x_in, int32_t B, int32_t T, void* x_out) {
  if (!c) return LADDER_E_ARG;
  if (!x_in || !x_out) return fail(c, LADDER_E_ARG, "null x_in / x_out");
  const ladder_config& g = c->cfg;
  if (B <= 0 || T <= 0) return fail(c, LADDER_E_ARG, "B and T must be positive");
  if (B > g.max_batch) return fail(c, LADDER_E_SHAPE, "B exceeds max_batch");
  if (T > g.max_seq) return fail(c, LADDER_E_OVERFLOW, "T exceeds max_seq");
  if (T > g.max_tokens) return fail(c, LADDER_E_SHAPE, "T exceeds max_tokens");
  if (c->peers && B * T > g.peer_rows) return fail(c, LADDER_E_SHAPE, "B*T exceeds peer_rows");
  int rc = check_device_error(c);
  if (rc) return rc;
  rc = all_loaded(c);
  if (rc) return rc;
  rc = forward(c, x_in, B, T, 0, x_out);
  if (rc) return rc;
  for (auto& X : c->store) { X.kv_B = 0; X.kv_S = 0; }
  c->pos = T;
  c->batch = B;
  hipLaunchKernelGGL(set_pos_kernel, dim3(1), dim3(1), 0, c->main, c->pos_dev, T);
  HIP_TRY(c, hipGetLastError());
  return LADDER_OK;
}

int ladder_decode_step(ladder_ctx* c, const void* x_in, void* x_out) {
  if (!c) return LADDER_E_ARG;
  if (!x_in || !x_out) return fail(c, LADDER_E_ARG, "null x_in / x_out");
  if (c->batch <= 0 || c->pos <= 0) return fail(c, LADDER_E_STATE, "decode before prefill / load_kv");
  if (c->pos + 1 > c->cfg.max_seq) return fail(c, LADDER_E_OVERFLOW, "KV cache is full");
  if (c->peers && c->batch > c->cfg.peer_rows) return fail(c, LADDER_E_SHAPE, "batch exceeds peer_rows");
  int rc = check_device_error(c);
  if (rc) return rc;
  rc = all_loaded(c);
  if (rc) return rc;
  if (c->fast && c->cfg.decode_graph && !c->prof) {
    rc = decode_graph_step(c, x_in, x_out);
    if (rc) return rc;
  } else if (c->fused) {
    rc = decode_fused_step(c, x_in, x_out);
    if (rc) return rc;
  } else {
    rc = forward(c, x_in, c->batch, 1, c->pos, x_out);
    if (rc) return rc;
    hipLaunchKernelGGL(inc_pos_kernel, dim3(1), dim3(1), 0, c->main, c->pos_dev);
    HIP_TRY(c, hipGetLastError());
  }
  c->pos += 1;
  return LADDER_OK;
}

static int stage_args(ladder_ctx* c, const float* res, const float* att, const float* mlp, float* r, float* a, float* m, StageIo* st) {
  if (!res || !r || !a || !m) return fail(c, LADDER_E_ARG, "null residual_in / output tensor");
  if (r == a || r == m || a == m) return fail(c, LADDER_E_ARG, "the three output tensors must be distinct");
  for (const void* p : {(const void*)res, (const void*)att, (const void*)mlp, (const void*)r, (const void*)a, (const void*)m})
    if ((uintptr_t)p & 15) return fail(c, LADDER_E_ARG, "stage tensors must be 16-byte aligned");
  for (int q = 1; q <= c->n_mod; ++q)
    if (lag_of(c, q) != 2) return fail(c, LADDER_E_STATE, "pipeline-stage calls need the ladder wiring in every layer");
  *st = StageIo{res, att, mlp, r, a, m};
  return LADDER_OK;
}

int ladder_prefill_stage(ladder_ctx* c, const float* residual_in, const float* attn_in, const float* mlp_in, int32_t B, int32_t T,
                         float* residual_out, float* attn_out, float* mlp_out) {
  if (!c) return LADDER_E_ARG;
  StageIo st{};
  int rc = stage_args(c, residual_in, attn_in, mlp_in, residual_out, attn_out, mlp_out, &st);
  if (rc) return rc;
  const ladder_config& g = c->cfg;
  if (B <= 0 || T <= 0) return fail(c, LADDER_E_ARG, "B and T must be positive");
  if (B > g.max_batch) return fail(c, LADDER_E_SHAPE, "B exceeds max_batch");
  if (T > g.max_seq) return fail(c, LADDER_E_OVERFLOW, "T exceeds max_seq");
  if (T > g.max_tokens) return fail(c, LADDER_E_SHAPE, "T exceeds max_tokens");
  if (c->peers && B * T > g.peer_rows) return fail(c, LADDER_E_SHAPE, "B*T exceeds peer_rows");
  rc = check_device_error(c);
  if (rc) return rc;
  rc = all_loaded(c);
  if (rc) return rc;
  rc = forward(c, nullptr, B, T, 0, nullptr, &st);
  if (rc) return rc;
  for (auto& X : c->store) { X.kv_B = 0; X.kv_S = 0; }
  c->pos = T;
  c->batch = B;
  hipLaunchKernelGGL(set_pos_kernel, dim3(1), dim3(1), 0, c->main, c->pos_dev, T);
  HIP_TRY(c, hipGetLastError());
  return LADDER_OK;
}

int ladder_decode_step_stage(ladder_ctx* c, const float* residual_in, const float* attn_in, const float* mlp_in,
                             float* residual_out, float* attn_out, float* mlp_out) {
  if (!c) return LADDER_E_ARG;
  StageIo st{};
  int rc = stage_args(c, residual_in, attn_in, mlp_in, residual_out, attn_out, mlp_out, &st);
  if (rc) return rc;
  if (c->batch <= 0 || c->pos <= 0) return fail(c, LADDER_E_STATE, "decode before prefill / load_kv");
  if (c->pos + 1 > c->cfg.max_seq) return fail(c, LADDER_E_OVERFLOW, "KV cache is full");
  if (c->peers && c->batch > c->cfg.peer_rows) return fail(c, LADDER_E_SHAPE, "batch exceeds peer_rows");
  rc = check_device_error(c);
  if (rc) return rc;
  rc = all_loaded(c);
  if (rc) return rc;
  // (launched eagerly also where ladder_decode_step replays a captured graph: the graph holds that call's staging)
  if (c->fused) {
    rc = decode_fused_step(c, nullptr, nullptr, &st);
    if (rc) return rc;
  } else {
    rc = forward(c, nullptr, c->batch, 1, c->pos, nullptr, &st);
    if (rc) return rc;
    hipLaunchKernelGGL(inc_pos_kernel, dim3(1), dim3(1), 0, c->main, c->pos_dev);
    HIP_TRY(c, hipGetLastError());
  }
  c->pos += 1;
  return LADDER_OK;
}

void ladder_free(ladder_ctx* c) {
  if (!c) return;
  (void)hipStreamSynchronize(c->main);
  for (hipStream_t* st : {&c->s_attn, &c->s_mlp, &c->side}) {
    if (*st) {
      (void)hipStreamSynchronize(*st);
      (void)hipStreamDestroy(*st);
    }
  }
  if (c->graph_exec) (void)hipGraphExecDestroy(c->graph_exec);
  if (c->ev_begin) (void)hipEventDestroy(c->ev_begin);
  if (c->ev_end) (void)hipEventDestroy(c->ev_end);
  if (c->ev_fork) (void)hipEventDestroy(c->ev_fork);
  for (auto& r : c->prof_pending) {
    (void)hipEventDestroy(r.start);
    (void)hipEventDestroy(r.stop);
  }
  for (auto e : c->prof_pool) (void)hipEventDestroy(e);
  for (int i = 0; i < 2; ++i) {
    if (c->ev_mod[i]) (void)hipEventDestroy(c->ev_mod[i]);
    if (c->ev_red[i]) (void)hipEventDestroy(c->ev_red[i]);
  }
  for (void* p : c->allocs) (void)hipFree(p);
  if (c->err_word) (void)hipHostFree(c->err_word);
  delete c;
}

const char* ladder_last_error(const ladder_ctx* c) { return c ? c->err.c_str() : g_init_error.c_str(); }

int ladder_position(const ladder_ctx* c, int32_t* pos, int32_t* batch) {
  if (!c) return LADDER_E_ARG;
  if (pos) *pos = c->pos;
  if (batch) *batch = c->batch;
  return LADDER_OK;
}

size_t ladder_device_bytes(const ladder_ctx* c) { return c ? c->dev_bytes : 0; }

int ladder_profile_enable(ladder_ctx* c, int32_t on) {
  if (!c) return LADDER_E_ARG;
  if (!on) {
    int rc = collect_profile(c);
    if (rc) return rc;
  }
  c->prof = on != 0;
  return LADDER_OK;
}

int ladder_profile_read(ladder_ctx* c, int32_t cls, int64_t* launches, double* total_ms) {
  if (!c) return LADDER_E_ARG;
  if (cls < 0 || cls >= LADDER_K_COUNT) return fail(c, LADDER_E_ARG, "unknown kernel class");
  int rc = collect_profile(c);
  if (rc) return rc;
  if (launches) *launches = c->prof_n[cls];
  if (total_ms) *total_ms = c->prof_ms[cls];
  return LADDER_OK;
}

int ladder_load_head(ladder_ctx* c, const void* table, const void* final_norm, const void* w_lm, int32_t vocab,
                     int32_t vocab_local) {
  if (!c) return LADDER_E_ARG;
  if (!table || !final_norm || !w_lm) return fail(c, LADDER_E_ARG, "null table / final_norm / w_lm");
  if (vocab <= 0 || vocab_local <= 0 || vocab_local > vocab) return fail(c, LADDER_E_SHAPE, "vocab sizes out of range");
  if (c->head_table) return fail(c, LADDER_E_STATE, "the head is already loaded");
  const ladder_config& g = c->cfg;
  const int H = g.hidden;
  const size_t esz = c->esz;
  int rc;
  if ((rc = dev_alloc(c, (void**)&c->head_table, (size_t)vocab * H * esz, false))) return rc;
  if ((rc = dev_alloc(c, (void**)&c->head_y, (size_t)g.max_batch * H * esz, false))) return rc;
  if ((rc = dev_alloc(c, (void**)&c->head_logits, (size_t)g.max_batch * vocab_local * 4, false))) return rc;
  HIP_TRY(c, hipMemcpyAsync(c->head_table, table, (size_t)vocab * H * esz, hipMemcpyDeviceToDevice, c->main));
  c->head_fast = c->fast && vocab_local % 16 == 0;
  if ((rc = dev_alloc(c, (void**)&c->head_gain, (size_t)H * esz, false))) return rc;
  HIP_TRY(c, hipMemcpyAsync(c->head_gain, final_norm, (size_t)H * esz, hipMemcpyDeviceToDevice, c->main));
  if (c->head_fast) {   // packed tiles, as for the block projections
    if ((rc = dev_alloc(c, (void**)&c->head_wp, (size_t)H * vocab_local * 2, false))) return rc;
    HIP_TRY(c, launch_repack_tiles((const bf16_t*)w_lm, c->head_wp, H, vocab_local, vocab_local, 0, 0, c->main));
  } else {
    if ((rc = dev_alloc(c, (void**)&c->head_w, (size_t)H * vocab_local * esz, false))) return rc;
    HIP_TRY(c, hipMemcpyAsync(c->head_w, w_lm, (size_t)H * vocab_local * esz, hipMemcpyDeviceToDevice, c->main));
  }
  c->vocab = vocab;
  c->vocab_local = vocab_local;
  return LADDER_OK;
}

int ladder_embed(ladder_ctx* c, const int32_t* tokens, int32_t rows, void* x_out) {
  if (!c) return LADDER_E_ARG;
  if (!tokens || !x_out) return fail(c, LADDER_E_ARG, "null tokens / x_out");
  if (!c->head_table) return fail(c, LADDER_E_STATE, "the head is not loaded");
  if (rows <= 0) return fail(c, LADDER_E_ARG, "rows must be positive");
  if ((long long)rows > (long long)c->cfg.max_batch * c->cfg.max_tokens) return fail(c, LADDER_E_SHAPE, "rows exceed max_batch * max_tokens");
  const int rc = check_device_error(c);
  if (rc) return rc;
  HIP_TRY(c, launch_embed_gather(tokens, c->head_table, x_out, rows, c->cfg.hidden, c->vocab, c->err_word_dev ? c->err_word_dev + 1 : nullptr, c->bf16, c->main));
  return LADDER_OK;
}

// final norm -> output projection -> (arg max) with the normed rows in y and the logits in `logits`
static int head_body(ladder_ctx* c, const float* x, int rows, char* y, float* logits, int32_t* tokens_out) {
  const ladder_config& g = c->cfg;
  const int H = g.hidden, V = c->vocab_local;
  hipStream_t s = c->main;
  HIP_TRY(c, launch_head_norm(x, c->head_gain, y, rows, H, g.rms_eps, c->bf16, s));
  if (!c->head_fast) {
    HIP_TRY(c, launch_gemm_generic(y, c->head_w, logits, rows, V, H, V, 0, c->bf16, s));
  } else if (rows <= 64) {
    GemvArgs a{};
    a.x = (const bf16_t*)y; a.ldx = H; a.wp = c->head_wp; a.M = rows; a.K = H; a.N = V; a.ksplit = 1;
    a.out = logits; a.out_stride = (size_t)rows * V; a.slot0 = 0; a.epilogue = 0;
    HIP_TRY(c, launch_gemv(a, s));
  } else {
    GemmArgs a{};
    a.x = (const bf16_t*)y; a.ldx = H; a.wp = c->head_wp; a.M = rows; a.K = H; a.N = V; a.out = logits; a.epilogue = 0;
    HIP_TRY(c, launch_gemm_mfma(a, s));
  }
  if (tokens_out) HIP_TRY(c, launch_argmax(logits, tokens_out, rows, V, s));
  return LADDER_OK;
}

int ladder_head(ladder_ctx* c, const float* x, int32_t rows, float* logits_out, int32_t* tokens_out) {
  if (!c) return LADDER_E_ARG;
  if (!x || (!logits_out && !tokens_out)) return fail(c, LADDER_E_ARG, "null x, or neither logits_out nor tokens_out");
  if (!c->head_table) return fail(c, LADDER_E_STATE, "the head is not loaded");
  if (rows <= 0) return fail(c, LADDER_E_ARG, "rows must be positive");
  if (rows > c->cfg.max_batch) return fail(c, LADDER_E_SHAPE, "rows exceed max_batch (the head serves one position per sequence)");
  return head_body(c, x, rows, c->head_y, logits_out ? logits_out : c->head_logits, tokens_out);
}

int ladder_head_static(ladder_ctx* c, const float* x, int32_t rows, int32_t* tokens_out) {
  if (!c) return LADDER_E_ARG;
  if (!x || !tokens_out) return fail(c, LADDER_E_ARG, "null x / tokens_out");
  if (!c->head_table) return fail(c, LADDER_E_STATE, "the head is not loaded");
  if (rows <= 0) return fail(c, LADDER_E_ARG, "rows must be positive");
  if (rows > c->cfg.max_batch) return fail(c, LADDER_E_SHAPE, "rows exceed max_batch (the head serves one position per sequence)");
  if (rows > LADDER_HEAD_STATIC_MAX_ROWS || c->cfg.hidden > LADDER_HEAD_STATIC_MAX_HIDDEN || c->vocab_local > LADDER_HEAD_STATIC_MAX_VOCAB)
    return fail(c, LADDER_E_SHAPE, "ladder_head_static: rows, hidden or vocab_local beyond the LADDER_HEAD_STATIC_MAX_* limits of the static scratch");
  int dev = -1;
  HIP_TRY(c, hipGetDevice(&dev));
  if (dev != c->device || !c->static_scratch) return fail(c, LADDER_E_STATE, "ladder_head_static: the context's device is not the current device");
  char* y = (char*)c->static_scratch;                                   // the looked-up device address, never the array's name
  float* logits = (float*)((char*)c->static_scratch + HEAD_STATIC_Y_BYTES);
  return head_body(c, x, rows, y, logits, tokens_out);
}

int ladder_calibration_copy(ladder_ctx* c, void* dst, const void* src, size_t bytes) {
  if (!c || !dst || !src) return LADDER_E_ARG;
  if (bytes == 0 || (bytes & 15) || ((uintptr_t)dst & 15) || ((uintptr_t)src & 15)) return fail(c, LADDER_E_SHAPE, "copy: pointers and size must be multiples of 16 bytes");
  const size_t n16 = bytes / 16;
  const int blocks = (int)std::min<size_t>((n16 + 255) / 256, 256 * 32);
  hipLaunchKernelGGL(calibration_copy_kernel, dim3(blocks), dim3(256), 0, c->main, (const uint4*)src, (uint4*)dst, n16);
  HIP_TRY(c, hipGetLastError());
  return LADDER_OK;
}

int ladder_timeline_enable(ladder_ctx* c, int32_t on) {
  if (!c) return LADDER_E_ARG;
  if (!c->chain) return fail(c, LADDER_E_STATE, "the timeline belongs to the chained decode step (decode_fused = 3 on the fused path)");
  if (on && c->cfg.decode_graph) return fail(c, LADDER_E_STATE, "the timeline is recorded by eager steps (decode_graph = 0)");
  if (on && !c->chain_tl_dev) {
    const size_t bytes = (size_t)c->chain_slots * c->chain_items_cap * 3 * sizeof(unsigned long long);
    const int rc = dev_alloc(c, (void**)&c->chain_tl_dev, bytes, true);
    if (rc) return rc;
  }
  HIP_TRY(c, hipStreamSynchronize(c->s_attn));
  c->timeline_on = on != 0;
  return LADDER_OK;
}

int ladder_timeline_read(ladder_ctx* c, ladder_timeline_rec* out, int64_t cap, int64_t* n_out, double* ticks_per_us) {
  if (!c || !n_out) return LADDER_E_ARG;
  if (!c->chain || !c->chain_tl_dev) return fail(c, LADDER_E_STATE, "no timeline: ladder_timeline_enable first");
  if (c->fused_plan.empty() || c->chain_items <= 0) return fail(c, LADDER_E_STATE, "no timeline: no decode step has run");
  HIP_TRY(c, hipStreamSynchronize(c->s_attn));
  const size_t n_items = (size_t)c->chain_items;
  std::vector<unsigned long long> t((size_t)c->chain_slots * n_items * 3);
  HIP_TRY(c, hipMemcpy(t.data(), c->chain_tl_dev, t.size() * sizeof(unsigned long long), hipMemcpyDeviceToHost));
  int64_t n = 0;
  for (size_t w = 0; w < c->chain_meta.size(); ++w)
    for (size_t i = 0; i < c->chain_meta[w].size(); ++i, ++n) {
      const ladder_ctx::ChainMeta& m = c->chain_meta[w][i];
      if (m.kind < 0) { --n; continue; }   // (a surplus list's item: its blocks are not recorded)
      if (!out || n >= cap) continue;
      const unsigned long long* ts = t.data() + (w * n_items + i) * 3;
      out[n] = ladder_timeline_rec{(int32_t)w, m.launch, m.kind, m.tiles, m.weight_bytes, ts[0], ts[1], ts[2]};
    }
  *n_out = n;
  if (ticks_per_us) *ticks_per_us = (double)c->wall_khz / 1000.0;
  return LADDER_OK;
}

int ladder_profile_reset(ladder_ctx* c) {
  if (!c) return LADDER_E_ARG;
  int rc = collect_profile(c);
  if (rc) return rc;
  for (int i = 0; i < LADDER_K_COUNT; ++i) {
    c->prof_n[i] = 0;
    c->prof_ms[i] = 0.0;
  }
  return LADDER_OK;
}

}  // extern "C"
