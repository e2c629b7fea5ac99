// ladder_cdriver: a host-only C++ program that drives the C-ABI of libladder.so without Python.
//
//   ladder_cdriver [--layers N] [--steps K] [--warmup W] [--kv S] [--copies C] [--fused F]   (F = decode_fused: 3 chained step (default), 1, 2, 0)
//   ladder_cdriver --prefill 1 [--layers N] [--steps K] [--warmup W] [--batch B] [--tokens T]
//
// With --prefill 1 it builds the prefill workload's shard instead (one rank at R = 4: hidden 8192, 16 q / 2 kv heads,
// d = 128, intermediate 7168, 3 synthetic peers), fills weights, peers and embeddings with pseudo-random bf16
// values (matrix-core power, and with it the clock, depends on the operands' bit patterns) and times K prefill
// calls of B x T tokens: the target for hardware counters on the prefill GEMMs.
//
// Without it, it builds the 70B-shard decode configuration (one tensor-parallel rank at R = 8: hidden 8192,
// 8 q heads on 1 kv head, d = 128, intermediate 3584, batch 4, 7 synthetic peer partial sums per
// module), fills weights, KV cache and peers with constant bf16 patterns (hipMemsetD16: the values
// are irrelevant to timing and to the bytes moved), runs C plain copies of 1 GiB (the known-size
// dispatches hardware byte counters are scaled by), then W + K decode steps, and prints the time per
// step.  It exists for two things: as a C usage example of the boundary, and as a profiling target
// for counter collection (rocprofv3 --pmc), which on some stacks cannot follow a Python process.
// Results of the computation are checked elsewhere (the parity tests go through the same entry points).
#include <hip/hip_runtime.h>

#include <chrono>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "../../include/ladder.h"

#define HIP_OK(x)                                                                                   \
  do {                                                                                              \
    hipError_t e_ = (x);                                                                            \
    if (e_ != hipSuccess) {                                                                         \
      fprintf(stderr, "HIP error %s at %s:%d\n", hipGetErrorString(e_), __FILE__, __LINE__);        \
      return 1;                                                                                     \
    }                                                                                               \
  } while (0)
#define LADDER_OK_OR_DIE(x)                                                                         \
  do {                                                                                              \
    int rc_ = (x);                                                                                  \
    if (rc_ != LADDER_OK) {                                                                         \
      fprintf(stderr, "ladder error %d (%s) at %s:%d\n", rc_, ladder_last_error(ctx), __FILE__, __LINE__); \
      return 1;                                                                                     \
    }                                                                                               \
  } while (0)

static int arg_int(int argc, char** argv, const char* name, int dflt) {
  for (int i = 1; i + 1 < argc; ++i)
    if (!strcmp(argv[i], name)) return atoi(argv[i + 1]);
  return dflt;
}

// pseudo-random bf16 values with magnitudes in [lo_exp pattern, twice that) and random signs / mantissas
static hipError_t dmalloc_random16(size_t n, unsigned short exp_pattern, void** out) {
  std::vector<unsigned short> h(n);
  unsigned long long st = 0x9E3779B97F4A7C15ull ^ (unsigned long long)n;
  for (size_t i = 0; i < n; ++i) {
    st ^= st << 13; st ^= st >> 7; st ^= st << 17;      // xorshift64
    h[i] = (unsigned short)(exp_pattern | ((unsigned)(st >> 20) & 0x807Fu));
  }
  hipError_t e = hipMalloc(out, n * 2);
  if (e != hipSuccess) return e;
  return hipMemcpy(*out, h.data(), n * 2, hipMemcpyHostToDevice);
}

static int run_prefill(int argc, char** argv) {
  const int n_layers = arg_int(argc, argv, "--layers", 2);
  const int steps = arg_int(argc, argv, "--steps", 3);
  const int warmup = arg_int(argc, argv, "--warmup", 1);
  const int B = arg_int(argc, argv, "--batch", 16);
  const int T = arg_int(argc, argv, "--tokens", 2048);
  const int H = 8192, NQ = 16, NKV = 2, D = 128, I = 7168, R = 4;
  if (n_layers < 1 || steps < 1 || warmup < 0 || B < 1 || T < 1) {
    fprintf(stderr, "bad arguments\n");
    return 2;
  }
  ladder_config cfg;
  memset(&cfg, 0, sizeof(cfg));
  cfg.n_layers = n_layers; cfg.hidden = H; cfg.n_q_heads = NQ; cfg.n_kv_heads = NKV; cfg.head_dim = D; cfg.inter = I;
  cfg.tp_degree = R; cfg.n_real_shards = 1; cfg.max_batch = B; cfg.max_seq = T + 8;
  cfg.max_tokens = T; cfg.dtype = LADDER_BF16; cfg.wiring = LADDER_WIRING_LADDER; cfg.n_standard_layers = 0;
  cfg.reduce_on_side_stream = 1; cfg.peer_pool = 2; cfg.peer_rows = B * T; cfg.kernel_path = LADDER_PATH_AUTO;
  cfg.overlap_modules = 1; cfg.decode_graph = 0; cfg.decode_fused = 1; cfg.rms_eps = 1e-5f; cfg.rope_theta = 500000.0f;
  ladder_ctx* ctx = nullptr;
  LADDER_OK_OR_DIE(ladder_init(&cfg, nullptr, &ctx));
  const unsigned short ONE = 0x3f80, SMALL = 0x3c00;   // bf16 exponent patterns of 1.0 and 2^-7
  void *g1, *g2, *wq, *wk, *wv, *wo, *wg, *wu, *wd;
  HIP_OK(dmalloc_random16(H, ONE, &g1));
  HIP_OK(dmalloc_random16(H, ONE, &g2));
  HIP_OK(hipMemsetD16(g1, ONE, H));     // gains of exactly 1
  HIP_OK(hipMemsetD16(g2, ONE, H));
  HIP_OK(dmalloc_random16((size_t)H * NQ * D, SMALL, &wq));
  HIP_OK(dmalloc_random16((size_t)H * NKV * D, SMALL, &wk));
  HIP_OK(dmalloc_random16((size_t)H * NKV * D, SMALL, &wv));
  HIP_OK(dmalloc_random16((size_t)NQ * D * H, SMALL, &wo));
  HIP_OK(dmalloc_random16((size_t)H * I, SMALL, &wg));
  HIP_OK(dmalloc_random16((size_t)H * I, SMALL, &wu));
  HIP_OK(dmalloc_random16((size_t)I * H, SMALL, &wd));
  ladder_layer_weights lw = {g1, wq, wk, wv, wo, g2, wg, wu, wd};
  for (int l = 0; l < n_layers; ++l) LADDER_OK_OR_DIE(ladder_load_layer(ctx, l, 0, &lw));
  void* peers;
  {   // (the peers only pass through an epilogue: a constant pattern)
    const size_t n = (size_t)cfg.peer_pool * (R - 1) * B * T * H;
    HIP_OK(hipMalloc(&peers, n * 2));
    HIP_OK(hipMemsetD16(peers, SMALL, n));
  }
  LADDER_OK_OR_DIE(ladder_set_peer_partials(ctx, peers));
  void *x_in, *x_out;
  HIP_OK(dmalloc_random16((size_t)B * T * H, ONE, &x_in));
  HIP_OK(hipMalloc(&x_out, (size_t)B * T * H * 4));
  HIP_OK(hipDeviceSynchronize());
  fprintf(stderr, "[cdriver] prefill: %d layers, %d x %d tokens, %.2f GiB on device\n", n_layers, B, T,
          ladder_device_bytes(ctx) / 1073741824.0);
  for (int i = 0; i < warmup; ++i) LADDER_OK_OR_DIE(ladder_prefill(ctx, x_in, B, T, x_out));
  HIP_OK(hipDeviceSynchronize());
  const auto t0 = std::chrono::steady_clock::now();
  for (int i = 0; i < steps; ++i) LADDER_OK_OR_DIE(ladder_prefill(ctx, x_in, B, T, x_out));
  HIP_OK(hipDeviceSynchronize());
  const double ms = std::chrono::duration<double, std::milli>(std::chrono::steady_clock::now() - t0).count() / steps;
  const double params = (double)H * (NQ + 2 * NKV) * D + (double)NQ * D * H + 3.0 * H * I;
  const double gemm_tflops = 2.0 * params * n_layers * B * T / (ms * 1e-3) / 1e12;
  float first = 0.f;
  HIP_OK(hipMemcpy(&first, x_out, 4, hipMemcpyDeviceToHost));
  printf("{\"driver\": \"ladder_cdriver\", \"mode\": \"prefill\", \"n_layers\": %d, \"rows\": %d, \"steps\": %d, "
         "\"ms_per_call\": %.3f, \"gemm_TFLOPs_over_call_time\": %.1f, \"x_out_0\": %g}\n",
         n_layers, B * T, steps, ms, gemm_tflops, first);
  ladder_free(ctx);
  return 0;
}

int main(int argc, char** argv) {
  if (arg_int(argc, argv, "--prefill", 0)) return run_prefill(argc, argv);
  const int n_layers = arg_int(argc, argv, "--layers", 80);
  const int steps = arg_int(argc, argv, "--steps", 32);
  const int warmup = arg_int(argc, argv, "--warmup", 4);
  const int kv = arg_int(argc, argv, "--kv", 1024);
  const int copies = arg_int(argc, argv, "--copies", 4);
  const int fused = arg_int(argc, argv, "--fused", 3);
  const int H = 8192, NQ = 8, NKV = 1, D = 128, I = 3584, R = 8, B = 4;
  if (n_layers < 1 || steps < 1 || warmup < 0 || kv < 1 || copies < 0) {
    fprintf(stderr, "bad arguments\n");
    return 2;
  }

  ladder_config cfg;
  memset(&cfg, 0, sizeof(cfg));
  cfg.n_layers = n_layers; cfg.hidden = H; cfg.n_q_heads = NQ; cfg.n_kv_heads = NKV; cfg.head_dim = D; cfg.inter = I;
  cfg.tp_degree = R; cfg.n_real_shards = 1; cfg.max_batch = B; cfg.max_seq = kv + warmup + steps + 8;
  cfg.max_tokens = 1; cfg.dtype = LADDER_BF16; cfg.wiring = LADDER_WIRING_LADDER; cfg.n_standard_layers = 0;
  cfg.reduce_on_side_stream = 1; cfg.peer_pool = 2; cfg.peer_rows = B; cfg.kernel_path = LADDER_PATH_AUTO;
  cfg.overlap_modules = 1; cfg.decode_graph = 0; cfg.decode_fused = fused; cfg.rms_eps = 1e-5f; cfg.rope_theta = 500000.0f;

  ladder_ctx* ctx = nullptr;
  LADDER_OK_OR_DIE(ladder_init(&cfg, nullptr, &ctx));

  // one set of caller-side tensors, reused for every layer (load_layer copies / repacks them)
  auto dmalloc16 = [](size_t n, unsigned short pattern, void** out) -> hipError_t {
    hipError_t e = hipMalloc(out, n * 2);
    if (e != hipSuccess) return e;
    return hipMemsetD16(*out, pattern, n);
  };
  const unsigned short ONE = 0x3f80, SMALL = 0x3c00;   // bf16 1.0 and 2^-7
  void *g1, *g2, *wq, *wk, *wv, *wo, *wg, *wu, *wd;
  HIP_OK(dmalloc16(H, ONE, &g1));
  HIP_OK(dmalloc16(H, ONE, &g2));
  HIP_OK(dmalloc16((size_t)H * NQ * D, SMALL, &wq));
  HIP_OK(dmalloc16((size_t)H * NKV * D, SMALL, &wk));
  HIP_OK(dmalloc16((size_t)H * NKV * D, SMALL, &wv));
  HIP_OK(dmalloc16((size_t)NQ * D * H, SMALL, &wo));
  HIP_OK(dmalloc16((size_t)H * I, SMALL, &wg));
  HIP_OK(dmalloc16((size_t)H * I, SMALL, &wu));
  HIP_OK(dmalloc16((size_t)I * H, SMALL, &wd));
  ladder_layer_weights lw = {g1, wq, wk, wv, wo, g2, wg, wu, wd};
  void *kbuf, *vbuf;
  HIP_OK(dmalloc16((size_t)B * NKV * kv * D, SMALL, &kbuf));
  HIP_OK(dmalloc16((size_t)B * NKV * kv * D, SMALL, &vbuf));
  for (int l = 0; l < n_layers; ++l) {
    LADDER_OK_OR_DIE(ladder_load_layer(ctx, l, 0, &lw));
    LADDER_OK_OR_DIE(ladder_load_kv(ctx, l, 0, kbuf, vbuf, B, kv));
  }
  void* peers;
  HIP_OK(dmalloc16((size_t)cfg.peer_pool * (R - 1) * B * H, SMALL, &peers));
  LADDER_OK_OR_DIE(ladder_set_peer_partials(ctx, peers));
  void *x_in, *x_out;
  HIP_OK(dmalloc16((size_t)B * H, SMALL, &x_in));
  HIP_OK(hipMalloc(&x_out, (size_t)B * H * 4));
  HIP_OK(hipDeviceSynchronize());
  fprintf(stderr, "[cdriver] %d layers, %.2f GiB on device, cache preloaded with %d positions\n", n_layers,
          ladder_device_bytes(ctx) / 1073741824.0, kv);

  if (copies > 0) {
    const size_t gib = (size_t)1 << 30;
    void *src, *dst;
    HIP_OK(hipMalloc(&src, gib));
    HIP_OK(hipMalloc(&dst, gib));
    HIP_OK(hipMemset(src, 1, gib));
    for (int i = 0; i < copies; ++i) LADDER_OK_OR_DIE(ladder_calibration_copy(ctx, dst, src, gib));
    HIP_OK(hipDeviceSynchronize());
    HIP_OK(hipFree(src));
    HIP_OK(hipFree(dst));
  }

  for (int i = 0; i < warmup; ++i) LADDER_OK_OR_DIE(ladder_decode_step(ctx, x_in, x_out));
  HIP_OK(hipDeviceSynchronize());
  const auto t0 = std::chrono::steady_clock::now();
  for (int i = 0; i < steps; ++i) LADDER_OK_OR_DIE(ladder_decode_step(ctx, x_in, x_out));
  HIP_OK(hipDeviceSynchronize());
  const double ms = std::chrono::duration<double, std::milli>(std::chrono::steady_clock::now() - t0).count() / steps;
  int32_t pos = 0, batch = 0;
  LADDER_OK_OR_DIE(ladder_position(ctx, &pos, &batch));
  std::vector<float> host((size_t)B * H);
  HIP_OK(hipMemcpy(host.data(), x_out, host.size() * 4, hipMemcpyDeviceToHost));
  printf("{\"driver\": \"ladder_cdriver\", \"n_layers\": %d, \"batch\": %d, \"position\": %d, \"steps\": %d, "
         "\"ms_per_step\": %.4f, \"tokens_per_s\": %.1f, \"x_out_0\": %g}\n",
         n_layers, batch, pos, steps, ms, B * 1e3 / ms, host[0]);
  ladder_free(ctx);
  return 0;
}
