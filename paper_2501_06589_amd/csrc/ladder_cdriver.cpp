// ladder_cdriver: a host-only C++ program that drives the C-ABI of libladder.so without Python.
//
//   ladder_cdriver [--layers N] [--steps K] [--warmup W] [--kv S] [--copies C]
//
// It builds the 70B-shard decode configuration (one tensor-parallel rank at R = 8: hidden 8192,
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

int main(int argc, char** argv) {
  const int n_layers = arg_int(argc, argv, "--layers", 80);
  const int steps = arg_int(argc, argv, "--steps", 32);
  const int warmup = arg_int(argc, argv, "--warmup", 4);
  const int kv = arg_int(argc, argv, "--kv", 1024);
  const int copies = arg_int(argc, argv, "--copies", 4);
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
  cfg.overlap_modules = 1; cfg.decode_graph = 0; cfg.decode_fused = 1; cfg.rms_eps = 1e-5f; cfg.rope_theta = 500000.0f;

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
