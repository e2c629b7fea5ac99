// Shared declarations of the HIP sources: storage-type helpers and the host-side launchers
// that the API file calls.  gfx950 only.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

typedef uint16_t bf16_t;  // bfloat16 bit pattern

__device__ __forceinline__ float bf16_to_f32(bf16_t v) { return __uint_as_float(((uint32_t)v) << 16); }

// round to nearest even; inputs here are finite
__device__ __forceinline__ bf16_t f32_to_bf16(float f) {
  uint32_t u = __float_as_uint(f);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return (bf16_t)(u >> 16);
}

template <typename T> __device__ __forceinline__ float load_f(const T* p);
template <> __device__ __forceinline__ float load_f<float>(const float* p) { return *p; }
template <> __device__ __forceinline__ float load_f<bf16_t>(const bf16_t* p) { return bf16_to_f32(*p); }
template <typename T> __device__ __forceinline__ void store_f(T* p, float v);
template <> __device__ __forceinline__ void store_f<float>(float* p, float v) { *p = v; }
template <> __device__ __forceinline__ void store_f<bf16_t>(bf16_t* p, float v) { *p = f32_to_bf16(v); }

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}

// ---------------------------------------------------------------------------------------------
// launchers (host).  is_bf16 selects the storage type T of the operands marked T.
// All return the hipError_t of the launch.
// ---------------------------------------------------------------------------------------------

// x (f32 [rows][H], in place) = (emb ? emb : x) + sum_{s<n_parts} parts[s] + sum_{j<n_peers} peers[j];
// then up to two normed copies out_a = rmsnorm(x) * gain_a, out_b likewise (T), and an optional
// f32 copy x_out.  parts: f32, slot s at parts + s*part_stride; peers: T, peer j at peers + j*peer_stride.
struct ReduceNormArgs {
  float* x;
  const void* emb;         // T [rows][H] or null
  const float* parts;      // f32 or null
  int n_parts;
  size_t part_stride;      // elements
  const void* peers;       // T or null
  int n_peers;
  size_t peer_stride;      // elements
  void* out_a;             // T or null
  const void* gain_a;      // T, or null = no gain
  void* out_b;
  const void* gain_b;
  float* x_out;            // f32 or null
  int rows, H;
  float eps;
};
hipError_t launch_reduce_norm(const ReduceNormArgs& a, bool is_bf16, hipStream_t s);

// out[m][col0 + n] (f32, row stride ldo) = sum_k x[m][k] * w[k][n];  x: T [M][K], w: T [K][N]
hipError_t launch_gemm_generic(const void* x, const void* w, float* out, int M, int N, int K, int ldo,
                               int col0, bool is_bf16, hipStream_t s);

// qkv: f32 [n_parts][rows][(nq+2nkv)*d] (slots summed).  rows = B*T, row = b*T + t, position = pos0 + t.
// q -> T [rows][nq*d] rotated; k rotated -> cache_k T [B_cap][nkv][max_seq][d]; v -> cache_v kept
// TRANSPOSED, T [B_cap][nkv][d][max_seq] (positions contiguous: the layout the P*V contraction wants).
// max_seq here is the cache row capacity (a multiple of 64).
struct RopeAppendArgs {
  const float* qkv;
  int n_parts;
  size_t part_stride;
  void* q_out;
  void* cache_k;
  void* cache_v;
  const float* cos_tab;    // [max_seq][d/2]
  const float* sin_tab;
  int B, T, pos0, nq, nkv, d, max_seq;
  const int* pos_dev;      // if non-null the position is read from device memory (pos0 ignored)
};
hipError_t launch_rope_append(const RopeAppendArgs& a, bool is_bf16, hipStream_t s);

// plain causal GQA attention over the cache: one wavefront per (row, q head).
struct AttnGenericArgs {
  const void* q;           // T [rows][nq*d]
  const void* cache_k;     // T [B_cap][nkv][max_seq][d]
  const void* cache_v;     // T [B_cap][nkv][d][max_seq]
  void* o;                 // T [rows][nq*d]
  int B, T, pos0, nq, nkv, d, max_seq;
};
hipError_t launch_attn_generic(const AttnGenericArgs& a, bool is_bf16, hipStream_t s);

// act[m][i] (T) = silu(gu[m][i]) * gu[m][I + i];  gu: f32 [M][2I]
hipError_t launch_swiglu(const float* gu, void* act, int M, int I, bool is_bf16, hipStream_t s);

// ---- generation head ----------------------------------------------------------------------------
// x_out[r][:] = table[tokens[r]][:]  (T [rows][H]); an id outside [0, vocab) reads the nearest valid row and sets
// *bad_id (host-visible memory, may be null) to 1
hipError_t launch_embed_gather(const int* tokens, const void* table, void* x_out, int rows, int H, int vocab,
                               unsigned* bad_id, bool is_bf16, hipStream_t s);
// y[r][:] = x[r][:] / sqrt(mean(x[r]^2) + eps) * gain   (gain may be null = 1); y: T
hipError_t launch_head_norm(const float* x, const void* gain, void* y, int rows, int H, float eps, bool is_bf16,
                            hipStream_t s);
// tokens_out[r] = index of the largest of logits[r][0..V), the lowest index among equal maxima
hipError_t launch_argmax(const float* logits, int* tokens_out, int rows, int V, hipStream_t s);

// ---- bf16 streaming / MFMA path ----------------------------------------------------------------
// Packed weight format ("tiles"): the [K][N] matrix is cut into tiles of 32 k x 16 n; tile (nt, kt)
// is 1 KiB at ((nt*KT + kt)*64 + lane)*16 bytes, lane holding W[kt*32 + (lane/16)*8 + e][nt*16 + lane%16]
// for e = 0..7 -- exactly one wavefront's A operand of a 16x16x32 bf16 MFMA, so a wave reads a tile
// with one fully coalesced 16-byte-per-lane load.  K and N are zero-padded to multiples of 32 / 16.
static inline size_t packed_tiles_bytes(int K, int N) {
  return (size_t)((N + 15) / 16) * (size_t)((K + 31) / 32) * 1024;
}
// Repack src (bf16 [K][N], row stride N) into dst tiles at column-tile offset: column n of src becomes
// packed column map(n).  mode 0: n -> col0 + n.  mode 1 (gate) / 2 (up): SwiGLU interleave,
// n -> 16*(n/8) + (n%8) + (mode==2 ? 8 : 0), so each 16-wide tile holds 8 gate and the 8 matching up columns.
// The values are copied bit for bit.
hipError_t launch_repack_tiles(const bf16_t* src, void* dst, int K, int N, int N_total, int col0, int mode, hipStream_t s);

struct GemvArgs {
  const bf16_t* x;         // bf16 [M][ldx]
  int ldx;
  const void* wp;          // packed tiles, N_total columns, K rows
  int M, K, N;             // N = packed column count (multiple of 16 after padding)
  int ksplit;              // workgroups along K; out slot = slot0 + ks
  float* out;              // epilogue 0: f32 [slot][M][N] partial sums, slot stride out_stride
  size_t out_stride;
  int slot0;
  bf16_t* act;             // epilogue 1 (ksplit must be 1): SwiGLU -> bf16 [M][N/2]
  int epilogue;
};
// launch shape of the skinny GEMM for a problem: column tiles per workgroup, wavefronts per workgroup,
// k tiles per register buffer, workgroups along K (1 unless allow_ksplit)
struct GemvPlan { int tn, waves, u, ksplit; };
GemvPlan gemv_plan(int M, int N, int K, bool allow_ksplit);
hipError_t launch_gemv(const GemvArgs& a, hipStream_t s);

struct AttnDecodeArgs {
  const bf16_t* q;         // [B][nq*d] rotated
  const bf16_t* cache_k;   // [B_cap][nkv][max_seq][d]
  const bf16_t* cache_v;   // [B_cap][nkv][d][max_seq]
  float* part_o;           // [B][nkv][n_chunks][g][d]
  float* part_ml;          // [B][nkv][n_chunks][g][2]
  bf16_t* o;               // [B][nq*d]
  int B, nq, nkv, d, max_seq;
  int n_pos;               // visible positions (incl. the new one)
  int chunk, n_chunks;     // chunk in {32, 64, 128}
  const int* pos_dev;      // if non-null: n_pos = *pos_dev + 1
};
hipError_t launch_attn_decode(const AttnDecodeArgs& a, hipStream_t s);

// ---- prefill MFMA path ---------------------------------------------------------------------------
struct GemmArgs {
  const bf16_t* x;         // bf16 [M][ldx]
  int ldx;
  const void* wp;          // packed tiles
  int M, K, N;
  float* out;              // epilogue 0: f32 [M][N] (row stride N)
  bf16_t* act;             // epilogue 1: SwiGLU -> bf16 [M][N/2]
  int epilogue;
  // epilogue 2: the columns are q | k | v heads of d columns each; row m is token m % T of sequence m / T at
  // position pos0 + m % T: rotary embedding of q and k (adjacent pairs), q -> q_out bf16 [M][nq*d], k and v ->
  // the cache (k [seq][nkv][max_seq][d], v transposed [seq][nkv][d][max_seq])
  bf16_t* q_out;
  bf16_t* cache_k;
  bf16_t* cache_v;
  const float* cos_tab;    // [max_seq][d/2]
  const float* sin_tab;
  int T, pos0, nq, nkv, d, max_seq;
  // epilogue 3: the residual update of Algorithm 1 (a module's reduced output joins the stream) with the AllReduce written as a sum
  // over rank partial sums (Eq. 2): x_res[m][n] = x_res[m][n] + product + peers_0[m][n] + peers_1[m][n] + ...
  // (in this order, in place, row stride N), an optional f32 copy, for each module that reads the new rows a bf16
  // copy of them times the gain of that module's RMSNorm (the product in fp32, one rounding), and the rows' sums
  // of squares per column block: ssq_part[block][m], gemm_ssq_parts() blocks
  float* x_res;
  float* x_copy;           // or null
  bf16_t* xh_a;            // bf16 [M][N], or null
  const bf16_t* gain_a;    // bf16 [N] (with xh_a)
  bf16_t* xh_b;            // or null (only with xh_a)
  const bf16_t* gain_b;    // bf16 [N] (with xh_b)
  const bf16_t* peers;     // bf16 [n_peers][peer_stride], row stride N; or null
  int n_peers;
  size_t peer_stride;      // elements
  float* ssq_part;         // f32 [gemm_ssq_parts()][M] (at most ceil(N / 64) blocks), or null
  // every epilogue: if non-null, row m of the product is multiplied by row_scale[m] first (the 1/rms of an
  // RMSNorm whose gain the producer of x has already applied: the factor commutes with the product)
  const float* row_scale;
};
hipError_t launch_gemm_mfma(const GemmArgs& a, hipStream_t s);
int gemm_ssq_parts(const GemmArgs& a);   // epilogue 3: the number of column blocks that launch_gemm_mfma(a) leaves in ssq_part
// rs_a[m] (and rs_b[m] if non-null) = 1 / sqrt(sum_p ssq_part[p][m] / H + eps), p < n_part, fixed summation order
hipError_t launch_row_rms(const float* ssq_part, int n_part, int M, int H, float eps, float* rs_a, float* rs_b, hipStream_t s);

struct AttnPrefillArgs {
  const bf16_t* q;         // [B*T][nq*d] rotated
  const bf16_t* cache_k;   // [B_cap][nkv][max_seq][d]
  const bf16_t* cache_v;   // [B_cap][nkv][d][max_seq]
  bf16_t* o;               // [B*T][nq*d]
  int B, T, pos0, nq, nkv, d, max_seq;
};
hipError_t launch_attn_prefill(const AttnPrefillArgs& a, hipStream_t s);

// transposes caller-made V content [B][nkv][S][d] into the cache layout [B_cap][nkv][d][max_seq] and copies K
hipError_t launch_load_kv(const void* k, const void* v, void* cache_k, void* cache_v, int B, int nkv, int S, int d,
                          int max_seq, bool is_bf16, hipStream_t s);
