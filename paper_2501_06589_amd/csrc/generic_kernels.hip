// Plain kernels: any size, both storage types, fp32 arithmetic.  They are the whole path for the
// fp32 storage type and the fallback of the bf16 one; reduce_norm and rope_append are also used by
// the streaming / MFMA path.  gfx950 only.
#include "common.h"

// ------------------------------------------------------------------------------------------------
template <typename T> __device__ __forceinline__ void load4(const T* p, float v[4]);
template <> __device__ __forceinline__ void load4<float>(const float* p, float v[4]) {
  float4 t = *reinterpret_cast<const float4*>(p);
  v[0] = t.x; v[1] = t.y; v[2] = t.z; v[3] = t.w;
}
template <> __device__ __forceinline__ void load4<bf16_t>(const bf16_t* p, float v[4]) {
  uint2 t = *reinterpret_cast<const uint2*>(p);
  v[0] = __uint_as_float(t.x << 16); v[1] = __uint_as_float(t.x & 0xFFFF0000u);
  v[2] = __uint_as_float(t.y << 16); v[3] = __uint_as_float(t.y & 0xFFFF0000u);
}
template <typename T> __device__ __forceinline__ void store4(T* p, const float v[4]);
template <> __device__ __forceinline__ void store4<float>(float* p, const float v[4]) {
  *reinterpret_cast<float4*>(p) = make_float4(v[0], v[1], v[2], v[3]);
}
template <> __device__ __forceinline__ void store4<bf16_t>(bf16_t* p, const float v[4]) {
  uint2 t;
  t.x = (uint32_t)f32_to_bf16(v[0]) | ((uint32_t)f32_to_bf16(v[1]) << 16);
  t.y = (uint32_t)f32_to_bf16(v[2]) | ((uint32_t)f32_to_bf16(v[3]) << 16);
  *reinterpret_cast<uint2*>(p) = t;
}

// ------------------------------------------------------------------------------------------------
// Reduce + residual add + RMSNorm: the local image of the residual update and the norm that follows it
// (Algorithm 1) with the AllReduce written as a sum over rank partial sums (Eq. 2).
// One workgroup per row; the summation order is fixed: x, parts 0.., peers 0.. .
// ------------------------------------------------------------------------------------------------
template <typename T>
__global__ void reduce_norm_kernel(ReduceNormArgs a) {
  const int row = blockIdx.x;
  const int H = a.H;
  float* xr = a.x + (size_t)row * H;
  const T* emb = reinterpret_cast<const T*>(a.emb);
  const T* peers = reinterpret_cast<const T*>(a.peers);
  float ss = 0.f;
  for (int i = threadIdx.x * 4; i < H; i += blockDim.x * 4) {
    float v[4], t[4];
    if (emb) load4<T>(emb + (size_t)row * H + i, v);
    else load4<float>(xr + i, v);
    for (int s = 0; s < a.n_parts; ++s) {
      load4<float>(a.parts + s * a.part_stride + (size_t)row * H + i, t);
      v[0] += t[0]; v[1] += t[1]; v[2] += t[2]; v[3] += t[3];
    }
    for (int j = 0; j < a.n_peers; ++j) {
      load4<T>(peers + j * a.peer_stride + (size_t)row * H + i, t);
      v[0] += t[0]; v[1] += t[1]; v[2] += t[2]; v[3] += t[3];
    }
    store4<float>(xr + i, v);
    if (a.x_out) store4<float>(a.x_out + (size_t)row * H + i, v);
    ss += v[0] * v[0] + v[1] * v[1] + v[2] * v[2] + v[3] * v[3];
  }
  if (!a.out_a && !a.out_b) return;
  __shared__ float red[16];
  ss = wave_sum(ss);
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, nw = blockDim.x >> 6;
  if (lane == 0) red[wave] = ss;
  __syncthreads();
  float tot = 0.f;
  for (int w = 0; w < nw; ++w) tot += red[w];
  const float rs = 1.0f / sqrtf(tot / (float)H + a.eps);
  T* oa = reinterpret_cast<T*>(a.out_a);
  T* ob = reinterpret_cast<T*>(a.out_b);
  const T* ga = reinterpret_cast<const T*>(a.gain_a);
  const T* gb = reinterpret_cast<const T*>(a.gain_b);
  for (int i = threadIdx.x * 4; i < H; i += blockDim.x * 4) {
    float v[4], g[4], y[4];
    load4<float>(xr + i, v);  // this thread's own writes
    if (oa) {
      if (ga) load4<T>(ga + i, g);
      else g[0] = g[1] = g[2] = g[3] = 1.f;
      for (int e = 0; e < 4; ++e) y[e] = v[e] * rs * g[e];
      store4<T>(oa + (size_t)row * H + i, y);
    }
    if (ob) {
      if (gb) load4<T>(gb + i, g);
      else g[0] = g[1] = g[2] = g[3] = 1.f;
      for (int e = 0; e < 4; ++e) y[e] = v[e] * rs * g[e];
      store4<T>(ob + (size_t)row * H + i, y);
    }
  }
}

hipError_t launch_reduce_norm(const ReduceNormArgs& a, bool is_bf16, hipStream_t s) {
  if (a.rows <= 0) return hipSuccess;
  const int threads = a.H >= 4096 ? 1024 : 256;
  if (is_bf16) hipLaunchKernelGGL(reduce_norm_kernel<bf16_t>, dim3(a.rows), dim3(threads), 0, s, a);
  else hipLaunchKernelGGL(reduce_norm_kernel<float>, dim3(a.rows), dim3(threads), 0, s, a);
  return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// Plain tiled GEMM, 64x64 output tile per workgroup, 4x4 per thread, fully bounds-checked.
// ------------------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void gemm_generic_kernel(const T* __restrict__ x, const T* __restrict__ w,
                                                           float* __restrict__ out, int M, int N, int K,
                                                           int ldo, int col0) {
  __shared__ float xs[16][64 + 4];
  __shared__ float ws[16][64 + 4];
  const int t = threadIdx.x;
  const int m0 = blockIdx.y * 64, n0 = blockIdx.x * 64;
  const int ty = t >> 4, tx = t & 15;
  float acc[4][4] = {};
  for (int k0 = 0; k0 < K; k0 += 16) {
    {
      const int r = t >> 2, kq = (t & 3) * 4;
      for (int e = 0; e < 4; ++e) {
        const int m = m0 + r, k = k0 + kq + e;
        xs[kq + e][r] = (m < M && k < K) ? load_f<T>(x + (size_t)m * K + k) : 0.f;
      }
      const int kr = t >> 4, nq4 = (t & 15) * 4;
      for (int e = 0; e < 4; ++e) {
        const int k = k0 + kr, n = n0 + nq4 + e;
        ws[kr][nq4 + e] = (k < K && n < N) ? load_f<T>(w + (size_t)k * N + n) : 0.f;
      }
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < 16; ++kk) {
      float av[4], bv[4];
      for (int i = 0; i < 4; ++i) av[i] = xs[kk][ty * 4 + i];
      for (int j = 0; j < 4; ++j) bv[j] = ws[kk][tx * 4 + j];
      for (int i = 0; i < 4; ++i)
        for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(av[i], bv[j], acc[i][j]);
    }
    __syncthreads();
  }
  for (int i = 0; i < 4; ++i) {
    const int m = m0 + ty * 4 + i;
    if (m >= M) continue;
    for (int j = 0; j < 4; ++j) {
      const int n = n0 + tx * 4 + j;
      if (n < N) out[(size_t)m * ldo + col0 + n] = acc[i][j];
    }
  }
}

hipError_t launch_gemm_generic(const void* x, const void* w, float* out, int M, int N, int K, int ldo,
                               int col0, bool is_bf16, hipStream_t s) {
  if (M <= 0 || N <= 0) return hipSuccess;
  dim3 grid((N + 63) / 64, (M + 63) / 64);
  if (is_bf16)
    hipLaunchKernelGGL(gemm_generic_kernel<bf16_t>, grid, dim3(256), 0, s, (const bf16_t*)x, (const bf16_t*)w, out,
                       M, N, K, ldo, col0);
  else
    hipLaunchKernelGGL(gemm_generic_kernel<float>, grid, dim3(256), 0, s, (const float*)x, (const float*)w, out, M,
                       N, K, ldo, col0);
  return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// Rotary embedding of q and k (adjacent pairs, angle = position * theta^(-2j/d), cos/sin from a
// host-made table) and append of k, v to the cache.  One thread per pair.
// ------------------------------------------------------------------------------------------------
template <typename T>
__global__ void rope_append_kernel(RopeAppendArgs a) {
  const int half = a.d >> 1;
  const int per_row = (a.nq + 2 * a.nkv) * half;
  const int rows = a.B * a.T;
  const long long gid = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (gid >= (long long)rows * per_row) return;
  const int row = (int)(gid / per_row);
  const int u = (int)(gid % per_row);
  const int b = row / a.T, t = row % a.T;
  const int pos0 = a.pos_dev ? *a.pos_dev : a.pos0;
  const int pos = pos0 + t;
  const int nqkv = (a.nq + 2 * a.nkv) * a.d;
  const int head = u / half, j = u % half;  // head index over q heads, then k heads, then v heads
  const int col = head * a.d + 2 * j;
  float e = 0.f, o = 0.f;
  for (int s = 0; s < a.n_parts; ++s) {
    const float* p = a.qkv + s * a.part_stride + (size_t)row * nqkv + col;
    e += p[0];
    o += p[1];
  }
  if (head < a.nq + a.nkv) {
    const float c = a.cos_tab[(size_t)pos * half + j], sn = a.sin_tab[(size_t)pos * half + j];
    const float re = e * c - o * sn, ro = e * sn + o * c;
    e = re;
    o = ro;
  }
  T* dst;
  if (head < a.nq) {
    dst = reinterpret_cast<T*>(a.q_out) + (size_t)row * a.nq * a.d + head * a.d + 2 * j;
  } else {
    const bool is_k = head < a.nq + a.nkv;
    if (!is_k) {  // V is kept transposed: [b][kv head][dim][position]
      const int kvh = head - a.nq - a.nkv;
      T* vt = reinterpret_cast<T*>(a.cache_v) + (((size_t)b * a.nkv + kvh) * a.d + 2 * j) * a.max_seq + pos;
      store_f<T>(vt, e);
      store_f<T>(vt + a.max_seq, o);
      return;
    }
    const int kvh = head - a.nq;
    dst = reinterpret_cast<T*>(a.cache_k) + (((size_t)b * a.nkv + kvh) * a.max_seq + pos) * a.d + 2 * j;
  }
  store_f<T>(dst, e);
  store_f<T>(dst + 1, o);
}

hipError_t launch_rope_append(const RopeAppendArgs& a, bool is_bf16, hipStream_t s) {
  const long long total = (long long)a.B * a.T * (a.nq + 2 * a.nkv) * (a.d / 2);
  if (total <= 0) return hipSuccess;
  const unsigned blocks = (unsigned)((total + 255) / 256);
  if (is_bf16) hipLaunchKernelGGL(rope_append_kernel<bf16_t>, dim3(blocks), dim3(256), 0, s, a);
  else hipLaunchKernelGGL(rope_append_kernel<float>, dim3(blocks), dim3(256), 0, s, a);
  return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// Plain attention: one wavefront per (row, q head), streaming softmax over the visible positions.
// ------------------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void attn_generic_kernel(AttnGenericArgs a) {
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const long long unit = (long long)blockIdx.x * 4 + wave;
  const int rows = a.B * a.T;
  if (unit >= (long long)rows * a.nq) return;
  const int row = (int)(unit / a.nq), h = (int)(unit % a.nq);
  const int b = row / a.T, t = row % a.T;
  const int kvh = h / (a.nq / a.nkv);
  const int n_vis = a.pos0 + t + 1;
  const T* q = reinterpret_cast<const T*>(a.q) + (size_t)row * a.nq * a.d + h * a.d;
  const T* kb = reinterpret_cast<const T*>(a.cache_k) + ((size_t)b * a.nkv + kvh) * a.max_seq * a.d;
  const T* vb = reinterpret_cast<const T*>(a.cache_v) + ((size_t)b * a.nkv + kvh) * a.max_seq * a.d;
  float qr[4], acc[4] = {0.f, 0.f, 0.f, 0.f};
  for (int e = 0; e < 4; ++e) {
    const int i = lane + 64 * e;
    qr[e] = i < a.d ? load_f<T>(q + i) : 0.f;
  }
  const float scale = 1.0f / sqrtf((float)a.d);
  float mx = -INFINITY, l = 0.f;
  for (int j = 0; j < n_vis; ++j) {
    float part = 0.f;
    for (int e = 0; e < 4; ++e) {
      const int i = lane + 64 * e;
      if (i < a.d) part = fmaf(qr[e], load_f<T>(kb + (size_t)j * a.d + i), part);
    }
    const float sc = wave_sum(part) * scale;
    const float mn = fmaxf(mx, sc);
    const float corr = expf(mx - mn), p = expf(sc - mn);
    l = l * corr + p;
    for (int e = 0; e < 4; ++e) {
      const int i = lane + 64 * e;
      if (i < a.d) acc[e] = acc[e] * corr + p * load_f<T>(vb + (size_t)i * a.max_seq + j);
    }
    mx = mn;
  }
  T* o = reinterpret_cast<T*>(a.o) + (size_t)row * a.nq * a.d + h * a.d;
  for (int e = 0; e < 4; ++e) {
    const int i = lane + 64 * e;
    if (i < a.d) store_f<T>(o + i, acc[e] / l);
  }
}

hipError_t launch_attn_generic(const AttnGenericArgs& a, bool is_bf16, hipStream_t s) {
  const long long units = (long long)a.B * a.T * a.nq;
  if (units <= 0) return hipSuccess;
  const unsigned blocks = (unsigned)((units + 3) / 4);
  if (is_bf16) hipLaunchKernelGGL(attn_generic_kernel<bf16_t>, dim3(blocks), dim3(256), 0, s, a);
  else hipLaunchKernelGGL(attn_generic_kernel<float>, dim3(blocks), dim3(256), 0, s, a);
  return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
template <typename T>
__global__ void swiglu_kernel(const float* __restrict__ gu, T* __restrict__ act, int M, int I) {
  const long long gid = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (gid >= (long long)M * I) return;
  const int m = (int)(gid / I), i = (int)(gid % I);
  const float g = gu[(size_t)m * 2 * I + i], u = gu[(size_t)m * 2 * I + I + i];
  store_f<T>(act + gid, g / (1.0f + expf(-g)) * u);
}

hipError_t launch_swiglu(const float* gu, void* act, int M, int I, bool is_bf16, hipStream_t s) {
  const long long total = (long long)M * I;
  if (total <= 0) return hipSuccess;
  const unsigned blocks = (unsigned)((total + 255) / 256);
  if (is_bf16) hipLaunchKernelGGL(swiglu_kernel<bf16_t>, dim3(blocks), dim3(256), 0, s, gu, (bf16_t*)act, M, I);
  else hipLaunchKernelGGL(swiglu_kernel<float>, dim3(blocks), dim3(256), 0, s, gu, (float*)act, M, I);
  return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// Caller-made cache content [B][nkv][S][d] -> K cache rows, V cache transposed.
// ------------------------------------------------------------------------------------------------
template <typename T>
__global__ void load_kv_kernel(const T* __restrict__ k, const T* __restrict__ v, T* __restrict__ ck,
                               T* __restrict__ cv, int B, int nkv, int S, int d, int max_seq) {
  const long long gid = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  const long long total = (long long)B * nkv * S * d;
  if (gid >= total) return;
  const int i = (int)(gid % d);
  const int p = (int)((gid / d) % S);
  const long long bh = gid / ((long long)d * S);
  ck[((size_t)bh * max_seq + p) * d + i] = k[gid];
  cv[((size_t)bh * d + i) * max_seq + p] = v[gid];
}

hipError_t launch_load_kv(const void* k, const void* v, void* cache_k, void* cache_v, int B, int nkv, int S, int d,
                          int max_seq, bool is_bf16, hipStream_t s) {
  const long long total = (long long)B * nkv * S * d;
  if (total <= 0) return hipSuccess;
  const unsigned blocks = (unsigned)((total + 255) / 256);
  if (is_bf16)
    hipLaunchKernelGGL(load_kv_kernel<bf16_t>, dim3(blocks), dim3(256), 0, s, (const bf16_t*)k, (const bf16_t*)v,
                       (bf16_t*)cache_k, (bf16_t*)cache_v, B, nkv, S, d, max_seq);
  else
    hipLaunchKernelGGL(load_kv_kernel<float>, dim3(blocks), dim3(256), 0, s, (const float*)k, (const float*)v,
                       (float*)cache_k, (float*)cache_v, B, nkv, S, d, max_seq);
  return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// Generation head: token embedding (row gather), final RMSNorm, greedy sampling (first arg max).
// ------------------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void embed_gather_kernel(const int* __restrict__ tokens, const T* __restrict__ table,
                                                           T* __restrict__ out, int H, int vocab, unsigned* bad_id) {
  const int r = blockIdx.x;
  const int raw = tokens[r];
  const int tok = min(max(raw, 0), vocab - 1);   // no access leaves the table; an id outside it is reported
  if (raw != tok && bad_id && threadIdx.x == 0) __hip_atomic_store(bad_id, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
  for (int i = threadIdx.x; i < H; i += 256) out[(size_t)r * H + i] = table[(size_t)tok * H + i];
}

hipError_t launch_embed_gather(const int* tokens, const void* table, void* x_out, int rows, int H, int vocab,
                               unsigned* bad_id, bool is_bf16, hipStream_t s) {
  if (rows <= 0) return hipSuccess;
  if (is_bf16) hipLaunchKernelGGL(embed_gather_kernel<bf16_t>, dim3(rows), dim3(256), 0, s, tokens, (const bf16_t*)table, (bf16_t*)x_out, H, vocab, bad_id);
  else hipLaunchKernelGGL(embed_gather_kernel<float>, dim3(rows), dim3(256), 0, s, tokens, (const float*)table, (float*)x_out, H, vocab, bad_id);
  return hipGetLastError();
}

template <typename T>
__global__ __launch_bounds__(256) void head_norm_kernel(const float* __restrict__ x, const T* __restrict__ gain,
                                                        T* __restrict__ y, int H, float eps) {
  __shared__ float part[4];
  const float* xr = x + (size_t)blockIdx.x * H;
  float ss = 0.f;
  for (int i = threadIdx.x; i < H; i += 256) ss = fmaf(xr[i], xr[i], ss);
  ss = wave_sum(ss);
  if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = ss;
  __syncthreads();
  const float rs = 1.0f / sqrtf((part[0] + part[1] + part[2] + part[3]) / (float)H + eps);
  for (int i = threadIdx.x; i < H; i += 256)
    store_f(y + (size_t)blockIdx.x * H + i, xr[i] * rs * (gain ? load_f(gain + i) : 1.0f));
}

hipError_t launch_head_norm(const float* x, const void* gain, void* y, int rows, int H, float eps, bool is_bf16,
                            hipStream_t s) {
  if (rows <= 0) return hipSuccess;
  if (is_bf16) hipLaunchKernelGGL(head_norm_kernel<bf16_t>, dim3(rows), dim3(256), 0, s, x, (const bf16_t*)gain, (bf16_t*)y, H, eps);
  else hipLaunchKernelGGL(head_norm_kernel<float>, dim3(rows), dim3(256), 0, s, x, (const float*)gain, (float*)y, H, eps);
  return hipGetLastError();
}

// one workgroup per row; a thread keeps the first maximum of its strided share, the merge prefers the
// lower index among equal values, so the result is the first arg max of the row
__global__ __launch_bounds__(256) void argmax_kernel(const float* __restrict__ logits, int* __restrict__ out, int V) {
  __shared__ float bv[256];
  __shared__ int bi[256];
  const float* lr = logits + (size_t)blockIdx.x * V;
  float best = -INFINITY;
  int at = 0x7fffffff;
  for (int i = threadIdx.x; i < V; i += 256) {
    const float v = lr[i];
    if (v > best || at == 0x7fffffff) { best = v; at = i; }   // strictly greater: the earliest index stays
  }
  bv[threadIdx.x] = best;
  bi[threadIdx.x] = at;
  __syncthreads();
  for (int w = 128; w > 0; w >>= 1) {
    if ((int)threadIdx.x < w) {
      const float ov = bv[threadIdx.x + w];
      const int oi = bi[threadIdx.x + w];
      if (oi != 0x7fffffff && (bi[threadIdx.x] == 0x7fffffff || ov > bv[threadIdx.x] || (ov == bv[threadIdx.x] && oi < bi[threadIdx.x]))) {
        bv[threadIdx.x] = ov;
        bi[threadIdx.x] = oi;
      }
    }
    __syncthreads();
  }
  if (threadIdx.x == 0) out[blockIdx.x] = bi[0] == 0x7fffffff ? 0 : bi[0];
}

hipError_t launch_argmax(const float* logits, int* tokens_out, int rows, int V, hipStream_t s) {
  if (rows <= 0) return hipSuccess;
  hipLaunchKernelGGL(argmax_kernel, dim3(rows), dim3(256), 0, s, logits, tokens_out, V);
  return hipGetLastError();
}
