// Decode-shape kernels of the bf16 path (gfx950): weight repacking into MFMA tiles, the
// weight-streaming skinny GEMM, and split-KV attention over the cache with its combine step.
#include "common.h"

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8_t;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4_t;

// ------------------------------------------------------------------------------------------------
// Repack: one thread per (tile, lane); writes the lane's 8 consecutive k of its packed column.
// ------------------------------------------------------------------------------------------------
__global__ void repack_tiles_kernel(const bf16_t* __restrict__ src, uint4* __restrict__ dst, int K, int N,
                                    int N_total, int col0, int mode) {
  const int KT = (K + 31) / 32, NT = (N_total + 15) / 16;
  const long long gid = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (gid >= (long long)NT * KT * 64) return;
  const int lane = (int)(gid & 63);
  const long long tile = gid >> 6;
  const int kt = (int)(tile % KT), nt = (int)(tile / KT);
  const int pc = nt * 16 + (lane & 15);
  int n_src;
  if (mode == 0) {
    n_src = pc - col0;
  } else {
    const int in_tile = pc & 15;
    if ((mode == 1) != (in_tile < 8)) return;  // gate owns the low 8 columns of a tile, up the high 8
    n_src = 8 * (pc >> 4) + (in_tile & 7);
  }
  if (n_src < 0 || n_src >= N) return;
  const int k0 = kt * 32 + (lane >> 4) * 8;
  uint32_t w[4];
  for (int e = 0; e < 4; ++e) {
    const int ka = k0 + 2 * e, kb = ka + 1;
    const uint32_t lo = ka < K ? src[(size_t)ka * N + n_src] : 0;
    const uint32_t hi = kb < K ? src[(size_t)kb * N + n_src] : 0;
    w[e] = lo | (hi << 16);
  }
  dst[gid] = make_uint4(w[0], w[1], w[2], w[3]);
}

hipError_t launch_repack_tiles(const bf16_t* src, void* dst, int K, int N, int N_total, int col0, int mode,
                               hipStream_t s) {
  const long long total = (long long)((N_total + 15) / 16) * ((K + 31) / 32) * 64;
  const unsigned blocks = (unsigned)((total + 255) / 256);
  hipLaunchKernelGGL(repack_tiles_kernel, dim3(blocks), dim3(256), 0, s, src, (uint4*)dst, K, N, N_total, col0,
                     mode);
  return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// Weight-streaming skinny GEMM  out[m][n] = sum_k x[m][k] W[k][n]  for M <= 16*MT rows.
// HBM-bound: every weight byte is read once, as one coalesced 1 KiB tile per wavefront load, and
// goes straight into the A operand of a 16x16x32 bf16 MFMA; the B operand is the matching
// 16 rows x 32 k slice of x (rows >= M are zero), read from L1/L2.  A workgroup owns one 16-column
// tile and a K range; its 4 wavefronts split that range, keep UNROLL tiles in flight each, and
// add up through LDS.  Summation order is fixed (wave 0..3, then ksplit slots by the consumer).
// ------------------------------------------------------------------------------------------------
#define GEMV_WAVES 4
#define GEMV_UNROLL 8

template <int MT>
__global__ __launch_bounds__(GEMV_WAVES * 64) void gemv_mfma_kernel(GemvArgs a) {
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int b = lane & 15, q = lane >> 4;
  const int nt = blockIdx.x, ks = blockIdx.y;
  const int KT = (a.K + 31) >> 5;
  const int kt_per_wg = (KT + a.ksplit - 1) / a.ksplit;
  const int wg0 = ks * kt_per_wg;
  const int wg1 = min(KT, wg0 + kt_per_wg);
  const int per_wave = (wg1 - wg0 + GEMV_WAVES - 1) / GEMV_WAVES;
  const int kt0 = wg0 + wave * per_wave;
  const int kt1 = min(wg1, kt0 + per_wave);

  f32x4_t acc[MT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) acc[mt] = (f32x4_t){0.f, 0.f, 0.f, 0.f};

  const uint4* wptr = reinterpret_cast<const uint4*>(a.wp) + ((size_t)nt * KT) * 64 + lane;
  const uint4 zero4 = make_uint4(0, 0, 0, 0);
  for (int kt = kt0; kt < kt1; kt += GEMV_UNROLL) {
    uint4 wv[GEMV_UNROLL];
    uint4 xv[MT][GEMV_UNROLL];
#pragma unroll
    for (int u = 0; u < GEMV_UNROLL; ++u) {
      const bool in = kt + u < kt1;
      wv[u] = in ? wptr[(size_t)(kt + u) * 64] : zero4;
    }
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
      const int row = mt * 16 + b;
#pragma unroll
      for (int u = 0; u < GEMV_UNROLL; ++u) {
        const bool in = (kt + u < kt1) && (row < a.M);
        xv[mt][u] = in ? *reinterpret_cast<const uint4*>(a.x + (size_t)row * a.ldx + (kt + u) * 32 + q * 8) : zero4;
      }
    }
#pragma unroll
    for (int u = 0; u < GEMV_UNROLL; ++u) {
#pragma unroll
      for (int mt = 0; mt < MT; ++mt)
        acc[mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, wv[u]),
                                                          __builtin_bit_cast(bf16x8_t, xv[mt][u]), acc[mt], 0, 0, 0);
    }
  }

  // acc[mt][r] = out[row = mt*16 + b][col = nt*16 + 4q + r]
  __shared__ float red[GEMV_WAVES][MT][16][17];  // [wave][mt][col in tile][row in tile]
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int r = 0; r < 4; ++r) red[wave][mt][4 * q + r][b] = acc[mt][r];
  __syncthreads();

  if (a.epilogue == 0) {
    // thread t -> (mt, row, col): coalesced along columns
    for (int i = threadIdx.x; i < MT * 256; i += GEMV_WAVES * 64) {
      const int mt = i >> 8, row16 = (i >> 4) & 15, col16 = i & 15;
      const int row = mt * 16 + row16, col = nt * 16 + col16;
      if (row < a.M && col < a.N) {
        float s = 0.f;
#pragma unroll
        for (int w = 0; w < GEMV_WAVES; ++w) s += red[w][mt][col16][row16];
        a.out[(size_t)(a.slot0 + ks) * a.out_stride + (size_t)row * a.N + col] = s;
      }
    }
  } else {
    // SwiGLU: tile columns 0..7 are gate columns 8nt..8nt+7, columns 8..15 the matching up columns
    const int I = a.N >> 1;
    for (int i = threadIdx.x; i < MT * 128; i += GEMV_WAVES * 64) {
      const int mt = i >> 7, row16 = (i >> 3) & 15, c8 = i & 7;
      const int row = mt * 16 + row16, col = nt * 8 + c8;
      if (row < a.M && col < I) {
        float g = 0.f, u = 0.f;
#pragma unroll
        for (int w = 0; w < GEMV_WAVES; ++w) {
          g += red[w][mt][c8][row16];
          u += red[w][mt][c8 + 8][row16];
        }
        a.act[(size_t)row * I + col] = f32_to_bf16(g / (1.0f + __expf(-g)) * u);
      }
    }
  }
}

hipError_t launch_gemv(const GemvArgs& a, hipStream_t s) {
  if (a.M <= 0 || a.M > 64 || a.ksplit < 1) return hipErrorInvalidValue;
  if (a.epilogue == 1 && a.ksplit != 1) return hipErrorInvalidValue;
  dim3 grid((a.N + 15) / 16, a.ksplit), block(GEMV_WAVES * 64);
  const int mt = (a.M + 15) / 16;
  switch (mt) {
    case 1: hipLaunchKernelGGL(gemv_mfma_kernel<1>, grid, block, 0, s, a); break;
    case 2: hipLaunchKernelGGL(gemv_mfma_kernel<2>, grid, block, 0, s, a); break;
    case 3: hipLaunchKernelGGL(gemv_mfma_kernel<3>, grid, block, 0, s, a); break;
    default: hipLaunchKernelGGL(gemv_mfma_kernel<4>, grid, block, 0, s, a); break;
  }
  return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// Decode attention, split over the cached positions.  Workgroup (chunk, kv head, sequence):
// all G = nq/nkv query heads of the group share every K/V load.
//   scores : D/8 lanes cover one K row with 16-byte loads (a wavefront load = whole rows, contiguous),
//            the dot products are reduced over those lanes with wavefront shuffles;
//   softmax: within the chunk, one wavefront per head;
//   P*V    : V is cached transposed, CHUNK/8 lanes cover one dim's CHUNK positions with 16-byte loads,
//            reduced over those lanes with shuffles.
// (max, sum, unnormalised output) of the chunk go to the combine kernel.
// ------------------------------------------------------------------------------------------------
__device__ __forceinline__ void unpack8(const uint4 v, float f[8]) {
  f[0] = __uint_as_float(v.x << 16); f[1] = __uint_as_float(v.x & 0xFFFF0000u);
  f[2] = __uint_as_float(v.y << 16); f[3] = __uint_as_float(v.y & 0xFFFF0000u);
  f[4] = __uint_as_float(v.z << 16); f[5] = __uint_as_float(v.z & 0xFFFF0000u);
  f[6] = __uint_as_float(v.w << 16); f[7] = __uint_as_float(v.w & 0xFFFF0000u);
}

template <int D, int G, int CHUNK>
__global__ __launch_bounds__(256) void attn_decode_kernel(AttnDecodeArgs a) {
  constexpr int LPR = D / 8;         // lanes per K row
  constexpr int RPP = 256 / LPR;     // K rows per pass of the workgroup
  constexpr int SEGS = CHUNK / 8;    // lanes per V^T row (8 positions each)
  constexpr int DPP = 256 / SEGS;    // dims per pass
  __shared__ float qs[G * D];
  __shared__ float sc[G * CHUNK];
  __shared__ float hmax[G], hsum[G];

  const int c = blockIdx.x, kvh = blockIdx.y, bi = blockIdx.z;
  const int n_pos = a.pos_dev ? (*a.pos_dev + 1) : a.n_pos;
  const int p0 = c * CHUNK;
  const int p1 = min(n_pos, p0 + CHUNK);
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const size_t part_idx = ((size_t)bi * a.nkv + kvh) * a.n_chunks + c;
  if (p0 >= p1) {  // chunk beyond the visible range: neutral element for the combine
    if (tid < G) {
      a.part_ml[(part_idx * G + tid) * 2 + 0] = -INFINITY;
      a.part_ml[(part_idx * G + tid) * 2 + 1] = 0.f;
    }
    return;
  }
  const int len = p1 - p0;
  const float scale = 1.0f / sqrtf((float)D);
  const bf16_t* qg = a.q + (size_t)bi * a.nq * D + (size_t)kvh * G * D;
  for (int i = tid; i < G * D; i += 256) qs[i] = bf16_to_f32(qg[i]) * scale;
  for (int i = tid; i < G * CHUNK; i += 256) sc[i] = 0.f;
  __syncthreads();

  const bf16_t* kb = a.cache_k + (((size_t)bi * a.nkv + kvh) * a.max_seq + p0) * D;
  const bf16_t* vb = a.cache_v + ((size_t)bi * a.nkv + kvh) * D * a.max_seq + p0;

  // phase 1: scores
  {
    const int rsel = tid / LPR, csel = tid % LPR;  // row within a pass, 8-dim slice
    for (int r0 = 0; r0 < len; r0 += RPP) {
      const int r = r0 + rsel;
      float kf[8];
      if (r < len) {
        unpack8(*reinterpret_cast<const uint4*>(kb + (size_t)r * D + csel * 8), kf);
      } else {
#pragma unroll
        for (int e = 0; e < 8; ++e) kf[e] = 0.f;
      }
#pragma unroll
      for (int h = 0; h < G; ++h) {
        float p = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) p = fmaf(qs[h * D + csel * 8 + e], kf[e], p);
#pragma unroll
        for (int o = LPR / 2; o > 0; o >>= 1) p += __shfl_xor(p, o, 64);
        if (csel == 0 && r < len) sc[h * CHUNK + r] = p;
      }
    }
  }
  __syncthreads();

  // phase 2: softmax within the chunk, one wavefront per head (round robin); entries >= len stay 0
  for (int h = wave; h < G; h += 4) {
    float m = -INFINITY;
    for (int r = lane; r < len; r += 64) m = fmaxf(m, sc[h * CHUNK + r]);
    m = wave_max(m);
    float l = 0.f;
    for (int r = lane; r < len; r += 64) {
      const float e = __expf(sc[h * CHUNK + r] - m);
      sc[h * CHUNK + r] = e;
      l += e;
    }
    l = wave_sum(l);
    if (lane == 0) { hmax[h] = m; hsum[h] = l; }
  }
  __syncthreads();

  // phase 3: unnormalised output  o[h][dim] = sum_r p[h][r] V^T[dim][r]
  {
    const int seg = tid % SEGS, dsel = tid / SEGS;
    float pr[G][8];
#pragma unroll
    for (int h = 0; h < G; ++h)
#pragma unroll
      for (int e = 0; e < 8; ++e) pr[h][e] = sc[h * CHUNK + seg * 8 + e];
    float* po = a.part_o + part_idx * G * D;
    for (int d0 = 0; d0 < D; d0 += DPP) {
      const int dim = d0 + dsel;
      float vf[8];
      unpack8(*reinterpret_cast<const uint4*>(vb + (size_t)dim * a.max_seq + seg * 8), vf);
#pragma unroll
      for (int e = 0; e < 8; ++e) vf[e] = (seg * 8 + e < len) ? vf[e] : 0.f;  // never touch unwritten cache
#pragma unroll
      for (int h = 0; h < G; ++h) {
        float s = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) s = fmaf(pr[h][e], vf[e], s);
#pragma unroll
        for (int o = SEGS / 2; o > 0; o >>= 1) s += __shfl_xor(s, o, 64);
        if (seg == 0) po[h * D + dim] = s;
      }
    }
  }
  if (tid < G) {
    a.part_ml[(part_idx * G + tid) * 2 + 0] = hmax[tid];
    a.part_ml[(part_idx * G + tid) * 2 + 1] = hsum[tid];
  }
}

// combine: one workgroup of D threads per (sequence, q head)
template <int D>
__global__ void attn_combine_kernel(AttnDecodeArgs a) {
  const int h = blockIdx.x, bi = blockIdx.y;
  const int g = a.nq / a.nkv;
  const int kvh = h / g, hg = h % g;
  const size_t base = ((size_t)bi * a.nkv + kvh) * a.n_chunks;
  float m = -INFINITY;
  for (int c = 0; c < a.n_chunks; ++c) m = fmaxf(m, a.part_ml[((base + c) * g + hg) * 2]);
  float l = 0.f, o = 0.f;
  for (int c = 0; c < a.n_chunks; ++c) {
    const float mc = a.part_ml[((base + c) * g + hg) * 2], lc = a.part_ml[((base + c) * g + hg) * 2 + 1];
    if (lc > 0.f) {
      const float w = __expf(mc - m);
      l += lc * w;
      o += a.part_o[((base + c) * g + hg) * D + threadIdx.x] * w;
    }
  }
  a.o[(size_t)bi * a.nq * D + h * D + threadIdx.x] = f32_to_bf16(o / l);
}

template <int D, int G>
static hipError_t launch_attn_decode_t(const AttnDecodeArgs& a, hipStream_t s) {
  const dim3 grid(a.n_chunks, a.nkv, a.B);
  switch (a.chunk) {
    case 32: hipLaunchKernelGGL((attn_decode_kernel<D, G, 32>), grid, dim3(256), 0, s, a); break;
    case 64: hipLaunchKernelGGL((attn_decode_kernel<D, G, 64>), grid, dim3(256), 0, s, a); break;
    case 128: hipLaunchKernelGGL((attn_decode_kernel<D, G, 128>), grid, dim3(256), 0, s, a); break;
    default: return hipErrorInvalidValue;
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(attn_combine_kernel<D>, dim3(a.nq, a.B), dim3(D), 0, s, a);
  return hipGetLastError();
}

hipError_t launch_attn_decode(const AttnDecodeArgs& a, hipStream_t s) {
  const int g = a.nq / a.nkv;
  if (a.d == 128) {
    switch (g) {
      case 1: return launch_attn_decode_t<128, 1>(a, s);
      case 2: return launch_attn_decode_t<128, 2>(a, s);
      case 4: return launch_attn_decode_t<128, 4>(a, s);
      case 8: return launch_attn_decode_t<128, 8>(a, s);
    }
  } else if (a.d == 64) {
    switch (g) {
      case 1: return launch_attn_decode_t<64, 1>(a, s);
      case 2: return launch_attn_decode_t<64, 2>(a, s);
      case 4: return launch_attn_decode_t<64, 4>(a, s);
      case 8: return launch_attn_decode_t<64, 8>(a, s);
    }
  }
  return hipErrorInvalidValue;
}
