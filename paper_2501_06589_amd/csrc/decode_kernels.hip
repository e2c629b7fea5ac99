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

hipError_t launch_repack_tiles(const bf16_t* src, void* dst, int K, int N, int N_total, int col0, int mode, hipStream_t s) {
  const long long total = (long long)((N_total + 15) / 16) * ((K + 31) / 32) * 64;
  const unsigned blocks = (unsigned)((total + 255) / 256);
  hipLaunchKernelGGL(repack_tiles_kernel, dim3(blocks), dim3(256), 0, s, src, (uint4*)dst, K, N, N_total, col0, mode);
  return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// Weight-streaming skinny GEMM  out[m][n] = sum_k x[m][k] W[k][n]  for M <= 16*MT rows.
// HBM-bound: every weight byte is read once, as one coalesced 1 KiB tile per wavefront load
// (non-temporal: the stream must not evict x from the caches), and goes straight into the A operand
// of a 16x16x32 bf16 MFMA; the B operand is the matching 16 rows x 32 k slice of x (rows >= M zeroed),
// read from L1/L2 once per k tile and shared by the wave's TN column tiles.  A workgroup owns TN
// adjacent 16-column tiles and a K range; its WAVES wavefronts split that range and add up through
// LDS in a fixed order (wave 0.., then the ksplit slots by the consumer).
// Latency hiding is explicit: two register buffers of U k-tiles each, the next batch is always in
// flight while the current one is multiplied.  All loads are unconditional (addresses clamped into
// the wave's range, contributions masked at use) and the K loop is wave-uniform, so the compiler can
// count outstanding loads exactly instead of draining them.
// ------------------------------------------------------------------------------------------------
typedef __attribute__((__vector_size__(4 * sizeof(uint32_t)))) uint32_t u32x4_t;

template <int MT, int WAVES, int U, int TN>
__global__ __launch_bounds__(WAVES * 64) void gemv_mfma_kernel(GemvArgs a) {
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
  const int b = lane & 15, q = lane >> 4;
  const int nt0 = blockIdx.x * TN, ks = blockIdx.y;
  const int KT = a.K >> 5;
  const int kt_per_wg = (KT + a.ksplit - 1) / a.ksplit;
  const int wg0 = ks * kt_per_wg;
  const int wg1 = min(KT, wg0 + kt_per_wg);
  // the wavefronts take groups of U k tiles round robin: the workgroup sweeps its weight range once (DRAM page
  // locality: measured faster than a contiguous share per wavefront)
  constexpr int KB = WAVES * U, KA = 2 * WAVES * U;   // tile distance to the second register buffer / to the next turn
  const int kt0 = wg0 + wave * U;
  const int kt1 = wg1;

  f32x4_t acc[TN][MT];
#pragma unroll
  for (int j = 0; j < TN; ++j)
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) acc[j][mt] = (f32x4_t){0.f, 0.f, 0.f, 0.f};

  const u32x4_t* wptr = reinterpret_cast<const u32x4_t*>(a.wp) + ((size_t)nt0 * KT) * 64 + lane;
  const bf16_t* xptr[MT];
  bool rowok[MT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) {
    rowok[mt] = mt * 16 + b < a.M;
    xptr[mt] = a.x + (size_t)min(mt * 16 + b, a.M - 1) * a.ldx + q * 8;
  }
  u32x4_t wa[TN][U], wb[TN][U], xa[MT][U], xb[MT][U];
  auto load = [&](u32x4_t (&wv)[TN][U], u32x4_t (&xv)[MT][U], int kt) {
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int ktc = min(kt + u, kt1 - 1);
#pragma unroll
      for (int j = 0; j < TN; ++j) wv[j][u] = __builtin_nontemporal_load(wptr + ((size_t)j * KT + ktc) * 64);
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) xv[mt][u] = *reinterpret_cast<const u32x4_t*>(xptr[mt] + (size_t)ktc * 32);
    }
  };
  auto fma = [&](const u32x4_t (&wv)[TN][U], const u32x4_t (&xv)[MT][U], int kt) {
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const bool kok = kt + u < kt1;
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) {
        const u32x4_t xz = (kok && rowok[mt]) ? xv[mt][u] : (u32x4_t){0u, 0u, 0u, 0u};
#pragma unroll
        for (int j = 0; j < TN; ++j)
          acc[j][mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, wv[j][u]),
                                                              __builtin_bit_cast(bf16x8_t, xz), acc[j][mt], 0, 0, 0);
      }
    }
  };
  if (kt0 < kt1) {
    load(wa, xa, kt0);
    for (int kt = kt0; kt < kt1; kt += KA) {
      load(wb, xb, kt + KB);
      __builtin_amdgcn_sched_barrier(0);
      fma(wa, xa, kt);
      __builtin_amdgcn_sched_barrier(0);
      load(wa, xa, kt + KA);
      __builtin_amdgcn_sched_barrier(0);
      fma(wb, xb, kt + KB);
      __builtin_amdgcn_sched_barrier(0);
    }
  }

  // acc[j][mt][r] = out[row = mt*16 + b][col = (nt0 + j)*16 + 4q + r]; reduce over the waves through LDS,
  // 4 (tile, row-tile) slots per round
  constexpr int SLOTS = TN * MT, PER_ROUND = SLOTS < 4 ? SLOTS : 4;
  __shared__ float red[WAVES][PER_ROUND][16][17];  // [wave][slot][col in tile][row in tile]
  const int I = a.N >> 1;
#pragma unroll
  for (int s0 = 0; s0 < SLOTS; s0 += PER_ROUND) {
    if (s0 > 0) __syncthreads();
#pragma unroll
    for (int s = 0; s < PER_ROUND; ++s) {
      const int j = (s0 + s) / MT, mt = (s0 + s) % MT;
#pragma unroll
      for (int r = 0; r < 4; ++r) red[wave][s][4 * q + r][b] = acc[j][mt][r];
    }
    __syncthreads();
    if (a.epilogue == 0) {
      for (int i = threadIdx.x; i < PER_ROUND * 256; i += WAVES * 64) {
        const int s = i >> 8, row16 = (i >> 4) & 15, col16 = i & 15;
        const int j = (s0 + s) / MT, mt = (s0 + s) % MT;
        const int row = mt * 16 + row16, col = (nt0 + j) * 16 + col16;
        if (row < a.M && col < a.N) {
          float v = 0.f;
#pragma unroll
          for (int w = 0; w < WAVES; ++w) v += red[w][s][col16][row16];
          a.out[(size_t)(a.slot0 + ks) * a.out_stride + (size_t)row * a.N + col] = v;
        }
      }
    } else {
      // SwiGLU: tile columns 0..7 are gate columns 8nt..8nt+7, columns 8..15 the matching up columns
      for (int i = threadIdx.x; i < PER_ROUND * 128; i += WAVES * 64) {
        const int s = i >> 7, row16 = (i >> 3) & 15, c8 = i & 7;
        const int j = (s0 + s) / MT, mt = (s0 + s) % MT;
        const int row = mt * 16 + row16, col = (nt0 + j) * 8 + c8;
        if (row < a.M && col < I) {
          float g = 0.f, u = 0.f;
#pragma unroll
          for (int w = 0; w < WAVES; ++w) {
            g += red[w][s][c8][row16];
            u += red[w][s][c8 + 8][row16];
          }
          a.act[(size_t)row * I + col] = f32_to_bf16(g / (1.0f + __expf(-g)) * u);
        }
      }
    }
  }
}

GemvPlan gemv_plan(int M, int N, int K, bool allow_ksplit) {
  GemvPlan p;
  const int NT = N / 16, KT = K / 32;
  p.tn = (NT <= 192 && NT % 4 == 0) ? 4 : 2;
  p.waves = KT >= 64 ? 8 : 4;
  const int groups = NT / p.tn;
  p.ksplit = 1;
  if (allow_ksplit)
    while (groups * p.ksplit * p.waves < 1536 && KT / (p.ksplit * 2 * p.waves) >= 8 && p.ksplit < 8) p.ksplit *= 2;
  p.u = (M <= 16 && p.waves == 4 && p.tn == 2) ? 4 : 2;
  return p;
}

template <int MT>
static hipError_t launch_gemv_mt(const GemvArgs& a, const GemvPlan& p, hipStream_t s) {
  const dim3 grid(a.N / 16 / p.tn, a.ksplit), block(p.waves * 64);
  if (p.waves == 8 && p.tn == 2) hipLaunchKernelGGL((gemv_mfma_kernel<MT, 8, 2, 2>), grid, block, 0, s, a);
  else if (p.waves == 8 && p.tn == 4) hipLaunchKernelGGL((gemv_mfma_kernel<MT, 8, 2, 4>), grid, block, 0, s, a);
  else if (p.waves == 4 && p.tn == 4) hipLaunchKernelGGL((gemv_mfma_kernel<MT, 4, 2, 4>), grid, block, 0, s, a);
  else if (p.u == 4) hipLaunchKernelGGL((gemv_mfma_kernel<MT, 4, 4, 2>), grid, block, 0, s, a);
  else hipLaunchKernelGGL((gemv_mfma_kernel<MT, 4, 2, 2>), grid, block, 0, s, a);
  return hipGetLastError();
}

hipError_t launch_gemv(const GemvArgs& a, hipStream_t s) {
  if (a.M <= 0 || a.M > 64 || (a.N & 31) || (a.K & 31)) return hipErrorInvalidValue;
  GemvPlan p = gemv_plan(a.M, a.N, a.K, a.epilogue == 0);
  if (a.ksplit != p.ksplit) return hipErrorInvalidValue;  // the caller sizes its slots from the same plan
  const int mt = (a.M + 15) / 16;
  if (mt == 1) return launch_gemv_mt<1>(a, p, s);
  if (mt == 2) return launch_gemv_mt<2>(a, p, s);
  return launch_gemv_mt<4>(a, p, s);
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

// combine: one workgroup of D threads per (sequence, q head); the chunk statistics go through LDS
// so that no thread walks a chain of dependent global loads
template <int D>
__global__ void attn_combine_kernel(AttnDecodeArgs a) {
  __shared__ float wgt[512];
  __shared__ float stat[2];
  const int h = blockIdx.x, bi = blockIdx.y, t = threadIdx.x;
  const int g = a.nq / a.nkv;
  const int kvh = h / g, hg = h % g;
  const int n_pos = a.pos_dev ? (*a.pos_dev + 1) : a.n_pos;
  const int nc = min(a.n_chunks, (n_pos + a.chunk - 1) / a.chunk);   // chunks that hold visible positions
  const size_t base = ((size_t)bi * a.nkv + kvh) * a.n_chunks;
  for (int c = t; c < nc; c += D) wgt[c] = a.part_ml[((base + c) * g + hg) * 2];
  __syncthreads();
  if (t < 64) {   // first wavefront: max, then weights and the normaliser
    float m = -INFINITY;
    for (int c = t; c < nc; c += 64) m = fmaxf(m, wgt[c]);
    m = wave_max(m);
    float l = 0.f;
    for (int c = t; c < nc; c += 64) {
      const float w = __expf(wgt[c] - m);
      wgt[c] = w;
      l += a.part_ml[((base + c) * g + hg) * 2 + 1] * w;
    }
    l = wave_sum(l);
    if (t == 0) stat[0] = l;
  }
  __syncthreads();
  float o = 0.f;
#pragma unroll 8
  for (int c = 0; c < nc; ++c) o += a.part_o[((base + c) * g + hg) * D + t] * wgt[c];
  a.o[(size_t)bi * a.nq * D + h * D + t] = f32_to_bf16(o / stat[0]);
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
