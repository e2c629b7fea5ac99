// Prefill-shape kernels of the bf16 path (gfx950): MFMA GEMM on the packed weight tiles and causal
// GQA flash attention over the cache, both on v_mfma_f32_16x16x32_bf16.
#include "common.h"
#include <type_traits>

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8_t;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4_t;
typedef __attribute__((__vector_size__(4 * sizeof(uint32_t)))) uint32_t u32x4_t;

// workgroup tile of the large-M GEMM: 16 row tiles (256 x 256) at one wave per SIMD, or 8 (128 x 256) at two
#define GEMM_WM_LARGE 8
#define GEMM_WAVES_LARGE 2

__device__ __forceinline__ void unpack8(const uint4 v, float (&f)[8]) {
  f[0] = __uint_as_float(v.x << 16); f[1] = __uint_as_float(v.x & 0xFFFF0000u);
  f[2] = __uint_as_float(v.y << 16); f[3] = __uint_as_float(v.y & 0xFFFF0000u);
  f[4] = __uint_as_float(v.z << 16); f[5] = __uint_as_float(v.z & 0xFFFF0000u);
  f[6] = __uint_as_float(v.w << 16); f[7] = __uint_as_float(v.w & 0xFFFF0000u);
}

__device__ __forceinline__ f32x4_t mfma16(const uint4 a, const uint4 b, const f32x4_t c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, a), __builtin_bit_cast(bf16x8_t, b), c,
                                                 0, 0, 0);
}

// ------------------------------------------------------------------------------------------------
// C[M][N] = X[M][K] W[K][N].  Workgroup tile: BM = 16*WM rows x 256 columns, 4 wavefronts side by
// side along N (64 columns = 4 weight tiles each).  The weights are the MFMA A operand and come
// straight from global memory in their packed tile order (1 KiB coalesced per wave load, each tile
// read by exactly one wave of the workgroup); the activations are the B operand, staged once per
// workgroup through double-buffered LDS and shared by the 4 waves.  One k tile (32) per stage: the
// next stage's weights and activations are requested before the MFMAs of the current one.
// Output element (m, n) sits in lane (n%16)/4*16 + m%16, register n%4: a lane stores 4 consecutive
// columns.
// All global loads are unconditional (row / tile / k indices clamped into range): a guarded load makes
// the compiler drain every outstanding load before the MFMAs.  What a clamped load brings in is
// neutralised later: rows >= M become zeros when the X tile is written to LDS, columns >= N are never
// stored, and the stage past the end is never multiplied.
// ------------------------------------------------------------------------------------------------
#define GEMM_BK 32
#define GEMM_LDS_STRIDE (GEMM_BK + 8)  // bf16 elements per LDS row: 80 bytes, conflict-free 16-byte reads
#define GEMM_GROUP_M 16

// Epilogue of a wavefront's 64-column x (16 WM)-row accumulator block: row base m0, first weight tile nt0.
// Output element (m, n) sits in lane (n%16)/4*16 + m%16, register n%4: a lane stores 4 consecutive columns.
template <int WM>
__device__ __forceinline__ void gemm_epilogue(const GemmArgs& a, f32x4_t (&acc)[4][WM], int m0, int nt0, int NT, int lane) {
  const int b = lane & 15, q = lane >> 4;
  // row scale (1.0 where there is none: the multiplication is exact then), applied where an accumulator is read
  auto scale_of = [&](int mt) { return a.row_scale ? a.row_scale[min(m0 + mt * 16 + b, a.M - 1)] : 1.0f; };
  if (a.epilogue == 0) {
#pragma unroll
    for (int mt = 0; mt < WM; ++mt) {
      const int m = m0 + mt * 16 + b;
      const float rs = scale_of(mt);
      if (m >= a.M) continue;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        if (nt0 + j >= NT) continue;
        const int n = (nt0 + j) * 16 + 4 * q;
        *reinterpret_cast<float4*>(a.out + (size_t)m * a.N + n) =
            make_float4(acc[j][mt][0] * rs, acc[j][mt][1] * rs, acc[j][mt][2] * rs, acc[j][mt][3] * rs);
      }
    }
  } else if (a.epilogue == 3) {
    // residual update; the summation order per element is fixed: old value, product, peers 0, 1, ...
    // The operands (old values, the first three peers) of two column tiles are requested at once.
    constexpr int PB = 3, JB = 2, JG = 4 / JB, STEPS = WM * JG;
    struct Operands { float4 xo[JB]; uint2 pk[JB][PB]; };
    Operands o;
    auto row_of = [&](int mt) { return (size_t)min(m0 + mt * 16 + b, a.M - 1) * a.N; };
    auto request = [&](Operands& o, int st) {
      const size_t row = row_of(st / JG);
#pragma unroll
      for (int jj = 0; jj < JB; ++jj) {
        const size_t off = row + min(nt0 + (st % JG) * JB + jj, NT - 1) * 16 + 4 * q;
        o.xo[jj] = *reinterpret_cast<const float4*>(a.x_res + off);
#pragma unroll
        for (int p = 0; p < PB; ++p)
          if (p < a.n_peers) o.pk[jj][p] = *reinterpret_cast<const uint2*>(a.peers + p * a.peer_stride + off);
      }
    };
    auto add_peer = [&](float (&v4)[4], const uint2 pk) {
      v4[0] += __uint_as_float(pk.x << 16);
      v4[1] += __uint_as_float(pk.x & 0xFFFF0000u);
      v4[2] += __uint_as_float(pk.y << 16);
      v4[3] += __uint_as_float(pk.y & 0xFFFF0000u);
    };
    float ss = 0.f;
#pragma unroll
    for (int st = 0; st < STEPS; ++st) {
      request(o, st);
      const int mt = st / JG;
      const int m = m0 + mt * 16 + b;
      const bool ok = m < a.M;
      const size_t row = row_of(mt);
#pragma unroll
      for (int jj = 0; jj < JB; ++jj) {
        const int j = (st % JG) * JB + jj;
        if (nt0 + j >= NT) continue;   // (uniform over the wavefront)
        const size_t off = row + (nt0 + j) * 16 + 4 * q;
        float v4[4] = {o.xo[jj].x + acc[j][mt][0], o.xo[jj].y + acc[j][mt][1], o.xo[jj].z + acc[j][mt][2], o.xo[jj].w + acc[j][mt][3]};
#pragma unroll
        for (int p = 0; p < PB; ++p)
          if (p < a.n_peers) add_peer(v4, o.pk[jj][p]);
        for (int p = PB; p < a.n_peers; ++p) add_peer(v4, *reinterpret_cast<const uint2*>(a.peers + p * a.peer_stride + off));
        if (ok) {
          *reinterpret_cast<float4*>(a.x_res + off) = make_float4(v4[0], v4[1], v4[2], v4[3]);
          if (a.x_copy) *reinterpret_cast<float4*>(a.x_copy + off) = make_float4(v4[0], v4[1], v4[2], v4[3]);
          // the rows as the modules that read them want them: times their norm's gain (fp32 product, one rounding)
          auto store_gained = [&](bf16_t* dst, const bf16_t* gain) {
            const uint2 gk = *reinterpret_cast<const uint2*>(gain + (nt0 + j) * 16 + 4 * q);
            const float g4[4] = {__uint_as_float(gk.x << 16), __uint_as_float(gk.x & 0xFFFF0000u),
                                 __uint_as_float(gk.y << 16), __uint_as_float(gk.y & 0xFFFF0000u)};
            uint2 pk;
            pk.x = (uint32_t)f32_to_bf16(v4[0] * g4[0]) | ((uint32_t)f32_to_bf16(v4[1] * g4[1]) << 16);
            pk.y = (uint32_t)f32_to_bf16(v4[2] * g4[2]) | ((uint32_t)f32_to_bf16(v4[3] * g4[3]) << 16);
            *reinterpret_cast<uint2*>(dst + off) = pk;
          };
          if (a.xh_a) store_gained(a.xh_a, a.gain_a);
          if (a.xh_b) store_gained(a.xh_b, a.gain_b);
        }
        ss += v4[0] * v4[0] + v4[1] * v4[1] + v4[2] * v4[2] + v4[3] * v4[3];
      }
      if (st % JG == JG - 1) {   // the row block is complete: its rows' sums of squares over this wavefront's 64 columns
        ss += __shfl_xor(ss, 16, 64);
        ss += __shfl_xor(ss, 32, 64);
        if (a.ssq_part && q == 0 && ok && nt0 < NT) a.ssq_part[(size_t)(nt0 >> 2) * a.M + m] = ss;
        ss = 0.f;
      }
    }
  } else if (a.epilogue == 2) {
    // rotary embedding + cache append: a lane's 4 columns are two adjacent pairs of one head
    const int half = a.d >> 1;
#pragma unroll
    for (int mt = 0; mt < WM; ++mt) {
      const int m = m0 + mt * 16 + b;
      const float rs = scale_of(mt);
      if (m >= a.M) continue;
      const int seq = m / a.T, pos = a.pos0 + m % a.T;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        if (nt0 + j >= NT) continue;
        const int col = (nt0 + j) * 16 + 4 * q;
        const int head = col / a.d, dim = col % a.d;
        float v4[4] = {acc[j][mt][0] * rs, acc[j][mt][1] * rs, acc[j][mt][2] * rs, acc[j][mt][3] * rs};
        if (head < a.nq + a.nkv) {
#pragma unroll
          for (int p = 0; p < 2; ++p) {
            const float c = a.cos_tab[(size_t)pos * half + (dim >> 1) + p], sn = a.sin_tab[(size_t)pos * half + (dim >> 1) + p];
            const float e = v4[2 * p], o = v4[2 * p + 1];
            v4[2 * p] = e * c - o * sn;
            v4[2 * p + 1] = e * sn + o * c;
          }
        }
        if (head < a.nq + a.nkv) {
          uint2 pk;
          pk.x = (uint32_t)f32_to_bf16(v4[0]) | ((uint32_t)f32_to_bf16(v4[1]) << 16);
          pk.y = (uint32_t)f32_to_bf16(v4[2]) | ((uint32_t)f32_to_bf16(v4[3]) << 16);
          bf16_t* dst = head < a.nq ? a.q_out + (size_t)m * a.nq * a.d + head * a.d + dim
                                    : a.cache_k + (((size_t)seq * a.nkv + (head - a.nq)) * a.max_seq + pos) * a.d + dim;
          *reinterpret_cast<uint2*>(dst) = pk;
        } else {
          bf16_t* vt = a.cache_v + (((size_t)seq * a.nkv + (head - a.nq - a.nkv)) * a.d + dim) * a.max_seq + pos;
#pragma unroll
          for (int r = 0; r < 4; ++r) vt[(size_t)r * a.max_seq] = f32_to_bf16(v4[r]);
        }
      }
    }
  } else {
    // SwiGLU: tile columns 0..7 = gate columns 8nt..8nt+7 (lanes q = 0, 1), columns 8..15 = the matching
    // up columns (lanes q = 2, 3): lane + 32 holds the up partner of this lane's gate value.
    const int I = a.N >> 1;
#pragma unroll
    for (int mt = 0; mt < WM; ++mt) {
      const int m = m0 + mt * 16 + b;
      const float rs = scale_of(mt);   // (lane + 32 holds the same row)
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        float r4[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const float g = acc[j][mt][r] * rs;
          const float u = __shfl(g, (lane + 32) & 63, 64);
          r4[r] = g / (1.0f + __expf(-g)) * u;
        }
        if (q < 2 && m < a.M && nt0 + j < NT) {
          uint2 pk;
          pk.x = (uint32_t)f32_to_bf16(r4[0]) | ((uint32_t)f32_to_bf16(r4[1]) << 16);
          pk.y = (uint32_t)f32_to_bf16(r4[2]) | ((uint32_t)f32_to_bf16(r4[3]) << 16);
          *reinterpret_cast<uint2*>(a.act + (size_t)m * I + (nt0 + j) * 8 + 4 * q) = pk;
        }
      }
    }
  }
}

template <int WM, int MIN_WAVES>
__global__ __launch_bounds__(256, MIN_WAVES) void gemm_mfma_kernel(GemmArgs a) {
  constexpr int BM = 16 * WM;
  constexpr int XV = BM * 4 / 256;  // 16-byte segments per thread per stage of the X tile (BM rows x 64 bytes)
  static_assert(XV >= 1, "tile too small");
  extern __shared__ __attribute__((aligned(16))) bf16_t xs_raw[];   // [2][BM][GEMM_LDS_STRIDE]
  bf16_t (*xs)[BM][GEMM_LDS_STRIDE] = reinterpret_cast<bf16_t (*)[BM][GEMM_LDS_STRIDE]>(xs_raw);

  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int b = lane & 15, q = lane >> 4;
  const int KT = a.K >> 5, NT = a.N >> 4;
  const int tiles_m = (a.M + BM - 1) / BM, tiles_n = (a.N + 255) / 256;
  // Workgroups are handed to the 8 XCDs round robin by block index and every XCD has its own L2: block
  // index i is mapped to position (i % 8) * (n / 8) + i / 8 of the tile order, so that each XCD works
  // through one contiguous eighth of it and neighbours in the order (which share operands) meet in one L2.
  const int nblk = gridDim.x, nblk8 = nblk & ~7;
  const int bid = (int)blockIdx.x < nblk8 ? ((int)blockIdx.x & 7) * (nblk8 >> 3) + ((int)blockIdx.x >> 3) : (int)blockIdx.x;
  // grouped rasterisation: GROUP_M row blocks share one column block back to back
  const int per_group = GEMM_GROUP_M * tiles_n;
  const int group = bid / per_group, in_group = bid % per_group;
  const int gm = min(GEMM_GROUP_M, tiles_m - group * GEMM_GROUP_M);
  const int m_blk = group * GEMM_GROUP_M + in_group % gm;
  const int n_blk = in_group / gm;
  const int m0 = m_blk * BM;
  const int nt0 = n_blk * 16 + wave * 4;

  f32x4_t acc[4][WM];
#pragma unroll
  for (int j = 0; j < 4; ++j)
#pragma unroll
    for (int mt = 0; mt < WM; ++mt) acc[j][mt] = (f32x4_t){0.f, 0.f, 0.f, 0.f};

  // per-thread source addresses of the X tile (row clamped) and of the 4 weight tiles (tile clamped)
  const bf16_t* xsrc[XV];
  bool xok[XV];
#pragma unroll
  for (int i = 0; i < XV; ++i) {
    const int idx = tid + i * 256, row = idx >> 2, seg = idx & 3;
    xok[i] = m0 + row < a.M;
    xsrc[i] = a.x + (size_t)min(m0 + row, a.M - 1) * a.ldx + seg * 8;
  }
  const u32x4_t* wsrc[4];
#pragma unroll
  for (int j = 0; j < 4; ++j)
    wsrc[j] = reinterpret_cast<const u32x4_t*>(a.wp) + (size_t)min(nt0 + j, NT - 1) * KT * 64 + lane;

  u32x4_t xg[XV], w0[4], w1[4];
  auto load_stage = [&](u32x4_t (&w)[4], int kt) {
    const int ktc = min(kt, KT - 1);
#pragma unroll
    for (int i = 0; i < XV; ++i) xg[i] = *reinterpret_cast<const u32x4_t*>(xsrc[i] + (size_t)ktc * 32);
#pragma unroll
    for (int j = 0; j < 4; ++j) w[j] = wsrc[j][(size_t)ktc * 64];
  };
  auto store_x = [&](int buf) {
#pragma unroll
    for (int i = 0; i < XV; ++i) {
      const int idx = tid + i * 256, row = idx >> 2, seg = idx & 3;
      *reinterpret_cast<u32x4_t*>(&xs[buf][row][seg * 8]) = xok[i] ? xg[i] : (u32x4_t){0u, 0u, 0u, 0u};
    }
  };
  // LDS fragments are read two row tiles ahead of the MFMAs that consume them; the scheduling barriers
  // keep that distance (left alone, the compiler hoists every read to the top and runs out of registers)
  auto compute = [&](const u32x4_t (&w)[4], int buf) {
    auto frag = [&](int mt) { return *reinterpret_cast<const u32x4_t*>(&xs[buf][mt * 16 + b][q * 8]); };
    u32x4_t f0 = frag(0), f1 = frag(1), f2;
#pragma unroll
    for (int mt = 0; mt < WM; ++mt) {
      f2 = frag(mt + 2 < WM ? mt + 2 : WM - 1);
#pragma unroll
      for (int j = 0; j < 4; ++j)
        acc[j][mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, w[j]),
                                                            __builtin_bit_cast(bf16x8_t, f0), acc[j][mt], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
      f0 = f1;
      f1 = f2;
    }
  };

  load_stage(w0, 0);
  store_x(0);
  __syncthreads();
  for (int kt = 0; kt < KT; kt += 2) {
    load_stage(w1, kt + 1);
    __builtin_amdgcn_sched_barrier(0);
    compute(w0, 0);
    __builtin_amdgcn_sched_barrier(0);
    store_x(1);
    __syncthreads();
    if (kt + 1 >= KT) break;
    load_stage(w0, kt + 2);
    __builtin_amdgcn_sched_barrier(0);
    compute(w1, 1);
    __builtin_amdgcn_sched_barrier(0);
    store_x(0);
    __syncthreads();
  }

  gemm_epilogue<WM>(a, acc, m0, nt0, NT, lane);
}

__global__ __launch_bounds__(256) void row_rms_kernel(const float* __restrict__ part, int n_part, int M, float h, float eps,
                                                      float* __restrict__ rs_a, float* __restrict__ rs_b) {
  const int m = blockIdx.x * 256 + threadIdx.x;
  if (m >= M) return;
  float tot = 0.f;
  for (int p = 0; p < n_part; ++p) tot += part[(size_t)p * M + m];
  const float rs = 1.0f / sqrtf(tot / h + eps);
  rs_a[m] = rs;
  if (rs_b) rs_b[m] = rs;
}

hipError_t launch_row_rms(const float* ssq_part, int n_part, int M, int H, float eps, float* rs_a, float* rs_b, hipStream_t s) {
  if (M <= 0) return hipSuccess;
  hipLaunchKernelGGL(row_rms_kernel, dim3((M + 255) / 256), dim3(256), 0, s, ssq_part, n_part, M, (float)H, eps, rs_a, rs_b);
  return hipGetLastError();
}

template <int WM, int MIN_WAVES>
static hipError_t launch_gemm_wm(const GemmArgs& a, hipStream_t s) {
  constexpr int BM = 16 * WM;
  const size_t lds = (size_t)2 * BM * GEMM_LDS_STRIDE * sizeof(bf16_t);
  const int tiles_m = (a.M + BM - 1) / BM, tiles_n = (a.N + 255) / 256;
  hipLaunchKernelGGL((gemm_mfma_kernel<WM, MIN_WAVES>), dim3(tiles_m * tiles_n), dim3(256), lds, s, a);
  return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// Large-M GEMM: 256 x 256 workgroup tile, 8 wavefronts (2 along M x 4 along N, 128 x 64 each), one
// workgroup per CU.  Both operands travel global memory -> LDS without passing through registers
// (16-byte direct-to-LDS loads: the 64 lanes of one load fill 1 KiB of LDS in lane order), so loads are
// in flight two to three k tiles ahead of the MFMAs that consume them and cost no registers.
//   Weights: a ring of 4 stages of one k tile (32): 16 packed tiles of 1 KiB, each the register image of
//   an MFMA operand (read back as one contiguous 1 KiB).
//   Activations: a ring of 3 blocks of TWO k tiles (256 rows x 128 bytes): one load covers 8 rows x 64 k,
//   i.e. whole 128-byte cache lines (a load of 16 rows x 32 k would request every line twice, half a line
//   per k tile: measured 4 - 7 % slower).  Within a block the 16-byte segments of fragment row b are
//   stored XOR-swizzled by b / 2 (the lane that fetches segment s of row b sits at position s ^ (b / 2) of
//   the row's eight lanes), so that the 16 lanes of a fragment read that hold the same k segment hit 16
//   different bank groups.
// 160 KiB of LDS in all.  One bare barrier per k tile, in the middle of its MFMAs: after the barrier of k
// tile kt every wave's loads for k tile kt + 1 have landed and every wave has finished reading k tile
// kt - 1, whose buffers the next loads overwrite.  The first fragments of k tile kt + 1 are read right
// after that barrier, sixteen MFMAs before their first use, and a wave's loads are spread over its MFMA
// rows (issued in one burst by all eight waves they fill the address pipeline, and a wave that cannot
// issue its load cannot issue the MFMAs behind it either).
// Rows >= M and weight tiles >= N/16 are clamped on load (they only reach outputs that are not stored).
// K must be a multiple of 64.
// Tile order: the XCD-aware order of gemm_mfma_kernel with groups of GEMM2_GROUP_M row blocks; the 32 CUs
// of an XCD then work on 4 row blocks x 8 column blocks at a time (groups of 2 / 4 / 8 row blocks:
// 1309 / 1335 / 1297 TFLOP/s on 32768 x 8192 x 14336).
// Against gemm_mfma_kernel at 128 x 256 (two workgroups per CU): a third less operand traffic per CU
// and no register staging; 971 -> 1129, 908 -> 993, 1098 -> 1271, 1158 -> 1338 TFLOP/s on the QKV / O / down /
// gate-up shapes of the 70B R = 4 shard at 32768 rows.
// ------------------------------------------------------------------------------------------------
#define GEMM2_GROUP_M 4
#define GEMM2_LDSP(p) ((__attribute__((address_space(3))) void*)(p))
#define GEMM2_GLBP(p) ((const __attribute__((address_space(1))) void*)(p))

// s_waitcnt vmcnt(N) (at most N of this wave's vector-memory operations still in flight; the other counters
// are left alone: gfx9 encoding, vmcnt in bits 3:0 and 15:14, expcnt 6:4, lgkmcnt 11:8) and a bare
// workgroup barrier, without the fence of __syncthreads(), which would wait for ALL outstanding loads.
// Written with builtins, not inline assembly: after an asm statement the compiler no longer knows which
// LDS reads are pending and waits for all of them at the next use.
template <int N>
__device__ __forceinline__ void gemm2_wait_and_meet() {
  static_assert(N >= 0 && N < 64, "vmcnt range");
  __builtin_amdgcn_sched_barrier(0);
  __builtin_amdgcn_s_waitcnt(0x0F70 | (N & 15) | ((N >> 4) << 14));
  __builtin_amdgcn_s_barrier();
  __builtin_amdgcn_sched_barrier(0);
}

#define GEMM2_XBLOCK_BYTES 32768
#define GEMM2_WSTAGE_BYTES 16384
#define GEMM2_XBLOCKS 3
#define GEMM2_WSTAGES 4
#define GEMM2_LDS_BYTES (GEMM2_XBLOCKS * GEMM2_XBLOCK_BYTES + GEMM2_WSTAGES * GEMM2_WSTAGE_BYTES)

// Epilogue 3 of the 256 x 256 tile (see GemmArgs), with whole rows per memory instruction.  In the accumulator
// layout a wavefront's load or store touches 16 rows, 64 (fp32) or 32 (bf16) bytes of each; this epilogue
// moves 16 bytes per element through memory (the old row, three peers, the new row twice), and in that shape it
// cost as much as the separate reduce kernel it replaces.  So the tile passes through LDS (free once the
// workgroup is past its last k tile), 64 rows at a time: the wavefronts write their accumulator blocks, meet,
// and read back one row of 256 columns per half-wavefront, eight columns per lane, so that every access to
// memory is a whole row segment of 1 KiB (fp32) or 512 bytes (bf16), 16 bytes per lane and instruction.  The rows' sums of squares are left per 256-column
// block: ssq_part[n_blk][m].  The summation order per element is fixed: old value, product, peers 0, 1, ...
#define GEMM2_EPI_STRIDE 260   // floats per staged row: 256 + 4, so that the 16 rows of a write spread over the banks
static_assert(64 * GEMM2_EPI_STRIDE * 4 <= GEMM2_LDS_BYTES, "staging area");
__device__ __forceinline__ void gemm2_residual_epilogue(const GemmArgs& a, f32x4_t (&acc)[4][8], unsigned char* lds, int m0,
                                                        int n_blk, int wave, int lane) {
  float* stage = reinterpret_cast<float*>(lds);
  const int b = lane & 15, q = lane >> 4;
  const int wm = wave >> 2, wn = wave & 3;
  const int half = lane >> 5, l32 = lane & 31;
  const int n = n_blk * 256 + 8 * l32;       // on the way back: a half-wavefront per row, eight columns per lane
  const bool col_ok = n < a.N;               // (N is a multiple of 16)
  const int nc = col_ok ? n : 0;
  constexpr int PB = 3, RB = 2;              // peers and row pairs requested at once
  // the gains of the modules that read the new rows, for this lane's eight columns (the same for every row)
  float ga8[8], gb8[8];
  {
    const uint4 za = a.xh_a ? *reinterpret_cast<const uint4*>(a.gain_a + nc) : make_uint4(0, 0, 0, 0);
    const uint4 zb = a.xh_b ? *reinterpret_cast<const uint4*>(a.gain_b + nc) : make_uint4(0, 0, 0, 0);
    unpack8(za, ga8);
    unpack8(zb, gb8);
  }
#pragma unroll
  for (int pass = 0; pass < 4; ++pass) {     // row blocks mt = 2 pass, 2 pass + 1 of both halves of the tile
    if (pass > 0) __syncthreads();           // the previous pass has been read
#pragma unroll
    for (int h = 0; h < 2; ++h)
#pragma unroll
      for (int j = 0; j < 4; ++j)
        *reinterpret_cast<f32x4_t*>(stage + (wm * 32 + h * 16 + b) * GEMM2_EPI_STRIDE + wn * 64 + j * 16 + 4 * q) = acc[j][2 * pass + h];
    __syncthreads();
    // wavefront w takes the staged row pairs (2 w, 2 w + 1), (2 w + 16, 2 w + 17), ..., RB of them at a time
#pragma unroll
    for (int g = 0; g < 4 / RB; ++g) {
      float4 xo[RB][2];
      uint4 pk[RB][PB];
      size_t off[RB];
      bool ok[RB];
      int mrow[RB];
#pragma unroll
      for (int r = 0; r < RB; ++r) {
        const int lr = 2 * wave + 16 * (g * RB + r) + half;              // staged row: half lr / 32, row lr % 32 of the pass
        mrow[r] = m0 + (lr >> 5) * 128 + pass * 32 + (lr & 31);
        ok[r] = col_ok && mrow[r] < a.M;
        off[r] = (size_t)min(mrow[r], a.M - 1) * a.N + nc;
        xo[r][0] = *reinterpret_cast<const float4*>(a.x_res + off[r]);
        xo[r][1] = *reinterpret_cast<const float4*>(a.x_res + off[r] + 4);
#pragma unroll
        for (int p = 0; p < PB; ++p)
          if (p < a.n_peers) pk[r][p] = *reinterpret_cast<const uint4*>(a.peers + p * a.peer_stride + off[r]);
      }
#pragma unroll
      for (int r = 0; r < RB; ++r) {
        const int lr = 2 * wave + 16 * (g * RB + r) + half;
        const float4 p0 = *reinterpret_cast<const float4*>(stage + lr * GEMM2_EPI_STRIDE + 8 * l32);
        const float4 p1 = *reinterpret_cast<const float4*>(stage + lr * GEMM2_EPI_STRIDE + 8 * l32 + 4);
        float v8[8] = {xo[r][0].x + p0.x, xo[r][0].y + p0.y, xo[r][0].z + p0.z, xo[r][0].w + p0.w,
                       xo[r][1].x + p1.x, xo[r][1].y + p1.y, xo[r][1].z + p1.z, xo[r][1].w + p1.w};
        auto add_peer = [&](const uint4 u) {
          const uint32_t w4[4] = {u.x, u.y, u.z, u.w};
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            v8[2 * e] += __uint_as_float(w4[e] << 16);
            v8[2 * e + 1] += __uint_as_float(w4[e] & 0xFFFF0000u);
          }
        };
#pragma unroll
        for (int p = 0; p < PB; ++p)
          if (p < a.n_peers) add_peer(pk[r][p]);
        for (int p = PB; p < a.n_peers; ++p) add_peer(*reinterpret_cast<const uint4*>(a.peers + p * a.peer_stride + off[r]));
        if (ok[r]) {
          *reinterpret_cast<float4*>(a.x_res + off[r]) = make_float4(v8[0], v8[1], v8[2], v8[3]);
          *reinterpret_cast<float4*>(a.x_res + off[r] + 4) = make_float4(v8[4], v8[5], v8[6], v8[7]);
          if (a.x_copy) {
            *reinterpret_cast<float4*>(a.x_copy + off[r]) = make_float4(v8[0], v8[1], v8[2], v8[3]);
            *reinterpret_cast<float4*>(a.x_copy + off[r] + 4) = make_float4(v8[4], v8[5], v8[6], v8[7]);
          }
          // the rows as the modules that read them want them: times their norm's gain (fp32 product, one rounding)
          auto store_gained = [&](bf16_t* dst, const float (&g8)[8]) {
            uint4 u;
            u.x = (uint32_t)f32_to_bf16(v8[0] * g8[0]) | ((uint32_t)f32_to_bf16(v8[1] * g8[1]) << 16);
            u.y = (uint32_t)f32_to_bf16(v8[2] * g8[2]) | ((uint32_t)f32_to_bf16(v8[3] * g8[3]) << 16);
            u.z = (uint32_t)f32_to_bf16(v8[4] * g8[4]) | ((uint32_t)f32_to_bf16(v8[5] * g8[5]) << 16);
            u.w = (uint32_t)f32_to_bf16(v8[6] * g8[6]) | ((uint32_t)f32_to_bf16(v8[7] * g8[7]) << 16);
            *reinterpret_cast<uint4*>(dst + off[r]) = u;
          };
          if (a.xh_a) store_gained(a.xh_a, ga8);
          if (a.xh_b) store_gained(a.xh_b, gb8);
        }
        if (a.ssq_part) {   // (uniform)
          float ss = 0.f;
#pragma unroll
          for (int e = 0; e < 8; ++e) ss += v8[e] * v8[e];
          if (!ok[r]) ss = 0.f;
#pragma unroll
          for (int o = 16; o > 0; o >>= 1) ss += __shfl_xor(ss, o, 64);   // over the half-wavefront of the row
          if (l32 == 0 && mrow[r] < a.M) a.ssq_part[(size_t)n_blk * a.M + mrow[r]] = ss;
        }
      }
    }
  }
}

__global__ __launch_bounds__(512, 2) void gemm_lds_kernel(GemmArgs a) {
  constexpr int WM = 8;
  extern __shared__ __attribute__((aligned(16))) unsigned char g2_lds[];
  unsigned char* const xring = g2_lds;
  unsigned char* const wring = g2_lds + GEMM2_XBLOCKS * GEMM2_XBLOCK_BYTES;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int b = lane & 15, q = lane >> 4;
  const int wm = wave >> 2, wn = wave & 3;
  const int KT = a.K >> 5, KB = a.K >> 6, NT = a.N >> 4;
  const int tiles_m = (a.M + 255) / 256, tiles_n = (a.N + 255) / 256;
  const int nblk = gridDim.x, nblk8 = nblk & ~7;   // XCD-aware order, as in gemm_mfma_kernel
  const int bid = (int)blockIdx.x < nblk8 ? ((int)blockIdx.x & 7) * (nblk8 >> 3) + ((int)blockIdx.x >> 3) : (int)blockIdx.x;
  const int per_group = GEMM2_GROUP_M * tiles_n;
  const int group = bid / per_group, in_group = bid % per_group;
  const int gm = min(GEMM2_GROUP_M, tiles_m - group * GEMM2_GROUP_M);
  const int m_blk = group * GEMM2_GROUP_M + in_group % gm;
  const int n_blk = in_group / gm;
  const int m0 = m_blk * 256;
  const int nt0 = n_blk * 16;

  // this wave's share of the loads: row groups (8 rows) 4 wave .. 4 wave + 3 of an activation block, weight
  // tiles 2 wave, 2 wave + 1 of a stage
  const bf16_t* xsrc[4];
  const u32x4_t* wsrc[2];
  {
    const int r = lane >> 3;   // row within the group of 8
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int g = 4 * wave + i;                  // row group of the tile
      const int brow = 8 * (g & 1) + r;            // row within its 16-row fragment
      const int seg = (lane & 7) ^ ((brow >> 1) & 7);
      xsrc[i] = a.x + (size_t)min(m0 + 8 * g + r, a.M - 1) * a.ldx + seg * 8;
    }
#pragma unroll
    for (int i = 0; i < 2; ++i)
      wsrc[i] = reinterpret_cast<const u32x4_t*>(a.wp) + (size_t)min(nt0 + 2 * wave + i, NT - 1) * KT * 64 + lane;
  }
  auto issue_x = [&](int xbuf, int kb, int i) {   // row group i of this wave, activation block kb (k tiles 2 kb, 2 kb + 1)
    const int kbc = min(kb, KB - 1);
    __builtin_amdgcn_global_load_lds(GEMM2_GLBP(xsrc[i] + (size_t)kbc * 64),
                                     GEMM2_LDSP(xring + xbuf * GEMM2_XBLOCK_BYTES + (4 * wave + i) * 1024), 16, 0, 0);
  };
  auto issue_w = [&](int wbuf, int kt, int i) {   // weight tile i of this wave, k tile kt
    const int ktc = min(kt, KT - 1);
    __builtin_amdgcn_global_load_lds(GEMM2_GLBP(wsrc[i] + (size_t)ktc * 64),
                                     GEMM2_LDSP(wring + wbuf * GEMM2_WSTAGE_BYTES + (2 * wave + i) * 1024), 16, 0, 0);
  };

  f32x4_t acc[4][WM];
#pragma unroll
  for (int j = 0; j < 4; ++j)
#pragma unroll
    for (int mt = 0; mt < WM; ++mt) acc[j][mt] = (f32x4_t){0.f, 0.f, 0.f, 0.f};

  // per-lane read offsets inside an activation block, for the even and the odd k tile of the block
  const int xoff0 = (b >> 3) * 1024 + ((b & 7) * 8 + ((q) ^ ((b >> 1) & 7))) * 16 + wm * 8 * 2048;
  const int xoff1 = (b >> 3) * 1024 + ((b & 7) * 8 + ((4 + q) ^ ((b >> 1) & 7))) * 16 + wm * 8 * 2048;
  auto xfrag = [&](const unsigned char* xb, int mt) { return *reinterpret_cast<const u32x4_t*>(xb + mt * 2048); };
  auto wfrag = [&](const unsigned char* wb, int j) { return *reinterpret_cast<const u32x4_t*>(wb + (wn * 4 + j) * 1024); };
  auto mfma_row = [&](const u32x4_t (&w)[4], const u32x4_t& f, int mt) {
#pragma unroll
    for (int j = 0; j < 4; ++j)
      acc[j][mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, w[j]),
                                                          __builtin_bit_cast(bf16x8_t, f), acc[j][mt], 0, 0, 0);
  };

  // Issue order of a wave, per pair of k tiles (2j, 2j + 1); s = weight stage = k tile, blk = activation block:
  //   2j   first half : W1(s 2j+2)                       barrier 2j   needs W(2j+1)            -> vmcnt(4)
  //   2j   second half: W0(s 2j+3) X0 X1(blk j+2)
  //   2j+1 first half : W1(s 2j+3) X2 X3(blk j+2)        barrier 2j+1 needs W(2j+2), X(j+1)    -> vmcnt(6)
  //   2j+1 second half: W0(s 2j+4)
  // prologue in the same order: X(blk 0) W(0) | W0(1) X0 X1(blk 1) | W1(1) X2 X3(blk 1) | W0(2)
#pragma unroll
  for (int i = 0; i < 4; ++i) issue_x(0, 0, i);
  issue_w(0, 0, 0);
  issue_w(0, 0, 1);
  issue_w(1, 1, 0);
  issue_x(1, 1, 0);
  issue_x(1, 1, 1);
  issue_w(1, 1, 1);
  issue_x(1, 1, 2);
  issue_x(1, 1, 3);
  issue_w(2, 2, 0);
  gemm2_wait_and_meet<7>();   // block 0 and stage 0 have landed
  u32x4_t wA[4], wB[4], fA[3], fB[3];
#pragma unroll
  for (int j = 0; j < 4; ++j) wA[j] = wfrag(wring + lane * 16, j);
#pragma unroll
  for (int mt = 0; mt < 3; ++mt) fA[mt] = xfrag(xring + xoff0, mt);

  int wstage = 0;   // weight stage of the current k tile
  int xblk = 0;     // activation block of the current pair of k tiles
  // one k tile; ODD: second tile of its activation block
  auto step = [&](auto odd_tag, const u32x4_t (&w)[4], const u32x4_t (&f012)[3], u32x4_t (&wn4)[4], u32x4_t (&g012)[3], int kt) {
    constexpr bool ODD = decltype(odd_tag)::value;
    const unsigned char* xb = xring + xblk * GEMM2_XBLOCK_BYTES + (ODD ? xoff1 : xoff0);
    const int wnext = (wstage + 1) & 3, w2 = (wstage + 2) & 3, w3 = (wstage + 3) & 3;
    const int xnext = xblk + 1 == GEMM2_XBLOCKS ? 0 : xblk + 1;
    const int xfill = xblk + 2 >= GEMM2_XBLOCKS ? xblk + 2 - GEMM2_XBLOCKS : xblk + 2;
    u32x4_t f[WM];
    mfma_row(w, f012[0], 0);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int mt = 3; mt < WM; ++mt) f[mt] = xfrag(xb, mt);
    __builtin_amdgcn_sched_barrier(0);
    mfma_row(w, f012[1], 1);
    __builtin_amdgcn_sched_barrier(0);
    if (ODD) {
      issue_w(w2, kt + 2, 1);
      issue_x(xfill, (kt >> 1) + 2, 2);
    } else {
      issue_w(w2, kt + 2, 1);
    }
    __builtin_amdgcn_sched_barrier(0);
    mfma_row(w, f012[2], 2);
    __builtin_amdgcn_sched_barrier(0);
    mfma_row(w, f[3], 3);
    __builtin_amdgcn_sched_barrier(0);
    if (ODD) issue_x(xfill, (kt >> 1) + 2, 3);
    __builtin_amdgcn_sched_barrier(0);
    // after the barrier: weight stage kt + 1 (and, behind an odd tile, the next activation block) are readable,
    // and nobody reads weight stage kt - 1 (behind an even tile: activation block j - 1) any more
    if (ODD) gemm2_wait_and_meet<6>(); else gemm2_wait_and_meet<4>();
    const unsigned char* nxb = ODD ? xring + xnext * GEMM2_XBLOCK_BYTES + xoff0 : xring + xblk * GEMM2_XBLOCK_BYTES + xoff1;
    const unsigned char* nwb = wring + wnext * GEMM2_WSTAGE_BYTES + lane * 16;
#pragma unroll
    for (int j = 0; j < 4; ++j) wn4[j] = wfrag(nwb, j);
#pragma unroll
    for (int mt = 0; mt < 3; ++mt) g012[mt] = xfrag(nxb, mt);
    __builtin_amdgcn_sched_barrier(0);
    mfma_row(w, f[4], 4);
    __builtin_amdgcn_sched_barrier(0);
    issue_w(w3, kt + 3, 0);
    if (!ODD) issue_x(xfill, (kt >> 1) + 2, 0);
    __builtin_amdgcn_sched_barrier(0);
    mfma_row(w, f[5], 5);
    mfma_row(w, f[6], 6);
    __builtin_amdgcn_sched_barrier(0);
    if (!ODD) issue_x(xfill, (kt >> 1) + 2, 1);
    __builtin_amdgcn_sched_barrier(0);
    mfma_row(w, f[7], 7);
    __builtin_amdgcn_sched_barrier(0);
    wstage = wnext;
    if (ODD) xblk = xnext;
  };
  for (int kt = 0; kt < KT; kt += 2) {   // KT is even
    step(std::false_type{}, wA, fA, wB, fB, kt);
    step(std::true_type{}, wB, fB, wA, fA, kt + 1);
  }
  // the clamped loads past the last k tile are still in flight into LDS: they must land before the workgroup ends
  gemm2_wait_and_meet<0>();
  if (a.epilogue == 3) gemm2_residual_epilogue(a, acc, g2_lds, m0, n_blk, wave, lane);
  else gemm_epilogue<WM>(a, acc, m0 + wm * 128, nt0 + wn * 4, NT, lane);
}

static hipError_t launch_gemm_lds(const GemmArgs& a, hipStream_t s) {
  static bool prepared[64] = {};
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= 64) return hipErrorInvalidDevice;
  if (!prepared[dev]) {   // more than the default 64 KiB of dynamic LDS: asked for once per device
    e = hipFuncSetAttribute(reinterpret_cast<const void*>(gemm_lds_kernel), hipFuncAttributeMaxDynamicSharedMemorySize, (int)GEMM2_LDS_BYTES);
    if (e != hipSuccess) return e;
    prepared[dev] = true;
  }
  const int tiles_m = (a.M + 255) / 256, tiles_n = (a.N + 255) / 256;
  hipLaunchKernelGGL(gemm_lds_kernel, dim3(tiles_m * tiles_n), dim3(512), GEMM2_LDS_BYTES, s, a);
  return hipGetLastError();
}

static bool gemm_takes_lds_kernel(const GemmArgs& a) {
  // 256 x 256 tiles, one per CU, when they fill the chip at least once; else the smaller tiles
  return (long)((a.M + 255) / 256) * ((a.N + 255) / 256) >= 256 && (a.K & 63) == 0 && a.K >= 256;
}

int gemm_ssq_parts(const GemmArgs& a) { return gemm_takes_lds_kernel(a) ? (a.N + 255) / 256 : (a.N + 63) / 64; }

hipError_t launch_gemm_mfma(const GemmArgs& a, hipStream_t s) {
  if (a.M <= 0 || (a.K & 31) || (a.N & 15) || a.K < 32) return hipErrorInvalidValue;
  // operands of the chosen epilogue
  if (a.epilogue < 0 || a.epilogue > 3) return hipErrorInvalidValue;
  if (a.epilogue == 0 && !a.out) return hipErrorInvalidValue;
  if (a.epilogue == 1 && !a.act) return hipErrorInvalidValue;
  if (a.epilogue == 2 && (!a.q_out || !a.cache_k || !a.cache_v || !a.cos_tab || !a.sin_tab || a.T <= 0 || a.d <= 0)) return hipErrorInvalidValue;
  if (a.epilogue == 3 && (!a.x_res || a.n_peers < 0 || (a.n_peers > 0 && !a.peers) || (a.xh_b && !a.xh_a) || (a.ssq_part && !a.xh_a) ||
                          (a.xh_a && !a.gain_a) || (a.xh_b && !a.gain_b)))
    return hipErrorInvalidValue;
  if (gemm_takes_lds_kernel(a)) return launch_gemm_lds(a, s);
  // few rows: where 128-row tiles would not give every CU a workgroup, 64-row tiles (1.2B shape, 1024 rows: 9.0 -> 8.4 ms per call)
  if (a.M > 64 && (long)((a.M + 127) / 128) * ((a.N + 255) / 256) < 256) return launch_gemm_wm<4, 2>(a, s);
  if (a.M >= 1024) return launch_gemm_wm<GEMM_WM_LARGE, GEMM_WAVES_LARGE>(a, s);
  if (a.M > 64) return launch_gemm_wm<8, 2>(a, s);   // 128 x 256
  return launch_gemm_wm<4, 2>(a, s);                 //  64 x 256
}

// ------------------------------------------------------------------------------------------------
// Causal GQA flash attention for T new tokens per sequence over the cache (which already holds
// them).  Everything is computed transposed so that no operand needs a shuffle:
//   S^T[key][query] = K Q^T       A = K tile (16 keys x 32 dims, straight from the row-major K cache),
//                                 B = Q^T (16 queries x 32 dims, kept in registers);
//   a lane then owns, for ITS query (lane%16), keys 4*(lane/16)+r of each 16-key tile: the softmax
//   statistics of a query need two shuffles, and the lane's 8 probabilities of a 32-key block are,
//   as they stand, the B operand of
//   O^T[dim][query] = V^T P^T     A = V^T tile (16 dims x 32 keys) from the transposed V cache, with
//                                 the same key order (two 8-byte loads per lane).
// One wavefront owns QT tiles of 16 queries of one q head; a workgroup = 4 wavefronts.
// ------------------------------------------------------------------------------------------------
template <int D, int QT>
__global__ __launch_bounds__(256) void attn_prefill_kernel(AttnPrefillArgs a) {
  constexpr int DS = D / 32;  // 32-dim slabs
  constexpr int DT = D / 16;  // 16-dim output tiles
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int b = lane & 15, q = lane >> 4;
  const int n_qblk = gridDim.x;
  const int qblk = n_qblk - 1 - blockIdx.x;  // longest rows first
  const int h = blockIdx.y, bi = blockIdx.z;
  const int kvh = h / (a.nq / a.nkv);
  const int t0 = (qblk * 4 + wave) * QT * 16;
  if (t0 >= a.T) return;
  const float scale = 1.0f / sqrtf((float)D);
  const uint4 zero4 = make_uint4(0, 0, 0, 0);

  uint4 qreg[QT][DS];
#pragma unroll
  for (int qt = 0; qt < QT; ++qt) {
    const int t = t0 + qt * 16 + b;
#pragma unroll
    for (int s = 0; s < DS; ++s)
      qreg[qt][s] = t < a.T ? *reinterpret_cast<const uint4*>(a.q + ((size_t)bi * a.T + t) * a.nq * D + h * D +
                                                              s * 32 + q * 8)
                            : zero4;
  }
  f32x4_t oacc[QT][DT];
  float mrun[QT], lrun[QT];
#pragma unroll
  for (int qt = 0; qt < QT; ++qt) {
    mrun[qt] = -INFINITY;
    lrun[qt] = 0.f;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) oacc[qt][dt] = (f32x4_t){0.f, 0.f, 0.f, 0.f};
  }
  const bf16_t* kc = a.cache_k + ((size_t)bi * a.nkv + kvh) * a.max_seq * D;
  const bf16_t* vc = a.cache_v + ((size_t)bi * a.nkv + kvh) * D * a.max_seq;
  const int last_t = min(a.T, t0 + QT * 16) - 1;
  const int n_keys = a.pos0 + last_t + 1;

  for (int kb = 0; kb < n_keys; kb += 32) {
    uint4 kreg[2][DS];
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int s = 0; s < DS; ++s)
        kreg[t][s] = *reinterpret_cast<const uint4*>(kc + (size_t)(kb + 16 * t + b) * D + s * 32 + q * 8);
    uint4 vreg[DT];
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) {
      const bf16_t* vp = vc + (size_t)(dt * 16 + b) * a.max_seq + kb + 4 * q;
      const uint2 lo = *reinterpret_cast<const uint2*>(vp);
      const uint2 hi = *reinterpret_cast<const uint2*>(vp + 16);
      vreg[dt] = make_uint4(lo.x, lo.y, hi.x, hi.y);
    }
#pragma unroll
    for (int qt = 0; qt < QT; ++qt) {
      f32x4_t st[2];
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        st[t] = (f32x4_t){0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int s = 0; s < DS; ++s) st[t] = mfma16(kreg[t][s], qreg[qt][s], st[t]);
      }
      const int qpos = a.pos0 + t0 + qt * 16 + b;
      float sv[8];
      float mloc = -INFINITY;
#pragma unroll
      for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const int key = kb + 16 * t + 4 * q + r;
          const float v = key <= qpos ? st[t][r] * scale : -INFINITY;
          sv[t * 4 + r] = v;
          mloc = fmaxf(mloc, v);
        }
      mloc = fmaxf(mloc, __shfl_xor(mloc, 16, 64));
      mloc = fmaxf(mloc, __shfl_xor(mloc, 32, 64));
      const float mnew = fmaxf(mrun[qt], mloc);   // finite from the first block on (key 0 is always visible)
      const float corr = __expf(mrun[qt] - mnew);
      float psum = 0.f;
      float pv[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        pv[e] = __expf(sv[e] - mnew);
        psum += pv[e];
      }
      lrun[qt] = lrun[qt] * corr + psum;
      mrun[qt] = mnew;
      uint4 pb;
      pb.x = (uint32_t)f32_to_bf16(pv[0]) | ((uint32_t)f32_to_bf16(pv[1]) << 16);
      pb.y = (uint32_t)f32_to_bf16(pv[2]) | ((uint32_t)f32_to_bf16(pv[3]) << 16);
      pb.z = (uint32_t)f32_to_bf16(pv[4]) | ((uint32_t)f32_to_bf16(pv[5]) << 16);
      pb.w = (uint32_t)f32_to_bf16(pv[6]) | ((uint32_t)f32_to_bf16(pv[7]) << 16);
#pragma unroll
      for (int dt = 0; dt < DT; ++dt) {
#pragma unroll
        for (int r = 0; r < 4; ++r) oacc[qt][dt][r] *= corr;
        oacc[qt][dt] = mfma16(vreg[dt], pb, oacc[qt][dt]);
      }
    }
  }
#pragma unroll
  for (int qt = 0; qt < QT; ++qt) {
    float l = lrun[qt];
    l += __shfl_xor(l, 16, 64);
    l += __shfl_xor(l, 32, 64);
    const float inv = 1.0f / l;
    const int t = t0 + qt * 16 + b;
    if (t < a.T) {
      bf16_t* op = a.o + ((size_t)bi * a.T + t) * a.nq * D + h * D;
#pragma unroll
      for (int dt = 0; dt < DT; ++dt) {
        uint2 pk;
        pk.x = (uint32_t)f32_to_bf16(oacc[qt][dt][0] * inv) | ((uint32_t)f32_to_bf16(oacc[qt][dt][1] * inv) << 16);
        pk.y = (uint32_t)f32_to_bf16(oacc[qt][dt][2] * inv) | ((uint32_t)f32_to_bf16(oacc[qt][dt][3] * inv) << 16);
        *reinterpret_cast<uint2*>(op + dt * 16 + 4 * q) = pk;
      }
    }
  }
}

// ------------------------------------------------------------------------------------------------
// The same computation with the K / V^T tiles of a 32-key block staged once per workgroup in LDS
// (double buffered) and shared by its 4 wavefronts, each of which owns QT tiles of 16 queries of
// one q head.  With grouped-query attention the wavefronts of a workgroup are HW = min(G, 4) q heads
// of ONE kv head over the same query block, so they walk exactly the same keys.  Per block a
// wavefront issues 64 matrix instructions against 16 KiB of LDS reads; the running-max rescale of the
// output accumulators (the largest vector cost) is skipped for a tile whenever no lane's maximum moved.
// ------------------------------------------------------------------------------------------------
template <int D, int HW, int QT>
__global__ __launch_bounds__(256, QT <= 3 ? 2 : 1) void attn_prefill_lds_kernel(AttnPrefillArgs a) {
  constexpr int DS = D / 32, DT = D / 16;
  constexpr int QW = 4 / HW;                 // query sub-blocks (of QT * 16) per workgroup
  constexpr int KROW = D * 2 + 16;           // bytes per staged K row (key): 16-byte pad, conflict-free b128 reads
  constexpr int VROW = 64 + 16;              // bytes per staged V^T row (dim): 32 keys + pad
  constexpr int KBYTES = 32 * KROW, VBYTES = D * VROW;
  constexpr int SEGS = D / 64;               // 16-byte segments per thread and tile
  __shared__ __attribute__((aligned(16))) unsigned char lds[2][KBYTES + VBYTES];

  const int tid = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
  const int b = lane & 15, q = lane >> 4;
  const int qblk = (int)gridDim.x - 1 - (int)blockIdx.x;   // longest rows first
  const int h = blockIdx.y * HW + wave % HW, bi = blockIdx.z;
  const int kvh = h / (a.nq / a.nkv);
  const int t0 = (qblk * QW + wave / HW) * (QT * 16);       // this wavefront's first query
  const float scale = 1.0f / sqrtf((float)D);
  const uint4 zero4 = make_uint4(0, 0, 0, 0);

  uint4 qreg[QT][DS];
#pragma unroll
  for (int qt = 0; qt < QT; ++qt) {
    const int t = min(t0 + qt * 16 + b, a.T - 1);           // rows past T: a valid address, never stored
#pragma unroll
    for (int s = 0; s < DS; ++s)
      qreg[qt][s] = *reinterpret_cast<const uint4*>(a.q + ((size_t)bi * a.T + t) * a.nq * D + h * D + s * 32 + q * 8);
  }
  f32x4_t oacc[QT][DT];
  float mrun[QT], lrun[QT];
#pragma unroll
  for (int qt = 0; qt < QT; ++qt) {
    mrun[qt] = -INFINITY;
    lrun[qt] = 0.f;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) oacc[qt][dt] = (f32x4_t){0.f, 0.f, 0.f, 0.f};
  }
  const bf16_t* kc = a.cache_k + ((size_t)bi * a.nkv + kvh) * a.max_seq * D;
  const bf16_t* vc = a.cache_v + ((size_t)bi * a.nkv + kvh) * D * a.max_seq;
  const int wg_last_t = min(a.T, (qblk + 1) * QW * QT * 16) - 1;
  const int n_keys = a.pos0 + wg_last_t + 1;                 // keys the workgroup walks (same for all its waves)
  const int my_last = a.pos0 + min(a.T - 1, t0 + QT * 16 - 1);  // last position this wavefront's queries see
  const int n_blk = (n_keys + 31) / 32;

  u32x4_t kst[SEGS], vst[SEGS];
  auto fetch = [&](int blk) {   // global -> registers (unconditional: blk is clamped by the caller)
    const int kb = blk * 32;
#pragma unroll
    for (int i = 0; i < SEGS; ++i) {
      const int seg = tid + 256 * i;
      const int krow = seg / (D / 8), kcx = seg % (D / 8);
      kst[i] = *reinterpret_cast<const u32x4_t*>(kc + (size_t)(kb + krow) * D + kcx * 8);
      const int vrow = seg >> 2, vcx = seg & 3;
      vst[i] = *reinterpret_cast<const u32x4_t*>(vc + (size_t)vrow * a.max_seq + kb + vcx * 8);
    }
  };
  auto stash = [&](int buf) {   // registers -> LDS
#pragma unroll
    for (int i = 0; i < SEGS; ++i) {
      const int seg = tid + 256 * i;
      const int krow = seg / (D / 8), kcx = seg % (D / 8);
      *reinterpret_cast<u32x4_t*>(&lds[buf][krow * KROW + kcx * 16]) = kst[i];
      const int vrow = seg >> 2, vcx = seg & 3;
      *reinterpret_cast<u32x4_t*>(&lds[buf][KBYTES + vrow * VROW + vcx * 16]) = vst[i];
    }
  };

  fetch(0);
  stash(0);
  __syncthreads();
  for (int blk = 0; blk < n_blk; ++blk) {
    const int buf = blk & 1;
    const int kb = blk * 32;
    fetch(min(blk + 1, n_blk - 1));   // next block's tiles travel while this one is computed
    if (kb <= my_last && t0 < a.T) {
      const unsigned char* kl = &lds[buf][0];
      const unsigned char* vl = &lds[buf][KBYTES];
      f32x4_t st[QT][2];
#pragma unroll
      for (int qt = 0; qt < QT; ++qt) st[qt][0] = st[qt][1] = (f32x4_t){0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int s = 0; s < DS; ++s) {
          const uint4 kf = *reinterpret_cast<const uint4*>(kl + (16 * t + b) * KROW + s * 64 + q * 16);
#pragma unroll
          for (int qt = 0; qt < QT; ++qt) st[qt][t] = mfma16(kf, qreg[qt][s], st[qt][t]);
        }
      uint4 pb[QT];
#pragma unroll
      for (int qt = 0; qt < QT; ++qt) {
        const int qpos = a.pos0 + t0 + qt * 16 + b;
        float sv[8];
        float mloc = -INFINITY;
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
          for (int r = 0; r < 4; ++r) {
            const int key = kb + 16 * t + 4 * q + r;
            const float v = key <= qpos ? st[qt][t][r] * scale : -INFINITY;
            sv[t * 4 + r] = v;
            mloc = fmaxf(mloc, v);
          }
        mloc = fmaxf(mloc, __shfl_xor(mloc, 16, 64));
        mloc = fmaxf(mloc, __shfl_xor(mloc, 32, 64));
        const float mnew = fmaxf(mrun[qt], mloc);   // finite from the first block on (key 0 is always visible)
        const float corr = __expf(mrun[qt] - mnew);  // exactly 1 when the maximum did not move
        float psum = 0.f;
        float pv[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          pv[e] = __expf(sv[e] - mnew);
          psum += pv[e];
        }
        lrun[qt] = lrun[qt] * corr + psum;
        mrun[qt] = mnew;
        pb[qt].x = (uint32_t)f32_to_bf16(pv[0]) | ((uint32_t)f32_to_bf16(pv[1]) << 16);
        pb[qt].y = (uint32_t)f32_to_bf16(pv[2]) | ((uint32_t)f32_to_bf16(pv[3]) << 16);
        pb[qt].z = (uint32_t)f32_to_bf16(pv[4]) | ((uint32_t)f32_to_bf16(pv[5]) << 16);
        pb[qt].w = (uint32_t)f32_to_bf16(pv[6]) | ((uint32_t)f32_to_bf16(pv[7]) << 16);
        if (__any(corr != 1.0f)) {   // wave-uniform: some query of the tile has a new maximum
#pragma unroll
          for (int dt = 0; dt < DT; ++dt)
#pragma unroll
            for (int r = 0; r < 4; ++r) oacc[qt][dt][r] *= corr;
        }
      }
#pragma unroll
      for (int dt = 0; dt < DT; ++dt) {
        const unsigned char* vp = vl + (dt * 16 + b) * VROW + q * 8;
        const uint2 lo = *reinterpret_cast<const uint2*>(vp);
        const uint2 hi = *reinterpret_cast<const uint2*>(vp + 32);
        const uint4 vf = make_uint4(lo.x, lo.y, hi.x, hi.y);
#pragma unroll
        for (int qt = 0; qt < QT; ++qt) oacc[qt][dt] = mfma16(vf, pb[qt], oacc[qt][dt]);
      }
    }
    stash(buf ^ 1);   // that buffer was last read before the previous barrier
    __syncthreads();
  }
  if (t0 >= a.T) return;
#pragma unroll
  for (int qt = 0; qt < QT; ++qt) {
    float l = lrun[qt];
    l += __shfl_xor(l, 16, 64);
    l += __shfl_xor(l, 32, 64);
    const float inv = 1.0f / l;
    const int t = t0 + qt * 16 + b;
    if (t < a.T) {
      bf16_t* op = a.o + ((size_t)bi * a.T + t) * a.nq * D + h * D;
#pragma unroll
      for (int dt = 0; dt < DT; ++dt) {
        uint2 pk;
        pk.x = (uint32_t)f32_to_bf16(oacc[qt][dt][0] * inv) | ((uint32_t)f32_to_bf16(oacc[qt][dt][1] * inv) << 16);
        pk.y = (uint32_t)f32_to_bf16(oacc[qt][dt][2] * inv) | ((uint32_t)f32_to_bf16(oacc[qt][dt][3] * inv) << 16);
        *reinterpret_cast<uint2*>(op + dt * 16 + 4 * q) = pk;
      }
    }
  }
}

#define ATTN_LDS_QT 3   // 16-query tiles per wavefront.  Measured on 16 x 2048 tokens, 16 q / 2 kv heads, d = 128:
                        // 2 tiles 0.80 ms, 3 tiles 0.55 ms, 4 tiles 1.45 ms per layer (4 leaves one wavefront
                        // per SIMD, which cannot hide the global -> LDS latency; 2 doubles the LDS reads per flop)
template <int D>
static hipError_t launch_attn_prefill_lds(const AttnPrefillArgs& a, hipStream_t s) {
  const int g = a.nq / a.nkv;
  const int hw = g >= 4 && g % 4 == 0 ? 4 : (g % 2 == 0 ? 2 : 1);
  constexpr int QT = ATTN_LDS_QT;
  const int qrows = (4 / hw) * QT * 16;
  const dim3 grid((a.T + qrows - 1) / qrows, a.nq / hw, a.B), block(256);
  if (hw == 4) hipLaunchKernelGGL((attn_prefill_lds_kernel<D, 4, QT>), grid, block, 0, s, a);
  else if (hw == 2) hipLaunchKernelGGL((attn_prefill_lds_kernel<D, 2, QT>), grid, block, 0, s, a);
  else hipLaunchKernelGGL((attn_prefill_lds_kernel<D, 1, QT>), grid, block, 0, s, a);
  return hipGetLastError();
}

hipError_t launch_attn_prefill(const AttnPrefillArgs& a, hipStream_t s) {
  // long prompts: the LDS-shared kernel (its reads run to the end of the last 32-key block, which the
  // cache capacity, a multiple of 128, always covers); short ones keep more workgroups with the direct one
  if (a.T >= 256 && (a.max_seq & 31) == 0) {
    if (a.d == 128) return launch_attn_prefill_lds<128>(a, s);
    if (a.d == 64) return launch_attn_prefill_lds<64>(a, s);
    return hipErrorInvalidValue;
  }
  constexpr int QT = 2;
  const int bq = 4 * QT * 16;
  const dim3 grid((a.T + bq - 1) / bq, a.nq, a.B);
  if (a.d == 128) hipLaunchKernelGGL((attn_prefill_kernel<128, QT>), grid, dim3(256), 0, s, a);
  else if (a.d == 64) hipLaunchKernelGGL((attn_prefill_kernel<64, QT>), grid, dim3(256), 0, s, a);
  else return hipErrorInvalidValue;
  return hipGetLastError();
}
