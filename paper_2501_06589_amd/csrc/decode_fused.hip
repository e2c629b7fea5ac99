// Fused decode path of the bf16 storage type (gfx950), batch <= 16, one computed shard.
//
// One launch runs up to four JOBS side by side (workgroups pick their job from the block index).
// Under the ladder wiring module m+1 needs only x_{m-1}, so the MLP projections of layer l and the
// attention-side work around them have no dependency on each other: putting them into ONE launch
// keeps HBM streaming while the small, latency-bound attention work runs, with no stream, event or
// graph edge in between.  A decode step is two launches per layer:
//     { attention_l , gate/up_l (+ RMSNorm, SwiGLU) , o_l (+ residual add; waits for attention_l) }
//     { qkv_{l+1} (+ RMSNorm, rotary, cache append) , down_l (+ residual add) }
// Everything that used to be a kernel of its own is an epilogue or a prologue here.  Workgroups do not
// talk to each other, with two exceptions that involve a few dozen producers only: the splits of a long
// attention meet through an arrival ticket, and o_l waits on a counter that the attention workgroups
// raise.  Neither hand-off uses a fence (an agent-scope release writes back, and an acquire invalidates, the
// XCD's whole L2 under the weight streams: 1.2 - 2.5 us each where measured, and a release per workgroup of
// a whole projection cost more than the projection itself): the producer writes with device-coherent stores,
// waits for them, then takes the ticket or raises the counter; the consumer reads with device-coherent loads:
//   * the residual update of Algorithm 1 with the all-reduce written as a sum over rank partial
//     sums (Eq. 2) is the epilogue of the module's last projection: x_m = x_{m-1} + h_m + sum(peers),
//     written to a ring of three residual buffers (x_{m-1} is still read by the job that runs beside);
//   * RMSNorm: that same epilogue multiplies the new rows by the gain of the module that will read them (in
//     fp32) and leaves them as the split matrix-core operand of that module, together with the rows' sums of
//     squares per 16-column tile; the reading projection adds those up and scales its outputs by 1/rms at the
//     end (the factor commutes with the product);
//   * rotary embedding + KV append: epilogue of the QKV projection;
//   * attention: one workgroup per (sequence, kv head); its 8 wavefronts share out the visible
//     positions, each with a running softmax on the matrix cores, and merge through LDS, so nothing is
//     left to combine across workgroups; only when the cache is long enough to be split do the splits
//     meet through an arrival ticket.
// Precision: the weights and the cache are bf16 (storage); every operand this path itself produces for the
// matrix core (stream rows, q, softmax weights, attention output, SwiGLU output) is SPLIT into a high and a
// low bf16 part (see decode_fused.h), so nothing is rounded to 8 bits between the modules; sums are fp32.
// All sums are taken in a fixed order, so results are bit-reproducible run to run.
#include <hip/hip_ext.h>

#include <algorithm>

#include "common.h"
#include <cstddef>
#include "decode_fused.h"

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8_t;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4_t;
typedef __attribute__((__vector_size__(4 * sizeof(uint32_t)))) uint32_t u32x4_t;

#define FUSED_THREADS 512
#define FUSED_WAVES 8
// descriptor byte of a job in the preloaded `kinds` argument of the kernel
#define FUSED_K_ROTATE 13           // k tiles by which neighbouring tile groups' sweeps of the K range are apart
#define FUSED_KIND_MASK 3u          // JOB_NONE / JOB_GEMV / JOB_ATTN
#define FUSED_KIND_TN_SHIFT 2       // two bits: tiles per workgroup - 1 (1 .. 4 tiles)
#define FUSED_KIND_WAITS 32u        // the job waits for another job of the launch
#define FUSED_KIND_SLOT_SHIFT 6     // two bits: index of the job's preloaded (weights, operand) pointer pair, 3 = none

// k tiles per register buffer (two buffers) of a one-tile / a two-tile workgroup: 4 KiB of weights in flight
// per wavefront.  With the round-robin assignment of k tiles below, 2 beat 4 (3.57 against 3.65 ms per step;
// 1 gave 4.04, 3 gave 3.74: its turns do not divide the k range).  Two-tile workgroups take two k tiles per
// buffer as well: in a chained step 3.26 -> 3.23 ms per step (the output projection's whole weight share, 64 KiB,
// is then requested before its wait); as separate launches that costs 1.4 %, accepted so that both schedules sum
// in the same order and give the same bits (the k tiles a wavefront takes follow from this number).  Three- and
// four-tile workgroups: one (two: 2.6 % slower).
#define FUSED_U 2
#define FUSED_U2 2
#define FUSED_POLL_SLEEP 8      // s_sleep units (64 clocks) between two polls of a wait (2 measured the same)
#define FUSED_LDS_FLOATS 9216   // attention job: per-wave statistics and outputs

__device__ __forceinline__ uint32_t pack_bf16(float a, float b) {
  return (uint32_t)f32_to_bf16(a) | ((uint32_t)f32_to_bf16(b) << 16);
}

__device__ __forceinline__ void unpack8f(const uint4 v, float f[8]) {
  f[0] = __uint_as_float(v.x << 16); f[1] = __uint_as_float(v.x & 0xFFFF0000u);
  f[2] = __uint_as_float(v.y << 16); f[3] = __uint_as_float(v.y & 0xFFFF0000u);
  f[4] = __uint_as_float(v.z << 16); f[5] = __uint_as_float(v.z & 0xFFFF0000u);
  f[6] = __uint_as_float(v.w << 16); f[7] = __uint_as_float(v.w & 0xFFFF0000u);
}

// v as two bf16 numbers: hi = bf16(v), lo = bf16(v - hi); hi + lo carries 16 significant bits of v
// (the subtraction is kept out of fused multiply-adds: where v is a product, fma(a, b, -hi) would take the low part
// from the unrounded product, and whether the compiler forms it depends on the code around the call)
__device__ __forceinline__ void split_bf16(float v, uint32_t& hi, uint32_t& lo) {
#pragma clang fp contract(off)
  hi = f32_to_bf16(v);
  const float rest = v - __uint_as_float(hi << 16);
  lo = f32_to_bf16(rest);
}

// the value that lane ^ 8 holds (DPP rotation by 8 within each row of 16 lanes): joins the two halves of a split
// operand's result, whose high parts sit in operand columns 0..7 and low parts in columns 8..15
__device__ __forceinline__ float other_half(float v) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x128 /* row_ror:8 */, 0xF, 0xF, false));
}

// The thread index as a value the compiler knows nothing about.  A job is inlined into a loop over a
// workgroup's jobs (chained step): everything derived from the plain thread index is loop invariant, and the
// compiler would compute the LDS addresses and lane masks of every job variant ahead of the loop and keep them
// in private memory.
__device__ __forceinline__ int opaque_tid() {
  int t = (int)threadIdx.x;
  asm volatile("" : "+v"(t));
  return t;
}

// Cross-lane sums on the DPP path of the vector ALU (a __shfl_xor goes through the LDS crossbar instead: some
// sixty cycles each, in a dependent chain).  All 64 lanes must be active.
template <int CTRL>
__device__ __forceinline__ float dpp_read(float v) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xF, 0xF, false));
}
// every lane: the sum over its row of 16 lanes (neighbour, other pair, other quad of 8 mirrored, other half mirrored)
__device__ __forceinline__ float row16_sum(float v) {
  v += dpp_read<0xB1>(v);    // quad_perm [1,0,3,2]
  v += dpp_read<0x4E>(v);    // quad_perm [2,3,0,1]
  v += dpp_read<0x141>(v);   // row_half_mirror
  v += dpp_read<0x140>(v);   // row_mirror
  return v;
}
// every lane: the sum over the wavefront, rows added in the order 0, 1, 2, 3
__device__ __forceinline__ float wave_sum_dpp(float v) {
  v = row16_sum(v);
  const int i = __float_as_int(v);
  return __int_as_float(__builtin_amdgcn_readlane(i, 0)) + __int_as_float(__builtin_amdgcn_readlane(i, 16)) +
         __int_as_float(__builtin_amdgcn_readlane(i, 32)) + __int_as_float(__builtin_amdgcn_readlane(i, 48));
}

// Device-coherent stores / loads (agent-scope relaxed atomics: written through to memory, read past the caches
// that are not coherent across the chip) for the few values one workgroup hands to another inside a launch.
// A producer waits until its coherent stores have completed (s_waitcnt) before it takes a ticket or raises a
// counter; a consumer reads the data with coherent loads after it has seen the ticket or the counter.  No
// fence on either side: an agent-scope release writes back, and an acquire invalidates, the whole L2 of the XCD
// under the weight streams that run beside (1.2 - 2.5 us each on this path).
__device__ __forceinline__ void st_coherent(uint32_t* p, uint32_t v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void st_coherent(float* p, float v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void st_coherent(bf16_t* p, bf16_t v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float ld_coherent(const float* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// stores a split value whose high part belongs at hi_at and whose low part at lo_at, for an element with an even
// index i whose neighbour i ^ 1 lies right behind it: lanes i and i ^ 1 pair up for one 32-bit coherent store
// each (all lanes of the wave must call; ok = this pair is to be stored, the same on both of its lanes)
__device__ __forceinline__ void st_coherent_split_pair(bf16_t* hi_at, bf16_t* lo_at, int i, float v, bool ok = true) {
  uint32_t h, l;
  split_bf16(v, h, l);
  const uint32_t oh = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)h, 0xB1, 0xF, 0xF, false);   // the neighbour lane's (quad_perm [1,0,3,2])
  const uint32_t ol = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)l, 0xB1, 0xF, 0xF, false);
  if ((i & 1) == 0 && ok) {
    st_coherent(reinterpret_cast<uint32_t*>(hi_at), h | (oh << 16));
    st_coherent(reinterpret_cast<uint32_t*>(lo_at), l | (ol << 16));
  }
}

// Completion words of a producer (a projection, or the attention job of a layer): FUSED_SYNC_WORDS words, used in
// one of two ways.
// Counted: eight sub-counters, a cache line each, and ONE further line of eight flag words that the consumers
// poll.  A producer workgroup whose coherent stores have completed counts itself on the sub-counter of its ordinal
// mod 8; the one that completes a sub-counter raises that counter's flag word, and a consumer goes on when all
// eight are up (one 32-byte load per poll).  Hundreds of atomics on ONE line queue up behind each other, and behind
// the loads of whoever polls that line (microseconds for a whole projection): hence eight lines to count on and
// nobody polling a line that is counted on.  (A ninth counter for the eight finishers, whose last raised a single
// flag, cost every hand-off one more atomic round trip.  Counting without waiting for the atomics' results and
// letting every consumer poll all eight counters made every hand-off 2 - 3 us longer, the polls of 512 workgroups
// on eight lines being traffic of their own.)
// Flagged (n_flags > 0, at most 256): word i is the flag of producer workgroup i, which stores a 1 there, and a
// consumer polls all n_flags words with one load of its first wavefront.  No atomic, so the producer's end is a
// memory round trip (or two) shorter; the polls read up to eight lines instead of one, which is affordable where
// the producer is small or its consumers are few (the host decides).
__device__ __forceinline__ void sync_count(unsigned* words, unsigned ordinal, unsigned total, bool flagged) {
  if (flagged) {
    __hip_atomic_store(words + ordinal, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    return;
  }
  if (total > 16u) {
    const unsigned k = ordinal & 7u;
    const unsigned n_k = (total + 7u - k) >> 3;   // workgroups with this ordinal mod 8 (at least two)
    if (atomicAdd(words + 32u * k, 1u) == n_k - 1u)
      __hip_atomic_store(words + FUSED_SYNC_FLAG_WORD + k, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  } else if (atomicAdd(words, 1u) == total - 1u) {   // a small producer: one counter, its finisher raises all eight words
#pragma unroll
    for (unsigned k = 0; k < 8u; ++k)
      __hip_atomic_store(words + FUSED_SYNC_FLAG_WORD + k, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
}
// One poll of a producer's words by a whole wavefront: counted (n_flags = 0): lanes 0..3 read the eight flag words,
// two each; flagged: lane i reads the words 4i .. 4i+3 (two 8-byte coherent loads).  True if every word in use has reached 1 + bias (bias: a
// test's way of making the wait fail).
__device__ __forceinline__ bool sync_poll(const unsigned* words, unsigned n_flags, unsigned bias, int lane) {
  bool ok = true;
  if (n_flags == 0u) {
    if (lane < 4) {
      const unsigned long long v = __hip_atomic_load(reinterpret_cast<const unsigned long long*>(words + FUSED_SYNC_FLAG_WORD) + lane,
                                                     __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      ok = (unsigned)v >= 1u + bias && (unsigned)(v >> 32) >= 1u + bias;
    }
  } else if (4u * (unsigned)lane < n_flags) {
    const unsigned long long* p = reinterpret_cast<const unsigned long long*>(words) + 2 * lane;
    const unsigned long long a = __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    const unsigned long long b = __hip_atomic_load(p + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    const unsigned w[4] = {(unsigned)a, (unsigned)(a >> 32), (unsigned)b, (unsigned)(b >> 32)};
#pragma unroll
    for (int i = 0; i < 4; ++i)
      if (4u * (unsigned)lane + (unsigned)i < n_flags) ok = ok && w[i] >= 1u + bias;
  }
  return ok;
}
// waits (bounded) for one or two producers (w2 null: one); all 64 lanes of the wavefront must call
__device__ __forceinline__ bool sync_wait(const unsigned* w1, unsigned n1, const unsigned* w2, unsigned n2, unsigned bias,
                                          int spins, int lane) {
  for (int spin = 0; spin < spins; ++spin) {
    bool ok = sync_poll(w1, n1, bias, lane);
    if (w2) ok = sync_poll(w2, n2, bias, lane) && ok;   // (both polls' loads are in flight together)
    if (__all(ok)) return true;
    __builtin_amdgcn_s_sleep(FUSED_POLL_SLEEP);
  }
  return false;
}
// A producer job of a chained step: the workgroup's coherent stores have completed, count it.
__device__ __forceinline__ void gemv_signal_done(const GemvJob& j, int lb) {
  if (!j.done_ctr) return;
  __builtin_amdgcn_s_waitcnt(0);   // this thread's coherent stores have completed
  __syncthreads();
  if (threadIdx.x == 0) sync_count(j.done_ctr, j.done_ord0 + (unsigned)lb, j.done_target, j.done_flagged != 0);
}

// ------------------------------------------------------------------------------------------------
// skinny GEMM job: see gemv_mfma_kernel for the streaming scheme (same tiles, same pipeline).
// A workgroup owns TN adjacent 16-column tiles and the whole K range; U k-tiles per register buffer.
// A wavefront's streaming rate is its bytes in flight over the memory latency, so the launch time is
// set by the workgroup with the most bytes: one tile per workgroup keeps the jobs of a launch even
// and the number of streaming workgroups high.
// ------------------------------------------------------------------------------------------------
// wp, xop, KT, group0 and M repeat j.wp, j.xb, j.K / 32, j.group0 and j.M (the x rows are K elements apart): the
// kernel hands them over from preloaded kernel arguments where it can, so that the first weight tiles and
// operand slices are requested before the job's descriptor (j) has arrived from memory.
// WIDE = more than 8 rows: the high and the low parts of the operand are two MFMA operands (rows 0..15 each);
// else one: lanes 0..7 of a row of 16 carry the high parts of rows 0..7, lanes 8..15 their low parts.
// Operand columns beyond the rows in use hold whatever their slots hold (finite): a column of the operand only
// reaches its own column of the result, which nobody reads.
// CHAIN: the job is part of a chained step: other jobs of the same launch read what it writes, so the results go
// out with device-coherent stores (else: ordinary stores, the launch's end publishes them), and it may be waiting for
// any of its inputs, so the operand is requested behind the waits (else, unless COH: at once, with the weights).
// x_out: where a job with x_copy set leaves its second copy of the new rows, if not null (the chained step hands the
// caller's buffer over as a kernel argument; else x_copy itself is the place).  t_ready: if not null, thread 0
// leaves the wall-clock time there at which the job's waits were over.
// Returns false if a wait gave up (nothing stored, error word raised).
template <int U, int TN, bool COH, bool WIDE, bool CHAIN>
__device__ __forceinline__ bool gemv_job(const GemvJob& j, const void* wp, const bf16_t* xop, int KT, int group0, int M, int lb,
                                         float* smem, unsigned* s_flag, float* x_out, unsigned long long* t_ready) {
  constexpr bool EARLY_X = !COH && !CHAIN;
  constexpr int WAVES = FUSED_WAVES;
  constexpr int XP = WIDE ? 2 : 1;   // operand registers per k tile
  const int grp = group0 + lb;
  const int tid = opaque_tid();
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
  const int b = lane & 15, q = lane >> 4;
  const int nt0 = grp * TN;
  // The wavefronts take groups of U k tiles round robin, so that the workgroup as a whole sweeps its weight range
  // once, 8 U tiles (16 KiB) at a time: measured 3 % faster over a decode step than a contiguous eighth of the
  // range per wavefront (DRAM page locality); tile-wise round robin and 2 U tiles per turn were slower.
  constexpr int KB = WAVES * U, KA = 2 * WAVES * U;   // tile distance to the second register buffer / to the next turn
  const int kt0 = wave * U;
  const int kt1 = KT;

  f32x4_t acc[TN];
#pragma unroll
  for (int t = 0; t < TN; ++t) acc[t] = (f32x4_t){0.f, 0.f, 0.f, 0.f};
  const u32x4_t* wptr = reinterpret_cast<const u32x4_t*>(wp) + ((size_t)nt0 * KT) * 64 + lane;
  // operand slot of this lane (decode_fused.h): WIDE: slot b = row b of the high parts, the low parts 16 slots
  // further; else the k tile has S = 2, 4, 8 or 16 slots, the first half high parts, the second half low parts:
  // lanes 0..7 of a row of 16 take the high slots (repeating them when there are fewer than 8), lanes 8..15 the low ones
  const int S = WIDE ? 32 : fused_slots(M);
  const int slot = WIDE ? b : ((b & ((S >> 1) - 1)) + ((b & 8) ? (S >> 1) : 0));
  const int tile_stride = S * 32;                      // elements per k tile
  const bf16_t* xbp = xop + (q * S + slot) * 8;
  constexpr int low_off = 16 * 8;                      // WIDE: the low parts' slots
  u32x4_t wa[TN][U], wb[TN][U], xa[U][XP], xb[U][XP];
  // Where in its K range a workgroup starts: rotated by a number of k tiles that depends on its tile group, so that
  // the workgroups that stream side by side are not all at the same offset of their tiles, which lie a power of two
  // apart, at the same time (memory channels; headline shape: 3.22 -> 3.19 ms per step chained, 3.43 -> 3.38 as separate
  // launches).  A group of four tiles shares a rotation: a tile's sum has the same order whether its workgroup takes
  // one tile or two (four-tile workgroups split the k tiles over their wavefronts differently anyway).
  const int rot = ((nt0 >> 2) * FUSED_K_ROTATE) % KT;
  auto rotated = [&](int k) { return k + rot >= KT ? k + rot - KT : k + rot; };
  auto loadw = [&](u32x4_t (&wv)[TN][U], int kt) {
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int ktc = rotated(min(kt + u, kt1 - 1));
#pragma unroll
      for (int t = 0; t < TN; ++t) wv[t][u] = __builtin_nontemporal_load(wptr + ((size_t)t * KT + ktc) * 64);
    }
  };
  auto loadx = [&](u32x4_t (&xv)[U][XP], int kt) {
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int ktc = rotated(min(kt + u, kt1 - 1));
#pragma unroll
      for (int h = 0; h < XP; ++h) {
        const bf16_t* src = xbp + (size_t)ktc * tile_stride + (h ? low_off : 0);
        if (COH) {   // operand written by another workgroup of this launch: device-coherent loads, past L1 and the XCD's L2
          const unsigned long long* p8 = reinterpret_cast<const unsigned long long*>(src);
          const unsigned long long lo = __hip_atomic_load(p8, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          const unsigned long long hi = __hip_atomic_load(p8 + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          xv[u][h] = (u32x4_t){(uint32_t)lo, (uint32_t)(lo >> 32), (uint32_t)hi, (uint32_t)(hi >> 32)};
        } else {
          xv[u][h] = *reinterpret_cast<const u32x4_t*>(src);
        }
      }
    }
  };
  auto load = [&](u32x4_t (&wv)[TN][U], u32x4_t (&xv)[U][XP], int kt) {
    loadw(wv, kt);
    loadx(xv, kt);
  };
  // the first tiles depend on nothing but the (preloaded) arguments: requested before anything else; the operand
  // of a job that waits for its producer only behind the wait
  // both register buffers
  if (kt0 < kt1) loadw(wa, kt0);
  if (kt0 + KB < kt1) loadw(wb, kt0 + KB);
  if (EARLY_X && kt0 < kt1) loadx(xa, kt0);
  if (EARLY_X && kt0 + KB < kt1) loadx(xb, kt0 + KB);
  __builtin_amdgcn_sched_barrier(0);

  if (j.wait_on) {
    // What the job reads comes from other jobs of this launch.  A workgroup only waits for workgroups that come
    // before it in the launch's order and that wait, in turn, only for earlier ones: the words always arrive.  The
    // wait is bounded all the same, so that the kernel ends whatever happens; a workgroup whose wait gives up stores
    // nothing and raises the error word, which the host reads at the library's next call.
    if (wave == 0) {
      const bool arrived = sync_wait(j.wait_on, j.wait_flags, j.wait_on2, j.wait_flags2, j.wait_bias, j.wait_spins, lane);
      if (lane == 0) {
        *s_flag = arrived ? 1u : 0u;
        if (!arrived && j.err_word) __hip_atomic_store(j.err_word, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
      }
    }
    __syncthreads();   // (workgroup-scope ordering.  No cache invalidation: the attention output is read with
                       // device-coherent loads, and what a projection of the same launch has written is in no cache
                       // of this XCD yet, having been read by nobody before; an agent-scope acquire per workgroup
                       // would flush the L2 under the weight streams that run beside)
    if (*s_flag == 0u) return false;
  }

  if (j.t_ready) {
    // emulated collective: the stream this job reads counts as reduced delay_ticks after the time its producer
    // left; a wait on the clock alone (it ends whatever other workgroups do), bounded all the same
    if (tid == 0) {
      const unsigned long long t1 = __hip_atomic_load(j.t_ready, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) + j.delay_ticks;
      for (int spin = 0; spin < (1 << 20); ++spin) {
        if (wall_clock64() >= t1) break;
        __builtin_amdgcn_s_sleep(FUSED_POLL_SLEEP);
      }
    }
    __syncthreads();
  }

  if (t_ready && tid == 0) *t_ready = wall_clock64();
  if (!EARLY_X && kt0 < kt1) loadx(xa, kt0);
  if (!EARLY_X && kt0 + KB < kt1) loadx(xb, kt0 + KB);
  // results: coherent stores in a chained step (a split value's two halves as 32-bit stores of a column pair, all
  // lanes of the wavefront taking part), ordinary stores else
  auto store_f32 = [&](float* p, float v) {
    if (CHAIN) st_coherent(p, v);
    else *p = v;
  };
  auto store_u32 = [&](uint32_t* p, uint32_t v) {
    if (CHAIN) st_coherent(p, v);
    else *p = v;
  };
  auto store_b16 = [&](bf16_t* p, bf16_t v) {
    if (CHAIN) st_coherent(p, v);
    else *p = v;
  };
  auto store_split = [&](bf16_t* hi_at, bf16_t* lo_at, int i, float v, bool ok) {
    if (CHAIN) {
      st_coherent_split_pair(hi_at, lo_at, i, v, ok);
    } else if (ok) {
      uint32_t hi, lo;
      split_bf16(v, hi, lo);
      *hi_at = (bf16_t)hi;
      *lo_at = (bf16_t)lo;
    }
  };
  auto fma = [&](const u32x4_t (&wv)[TN][U], const u32x4_t (&xv)[U][XP], int kt) {
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const bool ok = kt + u < kt1;
#pragma unroll
      for (int h = 0; h < XP; ++h) {
        const u32x4_t xz = ok ? xv[u][h] : (u32x4_t){0u, 0u, 0u, 0u};
#pragma unroll
        for (int t = 0; t < TN; ++t)
          acc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, wv[t][u]),
                                                          __builtin_bit_cast(bf16x8_t, xz), acc[t], 0, 0, 0);
      }
    }
  };
  // The epilogue's own operands do not depend on the product: they are requested now, before the
  // weight stream, so their memory latency is hidden behind it instead of trailing the last tile.
  // (a thread owns output elements tid, tid + 512, ...: one for one or two tiles per workgroup, two for three)
  constexpr int PRE_PEERS = 8;
  constexpr int E_RES = (TN * 256 + FUSED_THREADS - 1) / FUSED_THREADS;   // residual epilogue: elements per thread
  float pre_old[E_RES], pre_cos = 0.f, pre_sin = 0.f;
  uint16_t pre_peer[E_RES][PRE_PEERS], pre_ga[E_RES], pre_gb[E_RES];
  int pre_pos = 0;
  // normed: this thread's share of the rows' sums of squares, tile tid of the stream, four rows per register quad
  float4 pre_ss[4];
  const int n_st = KT * 2;   // 16-column tiles of the stream the operand was made from
  if (j.normed) {
#pragma unroll
    for (int rq = 0; rq < 4; ++rq) {
      pre_ss[rq] = make_float4(0.f, 0.f, 0.f, 0.f);
      if (rq * 4 < M) pre_ss[rq] = *reinterpret_cast<const float4*>(j.ssq + (size_t)min(tid, n_st - 1) * 16 + rq * 4);
    }
  }
  if (j.epi == EPI_RESIDUAL) {
#pragma unroll
    for (int e = 0; e < E_RES; ++e) {
      const int idx = tid + e * FUSED_THREADS;
      pre_old[e] = 0.f;
      pre_ga[e] = pre_gb[e] = 0x3F80;   // 1.0
      if (idx < TN * 256) {
        const int t = idx >> 8, row = min((idx >> 4) & 15, j.M - 1), col = (nt0 + t) * 16 + (idx & 15);
        pre_old[e] = j.x_old[(size_t)row * j.N + col];
        if (j.xop_a) pre_ga[e] = j.gain_a[col];
        if (j.xop_b) pre_gb[e] = j.gain_b[col];
        if (j.n_peers > 0) {
#pragma unroll
          for (int p = 0; p < PRE_PEERS; ++p)
            pre_peer[e][p] = j.peers[min(p, j.n_peers - 1) * j.peer_stride + (size_t)row * j.N + col];
        }
      }
    }
  } else if (j.epi == EPI_QKV_ROPE) {
    pre_pos = *j.pos_dev;
    if (tid < 16 * TN * 8) {
      const int pr = tid % (TN * 8);
      const int jj = ((grp * (TN * 16) + 2 * pr) % j.d) >> 1;
      pre_cos = j.cos_tab[(size_t)pre_pos * (j.d >> 1) + jj];
      pre_sin = j.sin_tab[(size_t)pre_pos * (j.d >> 1) + jj];
    }
  }

  if (kt0 < kt1) {
    // buffer a holds the tiles of kt, buffer b those of kt + KB (where the range reaches that far): each is
    // requested again, a turn ahead, as soon as it has been used.  Nothing is requested beyond the range: a load
    // left in flight at the end (even one clamped onto the last tile, which the caches serve) is waited for by
    // whatever the epilogue reads first, a memory round trip at the end of every workgroup.
    int kt = kt0;
    for (; kt + KA < kt1; kt += KA) {
      fma(wa, xa, kt);
      __builtin_amdgcn_sched_barrier(0);
      load(wa, xa, kt + KA);
      __builtin_amdgcn_sched_barrier(0);
      fma(wb, xb, kt + KB);
      __builtin_amdgcn_sched_barrier(0);
      if (kt + KA + KB < kt1) load(wb, xb, kt + KA + KB);   // (uniform over the wavefront)
      __builtin_amdgcn_sched_barrier(0);
    }
    fma(wa, xa, kt);
    __builtin_amdgcn_sched_barrier(0);
    if (kt + KB < kt1) fma(wb, xb, kt + KB);
  }

  // cross-wave sums through LDS: red[wave][tile][col in tile][operand column], ssq[wave][row]
  float* red = smem;                            // WAVES * TN * 16 * 17 floats
  float* ssq = smem + WAVES * TN * 16 * 17;     // WAVES * 16 floats
#pragma unroll
  for (int t = 0; t < TN; ++t)
#pragma unroll
    for (int r = 0; r < 4; ++r) red[((wave * TN + t) * 16 + 4 * q + r) * 17 + b] = acc[t][r];
  if (j.normed) {
    // the rows' sums of squares: this thread's tile (and, for streams of more than 512 tiles, the tiles beyond),
    // then the wavefront, then (below) the eight wavefronts, always in this order
#pragma unroll
    for (int rq = 0; rq < 4; ++rq) {
      if (rq * 4 >= M) break;
      float4 v = tid < n_st ? pre_ss[rq] : make_float4(0.f, 0.f, 0.f, 0.f);
      for (int tile = tid + FUSED_THREADS; tile < n_st; tile += FUSED_THREADS) {
        const float4 t4 = *reinterpret_cast<const float4*>(j.ssq + (size_t)tile * 16 + rq * 4);
        v.x += t4.x; v.y += t4.y; v.z += t4.z; v.w += t4.w;
      }
      v.x = wave_sum_dpp(v.x); v.y = wave_sum_dpp(v.y); v.z = wave_sum_dpp(v.z); v.w = wave_sum_dpp(v.w);
      if (lane == 0) {
        float* dst = ssq + wave * 16 + rq * 4;
        dst[0] = v.x; dst[1] = v.y; dst[2] = v.z; dst[3] = v.w;
      }
    }
  }
  __syncthreads();
  auto out_of = [&](int t, int col16, int row) {  // finished output element: wave sums (high + low half), then 1/rms of the row
    float v = 0.f;
#pragma unroll
    for (int w = 0; w < WAVES; ++w) {
      const float* r = red + ((w * TN + t) * 16 + col16) * 17;
      v += WIDE ? r[row] : r[row] + r[row + 8];
    }
    if (j.normed) {
      float s = 0.f;
#pragma unroll
      for (int w = 0; w < WAVES; ++w) s += ssq[w * 16 + row];
      v *= 1.0f / sqrtf(s / (float)j.K + j.eps);
    }
    return v;
  };

  if (j.epi == EPI_SWIGLU) {
    // tile columns 0..7 = gate columns 8nt..8nt+7, columns 8..15 = the matching up columns
    const int I = j.N >> 1;
    if (tid < TN * 128) {   // (whole wavefronts: the lanes of a column pair store together)
      const int t = tid >> 7, row = (tid >> 3) & 15, c8 = tid & 7;
      const int col = (nt0 + t) * 8 + c8;
      const bool ok = row < j.M && col < I;   // (I is even: a pair is in or out as a whole)
      float v = 0.f;
      if (ok) {
        const float g = out_of(t, c8, row), u = out_of(t, c8 + 8, row);
        v = g / (1.0f + __expf(-g)) * u;
      }
      bf16_t* const at = j.act + fused_xop_offset(S, ok ? row : 0, ok ? col : 0);
      store_split(at, at + (S / 2) * 8, c8, v, ok);
    }
    if (CHAIN) gemv_signal_done(j, lb);
    return true;
  }

  if (j.epi == EPI_RESIDUAL) {
#pragma unroll
    for (int e = 0; e < E_RES; ++e) {
      const int idx = tid + e * FUSED_THREADS;
      if (idx >= TN * 256) break;   // (uniform over a wavefront: TN * 256 is a multiple of 64)
      const int t = idx >> 8, row = (idx >> 4) & 15, col16 = idx & 15;
      const int col = (nt0 + t) * 16 + col16;
      const bool ok = row < j.M;
      float v = 0.f;
      if (ok) {
        v = pre_old[e] + out_of(t, col16, row);
#pragma unroll
        for (int p = 0; p < PRE_PEERS; ++p)
          if (p < j.n_peers) v += bf16_to_f32(pre_peer[e][p]);
        for (int p = PRE_PEERS; p < j.n_peers; ++p) v += bf16_to_f32(j.peers[p * j.peer_stride + (size_t)row * j.N + col]);
        store_f32(j.x_new + (size_t)row * j.N + col, v);
        if (j.x_copy) (x_out ? x_out : j.x_copy)[(size_t)row * j.N + col] = v;
      }
      // what the modules that read x_m multiply: x_m times their norm's gain, split (the lanes of a column pair
      // store together, so all lanes of the wavefront take part)
      const size_t at = fused_xop_offset(S, ok ? row : 0, col);
      if (j.xop_a) store_split(j.xop_a + at, j.xop_a + at + (S / 2) * 8, col16, v * bf16_to_f32(pre_ga[e]), ok);
      if (j.xop_b) store_split(j.xop_b + at, j.xop_b + at + (S / 2) * 8, col16, v * bf16_to_f32(pre_gb[e]), ok);
      // the row's sum of squares over this tile's 16 columns (the 16 lanes that share t and row)
      const float s = row16_sum(v * v);
      if (col16 == 0 && ok && j.ssq_new) store_f32(j.ssq_new + (size_t)(nt0 + t) * 16 + row, s);
    }
    if (j.t_done && tid == 0) atomicMax(j.t_done, (unsigned long long)wall_clock64());   // (emulated collectives only)
    if (CHAIN) gemv_signal_done(j, lb);
    if (j.pos_inc && lb == 0 && tid == 0) *j.pos_inc += 1;
    return true;
  }

  // EPI_QKV_ROPE: TN*8 adjacent pairs in this workgroup's columns, all inside one head
  if (tid < 16 * TN * 8) {
    const int row = tid / (TN * 8), pr = tid % (TN * 8);
    if (row < j.M) {
      const int col = grp * (TN * 16) + 2 * pr;
      const int c16 = (2 * pr) & 15, t = (2 * pr) >> 4;
      float e = out_of(t, c16, row), o = out_of(t, c16 + 1, row);
      const int pos = pre_pos;
      const int head = col / j.d, jj = (col % j.d) >> 1;
      if (head < j.nq + j.nkv) {
        const float c = pre_cos, sn = pre_sin;
        const float re = e * c - o * sn, ro = e * sn + o * c;
        e = re;
        o = ro;
      }
      if (head < j.nq) {
        uint32_t eh, el, oh, ol;
        split_bf16(e, eh, el);
        split_bf16(o, oh, ol);
        const size_t at = (size_t)row * j.nq * j.d + col;
        store_u32(reinterpret_cast<uint32_t*>(j.q_out + at), eh | (oh << 16));
        store_u32(reinterpret_cast<uint32_t*>(j.q_out + (size_t)FUSED_LOW_ROW * j.nq * j.d + at), el | (ol << 16));
      } else if (head < j.nq + j.nkv) {
        const int kvh = head - j.nq;
        store_u32(reinterpret_cast<uint32_t*>(j.cache_k + (((size_t)row * j.nkv + kvh) * j.max_seq + pos) * j.d + 2 * jj),
                  pack_bf16(e, o));
      } else {
        const int kvh = head - j.nq - j.nkv;
        bf16_t* vt = j.cache_v + (((size_t)row * j.nkv + kvh) * j.d + 2 * jj) * j.max_seq + pos;
        store_b16(vt, f32_to_bf16(e));
        store_b16(vt + j.max_seq, f32_to_bf16(o));
      }
    }
  }
  if (CHAIN) gemv_signal_done(j, lb);
  return true;
}

// ------------------------------------------------------------------------------------------------
// decode attention job (MFMA, computed transposed as in the prefill kernel):
//   S^T[key][head] = K Q^T        A = K tile (16 keys x 32 dims, straight from the K cache rows),
//                                 B = Q^T (the G heads of this kv head as columns, rest zero);
//   O^T[dim][head] = V^T P^T      A = V^T tile (16 dims x 32 keys, from the transposed V cache),
//                                 B = the lane's own 8 probabilities of the 32-key block.
// Q and P are split operands: operand column h < 8 carries the high part of head h's row, column 8 + h its
// low part (at most 8 q heads share a kv head), so the two halves of S^T and of O^T are added across lanes
// b and b ^ 8; the cache rows (K, V) are bf16 as stored.
// The 8 wavefronts take the 32-key blocks of the split round robin, each with its own running
// softmax and no barrier in the loop; they merge once, through LDS, at the end.
// ------------------------------------------------------------------------------------------------
// The workgroup has stored the final attention output of its (sequence, kv head) with coherent stores: wait for
// them and count it, for the projection job of the same launch that consumes it.
// (The counter is the word the consumers poll.  That is affordable for these few increments only: an atomic
// on a cache line that hundreds of workgroups poll takes microseconds, and the workgroup keeps its CU slot
// until the atomic has completed.  A producer job of many workgroups must count on one line and have the
// workgroup that completes the count set a flag on another line, which the consumers poll.)
__device__ __forceinline__ void attn_signal_done(const AttnJob& a, int ordinal) {
  if (!a.done) return;
  __builtin_amdgcn_s_waitcnt(0);   // this thread's coherent stores of the output have completed
  __syncthreads();
  if (threadIdx.x == 0) sync_count(a.done, (unsigned)ordinal, (unsigned)(a.B * a.nkv), a.done_flagged != 0);
}

// Returns false if the job's wait gave up (nothing stored, error word raised).
template <int D, int G>
__device__ __forceinline__ bool attn_job(const AttnJob& a, int lb, float* smem, unsigned* s_flag, unsigned long long* t_ready) {
  constexpr int DS = D / 32, DT = D / 16;
  const int tid0 = opaque_tid();
  const int wave = __builtin_amdgcn_readfirstlane(tid0 >> 6);
  if (a.wait_on) {
    // chained step: q and the new cache rows come from the QKV projection of the same launch (see gemv_job)
    if (wave == 0) {
      const bool arrived = sync_wait(a.wait_on, a.wait_flags, nullptr, 0u, a.wait_bias, a.wait_spins, tid0 & 63);
      if (tid0 == 0) {
        *s_flag = arrived ? 1u : 0u;
        if (!arrived && a.err_word) __hip_atomic_store(a.err_word, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
      }
    }
    __syncthreads();
    if (*s_flag == 0u) return false;
    __syncthreads();   // (s_flag is written again below)
  }
  if (t_ready && tid0 == 0) *t_ready = wall_clock64();
  const int b = tid0 & 15, q = (tid0 & 63) >> 4;   // (valid up to the end of the key loop: see below)
  const int sp = lb % a.n_splits, kvh = (lb / a.n_splits) % a.nkv, bi = lb / (a.n_splits * a.nkv);
  const int pbeg = sp * a.split_len;
  const float scale = 1.0f / sqrtf((float)D);

  const bf16_t* kc = a.cache_k + ((size_t)bi * a.nkv + kvh) * a.max_seq * D;
  const bf16_t* vc = a.cache_v + ((size_t)bi * a.nkv + kvh) * D * a.max_seq;
  uint4 kreg[2][DS], vreg[DT];
  auto load_kv = [&](int kb) {   // keys kb .. kb + 31 (inside the cache's capacity)
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int s = 0; s < DS; ++s)
        kreg[t][s] = *reinterpret_cast<const uint4*>(kc + (size_t)(kb + 16 * t + b) * D + s * 32 + q * 8);
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) {
      const bf16_t* vp = vc + (size_t)(dt * 16 + b) * a.max_seq + kb + 4 * q;
      const uint2 lo = *reinterpret_cast<const uint2*>(vp);
      const uint2 hi = *reinterpret_cast<const uint2*>(vp + 16);
      vreg[dt] = make_uint4(lo.x, lo.y, hi.x, hi.y);
    }
  };
  // The wave's first key block and the queries are requested before the position is known (one memory round
  // trip instead of two; a block beyond the new token is masked or never used).
  const int kb0 = pbeg + 32 * wave;
  const bool early = kb0 + 32 <= a.max_seq;
  if (early) load_kv(kb0);
  const uint4 zero4 = make_uint4(0, 0, 0, 0);
  static_assert(G <= 8, "high and low parts of the heads of a kv head share one 16-column operand");
  const int hsel = b & 7;             // head of this lane's operand column
  const bool low = (b & 8) != 0;      // its column carries the low parts
  uint4 qreg[DS];
  {
    const bf16_t* qg = a.q + ((size_t)((low ? FUSED_LOW_ROW : 0) + bi) * a.nq + kvh * G + min(hsel, G - 1)) * D;
#pragma unroll
    for (int s = 0; s < DS; ++s) {
      const uint4 v = *reinterpret_cast<const uint4*>(qg + s * 32 + q * 8);
      qreg[s] = hsel < G ? v : zero4;
    }
  }
  const int n_pos = *a.pos_dev + 1;
  if (pbeg >= n_pos) return true;  // nothing visible in this split: the workgroup leaves, no ticket taken
  const int pend = min(n_pos, pbeg + a.split_len);
  f32x4_t oacc[DT];
#pragma unroll
  for (int dt = 0; dt < DT; ++dt) oacc[dt] = (f32x4_t){0.f, 0.f, 0.f, 0.f};
  float mrun = -INFINITY, lrun = 0.f;

  auto process = [&](int kb) {   // keys kb .. kb + 31, already in kreg / vreg
    f32x4_t st[2];
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      st[t] = (f32x4_t){0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int s = 0; s < DS; ++s)
        st[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, kreg[t][s]),
                                                       __builtin_bit_cast(bf16x8_t, qreg[s]), st[t], 0, 0, 0);
    }
    float sv[8], mloc = -INFINITY;
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int key = kb + 16 * t + 4 * q + r;
        const float sc = st[t][r] + other_half(st[t][r]);             // q = high + low part: both halves now hold the score
        const float v = key < pend ? sc * scale : -INFINITY;          // positions past the new token: masked
        sv[t * 4 + r] = v;
        mloc = fmaxf(mloc, v);
      }
    mloc = fmaxf(mloc, __shfl_xor(mloc, 16, 64));
    mloc = fmaxf(mloc, __shfl_xor(mloc, 32, 64));
    const float mnew = fmaxf(mrun, mloc);      // finite: key kb itself is < pend
    const float corr = __expf(mrun - mnew);
    float pv[8], psum = 0.f;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      pv[e] = __expf(sv[e] - mnew);
      psum += pv[e];
    }
    lrun = lrun * corr + psum;
    mrun = mnew;
    uint32_t pe[8];   // this column's part of the probabilities: high parts in columns 0..7, low parts in 8..15
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      uint32_t h, l;
      split_bf16(pv[e], h, l);
      pe[e] = low ? l : h;
    }
    uint4 pb;
    pb.x = pe[0] | (pe[1] << 16); pb.y = pe[2] | (pe[3] << 16);
    pb.z = pe[4] | (pe[5] << 16); pb.w = pe[6] | (pe[7] << 16);
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) {
#pragma unroll
      for (int r = 0; r < 4; ++r) oacc[dt][r] *= corr;
      oacc[dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, vreg[dt]),
                                                        __builtin_bit_cast(bf16x8_t, pb), oacc[dt], 0, 0, 0);
    }
  };
  if (kb0 < pend) {
    if (!early) load_kv(kb0);
    process(kb0);
  }
  for (int kb = kb0 + 32 * FUSED_WAVES; kb < pend; kb += 32 * FUSED_WAVES) {
    load_kv(kb);
    process(kb);
  }
  // per-wave (max, sum, O^T) -> LDS; oacc[dt][r] = O^T[dim = dt*16 + 4q + r][head b]
  lrun += __shfl_xor(lrun, 16, 64);
  lrun += __shfl_xor(lrun, 32, 64);
  // (the lane's coordinates are taken afresh from the hardware here, so that the ones above need not stay in
  // registers across the key loop, where every register is wanted for rows in flight)
  unsigned zero_m = 0u;
  asm volatile("" : "+v"(zero_m));   // (so that this is computed here and not kept from the top of an enclosing loop)
  const int lane_m = (int)__builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, zero_m));
  const int tid_m = wave * 64 + lane_m;
  float* wm = smem;                          // [WAVES][16]
  float* wl = wm + FUSED_WAVES * 16;         // [WAVES][16]
  float* wo = wl + FUSED_WAVES * 16;         // [WAVES][G][D]
  const int b2 = lane_m & 15, q2 = lane_m >> 4;
  if (q2 == 0) { wm[wave * 16 + b2] = mrun; wl[wave * 16 + b2] = lrun; }
#pragma unroll
  for (int dt = 0; dt < DT; ++dt)
#pragma unroll
    for (int r = 0; r < 4; ++r) oacc[dt][r] += other_half(oacc[dt][r]);   // P = high + low part
  if (b2 < G) {
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
      for (int r = 0; r < 4; ++r) wo[(wave * G + b2) * D + dt * 16 + 4 * q2 + r] = oacc[dt][r];
  }
  __syncthreads();
  const size_t pbase = ((size_t)bi * a.nkv + kvh) * a.n_splits;
  // the output is the output projection's operand: a split operand matrix of B rows, column = head * D + dim
  const int So = fused_slots(a.B);
  const int ocol0 = kvh * G * D;
  for (int i = tid_m; i < G * D; i += FUSED_THREADS) {
    const int h = i / D, dim = i % D;
    float m = -INFINITY;
#pragma unroll
    for (int w = 0; w < FUSED_WAVES; ++w) m = fmaxf(m, wm[w * 16 + h]);
    float l = 0.f, o = 0.f;
#pragma unroll
    for (int w = 0; w < FUSED_WAVES; ++w) {
      const float f = __expf(wm[w * 16 + h] - m);   // 0 for a wave that saw no block
      l += wl[w * 16 + h] * f;
      o += wo[(w * G + h) * D + dim] * f;
    }
    if (a.n_splits == 1) {
      {
        bf16_t* const at = a.o + fused_xop_offset(So, bi, ocol0 + i);
        st_coherent_split_pair(at, at + (So / 2) * 8, i, o / l);
      }
    } else {
      st_coherent(a.part_o + ((pbase + sp) * G + h) * D + dim, o);
      if (dim == 0) {
        st_coherent(a.part_ml + ((pbase + sp) * G + h) * 2 + 0, m);
        st_coherent(a.part_ml + ((pbase + sp) * G + h) * 2 + 1, l);
      }
    }
  }
  if (a.n_splits == 1) {
    attn_signal_done(a, bi * a.nkv + kvh);
    return true;
  }

  // several splits: the last one to arrive merges them (fixed order)
  const int n_active = min(a.n_splits, (n_pos + a.split_len - 1) / a.split_len);
  __builtin_amdgcn_s_waitcnt(0);   // this thread's coherent stores of the partial result have completed
  __syncthreads();
  if (tid_m == 0) {
    const unsigned t = atomicAdd(a.tickets + bi * a.nkv + kvh, 1u);
    *s_flag = t;
    if (t == (unsigned)n_active - 1) st_coherent(a.tickets + bi * a.nkv + kvh, 0u);  // ready for the next attention job
  }
  __syncthreads();
  if (*s_flag != (unsigned)n_active - 1) return true;
  // The last arrival reads the other splits' partial results with coherent loads.  Every thread merges its
  // own output elements from all splits, sixteen splits per pass with all of the pass's loads issued
  // together (one memory round trip per pass), in split order.
  constexpr int SP = 16;
  for (int i = tid_m; i < G * D; i += FUSED_THREADS) {
    const int h = i / D;
    float m = -INFINITY, l = 0.f, o = 0.f;
    for (int s0 = 0; s0 < n_active; s0 += SP) {
      float ms[SP], ls[SP], os[SP];
#pragma unroll
      for (int k = 0; k < SP; ++k) {
        ms[k] = -INFINITY; ls[k] = 0.f; os[k] = 0.f;
        if (s0 + k < n_active) {   // (uniform: no request for a split that is not there)
          const int s = s0 + k;
          ms[k] = ld_coherent(a.part_ml + ((pbase + s) * G + h) * 2 + 0);
          ls[k] = ld_coherent(a.part_ml + ((pbase + s) * G + h) * 2 + 1);
          os[k] = ld_coherent(a.part_o + (pbase + s) * G * D + i);
        }
      }
      float mnew = m;
#pragma unroll
      for (int k = 0; k < SP; ++k) mnew = fmaxf(mnew, s0 + k < n_active ? ms[k] : -INFINITY);
      const float f0 = __expf(m - mnew);   // 0 on the first pass (m = -inf, mnew finite: split 0 saw a key)
      l *= f0;
      o *= f0;
#pragma unroll
      for (int k = 0; k < SP; ++k) {
        const float f = s0 + k < n_active ? __expf(ms[k] - mnew) : 0.f;
        l += ls[k] * f;
        o += os[k] * f;
      }
      m = mnew;
    }
    {
        bf16_t* const at = a.o + fused_xop_offset(So, bi, ocol0 + i);
        st_coherent_split_pair(at, at + (So / 2) * 8, i, o / l);
      }
  }
  attn_signal_done(a, bi * a.nkv + kvh);
  return true;
}


// The leading arguments repeat what a workgroup needs first: two (weights, operand) pointer pairs that cover the
// GEMV jobs of a launch (jobs that are parts of one projection share theirs), the block boundaries of the jobs
// and the row count, one descriptor byte per job (FUSED_KIND_* below), and K / 32 and the first tile group of the
// first three GEMV jobs.  With kernel-argument preloading (the build passes -mllvm
// -amdgpu-kernarg-preload-count=10; 14 dwords) they are in SGPRs when a wave starts: a workgroup knows its job
// and requests its first weight tiles and operand slices at once, while the job's descriptor is still on its
// way from memory (a cold scalar load costs 0.7 - 2 us here, and it used to stand in front of every
// workgroup's first request).
// The kernel's parameter list as a struct: kernel arguments are laid out in the argument segment like the members
// of a C struct, so offsetof() of the last member is where the by-value FusedArgs block starts.  Keep it in step
// with the parameter list of fused_decode_kernel.
struct FusedKernelParams {
  const void* wp_a;
  const void* wp_b;
  const bf16_t* x_a;
  const bf16_t* x_b;
  unsigned ends01, end2_m, kinds, geo0, geo1, geo2;
  FusedArgs fa;
};
static_assert(FUSED_MAX_JOBS == 4, "the preloaded arguments carry three block boundaries and four descriptor bytes");
template <int D, int G>
__global__ __launch_bounds__(FUSED_THREADS, 4) void fused_decode_kernel(const void* wp_a, const void* wp_b, const bf16_t* x_a,
                                                                       const bf16_t* x_b, unsigned ends01, unsigned end2_m,
                                                                       unsigned kinds, unsigned geo0, unsigned geo1,
                                                                       unsigned geo2, FusedArgs fa) {
  extern __shared__ float smem[];   // fa.lds_bytes: the largest need of the launch's jobs
  __shared__ unsigned s_flag;
  const int end0 = (int)(ends01 & 0xFFFFu), end1 = (int)(ends01 >> 16), end2 = (int)(end2_m & 0xFFFFu);
  int lb = blockIdx.x, job = 0;
  if ((int)blockIdx.x >= end0) { lb = blockIdx.x - end0; job = 1; }
  if ((int)blockIdx.x >= end1) { lb = blockIdx.x - end1; job = 2; }
  if ((int)blockIdx.x >= end2) { lb = blockIdx.x - end2; job = 3; }
  const unsigned kb = (kinds >> (8 * job)) & 0xFFu;
  // The jobs' descriptors are read in place from the kernel-argument segment (uniform index -> scalar loads).
  // Touching the by-value argument itself makes the compiler, beyond some amount of code that uses it, keep a
  // copy of all of it in private memory (a kilobyte of scratch stores at the head of every wavefront).  The
  // block's offset in the segment is that of the last member of FusedKernelParams.
  typedef __attribute__((address_space(4))) const char* kernarg_ptr_t;
  const kernarg_ptr_t ka = (kernarg_ptr_t)__builtin_amdgcn_kernarg_segment_ptr();
  if ((kb & FUSED_KIND_MASK) == (unsigned)JOB_ATTN) {
    const AttnJob& aj = *(const AttnJob*)(ka + offsetof(FusedKernelParams, fa) + offsetof(FusedArgs, a));
    (void)attn_job<D, G>(aj, lb, smem, &s_flag, nullptr);
  } else {
    const GemvJob& j = *(const GemvJob*)(ka + offsetof(FusedKernelParams, fa) + offsetof(FusedArgs, g) + (size_t)job * sizeof(GemvJob));
    const unsigned slot = kb >> FUSED_KIND_SLOT_SHIFT;   // which preloaded pointer pair: 0, 1, or 3 = none
    const int gi = job - ((kinds & FUSED_KIND_MASK) == (unsigned)JOB_ATTN ? 1 : 0);   // index among the GEMV jobs
    const void* wp = slot == 0 ? wp_a : wp_b;
    const bf16_t* xop = slot == 0 ? x_a : x_b;
    const unsigned geo = gi == 0 ? geo0 : gi == 1 ? geo1 : geo2;
    int KT = (int)(geo >> 16), group0 = (int)(geo & 0xFFFFu), M = (int)(end2_m >> 16);
    if (slot == 3) { wp = j.wp; xop = j.xb; KT = j.K >> 5; group0 = j.group0; M = j.M; }
    const unsigned tn = ((kb >> FUSED_KIND_TN_SHIFT) & 3u) + 1u;
    // more than 8 rows: high and low operand parts are two MFMA operands (else they share one)
    // (the one wait of these launches is for the attention output, read with coherent loads; every other operand
    // was complete before the launch: requested at once)
#define FUSED_GEMV(U_, TN_, COH_)                                                                                  \
  do {                                                                                                             \
    if (M > 8) (void)gemv_job<U_, TN_, COH_, true, false>(j, wp, xop, KT, group0, M, lb, smem, &s_flag, nullptr, nullptr);  \
    else (void)gemv_job<U_, TN_, COH_, false, false>(j, wp, xop, KT, group0, M, lb, smem, &s_flag, nullptr, nullptr);       \
  } while (0)
    if (kb & FUSED_KIND_WAITS) {
      if (tn == 4) FUSED_GEMV(1, 4, true);
      else if (tn == 2) FUSED_GEMV(FUSED_U2, 2, true);
      else FUSED_GEMV(FUSED_U, 1, true);
    } else if (tn == 4) {
      FUSED_GEMV(1, 4, false);
    } else if (tn == 3) {
      FUSED_GEMV(1, 3, false);
    } else if (tn == 2) {
      FUSED_GEMV(FUSED_U2, 2, false);
    } else {
      FUSED_GEMV(FUSED_U, 1, false);
    }
#undef FUSED_GEMV
  }
}

// ------------------------------------------------------------------------------------------------
// Chained step: the whole launch list of a decode step in ONE launch of persistent workgroups.
// Workgroup w (a "slot"; the launch has as many as are resident together) runs the blocks w, w + n_slots, ... of
// every launch of the list, in the list's order.  Where the list relies on one launch ending before the next
// begins, a job now waits for the flags of the jobs that produce what it reads (gemv_job, attn_job): a
// workgroup requests its first weight tiles, then sleeps on the flag.  What this saves is the end of every launch
// (the chip draining while the last workgroups finish, the caches written back), its start (descriptor loads,
// the first memory round trip with nothing in flight) and the gap between the two; and the two chains that the
// ladder wiring leaves independent (attention side, MLP side) drift against each other instead of meeting at
// every launch boundary.
// Every wait is for a block that comes earlier in (launch, block) order, and every slot runs its blocks in that
// order: the earliest unfinished block of the step never waits for anything unfinished, so the step always ends
// (the waits are bounded all the same; a workgroup whose wait gives up leaves the kernel).
// A slot's item list is read in chunks of 32 items into LDS; an item carries what the first requests need.
// ------------------------------------------------------------------------------------------------
#define FUSED_CHAIN_CHUNK 32
#define FUSED_KIND_COH 32u
static_assert(sizeof(StepItem) == 32, "the kernel reads an item as two 16-byte words");
template <int D, int G>
__global__ __launch_bounds__(FUSED_THREADS, 4) void fused_chain_kernel(const StepItem* __restrict__ items, int n_items,
                                                                      const GemvJob* __restrict__ gemv_jobs,
                                                                      const AttnJob* __restrict__ attn_jobs, float* x_out,
                                                                      unsigned long long* timeline) {
  extern __shared__ float smem[];
  __shared__ unsigned s_flag;
  __shared__ unsigned s_claim, s_claim_n;
  __shared__ uint4 s_items[2 * FUSED_CHAIN_CHUNK];
  __shared__ uint4 s_surplus[2 * FUSED_CLAIM_MAX];
  // the job tables are read-only for the launch: scalar loads (constant address space), as for kernel arguments
  typedef __attribute__((address_space(4))) const char* const_ptr_t;
  typedef __attribute__((address_space(1))) const char* global_ptr_t;
  const const_ptr_t gj = (const_ptr_t)(unsigned long long)gemv_jobs;
  const const_ptr_t aj = (const_ptr_t)(unsigned long long)attn_jobs;
  const uint4* mine = reinterpret_cast<const uint4*>(items + (size_t)blockIdx.x * n_items);
  // (whether the slot is inside a surplus list is kept in LDS, not in a register that would stay live across the
  // jobs' code: the kernel is at its register limit)
  if (threadIdx.x == 0) s_claim_n = 0u;
  for (int it = 0; it < n_items; ++it) {
    const int ic = it % FUSED_CHAIN_CHUNK;
    if (ic == 0) {
      if ((int)threadIdx.x < 2 * FUSED_CHAIN_CHUNK && 2 * it + (int)threadIdx.x < 2 * n_items)
        s_items[threadIdx.x] = mine[2 * it + threadIdx.x];
      __syncthreads();
    }
    uint4 i0 = s_items[2 * ic], i1 = s_items[2 * ic + 1];
    unsigned kb = (unsigned)__builtin_amdgcn_readfirstlane((int)i1.z) & 0xFFu;
    if (kb == 0u) break;
    bool taken_block = false;
    if ((kb & FUSED_KIND_MASK) == (unsigned)JOB_CLAIM) {
      // a surplus list: the slot stays on this item, taking one block per visit, until the list is used up
      const unsigned n = min((unsigned)__builtin_amdgcn_readfirstlane((int)i1.w), (unsigned)FUSED_CLAIM_MAX);
      if (__builtin_amdgcn_readfirstlane((int)s_claim_n) == 0) {   // first visit: the list into LDS
        const unsigned long long lp = (unsigned long long)(unsigned)__builtin_amdgcn_readfirstlane((int)i0.x) |
                                      ((unsigned long long)(unsigned)__builtin_amdgcn_readfirstlane((int)i0.y) << 32);
        const uint4* list = (const uint4*)(global_ptr_t)lp;
        for (unsigned k = threadIdx.x; k < 2u * n; k += FUSED_THREADS) s_surplus[k] = list[k];
      }
      if (threadIdx.x == 0) {
        const unsigned long long cp = (unsigned long long)i0.z | ((unsigned long long)i0.w << 32);
        s_claim = __hip_atomic_fetch_add((unsigned*)cp, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      }
      __syncthreads();     // (every thread has read s_claim_n; the list and the number taken are in LDS)
      const unsigned taken = (unsigned)__builtin_amdgcn_readfirstlane((int)s_claim);
      if (threadIdx.x == 0) s_claim_n = taken < n ? n : 0u;   // (read next at the next visit of a list, behind a block's barriers)
      if (taken >= n) {
        __syncthreads();   // (every thread has read s_claim: the next list's first visit may follow at once)
        continue;
      }
      i0 = s_surplus[2 * taken];
      i1 = s_surplus[2 * taken + 1];
      kb = (unsigned)__builtin_amdgcn_readfirstlane((int)i1.z) & 0xFFu;
      taken_block = true;
      --it;   // the same item again after this block (s_claim and s_surplus are next written behind its __syncthreads)
    }
    // timeline (measurement; null in normal operation): when the slot took the item, when its waits were over, when it
    // ended (blocks taken from a surplus list are not recorded)
    unsigned long long* const tl = (timeline && !taken_block) ? timeline + ((size_t)blockIdx.x * n_items + it) * 3 : nullptr;
    const unsigned geo = (unsigned)__builtin_amdgcn_readfirstlane((int)i1.x);
    const unsigned lbj = (unsigned)__builtin_amdgcn_readfirstlane((int)i1.y);
    const int lb = (int)(lbj & 0xFFFFu), job = (int)(lbj >> 16);
    if (tl && threadIdx.x == 0) tl[0] = wall_clock64();
    bool ok;
    if ((kb & FUSED_KIND_MASK) == (unsigned)JOB_ATTN) {
      ok = attn_job<D, G>(*(const AttnJob*)(aj + (size_t)job * sizeof(AttnJob)), lb, smem, &s_flag, tl ? tl + 1 : nullptr);
    } else {
      const GemvJob& j = *(const GemvJob*)(gj + (size_t)job * sizeof(GemvJob));
      const unsigned long long wpu = (unsigned long long)(unsigned)__builtin_amdgcn_readfirstlane((int)i0.x) |
                                     ((unsigned long long)(unsigned)__builtin_amdgcn_readfirstlane((int)i0.y) << 32);
      const unsigned long long xpu = (unsigned long long)(unsigned)__builtin_amdgcn_readfirstlane((int)i0.z) |
                                     ((unsigned long long)(unsigned)__builtin_amdgcn_readfirstlane((int)i0.w) << 32);
      // (pointers into global memory, and said to be: through a pointer of unknown address space every load is a
      // flat load, which counts as an LDS and scalar-memory operation too, so that each wait for a descriptor field
      // would wait for all weight tiles in flight)
      const void* wp = (const void*)(global_ptr_t)wpu;
      const bf16_t* xop = (const bf16_t*)(global_ptr_t)xpu;
      const int KT = (int)(geo & 0xFFFFu), group0 = (int)(geo >> 16);
      const int M = (int)(((unsigned)__builtin_amdgcn_readfirstlane((int)i1.z) >> 8) & 0xFFu);
      const unsigned tn = ((kb >> FUSED_KIND_TN_SHIFT) & 3u) + 1u;
#define CHAIN_GEMV(U_, TN_, COH_)                                                                                   \
  do {                                                                                                              \
    if (M > 8) ok = gemv_job<U_, TN_, COH_, true, true>(j, wp, xop, KT, group0, M, lb, smem, &s_flag, x_out, tl ? tl + 1 : nullptr);   \
    else ok = gemv_job<U_, TN_, COH_, false, true>(j, wp, xop, KT, group0, M, lb, smem, &s_flag, x_out, tl ? tl + 1 : nullptr);        \
  } while (0)
      if (kb & FUSED_KIND_COH) {
        if (tn == 4) CHAIN_GEMV(1, 4, true);
        else if (tn == 2) CHAIN_GEMV(FUSED_U2, 2, true);
        else CHAIN_GEMV(FUSED_U, 1, true);
      } else if (tn == 4) {
        CHAIN_GEMV(1, 4, false);
      } else if (tn == 3) {
        CHAIN_GEMV(1, 3, false);
      } else if (tn == 2) {
        CHAIN_GEMV(FUSED_U2, 2, false);
      } else {
        CHAIN_GEMV(FUSED_U, 1, false);
      }
#undef CHAIN_GEMV
    }
    if (!ok) break;      // (the same for the whole workgroup)
    __syncthreads();     // the job's LDS is free again; the item chunk may be overwritten
    if (tl && threadIdx.x == 0) tl[2] = wall_clock64();
  }
}

// x_0 = embeddings: fp32 for the residual chain, split operands (times the readers' gains) for the projections,
// sums of squares per 16-column tile and row (a tile = 16 adjacent threads: H is a multiple of 16)
// (also clears the step's arrival counters: a fill kernel, not a memset node, so that a captured step replays)
__global__ __launch_bounds__(256) void embed_kernel(EmbedArgs a) {
  const int i = blockIdx.x * 256 + threadIdx.x, n = a.rows * a.H;
  const bool ok = i < n;
  const int ic = min(i, n - 1);
  const int row = ic / a.H, col = ic % a.H;
  float v, vp;   // x_0, and what module 1 reads (x_{-1}: the same rows unless a pipeline stage hands over)
  if (a.res) {
    vp = a.res[ic] + (a.att ? a.att[ic] : 0.f);
    v = vp + (a.mlp ? a.mlp[ic] : 0.f);
  } else {
    v = vp = bf16_to_f32(a.emb[ic]);
  }
  if (ok) {
    a.x0[ic] = v;
    const int S = fused_slots(a.rows);
    const size_t at = fused_xop_offset(S, row, col);
    if (a.xop_a) {
      uint32_t hi, lo;
      split_bf16(vp * bf16_to_f32(a.gain_a[col]), hi, lo);
      a.xop_a[at] = (bf16_t)hi;
      a.xop_a[at + (S / 2) * 8] = (bf16_t)lo;
    }
    if (a.xop_b) {
      uint32_t hi, lo;
      split_bf16(v * bf16_to_f32(a.gain_b[col]), hi, lo);
      a.xop_b[at] = (bf16_t)hi;
      a.xop_b[at + (S / 2) * 8] = (bf16_t)lo;
    }
  }
  float s = ok ? v * v : 0.f;
  s += __shfl_xor(s, 1, 64);
  s += __shfl_xor(s, 2, 64);
  s += __shfl_xor(s, 4, 64);
  s += __shfl_xor(s, 8, 64);
  if (ok && (col & 15) == 0) a.ssq[(size_t)(col >> 4) * 16 + row] = s;
  if (a.ssq_a) {
    float sp = ok ? vp * vp : 0.f;
    sp += __shfl_xor(sp, 1, 64);
    sp += __shfl_xor(sp, 2, 64);
    sp += __shfl_xor(sp, 4, 64);
    sp += __shfl_xor(sp, 8, 64);
    if (ok && (col & 15) == 0) a.ssq_a[(size_t)(col >> 4) * 16 + row] = sp;
  }
  if (i < a.n_zero) a.zero_words[i] = 0u;
}

hipError_t launch_embed(const EmbedArgs& a, hipStream_t s, hipEvent_t ev0, hipEvent_t ev1) {
  if (a.rows <= 0 || a.rows > 16 || a.H <= 0 || (a.H & 15) || (!a.emb == !a.res) || !a.x0 || !a.ssq) return hipErrorInvalidValue;
  if (!a.res && (a.att || a.mlp)) return hipErrorInvalidValue;
  if ((a.xop_a && !a.gain_a) || (a.xop_b && !a.gain_b)) return hipErrorInvalidValue;
  const dim3 grid((std::max(a.rows * a.H, a.n_zero) + 255) / 256), block(256);
  if (ev0 || ev1) hipExtLaunchKernelGGL(embed_kernel, grid, block, 0, s, ev0, ev1, 0, a);
  else hipLaunchKernelGGL(embed_kernel, grid, block, 0, s, a);
  return hipGetLastError();
}

// what the kernels take for granted about a GEMV job
static bool gemv_job_valid(const GemvJob& j) {
  const int tn = j.tn >= 2 ? j.tn : 1;
  if (j.ldx != j.K) return false;   // (the x rows are taken to be K elements apart)
  // tiles per workgroup the kernels have code for: 1, 2 and 4 for every job, 3 for jobs with ordinary operand loads
  if (tn > 4) return false;
  if (j.M < 1 || j.M > 16 || (j.K & 31) || (j.N & 15) || j.K <= 0) return false;
  if (j.normed && !j.ssq) return false;
  if (j.wait_on && j.wait_spins <= 0) return false;
  if (j.wait_on2 && !j.wait_on) return false;
  if (j.done_ctr && j.done_target == 0) return false;
  if (j.epi == EPI_RESIDUAL && ((j.xop_a && !j.gain_a) || (j.xop_b && !j.gain_b) || !j.x_old || !j.x_new)) return false;
  if (j.epi == EPI_SWIGLU && (!j.act || ((j.N / 2) & 1))) return false;
  return j.epi == EPI_RESIDUAL || j.epi == EPI_SWIGLU || j.epi == EPI_QKV_ROPE;
}

hipError_t fused_chain_item(const GemvJob& j, int job_index, int lb, StepItem* out) {
  if (!gemv_job_valid(j) || !out) return hipErrorInvalidValue;
  const int tn = j.tn >= 2 ? j.tn : 1, kt = j.K >> 5;
  if (kt > 0xFFFF || j.group0 < 0 || j.group0 > 0xFFFF || lb < 0 || lb > 0xFFFF || job_index < 0 || job_index > 0xFFFF)
    return hipErrorInvalidValue;
  const bool coh = j.coherent_x != 0;
  if (tn == 3 && coh) return hipErrorInvalidValue;
  StepItem it{};
  it.wp = j.wp; it.xb = j.xb; it.kt = (uint16_t)kt; it.group0 = (uint16_t)j.group0; it.lb = (uint16_t)lb; it.job = (uint16_t)job_index;
  it.kind = (uint8_t)((unsigned)JOB_GEMV | ((unsigned)(tn - 1) << FUSED_KIND_TN_SHIFT) | (coh ? FUSED_KIND_COH : 0u));
  it.M = (uint8_t)j.M;
  *out = it;
  return hipSuccess;
}

hipError_t fused_chain_claim_item(const StepItem* surplus_dev, unsigned* counter_dev, int n, StepItem* out) {
  if (!surplus_dev || !counter_dev || !out || n < 1 || n > FUSED_CLAIM_MAX) return hipErrorInvalidValue;
  StepItem it{};
  it.wp = surplus_dev; it.xb = reinterpret_cast<const bf16_t*>(counter_dev); it.kind = (uint8_t)JOB_CLAIM; it.pad1 = (uint32_t)n;
  *out = it;
  return hipSuccess;
}

hipError_t fused_chain_attn_item(const AttnJob& a, int job_index, int lb, StepItem* out) {
  if (!out || lb < 0 || lb > 0xFFFF || job_index < 0 || job_index > 0xFFFF) return hipErrorInvalidValue;
  if (a.wait_on && a.wait_spins <= 0) return hipErrorInvalidValue;
  if (a.B < 1 || a.B > 16 || a.n_splits < 1 || (a.split_len & 63)) return hipErrorInvalidValue;
  StepItem it{};
  it.lb = (uint16_t)lb; it.job = (uint16_t)job_index; it.kind = (uint8_t)JOB_ATTN; it.M = (uint8_t)a.B;
  *out = it;
  return hipSuccess;
}

template <int D>
static hipError_t launch_fused_d(const FusedArgs& fa, int g, dim3 grid, hipStream_t s, hipEvent_t ev0, hipEvent_t ev1) {
  const dim3 block(FUSED_THREADS);
  // with events: the dispatch itself carries them, so their distance is the kernel's own run time
  // preloaded arguments: a GEMV job is "hot" when it is among the first three, its numbers fit 16 bits and its
  // (weights, operand) pair is one of the two the launch can carry
  unsigned kinds = 0, geo[3] = {0u, 0u, 0u};
  const void* wp[2] = {nullptr, nullptr};
  const bf16_t* xp[2] = {nullptr, nullptr};
  int n_pairs = 0, n_gemv = 0, rows = -1;
  if (fa.block_end[0] > 0xFFFF || fa.block_end[1] > 0xFFFF || fa.block_end[2] > 0xFFFF) return hipErrorInvalidValue;
  for (int i = 0; i < FUSED_MAX_JOBS; ++i) {
    unsigned kb = (unsigned)fa.kind[i] & FUSED_KIND_MASK;
    if (i < fa.n_jobs && fa.kind[i] == JOB_ATTN && i != 0) return hipErrorInvalidValue;   // (the kernel counts on it)
    if (i < fa.n_jobs && fa.kind[i] == JOB_GEMV) {
      const GemvJob& j = fa.g[i];
      if (!gemv_job_valid(j) || j.wait_on2 || j.done_ctr) return hipErrorInvalidValue;   // (the last two: chained steps only)
      const int kt = j.K >> 5, gi = n_gemv++;
      unsigned slot = 3;
      if (gi < 3 && kt <= 0xFFFF && j.group0 >= 0 && j.group0 <= 0xFFFF && j.M >= 1 && j.M <= 0xFFFF &&
          (rows < 0 || rows == j.M)) {
        int p = 0;
        while (p < n_pairs && !(wp[p] == j.wp && xp[p] == j.xb)) ++p;
        if (p == n_pairs && n_pairs < 2) { wp[p] = j.wp; xp[p] = j.xb; ++n_pairs; }
        if (p < n_pairs) {
          slot = (unsigned)p;
          geo[gi] = ((unsigned)kt << 16) | (unsigned)j.group0;
          rows = j.M;
        }
      }
      // tiles per workgroup the kernel has code for: 1, 2 and 4 for every job, 3 for jobs without a wait
      const int tn = j.tn >= 2 ? j.tn : 1;
      if (tn == 3 && j.wait_on) return hipErrorInvalidValue;
      kb |= (unsigned)(tn - 1) << FUSED_KIND_TN_SHIFT;
      if (j.wait_on) kb |= FUSED_KIND_WAITS;
      kb |= slot << FUSED_KIND_SLOT_SHIFT;
    }
    kinds |= kb << (8 * i);
  }
  const unsigned ends01 = (unsigned)fa.block_end[0] | ((unsigned)fa.block_end[1] << 16);
  const unsigned end2_m = (unsigned)fa.block_end[2] | ((unsigned)(rows < 0 ? 0 : rows) << 16);
#define FUSED_LAUNCH(GQ)                                                                                    \
  do {                                                                                                      \
    if (ev0 || ev1)                                                                                          \
      hipExtLaunchKernelGGL((fused_decode_kernel<D, GQ>), grid, block, fa.lds_bytes, s, ev0, ev1, 0,         \
                            wp[0], wp[1], xp[0], xp[1], ends01, end2_m, kinds, geo[0], geo[1], geo[2], fa);  \
    else                                                                                                    \
      hipLaunchKernelGGL((fused_decode_kernel<D, GQ>), grid, block, fa.lds_bytes, s,                         \
                         wp[0], wp[1], xp[0], xp[1], ends01, end2_m, kinds, geo[0], geo[1], geo[2], fa);     \
  } while (0)
  switch (g) {
    case 1: FUSED_LAUNCH(1); break;
    case 2: FUSED_LAUNCH(2); break;
    case 4: FUSED_LAUNCH(4); break;
    case 8: FUSED_LAUNCH(8); break;
    default: return hipErrorInvalidValue;
  }
#undef FUSED_LAUNCH
  return hipGetLastError();
}

// LDS a job needs: the attention job's merge area or the GEMV job's cross-wave sums
size_t fused_attn_lds_bytes(int d, int g) { return (size_t)(2 * FUSED_WAVES * 16 + FUSED_WAVES * g * d + g * 64) * 4; }
size_t fused_gemv_lds_bytes() {
  return (size_t)(FUSED_WAVES * 4 * 16 * 17 + FUSED_WAVES * 16) * 4;   // sized for four-tile workgroups
}

// dynamic LDS above 64 KiB has to be allowed per kernel, once (outside any stream capture)
template <int D>
static hipError_t prepare_d(int g) {
  const int bytes = FUSED_MAX_LDS_BYTES;
  switch (g) {
    case 1: return hipFuncSetAttribute((const void*)fused_decode_kernel<D, 1>, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    case 2: return hipFuncSetAttribute((const void*)fused_decode_kernel<D, 2>, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    case 4: return hipFuncSetAttribute((const void*)fused_decode_kernel<D, 4>, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    case 8: return hipFuncSetAttribute((const void*)fused_decode_kernel<D, 8>, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
  }
  return hipErrorInvalidValue;
}
hipError_t fused_decode_prepare(int d, int g) {
  if (d == 128) return prepare_d<128>(g);
  if (d == 64) return prepare_d<64>(g);
  return hipErrorInvalidValue;
}

template <int D, int GQ>
static hipError_t launch_chain_dg(const StepItem* items, int n_items, const GemvJob* gj, const AttnJob* aj, float* x_out,
                                  unsigned long long* tl, int n_slots, int lds_bytes, hipStream_t s, hipEvent_t ev0, hipEvent_t ev1) {
  const dim3 grid(n_slots), block(FUSED_THREADS);
  if (ev0 || ev1) hipExtLaunchKernelGGL((fused_chain_kernel<D, GQ>), grid, block, lds_bytes, s, ev0, ev1, 0, items, n_items, gj, aj, x_out, tl);
  else hipLaunchKernelGGL((fused_chain_kernel<D, GQ>), grid, block, lds_bytes, s, items, n_items, gj, aj, x_out, tl);
  return hipGetLastError();
}
template <int D>
static const void* chain_kernel_of(int g) {
  switch (g) {
    case 1: return (const void*)fused_chain_kernel<D, 1>;
    case 2: return (const void*)fused_chain_kernel<D, 2>;
    case 4: return (const void*)fused_chain_kernel<D, 4>;
    case 8: return (const void*)fused_chain_kernel<D, 8>;
  }
  return nullptr;
}

int fused_chain_slots(int d, int g, int n_cu) {
  const void* k = d == 128 ? chain_kernel_of<128>(g) : d == 64 ? chain_kernel_of<64>(g) : nullptr;
  if (!k || n_cu <= 0) return 0;
  if (hipFuncSetAttribute(k, hipFuncAttributeMaxDynamicSharedMemorySize, FUSED_MAX_LDS_BYTES) != hipSuccess) return 0;
  int per_cu = 0;
  if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, k, FUSED_THREADS, FUSED_MAX_LDS_BYTES) != hipSuccess) return 0;
  return std::min(per_cu, 2) * n_cu;   // (the launch lists are laid out for two workgroups per CU)
}

hipError_t launch_fused_chain(const StepItem* items, int n_items, const GemvJob* gemv_jobs, const AttnJob* attn_jobs,
                              float* x_out, unsigned long long* timeline, int n_slots, int lds_bytes, int d, int g,
                              hipStream_t s, hipEvent_t ev0, hipEvent_t ev1) {
  if (!items || n_items <= 0 || n_slots <= 0 || lds_bytes <= 0 || lds_bytes > FUSED_MAX_LDS_BYTES) return hipErrorInvalidValue;
#define CHAIN_LAUNCH(D_)                                                                                                    \
  switch (g) {                                                                                                              \
    case 1: return launch_chain_dg<D_, 1>(items, n_items, gemv_jobs, attn_jobs, x_out, timeline, n_slots, lds_bytes, s, ev0, ev1);    \
    case 2: return launch_chain_dg<D_, 2>(items, n_items, gemv_jobs, attn_jobs, x_out, timeline, n_slots, lds_bytes, s, ev0, ev1);    \
    case 4: return launch_chain_dg<D_, 4>(items, n_items, gemv_jobs, attn_jobs, x_out, timeline, n_slots, lds_bytes, s, ev0, ev1);    \
    case 8: return launch_chain_dg<D_, 8>(items, n_items, gemv_jobs, attn_jobs, x_out, timeline, n_slots, lds_bytes, s, ev0, ev1);    \
  }
  if (d == 128) { CHAIN_LAUNCH(128) }
  if (d == 64) { CHAIN_LAUNCH(64) }
#undef CHAIN_LAUNCH
  return hipErrorInvalidValue;
}

hipError_t launch_fused_decode(const FusedArgs& fa, int d, int g, hipStream_t s, hipEvent_t ev0, hipEvent_t ev1) {
  if (fa.lds_bytes <= 0 || fa.lds_bytes > FUSED_MAX_LDS_BYTES) return hipErrorInvalidValue;
  const int total = fa.block_end[fa.n_jobs - 1];
  if (total <= 0) return hipErrorInvalidValue;
  if (d == 128) return launch_fused_d<128>(fa, g, dim3(total), s, ev0, ev1);
  if (d == 64) return launch_fused_d<64>(fa, g, dim3(total), s, ev0, ev1);
  return hipErrorInvalidValue;
}
