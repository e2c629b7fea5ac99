// Argument blocks of the fused decode launches (see decode_fused.hip).
#pragma once

#include "common.h"

enum { JOB_NONE = 0, JOB_GEMV = 1, JOB_ATTN = 2, JOB_CLAIM = 3 };   // (JOB_CLAIM: chained steps only, see StepItem)
enum { EPI_SWIGLU = 1, EPI_RESIDUAL = 2, EPI_QKV_ROPE = 3 };

// Operands of the matrix core on this path are SPLIT: a value v travels as two bf16 numbers, high = bf16(v) and
// low = bf16(v - high), so that high + low carries 16 significant bits and the products with the (bf16) weights
// lose nothing that an fp32 operand would keep.  Up to 8 rows, high and low parts share ONE 16-column MFMA
// operand (the columns that a small batch leaves empty) and the two halves of the result are added afterwards;
// from 9 rows on they are two operands and two MFMAs into the same accumulator.  Decode is bound by the
// weight stream: the matrix core has the time.
//
// Layout of a split operand matrix of M rows (M = the batch of the step) and K columns, in the order the matrix
// core reads it: the K range is cut into k tiles of 32; a k tile holds S row slots, S = fused_slots(M) = 2, 4, 8,
// 16 or 32 (twice the batch rounded up to a power of two; 32 from 9 rows on): slots 0 .. S/2-1 the high parts of rows 0 .., slots S/2 .. S-1 their low parts; a slot's 32 values
// are stored as four groups of 8 (16 bytes: one lane's share of the MFMA operand), group-major:
//     element (row r, part p, column k)  at  (k / 32) * S * 32 + (((k % 32) / 8) * S + r + p * S/2) * 8 + k % 8
// A wavefront's load of a k tile is then S * 64 contiguous bytes (512 bytes for a batch of 4, 128 for a single
// sequence) instead of 16 bytes from each of 2 M rows that lie K elements apart.  Every such matrix is allocated for S = 32 (K * 64 bytes).
// The queries of the attention job are the exception: a split matrix in plain rows, bf16 [32][nq * d], rows
// 0..15 the high parts, rows 16..31 (FUSED_LOW_ROW) the low parts.
#define FUSED_LOW_ROW 16
#if defined(__HIPCC__)
#define FUSED_HD __host__ __device__
#else
#define FUSED_HD
#endif
static inline FUSED_HD int fused_slots(int M) { return M <= 1 ? 2 : (M <= 2 ? 4 : (M <= 4 ? 8 : (M <= 8 ? 16 : 32))); }
// element offset of (row, column) of the HIGH part in a split operand matrix with S slots; the low part sits
// (S / 2) * 8 elements further
static inline FUSED_HD size_t fused_xop_offset(int S, int row, int col) {
  return (size_t)(col >> 5) * (size_t)(S * 32) + (size_t)(((((col & 31) >> 3) * S) + row) << 3) + (size_t)(col & 7);
}

// One skinny GEMM  out[m][n] = sum_k x[m][k] W[k][n], M <= 16, on packed weight tiles; a workgroup
// owns tn adjacent 16-column tiles and the whole K range.
struct GemvJob {
  // x operand: a split bf16 matrix of M rows and K columns (see above).  normed != 0: it is the residual stream times the gain of
  // this module's RMSNorm (both applied in fp32 by the job that wrote the stream, before the split), and this
  // projection scales its output rows by 1/rms (the factor commutes with the product), the rows' sums of squares
  // coming from ssq: f32 [K/16][16], one value per 16-column tile of the stream and row, summed in a fixed order
  const bf16_t* xb;
  int ldx;
  int normed;
  float eps;
  const float* ssq;
  int reads_stream;        // host-side note: normed jobs read the stream x_m with this m (the kernel does not use it)
  int completes_stream;    // host-side note: a residual job after which the stream x_m is complete (a collective ends there): that m; else 0
  int after_attention;     // host-side note: the output projection of an attention module (its operand is the attention job's output)
  const void* wp;
  int M, K, N;
  // wait_on != null: the job's x operand is produced by the attention job of the SAME launch; the
  // workgroup starts by waiting (bounded: wait_spins polls) for the flag of that job's completion words (wait_on,
  // FUSED_SYNC_WORDS words), then reads that operand with device-coherent loads.  If the wait gives up, the
  // workgroup stores nothing and raises *err_word (host-visible memory), which the next call of the library reports.
  const unsigned* wait_on;
  unsigned wait_flags;     // 0: that producer counts itself and raises one flag; else: it has this many workgroups, each
                           // with a flag word of its own (see sync_count in decode_fused.hip)
  unsigned wait_bias;
  int wait_spins;
  unsigned* err_word;
  // Chained step (one launch for the whole decode step): every job waits for the jobs that produce what it reads.
  // wait_on (above) then is the flag (or, for the attention job's output, the arrival counter) of the producer
  // of the x operand, wait_on2 that of the producer of x_old where that is another job; operands whose producer
  // is a projection are read with ordinary loads after the wait (each such buffer is written once per launch and
  // read by nobody before, so no cache of the chip holds an older copy of it).
  // done_ctr != null: this job is a producer.  Its workgroups write their results with device-coherent stores,
  // wait for them and count themselves at done_ctr (FUSED_SYNC_WORDS words); done_target = the workgroups of the
  // whole projection (its jobs share done_ctr), done_ord0 = the ordinal of this job's first workgroup among them.
  // wait_on / wait_on2 point at such words of a producer (the job polls their flag); wait_bias is added to the
  // value the flag must reach (0; a test makes the wait fail with it).
  const unsigned* wait_on2;
  unsigned wait_flags2;
  int coherent_x;          // chained step: the x operand is read with device-coherent loads (a buffer that is written more than once per launch)
  unsigned* done_ctr;
  unsigned done_target;
  unsigned done_ord0;
  int done_flagged;        // the producer's workgroups raise a flag word each instead of counting themselves
  // Emulated collective latency (both null / 0 in normal operation).  t_ready: the job reads a stream whose
  // collective ends delay_ticks (wall clock) after the time stored there by an earlier launch; its workgroups
  // hold back until then (bounded).  t_done: every workgroup of this (residual) job leaves the time it ended there
  // (atomic maximum), which is when the collective of the stream it completes starts.
  const unsigned long long* t_ready;
  unsigned long long delay_ticks;
  unsigned long long* t_done;
  int tn;                  // 16-column tiles per workgroup: 1 (0 means 1), 2, 4, or 3 (jobs without a wait)
  int group0, n_groups;    // this job's workgroups own the tile groups [group0, group0 + n_groups), tn tiles
                           // each; a projection may be cut over two launches
  int epi;
  // EPI_SWIGLU: act = split operand matrix of M rows and N/2 columns
  bf16_t* act;
  // EPI_RESIDUAL: x_new = x_old + out + sum_p peers[p]   (the residual update of Algorithm 1 with the
  // all-reduce written as a sum over rank partial sums, Eq. 2); for each of the (at most two) modules that read
  // x_new: its operand xop = split(x_new * gain of that module's RMSNorm) (M rows, N columns), gain in the storage type [N];
  // and the sums of squares of x_new per 16-column tile and row, ssq_new f32 [N/16][16]
  const float* x_old;
  float* x_new;
  bf16_t* xop_a;
  const bf16_t* gain_a;
  bf16_t* xop_b;
  const bf16_t* gain_b;
  float* ssq_new;
  const bf16_t* peers;
  int n_peers;
  size_t peer_stride;
  float* x_copy;           // EPI_RESIDUAL, optional: a second f32 copy of the new rows (the caller's x_out for the last module)
  int* pos_inc;            // EPI_RESIDUAL, optional (last launch of a step, which holds no reader of the position): the
                           // job's first workgroup advances the position by one at its end
  // EPI_QKV_ROPE: rotary on q and k (adjacent pairs), q -> q_out (split bf16 [32][nq*d]), k and v rounded to the
  // cache's storage type and appended at *pos_dev
  bf16_t* q_out;
  bf16_t* cache_k;
  bf16_t* cache_v;
  const float* cos_tab;
  const float* sin_tab;
  const int* pos_dev;
  int nq, nkv, d, max_seq;
};

// Decode attention over the cache.  One workgroup per (split, kv head, sequence) walks its share of
// the positions in blocks of 32 with a running softmax; with one split the result is final, with several
// the last split to arrive (ticket) merges them.  Queries, probabilities and the output are split operands:
// the nq/nkv <= 8 heads of a kv head sit in operand columns 0..7 (high parts) and 8..15 (low parts).
struct AttnJob {
  const bf16_t* q;         // split [32][nq*d] rotated
  const bf16_t* cache_k;   // [B_cap][nkv][max_seq][d]
  const bf16_t* cache_v;   // [B_cap][nkv][d][max_seq]
  float* part_o;           // [B][nkv][n_splits][g][d]   (n_splits > 1 only)
  float* part_ml;          // [B][nkv][n_splits][g][2]
  bf16_t* o;               // split operand matrix of B rows and nq*d columns (the output projection's operand)
  unsigned* tickets;       // [B][nkv]
  int B, nq, nkv, max_seq;
  int n_splits, split_len; // split s covers positions [s*split_len, (s+1)*split_len); split_len % 64 == 0
  const int* pos_dev;      // position of the new token; positions 0..*pos_dev are visible
  unsigned* done;          // if non-null: completion words (FUSED_SYNC_WORDS) at which the workgroup that has written the
                           // final output of its (sequence, kv head) counts itself, once its device-coherent stores
                           // have completed; a projection job of the same launch waits on them
  // chained step: the job starts by waiting (bounded) for the flag of the completion words at wait_on: those of the
  // QKV projection that writes q and appends to the cache
  const unsigned* wait_on;
  unsigned wait_flags;     // as in GemvJob
  unsigned wait_bias;
  int wait_spins;
  unsigned* err_word;
  int done_flagged;        // the workgroups that write final outputs raise a flag word each at `done` (else: count themselves)
};

// completion words of one producer (a projection, the attention job of a layer): 10 cache lines of 32 words
// (sub-counters 0..7 on lines 0..7; eight flag words, which consumers poll, at the start of line 9); zero at the
// start of every step
#define FUSED_SYNC_WORDS 320
#define FUSED_SYNC_FLAG_WORD 288

#define FUSED_MAX_LDS_BYTES (48 * 1024)   // (the largest job needs 36.6 KiB; two workgroups per CU must fit with the chained kernel's static 13 KiB)
#define FUSED_MAX_JOBS 4

struct FusedArgs {
  int n_jobs;              // 1 .. FUSED_MAX_JOBS
  int lds_bytes;           // dynamic LDS of the launch = the largest need of its jobs
  int kind[FUSED_MAX_JOBS];       // JOB_GEMV | JOB_ATTN (at most one attention job, described by `a`)
  int block_end[FUSED_MAX_JOBS];  // cumulative workgroup counts: job i = [block_end[i-1], block_end[i])
  GemvJob g[FUSED_MAX_JOBS];
  AttnJob a;
};

hipError_t launch_fused_decode(const FusedArgs& fa, int d, int g, hipStream_t s, hipEvent_t ev0, hipEvent_t ev1);

// Chained step: ONE launch of persistent workgroups runs the whole list of launches of a step.  Workgroup w of the
// launch (a "slot") runs the blocks w, w + n_slots, ... of every launch of the list in turn; a job starts when the
// jobs it reads from have raised their flags.  An item is what a workgroup needs to request its first weight tiles
// before the job's descriptor has arrived from memory.
struct StepItem {
  const void* wp;          // GEMV job: the job's weights
  const bf16_t* xb;        //           and operand
  uint16_t kt;             // K / 32
  uint16_t group0;
  uint16_t lb;             // block index within the job
  uint16_t job;            // index into the GEMV or the attention job table
  uint8_t kind;            // descriptor byte: JOB_* | (tiles per workgroup - 1) << 2 | coherent operand loads << 5; 0 ends the list
  uint8_t M;
  uint16_t pad0;
  uint32_t pad1;
};
// Where a launch of the list has more blocks than there are slots, the blocks beyond the slots (at most
// FUSED_CLAIM_MAX of them) are not dealt out beforehand: they form the launch's surplus list, and a slot that has
// finished its own block of that launch takes blocks from it, one at a time (an atomic counter, zero at the start of
// the step), before it goes on to the next launch -- as a hardware dispatcher hands the next workgroup to the first
// free CU.  A JOB_CLAIM item in a slot's list says where: wp = the surplus list (StepItem[pad1], device), xb = its
// counter word, pad1 = its length.  The (launch, block) order that the waits rely on still holds: a block waits for
// earlier blocks only, and the earliest unfinished block is either on a slot that has reached it or in a surplus list
// that every slot passes after its own block of that launch.
#define FUSED_CLAIM_MAX 384
hipError_t fused_chain_claim_item(const StepItem* surplus_dev, unsigned* counter_dev, int n, StepItem* out);
// the item of block lb of a job; hipErrorInvalidValue if the job is outside what the kernel has code for
hipError_t fused_chain_item(const GemvJob& j, int job_index, int lb, StepItem* out);
hipError_t fused_chain_attn_item(const AttnJob& a, int job_index, int lb, StepItem* out);
// persistent workgroups that are resident together on a device of n_cu compute units (0: the kernel does not fit)
int fused_chain_slots(int d, int g, int n_cu);
// items: [n_slots][n_items] (device), each slot's list ended by an item of kind 0 (n_items includes it)
// timeline (null in normal operation): u64 [n_slots][n_items][3], the wall-clock times at which a slot took an item,
// had waited for its inputs, and had finished it
hipError_t launch_fused_chain(const StepItem* items, int n_items, const GemvJob* gemv_jobs, const AttnJob* attn_jobs,
                              float* x_out, unsigned long long* timeline, int n_slots, int lds_bytes, int d, int g,
                              hipStream_t s, hipEvent_t ev0, hipEvent_t ev1);
hipError_t fused_decode_prepare(int d, int g);   // once per context, before the first launch
size_t fused_attn_lds_bytes(int d, int g);
size_t fused_gemv_lds_bytes();
// x_0 = the embeddings (emb: bf16 [rows][H]): fp32 rows for the residual chain, the split operand matrices (rows
// rows, H columns) of the (at most two) modules that read x_0 (each times that module's gain), the sums of
// squares per tile and row; also clears
// n_zero words at zero_words (the step's arrival counters).
// A pipeline stage that is not the first starts from three fp32 tensors instead (res non-null, emb null; att and
// mlp may be null = zeros): x_{-1} = res + att is what operand a is made of, with its sums of squares in ssq_a,
// x_0 = x_{-1} + mlp is the stream, operand b and ssq.  With emb both are the embeddings (ssq_a, if given, = ssq).
struct EmbedArgs {
  const bf16_t* emb;
  const float* res;
  const float* att;
  const float* mlp;
  float* ssq_a;            // [H/16][16] or null
  float* x0;
  bf16_t* xop_a;
  const bf16_t* gain_a;
  bf16_t* xop_b;
  const bf16_t* gain_b;
  float* ssq;              // [H/16][16]
  int rows, H;
  unsigned* zero_words;
  int n_zero;
};
hipError_t launch_embed(const EmbedArgs& a, hipStream_t s, hipEvent_t ev0, hipEvent_t ev1);
