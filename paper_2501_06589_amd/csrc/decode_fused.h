// Argument blocks of the fused decode launches (see decode_fused.hip).
#pragma once

#include "common.h"

enum { JOB_NONE = 0, JOB_GEMV = 1, JOB_ATTN = 2 };
enum { EPI_SWIGLU = 1, EPI_RESIDUAL = 2, EPI_QKV_ROPE = 3 };

// One skinny GEMM  out[m][n] = sum_k x[m][k] W[k][n], M <= 16, on packed weight tiles; a workgroup
// owns 32 columns and the whole K range.
struct GemvJob {
  // x operand: a bf16 matrix.  normed != 0: it is the bf16 copy of the residual stream and this
  // projection applies RMSNorm: the gain is already folded into the weight rows, and the rows' 1/rms,
  // computed from the same operand loads, scales the output (the factor commutes with the product)
  const bf16_t* xb;
  int ldx;
  int normed;
  float eps;
  const void* wp;
  int M, K, N;
  // wait_on != null: the job's x operand is produced by the attention job of the SAME launch; the
  // workgroup starts by waiting (bounded) until *wait_on has reached wait_target, then reads that operand
  // with device-coherent loads
  const unsigned* wait_on;
  unsigned wait_target;
  int tn;                  // 16-column tiles per workgroup: 1 (0 means 1), 2, 3 (un-normed jobs without a wait)
                           // or 4 (normed jobs without a wait, un-normed jobs with one)
  int group0, n_groups;    // this job's workgroups own the tile groups [group0, group0 + n_groups), tn tiles
                           // each; a projection may be cut over two launches
  int epi;
  // EPI_SWIGLU: act[m][N/2] bf16
  bf16_t* act;
  // EPI_RESIDUAL: x_new = x_old + out + sum_p peers[p]   ("wait(); residual += out" with the
  // all-reduce written as a sum over rank partial sums)
  const float* x_old;
  float* x_new;
  bf16_t* xh_new;          // bf16 copy of x_new
  const bf16_t* peers;
  int n_peers;
  size_t peer_stride;
  // EPI_QKV_ROPE: rotary on q and k (adjacent pairs), q -> q_out, k and v appended at *pos_dev
  bf16_t* q_out;
  bf16_t* cache_k;
  bf16_t* cache_v;
  const float* cos_tab;
  const float* sin_tab;
  const int* pos_dev;
  int nq, nkv, d, max_seq;
};

// Decode attention over the cache.  One workgroup per (split, kv head, sequence) walks its share of
// the positions in passes of 64 with a running softmax; with one split (the usual case) the result
// is final, with several the last split to arrive (ticket) merges them.
struct AttnJob {
  const bf16_t* q;         // [B][nq*d] rotated
  const bf16_t* cache_k;   // [B_cap][nkv][max_seq][d]
  const bf16_t* cache_v;   // [B_cap][nkv][d][max_seq]
  float* part_o;           // [B][nkv][n_splits][g][d]   (n_splits > 1 only)
  float* part_ml;          // [B][nkv][n_splits][g][2]
  bf16_t* o;               // [B][nq*d]
  unsigned* tickets;       // [B][nkv]
  int B, nq, nkv, max_seq;
  int n_splits, split_len; // split s covers positions [s*split_len, (s+1)*split_len); split_len % 64 == 0
  const int* pos_dev;      // position of the new token; positions 0..*pos_dev are visible
  unsigned* done;          // if non-null: incremented by the workgroup that has written the final output of its
                           // (sequence, kv head), once its device-coherent stores have completed; a projection
                           // job of the same launch waits on it
};

#define FUSED_MAX_LDS_BYTES (72 * 1024)
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
hipError_t fused_decode_prepare(int d, int g);   // once per context, before the first launch
size_t fused_attn_lds_bytes(int d, int g);
size_t fused_gemv_lds_bytes();
hipError_t launch_embed(const bf16_t* emb, float* x0, bf16_t* xh0, int n, unsigned* zero_words, int n_zero,
                        hipStream_t s, hipEvent_t ev0, hipEvent_t ev1);
