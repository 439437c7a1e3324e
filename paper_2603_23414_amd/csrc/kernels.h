// Launchers and device-state layout shared by the engine and the kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

// ---- attention --------------------------------------------------------------------------------------
struct AttnArgs {
  const void* pool;        // this layer's KV pool
  const void* q;           // bf16 [n_rows][Hq][d]
  const int* row_slot;     // page-table row of each query row
  const int* row_pos;      // position of the query token (context = pos + 1)
  const int* page_table;   // int32 [slots][max_pages]
  int max_pages;
  const int4* work;        // (row, group, page-table row, context length) items: all a workgroup needs to start; full
                           // groups first, then the shorter last groups of the rows in descending length, so that the
                           // launch ends on its smallest items
  const int2* row_wstart;  // work items of each row: .x = first of its full groups (consecutive), .y = its last, shorter group
  int n_work, n_rows, Hkv;
  float* part_acc;         // [n_work][Hq][d]
  float* part_ml;          // [n_work][Hq][2]
  int* row_cnt;            // [n_rows][Hkv] arrival counters of rows that span several work items: zero before the
                           // first launch, left at zero by every launch
  void* out;               // [n_rows][Hq*d], bf16 or fp32
  int out_fp32;
  int chunk_tokens;        // cached tokens per work item (multiple of 64, at most 1024)
};
int attn_supported(int head_dim, int group);
void launch_decode_attn(const AttnArgs& a, int head_dim, int group, hipStream_t st, hipEvent_t ev0 = nullptr,
                        hipEvent_t ev1 = nullptr);
void launch_write_kv(void* pool, int Hkv, int head_dim, const void* k, const void* v, const int* tok_seq,
                     const int* tok_pos, const int* page_table, int max_pages, size_t n_tok, hipStream_t st);

// causal paged attention for prefill rows: one tile = up to 32 consecutive query tokens of one sequence
struct PfTileHost { int row0, n, slot, pos0; };
void launch_prefill_attn(const void* pool, const void* q, const void* tiles, int n_tiles, const int* page_table,
                         int max_pages, int Hq, int Hkv, int head_dim, void* out, hipStream_t st);

// ---- GEMM ---------------------------------------------------------------------------------------------
int gemm_pick_splits(int M, int N, int K);
// name of the kernel instantiation launch_gemm (epi 0) / launch_gemm_swiglu (epi 1) runs for this shape and split count
const char* gemm_kernel_name(int M, int N, int K, int S, int epi);
void launch_gemm(const void* A, const void* W, float* C, int M, int N, int K, int S, hipStream_t st);
void launch_gemm_swiglu(const void* A, const void* W, void* act, int M, int N, int K, hipStream_t st);
// The LM head with the emit statistics taken in its epilogue, so that no logits row is ever written: per row the
// candidate token (arg-max with the lowest index on ties, or the Gumbel-max draw when sampling), its scaled logit, the
// scaled logit of the EOS column and the log-sum-exp of the scaled logits.  Each workgroup (128 columns) leaves one
// partial record per row; lm_reduce combines a row's records in ascending column order (deterministic).
struct LmEpi {
  float scale;                       // logits multiplier: 1 / temperature when sampling, else 1
  int sampling;
  unsigned long long seed;           // key of the counter-based generator
  int eos_id;
  int n_tiles;                       // column tiles = workgroups along the vocabulary
  const int* row_slot;               // sampling only: row -> slot -> sequence -> (seq_id, tokens generated so far)
  const int* slot_seq;
  const unsigned long long* seq_id;
  const int* seq_gen_len;
  float4* part_f;                    // [rows][n_tiles]: best perturbed score, its scaled logit, max scaled logit, sum exp
  int* part_i;                       // [rows][n_tiles]: column of the best score
  float* row_zeos;                   // [rows]: scaled logit of the EOS column
};
void launch_gemm_lm_fused(const void* A, const void* W, int M, int N, int K, const LmEpi& epi, hipStream_t st);
void launch_lm_reduce(const LmEpi& epi, int M, int* row_argmax, float* row_ztok, float* row_lse, hipStream_t st);

// row-major [N, K] -> the packed fragment layout the GEMM kernels read (N * K elements; N a multiple of 32)
void launch_pack_weights(const void* src, void* dst, size_t N, size_t K, hipStream_t st);
void launch_reduce_splits(const float* part, float* c, size_t mn, int S, hipStream_t st);

struct SchedDev;
// ---- fused small kernels ------------------------------------------------------------------------------
void launch_embed(const void* table, const int* row_tok, float* h, int R, int D, hipStream_t st);
void launch_add_rmsnorm(float* h, const float* part, int S, size_t part_stride, const float* gain, float eps, void* x,
                        int R, int D, hipStream_t st);
void launch_rope_kvwrite(const float* part, int S, size_t part_stride, const float* bias, const int* row_slot,
                         const int* row_pos, const void* cs_table, void* q_out, void* pool, const int* page_table,
                         int max_pages, int Hq, int Hkv, int d, int R, hipStream_t st);
// greedy (inv_temp == 0) or Gumbel-max sampling; row_lse is the log-sum-exp of logits * inv_temp (of logits if greedy)
void launch_argmax_lse(const float* logits, int V, int* row_argmax, float* row_lse, float* row_ztok, float* row_zeos, int R,
                       const SchedDev* sched, hipStream_t st);
void launch_gather_rows(const float* src, const int* src_row, float* dst, int dst_row0, int n, int D, hipStream_t st);

// ---- scheduler state (device side of the rollout state manager / stateful buffer, Sec. 3.3) ----------
enum { SEQ_QUEUED = 0, SEQ_ACTIVE = 1, SEQ_FINISHED = 2, SEQ_HARVESTED = 3 };
enum {  // scalar cells in SchedDev::sc
  SC_STEP = 0, SC_VERSION, SC_NFREE, SC_QHEAD, SC_QCOUNT, SC_FINCOUNT, SC_NDEC, SC_NPRE, SC_NWORK, SC_MINFREE,
  SC_ADMIT_RAN, SC_QNE, SC_COUNT
};
enum {  // 64-bit counters in SchedDev::ctr
  CT_BUSY = 0, CT_IDLE, CT_STEPS_Q, CT_IDLE_Q, CT_GEN, CT_DISCARD, CT_PREFILL, CT_PREEMPT, CT_STALE, CT_COUNT
};
enum {  // int cells of the status block copied to the host after every scheduler kernel
  STAT_STEP = 0, STAT_R, STAT_NACTIVE, STAT_FIN, STAT_QUEUED, STAT_FREE, STAT_NADM, STAT_NFIN_STEP, STAT_NPRE_STEP,
  STAT_NDEC_NEXT, STAT_NWORK_NEXT, STAT_CTX_LO, STAT_CTX_HI, STAT_VERSION, STAT_CHUNK, STAT_HDR = 16
};  // followed by max_slots admission descriptors of STAT_ADM_INTS ints: slot, sequence-table index, end position
#define STAT_ADM_INTS 4   // ... and the first position to prefill (> 0 when the rollout attached to shared prompt pages)

struct SchedDev {
  int Q, max_pages, n_pages, max_seqs, qmask, tok_stride, cap, eos_id, eos_mode, mode, max_staleness, no_model, V, Hkv;
  float inv_temp;          // 1 / temperature, 0 = greedy
  unsigned long long sample_seed;
  int* sc;
  unsigned long long* ctr;
  int *slot_seq, *slot_npages, *page_table;
  int *seq_prompt_len, *seq_target_len, *seq_gen_len, *seq_state, *seq_slot, *seq_completion, *seq_kv_version,
      *seq_npreempt;
  int* seq_fin_version;    // policy version under which the rollout's last token was produced (set when it finishes)
  unsigned long long* seq_id;
  int* seq_tokens;
  float* seq_logp;
  // prompt groups: the rollouts of one prompt share the pages the prompt fills completely (Sec. 4.1: several
  // responses per prompt); grp_ref counts the running rollouts that read them
  int *seq_group;          // group-table index or -1
  int *grp_nshared, *grp_ref, *grp_version, *grp_pages;   // grp_pages: [max_seqs][max_shared]
  int max_shared;
  int *q_ring, *free_stack, *fin_list;
  int *row_slot, *row_pos, *row_tok;
  int2* row_wstart;
  int4* work;
  const int* row_argmax;
  const float* row_lse;
  const float* row_ztok;   // scaled logit of the candidate token of each row
  const float* row_zeos;   // scaled logit of the EOS column of each row
  const float* logits;     // fp32 logits rows: only the teacher-forced path has them
  const int* forced_tok;   // nullable
  int* status;
};

struct SubmitRec { int sidx, prompt_len, target_len, tok_off; unsigned long long seq_id; int group, nshared; };

void launch_sched_admit(const SchedDev& d, hipStream_t st);
void launch_sched_emit(const SchedDev& d, hipStream_t st);
void launch_sched_boundary(const SchedDev& d, int n_groups, hipStream_t st);
void launch_sched_submit(const SchedDev& d, const SubmitRec* recs, const int* tok_staging, int n, hipStream_t st);
void launch_sched_init(const SchedDev& d, hipStream_t st);

// harvest: one finished rollout whose gen_len tokens (and log-probs) go to offset `off` of the staging buffers
struct HarvestRec { int sidx, prompt_len, gen_len, off; };
void launch_harvest_gather(const SchedDev& d, const HarvestRec* recs, int n, int* tok_out, float* logp_out,
                           hipStream_t st);

// prefill planning: token rows of the admitted sequences
struct PrefillDesc { int slot, sidx, n_tok, pos_begin, row_begin; };   // a run of consecutive positions of one sequence
void launch_prefill_rows(const SchedDev& d, const PrefillDesc* descs, int n_desc, int* row_slot, int* row_pos,
                         int* row_tok, hipStream_t st);

// weight repacking at init: dst[dst_row(r)][c] = convert(src[r][c]), dst_row(r) = row0 + (r / blk) * blk_stride + r % blk
void launch_repack(const void* src, int src_fp32, void* dst, int dst_fp32, size_t rows, size_t cols, size_t row0,
                   size_t blk, size_t blk_stride, hipStream_t st);

// plain streaming kernels (counter calibration, measured HBM ceiling)
void launch_stream_copy(const void* src, void* dst, size_t bytes, hipStream_t st);
void launch_stream_read(const void* src, size_t bytes, void* sink, hipStream_t st);
