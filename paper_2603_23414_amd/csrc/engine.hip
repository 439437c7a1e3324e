// Host engine and C ABI of librollout: owns the weights, the paged KV pool, the device-resident scheduler
// state, and sequences the per-step kernel chain.  The host never computes any part of the method; it
// launches kernels, reads back the small status block the scheduler kernels publish, and copies
// trajectories out at harvest.
#include <algorithm>
#include <chrono>
#include <cmath>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <string>
#include <unordered_map>
#include <vector>

#include "../../include/rollout.h"
#include "common.h"
#include "kernels.h"

#define PF_ROWS 4096          // token rows per prefill pass

// Scratch of rollout_gemm_bf16_static (split-K partial sums for callers that cannot allocate).  The name is a host-side
// stand-in: host code only ever uses the per-device address static_scratch() looks up.
#define GEMM_STATIC_SCRATCH_BYTES (32ull << 20)
static __device__ __align__(256) unsigned char scratch[GEMM_STATIC_SCRATCH_BYTES];

namespace {

struct LayerW {
  float* attn_norm = nullptr;
  uint16_t* wqkv = nullptr;
  float* bqkv = nullptr;
  uint16_t* wo = nullptr;
  float* ffn_norm = nullptr;
  uint16_t* wgu = nullptr;
  uint16_t* wdown = nullptr;
};

struct SeqHost {
  uint64_t seq_id = 0;
  int prompt_len = 0;
  bool in_use = false;
  bool harvested = false;
  int group = -1;       // prompt-group table index (several responses of one prompt), -1 = none
};

}  // namespace

struct rollout_ctx {
  rollout_cfg cfg;
  std::string err;
  bool dead = false;
  hipStream_t stream = nullptr;
  int NL, D, Hq, Hkv, d, F, V, G, Nqkv, Q;
  // weights
  uint16_t* embed = nullptr;
  uint16_t* lm_head = nullptr;
  float* final_norm = nullptr;
  std::vector<LayerW> layers;
  // KV
  uint8_t* kv_pool = nullptr;
  size_t layer_pool_bytes = 0;
  int n_pages = 0, max_pages = 0;
  float2* cs_table = nullptr;
  // scheduler
  SchedDev sd;
  int* status_host = nullptr;  // pinned
  int status_ints = 0;
  int* forced_tok_dev = nullptr;
  // activations
  int rows_cap = 0;
  float* h = nullptr;
  uint16_t* x = nullptr;
  float* part = nullptr;
  uint16_t* qbuf = nullptr;
  uint16_t* attn_out = nullptr;
  uint16_t* act = nullptr;
  float* h_final = nullptr;
  uint16_t* x_final = nullptr;
  float* logits = nullptr;
  int* row_argmax = nullptr;
  float* row_lse = nullptr;
  float* row_ztok = nullptr;
  float* row_zeos = nullptr;
  float4* lm_part_f = nullptr;   // per-(row, column tile) records of the fused LM head
  int* lm_part_i = nullptr;
  int lm_tiles = 0;
  int* iota = nullptr;
  // prefill rows + attention workspace
  int *pf_row_slot = nullptr, *pf_row_pos = nullptr, *pf_row_tok = nullptr;
  PfTileHost* pf_tiles_dev = nullptr;
  PfTileHost* pf_tiles_host = nullptr;  // pinned
  PrefillDesc* pf_desc_dev = nullptr;
  PrefillDesc* pf_desc_host = nullptr;  // pinned
  int* pf_last_host = nullptr;          // pinned
  float* part_acc = nullptr;
  float* part_ml = nullptr;
  int* attn_row_cnt = nullptr;
  size_t max_work = 0;
  // submit staging (pinned + device)
  SubmitRec* sub_host = nullptr;
  SubmitRec* sub_dev = nullptr;
  int* tok_stage_host = nullptr;
  int* tok_stage_dev = nullptr;
  // harvest staging: records (pinned + device) and packed tokens / log-probs of one batch of trajectories
  HarvestRec* hv_rec_host = nullptr;
  HarvestRec* hv_rec_dev = nullptr;
  int* hv_tok_dev = nullptr;
  float* hv_logp_dev = nullptr;
  size_t hv_cap = 0;
  // host bookkeeping
  std::vector<SeqHost> seqs;
  std::vector<int> free_sidx;
  std::vector<int> free_group;        // prompt-group table: free indices and unharvested members per group
  std::vector<int> group_members;
  std::unordered_map<uint64_t, int> id2sidx;
  uint64_t next_seq_id = 0, n_submitted = 0, n_harvested = 0, n_groups_total = 0;
  // timing
  std::vector<hipEvent_t> ev;
  uint64_t attn_launches = 0, attn_kv_tokens = 0;
  double attn_ms = 0.0, wall_ms_steps = 0.0;
  std::vector<void*> allocs;
  std::vector<void*> host_allocs;
};

namespace {

thread_local std::string g_err;

int fail(rollout_ctx* c, int code, const std::string& msg) {
  if (c) c->err = msg;
  g_err = msg;
  return code;
}

#define HIPCHK(c, expr)                                                                              \
  do {                                                                                               \
    hipError_t e_ = (expr);                                                                          \
    if (e_ != hipSuccess) {                                                                          \
      if (c) (c)->dead = true;                                                                       \
      return fail(c, ROLLOUT_EDEVICE, std::string(#expr) + ": " + hipGetErrorString(e_));            \
    }                                                                                                \
  } while (0)

template <typename T>
int dev_alloc(rollout_ctx* c, T** p, size_t n) {
  void* q = nullptr;
  hipError_t e = hipMalloc(&q, n * sizeof(T) + 256);
  if (e != hipSuccess) return fail(c, ROLLOUT_ENOMEM, std::string("hipMalloc failed: ") + hipGetErrorString(e));
  c->allocs.push_back(q);
  *p = (T*)q;
  return 0;
}
template <typename T>
int host_alloc(rollout_ctx* c, T** p, size_t n) {
  void* q = nullptr;
  hipError_t e = hipHostMalloc(&q, n * sizeof(T) + 64, hipHostMallocDefault);
  if (e != hipSuccess) return fail(c, ROLLOUT_ENOMEM, std::string("hipHostMalloc failed: ") + hipGetErrorString(e));
  c->host_allocs.push_back(q);
  *p = (T*)q;
  return 0;
}
#define TRY(expr)          \
  do {                     \
    int r_ = (expr);       \
    if (r_ != 0) return r_; \
  } while (0)

// splitmix64 (Steele, Lea, Flood 2014) driving a Fisher-Yates shuffle: initial order of the page free list
std::vector<int> page_permutation(int n, uint64_t seed) {
  std::vector<int> p(n);
  for (int i = 0; i < n; ++i) p[i] = i;
  uint64_t s = seed;
  for (int i = n - 1; i > 0; --i) {
    s += 0x9E3779B97F4A7C15ull;
    uint64_t z = s;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    z ^= z >> 31;
    std::swap(p[i], p[(int)(z % (uint64_t)(i + 1))]);
  }
  return p;
}

int sync_status(rollout_ctx* c) {
  HIPCHK(c, hipMemcpyAsync(c->status_host, c->sd.status, sizeof(int) * c->status_ints, hipMemcpyDeviceToHost, c->stream));
  HIPCHK(c, hipStreamSynchronize(c->stream));
  return 0;
}

// ---- weights ---------------------------------------------------------------------------------------
struct BlobReader {
  rollout_ctx* c;
  const uint8_t* base;
  size_t esz, off = 0, total;
  void* tmp = nullptr;  // device staging for host blobs
  size_t tmp_bytes = 0;
  uint16_t* rowmajor = nullptr;  // device staging: a projection matrix assembled row-major before it is packed
  // pack the assembled [n_rows, cols] matrix (rows padded with zeros to a multiple of 32) into dst
  int pack(size_t n_rows, size_t cols, uint16_t* dst) {
    const size_t n_pad = (n_rows + 31) / 32 * 32;
    if (n_pad > n_rows) HIPCHK(c, hipMemsetAsync(rowmajor + n_rows * cols, 0, (n_pad - n_rows) * cols * 2, c->stream));
    launch_pack_weights(rowmajor, dst, n_pad, cols, c->stream);
    HIPCHK(c, hipStreamSynchronize(c->stream));
    return 0;
  }
  int take(size_t rows, size_t cols, void* dst, int dst_fp32, size_t row0, size_t blk, size_t blk_stride) {
    const size_t bytes = rows * cols * esz;
    if (off + bytes > total) return fail(c, ROLLOUT_EINVAL, "weights blob smaller than the configured shape");
    const void* src = base + off;
    if (!c->cfg.weights_on_device) {
      HIPCHK(c, hipMemcpyAsync(tmp, src, bytes, hipMemcpyHostToDevice, c->stream));
      src = tmp;
    }
    launch_repack(src, c->cfg.weight_dtype == 0, dst, dst_fp32, rows, cols, row0, blk ? blk : rows, blk_stride, c->stream);
    if (!c->cfg.weights_on_device) HIPCHK(c, hipStreamSynchronize(c->stream));
    off += bytes;
    return 0;
  }
};

inline size_t pad32(size_t n) { return (n + 31) / 32 * 32; }

int alloc_weights(rollout_ctx* c) {
  const size_t D = c->D, F = c->F, V = c->V, qd = (size_t)c->Hq * c->d;
  TRY(dev_alloc(c, &c->embed, V * D));
  TRY(dev_alloc(c, &c->lm_head, pad32(V) * D));
  TRY(dev_alloc(c, &c->final_norm, D));
  c->layers.resize(c->NL);
  for (int l = 0; l < c->NL; ++l) {
    LayerW& L = c->layers[l];
    TRY(dev_alloc(c, &L.attn_norm, D));
    TRY(dev_alloc(c, &L.wqkv, pad32((size_t)c->Nqkv) * D));
    TRY(dev_alloc(c, &L.wo, pad32(D) * qd));
    TRY(dev_alloc(c, &L.ffn_norm, D));
    TRY(dev_alloc(c, &L.wgu, 2 * F * D));
    TRY(dev_alloc(c, &L.wdown, pad32(D) * F));
    if (c->cfg.qkv_bias) TRY(dev_alloc(c, &L.bqkv, (size_t)c->Nqkv));
  }
  return 0;
}

// Convert and repack a weights blob into the engine's buffers (used by rollout_init and rollout_update_weights).
int fill_weights(rollout_ctx* c, const void* weights, size_t weights_bytes) {
  const size_t D = c->D, F = c->F, V = c->V, qd = (size_t)c->Hq * c->d, kvd = (size_t)c->Hkv * c->d;
  BlobReader br{c, (const uint8_t*)weights, c->cfg.weight_dtype == 0 ? (size_t)4 : (size_t)2, 0, weights_bytes};
  // staging must hold the largest assembled matrix (with its padded rows)
  const size_t big = std::max({pad32(V) * D, 2 * F * D, pad32((size_t)c->Nqkv) * D, pad32(D) * qd, pad32(D) * F});
  if (!c->cfg.weights_on_device) {
    br.tmp_bytes = big * br.esz;
    if (hipMalloc(&br.tmp, br.tmp_bytes) != hipSuccess) return fail(c, ROLLOUT_ENOMEM, "hipMalloc failed (weight staging)");
  }
  if (hipMalloc((void**)&br.rowmajor, big * 2) != hipSuccess) {
    if (br.tmp) (void)hipFree(br.tmp);
    return fail(c, ROLLOUT_ENOMEM, "hipMalloc failed (weight staging)");
  }
  struct Guard {   // staging is only needed while loading
    BlobReader& b;
    ~Guard() { if (b.tmp) (void)hipFree(b.tmp); if (b.rowmajor) (void)hipFree(b.rowmajor); }
  } guard{br};
  TRY(br.take(V, D, c->embed, 0, 0, 0, 0));
  for (int l = 0; l < c->NL; ++l) {
    LayerW& L = c->layers[l];
    TRY(br.take(1, D, L.attn_norm, 1, 0, 0, 0));
    TRY(br.take(qd, D, br.rowmajor, 0, 0, 0, 0));
    TRY(br.take(kvd, D, br.rowmajor, 0, qd, 0, 0));
    TRY(br.take(kvd, D, br.rowmajor, 0, qd + kvd, 0, 0));
    TRY(br.pack((size_t)c->Nqkv, D, L.wqkv));
    if (c->cfg.qkv_bias) {
      // biases are [1, n] rows in the blob: load them as n rows of one column so they land contiguously
      TRY(br.take(qd, 1, L.bqkv, 1, 0, 0, 0));
      TRY(br.take(kvd, 1, L.bqkv, 1, qd, 0, 0));
      TRY(br.take(kvd, 1, L.bqkv, 1, qd + kvd, 0, 0));
    }
    TRY(br.take(D, qd, br.rowmajor, 0, 0, 0, 0));
    TRY(br.pack(D, qd, L.wo));
    TRY(br.take(1, D, L.ffn_norm, 1, 0, 0, 0));
    TRY(br.take(F, D, br.rowmajor, 0, 0, 16, 32));    // gate rows -> blocks 0,2,4,.. of 16
    TRY(br.take(F, D, br.rowmajor, 0, 16, 16, 32));   // up rows   -> blocks 1,3,5,..
    TRY(br.pack(2 * F, D, L.wgu));
    TRY(br.take(D, F, br.rowmajor, 0, 0, 0, 0));
    TRY(br.pack(D, F, L.wdown));
  }
  TRY(br.take(1, D, c->final_norm, 1, 0, 0, 0));
  TRY(br.take(V, D, br.rowmajor, 0, 0, 0, 0));
  TRY(br.pack(V, D, c->lm_head));
  if (br.off != weights_bytes) return fail(c, ROLLOUT_EINVAL, "weights blob larger than the configured shape");
  HIPCHK(c, hipStreamSynchronize(c->stream));
  return 0;
}

// ---- the per-step kernel chain over a set of rows (decode rows or one prefill pass) ---------------------
void run_layers(rollout_ctx* c, int R, const int* row_slot, const int* row_pos, const int* row_tok, const int4* work,
                const int2* row_wstart, int n_work, int chunk_tokens, bool time_attn, const PfTileHost* pf_tiles = nullptr,
                int n_tiles = 0) {
  hipStream_t st = c->stream;
  const int D = c->D, F = c->F, Hq = c->Hq, Hkv = c->Hkv, d = c->d, Nqkv = c->Nqkv;
  const float eps = c->cfg.rms_eps;
  launch_embed(c->embed, row_tok, c->h, R, D, st);
  launch_add_rmsnorm(c->h, nullptr, 0, 0, c->layers[0].attn_norm, eps, c->x, R, D, st);
  const int S1 = gemm_pick_splits(R, Nqkv, D), S2 = gemm_pick_splits(R, D, Hq * d), S4 = gemm_pick_splits(R, D, F);
  for (int l = 0; l < c->NL; ++l) {
    const LayerW& L = c->layers[l];
    uint8_t* pool_l = c->kv_pool + (size_t)l * c->layer_pool_bytes;
    launch_gemm(c->x, L.wqkv, c->part, R, Nqkv, D, S1, st);
    launch_rope_kvwrite(c->part, S1, (size_t)R * Nqkv, L.bqkv, row_slot, row_pos, c->cs_table, c->qbuf, pool_l,
                        c->sd.page_table, c->max_pages, Hq, Hkv, d, R, st);
    AttnArgs a;
    a.pool = pool_l;
    a.q = c->qbuf;
    a.row_slot = row_slot;
    a.row_pos = row_pos;
    a.page_table = c->sd.page_table;
    a.max_pages = c->max_pages;
    a.work = work;
    a.row_wstart = row_wstart;
    a.n_work = n_work;
    a.n_rows = R;
    a.Hkv = Hkv;
    a.part_acc = c->part_acc;
    a.part_ml = c->part_ml;
    a.row_cnt = c->attn_row_cnt;
    a.out = c->attn_out;
    a.out_fp32 = 0;
    a.chunk_tokens = chunk_tokens;
    if (n_tiles > 0) {
      launch_prefill_attn(pool_l, c->qbuf, pf_tiles, n_tiles, c->sd.page_table, c->max_pages, Hq, Hkv, d, c->attn_out, st);
    } else {
      launch_decode_attn(a, d, c->G, st, time_attn ? c->ev[2 * l] : nullptr, time_attn ? c->ev[2 * l + 1] : nullptr);
    }
    launch_gemm(c->attn_out, L.wo, c->part, R, D, Hq * d, S2, st);
    launch_add_rmsnorm(c->h, c->part, S2, (size_t)R * D, L.ffn_norm, eps, c->x, R, D, st);
    launch_gemm_swiglu(c->x, L.wgu, c->act, R, 2 * F, D, st);
    launch_gemm(c->act, L.wdown, c->part, R, D, F, S4, st);
    const float* next_gain = l + 1 < c->NL ? c->layers[l + 1].attn_norm : c->final_norm;
    launch_add_rmsnorm(c->h, c->part, S4, (size_t)R * D, next_gain, eps, c->x, R, D, st);
  }
}

int run_prefill(rollout_ctx* c, int n_dec, int n_adm) {
  // admitted sequences in ascending slot order (= admission order, so a rollout that attaches to shared prompt
  // pages always comes after the sibling that fills them): (slot, sidx, end position, first position) per admission
  const int* desc = c->status_host + STAT_HDR;
  int a = 0, pos = desc[3];  // cursor: sequence a, next position pos
  hipStream_t st = c->stream;
  while (a < n_adm) {
    int rows = 0, n_desc = 0, n_last = 0, n_tiles = 0;
    while (a < n_adm && rows < PF_ROWS) {
      const int slot = desc[STAT_ADM_INTS * a], sidx = desc[STAT_ADM_INTS * a + 1], n = desc[STAT_ADM_INTS * a + 2];
      const int take = std::min(n - pos, PF_ROWS - rows);
      c->pf_desc_host[n_desc++] = PrefillDesc{slot, sidx, take, pos, rows};
      for (int t = 0; t < take; t += 32)   // query tiles of up to 32 consecutive tokens
        c->pf_tiles_host[n_tiles++] = PfTileHost{rows + t, std::min(32, take - t), slot, pos + t};
      rows += take;
      pos += take;
      if (pos == n) {
        c->pf_last_host[2 * n_last] = rows - 1;   // row holding the sequence's last token
        c->pf_last_host[2 * n_last + 1] = a;      // its index among the admitted
        ++n_last;
        ++a;
        pos = a < n_adm ? desc[STAT_ADM_INTS * a + 3] : 0;
      }
    }
    HIPCHK(c, hipMemcpyAsync(c->pf_desc_dev, c->pf_desc_host, sizeof(PrefillDesc) * n_desc, hipMemcpyHostToDevice, st));
    HIPCHK(c, hipMemcpyAsync(c->pf_tiles_dev, c->pf_tiles_host, sizeof(PfTileHost) * n_tiles, hipMemcpyHostToDevice, st));
    launch_prefill_rows(c->sd, c->pf_desc_dev, n_desc, c->pf_row_slot, c->pf_row_pos, c->pf_row_tok, st);
    run_layers(c, rows, c->pf_row_slot, c->pf_row_pos, c->pf_row_tok, nullptr, nullptr, 0, 0, false, c->pf_tiles_dev, n_tiles);
    for (int j = 0; j < n_last; ++j) {
      // one tiny gather per finished prompt: h row -> h_final row n_dec + (index among admitted)
      const int src_row = c->pf_last_host[2 * j], dst = n_dec + c->pf_last_host[2 * j + 1];
      launch_gather_rows(c->h, c->iota + src_row, c->h_final, dst, 1, c->D, st);
    }
    // the pinned descriptor buffers are reused by the next pass
    HIPCHK(c, hipStreamSynchronize(st));
  }
  return 0;
}

int step_impl(rollout_ctx* c, const int32_t* forced_tok, rollout_step_info* info) {
  if (!c) return ROLLOUT_EINVAL;
  if (c->dead) return fail(c, ROLLOUT_EDEVICE, "context unusable after an earlier device error");
  if (forced_tok)   // the emit kernel indexes the logits row and, next step, the embedding table with these
    for (int i = 0; i < c->Q; ++i)
      if (forced_tok[i] >= c->V) return fail(c, ROLLOUT_ERANGE, "forced token id outside the vocabulary; nothing consumed");
  const auto t0 = std::chrono::steady_clock::now();
  HIPCHK(c, hipSetDevice(c->cfg.device));
  hipStream_t st = c->stream;
  int* sh = c->status_host;
  const int Q = c->Q;
  const int n_dec = sh[STAT_NDEC_NEXT], n_work = sh[STAT_NWORK_NEXT], chunk_tokens = sh[STAT_CHUNK];
  const unsigned long long ctx_sum = (unsigned long long)(unsigned)sh[STAT_CTX_LO] | ((unsigned long long)(unsigned)sh[STAT_CTX_HI] << 32);
  const int n_active = sh[STAT_NACTIVE];
  int n_adm = 0;
  unsigned long long pf_tokens = 0, pf_pairs = 0;
  const bool can_admit = sh[STAT_QUEUED] > 0 && n_active < Q && !(c->cfg.mode == ROLLOUT_MODE_SYNC && n_active > 0);
  if (can_admit) {
    launch_sched_admit(c->sd, st);
    TRY(sync_status(c));
    n_adm = sh[STAT_NADM];
    for (int a = 0; a < n_adm; ++a) {   // positions first .. n-1 of each admitted rollout are computed; position p sees p+1 keys
      const unsigned long long n = (unsigned)sh[STAT_HDR + STAT_ADM_INTS * a + 2], first = (unsigned)sh[STAT_HDR + STAT_ADM_INTS * a + 3];
      pf_tokens += n - first;
      pf_pairs += (n * (n + 1) - first * (first + 1)) / 2;
    }
  }
  if (forced_tok) {
    HIPCHK(c, hipMemcpyAsync(c->forced_tok_dev, forced_tok, sizeof(int) * Q, hipMemcpyHostToDevice, st));
    c->sd.forced_tok = c->forced_tok_dev;
  } else {
    c->sd.forced_tok = nullptr;
  }
  const bool model = !(c->cfg.debug_flags & ROLLOUT_DEBUG_NO_MODEL);
  const bool time_attn = (c->cfg.debug_flags & ROLLOUT_DEBUG_TIME_ATTN) != 0;
  const int n_rows = n_dec + n_adm;
  if (model && n_rows > 0) {
    if (n_dec > 0) {
      run_layers(c, n_dec, c->sd.row_slot, c->sd.row_pos, c->sd.row_tok, c->sd.work, c->sd.row_wstart, n_work, chunk_tokens, time_attn);
      launch_gather_rows(c->h, c->iota, c->h_final, 0, n_dec, c->D, st);
    }
    if (n_adm > 0) TRY(run_prefill(c, n_dec, n_adm));
    launch_add_rmsnorm(c->h_final, nullptr, 0, 0, c->final_norm, c->cfg.rms_eps, c->x_final, n_rows, c->D, st);
    if (forced_tok) {
      // teacher forcing reads arbitrary logits: keep the fp32 rows and take the statistics from them
      launch_gemm(c->x_final, c->lm_head, c->logits, n_rows, c->V, c->D, 1, st);
      launch_argmax_lse(c->logits, c->V, c->row_argmax, c->row_lse, c->row_ztok, c->row_zeos, n_rows, &c->sd, st);
    } else {
      // the rollout step proper: arg-max / Gumbel-max draw, EOS logit and log-sum-exp in the LM head's epilogue
      LmEpi e;
      e.scale = c->sd.inv_temp > 0.f ? c->sd.inv_temp : 1.f;
      e.sampling = c->sd.inv_temp > 0.f ? 1 : 0;
      e.seed = c->sd.sample_seed;
      e.eos_id = c->sd.eos_id;
      e.n_tiles = c->lm_tiles;
      e.row_slot = c->sd.row_slot;
      e.slot_seq = c->sd.slot_seq;
      e.seq_id = c->sd.seq_id;
      e.seq_gen_len = c->sd.seq_gen_len;
      e.part_f = c->lm_part_f;
      e.part_i = c->lm_part_i;
      e.row_zeos = c->row_zeos;
      launch_gemm_lm_fused(c->x_final, c->lm_head, n_rows, c->V, c->D, e, st);
      launch_lm_reduce(e, n_rows, c->row_argmax, c->row_ztok, c->row_lse, st);
    }
  }
  launch_sched_emit(c->sd, st);
  TRY(sync_status(c));
  if (time_attn && model && n_dec > 0) {
    for (int l = 0; l < c->NL; ++l) {
      float ms = 0.f;
      if (hipEventElapsedTime(&ms, c->ev[2 * l], c->ev[2 * l + 1]) == hipSuccess) c->attn_ms += ms;
    }
    c->attn_launches += c->NL;
    c->attn_kv_tokens += ctx_sum * (unsigned long long)c->NL;
  }
  if (info) {
    info->step = (uint64_t)sh[STAT_STEP];
    info->n_ran = (uint32_t)sh[STAT_R];
    info->n_active = (uint32_t)sh[STAT_NACTIVE];
    info->n_finished_unharvested = (uint32_t)sh[STAT_FIN];
    info->n_queued = (uint32_t)sh[STAT_QUEUED];
    info->free_pages = (uint32_t)sh[STAT_FREE];
    info->n_admitted = (uint32_t)sh[STAT_NADM];
    info->n_finished_step = (uint32_t)sh[STAT_NFIN_STEP];
    info->n_preempted_step = (uint32_t)sh[STAT_NPRE_STEP];
    info->ctx_tokens = (uint64_t)(unsigned)sh[STAT_CTX_LO] | ((uint64_t)(unsigned)sh[STAT_CTX_HI] << 32);
    info->n_decode_rows = (uint32_t)n_dec;
    info->prefill_tokens = (uint32_t)pf_tokens;
    info->decode_ctx_tokens = n_dec > 0 ? ctx_sum : 0;
    info->prefill_ctx_pairs = pf_pairs;
  }
  c->wall_ms_steps += std::chrono::duration<double, std::milli>(std::chrono::steady_clock::now() - t0).count();
  return 0;
}

// ---- the projection GEMM for callers that cannot allocate ---------------------------------------------------
// Split-K partial sums live in a fixed array inside the library's device image instead of a caller workspace.  Each
// GPU holds its own copy of the array at its own address: the address is looked up once per device, with that device
// current, and only that pointer is ever handed to kernels (the array's name is a host-side stand-in, not a device
// address).
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mu;
void* g_scratch_ptr[kMaxDevices] = {};
int static_scratch(void** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices)
    return fail(nullptr, ROLLOUT_EDEVICE, "no current HIP device (or its ordinal is above 63)");
  std::lock_guard<std::mutex> lk(g_scratch_mu);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !p)
      return fail(nullptr, ROLLOUT_EDEVICE, std::string("hipGetSymbolAddress(scratch): ") + hipGetErrorString(e));
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return 0;
}

}  // namespace

// =====================================================================================================
extern "C" {

const char* rollout_last_error(rollout_ctx* c) { return c ? c->err.c_str() : g_err.c_str(); }

void rollout_destroy(rollout_ctx* c) {
  if (!c) return;
  (void)hipSetDevice(c->cfg.device);
  if (c->stream) (void)hipStreamSynchronize(c->stream);
  for (hipEvent_t e : c->ev) (void)hipEventDestroy(e);
  for (void* p : c->allocs) (void)hipFree(p);
  for (void* p : c->host_allocs) (void)hipHostFree(p);
  if (c->stream) (void)hipStreamDestroy(c->stream);
  delete c;
}

int rollout_init(rollout_ctx** out, const void* weights, size_t weights_bytes, const rollout_cfg* cfg) {
  if (!out || !cfg || !weights) return fail(nullptr, ROLLOUT_EINVAL, "null argument");
  *out = nullptr;
  const rollout_cfg& f = *cfg;
  if (f.n_layers == 0 || f.d_model == 0 || f.n_q_heads == 0 || f.n_kv_heads == 0 || f.d_ffn == 0 || f.vocab == 0)
    return fail(nullptr, ROLLOUT_EINVAL, "zero-sized model dimension");
  if (f.n_q_heads % f.n_kv_heads != 0 || !attn_supported((int)f.head_dim, (int)(f.n_q_heads / f.n_kv_heads)))
    return fail(nullptr, ROLLOUT_EINVAL, "unsupported head_dim / query-group size (head_dim 32 or 128, group 1, 4 or 5)");
  if (f.page_tokens != PAGE_TOKENS) return fail(nullptr, ROLLOUT_EINVAL, "page_tokens must be 16");
  if (f.max_slots == 0 || f.max_slots > 1024) return fail(nullptr, ROLLOUT_EINVAL, "max_slots must be in 1..1024");
  if (f.d_model % 64 || f.d_ffn % 64 || (f.n_q_heads * f.head_dim) % 64 || f.d_model > 8192 || f.d_ffn > (1u << 20) ||
      f.vocab > (1u << 24))
    return fail(nullptr, ROLLOUT_EINVAL,
                "d_model, d_ffn and n_q_heads*head_dim must be multiples of 64; d_model <= 8192, d_ffn <= 2^20, vocab <= 2^24");
  if (f.max_prompt_len == 0 || f.max_new_tokens == 0 || f.max_seqs == 0)
    return fail(nullptr, ROLLOUT_EINVAL, "max_prompt_len, max_new_tokens and max_seqs must be positive");
  if (f.eos_id < 0 || (uint32_t)f.eos_id >= f.vocab) return fail(nullptr, ROLLOUT_EINVAL, "eos_id outside the vocabulary");
  if (f.mode > 2 || f.eos_mode > 1 || f.weight_dtype > 1) return fail(nullptr, ROLLOUT_EINVAL, "bad mode / eos_mode / weight_dtype");
  if (!(f.temperature >= 0.f)) return fail(nullptr, ROLLOUT_EINVAL, "temperature must be >= 0");
  int ndev = 0;
  if (hipGetDeviceCount(&ndev) != hipSuccess || ndev <= 0 || f.device < 0 || f.device >= ndev)
    return fail(nullptr, ROLLOUT_EDEVICE, "no usable HIP device (this library has no CPU fallback)");

  rollout_ctx* c = new rollout_ctx();
  c->cfg = f;
  c->NL = f.n_layers; c->D = f.d_model; c->Hq = f.n_q_heads; c->Hkv = f.n_kv_heads; c->d = f.head_dim;
  c->F = f.d_ffn; c->V = f.vocab; c->G = c->Hq / c->Hkv; c->Nqkv = (c->Hq + 2 * c->Hkv) * c->d; c->Q = f.max_slots;
#define INIT_TRY(expr)        \
  do {                        \
    int r_ = (expr);          \
    if (r_ != 0) {            \
      g_err = c->err;         \
      rollout_destroy(c);     \
      return r_;              \
    }                         \
  } while (0)
#define INIT_HIP(expr)                                                                          \
  do {                                                                                          \
    hipError_t e_ = (expr);                                                                     \
    if (e_ != hipSuccess) {                                                                     \
      g_err = std::string(#expr) + ": " + hipGetErrorString(e_);                                \
      rollout_destroy(c);                                                                       \
      return ROLLOUT_EDEVICE;                                                                   \
    }                                                                                           \
  } while (0)
  INIT_HIP(hipSetDevice(f.device));
  INIT_HIP(hipStreamCreateWithFlags(&c->stream, hipStreamNonBlocking));

  // ---- KV pool --------------------------------------------------------------------------------------
  c->max_pages = (int)((f.max_prompt_len + f.max_new_tokens + PAGE_TOKENS - 1) / PAGE_TOKENS);
  const size_t page_layer_bytes = (size_t)c->Hkv * kv_block_bytes(c->d);
  const size_t page_bytes = page_layer_bytes * c->NL;
  long long n_pages = f.kv_pool_bytes ? (long long)(f.kv_pool_bytes / page_bytes) : (long long)c->Q * c->max_pages;
  if (n_pages < c->max_pages) {
    g_err = "kv_pool_bytes cannot hold one maximum-length rollout";
    rollout_destroy(c);
    return ROLLOUT_ENOMEM;
  }
  if (n_pages > (1ll << 30)) n_pages = 1ll << 30;
  c->n_pages = (int)n_pages;
  c->layer_pool_bytes = (size_t)c->n_pages * page_layer_bytes;
  if (!(f.debug_flags & ROLLOUT_DEBUG_NO_MODEL)) {   // a scheduler-only context counts pages but never touches them
    INIT_TRY(dev_alloc(c, &c->kv_pool, c->layer_pool_bytes * c->NL));
    INIT_HIP(hipMemsetAsync(c->kv_pool, 0, c->layer_pool_bytes * c->NL, c->stream));
  }

  // ---- RoPE table: cos/sin of pos * theta^(-2i/d), evaluated in double --------------------------------
  {
    const int max_pos = (int)(f.max_prompt_len + f.max_new_tokens), half = c->d / 2;
    std::vector<float2> tab((size_t)max_pos * half);
    for (int i = 0; i < half; ++i) {
      const double freq = std::pow((double)f.rope_theta, -2.0 * i / c->d);
      for (int p = 0; p < max_pos; ++p) {
        const double ang = (double)p * freq;
        tab[(size_t)p * half + i] = make_float2((float)std::cos(ang), (float)std::sin(ang));
      }
    }
    INIT_TRY(dev_alloc(c, &c->cs_table, tab.size()));
    INIT_HIP(hipMemcpy(c->cs_table, tab.data(), tab.size() * sizeof(float2), hipMemcpyHostToDevice));
  }

  // ---- scheduler state -------------------------------------------------------------------------------
  SchedDev& s = c->sd;
  memset(&s, 0, sizeof(s));
  s.Q = c->Q; s.max_pages = c->max_pages; s.n_pages = c->n_pages; s.max_seqs = f.max_seqs;
  int qcap = 1;
  while (qcap < (int)f.max_seqs + 1) qcap <<= 1;
  s.qmask = qcap - 1;
  s.tok_stride = f.max_prompt_len + f.max_new_tokens; s.cap = f.max_new_tokens; s.eos_id = f.eos_id;
  s.eos_mode = f.eos_mode; s.mode = f.mode; s.max_staleness = f.max_staleness;
  s.no_model = (f.debug_flags & ROLLOUT_DEBUG_NO_MODEL) ? 1 : 0; s.V = c->V; s.Hkv = c->Hkv;
  s.inv_temp = f.temperature > 0.f ? 1.0f / f.temperature : 0.f; s.sample_seed = f.sample_seed;
  const size_t MS = f.max_seqs, Q = c->Q;
  INIT_TRY(dev_alloc(c, &s.sc, SC_COUNT));
  INIT_TRY(dev_alloc(c, &s.ctr, CT_COUNT));
  INIT_TRY(dev_alloc(c, &s.slot_seq, Q));
  INIT_TRY(dev_alloc(c, &s.slot_npages, Q));
  INIT_TRY(dev_alloc(c, &s.page_table, Q * c->max_pages));
  INIT_TRY(dev_alloc(c, &s.seq_prompt_len, MS));
  INIT_TRY(dev_alloc(c, &s.seq_target_len, MS));
  INIT_TRY(dev_alloc(c, &s.seq_gen_len, MS));
  INIT_TRY(dev_alloc(c, &s.seq_state, MS));
  INIT_TRY(dev_alloc(c, &s.seq_slot, MS));
  INIT_TRY(dev_alloc(c, &s.seq_completion, MS));
  INIT_TRY(dev_alloc(c, &s.seq_kv_version, MS));
  INIT_TRY(dev_alloc(c, &s.seq_npreempt, MS));
  INIT_TRY(dev_alloc(c, &s.seq_fin_version, MS));
  INIT_TRY(dev_alloc(c, &s.seq_id, MS));
  INIT_TRY(dev_alloc(c, &s.seq_tokens, MS * s.tok_stride));
  INIT_TRY(dev_alloc(c, &s.seq_logp, MS * s.cap));
  s.max_shared = std::max(1, (int)((f.max_prompt_len - 1) / PAGE_TOKENS));
  INIT_TRY(dev_alloc(c, &s.seq_group, MS));
  INIT_TRY(dev_alloc(c, &s.grp_nshared, MS));
  INIT_TRY(dev_alloc(c, &s.grp_ref, MS));
  INIT_TRY(dev_alloc(c, &s.grp_version, MS));
  INIT_TRY(dev_alloc(c, &s.grp_pages, MS * (size_t)s.max_shared));
  INIT_TRY(dev_alloc(c, &s.q_ring, (size_t)qcap));
  INIT_TRY(dev_alloc(c, &s.free_stack, (size_t)c->n_pages));
  INIT_TRY(dev_alloc(c, &s.fin_list, MS));
  INIT_TRY(dev_alloc(c, &s.row_slot, Q));
  INIT_TRY(dev_alloc(c, &s.row_pos, Q));
  INIT_TRY(dev_alloc(c, &s.row_tok, Q));
  INIT_TRY(dev_alloc(c, &s.row_wstart, Q));
  const size_t dec_work = Q * (size_t)((s.tok_stride + ATTN_CHUNK_MIN - 1) / ATTN_CHUNK_MIN);
  INIT_TRY(dev_alloc(c, &s.work, dec_work));
  c->status_ints = STAT_HDR + STAT_ADM_INTS * c->Q;
  INIT_TRY(dev_alloc(c, &s.status, (size_t)c->status_ints));
  INIT_TRY(host_alloc(c, &c->status_host, (size_t)c->status_ints));
  INIT_TRY(dev_alloc(c, &c->forced_tok_dev, Q));
  INIT_HIP(hipMemsetAsync(s.seq_tokens, 0, MS * s.tok_stride * sizeof(int), c->stream));
  {
    std::vector<int> perm = page_permutation(c->n_pages, f.page_seed);
    INIT_HIP(hipMemcpy(s.free_stack, perm.data(), perm.size() * sizeof(int), hipMemcpyHostToDevice));
  }
  launch_sched_init(s, c->stream);
  c->seqs.resize(MS);
  for (int i = (int)MS - 1; i >= 0; --i) c->free_sidx.push_back(i);
  for (int i = (int)MS - 1; i >= 0; --i) c->free_group.push_back(i);
  c->group_members.assign(MS, 0);
  INIT_TRY(host_alloc(c, &c->sub_host, MS));
  INIT_TRY(dev_alloc(c, &c->sub_dev, MS));
  INIT_TRY(host_alloc(c, &c->tok_stage_host, MS * f.max_prompt_len));
  INIT_TRY(dev_alloc(c, &c->tok_stage_dev, MS * f.max_prompt_len));
  c->hv_cap = std::max<size_t>(f.max_new_tokens, std::min<size_t>(MS * (size_t)f.max_new_tokens, (size_t)1 << 22));
  INIT_TRY(host_alloc(c, &c->hv_rec_host, MS));
  INIT_TRY(dev_alloc(c, &c->hv_rec_dev, MS));
  INIT_TRY(dev_alloc(c, &c->hv_tok_dev, c->hv_cap));
  INIT_TRY(dev_alloc(c, &c->hv_logp_dev, c->hv_cap));

  // ---- activations / workspaces ----------------------------------------------------------------------
  const bool model = !(f.debug_flags & ROLLOUT_DEBUG_NO_MODEL);
  if (model) {
    const size_t R = std::max<size_t>(Q, PF_ROWS);
    c->rows_cap = (int)R;
    const size_t D = c->D, F = c->F, V = c->V;
    INIT_TRY(dev_alloc(c, &c->h, R * D));
    INIT_TRY(dev_alloc(c, &c->x, R * D));
    size_t part_elems = 0;   // split-K partials: worst case over every row count a chain can run with
    for (size_t rows = 1; rows <= R; ++rows) {
      const int r = (int)rows;
      part_elems = std::max(part_elems, (size_t)gemm_pick_splits(r, c->Nqkv, c->D) * rows * c->Nqkv);
      part_elems = std::max(part_elems, (size_t)gemm_pick_splits(r, c->D, c->Hq * c->d) * rows * D);
      part_elems = std::max(part_elems, (size_t)gemm_pick_splits(r, c->D, c->F) * rows * D);
    }
    INIT_TRY(dev_alloc(c, &c->part, part_elems));
    INIT_TRY(dev_alloc(c, &c->qbuf, R * c->Hq * c->d));
    INIT_TRY(dev_alloc(c, &c->attn_out, R * c->Hq * c->d));
    INIT_TRY(dev_alloc(c, &c->act, R * F));
    INIT_TRY(dev_alloc(c, &c->h_final, Q * D));
    INIT_TRY(dev_alloc(c, &c->x_final, Q * D));
    INIT_TRY(dev_alloc(c, &c->logits, Q * V));
    INIT_TRY(dev_alloc(c, &c->row_argmax, Q));
    INIT_TRY(dev_alloc(c, &c->row_lse, Q));
    INIT_TRY(dev_alloc(c, &c->row_ztok, Q));
    INIT_TRY(dev_alloc(c, &c->row_zeos, Q));
    c->lm_tiles = (c->V + 127) / 128;
    INIT_TRY(dev_alloc(c, &c->lm_part_f, Q * (size_t)c->lm_tiles));
    INIT_TRY(dev_alloc(c, &c->lm_part_i, Q * (size_t)c->lm_tiles));
    INIT_TRY(dev_alloc(c, &c->iota, R));
    {
      std::vector<int> io(R);
      for (size_t i = 0; i < R; ++i) io[i] = (int)i;
      INIT_HIP(hipMemcpy(c->iota, io.data(), R * sizeof(int), hipMemcpyHostToDevice));
    }
    INIT_TRY(dev_alloc(c, &c->pf_row_slot, (size_t)PF_ROWS));
    INIT_TRY(dev_alloc(c, &c->pf_row_pos, (size_t)PF_ROWS));
    INIT_TRY(dev_alloc(c, &c->pf_row_tok, (size_t)PF_ROWS));
    c->max_work = dec_work;
    INIT_TRY(dev_alloc(c, &c->pf_tiles_dev, (size_t)PF_ROWS));
    INIT_TRY(host_alloc(c, &c->pf_tiles_host, (size_t)PF_ROWS));
    INIT_TRY(dev_alloc(c, &c->pf_desc_dev, (size_t)PF_ROWS));
    INIT_TRY(host_alloc(c, &c->pf_desc_host, (size_t)PF_ROWS));
    INIT_TRY(host_alloc(c, &c->pf_last_host, (size_t)2 * PF_ROWS));
    INIT_TRY(dev_alloc(c, &c->part_acc, c->max_work * c->Hq * c->d));
    INIT_TRY(dev_alloc(c, &c->part_ml, c->max_work * c->Hq * 2));
    INIT_TRY(dev_alloc(c, &c->attn_row_cnt, Q * (size_t)c->Hkv));   // zero now; every attention launch leaves it at zero
    INIT_HIP(hipMemsetAsync(c->attn_row_cnt, 0, Q * (size_t)c->Hkv * sizeof(int), c->stream));
    s.row_argmax = c->row_argmax;
    s.row_lse = c->row_lse;
    s.row_ztok = c->row_ztok;
    s.row_zeos = c->row_zeos;
    s.logits = c->logits;
    INIT_TRY(alloc_weights(c));
    INIT_TRY(fill_weights(c, weights, weights_bytes));
    if (f.debug_flags & ROLLOUT_DEBUG_TIME_ATTN) {
      c->ev.resize(2 * (size_t)c->NL);
      for (auto& e : c->ev) INIT_HIP(hipEventCreate(&e));
    }
  }
  INIT_TRY(sync_status(c));
  *out = c;
  return ROLLOUT_OK;
#undef INIT_TRY
#undef INIT_HIP
}

int rollout_submit_n(rollout_ctx* c, const int32_t* tokens, const uint32_t* offsets, const uint32_t* target_len,
                     uint32_t n, uint32_t k, uint64_t* first_seq_id) {
  if (!c || !tokens || !offsets || (!target_len && n)) return fail(c, ROLLOUT_EINVAL, "null argument");
  if (k == 0) return fail(c, ROLLOUT_EINVAL, "responses per prompt must be positive");
  if (c->dead) return fail(c, ROLLOUT_EDEVICE, "context unusable after an earlier device error");
  if (c->cfg.grouped_loading && c->n_submitted != c->n_harvested)
    return fail(c, ROLLOUT_EBUSY, "grouped loading: the previous group is not fully harvested");
  const uint64_t total = (uint64_t)n * k;
  if (total > c->free_sidx.size()) return fail(c, ROLLOUT_EBUSY, "sequence table full (max_seqs unharvested rollouts)");
  for (uint32_t i = 0; i < n; ++i) {
    if (offsets[i + 1] <= offsets[i] || offsets[i + 1] - offsets[i] > c->cfg.max_prompt_len)
      return fail(c, ROLLOUT_ERANGE, "empty or over-long prompt");
    for (uint32_t r = 0; r < k; ++r)
      if (target_len[(size_t)i * k + r] > c->cfg.max_new_tokens)
        return fail(c, ROLLOUT_ERANGE, "target_len exceeds max_new_tokens");
    for (uint32_t j = offsets[i]; j < offsets[i + 1]; ++j)
      if (tokens[j] < 0 || (uint32_t)tokens[j] >= c->cfg.vocab) return fail(c, ROLLOUT_ERANGE, "token id outside the vocabulary");
  }
  if (first_seq_id) *first_seq_id = c->next_seq_id;
  if (total == 0) return ROLLOUT_OK;
  HIPCHK(c, hipSetDevice(c->cfg.device));
  size_t tok_off = 0, rec = 0;
  for (uint32_t i = 0; i < n; ++i) {
    const int plen = (int)(offsets[i + 1] - offsets[i]);
    // the pages a prompt fills completely, not counting the one with its last token, are shared by its responses
    const int nshared = (plen - 1) / PAGE_TOKENS;
    int group = -1;
    if (k > 1 && nshared > 0) {
      group = c->free_group.back();
      c->free_group.pop_back();
      c->group_members[group] = (int)k;
    }
    for (uint32_t r = 0; r < k; ++r) {
      const int sidx = c->free_sidx.back();
      c->free_sidx.pop_back();
      SeqHost& sh = c->seqs[sidx];
      sh.seq_id = c->next_seq_id++;
      sh.prompt_len = plen;
      sh.in_use = true;
      sh.harvested = false;
      sh.group = group;
      c->id2sidx[sh.seq_id] = sidx;
      c->sub_host[rec++] = SubmitRec{sidx, plen, (int)target_len[(size_t)i * k + r], (int)tok_off, sh.seq_id, group, nshared};
    }
    memcpy(c->tok_stage_host + tok_off, tokens + offsets[i], sizeof(int) * plen);
    tok_off += plen;
  }
  c->n_submitted += total;
  HIPCHK(c, hipMemcpyAsync(c->sub_dev, c->sub_host, sizeof(SubmitRec) * total, hipMemcpyHostToDevice, c->stream));
  HIPCHK(c, hipMemcpyAsync(c->tok_stage_dev, c->tok_stage_host, sizeof(int) * tok_off, hipMemcpyHostToDevice, c->stream));
  launch_sched_submit(c->sd, c->sub_dev, c->tok_stage_dev, (int)total, c->stream);
  TRY(sync_status(c));
  return ROLLOUT_OK;
}

int rollout_submit(rollout_ctx* c, const int32_t* tokens, const uint32_t* offsets, const uint32_t* target_len,
                   uint32_t n, uint64_t* first_seq_id) {
  return rollout_submit_n(c, tokens, offsets, target_len, n, 1, first_seq_id);
}

int rollout_update_weights(rollout_ctx* c, const void* weights, size_t weights_bytes) {
  if (!c || !weights) return fail(c, ROLLOUT_EINVAL, "null argument");
  if (c->dead) return fail(c, ROLLOUT_EDEVICE, "context unusable after an earlier device error");
  if (c->cfg.debug_flags & ROLLOUT_DEBUG_NO_MODEL) return ROLLOUT_OK;
  HIPCHK(c, hipSetDevice(c->cfg.device));
  HIPCHK(c, hipStreamSynchronize(c->stream));
  const int r = fill_weights(c, weights, weights_bytes);
  if (r == ROLLOUT_EINVAL) c->dead = true;   // buffers may hold a mix of old and new tensors
  return r;
}

int rollout_step(rollout_ctx* c, rollout_step_info* info) { return step_impl(c, nullptr, info); }

int rollout_step_forced(rollout_ctx* c, const int32_t* forced_tok, float* logits_out, rollout_step_info* info) {
  if (!c) return ROLLOUT_EINVAL;
  if (!logits_out) return step_impl(c, forced_tok, info);
  // the emit kernel rewrites the row list, so capture this step's row -> slot map before it runs:
  // the decode rows are known before the step; admitted slots come from the status block afterwards
  const int n_dec = c->status_host[STAT_NDEC_NEXT];
  std::vector<int> row_slot(c->Q, -1);
  if (n_dec > 0) {
    HIPCHK(c, hipMemcpy(row_slot.data(), c->sd.row_slot, sizeof(int) * n_dec, hipMemcpyDeviceToHost));
  }
  const int r = step_impl(c, forced_tok, info);
  if (r != 0) return r;
  if (c->cfg.debug_flags & ROLLOUT_DEBUG_NO_MODEL) return 0;
  const int n_adm = c->status_host[STAT_NADM];
  for (int a = 0; a < n_adm; ++a) row_slot[n_dec + a] = c->status_host[STAT_HDR + STAT_ADM_INTS * a];
  for (int row = 0; row < n_dec + n_adm; ++row)
    HIPCHK(c, hipMemcpy(logits_out + (size_t)row_slot[row] * c->V, c->logits + (size_t)row * c->V, sizeof(float) * c->V,
                        hipMemcpyDeviceToHost));
  return 0;
}

int rollout_harvest(rollout_ctx* c, uint32_t group_size, uint32_t flags, rollout_traj* recs, uint32_t recs_cap,
                    int32_t* tok_buf, float* logp_buf, uint64_t tok_cap, uint32_t* n_groups, uint32_t* n_recs,
                    uint64_t* tok_needed) {
  if (!c || group_size == 0 || !n_groups) return fail(c, ROLLOUT_EINVAL, "null argument or zero group size");
  if (c->dead) return fail(c, ROLLOUT_EDEVICE, "context unusable after an earlier device error");
  HIPCHK(c, hipSetDevice(c->cfg.device));
  HIPCHK(c, hipStreamSynchronize(c->stream));
  *n_groups = 0;
  if (n_recs) *n_recs = 0;
  if (tok_needed) *tok_needed = 0;
  const int* sh = c->status_host;
  const int nfin = sh[STAT_FIN];
  const bool drained = sh[STAT_QUEUED] == 0 && sh[STAT_NACTIVE] == 0;
  int k = nfin / (int)group_size;
  int take = k * (int)group_size;
  if ((flags & ROLLOUT_FLUSH) && drained && nfin > take) {
    take = nfin;
    ++k;
  }
  if (k == 0) return ROLLOUT_OK;
  const size_t MS = c->cfg.max_seqs;
  std::vector<int> fin(nfin), comp(MS), glen(MS), slot(MS), npre(MS), fver(MS);
  HIPCHK(c, hipMemcpy(fin.data(), c->sd.fin_list, sizeof(int) * nfin, hipMemcpyDeviceToHost));
  HIPCHK(c, hipMemcpy(comp.data(), c->sd.seq_completion, sizeof(int) * MS, hipMemcpyDeviceToHost));
  HIPCHK(c, hipMemcpy(glen.data(), c->sd.seq_gen_len, sizeof(int) * MS, hipMemcpyDeviceToHost));
  HIPCHK(c, hipMemcpy(slot.data(), c->sd.seq_slot, sizeof(int) * MS, hipMemcpyDeviceToHost));
  HIPCHK(c, hipMemcpy(npre.data(), c->sd.seq_npreempt, sizeof(int) * MS, hipMemcpyDeviceToHost));
  HIPCHK(c, hipMemcpy(fver.data(), c->sd.seq_fin_version, sizeof(int) * MS, hipMemcpyDeviceToHost));
  // length-ordered: completion step, then generated length, then submission order
  std::sort(fin.begin(), fin.end(), [&](int a, int b) {
    if (comp[a] != comp[b]) return comp[a] < comp[b];
    if (glen[a] != glen[b]) return glen[a] < glen[b];
    return c->seqs[a].seq_id < c->seqs[b].seq_id;
  });
  uint64_t need_tok = 0;
  for (int i = 0; i < take; ++i) need_tok += (uint64_t)glen[fin[i]];
  if (n_recs) *n_recs = (uint32_t)take;
  if (tok_needed) *tok_needed = need_tok;
  if (!recs || (uint32_t)take > recs_cap || !tok_buf || need_tok > tok_cap)
    return fail(c, ROLLOUT_ERANGE, "output buffers too small (see n_recs / tok_needed); nothing consumed");
  // tokens and log-probs leave the device in batches: a gather kernel packs as many trajectories as the staging
  // buffers hold (always at least one: they hold max_new_tokens), then one copy per array moves the batch
  uint64_t off = 0;
  for (int i0 = 0; i0 < take;) {
    size_t fill = 0;
    int i1 = i0;
    while (i1 < take && fill + (size_t)glen[fin[i1]] <= c->hv_cap) {
      const int sidx = fin[i1];
      c->hv_rec_host[i1 - i0] = HarvestRec{sidx, c->seqs[sidx].prompt_len, glen[sidx], (int)fill};
      fill += (size_t)glen[sidx];
      ++i1;
    }
    HIPCHK(c, hipMemcpyAsync(c->hv_rec_dev, c->hv_rec_host, sizeof(HarvestRec) * (i1 - i0), hipMemcpyHostToDevice, c->stream));
    launch_harvest_gather(c->sd, c->hv_rec_dev, i1 - i0, c->hv_tok_dev, logp_buf ? c->hv_logp_dev : nullptr, c->stream);
    HIPCHK(c, hipStreamSynchronize(c->stream));
    if (fill > 0) {
      HIPCHK(c, hipMemcpy(tok_buf + off, c->hv_tok_dev, sizeof(int) * fill, hipMemcpyDeviceToHost));
      if (logp_buf) HIPCHK(c, hipMemcpy(logp_buf + off, c->hv_logp_dev, sizeof(float) * fill, hipMemcpyDeviceToHost));
    }
    off += fill;
    i0 = i1;
  }
  off = 0;
  for (int i = 0; i < take; ++i) {
    const int sidx = fin[i];
    rollout_traj& r = recs[i];
    r.seq_id = c->seqs[sidx].seq_id;
    r.slot = (uint32_t)slot[sidx];
    r.completion_step = (uint32_t)comp[sidx];
    r.gen_len = (uint32_t)glen[sidx];
    r.group_idx = (uint32_t)(c->n_groups_total + (uint64_t)(i / (int)group_size));
    r.tok_off = off;
    r.n_preempt = (uint32_t)npre[sidx];
    r.policy_version = (uint32_t)fver[sidx];
    off += glen[sidx];
    c->seqs[sidx].harvested = true;
    c->seqs[sidx].in_use = false;
    c->id2sidx.erase(c->seqs[sidx].seq_id);
    c->free_sidx.push_back(sidx);
    const int grp = c->seqs[sidx].group;
    if (grp >= 0 && --c->group_members[grp] == 0) c->free_group.push_back(grp);
  }
  // remainder stays finished-unharvested, in its sorted order; it goes through the pinned submit staging area and the
  // engine's own stream, so the boundary kernel below is ordered after it
  const int rest = nfin - take;
  int* stage = reinterpret_cast<int*>(c->sub_host);
  static_assert(sizeof(SubmitRec) >= 2 * sizeof(int), "staging area holds max_seqs + 1 ints");
  memcpy(stage, fin.data() + take, sizeof(int) * rest);
  stage[rest] = rest;
  if (rest > 0) HIPCHK(c, hipMemcpyAsync(c->sd.fin_list, stage, sizeof(int) * rest, hipMemcpyHostToDevice, c->stream));
  HIPCHK(c, hipMemcpyAsync(c->sd.sc + SC_FINCOUNT, stage + rest, sizeof(int), hipMemcpyHostToDevice, c->stream));
  c->n_harvested += take;
  c->n_groups_total += k;
  *n_groups = (uint32_t)k;
  launch_sched_boundary(c->sd, k, c->stream);   // update boundary: version += k, staleness / on-policy eviction
  TRY(sync_status(c));
  return ROLLOUT_OK;
}

int rollout_stats(rollout_ctx* c, rollout_stats_t* out) {
  if (!c || !out) return fail(c, ROLLOUT_EINVAL, "null argument");
  if (c->dead) return fail(c, ROLLOUT_EDEVICE, "context unusable after an earlier device error");
  HIPCHK(c, hipSetDevice(c->cfg.device));
  HIPCHK(c, hipStreamSynchronize(c->stream));
  unsigned long long ctr[CT_COUNT];
  int sc[SC_COUNT];
  HIPCHK(c, hipMemcpy(ctr, c->sd.ctr, sizeof(ctr), hipMemcpyDeviceToHost));
  HIPCHK(c, hipMemcpy(sc, c->sd.sc, sizeof(sc), hipMemcpyDeviceToHost));
  memset(out, 0, sizeof(*out));
  out->steps = (uint64_t)sc[SC_STEP];
  out->busy = ctr[CT_BUSY];
  out->idle = ctr[CT_IDLE];
  out->steps_q = ctr[CT_STEPS_Q];
  out->idle_q = ctr[CT_IDLE_Q];
  out->gen_tokens = ctr[CT_GEN];
  out->discarded_tokens = ctr[CT_DISCARD];
  out->prefill_tokens = ctr[CT_PREFILL];
  out->n_preempt = ctr[CT_PREEMPT];
  out->n_stale = ctr[CT_STALE];
  out->version = (uint64_t)sc[SC_VERSION];
  out->n_pages = (uint64_t)c->n_pages;
  out->max_pages_used = (uint64_t)(c->n_pages - sc[SC_MINFREE]);
  out->attn_launches = c->attn_launches;
  out->attn_kv_tokens = c->attn_kv_tokens;
  out->attn_ms = c->attn_ms;
  out->wall_ms_steps = c->wall_ms_steps;
  return ROLLOUT_OK;
}

int rollout_peek(rollout_ctx* c, uint64_t seq_id, int32_t* tok_buf, float* logp_buf, uint32_t cap, uint32_t* gen_len,
                 uint32_t* state, int32_t* slot) {
  if (!c) return ROLLOUT_EINVAL;
  if (c->dead) return fail(c, ROLLOUT_EDEVICE, "context unusable after an earlier device error");
  if (seq_id >= c->next_seq_id) return fail(c, ROLLOUT_ERANGE, "unknown seq_id");
  auto it = c->id2sidx.find(seq_id);
  if (it == c->id2sidx.end()) {   // harvested: its table entry has been recycled
    if (gen_len) *gen_len = 0;
    if (state) *state = SEQ_HARVESTED;
    if (slot) *slot = -1;
    return ROLLOUT_OK;
  }
  const int sidx = it->second;
  HIPCHK(c, hipSetDevice(c->cfg.device));
  HIPCHK(c, hipStreamSynchronize(c->stream));
  int g = 0, stt = 0, sl = -1;
  HIPCHK(c, hipMemcpy(&g, c->sd.seq_gen_len + sidx, sizeof(int), hipMemcpyDeviceToHost));
  HIPCHK(c, hipMemcpy(&stt, c->sd.seq_state + sidx, sizeof(int), hipMemcpyDeviceToHost));
  HIPCHK(c, hipMemcpy(&sl, c->sd.seq_slot + sidx, sizeof(int), hipMemcpyDeviceToHost));
  if (gen_len) *gen_len = (uint32_t)g;
  if (state) *state = (uint32_t)stt;
  if (slot) *slot = stt == SEQ_ACTIVE ? sl : -1;
  if ((tok_buf || logp_buf) && (uint32_t)g > cap) return fail(c, ROLLOUT_ERANGE, "buffer smaller than gen_len");
  if (tok_buf && g > 0)
    HIPCHK(c, hipMemcpy(tok_buf, c->sd.seq_tokens + (size_t)sidx * c->sd.tok_stride + c->seqs[sidx].prompt_len,
                        sizeof(int) * g, hipMemcpyDeviceToHost));
  if (logp_buf && g > 0)
    HIPCHK(c, hipMemcpy(logp_buf, c->sd.seq_logp + (size_t)sidx * c->sd.cap, sizeof(float) * g, hipMemcpyDeviceToHost));
  return ROLLOUT_OK;
}

int rollout_slot_pages(rollout_ctx* c, uint32_t slot, int32_t* pages, uint32_t cap, uint32_t* n) {
  if (!c || !n || slot >= (uint32_t)c->Q) return fail(c, ROLLOUT_EINVAL, "bad argument");
  if (c->dead) return fail(c, ROLLOUT_EDEVICE, "context unusable after an earlier device error");
  HIPCHK(c, hipSetDevice(c->cfg.device));
  HIPCHK(c, hipStreamSynchronize(c->stream));
  int sidx = -1, np = 0;
  HIPCHK(c, hipMemcpy(&sidx, c->sd.slot_seq + slot, sizeof(int), hipMemcpyDeviceToHost));
  HIPCHK(c, hipMemcpy(&np, c->sd.slot_npages + slot, sizeof(int), hipMemcpyDeviceToHost));
  if (sidx < 0) np = 0;
  *n = (uint32_t)np;
  if (np == 0) return ROLLOUT_OK;
  if (!pages || (uint32_t)np > cap) return fail(c, ROLLOUT_ERANGE, "buffer smaller than the page count");
  HIPCHK(c, hipMemcpy(pages, c->sd.page_table + (size_t)slot * c->max_pages, sizeof(int) * np, hipMemcpyDeviceToHost));
  return ROLLOUT_OK;
}

// ---- standalone attention ------------------------------------------------------------------------------
uint64_t rollout_attn_pool_bytes(uint32_t n_pages, uint32_t n_kv_heads, uint32_t head_dim) {
  return (uint64_t)n_pages * n_kv_heads * kv_block_bytes((int)head_dim);
}

int rollout_attn_write_kv(void* pool_dev, uint32_t n_kv_heads, uint32_t head_dim, const void* k_dev, const void* v_dev,
                          const int32_t* tok_seq_dev, const int32_t* tok_pos_dev, const int32_t* page_table_dev,
                          uint32_t max_pages, uint64_t n_tok, void* stream) {
  if (!pool_dev || !k_dev || !v_dev || !tok_seq_dev || !tok_pos_dev || !page_table_dev)
    return fail(nullptr, ROLLOUT_EINVAL, "null argument");
  if (head_dim != 128 && head_dim != 32) return fail(nullptr, ROLLOUT_EINVAL, "head_dim must be 32 or 128");
  launch_write_kv(pool_dev, (int)n_kv_heads, (int)head_dim, k_dev, v_dev, tok_seq_dev, tok_pos_dev, page_table_dev,
                  (int)max_pages, (size_t)n_tok, (hipStream_t)stream);
  return hipGetLastError() == hipSuccess ? ROLLOUT_OK : fail(nullptr, ROLLOUT_EDEVICE, "kernel launch failed");
}

static inline uint64_t align256(uint64_t x) { return (x + 255) & ~(uint64_t)255; }
struct AttnWs { uint64_t row_slot, row_pos, row_wstart, row_cnt, work, part_ml, part_acc, total; };
static AttnWs attn_ws_layout(uint32_t n, uint64_t max_work, uint32_t Hq, uint32_t d) {
  AttnWs w;
  uint64_t o = 0;
  w.row_slot = o; o = align256(o + 4ull * n);
  w.row_pos = o; o = align256(o + 4ull * n);
  w.row_wstart = o; o = align256(o + 8ull * n);
  w.row_cnt = o; o = align256(o + 4ull * n * Hq);     // n * n_kv_heads counters (n_kv_heads <= n_q_heads)
  w.work = o; o = align256(o + 16ull * max_work);
  w.part_ml = o; o = align256(o + 8ull * max_work * Hq);
  w.part_acc = o; o = align256(o + 4ull * max_work * Hq * d);
  w.total = o;
  return w;
}
uint64_t rollout_attn_workspace_bytes(uint32_t n, uint64_t total_ctx, uint32_t n_q_heads, uint32_t head_dim) {
  const uint64_t max_work = total_ctx / ATTN_CHUNK_MIN + n;
  return attn_ws_layout(n, max_work, n_q_heads, head_dim).total;
}

int rollout_attn_plan(const int32_t* ctx_len, uint32_t n, uint32_t n_q_heads, uint32_t n_kv_heads, uint32_t head_dim,
                      void* workspace_dev, uint64_t workspace_bytes, uint32_t* n_work, uint32_t* chunk_tokens) {
  if (!ctx_len || !workspace_dev || !n_work || !chunk_tokens || n == 0 || n_kv_heads == 0)
    return fail(nullptr, ROLLOUT_EINVAL, "null argument");
  uint64_t total = 0;
  for (uint32_t i = 0; i < n; ++i) {
    if (ctx_len[i] < 1) return fail(nullptr, ROLLOUT_EINVAL, "context lengths must be >= 1");
    total += (uint64_t)ctx_len[i];
  }
  const uint64_t max_work = total / ATTN_CHUNK_MIN + n;
  const int chunk = attn_pick_chunk(total, (int)n_kv_heads);
  const AttnWs w = attn_ws_layout(n, max_work, n_q_heads, head_dim);
  if (w.total > workspace_bytes) return fail(nullptr, ROLLOUT_EINVAL, "workspace too small");
  std::vector<int> rs(n), rp(n);
  std::vector<int2> ws(n);
  // full groups first (consecutive per sequence), then the shorter last groups in descending length (ties: ascending
  // sequence), so that the launch ends on its smallest items
  const int gt = ATTN_GROUP_CHUNKS * chunk;
  std::vector<int> rem_order;
  int n_full = 0;
  for (uint32_t i = 0; i < n; ++i) {
    rs[i] = (int)i;
    rp[i] = ctx_len[i] - 1;
    ws[i].x = n_full;
    n_full += ctx_len[i] / gt;
    if (ctx_len[i] % gt) rem_order.push_back((int)i);
  }
  std::stable_sort(rem_order.begin(), rem_order.end(), [&](int a, int b) { return ctx_len[a] % gt > ctx_len[b] % gt; });
  std::vector<int4> work((size_t)n_full + rem_order.size());
  for (uint32_t i = 0; i < n; ++i)
    for (int c = 0; c < ctx_len[i] / gt; ++c) work[ws[i].x + c] = make_int4((int)i, c, (int)i, ctx_len[i]);
  for (size_t k = 0; k < rem_order.size(); ++k) {
    const int i = rem_order[k];
    ws[i].y = n_full + (int)k;
    work[ws[i].y] = make_int4(i, ctx_len[i] / gt, i, ctx_len[i]);
  }
  if (work.size() > max_work) return fail(nullptr, ROLLOUT_EINVAL, "work list larger than planned");
  uint8_t* base = (uint8_t*)workspace_dev;
  if (hipMemcpy(base + w.row_slot, rs.data(), 4ull * n, hipMemcpyHostToDevice) != hipSuccess ||
      hipMemcpy(base + w.row_pos, rp.data(), 4ull * n, hipMemcpyHostToDevice) != hipSuccess ||
      hipMemcpy(base + w.row_wstart, ws.data(), 8ull * n, hipMemcpyHostToDevice) != hipSuccess ||
      hipMemset(base + w.row_cnt, 0, 4ull * n * n_q_heads) != hipSuccess ||
      hipMemcpy(base + w.work, work.data(), 16ull * work.size(), hipMemcpyHostToDevice) != hipSuccess)
    return fail(nullptr, ROLLOUT_EDEVICE, "hipMemcpy failed");
  *n_work = (uint32_t)work.size();
  *chunk_tokens = (uint32_t)chunk;
  return ROLLOUT_OK;
}

int rollout_attn_decode(const void* pool_dev, uint32_t n_q_heads, uint32_t n_kv_heads, uint32_t head_dim,
                        const void* q_dev, const int32_t* page_table_dev, uint32_t max_pages, uint32_t n, uint32_t n_work,
                        uint32_t chunk_tokens, void* out_dev, int out_fp32, void* workspace_dev, void* stream) {
  if (!pool_dev || !q_dev || !page_table_dev || !out_dev || !workspace_dev || n == 0 || n_work < n)
    return fail(nullptr, ROLLOUT_EINVAL, "null argument");
  if (chunk_tokens < 64 || chunk_tokens > ATTN_CHUNK_MAX || chunk_tokens % 64)
    return fail(nullptr, ROLLOUT_EINVAL, "chunk_tokens must be a multiple of 64 in 64..1024 (use the planned value)");
  if (n_kv_heads == 0 || n_q_heads % n_kv_heads || !attn_supported((int)head_dim, (int)(n_q_heads / n_kv_heads)))
    return fail(nullptr, ROLLOUT_EINVAL, "unsupported head_dim / query-group size");
  // row arrays and the work list sit where the plan put them (their offsets depend on n only); the partial
  // buffers are scratch of this call and are laid out for n_work items, which never exceeds the planned bound
  uint8_t* base = (uint8_t*)workspace_dev;
  const AttnWs w = attn_ws_layout(n, n_work, n_q_heads, head_dim);
  AttnArgs a;
  a.pool = pool_dev;
  a.q = q_dev;
  a.row_slot = (const int*)(base + w.row_slot);
  a.row_pos = (const int*)(base + w.row_pos);
  a.page_table = page_table_dev;
  a.max_pages = (int)max_pages;
  a.work = (const int4*)(base + w.work);
  a.row_wstart = (const int2*)(base + w.row_wstart);
  a.n_work = (int)n_work;
  a.n_rows = (int)n;
  a.Hkv = (int)n_kv_heads;
  a.part_ml = (float*)(base + w.part_ml);
  a.row_cnt = (int*)(base + w.row_cnt);
  a.part_acc = (float*)(base + w.part_acc);
  a.out = out_dev;
  a.out_fp32 = out_fp32;
  a.chunk_tokens = (int)chunk_tokens;
  launch_decode_attn(a, (int)head_dim, (int)(n_q_heads / n_kv_heads), (hipStream_t)stream);
  return hipGetLastError() == hipSuccess ? ROLLOUT_OK : fail(nullptr, ROLLOUT_EDEVICE, "kernel launch failed");
}

// ---- plain streaming kernels ---------------------------------------------------------------------------------
int rollout_stream_copy(const void* src_dev, void* dst_dev, uint64_t bytes, void* stream) {
  if (!src_dev || !dst_dev || bytes % 16) return fail(nullptr, ROLLOUT_EINVAL, "null pointer or size not a multiple of 16");
  launch_stream_copy(src_dev, dst_dev, (size_t)bytes, (hipStream_t)stream);
  return hipGetLastError() == hipSuccess ? ROLLOUT_OK : fail(nullptr, ROLLOUT_EDEVICE, "kernel launch failed");
}
int rollout_stream_read(const void* src_dev, uint64_t bytes, void* sink_dev, void* stream) {
  if (!src_dev || !sink_dev || bytes % 16) return fail(nullptr, ROLLOUT_EINVAL, "null pointer or size not a multiple of 16");
  launch_stream_read(src_dev, (size_t)bytes, sink_dev, (hipStream_t)stream);
  return hipGetLastError() == hipSuccess ? ROLLOUT_OK : fail(nullptr, ROLLOUT_EDEVICE, "kernel launch failed");
}

// ---- standalone GEMM ---------------------------------------------------------------------------------------
uint64_t rollout_gemm_packed_bytes(uint32_t N, uint32_t K) { return (uint64_t)((N + 31) / 32 * 32) * K * 2ull; }
int rollout_gemm_pack_weights(const void* w_dev, void* packed_dev, uint32_t N, uint32_t K, void* stream) {
  if (!w_dev || !packed_dev || N == 0 || K == 0) return fail(nullptr, ROLLOUT_EINVAL, "null argument");
  if (K % 64) return fail(nullptr, ROLLOUT_EINVAL, "K must be a multiple of 64");
  const uint32_t n_pad = (N + 31) / 32 * 32;
  if (n_pad > N) {   // rows past N inside the last tile: zero them, then pack the N real rows
    if (hipMemsetAsync((uint8_t*)packed_dev + (size_t)(N / 32) * 32 * K * 2, 0, (size_t)32 * K * 2, (hipStream_t)stream) != hipSuccess)
      return fail(nullptr, ROLLOUT_EDEVICE, "hipMemsetAsync failed");
  }
  launch_pack_weights(w_dev, packed_dev, N, K, (hipStream_t)stream);
  return hipGetLastError() == hipSuccess ? ROLLOUT_OK : fail(nullptr, ROLLOUT_EDEVICE, "kernel launch failed");
}
uint64_t rollout_gemm_workspace_bytes(uint32_t M, uint32_t N, uint32_t K) {
  return (uint64_t)gemm_pick_splits((int)M, (int)N, (int)K) * M * N * 4ull + 256;
}
int rollout_gemm_bf16(const void* a_dev, const void* w_packed_dev, float* c_dev, uint32_t M, uint32_t N, uint32_t K,
                      void* workspace_dev, uint64_t workspace_bytes, void* stream) {
  if (!a_dev || !w_packed_dev || !c_dev || M == 0 || N == 0 || K == 0) return fail(nullptr, ROLLOUT_EINVAL, "null argument");
  if (K % 64) return fail(nullptr, ROLLOUT_EINVAL, "K must be a multiple of 64");
  if (K > (1u << 20) || M > (1u << 24) || N > (1u << 24))   // byte offsets inside one row block / tile row are 32-bit
    return fail(nullptr, ROLLOUT_EINVAL, "matrix too large (K <= 2^20, M and N <= 2^24)");
  const int S = gemm_pick_splits((int)M, (int)N, (int)K);
  if (S == 1) {
    launch_gemm(a_dev, w_packed_dev, c_dev, (int)M, (int)N, (int)K, 1, (hipStream_t)stream);
  } else {
    if (!workspace_dev || workspace_bytes < (uint64_t)S * M * N * 4ull) return fail(nullptr, ROLLOUT_EINVAL, "workspace too small");
    launch_gemm(a_dev, w_packed_dev, (float*)workspace_dev, (int)M, (int)N, (int)K, S, (hipStream_t)stream);
    launch_reduce_splits((const float*)workspace_dev, c_dev, (size_t)M * N, S, (hipStream_t)stream);
  }
  return hipGetLastError() == hipSuccess ? ROLLOUT_OK : fail(nullptr, ROLLOUT_EDEVICE, "kernel launch failed");
}


// ---- the projection GEMM for callers that cannot allocate (static scratch: see static_scratch above) ----------
uint64_t rollout_gemm_static_scratch_bytes(void) { return GEMM_STATIC_SCRATCH_BYTES; }

int rollout_gemm_bf16_static(const void* a_dev, const void* w_packed_dev, float* c_dev, uint32_t M, uint32_t N, uint32_t K,
                             void* stream) {
  if (!a_dev || !w_packed_dev || !c_dev || M == 0 || N == 0 || K == 0) return fail(nullptr, ROLLOUT_EINVAL, "null argument");
  if (K % 64) return fail(nullptr, ROLLOUT_EINVAL, "K must be a multiple of 64");
  if (K > (1u << 20) || M > (1u << 24) || N > (1u << 24))
    return fail(nullptr, ROLLOUT_EINVAL, "matrix too large (K <= 2^20, M and N <= 2^24)");
  const int S = gemm_pick_splits((int)M, (int)N, (int)K);
  if (S == 1) {
    launch_gemm(a_dev, w_packed_dev, c_dev, (int)M, (int)N, (int)K, 1, (hipStream_t)stream);
  } else {
    const uint64_t need = (uint64_t)S * M * N * 4ull;
    if (need > GEMM_STATIC_SCRATCH_BYTES)
      return fail(nullptr, ROLLOUT_ERANGE,
                  "split-K partial sums of this shape (" + std::to_string(need) + " bytes) exceed the library's static scratch (" +
                      std::to_string(GEMM_STATIC_SCRATCH_BYTES) + " bytes): use rollout_gemm_bf16 with a workspace");
    void* part = nullptr;
    TRY(static_scratch(&part));
    // every split writes all M x N of its partial sums, so nothing has to start at zero
    launch_gemm(a_dev, w_packed_dev, (float*)part, (int)M, (int)N, (int)K, S, (hipStream_t)stream);
    launch_reduce_splits((const float*)part, c_dev, (size_t)M * N, S, (hipStream_t)stream);
  }
  return hipGetLastError() == hipSuccess ? ROLLOUT_OK : fail(nullptr, ROLLOUT_EDEVICE, "kernel launch failed");
}

int rollout_gemm_swiglu_bf16(const void* a_dev, const void* w_packed_dev, void* act_dev, uint32_t M, uint32_t F, uint32_t K,
                             void* stream) {
  if (!a_dev || !w_packed_dev || !act_dev || M == 0 || F == 0 || K == 0) return fail(nullptr, ROLLOUT_EINVAL, "null argument");
  if (K % 64 || F % 16) return fail(nullptr, ROLLOUT_EINVAL, "K must be a multiple of 64 and F of 16");
  if (K > (1u << 20) || M > (1u << 24) || F > (1u << 23)) return fail(nullptr, ROLLOUT_EINVAL, "matrix too large");
  launch_gemm_swiglu(a_dev, w_packed_dev, act_dev, (int)M, (int)(2 * F), (int)K, (hipStream_t)stream);
  return hipGetLastError() == hipSuccess ? ROLLOUT_OK : fail(nullptr, ROLLOUT_EDEVICE, "kernel launch failed");
}

const char* rollout_gemm_kernel_name(uint32_t M, uint32_t N, uint32_t K, uint32_t splits, int swiglu) {
  if (M == 0 || N == 0 || K == 0 || K % 64) return "";
  const int S = swiglu ? 1 : splits ? (int)splits : gemm_pick_splits((int)M, (int)N, (int)K);
  return gemm_kernel_name((int)M, (int)N, (int)K, S, swiglu ? 1 : 0);
}
uint32_t rollout_gemm_splits(uint32_t M, uint32_t N, uint32_t K) {
  if (M == 0 || N == 0 || K == 0 || K % 64) return 0;
  return (uint32_t)gemm_pick_splits((int)M, (int)N, (int)K);
}

}  // extern "C"
