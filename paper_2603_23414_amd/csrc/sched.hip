// Device side of the length-aware rollout scheduler (Sec. 3.1-3.3): admission / refill of free slots,
// token append + finish detection + eviction, page growth with preemption, update-boundary handling,
// and the order-preserving compaction of running slots into the decode row list.
//
// Every kernel is ONE workgroup of 1024 threads (thread = slot, max_slots <= 1024).  Anything whose order
// is observable (slot choice, page pops/pushes, finished list, queue) is produced by exclusive scans in
// ascending slot order or by a single thread, never by atomics, so the outcome is bit-reproducible.
#include "common.h"
#include "kernels.h"

__device__ __forceinline__ int block_scan_excl(int v, int* total, int* sh /* >= 17 ints */) {
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  int inc = v;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const int n = __shfl_up(inc, o, 64);
    if (lane >= o) inc += n;
  }
  if (lane == 63) sh[w] = inc;
  __syncthreads();
  if (w == 0) {
    const int x = lane < 16 ? sh[lane] : 0;
    int xi = x;
#pragma unroll
    for (int o = 1; o < 16; o <<= 1) {
      const int n = __shfl_up(xi, o, 64);
      if (lane >= o) xi += n;
    }
    if (lane < 16) sh[lane] = xi - x;
    if (lane == 15) sh[16] = xi;
  }
  __syncthreads();
  const int res = inc - v + sh[w];
  *total = sh[16];
  __syncthreads();
  return res;
}

__device__ __forceinline__ void q_push_front(const SchedDev& d, int sidx) {
  const int head = (d.sc[SC_QHEAD] - 1) & d.qmask;
  d.q_ring[head] = sidx;
  d.sc[SC_QHEAD] = head;
  d.sc[SC_QCOUNT] += 1;
}

// Rebuild the decode row list (ascending slot order = order-preserving compaction) and the attention work
// list for the next step, then publish the status block.  Called by all threads at the end of a kernel.
__device__ void rebuild_rows_and_status(const SchedDev& d, int* sh, int* big /* 1024 ints of LDS */, int r_this_step,
                                        int n_fin_step, int n_pre_step, int n_adm) {
  const int t = threadIdx.x;
  int sidx = -1, pos = 0;
  if (t < d.Q && (sidx = d.slot_seq[t]) >= 0) pos = d.seq_prompt_len[sidx] + d.seq_gen_len[sidx] - 1;
  // sum of contexts (chunk choice and byte accounting): reduced through the scan helper on 16-bit halves
  int lo_tot, hi_tot;
  block_scan_excl(sidx >= 0 ? ((pos + 1) & 0xFFFF) : 0, &lo_tot, sh);
  block_scan_excl(sidx >= 0 ? ((pos + 1) >> 16) : 0, &hi_tot, sh);
  const unsigned long long ctx_total = (unsigned long long)lo_tot + ((unsigned long long)hi_tot << 16);
  const int chunk = attn_pick_chunk(ctx_total, d.Hkv);
  // work items: a row's full groups (ATTN_GROUP_CHUNKS chunks each) go to the front of the list, its last, shorter group
  // to the back part, which is ordered by descending length (ties: ascending slot) -- the dispatcher hands out
  // workgroups in list order, so the launch ends on its smallest items instead of on whatever the last slots hold
  const int gt = ATTN_GROUP_CHUNKS * chunk;
  const int nfull = sidx >= 0 ? (pos + 1) / gt : 0;
  const int rem = sidx >= 0 ? (pos + 1) % gt : 0;
  big[t] = rem;
  int n_active, n_full;
  const int rank = block_scan_excl(sidx >= 0 ? 1 : 0, &n_active, sh);
  const int fstart = block_scan_excl(nfull, &n_full, sh);   // (its barriers also publish big[])
  int n_rem = 0, rrank = 0;
  for (int j = 0; j < d.Q; ++j) {
    const int rj = big[j];
    n_rem += rj > 0;
    rrank += rj > rem || (rj == rem && rj > 0 && j < t);
  }
  const int n_work = n_full + n_rem;
  if (sidx >= 0) {
    d.row_slot[rank] = t;
    d.row_pos[rank] = pos;
    d.row_tok[rank] = d.seq_tokens[(size_t)sidx * d.tok_stride + pos];
    d.row_wstart[rank] = make_int2(fstart, n_full + rrank);
    for (int c = 0; c < nfull; ++c) d.work[fstart + c] = make_int4(rank, c, t, pos + 1);
    if (rem > 0) d.work[n_full + rrank] = make_int4(rank, nfull, t, pos + 1);
  }
  __syncthreads();                                          // big[] is the caller's scratch again
  if (t == 0) {
    d.sc[SC_NDEC] = n_active;
    d.sc[SC_NPRE] = 0;
    d.sc[SC_NWORK] = n_work;
    const unsigned long long ctx = ctx_total;
    int* s = d.status;
    s[STAT_STEP] = d.sc[SC_STEP];
    s[STAT_R] = r_this_step;
    s[STAT_NACTIVE] = n_active;
    s[STAT_FIN] = d.sc[SC_FINCOUNT];
    s[STAT_QUEUED] = d.sc[SC_QCOUNT];
    s[STAT_FREE] = d.sc[SC_NFREE];
    s[STAT_NADM] = n_adm;
    s[STAT_NFIN_STEP] = n_fin_step;
    s[STAT_NPRE_STEP] = n_pre_step;
    s[STAT_NDEC_NEXT] = n_active;
    s[STAT_NWORK_NEXT] = n_work;
    s[STAT_CTX_LO] = (int)(ctx & 0xFFFFFFFFull);
    s[STAT_CTX_HI] = (int)(ctx >> 32);
    s[STAT_VERSION] = d.sc[SC_VERSION];
    s[STAT_CHUNK] = chunk;
  }
}

// Release the slot and the pages of every flagged slot, ascending slot order, pages in logical order.  Shared
// prompt pages stay with the group while another running rollout reads them; the last one to leave (the highest
// flagged slot of the group, if that empties it) returns them, ahead of its own.  `grp_of` is 1024 ints of LDS.
__device__ void release_flagged(const SchedDev& d, int* sh, int* grp_of, bool flag) {
  const int t = threadIdx.x;
  int g = -1;
  if (flag) g = d.seq_group[d.slot_seq[t]];
  grp_of[t] = g;
  __syncthreads();
  int first = 0, leavers = 0;
  bool highest = true;
  if (g >= 0) {
    for (int j = 0; j < d.Q; ++j)
      if (grp_of[j] == g) {
        ++leavers;
        if (j > t) highest = false;
      }
    const bool last = highest && d.grp_ref[g] == leavers;
    if (!last) first = d.grp_nshared[g];
  }
  const int npg = flag ? d.slot_npages[t] - first : 0;
  int freed;
  const int off = block_scan_excl(npg, &freed, sh);
  const int n_free0 = d.sc[SC_NFREE];
  __syncthreads();                                 // every grp_ref read above precedes the update below
  if (flag) {
    for (int j = 0; j < npg; ++j) d.free_stack[n_free0 + off + j] = d.page_table[(size_t)t * d.max_pages + first + j];
    d.slot_seq[t] = -1;
    d.slot_npages[t] = 0;
    if (g >= 0 && highest) d.grp_ref[g] -= leavers;
  }
  __syncthreads();
  if (t == 0) d.sc[SC_NFREE] = n_free0 + freed;
  __syncthreads();
}

// Phase A: refill free slots from the queue head (lowest slot first; FIFO head only; pages for the prefix
// plus the token it will emit; a reserve keeps this step's page growth from failing).
__global__ __launch_bounds__(1024) void k_sched_admit(SchedDev d) {
  __shared__ int sh[20];
  __shared__ int adm_slot[1024], adm_need[1024], adm_start[1024], adm_grp[1024], adm_first[1024];
  __shared__ int n_adm_sh;
  const int t = threadIdx.x;
  int need = 0, act = 0;
  if (t < d.Q) {
    const int sidx = d.slot_seq[t];
    if (sidx >= 0) {
      act = 1;
      const int next_pos = d.seq_prompt_len[sidx] + d.seq_gen_len[sidx] - 1;
      need = ((next_pos + 1) >> 4) >= d.slot_npages[t];
    }
  }
  int reserve, n_active;
  block_scan_excl(need, &reserve, sh);
  block_scan_excl(act, &n_active, sh);
  if (t == 0) {
    int n_adm = 0, cursor = 0, n_free = d.sc[SC_NFREE], qh = d.sc[SC_QHEAD], qc = d.sc[SC_QCOUNT];
    unsigned long long pf_tokens = 0;
    d.sc[SC_ADMIT_RAN] = 1;
    d.sc[SC_QNE] = qc > 0;
    const bool may = !(d.mode == 2 && n_active > 0);
    const int ver = d.sc[SC_VERSION];
    while (may && qc > 0) {
      while (cursor < d.Q && d.slot_seq[cursor] >= 0) ++cursor;
      if (cursor >= d.Q) break;
      const int sidx = d.q_ring[qh];
      const int n = d.seq_prompt_len[sidx] + d.seq_gen_len[sidx];
      const int total = (n + 1 + PAGE_TOKENS - 1) / PAGE_TOKENS;
      // a running sibling's prompt pages are reused: only the private tail is allocated and prefilled
      const int g = d.seq_group[sidx];
      const int shared = (g >= 0 && d.grp_ref[g] > 0) ? d.grp_nshared[g] : 0;
      const int pages = total - shared;
      if (n_free < pages + reserve) break;
      qh = (qh + 1) & d.qmask;
      --qc;
      d.slot_seq[cursor] = sidx;
      d.slot_npages[cursor] = total;
      d.seq_state[sidx] = SEQ_ACTIVE;
      d.seq_slot[sidx] = cursor;
      d.seq_kv_version[sidx] = shared ? d.grp_version[g] : ver;   // a cache is as old as its shared part
      if (g >= 0) {
        if (!shared) d.grp_version[g] = ver;
        d.grp_ref[g] += 1;
      }
      adm_slot[n_adm] = cursor;
      adm_need[n_adm] = pages;
      adm_start[n_adm] = n_free;
      adm_grp[n_adm] = g;
      adm_first[n_adm] = shared;
      n_free -= pages;
      pf_tokens += n - shared * PAGE_TOKENS;
      int* desc = d.status + STAT_HDR + STAT_ADM_INTS * n_adm;
      desc[0] = cursor;
      desc[1] = sidx;
      desc[2] = n;
      desc[3] = shared * PAGE_TOKENS;
      ++n_adm;
      ++cursor;
    }
    d.sc[SC_NFREE] = n_free;
    d.sc[SC_QHEAD] = qh;
    d.sc[SC_QCOUNT] = qc;
    d.sc[SC_NPRE] = n_adm;
    if (n_free < d.sc[SC_MINFREE]) d.sc[SC_MINFREE] = n_free;
    d.ctr[CT_PREFILL] += pf_tokens;
    d.status[STAT_NADM] = n_adm;
    d.status[STAT_QUEUED] = qc;
    d.status[STAT_FREE] = n_free;
    n_adm_sh = n_adm;
  }
  __syncthreads();
  const int n_adm = n_adm_sh;
  const int n_dec = d.sc[SC_NDEC];
  for (int a = 0; a < n_adm; ++a) {
    const int g = adm_grp[a], first = adm_first[a];
    int* row = d.page_table + (size_t)adm_slot[a] * d.max_pages;
    for (int j = t; j < adm_need[a]; j += 1024) row[first + j] = d.free_stack[adm_start[a] - 1 - j];
    if (g >= 0) {                                     // uniform
      int* gp = d.grp_pages + (size_t)g * d.max_shared;
      if (first > 0) {
        for (int j = t; j < first; j += 1024) row[j] = gp[j];
      } else {                                        // first of its group to run: its leading pages become the shared set
        const int ns = d.grp_nshared[g];
        for (int j = t; j < ns; j += 1024) gp[j] = d.free_stack[adm_start[a] - 1 - j];
      }
      __syncthreads();                                // a later admission of this launch may attach to them
    }
  }
  if (t < n_adm) d.row_slot[n_dec + t] = adm_slot[t];
}

// Phases C, D, E: emit one token per row, evict finished rollouts, grow pages (preempting if the pool is
// empty), account the step, rebuild the row list for the next step.
__global__ __launch_bounds__(1024) void k_sched_emit(SchedDev d) {
  __shared__ int sh[20];
  __shared__ int slot_row[1024], grp_of[1024];
  const int t = threadIdx.x;
  const int n_dec = d.sc[SC_NDEC], n_pre = d.sc[SC_NPRE];
  const int n_rows = n_dec + n_pre;
  const int step = d.sc[SC_STEP];
  slot_row[t] = -1;
  __syncthreads();
  if (t < n_rows) slot_row[d.row_slot[t]] = t;
  __syncthreads();

  // ---- C: emit ----------------------------------------------------------------------------------
  int fin = 0;
  int my_sidx = -1;
  if (t < d.Q && slot_row[t] >= 0) {
    const int r = slot_row[t];
    const int sidx = d.slot_seq[t];
    my_sidx = sidx;
    int g = d.seq_gen_len[sidx];
    const int P = d.seq_prompt_len[sidx];
    const int tgt = d.seq_target_len[sidx];
    const bool forced = tgt > 0 && g + 1 == tgt;
    int tok = forced ? d.eos_id : (d.no_model ? 0 : d.row_argmax[r]);
    if (d.forced_tok && d.forced_tok[t] >= 0) tok = d.forced_tok[t];
    // log-prob under the distribution that was sampled: scaled logit of the emitted token minus the log-sum-exp.  The
    // candidate's and the EOS column's scaled logits come with the row statistics; only a teacher-forced token needs
    // the logits row itself (that path keeps it).
    float lp = 0.f;
    if (!d.no_model) {
      const float lscale = d.inv_temp > 0.f ? d.inv_temp : 1.f;
      const bool taught = d.forced_tok && d.forced_tok[t] >= 0;
      const float z = taught ? d.logits[(size_t)r * d.V + tok] * lscale : forced ? d.row_zeos[r] : d.row_ztok[r];
      lp = z - d.row_lse[r];
    }
    d.seq_tokens[(size_t)sidx * d.tok_stride + P + g] = tok;
    d.seq_logp[(size_t)sidx * d.cap + g] = lp;
    ++g;
    d.seq_gen_len[sidx] = g;
    fin = forced || (d.eos_mode == 1 && tok == d.eos_id) || g >= d.cap;
  }
  int n_fin;
  const int fin_rank = block_scan_excl(fin, &n_fin, sh);
  const int fin0 = d.sc[SC_FINCOUNT];
  if (fin) {
    d.fin_list[fin0 + fin_rank] = my_sidx;
    d.seq_completion[my_sidx] = step;
    d.seq_fin_version[my_sidx] = d.sc[SC_VERSION];
    d.seq_state[my_sidx] = SEQ_FINISHED;
  }
  release_flagged(d, sh, grp_of, fin != 0);
  if (t == 0) d.sc[SC_FINCOUNT] = fin0 + n_fin;

  // ---- D: page growth ---------------------------------------------------------------------------
  int grow = 0;
  if (t < d.Q) {
    const int sidx = d.slot_seq[t];
    if (sidx >= 0) {
      const int next_pos = d.seq_prompt_len[sidx] + d.seq_gen_len[sidx] - 1;
      grow = (next_pos >> 4) >= d.slot_npages[t];
    }
  }
  int n_grow;
  const int grow_rank = block_scan_excl(grow, &n_grow, sh);
  const int n_free = d.sc[SC_NFREE];
  __syncthreads();
  int n_preempted = 0;
  if (n_grow <= n_free) {
    if (grow) {
      d.page_table[(size_t)t * d.max_pages + d.slot_npages[t]] = d.free_stack[n_free - 1 - grow_rank];
      d.slot_npages[t] += 1;
    }
    if (t == 0) d.sc[SC_NFREE] = n_free - n_grow;
  } else if (t == 0) {
    // pool exhausted: sequential, preempting the running rollout with the fewest generated tokens
    // (ties: the latest submission); it keeps its tokens and waits at the queue front for re-prefill
    int nf = n_free;
    for (int i = 0; i < d.Q; ++i) {
      const int sidx = d.slot_seq[i];
      if (sidx < 0) continue;
      const int next_pos = d.seq_prompt_len[sidx] + d.seq_gen_len[sidx] - 1;
      if ((next_pos >> 4) < d.slot_npages[i]) continue;
      while (nf == 0) {
        int vs = -1, vg = 0;
        unsigned long long vid = 0;
        for (int j = 0; j < d.Q; ++j) {
          const int s2 = d.slot_seq[j];
          if (s2 < 0) continue;
          const int g2 = d.seq_gen_len[s2];
          const unsigned long long id2 = d.seq_id[s2];
          if (vs < 0 || g2 < vg || (g2 == vg && id2 > vid)) { vs = j; vg = g2; vid = id2; }
        }
        const int s2 = d.slot_seq[vs];
        const int grp = d.seq_group[s2];
        int first = 0;                                   // shared prompt pages stay while a sibling reads them
        if (grp >= 0 && (d.grp_ref[grp] -= 1) > 0) first = d.grp_nshared[grp];
        for (int j = first; j < d.slot_npages[vs]; ++j) d.free_stack[nf++] = d.page_table[(size_t)vs * d.max_pages + j];
        d.slot_seq[vs] = -1;
        d.slot_npages[vs] = 0;
        d.seq_state[s2] = SEQ_QUEUED;
        d.seq_npreempt[s2] += 1;
        q_push_front(d, s2);
        ++n_preempted;
      }
      if (d.slot_seq[i] == sidx) {
        d.page_table[(size_t)i * d.max_pages + d.slot_npages[i]] = d.free_stack[--nf];
        d.slot_npages[i] += 1;
      }
    }
    d.sc[SC_NFREE] = nf;
    d.ctr[CT_PREEMPT] += n_preempted;
  }
  __syncthreads();

  // ---- E: accounting (eq. 4 with one step as the time unit) ---------------------------------------
  if (t == 0) {
    const int qne = d.sc[SC_ADMIT_RAN] ? d.sc[SC_QNE] : (d.sc[SC_QCOUNT] - n_preempted > 0);
    d.sc[SC_ADMIT_RAN] = 0;
    d.ctr[CT_BUSY] += n_rows;
    d.ctr[CT_IDLE] += d.Q - n_rows;
    if (qne) {
      d.ctr[CT_STEPS_Q] += 1;
      d.ctr[CT_IDLE_Q] += d.Q - n_rows;
    }
    d.ctr[CT_GEN] += n_rows;
    if (d.sc[SC_NFREE] < d.sc[SC_MINFREE]) d.sc[SC_MINFREE] = d.sc[SC_NFREE];
    d.sc[SC_STEP] = step + 1;
    d.status[STAT_NPRE_STEP] = n_preempted;
  }
  __syncthreads();
  const int n_pre_step = d.status[STAT_NPRE_STEP];
  const int n_adm = n_pre;
  rebuild_rows_and_status(d, sh, grp_of, n_rows, n_fin, n_pre_step, n_adm);
  if (t == 0) d.status[STAT_STEP] = step;
}

// Update boundary after a harvest of n_groups groups: version += n_groups; partial mode releases caches
// older than max_staleness (tokens kept, re-prefilled later); on-policy mode terminates every running
// rollout and discards its tokens.  Evicted rollouts go to the queue front in ascending seq_id.
__global__ __launch_bounds__(1024) void k_sched_boundary(SchedDev d, int n_groups) {
  __shared__ int sh[20];
  __shared__ int grp_of[1024];
  __shared__ unsigned long long ids[1024];
  const int t = threadIdx.x;
  const int ver = d.sc[SC_VERSION] + n_groups;
  int sidx = -1;
  bool out = false;
  if (t < d.Q && (sidx = d.slot_seq[t]) >= 0) {
    if (d.mode == 1) out = true;
    else if (d.max_staleness >= 0) out = ver - d.seq_kv_version[sidx] > d.max_staleness;
  }
  ids[t] = out ? d.seq_id[sidx] : ~0ull;
  __syncthreads();
  int n_out;
  block_scan_excl(out ? 1 : 0, &n_out, sh);
  int rank = 0;
  unsigned long long disc = 0;
  if (out) {
    const unsigned long long me = ids[t];
    for (int j = 0; j < d.Q; ++j) rank += ids[j] < me;
    d.seq_state[sidx] = SEQ_QUEUED;
    if (d.mode == 1) {
      disc = d.seq_gen_len[sidx];
      d.seq_gen_len[sidx] = 0;
    }
  }
  release_flagged(d, sh, grp_of, out);
  const int head0 = d.sc[SC_QHEAD];
  __syncthreads();
  const int new_head = (head0 - n_out) & d.qmask;
  if (out) d.q_ring[(new_head + rank) & d.qmask] = sidx;
  // discarded-token total
  int dl, dh;
  block_scan_excl((int)(disc & 0xFFFF), &dl, sh);
  block_scan_excl((int)(disc >> 16), &dh, sh);
  if (t == 0) {
    d.sc[SC_VERSION] = ver;
    d.sc[SC_QHEAD] = new_head;
    d.sc[SC_QCOUNT] += n_out;
    if (d.mode == 1) d.ctr[CT_DISCARD] += (unsigned long long)dl + ((unsigned long long)dh << 16);
    else d.ctr[CT_STALE] += n_out;
  }
  __syncthreads();
  rebuild_rows_and_status(d, sh, grp_of, 0, 0, 0, 0);
}

// Feed prompts: one block per new sequence copies its record and prompt; the last step appends to the queue.
__global__ __launch_bounds__(256) void k_sched_submit_copy(SchedDev d, const SubmitRec* __restrict__ recs,
                                                           const int* __restrict__ tok_staging) {
  const SubmitRec r = recs[blockIdx.x];
  for (int i = threadIdx.x; i < r.prompt_len; i += 256)
    d.seq_tokens[(size_t)r.sidx * d.tok_stride + i] = tok_staging[r.tok_off + i];
  if (threadIdx.x == 0) {
    d.seq_prompt_len[r.sidx] = r.prompt_len;
    d.seq_target_len[r.sidx] = r.target_len;
    d.seq_gen_len[r.sidx] = 0;
    d.seq_state[r.sidx] = SEQ_QUEUED;
    d.seq_slot[r.sidx] = -1;
    d.seq_completion[r.sidx] = -1;
    d.seq_kv_version[r.sidx] = 0;
    d.seq_fin_version[r.sidx] = 0;
    d.seq_npreempt[r.sidx] = 0;
    d.seq_id[r.sidx] = r.seq_id;
    d.seq_group[r.sidx] = r.group;
    if (r.group >= 0) {           // every sibling writes the same values
      d.grp_nshared[r.group] = r.nshared;
      d.grp_ref[r.group] = 0;
      d.grp_version[r.group] = 0;
    }
  }
}
__global__ void k_sched_submit_enqueue(SchedDev d, const SubmitRec* __restrict__ recs, int n) {
  if (threadIdx.x != 0 || blockIdx.x != 0) return;
  const int head = d.sc[SC_QHEAD];
  int qc = d.sc[SC_QCOUNT];
  for (int i = 0; i < n; ++i) d.q_ring[(head + qc++) & d.qmask] = recs[i].sidx;
  d.sc[SC_QCOUNT] = qc;
  d.status[STAT_QUEUED] = qc;
}

__global__ __launch_bounds__(1024) void k_sched_init(SchedDev d) {
  for (int i = threadIdx.x; i < d.Q; i += 1024) {
    d.slot_seq[i] = -1;
    d.slot_npages[i] = 0;
  }
  if (threadIdx.x < SC_COUNT) d.sc[threadIdx.x] = 0;
  if (threadIdx.x < CT_COUNT) d.ctr[threadIdx.x] = 0;
  __syncthreads();
  if (threadIdx.x == 0) {
    d.sc[SC_NFREE] = d.n_pages;
    d.sc[SC_MINFREE] = d.n_pages;
    for (int i = 0; i < STAT_HDR; ++i) d.status[i] = 0;
    d.status[STAT_FREE] = d.n_pages;
  }
}

// Token rows of a prefill pass: row = one prompt (or already generated) token of an admitted sequence.
__global__ __launch_bounds__(256) void k_prefill_rows(SchedDev d, const PrefillDesc* __restrict__ descs,
                                                      int* __restrict__ row_slot, int* __restrict__ row_pos,
                                                      int* __restrict__ row_tok) {
  const PrefillDesc p = descs[blockIdx.x];
  for (int i = threadIdx.x; i < p.n_tok; i += 256) {
    const int row = p.row_begin + i;
    row_slot[row] = p.slot;
    row_pos[row] = p.pos_begin + i;
    row_tok[row] = d.seq_tokens[(size_t)p.sidx * d.tok_stride + p.pos_begin + i];
  }
}

// Harvest: pack the generated tokens and log-probs of a batch of finished rollouts into contiguous staging buffers
// (one workgroup per rollout), so that the host needs one copy per array instead of two per trajectory.
__global__ __launch_bounds__(256) void k_harvest_gather(SchedDev d, const HarvestRec* __restrict__ recs,
                                                        int* __restrict__ tok_out, float* __restrict__ logp_out) {
  const HarvestRec r = recs[blockIdx.x];
  const int* src = d.seq_tokens + (size_t)r.sidx * d.tok_stride + r.prompt_len;
  const float* lsrc = d.seq_logp + (size_t)r.sidx * d.cap;
  for (int i = threadIdx.x; i < r.gen_len; i += 256) {
    tok_out[r.off + i] = src[i];
    if (logp_out) logp_out[r.off + i] = lsrc[i];
  }
}
void launch_harvest_gather(const SchedDev& d, const HarvestRec* recs, int n, int* tok_out, float* logp_out,
                           hipStream_t st) {
  if (n > 0) hipLaunchKernelGGL(k_harvest_gather, dim3(n), dim3(256), 0, st, d, recs, tok_out, logp_out);
}

void launch_sched_admit(const SchedDev& d, hipStream_t st) { hipLaunchKernelGGL(k_sched_admit, dim3(1), dim3(1024), 0, st, d); }
void launch_sched_emit(const SchedDev& d, hipStream_t st) { hipLaunchKernelGGL(k_sched_emit, dim3(1), dim3(1024), 0, st, d); }
void launch_sched_boundary(const SchedDev& d, int n_groups, hipStream_t st) {
  hipLaunchKernelGGL(k_sched_boundary, dim3(1), dim3(1024), 0, st, d, n_groups);
}
void launch_sched_submit(const SchedDev& d, const SubmitRec* recs, const int* tok_staging, int n, hipStream_t st) {
  if (n <= 0) return;
  hipLaunchKernelGGL(k_sched_submit_copy, dim3(n), dim3(256), 0, st, d, recs, tok_staging);
  hipLaunchKernelGGL(k_sched_submit_enqueue, dim3(1), dim3(64), 0, st, d, recs, n);
}
void launch_sched_init(const SchedDev& d, hipStream_t st) { hipLaunchKernelGGL(k_sched_init, dim3(1), dim3(1024), 0, st, d); }
void launch_prefill_rows(const SchedDev& d, const PrefillDesc* descs, int n_desc, int* row_slot, int* row_pos,
                         int* row_tok, hipStream_t st) {
  if (n_desc > 0) hipLaunchKernelGGL(k_prefill_rows, dim3(n_desc), dim3(256), 0, st, d, descs, row_slot, row_pos, row_tok);
}
