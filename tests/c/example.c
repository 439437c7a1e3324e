/* A complete rollout job through the C ABI alone (no Python, no torch): a tiny randomly initialised policy, eight
 * prompts with pinned response lengths, steps until everything has drained, harvest in groups of three.
 * Checks what must hold whatever the weights are: every rollout comes back exactly once with its pinned length and
 * the end-of-sequence token last, groups are ordered by (completion step, length, id), log-probs are <= 0, and the
 * eq.-4 counters add up.  Exit status 0 = all checks passed. */
#include <math.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "rollout.h"

#define CHECK(cond)                                                         \
  do {                                                                      \
    if (!(cond)) {                                                          \
      fprintf(stderr, "check failed at line %d: %s\n", __LINE__, #cond);    \
      return 1;                                                             \
    }                                                                       \
  } while (0)
#define CALL(expr)                                                                        \
  do {                                                                                    \
    int rc_ = (expr);                                                                     \
    if (rc_ != ROLLOUT_OK) {                                                              \
      fprintf(stderr, "%s -> %d: %s\n", #expr, rc_, rollout_last_error(ctx));             \
      return 1;                                                                           \
    }                                                                                     \
  } while (0)

static uint64_t lcg_state = 12345;
static float lcg_normalish(void) { /* sum of four uniforms, centred: close enough to a bell for random weights */
  float s = 0.f;
  int i;
  for (i = 0; i < 4; ++i) {
    lcg_state = lcg_state * 6364136223846793005ull + 1442695040888963407ull;
    s += (float)((lcg_state >> 40) & 0xFFFFFF) / 16777216.0f;
  }
  return (s - 2.0f) * 1.7f;
}

int main(void) {
  enum { NL = 2, D = 128, HQ = 4, HKV = 4, HD = 32, F = 256, V = 300, NPROMPT = 8, PLEN = 20, CAP = 24, Q = 4, G = 3 };
  rollout_ctx* ctx = NULL;
  rollout_cfg cfg;
  size_t n_w, i;
  float* w;
  int32_t tokens[NPROMPT * PLEN];
  uint32_t offsets[NPROMPT + 1], target[NPROMPT];
  uint64_t first = 99;
  int seen[NPROMPT] = {0};
  uint32_t harvested = 0, groups_total = 0;
  rollout_stats_t st;

  memset(&cfg, 0, sizeof cfg);
  cfg.n_layers = NL; cfg.d_model = D; cfg.n_q_heads = HQ; cfg.n_kv_heads = HKV; cfg.head_dim = HD; cfg.d_ffn = F;
  cfg.vocab = V; cfg.rms_eps = 1e-5f; cfg.rope_theta = 1e4f; cfg.weight_dtype = 0; cfg.max_slots = Q;
  cfg.page_tokens = 16; cfg.max_prompt_len = PLEN; cfg.max_new_tokens = CAP; cfg.max_seqs = NPROMPT;
  cfg.eos_id = V - 1; cfg.eos_mode = ROLLOUT_EOS_FORCED_ONLY; cfg.mode = ROLLOUT_MODE_PARTIAL; cfg.max_staleness = -1;

  /* blob layout: embed, per layer {attn_norm, wq, wk, wv, wo, ffn_norm, w_gate, w_up, w_down}, final_norm, lm_head */
  n_w = (size_t)V * D + (size_t)NL * (D + (size_t)(HQ + 2 * HKV) * HD * D + (size_t)D * HQ * HD + D + 3 * (size_t)F * D) + D + (size_t)V * D;
  w = (float*)malloc(n_w * sizeof(float));
  CHECK(w != NULL);
  {
    size_t o = 0, l, k;
    for (k = 0; k < (size_t)V * D; ++k) w[o++] = 0.02f * lcg_normalish();
    for (l = 0; l < NL; ++l) {
      for (k = 0; k < D; ++k) w[o++] = 1.0f;
      for (k = 0; k < (size_t)(HQ + 2 * HKV) * HD * D + (size_t)D * HQ * HD; ++k) w[o++] = 0.02f * lcg_normalish();
      for (k = 0; k < D; ++k) w[o++] = 1.0f;
      for (k = 0; k < 3 * (size_t)F * D; ++k) w[o++] = 0.02f * lcg_normalish();
    }
    for (k = 0; k < D; ++k) w[o++] = 1.0f;
    for (k = 0; k < (size_t)V * D; ++k) w[o++] = 0.02f * lcg_normalish();
    CHECK(o == n_w);
  }
  {
    int rc = rollout_init(&ctx, w, n_w * sizeof(float), &cfg);
    if (rc != ROLLOUT_OK) {
      fprintf(stderr, "rollout_init -> %d: %s\n", rc, rollout_last_error(NULL));
      return 1;
    }
  }
  free(w);

  for (i = 0; i < NPROMPT; ++i) {
    size_t j;
    offsets[i] = (uint32_t)(i * PLEN);
    for (j = 0; j < PLEN; ++j) tokens[i * PLEN + j] = (int32_t)((i * 37 + j * 11) % (V - 1));
    target[i] = (uint32_t)(1 + (i * 7) % CAP);
  }
  offsets[NPROMPT] = NPROMPT * PLEN;
  CALL(rollout_submit(ctx, tokens, offsets, target, NPROMPT, &first));
  CHECK(first == 0);

  for (;;) {
    rollout_step_info info;
    CALL(rollout_step(ctx, &info));
    CHECK(info.n_ran <= Q && info.n_active <= Q);
    if (info.n_finished_unharvested >= G || (info.n_active == 0 && info.n_queued == 0)) {
      rollout_traj recs[NPROMPT];
      int32_t tok[NPROMPT * CAP];
      float logp[NPROMPT * CAP];
      uint32_t ng = 0, nr = 0, r;
      uint64_t need = 0;
      const uint32_t flags = (info.n_active == 0 && info.n_queued == 0) ? ROLLOUT_FLUSH : 0;
      CALL(rollout_harvest(ctx, G, flags, recs, NPROMPT, tok, logp, NPROMPT * CAP, &ng, &nr, &need));
      for (r = 0; r < nr; ++r) {
        const rollout_traj* t = &recs[r];
        uint32_t k;
        CHECK(t->seq_id < NPROMPT && !seen[t->seq_id]);
        seen[t->seq_id] = 1;
        CHECK(t->gen_len == target[t->seq_id]);
        CHECK(tok[t->tok_off + t->gen_len - 1] == V - 1);
        for (k = 0; k < t->gen_len; ++k) CHECK(logp[t->tok_off + k] <= 1e-6f && logp[t->tok_off + k] > -50.f);
        if (r > 0 && recs[r - 1].group_idx == t->group_idx)
          CHECK(recs[r - 1].completion_step < t->completion_step ||
                (recs[r - 1].completion_step == t->completion_step &&
                 (recs[r - 1].gen_len < t->gen_len || (recs[r - 1].gen_len == t->gen_len && recs[r - 1].seq_id < t->seq_id))));
      }
      harvested += nr;
      groups_total += ng;
    }
    if (info.n_active == 0 && info.n_queued == 0) break;
    CHECK(info.step < 10000);
  }
  CHECK(harvested == NPROMPT);
  CALL(rollout_stats(ctx, &st));
  {
    uint64_t sum = 0;
    for (i = 0; i < NPROMPT; ++i) sum += target[i];
    CHECK(st.gen_tokens == sum && st.busy == sum && st.busy + st.idle == (uint64_t)Q * st.steps);
    CHECK(st.version == groups_total && st.prefill_tokens == (uint64_t)NPROMPT * PLEN);
  }
  rollout_destroy(ctx);
  printf("ok: %u rollouts in %u groups, %llu steps, bubble ratio %.3f\n", harvested, groups_total,
         (unsigned long long)st.steps, (double)st.idle / ((double)Q * (double)st.steps));
  return 0;
}
