// Ragged paged GQA decode attention for gfx950 (the KV-streaming half of the rollout step; the paper,
// Sec. 2.2, names KV-cache loading as what bounds autoregressive rollout).
//
// One wavefront owns (row, kv head, chunk of cached tokens; the chunk size is picked per launch); the four wavefronts
// of a workgroup take four consecutive chunks of the same (row, kv head) and merge their results through LDS, so a
// row of up to four chunks leaves the kernel finished and a longer one writes one partial result per four chunks
// (those stores are what the kernel pays most for after the K/V stream itself: about 3 us per MB of partials,
// measured by removing them).  A row is one query token of one slot; all G query heads that share the kv head are
// computed from a single pass over the K/V bytes.  The page layout makes both phases stream 16-byte vectors that
// are contiguous across lanes with no LDS staging of K or V:
//   K block [d/8][16 tokens][8 dims]  -> score phase, one lane per token (16 lanes cover one page)
//   V block [2][d][8 tokens]          -> value phase, one lane per output dim, tokens paired for dot2
// Scores and values use v_dot2c_f32_bf16 with the query held in scalar registers; probabilities go
// through a 512-byte per-wave LDS tile (bf16) to be re-read as broadcast operands.  Softmax statistics
// and accumulators are fp32.  The chunk groups of one (row, kv head) are merged inside the kernel by whichever of them
// arrives last (log-sum-exp merge in group order).
#include "common.h"
#include "kernels.h"

#define ATTN_GROUP ATTN_GROUP_CHUNKS   // chunks per workgroup
// Workgroup id -> (work item, kv head).  With the kv head as the fastest-varying grid dimension, consecutive
// workgroup ids (which the dispatcher deals round-robin to the 8 XCDs) are the kv heads of one work item, so all the
// chunk groups of one (row, kv head) run on the same XCD and their partial results meet in one L2.
#ifndef ATTN_KVH_FASTEST
#define ATTN_KVH_FASTEST 1
#endif

#define NEG_BIG (-1.0e30f)

// Partial results travel between workgroups that may sit on different XCDs (each with its own L2): they are written and
// read with agent-scope accesses, which go through to the memory side instead of staying in the writer's L2.  That is
// all the coherence the exchange needs; an agent-scope FENCE would also write back / invalidate the whole L2 of the XCD
// and costs three times the kernel (measured: 1.5-1.9 ms against 0.48 ms).
__device__ __forceinline__ void st_agent(float* p, float v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float ld_agent(const float* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

template <int D, int G>
__global__ __launch_bounds__(64 * ATTN_GROUP) void k_decode_attn(
    const uint8_t* __restrict__ pool, const uint16_t* __restrict__ q, const int* __restrict__ page_table, int max_pages,
    const int4* __restrict__ work, const int2* __restrict__ row_wstart, int Hkv, float* __restrict__ part_acc,
    float* __restrict__ part_ml, int* __restrict__ row_cnt, void* __restrict__ out, int out_fp32, float scale_log2e,
    int chunk_tokens) {
  constexpr int NCH = D / 8;
  constexpr int DPL = (D + 63) / 64;
  constexpr int KBYTES = PAGE_TOKENS * D * 2;
  constexpr int BLK = 2 * KBYTES;
  __shared__ __align__(16) uint16_t p_lds[ATTN_GROUP][G][64];
  __shared__ float acc_s[ATTN_GROUP][G][DPL * 64];
  __shared__ float ml_s[ATTN_GROUP][G][2];
  __shared__ int last_s;

  const int lane = threadIdx.x & 63;
  const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // wave-uniform: keeps q addressing scalar
#if ATTN_KVH_FASTEST
  const int kvh = blockIdx.x, wi = blockIdx.y;
#else
  const int kvh = blockIdx.y, wi = blockIdx.x;
#endif
  const int4 it = work[wi];                       // one load, then page ids and query go out together
  const int row = it.x, group = it.y, slot = it.z, ctx = it.w;
  // the group's token range is cut evenly (in 64-token tiles) over the four wavefronts, so they finish together; a
  // wavefront left without tokens contributes weight zero to the merge
  const int r0 = group * (ATTN_GROUP * chunk_tokens);
  const int r1 = min(ctx, r0 + ATTN_GROUP * chunk_tokens);
  const int span = (r1 - r0 + ATTN_GROUP * 64 - 1) / (ATTN_GROUP * 64) * 64;   // <= chunk_tokens
  const int tok0 = r0 + w * span;
  const int tok_end = min(r1, tok0 + span);
  const int last_page = (ctx - 1) >> 4;
  const int* __restrict__ pt = page_table + (size_t)slot * max_pages;
  const int Hq = Hkv * G;
  const uint32_t* __restrict__ qp = (const uint32_t*)(q + ((size_t)row * Hq + (size_t)kvh * G) * D);

  float m[G], l[G], acc[G][DPL];
#pragma unroll
  for (int h = 0; h < G; ++h) {
    m[h] = NEG_BIG;
    l[h] = 0.f;
#pragma unroll
    for (int dd = 0; dd < DPL; ++dd) acc[h][dd] = 0.f;
  }

  // page ids of this wavefront's span (at most 64 pages), fetched once: lane i holds logical page tok0/16 + i
  const int pgs = pt[min((tok0 >> 4) + lane, last_page)];

  for (int t0 = tok0; t0 < tok_end; t0 += 64) {
    const int tile = (t0 - tok0) >> 6;
    const int pg0 = __builtin_amdgcn_readlane(pgs, tile * 4 + 0), pg1 = __builtin_amdgcn_readlane(pgs, tile * 4 + 1),
              pg2 = __builtin_amdgcn_readlane(pgs, tile * 4 + 2), pg3 = __builtin_amdgcn_readlane(pgs, tile * 4 + 3);
    const int pgv[4] = {pg0, pg1, pg2, pg3};
    // ---- issue every load of the tile up front: K rows (lane = token), then V (lane = dim) ------------
    const int tok = t0 + lane;
    const int grp = lane >> 4;
    const int pg = grp == 0 ? pg0 : grp == 1 ? pg1 : grp == 2 ? pg2 : pg3;
    const uint8_t* kb = pool + ((size_t)pg * Hkv + kvh) * BLK + (tok & 15) * 16;
    uint4 kr[NCH];
#pragma unroll
    for (int c = 0; c < NCH; ++c) kr[c] = ld_stream16(kb + c * 256);
    uint4 vr[4][2][DPL];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const uint8_t* vb = pool + ((size_t)pgv[j] * Hkv + kvh) * BLK + KBYTES;
#pragma unroll
      for (int half = 0; half < 2; ++half)
#pragma unroll
        for (int dd = 0; dd < DPL; ++dd) {
          const int dim = (D >= 64) ? lane + dd * 64 : (lane & (D - 1));
          vr[j][half][dd] = ld_stream16(vb + ((size_t)half * D + dim) * 16);
        }
    }
    // With up to four query heads per kv head they are kept up front: left alone, the scheduler sinks the V loads below
    // the score phase to save registers (three wavefronts per SIMD instead of two, but two memory round trips per tile
    // instead of one): 0.6 % slower on a full batch of the 8B shape, 0.5 % faster on its half batch, no difference in
    // the tail drain.  With five heads per kv head (the 32B shape, 64 rows) the third wavefront is worth more than the
    // round trip: pinned, its launches take 102-104 us instead of 97-99.
    if constexpr (G <= 4) __builtin_amdgcn_sched_barrier(0);
    // ---- scores -----------------------------------------------------------------------------------------
    const bool valid = tok < tok_end;
#pragma unroll
    for (int h = 0; h < G; ++h) {
      float s = 0.f;
#pragma unroll
      for (int c = 0; c < NCH; ++c) {
        const uint32_t* qq = qp + h * (D / 2) + c * 4;
        s = dot2_bf16(kr[c].x, qq[0], s);
        s = dot2_bf16(kr[c].y, qq[1], s);
        s = dot2_bf16(kr[c].z, qq[2], s);
        s = dot2_bf16(kr[c].w, qq[3], s);
      }
      s = valid ? s * scale_log2e : NEG_BIG;
      const float m_new = fmaxf(m[h], wave_max(s));
      const float alpha = __builtin_amdgcn_exp2f(m[h] - m_new);
      const float p = valid ? __builtin_amdgcn_exp2f(s - m_new) : 0.f;
      l[h] = l[h] * alpha + p;
      m[h] = m_new;
#pragma unroll
      for (int dd = 0; dd < DPL; ++dd) acc[h][dd] *= alpha;
      p_lds[w][h][lane] = f2bf(p);
    }
    // ---- values: operands = (token pair) x (probability pair) ---------------------------------------------
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int tj = t0 + j * 16;
#pragma unroll
      for (int half = 0; half < 2; ++half) {
        const int tb = tj + half * 8;
        if (tb < tok_end) {                       // wave-uniform
          uint4 pw[G];
#pragma unroll
          for (int h = 0; h < G; ++h) pw[h] = *(const uint4*)&p_lds[w][h][j * 16 + half * 8];
#pragma unroll
          for (int dd = 0; dd < DPL; ++dd) {
            if (D >= 64 || lane < D) {
              uint4 v = vr[j][half][dd];
              if (tb + 8 > tok_end) {             // ragged tail: bytes past the context may hold anything
                const int nv = tok_end - tb;      // 1..7 valid tokens
                uint32_t* vw = (uint32_t*)&v;
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                  const uint32_t keep = (2 * i < nv ? 0x0000FFFFu : 0u) | (2 * i + 1 < nv ? 0xFFFF0000u : 0u);
                  vw[i] &= keep;
                }
              }
#pragma unroll
              for (int h = 0; h < G; ++h) {
                float a = acc[h][dd];
                a = dot2_bf16(v.x, pw[h].x, a);
                a = dot2_bf16(v.y, pw[h].y, a);
                a = dot2_bf16(v.z, pw[h].z, a);
                a = dot2_bf16(v.w, pw[h].w, a);
                acc[h][dd] = a;
              }
            }
          }
        }
      }
    }
  }

  // ---- merge the workgroup's chunks through LDS (fixed order: the result does not depend on scheduling) -------
#pragma unroll
  for (int h = 0; h < G; ++h) {
    const float lsum = wave_sum(l[h]);
#pragma unroll
    for (int dd = 0; dd < DPL; ++dd) acc_s[w][h][lane + dd * 64] = acc[h][dd];
    if (lane == 0) {
      ml_s[w][h][0] = m[h];
      ml_s[w][h][1] = lsum;
    }
  }
  __syncthreads();
  const int nchunks = (ctx + chunk_tokens - 1) / chunk_tokens;
  const int ngroups = (nchunks + ATTN_GROUP - 1) / ATTN_GROUP;
  for (int h = w; h < G; h += ATTN_GROUP) {       // wave w finishes heads w, w + 4, ..
    float mx = NEG_BIG;
#pragma unroll
    for (int u = 0; u < ATTN_GROUP; ++u) mx = fmaxf(mx, ml_s[u][h][0]);
    float den = 0.f, num[DPL];
#pragma unroll
    for (int dd = 0; dd < DPL; ++dd) num[dd] = 0.f;
#pragma unroll
    for (int u = 0; u < ATTN_GROUP; ++u) {
      const float wgt = __builtin_amdgcn_exp2f(ml_s[u][h][0] - mx);
      den += wgt * ml_s[u][h][1];
#pragma unroll
      for (int dd = 0; dd < DPL; ++dd) num[dd] += wgt * acc_s[u][h][lane + dd * 64];
    }
    const int head = kvh * G + h;
    if (ngroups == 1) {
      const float inv = 1.f / den;
#pragma unroll
      for (int dd = 0; dd < DPL; ++dd) {
        const int dim = lane + dd * 64;
        if (D >= 64 || dim < D) {
          const size_t o = ((size_t)row * Hq + head) * D + dim;
          if (out_fp32) ((float*)out)[o] = num[dd] * inv;
          else ((uint16_t*)out)[o] = f2bf(num[dd] * inv);
        }
      }
    } else {
      const size_t pi = (size_t)wi * Hq + head;
#pragma unroll
      for (int dd = 0; dd < DPL; ++dd) {
        const int dim = lane + dd * 64;
#ifndef ATTN_ABLATE_PARTIAL_STORES
        if (D >= 64 || dim < D) st_agent(&part_acc[pi * D + dim], num[dd]);
#endif
      }
      if (lane == 0) {
        st_agent(&part_ml[pi * 2], mx);
        st_agent(&part_ml[pi * 2 + 1], den);
      }
    }
  }
  if (ngroups == 1) return;                       // uniform over the workgroup
  // ---- a row of several groups: the group that arrives last merges them all (log-sum-exp merge in group order, so the
  // result does not depend on which one that is).  Every thread waits until its own partial stores have completed
  // (they are write-through, see st_agent), the barrier collects the workgroup, then one thread counts the arrival;
  // the last group reads the others' partials with agent-scope loads.  The counter returns to zero for the next launch.
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();
  if (threadIdx.x == 0) last_s = atomicAdd(&row_cnt[row * Hkv + kvh], 1) == ngroups - 1;
  __syncthreads();
  if (!last_s) return;
  // work item of group c: the row's full groups are consecutive from ws.x, a last shorter group sits at ws.y
  const int2 ws = row_wstart[row];
  const int nfull = ctx / (ATTN_GROUP * chunk_tokens);
  // One wavefront per head.  The partials live at the memory side (uncached loads, a microsecond or two each), so
  // they are fetched in batches: lane c takes the (max, sum) pair of group c in one round trip, the accumulators come
  // eight groups at a time.  The order of every sum is fixed (butterfly over lanes, then ascending groups).
  for (int h = w; h < G; h += ATTN_GROUP) {
    const int head = kvh * G + h;
    float mx = NEG_BIG;
    for (int c0 = 0; c0 < ngroups; c0 += 64) {
      const int c = c0 + lane;
      const float mc = c < ngroups ? ld_agent(&part_ml[((size_t)(c < nfull ? ws.x + c : ws.y) * Hq + head) * 2]) : NEG_BIG;
      mx = fmaxf(mx, wave_max(mc));
    }
    float den = 0.f, num[DPL];
#pragma unroll
    for (int dd = 0; dd < DPL; ++dd) num[dd] = 0.f;
    for (int c0 = 0; c0 < ngroups; c0 += 64) {
      const int c = c0 + lane;
      float wgt = 0.f, lc = 0.f;
      if (c < ngroups) {
        const size_t pi = (size_t)(c < nfull ? ws.x + c : ws.y) * Hq + head;
        wgt = __builtin_amdgcn_exp2f(ld_agent(&part_ml[pi * 2]) - mx);
        lc = ld_agent(&part_ml[pi * 2 + 1]);
      }
      den += wave_sum(wgt * lc);
      const int nb = min(64, ngroups - c0);
      for (int u0 = 0; u0 < nb; u0 += 8) {
        float v[8][DPL];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
          const int cu = c0 + min(u0 + u, nb - 1);          // past the end: the last group again, with weight zero
          const size_t pi = (size_t)(cu < nfull ? ws.x + cu : ws.y) * Hq + head;
#pragma unroll
          for (int dd = 0; dd < DPL; ++dd) {
            const int dim = lane + dd * 64;
            v[u][dd] = (D >= 64 || dim < D) ? ld_agent(&part_acc[pi * D + dim]) : 0.f;
          }
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) {
          const float wu = u0 + u < nb ? __shfl(wgt, u0 + u, 64) : 0.f;
#pragma unroll
          for (int dd = 0; dd < DPL; ++dd) num[dd] += wu * v[u][dd];
        }
      }
    }
#pragma unroll
    for (int dd = 0; dd < DPL; ++dd) {
      const int dim = lane + dd * 64;
      if (D >= 64 || dim < D) {
        const size_t o = ((size_t)row * Hq + head) * D + dim;
        if (out_fp32) ((float*)out)[o] = num[dd] / den;
        else ((uint16_t*)out)[o] = f2bf(num[dd] / den);
      }
    }
  }
  if (threadIdx.x == 0) row_cnt[row * Hkv + kvh] = 0;
}

template <int D>
__global__ void k_write_kv(uint8_t* __restrict__ pool, int Hkv, const uint16_t* __restrict__ k,
                           const uint16_t* __restrict__ v, const int* __restrict__ tok_seq,
                           const int* __restrict__ tok_pos, const int* __restrict__ page_table, int max_pages,
                           size_t n_tok) {
  constexpr int KBYTES = PAGE_TOKENS * D * 2;
  const size_t total = n_tok * Hkv * D;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (size_t)gridDim.x * blockDim.x) {
    const int dim = (int)(i % D);
    const int kvh = (int)((i / D) % Hkv);
    const size_t t = i / ((size_t)D * Hkv);
    const int pos = tok_pos[t];
    const int pg = page_table[(size_t)tok_seq[t] * max_pages + (pos >> 4)];
    const int tk = pos & 15;
    uint16_t* blk = (uint16_t*)(pool + ((size_t)pg * Hkv + kvh) * 2 * KBYTES);
    blk[((dim >> 3) * 16 + tk) * 8 + (dim & 7)] = k[i];
    blk[KBYTES / 2 + ((size_t)(tk >> 3) * D + dim) * 8 + (tk & 7)] = v[i];
  }
}

// ---------------------------------------------------------------------------------------------------
int attn_supported(int head_dim, int group) {
  return (head_dim == 128 && (group == 1 || group == 4 || group == 5)) || (head_dim == 32 && (group == 1 || group == 4 || group == 5));
}

template <int D, int G>
static void launch_attn_t(const AttnArgs& a, hipStream_t st, hipEvent_t ev0, hipEvent_t ev1) {
  const float scale = 1.4426950408889634f / sqrtf((float)D);
#if ATTN_KVH_FASTEST
  dim3 grid(a.Hkv, a.n_work);
#else
  dim3 grid(a.n_work, a.Hkv);
#endif
  if (ev0) (void)hipEventRecord(ev0, st);
  hipLaunchKernelGGL((k_decode_attn<D, G>), grid, dim3(64 * ATTN_GROUP), 0, st, (const uint8_t*)a.pool, (const uint16_t*)a.q,
                     a.page_table, a.max_pages, a.work, a.row_wstart, a.Hkv, a.part_acc, a.part_ml, a.row_cnt, a.out,
                     a.out_fp32, scale, a.chunk_tokens);
  if (ev1) (void)hipEventRecord(ev1, st);
}

// ev0 / ev1 (nullable) bracket the kernel.
void launch_decode_attn(const AttnArgs& a, int head_dim, int group, hipStream_t st, hipEvent_t ev0, hipEvent_t ev1) {
  if (a.n_work <= 0) return;
  if (head_dim == 128 && group == 4) launch_attn_t<128, 4>(a, st, ev0, ev1);
  else if (head_dim == 128 && group == 5) launch_attn_t<128, 5>(a, st, ev0, ev1);
  else if (head_dim == 128 && group == 1) launch_attn_t<128, 1>(a, st, ev0, ev1);
  else if (head_dim == 32 && group == 1) launch_attn_t<32, 1>(a, st, ev0, ev1);
  else if (head_dim == 32 && group == 4) launch_attn_t<32, 4>(a, st, ev0, ev1);
  else if (head_dim == 32 && group == 5) launch_attn_t<32, 5>(a, st, ev0, ev1);
}

void launch_write_kv(void* pool, int Hkv, int head_dim, const void* k, const void* v, const int* tok_seq,
                     const int* tok_pos, const int* page_table, int max_pages, size_t n_tok, hipStream_t st) {
  if (n_tok == 0) return;
  const size_t total = n_tok * Hkv * head_dim;
  const int blocks = (int)((total + 255) / 256 < 65535 * 8 ? (total + 255) / 256 : 65535 * 8);
  if (head_dim == 128)
    hipLaunchKernelGGL((k_write_kv<128>), dim3(blocks), dim3(256), 0, st, (uint8_t*)pool, Hkv, (const uint16_t*)k,
                       (const uint16_t*)v, tok_seq, tok_pos, page_table, max_pages, n_tok);
  else
    hipLaunchKernelGGL((k_write_kv<32>), dim3(blocks), dim3(256), 0, st, (uint8_t*)pool, Hkv, (const uint16_t*)k,
                       (const uint16_t*)v, tok_seq, tok_pos, page_table, max_pages, n_tok);
}

// ---------------------------------------------------------------------------------------------------
// Causal paged attention for prefill rows (refilled or resumed rollouts): a dense contraction, so it runs
// on the matrix cores.  One wavefront = 32 consecutive query tokens of one sequence x one query head.
// Both products are taken transposed so that a lane always owns one query row:
//   S^T = K Q^T   (A = K tile straight from the page: lane -> key, 16-byte dim chunks; B = Q^T in registers)
//   O^T = V^T P^T (A = V^T straight from the page: lane -> dim, token runs; B = P^T = the softmaxed S^T
//                  accumulators)
// which keeps the online-softmax statistics, the rescaling and the final 1/l entirely lane-local.
// The accumulator layout of S^T gives a half-wave, per page, score rows {4g..4g+3} and {8+4g..8+4g+3} (g = lane / 32),
// while the value product wants from it the probabilities of eight CONSECUTIVE tokens (the run one 16-byte V load
// holds).  So the K rows are fetched in a permuted order -- the lane that feeds score row r loads the key whose token
// index within its page is r with bits 2 and 3 swapped -- which makes the rows a half-wave owns exactly tokens 8g..8g+7
// of each page: the P^T operand is then the packed accumulators as they are, and every V fragment is one 16-byte load.
struct PfTile { int row0, n, slot, pos0; };

// PF_KSPLIT wavefronts share one (query tile, head): wavefront w takes key tiles w, w + PF_KSPLIT, ..  A query tile deep
// in a long sequence has hundreds of key tiles (512 at 16k tokens) and a wavefront walks its tiles one after the other, so
// with one wavefront per query tile the launch lasted as long as its longest query tile while most of the chip had run
// out of work -- that, not the softmax arithmetic or the K/V traffic, is what held the kernel at a tenth of the matrix
// peak (a variant that shared K/V tiles between the heads of a group through a three-stage LDS ring was no faster).
// The partial results of the wavefronts are merged pairwise through LDS in a fixed order (log-sum-exp merge).
#define PF_KSPLIT 4
template <int D>
__global__ __launch_bounds__(64 * PF_KSPLIT, 2) void k_prefill_attn(const uint8_t* __restrict__ pool, const uint16_t* __restrict__ q,
                                                                const PfTile* __restrict__ tiles,
                                                                const int* __restrict__ page_table, int max_pages, int Hq,
                                                                int Hkv, int G, uint16_t* __restrict__ out, float scale_log2e) {
  typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
  typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
  constexpr int KBYTES = PAGE_TOKENS * D * 2;
  constexpr int BLK = 2 * KBYTES;
  constexpr int NDC = D / 16;   // k-steps of the score product
  constexpr int NMT = D / 32;   // 32-dim tiles of the output
  constexpr int MREC = NMT * 16 + 2;   // floats one lane hands over in a merge: its accumulators, m and l
  __shared__ float mrg[2][MREC][64];   // [sender][value][lane]: lane-contiguous, conflict-free
  const PfTile tile = tiles[blockIdx.x];
  const int head = blockIdx.y, kvh = head / G;
  const int lane = threadIdx.x & 63, g = lane >> 5, c = lane & 31;
  const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int row = tile.row0 + min(c, tile.n - 1);
  const int pos_c = tile.pos0 + c;
  const int last_key = tile.pos0 + tile.n - 1;
  const int last_page = last_key >> 4;
  const int* __restrict__ pt = page_table + (size_t)tile.slot * max_pages;
  // token (within its page) of the key this lane loads for score row c: bits 2 and 3 of c swapped
  const int tau = (c & 3) | ((c & 4) << 1) | ((c & 8) >> 1);

  bf16x8_t qf[NDC];
  {
    const uint16_t* qr = q + ((size_t)row * Hq + head) * D + g * 8;
#pragma unroll
    for (int dc = 0; dc < NDC; ++dc) qf[dc] = __builtin_bit_cast(bf16x8_t, *(const u32x4*)(qr + dc * 16));
  }
  f32x16_t o[NMT];
#pragma unroll
  for (int mt = 0; mt < NMT; ++mt)
#pragma unroll
    for (int j = 0; j < 16; ++j) o[mt][j] = 0.f;
  float m_run = NEG_BIG, l_run = 0.f;

  const int n_kt = (last_key >> 5) + 1;
  // software pipeline: the K fragments of this wavefront's next key tile are fetched as soon as the score product has
  // consumed the current ones, the V fragments as soon as the value product has
  int pg = 0;
  u32x4 kf[NDC], vw[2][NMT];
  // V fragments of key tile `t` (both pages; a page wholly past the tile's last query is skipped in the product, its
  // loads are clamped to the last valid page so they stay inside the slot's pages); pg_t holds the two page ids in
  // lanes 0 and 16
  auto load_v = [&](int pg_t, u32x4 (&v)[2][NMT]) {
#pragma unroll
    for (int s2 = 0; s2 < 2; ++s2) {
      const int pgs = __builtin_amdgcn_readlane(pg_t, s2 * 16);
      const uint8_t* vb = pool + ((size_t)pgs * Hkv + kvh) * BLK + KBYTES + (size_t)g * D * 16;
#pragma unroll
      for (int mt = 0; mt < NMT; ++mt) {
        const int dim = mt * 32 + c;
        v[s2][mt] = *(const u32x4*)(vb + (size_t)dim * 16);    // tokens 8g .. 8g+7 of the page, one dim
      }
    }
  };
  // Page ids run one tile further ahead than the fragments: pg holds the pages of the tile whose fragments are fetched
  // during the current iteration, pg2 those of the tile after it, requested at the top of the iteration.  Loads complete
  // in issue order, so an id requested right before it is used would make its user wait for every V load in flight (that
  // was a full drain of the queue between the score product and the softmax of every tile).  The prologue issues its loads
  // in the order an iteration leaves them in -- id, K fragments, V fragments -- so that the wait counts the compiler
  // derives for the loop are those of the steady state.
  int pg2 = 0;
  if (w < n_kt) {                                          // uniform
    const int pg0 = pt[min(w * 2 + (c >> 4), last_page)];
    const int kt1 = w + PF_KSPLIT < n_kt ? w + PF_KSPLIT : w;
    pg = pt[min(kt1 * 2 + (c >> 4), last_page)];
    __builtin_amdgcn_sched_barrier(0);
    const uint8_t* kb = pool + ((size_t)pg0 * Hkv + kvh) * BLK + tau * 16 + g * 256;
#pragma unroll
    for (int dc = 0; dc < NDC; ++dc) kf[dc] = *(const u32x4*)(kb + dc * 512);
    __builtin_amdgcn_sched_barrier(0);
    load_v(pg0, vw);
    __builtin_amdgcn_sched_barrier(0);
  }
  for (int kt = w; kt < n_kt; kt += PF_KSPLIT) {
    const int ktn = kt + PF_KSPLIT < n_kt ? kt + PF_KSPLIT : kt;   // past the end: this tile once more
    const int kt2 = ktn + PF_KSPLIT < n_kt ? ktn + PF_KSPLIT : ktn;
    pg2 = pt[min(kt2 * 2 + (c >> 4), last_page)];
    __builtin_amdgcn_sched_barrier(0);
    f32x16_t s;
#pragma unroll
    for (int j = 0; j < 16; ++j) s[j] = 0.f;
#pragma unroll
    for (int dc = 0; dc < NDC; ++dc)
      s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, kf[dc]), qf[dc], s, 0, 0, 0);
    {   // the next tile's K fragments go into the registers the score product has just consumed
      const uint8_t* kb = pool + ((size_t)pg * Hkv + kvh) * BLK + tau * 16 + g * 256;
#pragma unroll
      for (int dc = 0; dc < NDC; ++dc) kf[dc] = *(const u32x4*)(kb + dc * 512);
    }
    // s[j] = score of key kt*32 + (j/8)*16 + g*8 + j%8 against this lane's query row (K rows are loaded permuted).  Only key tiles that reach past
    // the tile's first query need the causal mask (the last one or two); the others are wholly visible.
    const bool diag = kt * 32 + 31 > tile.pos0;           // wave-uniform
    float mx = NEG_BIG;
    if (diag) {
#pragma unroll
      for (int j = 0; j < 16; ++j) {
        const int key = kt * 32 + (j >> 3) * 16 + g * 8 + (j & 7);   // score row (j/4)*8 + 4g + j%4 holds this key (see tau)
        s[j] = key <= pos_c ? s[j] * scale_log2e : NEG_BIG;
        mx = fmaxf(mx, s[j]);
      }
    } else {
#pragma unroll
      for (int j = 0; j < 16; ++j) {
        s[j] *= scale_log2e;
        mx = fmaxf(mx, s[j]);
      }
    }
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
    const float m_new = fmaxf(m_run, mx);
    // Rescaling the accumulators is 64 multiplies per lane, and with 64 rows-halves in a wavefront SOME row's maximum
    // moves in most tiles until a few thousand keys have been seen.  The running maximum is therefore only a reference
    // point: it is moved (and the accumulators rescaled) when some row's scores exceed it by more than 2^8; until then
    // probabilities up to 256 are accumulated against the old reference, which fp32 sums and bf16 operands (relative
    // precision) take without loss, and the final division by l cancels the reference exactly.
    if (__builtin_amdgcn_ballot_w64(m_new > m_run + 8.0f) != 0) {
      const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);
      l_run *= alpha;
#pragma unroll
      for (int mt = 0; mt < NMT; ++mt)
#pragma unroll
        for (int j = 0; j < 16; ++j) o[mt][j] *= alpha;
      m_run = m_new;
    }
    // a row whose keys in this wavefront's tiles are all masked so far still has m_run = -1e30: subtract a floor
    // instead, so that exp2 of a masked score underflows to exactly 0 whatever m_run is
    const float m_sub = fmaxf(m_run, -1.0e20f);
    float ls = 0.f;
    uint32_t pk[8];
#pragma unroll
    for (int j = 0; j < 16; j += 2) {
      const float p0 = __builtin_amdgcn_exp2f(s[j] - m_sub);
      const float p1 = __builtin_amdgcn_exp2f(s[j + 1] - m_sub);
      ls += p0 + p1;
      pk[j >> 1] = pack_bf2(p0, p1);
    }
    l_run += ls;
#pragma unroll
    for (int s2 = 0; s2 < 2; ++s2) {
      if (kt * 32 + s2 * 16 > last_key) break;          // wave-uniform: page wholly past the tile's last query
      u32x4 pw;
      pw.x = pk[4 * s2]; pw.y = pk[4 * s2 + 1]; pw.z = pk[4 * s2 + 2]; pw.w = pk[4 * s2 + 3];
      const bf16x8_t pf = __builtin_bit_cast(bf16x8_t, pw);
#pragma unroll
      for (int mt = 0; mt < NMT; ++mt)
        o[mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, vw[s2][mt]), pf, o[mt], 0, 0, 0);
    }
    load_v(pg, vw);                                      // the next tile's V fragments, into the registers just consumed
    pg = pg2;
  }

  // ---- merge the wavefronts' partial results: 2 -> 0 and 3 -> 1, then 1 -> 0 (lane-local: every wavefront keeps the
  // same (query row, dims) in the same lane and register).  A wavefront without tiles hands over weight zero.
  auto send = [&](int slot) {
#pragma unroll
    for (int mt = 0; mt < NMT; ++mt)
#pragma unroll
      for (int j = 0; j < 16; ++j) mrg[slot][mt * 16 + j][lane] = o[mt][j];
    mrg[slot][NMT * 16][lane] = m_run;
    mrg[slot][NMT * 16 + 1][lane] = l_run;
  };
  auto take = [&](int slot) {
    const float mb = mrg[slot][NMT * 16][lane], lb = mrg[slot][NMT * 16 + 1][lane];
    const float M = fmaxf(m_run, mb);
    const float wa = __builtin_amdgcn_exp2f(m_run - M), wb = __builtin_amdgcn_exp2f(mb - M);
    l_run = l_run * wa + lb * wb;
    m_run = M;
#pragma unroll
    for (int mt = 0; mt < NMT; ++mt)
#pragma unroll
      for (int j = 0; j < 16; ++j) o[mt][j] = o[mt][j] * wa + mrg[slot][mt * 16 + j][lane] * wb;
  };
  static_assert(PF_KSPLIT == 4, "the merge below is written for four wavefronts");
  if (w >= 2) send(w - 2);
  __syncthreads();
  if (w < 2) take(w);
  __syncthreads();
  if (w == 1) send(0);
  __syncthreads();
  if (w != 0) return;
  take(0);

  const float l_tot = l_run + __shfl_xor(l_run, 32, 64);
  if (c < tile.n) {
    const float inv = 1.f / l_tot;
    uint16_t* orow = out + ((size_t)(tile.row0 + c) * Hq + head) * D;
#pragma unroll
    for (int mt = 0; mt < NMT; ++mt)
#pragma unroll
      for (int jq = 0; jq < 4; ++jq) {
        const int dim = mt * 32 + jq * 8 + g * 4;
        u32x2 w2;
        w2.x = pack_bf2(o[mt][jq * 4] * inv, o[mt][jq * 4 + 1] * inv);
        w2.y = pack_bf2(o[mt][jq * 4 + 2] * inv, o[mt][jq * 4 + 3] * inv);
        *(u32x2*)(orow + dim) = w2;
      }
  }
}

void launch_prefill_attn(const void* pool, const void* q, const void* tiles, int n_tiles, const int* page_table,
                         int max_pages, int Hq, int Hkv, int head_dim, void* out, hipStream_t st) {
  if (n_tiles <= 0) return;
  const float scale = 1.4426950408889634f / sqrtf((float)head_dim);
  dim3 grid(n_tiles, Hq);
  if (head_dim == 128)
    hipLaunchKernelGGL((k_prefill_attn<128>), grid, dim3(64 * PF_KSPLIT), 0, st, (const uint8_t*)pool, (const uint16_t*)q,
                       (const PfTile*)tiles, page_table, max_pages, Hq, Hkv, Hq / Hkv, (uint16_t*)out, scale);
  else
    hipLaunchKernelGGL((k_prefill_attn<32>), grid, dim3(64 * PF_KSPLIT), 0, st, (const uint8_t*)pool, (const uint16_t*)q,
                       (const PfTile*)tiles, page_table, max_pages, Hq, Hkv, Hq / Hkv, (uint16_t*)out, scale);
}
