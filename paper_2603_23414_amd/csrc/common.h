// Shared device helpers for the rollout kernels (gfx950 / CDNA4, 64-wide wavefronts).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#define PAGE_TOKENS 16
// A decode-attention wavefront covers `chunk` cached tokens of one (row, kv head), a workgroup ATTN_GROUP_CHUNKS
// consecutive chunks (one work item of the list); the chunk is chosen per launch: a multiple of 64 between
// ATTN_CHUNK_MIN and ATTN_CHUNK_MAX, about (sum of contexts) * n_kv_heads / ATTN_TARGET_ITEMS wavefront spans, i.e.
// the largest chunks that still leave every resident wavefront slot (256 CUs x 4 SIMDs x 2) a span or two: with the
// rows finished inside the kernel and the work list ordered longest-first, fewer and longer items win (fewer partial
// results, fewer workgroup starts).  Measured, attention alone, us per launch at 12288 / 6144 / 4096 spans: 32 rows of
// 4-16 k tokens 240 / 228 / 229, 64 rows 390 / 377 / 378, a full batch 457 / 446 / 445; in the step 454.6 / 451.4 /
// 451.0 (full batch), 558 / 548 / 548 (123 rows), 247 / 240 / 237 (32 rows); 9 long rows and the 32B workload's 64 short
// ones sit at the 128-token floor either way (the floor beats 256 by 5 % there and 64 loses again), so that a few long
// rollouts still spread over the chip.
#ifndef ATTN_GROUP_CHUNKS
#define ATTN_GROUP_CHUNKS 4
#endif
#ifndef ATTN_CHUNK_MIN
#define ATTN_CHUNK_MIN 128
#endif
#define ATTN_CHUNK_MAX 1024         // 64 pages: their ids fit one register across a wavefront
#ifndef ATTN_TARGET_ITEMS
#define ATTN_TARGET_ITEMS 4096
#endif
__host__ __device__ __forceinline__ int attn_pick_chunk(unsigned long long total_ctx, int n_kv_heads) {
  unsigned long long c = (total_ctx * (unsigned long long)n_kv_heads + ATTN_TARGET_ITEMS - 1) / ATTN_TARGET_ITEMS;
  c = (c + 63) / 64 * 64;
  return c < ATTN_CHUNK_MIN ? ATTN_CHUNK_MIN : c > ATTN_CHUNK_MAX ? ATTN_CHUNK_MAX : (int)c;
}
// work items (workgroups per kv head) of a row with `ctx` cached tokens
__host__ __device__ __forceinline__ int attn_row_items(int ctx, int chunk) {
  return ((ctx + chunk - 1) / chunk + ATTN_GROUP_CHUNKS - 1) / ATTN_GROUP_CHUNKS;
}
#define WAVE 64

typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(16))) float f32x16_t;
typedef __attribute__((ext_vector_type(4))) float f32x4_t;

__device__ __forceinline__ float bf2f(uint16_t b) { return __uint_as_float(((uint32_t)b) << 16); }
__device__ __forceinline__ uint16_t f2bf(float f) {       // round to nearest even
  __bf16 b = (__bf16)f;
  return __builtin_bit_cast(uint16_t, b);
}
__device__ __forceinline__ uint32_t pack_bf2(float lo, float hi) {
  return (uint32_t)f2bf(lo) | ((uint32_t)f2bf(hi) << 16);
}
// acc + a.lo*b.lo + a.hi*b.hi on packed bf16 pairs (v_dot2c_f32_bf16)
__device__ __forceinline__ float dot2_bf16(uint32_t a, uint32_t b, float acc) {
  return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, a), __builtin_bit_cast(bf16x2_t, b), acc, false);
}

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}

// 16-byte streaming load: data that is read once per kernel (KV pages, weights) should not displace what is reused
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint4 ld_stream16(const void* p) {
  const u32x4_t t = __builtin_nontemporal_load((const u32x4_t*)p);
  return make_uint4(t.x, t.y, t.z, t.w);
}

// bytes of one (page, kv head) block: K then V, bf16
__host__ __device__ __forceinline__ size_t kv_block_bytes(int head_dim) { return (size_t)2 * PAGE_TOKENS * head_dim * 2; }

// Philox4x32-10 (Salmon et al., SC'11): first output word for counter (c0, c1, c2, c3) under key (k0, k1).
__device__ __forceinline__ uint32_t philox4x32_10_word0(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3, uint32_t k0,
                                                       uint32_t k1) {
#pragma unroll
  for (int r = 0; r < 10; ++r) {
    const uint32_t hi0 = __umulhi(0xD2511F53u, c0), lo0 = 0xD2511F53u * c0;
    const uint32_t hi1 = __umulhi(0xCD9E8D57u, c2), lo1 = 0xCD9E8D57u * c2;
    c0 = hi1 ^ c1 ^ k0;
    c1 = lo1;
    c2 = hi0 ^ c3 ^ k1;
    c3 = lo0;
    k0 += 0x9E3779B9u;
    k1 += 0xBB67AE85u;
  }
  return c0;
}

// The uniform behind the Gumbel-max draw of vocabulary column `col` for token `tok_index` of sequence `seq_id`:
// (top 24 bits of the first Philox word + 1/2) * 2^-24, strictly inside (0, 1).
__device__ __forceinline__ float gumbel_uniform(uint32_t col, uint32_t tok_index, unsigned long long seq_id,
                                                unsigned long long seed) {
  const uint32_t w = philox4x32_10_word0(col, tok_index, (uint32_t)seq_id, (uint32_t)(seq_id >> 32), (uint32_t)seed,
                                         (uint32_t)(seed >> 32));
  return ((float)(w >> 8) + 0.5f) * 5.9604644775390625e-8f;
}
