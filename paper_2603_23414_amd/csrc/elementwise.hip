// The small fused kernels around the projections: embedding gather, residual-add + RMSNorm (+ bf16 cast),
// RoPE + KV page write, arg-max / log-sum-exp over the vocabulary, row gather.
// All of them are HBM-trivial next to the weight and KV streams; each one also folds in the fixed-order
// sum over the split-K partials of the projection that feeds it.
#include "common.h"
#include "kernels.h"

__global__ __launch_bounds__(256) void k_embed(const uint16_t* __restrict__ table, const int* __restrict__ row_tok,
                                               float* __restrict__ h, int D) {
  const int r = blockIdx.x;
  const uint16_t* src = table + (size_t)row_tok[r] * D;
  for (int i = threadIdx.x; i < D; i += 256) h[(size_t)r * D + i] = bf2f(src[i]);
}

__device__ __forceinline__ float block_sum_1024(float v, float* sh) {
  v = wave_sum(v);
  if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = v;
  __syncthreads();
  float t = 0.f;
#pragma unroll
  for (int k = 0; k < 16; ++k) t += sh[k];
  __syncthreads();
  return t;
}

// t += part[0] + part[1] + .. in ascending split order (the order fixes the rounding); the loads of up to eight splits
// are issued before the first add, so a row's split-K partials arrive in one or two memory round trips instead of S
__device__ __forceinline__ void add_splits(float4& t, const float* __restrict__ p, size_t stride, int S) {
  int s = 0;
  for (; s + 8 <= S; s += 8) {
    float4 v[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) v[j] = *(const float4*)(p + (size_t)(s + j) * stride);
#pragma unroll
    for (int j = 0; j < 8; ++j) { t.x += v[j].x; t.y += v[j].y; t.z += v[j].z; t.w += v[j].w; }
  }
  if (s + 4 <= S) {
    float4 v[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) v[j] = *(const float4*)(p + (size_t)(s + j) * stride);
#pragma unroll
    for (int j = 0; j < 4; ++j) { t.x += v[j].x; t.y += v[j].y; t.z += v[j].z; t.w += v[j].w; }
    s += 4;
  }
  for (; s < S; ++s) {
    const float4 v = *(const float4*)(p + (size_t)s * stride);
    t.x += v.x; t.y += v.y; t.z += v.z; t.w += v.w;
  }
}

// h[r] += sum_s part[s][r] (S may be 0), then x[r] = bf16( h[r] * rsqrt(mean(h[r]^2) + eps) * gain ).
// One 1024-thread block per row, 16-byte accesses; D is a multiple of 4 and at most 8192.
__global__ __launch_bounds__(1024) void k_add_rmsnorm(float* __restrict__ h, const float* __restrict__ part, int S,
                                                      size_t part_stride, const float* __restrict__ gain, float eps,
                                                      uint16_t* __restrict__ x, int D) {
  __shared__ float sh[16];
  const int r = blockIdx.x;
  const int nv = D >> 2;
  float4 v[2];
  float ss = 0.f;
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int c = threadIdx.x + i * 1024;
    if (c < nv) {
      float4 t = ((const float4*)(h + (size_t)r * D))[c];
      add_splits(t, part + (size_t)r * D + 4 * c, part_stride, S);
      v[i] = t;
      ss += t.x * t.x + t.y * t.y + t.z * t.z + t.w * t.w;
    }
  }
  const float tot = block_sum_1024(ss, sh);
  const float inv = 1.0f / sqrtf(tot / (float)D + eps);
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int c = threadIdx.x + i * 1024;
    if (c < nv) {
      if (S > 0) ((float4*)(h + (size_t)r * D))[c] = v[i];
      const float4 g = ((const float4*)gain)[c];
      uint2 o;
      o.x = pack_bf2(v[i].x * inv * g.x, v[i].y * inv * g.y);
      o.y = pack_bf2(v[i].z * inv * g.z, v[i].w * inv * g.w);
      ((uint2*)(x + (size_t)r * D))[c] = o;
    }
  }
}

// qkv[r] = sum_s part[s][r] (+ bias); rotate-half RoPE on q and k heads at row_pos[r]; q -> bf16 [R][Hq][d];
// k, v -> the slot's KV page (K as [d/8][16][8], V as [2][d][8]).
__global__ __launch_bounds__(1024) void k_rope_kvwrite(const float* __restrict__ part, int S, size_t part_stride,
                                                      const float* __restrict__ bias, const int* __restrict__ row_slot,
                                                      const int* __restrict__ row_pos, const float2* __restrict__ cs_table,
                                                      uint16_t* __restrict__ q_out, uint8_t* __restrict__ pool,
                                                      const int* __restrict__ page_table, int max_pages, int Hq, int Hkv,
                                                      int d) {
  // one work item = four consecutive dims: (Hq + Hkv) * d/8 rotation items (dims i..i+3 paired with i+d/2..), then
  // Hkv * d/4 value items; head_dim is a multiple of 8, so every load is a float4 and q / K stores are 8 bytes
  const int r = blockIdx.x;
  const int pos = row_pos[r];
  const int slot = row_slot[r];
  const int Nqkv = (Hq + 2 * Hkv) * d;
  const int half = d / 2, hq4 = half / 4;
  const float* src = part + (size_t)r * Nqkv;
  const int pg = page_table[(size_t)slot * max_pages + (pos >> 4)];
  const int tk = pos & 15;
  const size_t kbytes = (size_t)PAGE_TOKENS * d * 2;
  const int n_rot = (Hq + Hkv) * hq4;
  const int n_v = Hkv * d / 4;
  const int voff = (Hq + Hkv) * d;
  for (int e = threadIdx.x; e < n_rot + n_v; e += 1024) {
    if (e < n_rot) {
      const int head = e / hq4, i = (e % hq4) * 4;
      const int c1 = head * d + i, c2 = c1 + half;
      float4 x1 = make_float4(0.f, 0.f, 0.f, 0.f), x2 = x1;
      add_splits(x1, src + c1, part_stride, S);
      add_splits(x2, src + c2, part_stride, S);
      if (bias) {
        const float4 a = *(const float4*)(bias + c1), b = *(const float4*)(bias + c2);
        x1.x += a.x; x1.y += a.y; x1.z += a.z; x1.w += a.w;
        x2.x += b.x; x2.y += b.y; x2.z += b.z; x2.w += b.w;
      }
      const float4 cs01 = *(const float4*)(cs_table + (size_t)pos * half + i);        // (cos, sin) of dims i, i+1
      const float4 cs23 = *(const float4*)(cs_table + (size_t)pos * half + i + 2);
      uint2 y1, y2;
      y1.x = pack_bf2(x1.x * cs01.x - x2.x * cs01.y, x1.y * cs01.z - x2.y * cs01.w);
      y1.y = pack_bf2(x1.z * cs23.x - x2.z * cs23.y, x1.w * cs23.z - x2.w * cs23.w);
      y2.x = pack_bf2(x2.x * cs01.x + x1.x * cs01.y, x2.y * cs01.z + x1.y * cs01.w);
      y2.y = pack_bf2(x2.z * cs23.x + x1.z * cs23.y, x2.w * cs23.z + x1.w * cs23.w);
      if (head < Hq) {
        uint16_t* qo = q_out + ((size_t)r * Hq + head) * d;
        *(uint2*)(qo + i) = y1;
        *(uint2*)(qo + i + half) = y2;
      } else {
        const int kvh = head - Hq;
        uint16_t* blk = (uint16_t*)(pool + ((size_t)pg * Hkv + kvh) * 2 * kbytes);
        const int d1 = i, d2 = i + half;                      // four dims stay inside one group of 8
        *(uint2*)(blk + ((d1 >> 3) * 16 + tk) * 8 + (d1 & 7)) = y1;
        *(uint2*)(blk + ((d2 >> 3) * 16 + tk) * 8 + (d2 & 7)) = y2;
      }
    } else {
      const int ev = (e - n_rot) * 4;
      const int kvh = ev / d, dim = ev % d;
      float4 x = make_float4(0.f, 0.f, 0.f, 0.f);
      add_splits(x, src + voff + ev, part_stride, S);
      if (bias) {
        const float4 a = *(const float4*)(bias + voff + ev);
        x.x += a.x; x.y += a.y; x.z += a.z; x.w += a.w;
      }
      uint16_t* vb = (uint16_t*)(pool + ((size_t)pg * Hkv + kvh) * 2 * kbytes) + kbytes / 2 +
                     ((size_t)(tk >> 3) * d + dim) * 8 + (tk & 7);
      vb[0] = f2bf(x.x);
      vb[8] = f2bf(x.y);
      vb[16] = f2bf(x.z);
      vb[24] = f2bf(x.w);
    }
  }
}

// Per row of fp32 logits: the emitted-token candidate and a log-sum-exp.
//   greedy (inv_temp == 0): arg-max with the lowest index on ties, lse of the logits;
//   sampling: Gumbel-max draw from softmax(logits * inv_temp) -- argmax_j logits_j * inv_temp - log(-log u_j), with
//   u_j from Philox4x32-10 at counter (j, token index, seq_id) under the sample seed -- and the lse of the scaled logits.
__global__ __launch_bounds__(1024) void k_argmax_lse(const float* __restrict__ logits, int V, int* __restrict__ row_argmax,
                                                     float* __restrict__ row_lse, float* __restrict__ row_ztok,
                                                     float* __restrict__ row_zeos, int eos_id, float inv_temp,
                                                     unsigned long long seed, const int* __restrict__ row_slot,
                                                     const int* __restrict__ slot_seq,
                                                     const unsigned long long* __restrict__ seq_id,
                                                     const int* __restrict__ seq_gen_len) {
  __shared__ float s_val[16];
  __shared__ int s_idx[16];
  __shared__ float s_sum[16];
  __shared__ float s_max[16];
  const float* x = logits + (size_t)blockIdx.x * V;
  const bool sampling = inv_temp > 0.f;
  const float scale = sampling ? inv_temp : 1.f;
  uint32_t tok_index = 0;
  unsigned long long id = 0;
  if (sampling) {
    const int sidx = slot_seq[row_slot[blockIdx.x]];
    id = seq_id[sidx];
    tok_index = (uint32_t)seq_gen_len[sidx];
  }
  float best = -INFINITY, mx = -INFINITY;
  int bi = 0x7fffffff;
  // every thread walks its elements in ascending index order, so its first hit is its lowest index
  auto visit = [&](int i, float xi) {
    const float z = xi * scale;
    mx = fmaxf(mx, z);
    float v = z;
    if (sampling) v = z - __logf(-__logf(gumbel_uniform((uint32_t)i, tok_index, id, seed)));
    if (v > best) { best = v; bi = i; }
  };
  const bool vec = (V & 3) == 0;     // rows are 16-byte aligned: four vectors of four logits in flight per thread
  const int nv = V >> 2;
  if (vec) {
    int i = threadIdx.x;
    for (; i + 3 * 1024 < nv; i += 4 * 1024) {
      float4 t[4];
#pragma unroll
      for (int j = 0; j < 4; ++j) t[j] = ((const float4*)x)[i + j * 1024];
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int e = (i + j * 1024) * 4;
        visit(e, t[j].x); visit(e + 1, t[j].y); visit(e + 2, t[j].z); visit(e + 3, t[j].w);
      }
    }
    for (; i < nv; i += 1024) {
      const float4 t = ((const float4*)x)[i];
      visit(i * 4, t.x); visit(i * 4 + 1, t.y); visit(i * 4 + 2, t.z); visit(i * 4 + 3, t.w);
    }
  } else {
    for (int i = threadIdx.x; i < V; i += 1024) visit(i, x[i]);
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    const float ov = __shfl_xor(best, o, 64);
    const int oi = __shfl_xor(bi, o, 64);
    if (ov > best || (ov == best && oi < bi)) { best = ov; bi = oi; }
    mx = fmaxf(mx, __shfl_xor(mx, o, 64));
  }
  const int w = threadIdx.x >> 6;
  if ((threadIdx.x & 63) == 0) { s_val[w] = best; s_idx[w] = bi; s_max[w] = mx; }
  __syncthreads();
  best = s_val[0]; bi = s_idx[0]; mx = s_max[0];
  for (int k = 1; k < 16; ++k) {
    if (s_val[k] > best || (s_val[k] == best && s_idx[k] < bi)) { best = s_val[k]; bi = s_idx[k]; }
    mx = fmaxf(mx, s_max[k]);
  }
  float sum = 0.f;
  if (vec) {
    int i = threadIdx.x;
    for (; i + 3 * 1024 < nv; i += 4 * 1024) {
      float4 t[4];
#pragma unroll
      for (int j = 0; j < 4; ++j) t[j] = ((const float4*)x)[i + j * 1024];
#pragma unroll
      for (int j = 0; j < 4; ++j)
        sum += __expf(t[j].x * scale - mx) + __expf(t[j].y * scale - mx) + __expf(t[j].z * scale - mx) + __expf(t[j].w * scale - mx);
    }
    for (; i < nv; i += 1024) {
      const float4 t = ((const float4*)x)[i];
      sum += __expf(t.x * scale - mx) + __expf(t.y * scale - mx) + __expf(t.z * scale - mx) + __expf(t.w * scale - mx);
    }
  } else {
    for (int i = threadIdx.x; i < V; i += 1024) sum += __expf(x[i] * scale - mx);
  }
  sum = wave_sum(sum);
  if ((threadIdx.x & 63) == 0) s_sum[w] = sum;
  __syncthreads();
  if (threadIdx.x == 0) {
    float t = 0.f;
    for (int k = 0; k < 16; ++k) t += s_sum[k];
    row_argmax[blockIdx.x] = bi;
    row_lse[blockIdx.x] = mx + __logf(t);
    row_ztok[blockIdx.x] = x[bi] * scale;
    row_zeos[blockIdx.x] = x[eos_id] * scale;
  }
}

__global__ __launch_bounds__(256) void k_gather_rows(const float* __restrict__ src, const int* __restrict__ src_row,
                                                     float* __restrict__ dst, int dst_row0, int D) {
  const float* s = src + (size_t)src_row[blockIdx.x] * D;
  float* t = dst + (size_t)(dst_row0 + blockIdx.x) * D;
  for (int i = threadIdx.x; i < D; i += 256) t[i] = s[i];
}

// Weight repacking at init: dst[row0 + (r / blk) * blk_stride + r % blk][c] = convert(src[r][c]).
__global__ __launch_bounds__(256) void k_repack(const void* __restrict__ src, int src_fp32, void* __restrict__ dst,
                                                int dst_fp32, size_t rows, size_t cols, size_t row0, size_t blk,
                                                size_t blk_stride) {
  const size_t total = rows * cols;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (size_t)gridDim.x * 256) {
    const size_t r = i / cols, c = i % cols;
    const size_t o = (row0 + (r / blk) * blk_stride + r % blk) * cols + c;
    if (dst_fp32) {
      ((float*)dst)[o] = src_fp32 ? ((const float*)src)[i] : bf2f(((const uint16_t*)src)[i]);
    } else {
      ((uint16_t*)dst)[o] = src_fp32 ? f2bf(((const float*)src)[i]) : ((const uint16_t*)src)[i];
    }
  }
}

// Plain streaming kernels used to calibrate the memory counters and to measure the practical HBM ceiling.
__global__ __launch_bounds__(256) void k_stream_copy(const uint4* __restrict__ src, uint4* __restrict__ dst, size_t n16) {
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += (size_t)gridDim.x * 256) dst[i] = src[i];
}
__global__ __launch_bounds__(256) void k_stream_read(const uint4* __restrict__ src, size_t n16, uint32_t* __restrict__ sink) {
  uint32_t acc = 0;
  const size_t stride = (size_t)gridDim.x * 256;
  size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  for (; i + 3 * stride < n16; i += 4 * stride) {       // four streaming loads in flight per lane
    uint4 v[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) v[u] = ld_stream16(src + i + u * stride);
#pragma unroll
    for (int u = 0; u < 4; ++u) acc ^= v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
  }
  for (; i < n16; i += stride) {
    const uint4 v = ld_stream16(src + i);
    acc ^= v.x ^ v.y ^ v.z ^ v.w;
  }
  if (acc == 0x9E3779B9u) sink[0] = acc;   // practically never taken; keeps the loads alive
}
void launch_stream_copy(const void* src, void* dst, size_t bytes, hipStream_t st) {
  const size_t n16 = bytes / 16;
  if (n16) hipLaunchKernelGGL(k_stream_copy, dim3(256 * 16), dim3(256), 0, st, (const uint4*)src, (uint4*)dst, n16);
}
void launch_stream_read(const void* src, size_t bytes, void* sink, hipStream_t st) {
  const size_t n16 = bytes / 16;
  if (n16) hipLaunchKernelGGL(k_stream_read, dim3(65536), dim3(256), 0, st, (const uint4*)src, n16, (uint32_t*)sink);
}

// ---------------------------------------------------------------------------------------------------
void launch_repack(const void* src, int src_fp32, void* dst, int dst_fp32, size_t rows, size_t cols, size_t row0,
                   size_t blk, size_t blk_stride, hipStream_t st) {
  const size_t total = rows * cols;
  if (total == 0) return;
  const size_t want = (total + 255) / 256;
  const unsigned blocks = (unsigned)(want < 262144 ? want : 262144);
  hipLaunchKernelGGL(k_repack, dim3(blocks), dim3(256), 0, st, src, src_fp32, dst, dst_fp32, rows, cols, row0, blk,
                     blk_stride);
}
void launch_embed(const void* table, const int* row_tok, float* h, int R, int D, hipStream_t st) {
  if (R > 0) hipLaunchKernelGGL(k_embed, dim3(R), dim3(256), 0, st, (const uint16_t*)table, row_tok, h, D);
}
void launch_add_rmsnorm(float* h, const float* part, int S, size_t part_stride, const float* gain, float eps, void* x,
                        int R, int D, hipStream_t st) {
  if (R > 0)
    hipLaunchKernelGGL(k_add_rmsnorm, dim3(R), dim3(1024), 0, st, h, part, S, part_stride, gain, eps, (uint16_t*)x, D);
}
void launch_rope_kvwrite(const float* part, int S, size_t part_stride, const float* bias, const int* row_slot,
                         const int* row_pos, const void* cs_table, void* q_out, void* pool, const int* page_table,
                         int max_pages, int Hq, int Hkv, int d, int R, hipStream_t st) {
  if (R > 0)
    hipLaunchKernelGGL(k_rope_kvwrite, dim3(R), dim3(1024), 0, st, part, S, part_stride, bias, row_slot, row_pos,
                       (const float2*)cs_table, (uint16_t*)q_out, (uint8_t*)pool, page_table, max_pages, Hq, Hkv, d);
}
void launch_argmax_lse(const float* logits, int V, int* row_argmax, float* row_lse, float* row_ztok, float* row_zeos, int R,
                       const SchedDev* sched, hipStream_t st) {
  if (R > 0)
    hipLaunchKernelGGL(k_argmax_lse, dim3(R), dim3(1024), 0, st, logits, V, row_argmax, row_lse, row_ztok, row_zeos,
                       sched->eos_id, sched->inv_temp, sched->sample_seed, sched->row_slot, sched->slot_seq, sched->seq_id,
                       sched->seq_gen_len);
}

// Combine the per-tile records the fused LM head left for each row (ascending column order: the first maximum a thread
// meets is its lowest index, and equal scores across threads go to the lower index).
__global__ __launch_bounds__(256) void k_lm_reduce(const float4* __restrict__ part_f, const int* __restrict__ part_i,
                                                   int n_tiles, int* __restrict__ row_argmax,
                                                   float* __restrict__ row_ztok, float* __restrict__ row_lse) {
  __shared__ float s_v[4], s_z[4], s_m[4], s_s[4];
  __shared__ int s_i[4];
  const int r = blockIdx.x;
  float bv = -INFINITY, bz = 0.f, mx = -INFINITY, sum = 0.f;
  int bi = 0x7fffffff;
  for (int t = threadIdx.x; t < n_tiles; t += 256) {
    const float4 f = part_f[(size_t)r * n_tiles + t];
    const int i = part_i[(size_t)r * n_tiles + t];
    if (f.x > bv || (f.x == bv && i < bi)) { bv = f.x; bi = i; bz = f.y; }
    const float m2 = fmaxf(mx, f.z);
    if (m2 > -INFINITY) sum = sum * __expf(mx - m2) + f.w * __expf(f.z - m2);
    mx = m2;
  }
  auto merge = [&](float ov, int oi, float oz, float om, float os) {
    if (ov > bv || (ov == bv && oi < bi)) { bv = ov; bi = oi; bz = oz; }
    const float m2 = fmaxf(mx, om);
    if (m2 > -INFINITY) sum = sum * __expf(mx - m2) + os * __expf(om - m2);
    mx = m2;
  };
#pragma unroll
  for (int o = 32; o > 0; o >>= 1)
    merge(__shfl_xor(bv, o, 64), __shfl_xor(bi, o, 64), __shfl_xor(bz, o, 64), __shfl_xor(mx, o, 64), __shfl_xor(sum, o, 64));
  const int w = threadIdx.x >> 6;
  if ((threadIdx.x & 63) == 0) { s_v[w] = bv; s_i[w] = bi; s_z[w] = bz; s_m[w] = mx; s_s[w] = sum; }
  __syncthreads();
  if (threadIdx.x == 0) {
    bv = s_v[0]; bi = s_i[0]; bz = s_z[0]; mx = s_m[0]; sum = s_s[0];
    for (int k = 1; k < 4; ++k) merge(s_v[k], s_i[k], s_z[k], s_m[k], s_s[k]);
    row_argmax[r] = bi;
    row_ztok[r] = bz;
    row_lse[r] = mx + __logf(sum);
  }
}
void launch_lm_reduce(const LmEpi& epi, int M, int* row_argmax, float* row_ztok, float* row_lse, hipStream_t st) {
  if (M > 0)
    hipLaunchKernelGGL(k_lm_reduce, dim3(M), dim3(256), 0, st, (const float4*)epi.part_f, (const int*)epi.part_i, epi.n_tiles,
                       row_argmax, row_ztok, row_lse);
}
void launch_gather_rows(const float* src, const int* src_row, float* dst, int dst_row0, int n, int D, hipStream_t st) {
  if (n > 0) hipLaunchKernelGGL(k_gather_rows, dim3(n), dim3(256), 0, st, src, src_row, dst, dst_row0, D);
}
