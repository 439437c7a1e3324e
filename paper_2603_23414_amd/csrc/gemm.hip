// bf16 MFMA projection GEMM for gfx950: C[M,N] (fp32) = A[M,K] (bf16, row-major) * W[N,K]^T (bf16, row-major).
//
// In decode M = running slots (<= 256), so every projection is a weight stream: each weight byte is read
// once and the MFMA work per byte is ~M flop, at or below the machine's ridge.  The kernel is built around
// that: a workgroup owns 128 output columns and all (<= 256) rows; each of its 4 wavefronts owns 32 columns
// and reads its W fragments straight from global memory in the v_mfma_f32_32x32x16_bf16 operand layout
// (lane -> row n, 16 contiguous bytes along K), so no weight byte is loaded twice or staged through LDS.
// Only the small activation tile A goes through LDS (rows padded to 144 bytes, or xor-swizzled where the tile
// is loaded global -> LDS directly, so that the 16-byte fragment reads are bank-conflict free).  Split-K over
// blockIdx.z writes fp32 partial sums that the consumer kernels (residual+norm, RoPE, SiLU*mul) add up in a
// fixed order, so results are deterministic.
//
// Two things about the k loops that the timings depend on and the source does not otherwise show:
//  - the compiler's wait-count pass merges the load-queue states of every path into a block.  A loop that may leave
//    after every block of its unrolled ring, or a prologue that issues its loads in another order than an iteration
//    does, makes it wait for (nearly) the whole queue at the top of some blocks.  So the loops run full groups of blocks
//    with no test in between, handle the last few blocks separately, and the prologues mimic an iteration's order;
//  - prefetches that would reach past a launch's last k block are issued against a buffer descriptor with zero records
//    (the range check then returns zeros without a memory access, and the load still counts in vmcnt), which keeps the
//    loops free of conditional loads without fetching the last block again and again.
#include <cstdio>
#include <type_traits>

#include "common.h"
#include "kernels.h"

#define GEMM_BK 64
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// Packed weight layout ("W fragments"): the matrix is cut into tiles of 32 rows (n) x 64 columns (k); tile
// (nt, kb) holds 4 k-steps x 64 lanes x 8 bf16, lane l of k-step j carrying W[nt*32 + l%32][kb*64 + (l/32)*32 + j*8 .. +8].
// A wavefront's 16-byte-per-lane load of one k-step is then one contiguous KiB (fully coalesced), where the same
// fragment read from a row-major matrix touches 32 different rows; that was the decode GEMM's real limit (address
// processing in the texture path, not HBM, LDS or MFMA).  Rows are padded with zeros to a multiple of 32.
#define WTILE_ELEMS 2048   // bf16 elements per (nt, kb) tile

#ifndef GEMM_STAGE_MI1      // k blocks per activation stage of k_gemm_bf16 at 32 / 64 / 128 rows
#define GEMM_STAGE_MI1 4
#endif
#ifndef GEMM_STAGE_MI2
#define GEMM_STAGE_MI2 2
#endif
#ifndef GEMM_STAGE_MI4
#define GEMM_STAGE_MI4 2
#endif
#define LDS_ROW 72   // bf16 elements per LDS row: 64 + 8 padding (144-byte stride: conflict-free 16-byte reads)

// One k-step pairs MFMA k index (lane/32)*8 + e with memory k = (lane/32)*32 + j*8 + e inside the 64-wide block,
// for A and W alike, so that every lane's four W loads of a block are 64 contiguous bytes (a row's two lanes
// cover a whole 128-byte line per block).
// EPI = 0: fp32 store of the (partial) sums.  EPI = 1: the SwiGLU epilogue -- W holds gate and up rows interleaved
// in blocks of 16 (cols 32q..32q+15 = gate of features 16q.., cols 32q+16..32q+31 = up of the same features), the
// two halves of a wave's 32 columns meet through one cross-lane exchange, and bf16 silu(gate)*up goes to
// act[M, N/2].  No split-K in that mode.
// STREAM = true reads W with streaming loads (the nt bit of the buffer load): right when every weight byte is used once per launch
// (M <= 256), wrong when several row blocks re-read the same W slab from L2 (prefill).
// EPI = 2 (greedy) / 3 (sampling): the LM head with the emit statistics in its epilogue (no logits are stored).  The two MFMA operands are
// swapped, which transposes the accumulator tile at no cost (both fragments have the same register layout): a lane
// then owns ONE row (lane % 32) and 16 of the wave's 32 columns, so the per-row arg-max / Gumbel-max draw, the
// maximum and the sum of exponentials are plain per-lane loops over registers; the two half-waves, then the four
// wavefronts, are merged in ascending column order, and the workgroup leaves one record per row.
template <int MI, int EPI, bool STREAM>
__global__ __launch_bounds__(256, 2) void k_gemm_bf16(const uint16_t* __restrict__ A, const uint16_t* __restrict__ W,
                                                      float* __restrict__ C, int M, int N, int K, int kb_per_split,
                                                      LmEpi lm) {
  constexpr int BM = 32 * MI;
  // The activation tile is staged SB k blocks at a time (global -> registers -> LDS, double-buffered), so the wait for
  // its loads and the workgroup barrier come once per SB blocks.  With one block per stage every iteration of a
  // small-M launch lasted one L2 round trip (0.7 us for 16 KiB of weights per workgroup): that chain, not the weight
  // stream, set the speed of the decode projections at M <= 128.  The W ring's depth is a multiple of SB so that a
  // block's position inside its stage is a compile-time constant.
  constexpr int SB = MI == 1 ? GEMM_STAGE_MI1 : MI == 2 ? GEMM_STAGE_MI2 : MI == 4 ? GEMM_STAGE_MI4 : 1;
  constexpr int RD = SB == 1 ? 3 : (SB == 2 ? 4 : SB);
  __shared__ __align__(16) uint16_t a_lds[2][SB][BM * LDS_ROW];
  const int tid = threadIdx.x, lane = tid & 63;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int n_base = blockIdx.x * 128 + w * 32;
  const int m_base = blockIdx.y * BM;
  const int nkb_total = K / GEMM_BK;
  const int kb0 = blockIdx.z * kb_per_split;
  const int nkb = min(kb_per_split, nkb_total - kb0);
  float* __restrict__ Cz = C + (size_t)blockIdx.z * M * N;

  // Operands are fetched with buffer loads: this row block of A and this wave's tile row of W (32 rows, clamped past the
  // edge: loaded, never stored) each get a descriptor, every offset used below stays inside it, and a prefetch that would
  // reach past the launch's last k block is issued against an EMPTY descriptor instead (zero records: the range check
  // returns zeros without touching memory, and the load still counts in the wave's load counter) -- the loop keeps its
  // fixed shape with no conditional register writes, and a short split-K range does not fetch its last block three
  // times over.
  const int nt = min(n_base, N - 1) >> 5;
  const int rows_here = min(BM, M - m_base);
  const uint16_t* a_base = A + (size_t)m_base * K;
  const uint16_t* w_base = W + (size_t)nt * nkb_total * WTILE_ELEMS;
  const int a_bytes = rows_here * K * 2, w_bytes = nkb_total * (WTILE_ELEMS * 2);
#define GEMM_RS_A(live) __builtin_amdgcn_make_buffer_rsrc((void*)a_base, 0, (live) ? a_bytes : 0, 0x00020000)
#define GEMM_RS_W(live) __builtin_amdgcn_make_buffer_rsrc((void*)w_base, 0, (live) ? w_bytes : 0, 0x00020000)
#define GEMM_LDW(rs, kb_, j) \
  __builtin_amdgcn_raw_buffer_load_b128(rs, w_voff + (j) * 1024, (kb0 + (kb_)) * (WTILE_ELEMS * 2), STREAM ? 2 : 0)
#define GEMM_LDA(rs, i, kb_) __builtin_amdgcn_raw_buffer_load_b128(rs, a_voff[i], (kb0 + (kb_)) * (GEMM_BK * 2), 0)
  const int w_voff = lane * 16;

  const int a_col = tid & 7;
  int a_voff[MI];
  int a_dst[MI];
#pragma unroll
  for (int i = 0; i < MI; ++i) {
    const int r = (tid >> 3) + i * 32;
    a_voff[i] = min(r, rows_here - 1) * K * 2 + a_col * 16;    // rows past M: the last row again (computed, never stored)
    a_dst[i] = r * LDS_ROW + a_col * 8;
  }
  const int a_frag = (lane & 31) * LDS_ROW + (lane >> 5) * 32;

  f32x16_t acc[MI];
#pragma unroll
  for (int i = 0; i < MI; ++i)
#pragma unroll
    for (int j = 0; j < 16; ++j) acc[i][j] = 0.f;

  u32x4 breg[RD][4];   // ring over k blocks; every index below is a compile-time constant after unrolling
  u32x4 areg[SB][MI];
#pragma unroll
  for (int s = 0; s < SB; ++s) {
    const __amdgpu_buffer_rsrc_t rs = GEMM_RS_A(s < nkb);
#pragma unroll
    for (int i = 0; i < MI; ++i) areg[s][i] = GEMM_LDA(rs, i, min(s, nkb - 1));
  }
#pragma unroll
  for (int r = 0; r < RD - 1; ++r) {
    const __amdgpu_buffer_rsrc_t rs = GEMM_RS_W(r < nkb);
#pragma unroll
    for (int j = 0; j < 4; ++j) breg[r][j] = GEMM_LDW(rs, min(r, nkb - 1), j);
  }
#pragma unroll
  for (int s = 0; s < SB; ++s)
#pragma unroll
    for (int i = 0; i < MI; ++i) *(u32x4*)&a_lds[0][s][a_dst[i]] = areg[s][i];
  __syncthreads();

  // one k block; u = kb % RD is a compile-time constant (ring slot, position inside the activation stage)
  auto block = [&](auto uc, const int kb) __attribute__((always_inline)) {
    constexpr int u = decltype(uc)::value;
    constexpr int pos = u % SB;                          // a group starts at a multiple of RD, RD is a multiple of SB
    const int cur = (kb / SB) & 1;
    // prefetch: the next stage of A at the first block of a stage (to registers, then LDS), W RD - 1 blocks ahead
    // (register ring); past the launch's last block the loads go against the empty descriptor
    if (pos == 0) {
#pragma unroll
      for (int s = 0; s < SB; ++s) {
        const __amdgpu_buffer_rsrc_t rs = GEMM_RS_A(kb + SB + s < nkb);
#pragma unroll
        for (int i = 0; i < MI; ++i) areg[s][i] = GEMM_LDA(rs, i, min(kb + SB + s, nkb - 1));
      }
    }
    {
      const __amdgpu_buffer_rsrc_t rs = GEMM_RS_W(kb + RD - 1 < nkb);
#pragma unroll
      for (int j = 0; j < 4; ++j) breg[(u + RD - 1) % RD][j] = GEMM_LDW(rs, min(kb + RD - 1, nkb - 1), j);
    }
    __builtin_amdgcn_sched_barrier(0);   // keep the prefetch loads ahead of this block's MFMAs
    const uint16_t* al = a_lds[cur][pos] + a_frag;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const bf16x8_t bf = __builtin_bit_cast(bf16x8_t, breg[u][j]);
#pragma unroll
      for (int i = 0; i < MI; ++i) {
        const u32x4 av = *(const u32x4*)(al + i * 32 * LDS_ROW + j * 8);
        if (EPI >= 2) acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bf, __builtin_bit_cast(bf16x8_t, av), acc[i], 0, 0, 0);
        else acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, av), bf, acc[i], 0, 0, 0);
      }
    }
    if (pos == SB - 1) {                                 // the stage is used up: publish the next one
#pragma unroll
      for (int s = 0; s < SB; ++s)
#pragma unroll
        for (int i = 0; i < MI; ++i) *(u32x4*)&a_lds[cur ^ 1][s][a_dst[i]] = areg[s][i];
      __syncthreads();
    }
  };
  // Full groups of RD blocks run without a test between the blocks (with an exit after every block the compiler's
  // wait-count pass merges the states of all those paths and drains most of the W ring once per group); the last
  // blocks follow, each behind its test.
  static_assert(RD == 3 || RD == 4, "the group calls below are written out for a ring of 3 or 4");
  int kbase = 0;
  for (; kbase + RD <= nkb; kbase += RD) {
    block(std::integral_constant<int, 0>{}, kbase);
    block(std::integral_constant<int, 1>{}, kbase + 1);
    block(std::integral_constant<int, 2>{}, kbase + 2);
    if constexpr (RD == 4) block(std::integral_constant<int, 3>{}, kbase + 3);
  }
  if (kbase < nkb) {
    block(std::integral_constant<int, 0>{}, kbase);
    if (kbase + 1 < nkb) {
      block(std::integral_constant<int, 1>{}, kbase + 1);
      if constexpr (RD == 4) {
        if (kbase + 2 < nkb) block(std::integral_constant<int, 2>{}, kbase + 2);
      }
    }
  }

#undef GEMM_LDA
#undef GEMM_LDW
#undef GEMM_RS_W
#undef GEMM_RS_A
  if (EPI >= 2) {
    constexpr bool SAMPLING = EPI == 3;                   // a separate instantiation: the generator is 128 x inlined
    // transposed tile: element j of lane -> column n_base + (j/4)*8 + (lane/32)*4 + j%4 (ascending in j), row lane%32
    if (SB > 1) __syncthreads();                          // a launch may end in the middle of a stage: no wave still reads A
    float* rec_f = (float*)&a_lds[0][0][0];               // [4 waves][BM rows][4]; the A tiles are dead (last barrier passed)
    int* rec_i = (int*)(rec_f + 4 * BM * 4);              // [4 waves][BM rows]
#pragma unroll
    for (int i = 0; i < MI; ++i) {
      const int m = m_base + i * 32 + (lane & 31);
      uint32_t tok_index = 0;
      unsigned long long sid = 0;
      if (SAMPLING && m < M) {
        const int sidx = lm.slot_seq[lm.row_slot[m]];
        sid = lm.seq_id[sidx];
        tok_index = (uint32_t)lm.seq_gen_len[sidx];
      }
      float bv = -INFINITY, bz = 0.f, mx = -INFINITY;
      int bi = 0x7fffffff;
      float z[16];
#pragma unroll
      for (int j = 0; j < 16; ++j) {
        const int n = n_base + (j >> 2) * 8 + (lane >> 5) * 4 + (j & 3);
        const bool valid = n < N;
        const float zz = valid ? acc[i][j] * lm.scale : -INFINITY;
        float v = zz;
        if (SAMPLING && valid) v = zz - __logf(-__logf(gumbel_uniform((uint32_t)n, tok_index, sid, lm.seed)));
        if (v > bv) { bv = v; bi = n; bz = zz; }          // ascending columns: the first maximum is the lowest index
        mx = fmaxf(mx, zz);
        z[j] = zz;
        if (n == lm.eos_id && m < M) lm.row_zeos[m] = zz;
      }
      float sum = 0.f;
      if (mx > -INFINITY) {
#pragma unroll
        for (int j = 0; j < 16; ++j) sum += __expf(z[j] - mx);   // exp(-inf) = 0 for columns past the vocabulary
      }
      // the other half-wave holds the interleaved other 16 columns of the same row
      {
        const float ov = __shfl_xor(bv, 32, 64), oz = __shfl_xor(bz, 32, 64), om = __shfl_xor(mx, 32, 64),
                    os = __shfl_xor(sum, 32, 64);
        const int oi = __shfl_xor(bi, 32, 64);
        if (ov > bv || (ov == bv && oi < bi)) { bv = ov; bi = oi; bz = oz; }
        const float m2 = fmaxf(mx, om);
        if (m2 > -INFINITY) sum = sum * __expf(mx - m2) + os * __expf(om - m2);
        mx = m2;
      }
      if (lane < 32) {
        const int row = i * 32 + lane;
        *(float4*)(rec_f + ((size_t)w * BM + row) * 4) = make_float4(bv, bz, mx, sum);
        rec_i[w * BM + row] = bi;
      }
    }
    __syncthreads();
    if (tid < BM && m_base + tid < M) {                    // one thread per row: the four wavefronts in column order
      float4 f = *(const float4*)(rec_f + (size_t)tid * 4);
      int bi = rec_i[tid];
#pragma unroll
      for (int u = 1; u < 4; ++u) {
        const float4 o = *(const float4*)(rec_f + ((size_t)u * BM + tid) * 4);
        const int oi = rec_i[u * BM + tid];
        if (o.x > f.x || (o.x == f.x && oi < bi)) { f.x = o.x; f.y = o.y; bi = oi; }
        const float m2 = fmaxf(f.z, o.z);
        if (m2 > -INFINITY) f.w = f.w * __expf(f.z - m2) + o.w * __expf(o.z - m2);
        f.z = m2;
      }
      const size_t o = (size_t)(m_base + tid) * lm.n_tiles + blockIdx.x;
      lm.part_f[o] = f;
      lm.part_i[o] = bi;
    }
    return;
  }
  // C fragment: element j of lane -> row (j/4)*8 + (lane/32)*4 + j%4, col lane%32
  const int n_out = n_base + (lane & 31);
  if (EPI == 1) {
    uint16_t* __restrict__ act = (uint16_t*)C;
    const int F = N >> 1;
    const int f_out = (n_base >> 1) + (lane & 15);
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
      for (int j = 0; j < 16; ++j) {
        const float mine = acc[i][j];
        const float other = __shfl_xor(mine, 16, 64);     // gate lanes (bit 4 clear) receive the up value
        const int mrow = m_base + i * 32 + (j >> 2) * 8 + (lane >> 5) * 4 + (j & 3);
        if ((lane & 16) == 0 && mrow < M && n_out < N)
          act[(size_t)mrow * F + f_out] = f2bf(mine / (1.0f + __expf(-mine)) * other);
      }
  } else if (n_out < N) {
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
      for (int j = 0; j < 16; ++j) {
        const int mrow = m_base + i * 32 + (j >> 2) * 8 + (lane >> 5) * 4 + (j & 3);
        if (mrow < M) Cz[(size_t)mrow * N + n_out] = acc[i][j];
      }
  }
}

// Variant for launches that cannot fill the chip twice over (<= ~1 workgroup per CU, i.e. every decode projection
// except the LM head): one workgroup per CU gets the whole register file (accumulators in AGPRs) and 128 KiB of LDS.
// A wave owns 8 x 1 MFMA tiles (256 rows x 32 columns).  The activation tile travels global memory -> LDS directly
// (buffer loads with the LDS flag: no staging registers, no LDS write instructions), four 32 KiB tiles deep: block
// kb + 3 is in flight while block kb is multiplied.  The W ring in registers runs three blocks ahead (loads complete
// in issue order, so a deeper ring than the tiles' would buy nothing).  The MFMA stream is continuous across the
// barrier: the next block's first fragments are read during the last k-step, and the fragments of k-step j + 1 while
// k-step j is multiplied.  A wave's LDS-direct load fills one contiguous KiB, so the tile cannot be padded; it is
// xor-swizzled instead: 16-byte chunk c of row r sits at chunk c ^ ((r ^ (r >> 3)) & 7) (conflict-free fragment reads).
// The four tiles are four separate arrays on purpose: the compiler's wait-count pass tells in-flight LDS-direct loads
// from LDS reads by the array they address, so fragment reads of one tile do not wait for the loads into another.
#define DEEP_TILE (256 * 64)
#ifndef DEEP_WAIT_VM
#define DEEP_WAIT_VM 16
#endif
typedef __attribute__((address_space(3))) void* lds_ptr_t;
template <int EPI>
__global__ __launch_bounds__(256, 1) void k_gemm_bf16_deep(const uint16_t* __restrict__ A, const uint16_t* __restrict__ W,
                                                           float* __restrict__ C, int M, int N, int K, int kb_per_split) {
  __shared__ __align__(1024) uint16_t a0[DEEP_TILE];
  __shared__ __align__(1024) uint16_t a1[DEEP_TILE];
  __shared__ __align__(1024) uint16_t a2[DEEP_TILE];
  __shared__ __align__(1024) uint16_t a3[DEEP_TILE];
#define DEEP_SEL(b) ((b) == 0 ? a0 : (b) == 1 ? a1 : (b) == 2 ? a2 : a3)   // b is a constant after unrolling
  const int tid = threadIdx.x, lane = tid & 63;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int n_base = blockIdx.x * 128 + w * 32;
  const int m_base = blockIdx.y * 256;
  const int nkb_total = K / GEMM_BK;
  const int kb0 = blockIdx.z * kb_per_split;
  const int nkb = min(kb_per_split, nkb_total - kb0);
  float* __restrict__ Cz = C + (size_t)blockIdx.z * M * N;
  // buffer descriptors: this row block of A, this wave's tile row of W (32 rows, clamped past the edge: loaded, never
  // stored).  Every offset below stays inside them; the hardware range check is only a second line of defence.
  // A prefetch that would reach past the launch's last k block goes against an EMPTY descriptor (zero records: the range
  // check answers with zeros and no memory access, and the load still counts in the wave's load counter), so the loop keeps
  // its fixed shape and its hand-counted waits while a short split-K range does not fetch its last block four times.
  const int rows_here = min(256, M - m_base);
  const uint16_t* a_base = A + (size_t)m_base * K;
  const uint16_t* w_base = W + (size_t)(min(n_base, N - 1) >> 5) * nkb_total * WTILE_ELEMS;
  const int a_bytes = rows_here * K * 2, w_bytes = nkb_total * (WTILE_ELEMS * 2);
#define DEEP_RS_A(live) __builtin_amdgcn_make_buffer_rsrc((void*)a_base, 0, (live) ? a_bytes : 0, 0x00020000)
#define DEEP_RS_W(live) __builtin_amdgcn_make_buffer_rsrc((void*)w_base, 0, (live) ? w_bytes : 0, 0x00020000)
  const int w_so = kb0 * (WTILE_ELEMS * 2);
  const int w_voff = lane * 16;
  // A load i of wave w fills tile rows i*32 + w*8 .. +8: lane -> row l/8, physical chunk l%8 <- logical chunk
  // (l%8) ^ f(row); rows past M are clamped to the last one (computed, never stored)
  const int lrow = w * 8 + (lane >> 3);
  const int a_chunk = ((lane & 7) ^ ((lrow ^ (lrow >> 3)) & 7)) * 16;      // f(row) is the same 32 rows further on
  int a_voff[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) a_voff[i] = min(i * 32 + lrow, rows_here - 1) * K * 2 + a_chunk;
  const int a_so = kb0 * (GEMM_BK * 2);
#define DEEP_LDA(rs, buf, i, kb_)                                                                                \
  __builtin_amdgcn_raw_ptr_buffer_load_lds(rs, (lds_ptr_t)(DEEP_SEL(buf) + ((i) * 32 + w * 8) * 64), 16, a_voff[i], \
                                           a_so + (kb_) * (GEMM_BK * 2), 0, 0)
#define DEEP_LDW(rs, kb_, j) __builtin_amdgcn_raw_buffer_load_b128(rs, w_voff, w_so + (kb_) * (WTILE_ELEMS * 2) + (j) * 1024, 2)
#define DEEP_MFMA8(AF, BF)                                                                                        \
  _Pragma("unroll") for (int i = 0; i < 8; ++i) acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(                  \
      __builtin_bit_cast(bf16x8_t, AF[i]), BF, acc[i], 0, 0, 0)
  // pin the interleave of a k-step: one LDS read and (with_mem) one global load per MFMA or per second MFMA
#define DEEP_PIN(mem_every)                                                                                       \
  _Pragma("unroll") for (int i = 0; i < 8; ++i) {                                                                  \
    __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);                                                             \
    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                                                             \
    if ((mem_every) == 1 || ((mem_every) == 2 && (i & 1))) __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);      \
  }                                                                                                                \
  __builtin_amdgcn_sched_barrier(0);
  // fragment read: row (lane & 31) + 32 i, logical chunk (lane >> 5) * 4 + j
  const int frow = lane & 31;
  const int ff = (frow ^ (frow >> 3)) & 7;
  int a_frag[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) a_frag[j] = frow * 64 + ((((lane >> 5) * 4 + j) ^ ff) * 8);
  f32x16_t acc[8];
#pragma unroll
  for (int i = 0; i < 8; ++i)
#pragma unroll
    for (int j = 0; j < 16; ++j) acc[i][j] = 0.f;
  u32x4 breg[4][4];   // W ring; every index is a compile-time constant after unrolling
  u32x4 af[2][8];     // A fragments of the current and the next k-step
  // prologue: W blocks 0..2, then A blocks 0..2 into tiles 0..2; everything has landed when the loop starts, so the
  // loop is entered in the state its own iterations leave behind
#pragma unroll
  for (int r = 0; r < 3; ++r) {
    const __amdgpu_buffer_rsrc_t rs = DEEP_RS_W(r < nkb);
#pragma unroll
    for (int j = 0; j < 4; ++j) breg[r][j] = DEEP_LDW(rs, min(r, nkb - 1), j);
  }
#pragma unroll
  for (int b = 0; b < 3; ++b) {
    const __amdgpu_buffer_rsrc_t rs = DEEP_RS_A(b < nkb);
#pragma unroll
    for (int i = 0; i < 8; ++i) DEEP_LDA(rs, b, i, min(b, nkb - 1));
  }
  __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0)
  __syncthreads();
#pragma unroll
  for (int i = 0; i < 8; ++i) af[0][i] = *(const u32x4*)(a0 + a_frag[0] + i * 32 * 64);

  // one k block; u = kb % 4 is a compile-time constant (ring slot and LDS tile)
  auto block = [&](auto uc, const int kb) __attribute__((always_inline)) {
    constexpr int u = decltype(uc)::value;
    const uint16_t* al = DEEP_SEL(u % 4);
    const uint16_t* al_next = DEEP_SEL((u + 1) % 4);
    const int k3 = min(kb + 3, nkb - 1);
    const __amdgpu_buffer_rsrc_t a_rs3 = DEEP_RS_A(kb + 3 < nkb), w_rs3 = DEEP_RS_W(kb + 3 < nkb);
    // k-step 0: + A block kb+3 straight into tile (kb+3) % 4 (last read before the previous barrier)
#pragma unroll
    for (int i = 0; i < 8; ++i) af[1][i] = *(const u32x4*)(al + a_frag[1] + i * 32 * 64);
    DEEP_MFMA8(af[0], __builtin_bit_cast(bf16x8_t, breg[u % 4][0]));
#pragma unroll
    for (int i = 0; i < 8; ++i) DEEP_LDA(a_rs3, (u + 3) % 4, i, k3);
    DEEP_PIN(1)
    // k-step 1
#pragma unroll
    for (int i = 0; i < 8; ++i) af[0][i] = *(const u32x4*)(al + a_frag[2] + i * 32 * 64);
    DEEP_MFMA8(af[1], __builtin_bit_cast(bf16x8_t, breg[u % 4][1]));
    DEEP_PIN(0)
    // k-step 2: + W block kb+3
#pragma unroll
    for (int i = 0; i < 8; ++i) af[1][i] = *(const u32x4*)(al + a_frag[3] + i * 32 * 64);
    DEEP_MFMA8(af[0], __builtin_bit_cast(bf16x8_t, breg[u % 4][2]));
#pragma unroll
    for (int j = 0; j < 4; ++j) breg[(u + 3) % 4][j] = DEEP_LDW(w_rs3, k3, j);
    DEEP_PIN(2)
    // k-step 3: first fragments of block kb+1 (published one barrier ago)
#pragma unroll
    for (int i = 0; i < 8; ++i) af[0][i] = *(const u32x4*)(al_next + a_frag[0] + i * 32 * 64);
    DEEP_MFMA8(af[1], __builtin_bit_cast(bf16x8_t, breg[u % 4][3]));
    DEEP_PIN(0)
    // the A tile of block kb+2 (loads issued one iteration ago) must have landed before this barrier publishes it:
    // its first fragments are read during the next iteration's last k-step.  Loads complete in issue order -- A then
    // W in every iteration -- so only the W loads of that iteration (block kb+2, not needed for another two
    // iterations; the compiler waits for those registers itself) and this iteration's 8 A + 4 W loads may still fly
    __builtin_amdgcn_s_waitcnt(0x0F70 | (DEEP_WAIT_VM & 15) | ((DEEP_WAIT_VM >> 4) << 14));
    __builtin_amdgcn_s_barrier();          // no fence: a release fence would wait for this iteration's loads too
    __builtin_amdgcn_sched_barrier(0);
  };
  // Full groups of four blocks run without a test between the blocks: with an exit after every block the compiler's
  // wait-count pass merges the states of all those paths and ends up draining the load queue (vmcnt 0..4) at the top of
  // two blocks in four.  The last one to three blocks follow, each behind its test.
  int kbase = 0;
  for (; kbase + 4 <= nkb; kbase += 4) {
    block(std::integral_constant<int, 0>{}, kbase);
    block(std::integral_constant<int, 1>{}, kbase + 1);
    block(std::integral_constant<int, 2>{}, kbase + 2);
    block(std::integral_constant<int, 3>{}, kbase + 3);
  }
  if (kbase < nkb) {
    block(std::integral_constant<int, 0>{}, kbase);
    if (kbase + 1 < nkb) {
      block(std::integral_constant<int, 1>{}, kbase + 1);
      if (kbase + 2 < nkb) block(std::integral_constant<int, 2>{}, kbase + 2);
    }
  }
  __builtin_amdgcn_s_waitcnt(0x0F70);   // the loads issued past the last block have completed before LDS is given up
#undef DEEP_PIN
#undef DEEP_MFMA8
#undef DEEP_LDW
#undef DEEP_LDA
#undef DEEP_RS_W
#undef DEEP_RS_A
#undef DEEP_SEL

  // C fragment: element j of lane -> row (j/4)*8 + (lane/32)*4 + j%4, col lane%32
  const int n_out = n_base + (lane & 31);
  if (EPI == 1) {
    uint16_t* __restrict__ act = (uint16_t*)C;
    const int F = N >> 1;
    const int f_out = (n_base >> 1) + (lane & 15);
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
      for (int j = 0; j < 16; ++j) {
        const float mine = acc[i][j];
        const float other = __shfl_xor(mine, 16, 64);
        const int mrow = m_base + i * 32 + (j >> 2) * 8 + (lane >> 5) * 4 + (j & 3);
        if ((lane & 16) == 0 && mrow < M && n_out < N)
          act[(size_t)mrow * F + f_out] = f2bf(mine / (1.0f + __expf(-mine)) * other);
      }
  } else if (n_out < N) {
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
      for (int j = 0; j < 16; ++j) {
        const int mrow = m_base + i * 32 + (j >> 2) * 8 + (lane >> 5) * 4 + (j & 3);
        if (mrow < M) Cz[(size_t)mrow * N + n_out] = acc[i][j];
      }
  }
}

// Variant for launches with several row blocks (prefill): a 256 x (64 NT) workgroup tile, NT = 4 or 3, 2 x 2
// wavefronts of 128 x (32 NT) (4 x NT MFMA tiles each), BOTH operands staged through LDS so that every fragment read
// feeds several MFMAs -- half the LDS reads, half the global-load and LDS-write instructions per MFMA of the 256 x 128
// kernels above, which is what bounds those.  The packed W tiles are copied to LDS verbatim (a fragment is then one
// contiguous KiB); the next block's global loads fly while the current one is multiplied; accumulators live in AGPRs.
// The 192-wide tile is for column counts that would leave the last round of 256-wide tiles half empty.
// XMAP: workgroups go to the 8 XCDs (each with its own L2) round-robin in launch order; give every XCD a contiguous
// run of tiles, ordered so that the 32 it runs at a time form 8 row blocks x 4 column blocks (fewer distinct operand
// slabs per k block through that L2).
#define BIG_A_ELEMS (256 * LDS_ROW)
#define BIG_LDS_BYTES(NT) (2 * (BIG_A_ELEMS + 2 * (NT) * WTILE_ELEMS) * 2)
template <int EPI, int NT, bool XMAP>
__global__ __launch_bounds__(256, 1) void k_gemm_bf16_big(const uint16_t* __restrict__ A, const uint16_t* __restrict__ W,
                                                          float* __restrict__ C, int M, int N, int K, int kb_per_split) {
  extern __shared__ __align__(16) uint16_t big_lds[];   // [2][A tile | W tiles]
  constexpr int BUF_ELEMS = BIG_A_ELEMS + 2 * NT * WTILE_ELEMS;
  const int tid = threadIdx.x, lane = tid & 63;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = w & 1, wn = w >> 1;
  int tx = blockIdx.x, ty = blockIdx.y, tz = blockIdx.z;
  if (XMAP) {
    const int gx = gridDim.x, gy = gridDim.y, T = gx * gy * gridDim.z;
    const int lin = blockIdx.x + gx * (blockIdx.y + gy * blockIdx.z);
    const int xcd = lin & 7, local = lin >> 3, q = T >> 3, r = T & 7;
    const int logical = xcd < r ? xcd * (q + 1) + local : r * (q + 1) + (xcd - r) * q + local;
    tz = logical / (gx * gy);
    const int id = logical - tz * gx * gy;
    const int g = id / (8 * gx), first = g * 8, gs = min(gy - first, 8), in = id - g * 8 * gx;
    ty = first + in % gs;
    tx = in / gs;
  }
  const int n_base = tx * (64 * NT);
  const int m_base = ty * 256;
  const int nkb_total = K / GEMM_BK;
  const int kb0 = tz * kb_per_split;
  const int nkb = min(kb_per_split, nkb_total - kb0);
  float* __restrict__ Cz = C + (size_t)tz * M * N;
  // global -> LDS copy plan: 8 A chunks (rows tid/8 + 32 i, 16-byte column tid%8) and 2 NT W chunks (tile i, chunk tid)
  const int a_col = tid & 7;
  const uint16_t* a_src[8];
  const uint16_t* w_src[2 * NT];
  int a_dst[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const int r = (tid >> 3) + i * 32;
    a_src[i] = A + (size_t)min(m_base + r, M - 1) * K + (size_t)kb0 * GEMM_BK + a_col * 8;
    a_dst[i] = r * LDS_ROW + a_col * 8;
  }
#pragma unroll
  for (int i = 0; i < 2 * NT; ++i) {
    const int nt = min(n_base + i * 32, N - 1) >> 5;             // clamped past the edge: loaded, never stored
    w_src[i] = W + ((size_t)nt * nkb_total + kb0) * WTILE_ELEMS + tid * 8;
  }
  const int a_frag = (wm * 128 + (lane & 31)) * LDS_ROW + (lane >> 5) * 32;
  const int w_frag = BIG_A_ELEMS + wn * NT * WTILE_ELEMS + lane * 8;

  f32x16_t acc[4][NT];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int t = 0; t < NT; ++t)
#pragma unroll
      for (int j = 0; j < 16; ++j) acc[i][t][j] = 0.f;
  u32x4 areg[8], wreg[2 * NT];
#pragma unroll
  for (int i = 0; i < 8; ++i) areg[i] = *(const u32x4*)(a_src[i]);
#pragma unroll
  for (int i = 0; i < 2 * NT; ++i) wreg[i] = *(const u32x4*)(w_src[i]);
#pragma unroll
  for (int i = 0; i < 8; ++i) *(u32x4*)&big_lds[a_dst[i]] = areg[i];
#pragma unroll
  for (int i = 0; i < 2 * NT; ++i) *(u32x4*)&big_lds[BIG_A_ELEMS + i * WTILE_ELEMS + tid * 8] = wreg[i];
  __syncthreads();

  // fragments of k-step j+1 are read while k-step j is multiplied; the global loads of the next block ride on k-steps
  // 0 and 1, its LDS writes on k-steps 2 and 3 (into the other buffer, which every wave left at the last barrier)
  u32x4 af[2][4], bf[2][NT];
#pragma unroll
  for (int i = 0; i < 4; ++i) af[0][i] = *(const u32x4*)(big_lds + a_frag + i * 32 * LDS_ROW);
#pragma unroll
  for (int t = 0; t < NT; ++t) bf[0][t] = *(const u32x4*)(big_lds + w_frag + t * WTILE_ELEMS);
  for (int kb = 0; kb < nkb; ++kb) {
    const int cur = kb & 1;
    const uint16_t* buf = big_lds + cur * BUF_ELEMS;
    uint16_t* nxt = big_lds + (cur ^ 1) * BUF_ELEMS;
    const size_t k1 = (size_t)min(kb + 1, nkb - 1);           // past the end the last block is simply loaded again
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      if (j < 3) {
#pragma unroll
        for (int i = 0; i < 4; ++i) af[(j + 1) & 1][i] = *(const u32x4*)(buf + a_frag + i * 32 * LDS_ROW + (j + 1) * 8);
#pragma unroll
        for (int t = 0; t < NT; ++t) bf[(j + 1) & 1][t] = *(const u32x4*)(buf + w_frag + t * WTILE_ELEMS + (j + 1) * 512);
      }
      if (j == 0) {
#pragma unroll
        for (int i = 0; i < 8; ++i) areg[i] = *(const u32x4*)(a_src[i] + k1 * GEMM_BK);
      } else if (j == 1) {
#pragma unroll
        for (int i = 0; i < 2 * NT; ++i) wreg[i] = *(const u32x4*)(w_src[i] + k1 * WTILE_ELEMS);
      } else if (j == 2) {
#pragma unroll
        for (int i = 0; i < 8; ++i) *(u32x4*)&nxt[a_dst[i]] = areg[i];
      } else {
#pragma unroll
        for (int i = 0; i < 2 * NT; ++i) *(u32x4*)&nxt[BIG_A_ELEMS + i * WTILE_ELEMS + tid * 8] = wreg[i];
      }
#pragma unroll
      for (int t = 0; t < NT; ++t)
#pragma unroll
        for (int i = 0; i < 4; ++i)
          acc[i][t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, af[j & 1][i]),
                                                              __builtin_bit_cast(bf16x8_t, bf[j & 1][t]), acc[i][t], 0, 0, 0);
      // pin the interleave over the 4 NT MFMAs of the k-step: the LDS reads (4 + NT of them) and the other memory
      // operations (8 or 2 NT of them) are spread between pairs of MFMAs
#pragma unroll
      for (int x = 0; x < 8; ++x) {
        if (NT == 4 || (x & 1) == 0) __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);
        else __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        if (j < 3 && x < 4 + NT) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
        if (x < ((j & 1) ? 2 * NT : 8)) {
          if (j < 2) __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
          else __builtin_amdgcn_sched_group_barrier(0x200, 1, 0);
        }
      }
      __builtin_amdgcn_sched_barrier(0);
    }
    __syncthreads();
    // first fragments of the next block (just published)
#pragma unroll
    for (int i = 0; i < 4; ++i) af[0][i] = *(const u32x4*)(nxt + a_frag + i * 32 * LDS_ROW);
#pragma unroll
    for (int t = 0; t < NT; ++t) bf[0][t] = *(const u32x4*)(nxt + w_frag + t * WTILE_ELEMS);
  }

#pragma unroll
  for (int t = 0; t < NT; ++t) {
    const int n_tile = n_base + wn * (32 * NT) + t * 32;
    const int n_out = n_tile + (lane & 31);
    if (EPI == 1) {
      uint16_t* __restrict__ act = (uint16_t*)C;
      const int F = N >> 1;
      const int f_out = (n_tile >> 1) + (lane & 15);
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 16; ++j) {
          const float mine = acc[i][t][j];
          const float other = __shfl_xor(mine, 16, 64);
          const int mrow = m_base + wm * 128 + i * 32 + (j >> 2) * 8 + (lane >> 5) * 4 + (j & 3);
          if ((lane & 16) == 0 && mrow < M && n_out < N)
            act[(size_t)mrow * F + f_out] = f2bf(mine / (1.0f + __expf(-mine)) * other);
        }
    } else if (n_out < N) {
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 16; ++j) {
          const int mrow = m_base + wm * 128 + i * 32 + (j >> 2) * 8 + (lane >> 5) * 4 + (j & 3);
          if (mrow < M) Cz[(size_t)mrow * N + n_out] = acc[i][t][j];
        }
    }
  }
}

// Row-major [N, K] bf16 -> packed W fragments (rows padded to a multiple of 32 must be zeroed by the caller).
__global__ __launch_bounds__(256) void k_pack_weights(const uint16_t* __restrict__ src, uint16_t* __restrict__ dst,
                                                      size_t N, size_t K) {
  const size_t total = N * K / 8;   // 16-byte groups
  const size_t nkb = K / GEMM_BK;
  for (size_t g = (size_t)blockIdx.x * 256 + threadIdx.x; g < total; g += (size_t)gridDim.x * 256) {
    const size_t n = g / (K / 8), k = (g % (K / 8)) * 8;
    const size_t kk = k % GEMM_BK;
    const size_t lane = (kk / 32) * 32 + n % 32, j = (kk % 32) / 8;
    const size_t o = ((n / 32) * nkb + k / GEMM_BK) * WTILE_ELEMS + j * 512 + lane * 8;
    *(u32x4*)(dst + o) = *(const u32x4*)(src + n * K + k);
  }
}
void launch_pack_weights(const void* src, void* dst, size_t N, size_t K, hipStream_t st) {
  const size_t total = N * K / 8;
  if (!total) return;
  const unsigned blocks = (unsigned)((total + 255) / 256 < 262144 ? (total + 255) / 256 : 262144);
  hipLaunchKernelGGL(k_pack_weights, dim3(blocks), dim3(256), 0, st, (const uint16_t*)src, (uint16_t*)dst, N, K);
}

__global__ void k_reduce_splits(const float* __restrict__ part, float* __restrict__ c, size_t mn, int S) {
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= mn) return;
  float s = 0.f;
  for (int z = 0; z < S; ++z) s += part[(size_t)z * mn + i];
  c[i] = s;
}

// Number of K splits: enough workgroups to cover the chip's 256 CUs without drowning the weight stream
// in partial-sum traffic.
int gemm_pick_splits(int M, int N, int K) {
  // Never more workgroups than the chip has CUs: a launch of 280-320 workgroups puts a second one on some CUs, which
  // then set its length (QKV at 8-128 rows: 6 splits = 288 workgroups 15.9-29.4 us, 5 splits = 240 workgroups 13.4-25.5 us;
  // the 32B shapes at 64 rows likewise).  At most 8 splits (partial-sum traffic), and with up to 128 rows at least 10 k
  // blocks per split (O projection: 6 splits of 11 blocks beat 8 of 8).  splits x tiles <= 256 also bounds the partial
  // sums of any shape by 256 x 256 x 128 fp32 = 32 MiB.
  const int mblocks = (M + 255) / 256;
  const int tiles = ((N + 127) / 128) * mblocks;
  const int nkb = K / GEMM_BK;
  int S = tiles < 192 ? 256 / tiles : 1;
  if (S > 8) S = 8;
  if (M <= 128 && S > nkb / 10) S = nkb / 10;
  if (S > nkb / 4) S = nkb / 4;
  if (S < 1) S = 1;
  const int per = (nkb + S - 1) / S;
  return (nkb + per - 1) / per;
}

// Which kernel a launch of M x N x K with S splits gets: every decision is taken here, once, so that a test can ask
// (gemm_kernel_name) which instantiation a shape reaches.
struct GemmPlan {
  int mi;          // row-block height in units of 32 rows
  dim3 grid;
  int per;         // k blocks per split
  int kind;        // 0 base kernel, 1 deep (one workgroup per CU), 2 big (several row blocks)
  bool narrow, xmap;
};
static GemmPlan gemm_plan(int M, int N, int K, int S) {
  GemmPlan p;
  const int nkb = K / GEMM_BK;
  p.per = (nkb + S - 1) / S;
  p.mi = M <= 32 ? 1 : M <= 64 ? 2 : M <= 128 ? 4 : 8;
  p.grid = dim3((N + 127) / 128, (M + 32 * p.mi - 1) / (32 * p.mi), S);
  p.narrow = p.xmap = false;
  p.kind = 0;
  if (p.mi == 8 && (long long)p.grid.x * p.grid.y * p.grid.z <= 256) {   // at most one workgroup per CU: the deep variant
    p.kind = 1;
  } else if (p.mi == 8 && p.grid.y > 1) {   // several row blocks (prefill): 256 x 256 or 256 x 192 tiles
    p.kind = 2;
    // tile width: fewer rounds of 256 workgroups weighted by the width; then fewer padded columns; then the wider
    const long long t4 = (long long)((N + 255) / 256) * p.grid.y * S, t3 = (long long)((N + 191) / 192) * p.grid.y * S;
    const long long c4 = (t4 + 255) / 256 * 256, c3 = (t3 + 255) / 256 * 192;
    p.narrow = c3 < c4 || (c3 == c4 && (N + 191) / 192 * 192 < (N + 255) / 256 * 256);
    // the XCD-aware order pays with many column tiles (gate||up: 112 of them, -7 %) and costs 2-3 % with 16
    const int gx = p.narrow ? (N + 191) / 192 : (N + 255) / 256;
    p.xmap = gx >= 32;
    p.grid.x = gx;
  }
  return p;
}

const char* gemm_kernel_name(int M, int N, int K, int S, int epi) {
  static thread_local char buf[64];
  const GemmPlan p = gemm_plan(M, N, K, S);
  if (p.kind == 1) snprintf(buf, sizeof buf, "k_gemm_bf16_deep<%d>", epi);
  else if (p.kind == 2) snprintf(buf, sizeof buf, "k_gemm_bf16_big<%d,%d,%s>", epi, p.narrow ? 3 : 4, p.xmap ? "true" : "false");
  else snprintf(buf, sizeof buf, "k_gemm_bf16<%d,%d,true>", p.mi, epi);
  return buf;
}

template <int EPI>
static void launch_gemm_t(const uint16_t* a, const uint16_t* w, float* C, int M, int N, int K, int S, hipStream_t st) {
  const GemmPlan p = gemm_plan(M, N, K, S);
  const dim3 grid = p.grid;
  const int per = p.per;
  if (p.kind == 1) {
    hipLaunchKernelGGL((k_gemm_bf16_deep<EPI>), grid, dim3(256), 0, st, a, w, C, M, N, K, per);
    return;
  }
  if (p.kind == 2) {
#define LAUNCH_BIG(NT_, XMAP_)                                                                                          \
  {                                                                                                                     \
    static const hipError_t attr = hipFuncSetAttribute((const void*)k_gemm_bf16_big<EPI, NT_, XMAP_>,                   \
                                                       hipFuncAttributeMaxDynamicSharedMemorySize, BIG_LDS_BYTES(NT_)); \
    (void)attr;                                                                                                         \
    hipLaunchKernelGGL((k_gemm_bf16_big<EPI, NT_, XMAP_>), grid, dim3(256), BIG_LDS_BYTES(NT_), st, a, w, C, M, N, K,   \
                       per);                                                                                            \
  }
    if (p.narrow && p.xmap) LAUNCH_BIG(3, true)
    else if (p.narrow) LAUNCH_BIG(3, false)
    else if (p.xmap) LAUNCH_BIG(4, true)
    else LAUNCH_BIG(4, false)
#undef LAUNCH_BIG
    return;
  }
  switch (p.mi) {   // a single row block (every decode launch) streams W
    case 1: hipLaunchKernelGGL((k_gemm_bf16<1, EPI, true>), grid, dim3(256), 0, st, a, w, C, M, N, K, per, LmEpi{}); break;
    case 2: hipLaunchKernelGGL((k_gemm_bf16<2, EPI, true>), grid, dim3(256), 0, st, a, w, C, M, N, K, per, LmEpi{}); break;
    case 4: hipLaunchKernelGGL((k_gemm_bf16<4, EPI, true>), grid, dim3(256), 0, st, a, w, C, M, N, K, per, LmEpi{}); break;
    default: hipLaunchKernelGGL((k_gemm_bf16<8, EPI, true>), grid, dim3(256), 0, st, a, w, C, M, N, K, per, LmEpi{}); break;
  }
}

// The LM head with fused emit statistics: always the base kernel (a single K split), one row block of up to 256 rows
// per blockIdx.y.  epi.n_tiles must equal ceil(N / 128); part_f / part_i hold M * n_tiles records.
void launch_gemm_lm_fused(const void* A, const void* W, int M, int N, int K, const LmEpi& epi, hipStream_t st) {
  if (M <= 0) return;
  const uint16_t* a = (const uint16_t*)A;
  const uint16_t* w = (const uint16_t*)W;
  const int mi = M <= 32 ? 1 : M <= 64 ? 2 : M <= 128 ? 4 : 8;
  const dim3 grid((N + 127) / 128, (M + 32 * mi - 1) / (32 * mi), 1);
  const int per = K / GEMM_BK;
#define LM_LAUNCH(MI_)                                                                                                   \
  if (epi.sampling) hipLaunchKernelGGL((k_gemm_bf16<MI_, 3, true>), grid, dim3(256), 0, st, a, w, nullptr, M, N, K, per, epi); \
  else hipLaunchKernelGGL((k_gemm_bf16<MI_, 2, true>), grid, dim3(256), 0, st, a, w, nullptr, M, N, K, per, epi)
  switch (mi) {
    case 1: LM_LAUNCH(1); break;
    case 2: LM_LAUNCH(2); break;
    case 4: LM_LAUNCH(4); break;
    default: LM_LAUNCH(8); break;
  }
#undef LM_LAUNCH
}

void launch_gemm(const void* A, const void* W, float* C, int M, int N, int K, int S, hipStream_t st) {
  if (M <= 0) return;
  launch_gemm_t<0>((const uint16_t*)A, (const uint16_t*)W, C, M, N, K, S, st);
}

// act[M, N/2] (bf16) = silu(A Wg^T) * (A Wu^T) with Wg / Wu interleaved in W as described at the kernel.
void launch_gemm_swiglu(const void* A, const void* W, void* act, int M, int N, int K, hipStream_t st) {
  if (M <= 0) return;
  launch_gemm_t<1>((const uint16_t*)A, (const uint16_t*)W, (float*)act, M, N, K, 1, st);
}

void launch_reduce_splits(const float* part, float* c, size_t mn, int S, hipStream_t st) {
  hipLaunchKernelGGL(k_reduce_splits, dim3((unsigned)((mn + 255) / 256)), dim3(256), 0, st, part, c, mn, S);
}
