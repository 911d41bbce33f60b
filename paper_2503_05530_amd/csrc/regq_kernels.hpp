// Corpus scan fused with top-k, query tile resident in registers.
//
// scan_mfma_dma_kernel and scan_bf16x3_kernel stage the query tile in LDS beside every corpus tile, so per
// multiply-add they move (TN + TM) / (TN TM) operand values from L2 to LDS, a third to three quarters of
// which are query values fetched again and again.  Here every wave keeps the B operand of the matrix
// instruction -- 16 queries, the whole dimension -- in its own registers for the life of the block: a
// CDNA4 SIMD has 512 registers per lane, 16 queries x 768 float32 columns take 192 of them, and 16 queries
// x 384 columns x 2 bfloat16 planes take 96.  Only corpus rows travel: each is brought from HBM to LDS
// once (global_load_lds_dwordx4, no register staging) and read from LDS once per wave that needs it.
//
// Shapes.  A block is NW waves (float32: 4, one per SIMD; bfloat16: 8, two per SIMD) over tiles of 128
// corpus rows.  The waves form WQ query groups of 16 queries and NW / WQ row groups: wave w holds query
// group w % WQ and multiplies rows (w / WQ) * 128 / (NW / WQ) .. of every tile, so a block serves
// 16 WQ queries; the shape is chosen by the number of queries so that no wave idles.
//
// Matrix instructions.  float32: v_mfma_f32_16x16x4_f32; lane l supplies A[l % 16][l / 16] (a corpus row
// and one of four columns) and B[l / 16][l % 16] (the same column of query l % 16).  A lane reads four
// consecutive floats of its row with one ds_read_b128 -- columns 16 t + 4 (l / 16) + e, e = 0..3 -- and
// register e of both operands then pairs those columns across the four lane groups; a dot product does not
// care in which order its terms are added, so four instructions consume sixteen columns.
// bfloat16: v_mfma_f32_16x16x32_bf16; lane l supplies eight consecutive columns 32 t + 8 (l / 16) .. +7 of
// its row (one ds_read_b128) and of its query, once per plane of the split q = hi + mid (+ lo, dropped here:
// see kRegqPlanes; bf16x3_kernels.hpp: products of bfloat16 values are exact in float32, so the sum over the
// planes rounds only where a float32 contraction rounds).  Result register v of lane l is row 4 (l / 16) + v,
// query l % 16.
//
// Pipeline.  Rows move in slabs of 128 bytes per row (32 float32 or 64 bfloat16 columns): a stage is
// 128 rows x 128 bytes = 16 KiB, the ring holds NS stages (NS - 1 slabs, 80 KiB at NS = 6, are in flight
// while one is multiplied; one block per CU).  LDS rows are unpadded; lane l of a load fetches the 16-byte
// chunk (l % 8) xor ((row / 2) % 8) of its row, so that the sixteen lanes that read one chunk of sixteen
// consecutive rows together cover all 64 banks exactly once.  One plain s_barrier per slab publishes the
// slab that has landed and retires the stage the next load group overwrites; it sits in the middle of the
// previous slab's multiplication (one wave per SIMD: nothing else would cover a wait at a slab boundary).  The body of a tile is fully
// unrolled (the B registers are indexed by column at compile time).
// Every LDS read on the usual path (operand fragments, row terms, candidate counters) is written in assembly
// with its own s_waitcnt lgkmcnt: the compiler guards an LDS read it can see with a wait for the global->LDS
// loads it cannot prove unrelated -- here that would be "all of them", draining the ring at every slab.
//
// Running top-k: as in scan_mfma_dma_kernel (bound per query, candidates appended to a global buffer,
// buffers cut back by a wave-level sort when the block agrees that one could overflow).
#pragma once

#include "bf16x3_kernels.hpp"
#include "mfma_kernels.hpp"

namespace prox {

typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kRegqTileRows = 128;
// Planes of the bfloat16 split this kernel multiplies: hi and mid.  What the third plane would add is below
// 2^-18 |q_i| per element, i.e. below 2^-17 |q| |x| in a score -- a tenth of the float32 accumulation error
// bound at 384 columns -- and the exactness check of the ranking (score_error_bound) carries that term, so
// the ranked lists stay provably exact while a third of the matrix work and of the query registers goes away.
constexpr int kRegqPlanes = 2;
constexpr int kRegqStageFloats = kRegqTileRows * 32;  // 16 KiB

// stages of the ring: a divisor of the slabs per tile, so that the stage of every slab of the unrolled
// tile body is known at compile time
__host__ __device__ constexpr int regq_stages(int slabs_per_tile) {
  return slabs_per_tile % 6 == 0 ? 6 : slabs_per_tile % 8 == 0 ? 8 : slabs_per_tile % 4 == 0 ? 4 : 0;
}
// Is there an instance for this corpus type and dimension?
__host__ __device__ constexpr bool regq_supported(int dtype, int dim) {
  return dtype == kDtypeF32 ? (dim == 768 || dim == 384) : (dim == 384 || dim == 256);
}

// 16 bytes from LDS into registers without a wait; regq_lds_wait orders the use of the value after the read.
// LDS reads return in order, so "at most `pending` reads issued after this one" is what has to be waited for.
template <typename V>
__device__ __forceinline__ V regq_lds_read128(uint32_t addr, int imm_offset = 0) {
  // (imm_offset must fold to a constant: loop indices of fully unrolled loops do)
  V v;
  asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "i"(imm_offset));
  return v;
}
// The matrix instructions, written out so that the query operand is read from the accumulation registers
// where it lives (a wave with 512 registers has 256 of each kind) instead of being copied to an ordinary
// register first: with one wave per SIMD every instruction between two matrix instructions delays the second
// (a single v_add per matrix instruction costs a quarter of the matrix rate), and those copies were one in three.
// acc += A x B; the accumulator is read and written by consecutive instructions at distance >= 4, the
// one dependency the matrix pipe resolves by itself.
__device__ __forceinline__ void regq_mfma_f32(f32x4& acc, float a, float b) {
  asm volatile("v_mfma_f32_16x16x4_f32 %0, %1, %2, %0" : "+a"(acc) : "v"(a), "a"(b));
}
__device__ __forceinline__ void regq_mfma_bf16(f32x4& acc, const bf16x8& a, const bf16x8& b) {
  asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+a"(acc) : "v"(a), "a"(b));
}
template <typename V>
__device__ __forceinline__ void regq_lds_wait(V& v, int pending) {
  if (pending <= 0)
    asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(v));
  else if (pending == 1)
    asm volatile("s_waitcnt lgkmcnt(1)" : "+v"(v));
  else if (pending == 2)
    asm volatile("s_waitcnt lgkmcnt(2)" : "+v"(v));
  else if (pending == 3)
    asm volatile("s_waitcnt lgkmcnt(3)" : "+v"(v));
  else
    asm volatile("s_waitcnt lgkmcnt(4)" : "+v"(v));
}
__device__ __forceinline__ int regq_lds_read_i32(uint32_t addr) {
  int v;
  asm volatile("ds_read_b32 %0, %1\n\ts_waitcnt lgkmcnt(0)" : "=v"(v) : "v"(addr));
  return v;
}
template <typename T>
__device__ __forceinline__ uint32_t regq_lds_addr(const T* p) {
  return uint32_t(uintptr_t((const __attribute__((address_space(3))) T*)p));
}

// The kernel serves the queries m_base .. m_base + 16 WQ - 1 of the miss list when the number of queries
// from m_base on, M - m_base, lies in (rem_lo, rem_hi]; otherwise it returns at once, so the host can launch
// the shapes for few, some and many queries back to back without knowing M.
// float32: queries are rows qlist[m] (or m) of Qbase.  bfloat16: Qbase is not used; Qplanes[p][m][:] are the
// three planes written by split_bf16x3_kernel.
// Output as scan_mfma_dma_kernel: out[((m) * gridDim.x + blockIdx.x) * kp ..], kp sorted keys per (query, block).
template <int DT, int DIM, int WQ>
__global__ __launch_bounds__(DT == kDtypeF32 ? 256 : 512, 1) void scan_regq_kernel(
    const void* __restrict__ Xv, const float* __restrict__ xnrm, long n_rows, const float* __restrict__ Qbase,
    const int* __restrict__ qlist, const uint16_t* __restrict__ Qplanes, long plane_stride,
    const int* __restrict__ m_count_ptr, int m_limit, int m_base, int rem_lo, int rem_hi, int kp,
    const uint64_t* __restrict__ seed, uint64_t* __restrict__ cand_buf, uint64_t* __restrict__ out, int cosine) {
  constexpr bool F32 = DT == kDtypeF32;
  constexpr int NW = F32 ? 4 : 8;                  // waves per block
  constexpr int NT = NW * 64;
  constexpr int WR = NW / WQ;                      // row groups
  constexpr int TM = 16 * WQ;                      // queries per block
  constexpr int TN = kRegqTileRows;
  constexpr int RPW = TN / WR;                     // rows of a tile one wave multiplies
  constexpr int NRB = RPW / 16;                    // 16-row blocks of those
  constexpr int SLAB_COLS = F32 ? 32 : 64;         // columns per slab (128 bytes per row)
  constexpr int SPT = DIM / SLAB_COLS;             // slabs per tile
  constexpr int NS = regq_stages(SPT);             // stages of the ring
  constexpr int NL = 16 / NW;                      // 1 KiB loads per wave per slab (a stage is 16 of them)
  static_assert(WQ >= 1 && NW % WQ == 0 && NRB >= 1, "bad shape");
  static_assert(NS >= 4 && NS <= SPT, "ring must not run more than one tile ahead (row norms are double-buffered)");
  static_assert(DIM % SLAB_COLS == 0, "whole slabs");

  const int M = m_count_ptr ? min(*m_count_ptr, m_limit) : m_limit;
  const int rem = M - m_base;
  if (rem <= rem_lo || rem > rem_hi) return;
  const int m0 = m_base;

  __shared__ __attribute__((aligned(1024))) float ring[NS][kRegqStageFloats];
#define PROX_RQ_RING(s) (ring[(s)])
  __shared__ __attribute__((aligned(16))) uint64_t wave_scratch[NW][kTopkCap];
  __shared__ __attribute__((aligned(256))) float nrm_ring[2][TN];   // [tile parity][row], filled by DMA
  __shared__ float bound[TM];
  __shared__ int count[TM];

  const int tid = threadIdx.x, lane = tid & 63;
  const int wib = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform, so everything derived from it is scalar
  const int r16 = lane & 15, g4 = lane >> 4;
  const int qg = wib % WQ, rg = wib / WQ;          // this wave's query group and row group
  const int q_local = qg * 16 + r16;               // this lane's query within the block's tile
  const int row_base = rg * RPW;                   // this wave's first row within a tile

  // ---- the wave's queries into registers (queries past M repeat the last one; their results are dropped) ----
  f32x4 bq_f[F32 ? DIM / 16 : 1];
  bf16x8 bq_h[F32 ? 1 : kRegqPlanes][F32 ? 1 : DIM / 32];
  {
    int m = m0 + q_local;
    m = m < M ? m : M - 1;
    if (F32) {
      const float* q = Qbase + long(qlist ? qlist[m] : m) * DIM;
#pragma unroll
      for (int t = 0; t < DIM / 16; ++t) {
        const float4 v = *reinterpret_cast<const float4*>(q + 16 * t + 4 * g4);
        bq_f[t] = f32x4{v.x, v.y, v.z, v.w};
      }
    } else {
#pragma unroll
      for (int p = 0; p < kRegqPlanes; ++p)
#pragma unroll
        for (int t = 0; t < DIM / 32; ++t)
          bq_h[p][t] = *reinterpret_cast<const bf16x8*>(Qplanes + long(p) * plane_stride + long(m) * DIM + 32 * t + 8 * g4);
    }
  }

  // The query loads are waited for here, once: left to the compiler the wait would sit at the first use, inside
  // the tile loop, where on every later round it would drain the global->LDS loads in flight.
  __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0)

  for (int i = tid; i < TM; i += NT) {
    // starting bound: the kp-th best score of a sample of the corpus, if the caller has one
    // (a padding key gives +inf); any value at or above the true kp-th best score is valid
    bound[i] = (seed && m0 + i < M) ? key_score(seed[long(m0 + i) * kp + kp - 1]) : __uint_as_float(0x7f800000u);
    count[i] = 0;
  }

  // (the block's share of the tiles: values every lane holds alike; passing them through readfirstlane keeps
  // the loop control in scalar registers)
  auto uniform = [](long v) {
    const unsigned lo = unsigned(__builtin_amdgcn_readfirstlane(int(unsigned(v))));
    const unsigned hi = unsigned(__builtin_amdgcn_readfirstlane(int(unsigned((unsigned long)v >> 32))));
    return long(((unsigned long)hi << 32) | lo);
  };
  const long n_tiles = (n_rows + TN - 1) / TN;
  const long t_begin = uniform(n_tiles * blockIdx.x / gridDim.x);
  const long t_end = uniform(n_tiles * (blockIdx.x + 1) / gridDim.x);
  uint64_t* my_buf = cand_buf + long(blockIdx.x) * long(TM) * kTopkCap;
  const char* X = static_cast<const char*>(Xv);
  constexpr long ROW_BYTES = long(DIM) * (F32 ? 4 : 2);

  // ---- load duty of this lane: load i of the wave covers stage rows 8 (wib NL + i) .. +7 ----
  // Everything about a load except the tile is fixed at compile time once the tile body is unrolled: the slab
  // within its row (an immediate offset of the load instruction) and the stage.  Per tile the lane's row
  // pointers are formed once.  Loads are issued NS - 1 slabs ahead unconditionally: past the block's last tile
  // they fetch rows of the following tiles (clamped to the corpus) into stages nobody reads any more -- a few
  // dozen KiB per block -- which keeps every branch out of the slab loop.
  int my_row[NL], my_chunk[NL];
#pragma unroll
  for (int i = 0; i < NL; ++i) {
    my_row[i] = 8 * (wib * NL + i) + (lane >> 3);
    my_chunk[i] = (lane & 7) ^ ((my_row[i] >> 1) & 7);
  }
  // A load's address is a wave-uniform base (tile and slab: scalar registers, scalar arithmetic) plus a 32-bit
  // per-lane offset (row within the tile and 16-byte piece) that changes only where a tile is cut by the end of
  // the corpus, so issuing a slab costs the vector pipeline nothing but the loads themselves.
  unsigned voff[NL];
  const char* x_tile = X;
  long itile = t_begin;   // tile of the next issue
  const long last_tile = (n_rows - 1) / TN;
  auto point_at_issue_tile = [&]() {
    const long tl = itile < last_tile ? itile : last_tile;
    const int rows_here = int(n_rows - tl * TN < TN ? n_rows - tl * TN : TN);
    x_tile = X + tl * (long(TN) * ROW_BYTES);
#pragma unroll
    for (int i = 0; i < NL; ++i) {
      const int r = my_row[i] < rows_here ? my_row[i] : rows_here - 1;
      voff[i] = unsigned(r) * unsigned(ROW_BYTES) + 16u * unsigned(my_chunk[i]);
    }
    if (wib < 2) {  // the tile's 128 row terms, 64 per wave, parked in LDS until the tile's scores are filtered
      long rn = itile * TN + wib * 64 + lane;
      rn = rn < n_rows ? rn : n_rows - 1;
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(xnrm + rn),
                                       (__attribute__((address_space(3))) void*)&nrm_ring[itile & 1][wib * 64], 4, 0,
                                       0);
    }
  };
  // slab `islab` (a constant after unrolling) of the issue tile into `stage`
  auto issue = [&](float* stage, const int islab) {
    if (islab == 0) point_at_issue_tile();
    float* base = stage + (wib * NL) * 256;
    const char* x_slab = x_tile + islab * 128;
#pragma unroll
    for (int i = 0; i < NL; ++i)  // corpus rows are read once: nontemporal (aux bit 1)
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(x_slab + size_t(voff[i])),
                                       (__attribute__((address_space(3))) void*)(base + i * 256), 16, 0, 2);
    if (islab == SPT - 1) ++itile;
  };

  constexpr int GB = NRB < 4 ? NRB : 4;            // row blocks multiplied side by side
  constexpr int NSPLIT = GB == 4 ? 1 : 2;          // partial sums per row block: up to 4 independent chains
  static_assert(GB == 1 || GB == 2 || GB == 4, "one, two or four row blocks per chunk");
  f32x4 acc[NRB][NSPLIT];
#pragma unroll
  for (int b = 0; b < NRB; ++b)
#pragma unroll
    for (int h = 0; h < NSPLIT; ++h) acc[b][h] = f32x4{0.f, 0.f, 0.f, 0.f};

  // One slab (number S within its tile) = 2 NRB operand reads, each feeding one group of matrix instructions.
  // Reads go in chunks of GB row blocks (same half t); the instructions of a chunk are issued column-major
  // over its row blocks, so that consecutive instructions accumulate into different registers (with fewer
  // than four row blocks per wave the accumulator of a row block is split in NSPLIT partial sums to the same
  // end).  The next chunk's reads are in flight while a chunk is multiplied.
  // Address of a read: stage + (row_base + 16 b + r16) * 128 bytes + the lane's swizzled chunk; the swizzle
  // (row / 2) % 8 = (r16 / 2) % 8 does not depend on the row block (row_base and 16 b are multiples of 16).
  using AFrag = typename std::conditional<F32, f32x4, bf16x8>::type;
  constexpr int NCHUNK = 2 * NRB / GB;             // chunk c: row blocks (c / 2) * GB .., half c % 2
  // The read address is a per-lane register plus an immediate: stage * 16 KiB + row block * 2 KiB must stay
  // below 64 KiB, so stages 4.. use a second register 64 KiB up.
  const uint32_t ring_lds = regq_lds_addr(&ring[0][0]);
  const uint32_t lane_off0 = ring_lds + uint32_t((row_base + r16) * 128 + ((g4 ^ ((r16 >> 1) & 7)) * 16));
  const uint32_t lane_off1 = ring_lds + (uint32_t((row_base + r16) * 128 + ((g4 ^ ((r16 >> 1) & 7)) * 16)) ^ 64u);
  const uint32_t lane_hi0 = lane_off0 + 65536u, lane_hi1 = lane_off1 + 65536u;
  auto read_chunk = [&](AFrag(&dst)[GB], const int stage, const int c) {
#pragma unroll
    for (int bb = 0; bb < GB; ++bb) {
      const uint32_t reg = stage < 4 ? ((c & 1) ? lane_off1 : lane_off0) : ((c & 1) ? lane_hi1 : lane_hi0);
      dst[bb] = regq_lds_read128<AFrag>(reg, (stage & 3) * (kRegqStageFloats * 4) + ((c >> 1) * GB + bb) * 2048);
    }
  };
  // the chunk is complete once at most `pending` (0 or GB) later reads are outstanding: LDS reads return in order
  auto wait_chunk = [&](AFrag(&f)[GB], const bool later_reads) {
    if constexpr (GB == 4) {
      if (later_reads)
        asm volatile("s_waitcnt lgkmcnt(4)\n\ts_nop 0" : "+v"(f[0]), "+v"(f[1]), "+v"(f[2]), "+v"(f[3]));
      else
        asm volatile("s_waitcnt lgkmcnt(0)\n\ts_nop 0" : "+v"(f[0]), "+v"(f[1]), "+v"(f[2]), "+v"(f[3]));
    } else if constexpr (GB == 2) {
      if (later_reads)
        asm volatile("s_waitcnt lgkmcnt(2)\n\ts_nop 0" : "+v"(f[0]), "+v"(f[1]));
      else
        asm volatile("s_waitcnt lgkmcnt(0)\n\ts_nop 0" : "+v"(f[0]), "+v"(f[1]));
    } else {
      if (later_reads)
        asm volatile("s_waitcnt lgkmcnt(1)\n\ts_nop 0" : "+v"(f[0]));
      else
        asm volatile("s_waitcnt lgkmcnt(0)\n\ts_nop 0" : "+v"(f[0]));
    }
  };
  AFrag a_first[GB];   // first chunk of the slab that is multiplied next, read ahead across the slab boundary
  // Slab S of a tile sits in `stage`.  Half way through, `mid_slab` publishes the next slab (see the main loop);
  // the last chunk's wait is overlapped with the first reads of that next slab, when there is one.
  // Rule for the reads written in assembly: the compiler takes their results for ready at once, so no result
  // may be in flight across anything it could use to move values around -- every chunk that is read ahead is
  // waited for in the same straight-line stretch of code, before any branch.
  auto multiply = [&](const int stage, const int S, const int next_stage, auto mid_slab) {
    AFrag a[NCHUNK][GB];
#pragma unroll
    for (int bb = 0; bb < GB; ++bb) a[0][bb] = a_first[bb];
#pragma unroll
    for (int c = 0; c < NCHUNK; ++c) {
      // the next chunk of this slab, or the first chunk of the next slab (published half a slab ago; after the
      // block's last slab the read is of a stage nobody writes any more and its result is not used)
      if (c + 1 < NCHUNK)
        read_chunk(a[c + 1], stage, c + 1);
      else
        read_chunk(a_first, next_stage, 0);
      wait_chunk(a[c], true);
      const int b0 = (c >> 1) * GB, t = c & 1;
      if constexpr (F32) {
        const f32x4 bv = bq_f[2 * S + t];
#pragma unroll
        for (int e = 0; e < 4; ++e)
#pragma unroll
          for (int bb = 0; bb < GB; ++bb) regq_mfma_f32(acc[b0 + bb][e % NSPLIT], a[c][bb][e], bv[e]);
      } else {
#pragma unroll
        for (int p = 0; p < kRegqPlanes; ++p)
#pragma unroll
          for (int bb = 0; bb < GB; ++bb) regq_mfma_bf16(acc[b0 + bb][p % NSPLIT], a[c][bb], bq_h[p][2 * S + t]);
      }
      if (c == NCHUNK / 2 - 1) {
        if (c + 1 < NCHUNK) wait_chunk(a[c + 1], false);  // nothing in flight across the branch below
        mid_slab();
      }
      if (c == NCHUNK - 1) wait_chunk(a_first, false);     // ... nor across the end of the slab
    }
  };

  // A buffer is cut back as soon as it holds clearly more than kp entries (so that the bound
  // tightens early), and in any case before the next tile could overflow it.
  const int trigger = min(kTopkCap - TN, max(2 * kp, 64));
  const uint32_t count_lds = uint32_t(uintptr_t((__attribute__((address_space(3))) int*)&count[0]));
  uint64_t* scratch = wave_scratch[wib];
  const bool q_real = m0 + q_local < M;
  uint64_t* my_q_buf = my_buf + long(q_local) * kTopkCap;

  const uint32_t nrm_lds = regq_lds_addr(&nrm_ring[0][0]);
  float T = -__builtin_inff();   // this lane's query's bound, refreshed from LDS only when a buffer was cut back
  bool T_stale = true;
  auto end_of_tile = [&](long tile) {
    // the last matrix instructions must have written the accumulators before ordinary instructions read them
    // (the compiler, which inserts these waits for instructions it knows, does not look into the assembly)
    asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");
    const long row0 = tile * TN + row_base + 4 * g4;
    if (T_stale) {
      T = q_real ? bound[q_local] : -__builtin_inff();
      T_stale = false;
    }
    // pass 1: accumulators into scores; which ones beat the query's bound.  The four row terms of a row block
    // that this lane needs are consecutive: one 16-byte read each.
    const uint32_t nr_addr = nrm_lds + uint32_t((int(tile & 1) * TN + row_base + 4 * g4) * 4);
    f32x4 nr[NRB];
    nr[0] = regq_lds_read128<f32x4>(nr_addr);
    uint32_t pass = 0;
#pragma unroll
    for (int b = 0; b < NRB; ++b) {
      if (b + 1 < NRB) nr[b + 1] = regq_lds_read128<f32x4>(nr_addr + uint32_t((b + 1) * 64));
      regq_lds_wait(nr[b], b + 1 < NRB ? 1 : 0);
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const float dot = NSPLIT == 1 ? acc[b][0][v] : acc[b][0][v] + acc[b][NSPLIT - 1][v];
        const float sc = row_score(nr[b][v], dot, cosine);
        acc[b][0][v] = sc;
        pass |= (sc <= T && row0 + 16 * b + v < n_rows) ? (1u << (4 * b + v)) : 0u;
      }
    }
    // pass 2: one LDS counter update per lane reserves room, then plain stores.  (Written in assembly so that
    // the compiler does not guard it with a wait for the global->LDS loads in flight, which never touch the counters.)
    if (pass) {
      uint32_t pos;
      asm volatile("ds_add_rtn_u32 %0, %1, %2\n\ts_waitcnt lgkmcnt(0)"
                   : "=v"(pos)
                   : "v"(count_lds + 4u * uint32_t(q_local)), "v"(uint32_t(__builtin_popcount(pass)))
                   : "memory");
#pragma unroll
      for (int b = 0; b < NRB; ++b)
#pragma unroll
        for (int v = 0; v < 4; ++v)
          if (pass & (1u << (4 * b + v))) my_q_buf[pos++] = pack_key(acc[b][0][v], uint32_t(row0 + 16 * b + v));
    }
#pragma unroll
    for (int b = 0; b < NRB; ++b)
#pragma unroll
      for (int h = 0; h < NSPLIT; ++h) acc[b][h] = f32x4{0.f, 0.f, 0.f, 0.f};
    // Do any buffers have to be cut back before the next tile?  Every wave reads the same counts
    // after a plain barrier (no memory fence: loads in flight stay in flight), so all agree.
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
    const bool mine = regq_lds_read_i32(count_lds + 4u * uint32_t(lane < TM ? lane : 0)) > trigger;   // TM <= 128: lanes
    const bool more = TM > 64 && regq_lds_read_i32(count_lds + 4u * uint32_t(64 + lane < TM ? 64 + lane : 0)) > trigger;
    if (__any(mine || more)) {
      __syncthreads();  // full fence: the candidates other waves appended must be visible
      for (int q = wib; q < TM; q += NW) {
        const int n = count[q];
        if (n > trigger) {
          const int keep = wave_compact_topk(my_buf + long(q) * kTopkCap, n, kp, scratch, &bound[q], lane);
          if (lane == 0) count[q] = keep;
        }
      }
      __syncthreads();  // the tightened bounds are read back at the next tile's end
      T_stale = true;
    }
    // the barrier at the top of the next slab orders these LDS writes
  };

  // ---- main loop ----
  // NS - 1 slabs are issued ahead.  Slab s + 1 is published (its loads waited for, then a plain barrier) half
  // way through the multiplication of slab s, with that slab's remaining operand reads already in flight, so
  // no wave ever sits at a barrier with nothing queued behind it; the same barrier retires the stage of slab
  // s - 1, which every wave has left by then, and slab s + NS - 1 is issued into it.
#pragma unroll
  for (int s = 0; s < NS - 1; ++s) issue(PROX_RQ_RING(s), s);
  asm volatile("s_waitcnt vmcnt(%0)\n\ts_barrier" ::"n"((NS - 2) * NL) : "memory");
  read_chunk(a_first, 0, 0);
  wait_chunk(a_first, false);
  for (long tile = t_begin; tile < t_end; ++tile) {
    // (fully unrolled: the slab number indexes the query registers and names the stages at compile time)
#pragma unroll
    for (int S = 0; S < SPT; ++S) {
      multiply(S % NS, S, (S + 1) % NS, [&]() {
        // slab S + 1 must have landed; the NS - 3 groups issued after it may stay in flight
        asm volatile("s_waitcnt vmcnt(%0)\n\ts_barrier" ::"n"((NS - 3) * NL) : "memory");
        issue(PROX_RQ_RING((S + NS - 1) % NS), (S + NS - 1) % SPT);
      });
    }
    end_of_tile(tile);
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // the loads issued past the last tile

  // ---- every query's buffer cut to kp sorted entries and written out ----
  __syncthreads();
  for (int q = wib; q < TM; q += NW) {
    if (m0 + q >= M) continue;
    const int n = count[q];
    uint64_t* buf = my_buf + long(q) * kTopkCap;
    const int keep = wave_compact_topk(buf, n, kp, wave_scratch[wib], &bound[q], lane);
    uint64_t* o = out + (long(m0 + q) * gridDim.x + blockIdx.x) * kp;
    for (int i = lane; i < kp; i += 64) o[i] = i < keep ? wave_scratch[wib][i] : kPadKey;
  }
#undef PROX_RQ_RING
}

}  // namespace prox
