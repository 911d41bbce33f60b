// Corpus scan fused with top-k, query tile resident in registers.
//
// scan_mfma_dma_kernel and scan_bf16x3_kernel stage the query tile in LDS beside every corpus tile, so per
// multiply-add they move (TN + TM) / (TN TM) operand values from L2 to LDS, a third to three quarters of
// which are query values fetched again and again.  Here every wave keeps the B operand of the matrix
// instruction -- its queries, the whole dimension -- in its own registers for the life of the block: a
// CDNA4 SIMD has 512 registers per lane (256 ordinary, 256 accumulation registers, and a matrix instruction
// reads either kind); 16 queries x 768 float32 columns take 192 of them, and so do 32 queries x 384 columns
// x 2 bfloat16 planes.  Only corpus rows travel: each is brought from HBM to LDS once
// (global_load_lds_dwordx4, no register staging) and read from LDS once per wave that needs it.
//
// Shapes.  A block is 4 waves, one per SIMD, over tiles of 128 corpus rows.  The waves form WQ query groups
// of QW queries (float32: 16, bfloat16: 32) and 4 / WQ row groups: wave w holds query group w % WQ and
// multiplies rows (w / WQ) * 128 / (4 / WQ) .. of every tile, so a block serves QW WQ queries; the shape is
// chosen by the number of queries so that no wave idles.
//
// Matrix instructions.  float32: v_mfma_f32_16x16x4_f32; lane l supplies A[l % 16][l / 16] (a corpus row
// and one of four columns) and B[l / 16][l % 16] (the same column of query l % 16).  A lane reads four
// consecutive floats of its row with one ds_read_b128 -- columns 16 t + 4 (l / 16) + e, e = 0..3 -- and
// register e of both operands then pairs those columns across the four lane groups; a dot product does not
// care in which order its terms are added, so four instructions consume sixteen columns.  Result register v
// of lane l is row 4 (l / 16) + v, query l % 16.
// bfloat16: v_mfma_f32_32x32x16_bf16; lane l supplies eight consecutive columns 16 t + 8 (l / 32) .. +7 of
// row l % 32 (one ds_read_b128) and of query l % 32, once per plane of the split q = hi + mid (+ lo, dropped
// here: see kRegqPlanes; bf16x3_kernels.hpp: products of bfloat16 values are exact in float32, so the sum over
// the planes rounds only where a float32 contraction rounds).  One 1 KiB operand read feeds 64 cycles of the
// matrix pipe (with the 16x16x32 form it feeds 32, and four SIMDs then ask LDS for exactly its peak rate).
// Result register j of lane l is row 8 (j / 4) + 4 (l / 32) + j % 4, query l % 32.
// Rounded operands (kRegqCoarse): only the first plane of the queries is multiplied, and float32 rows take the
// bfloat16 instruction too -- they stay float32 in HBM and LDS, and a lane rounds its eight columns of a step
// (two ds_read_b128) to bfloat16 on the way in.  Such scores only pick candidates; see kRegqCoarse below.
//
// Scores without arithmetic.  The registers hold -2 q instead of q (an exact scaling) and the accumulators of a
// tile start from the rows' terms |x|^2 (0 for the inner product), read from LDS straight into them: what the
// matrix pipe leaves behind is |x|^2 - 2 q.x, the score itself.  With one wave per SIMD nothing hides ordinary
// instructions -- each one between two matrix instructions delays the second, a single v_add per matrix
// instruction costs a quarter of the matrix rate -- so the end of a tile is one comparison per score against
// the query's bound and a (rare) append; the cosine distance alone multiplies each score by 1/|x| first.
//
// Pipeline.  Rows move in slabs of 128 bytes per row (32 float32 or 64 bfloat16 columns): a stage is
// 128 rows x 128 bytes = 16 KiB, the ring holds NS stages (NS - 1 slabs, 80 KiB at NS = 6, are in flight
// while one is multiplied; one block per CU).  LDS rows are unpadded; lane l of a load fetches the 16-byte
// chunk (l % 8) xor ((row / 2) % 8) of its row, so that the sixteen lanes that read one chunk of sixteen
// consecutive rows together cover all 64 banks exactly once.  A load's address is a scalar base (tile, slab)
// plus a per-lane offset that changes only at the corpus' last tile, and loads are issued unconditionally, so
// the slab loop has no branch and no address arithmetic on the vector pipe.  One plain s_barrier per slab
// publishes the slab that has landed and retires the stage the next load group overwrites; it sits in the
// middle of the previous slab's multiplication.  The body of a tile is fully unrolled (the B registers are
// indexed by column at compile time).
// Every LDS read on the usual path (operand fragments, row terms, candidate counters) is written in assembly
// with its own s_waitcnt lgkmcnt: the compiler guards an LDS read it can see with a wait for the global->LDS
// loads it cannot prove unrelated -- here that would be "all of them", draining the ring at every slab.  The
// matrix instructions are written in assembly too, so that the query operand is read from the accumulation
// registers where it lives instead of being copied to an ordinary register first.
//
// Running top-k: as in scan_mfma_dma_kernel (bound per query, candidates appended to a global buffer,
// buffers cut back by a wave-level sort when the block agrees that one could overflow).
#pragma once

#include <type_traits>

#include "bf16x3_kernels.hpp"
#include "cache_kernels.hpp"
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
// queries one wave holds: 16 with the float32 matrix instruction, 32 with the bfloat16 one (`coarse`: see
// kRegqCoarse, which multiplies float32 rows on the bfloat16 matrix cores too)
__host__ __device__ constexpr int regq_queries_per_wave(int dtype, bool coarse = false) {
  return dtype == kDtypeF32 && !coarse ? 16 : 32;
}

// 16 bytes from LDS into registers without a wait; a later s_waitcnt (regq_tie with the value as operand)
// orders the use of the value after the read.  LDS reads return in order, so "at most n reads issued after
// this one are outstanding" is what has to be waited for.
template <typename V>
__device__ __forceinline__ V regq_lds_read128(uint32_t addr, int imm_offset = 0) {
  // (imm_offset must fold to a constant: loop indices of fully unrolled loops do)
  V v;
  asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "i"(imm_offset));
  return v;
}
// acc += A x B with the query operand B in accumulation registers; the accumulator is read and written by
// consecutive instructions at distance >= 2, the one dependency the matrix pipe resolves by itself.
__device__ __forceinline__ void regq_mfma(f32x4& acc, float a, float b) {
  asm volatile("v_mfma_f32_16x16x4_f32 %0, %1, %2, %0" : "+v"(acc) : "v"(a), "a"(b));
}
__device__ __forceinline__ void regq_mfma(f32x16& acc, const bf16x8& a, const bf16x8& b) {
  asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(acc) : "v"(a), "a"(b));
}
// Instructions that order register traffic the compiler cannot see (results of the reads and matrix
// instructions above): the listed values count as rewritten by `CODE`, so every later use stays behind it
// and every earlier definition in front of it.
#define PROX_RQ_TIE1(CODE, a) asm volatile(CODE : "+v"(a))
#define PROX_RQ_TIE2(CODE, a, b) asm volatile(CODE : "+v"(a), "+v"(b))
#define PROX_RQ_TIE4(CODE, a, b, c, d) asm volatile(CODE : "+v"(a), "+v"(b), "+v"(c), "+v"(d))
template <int N, typename V>
__device__ __forceinline__ void regq_tie_wait_all(V (&v)[N]) {   // every LDS read has returned
  static_assert(N == 1 || N == 2 || N == 4 || N == 8 || N == 16, "operand count");
  if constexpr (N == 1) PROX_RQ_TIE1("s_waitcnt lgkmcnt(0)\n\ts_nop 0", v[0]);
  if constexpr (N == 2) PROX_RQ_TIE2("s_waitcnt lgkmcnt(0)\n\ts_nop 0", v[0], v[1]);
  if constexpr (N == 4) PROX_RQ_TIE4("s_waitcnt lgkmcnt(0)\n\ts_nop 0", v[0], v[1], v[2], v[3]);
  if constexpr (N == 8) {
    PROX_RQ_TIE4("s_waitcnt lgkmcnt(0)\n\ts_nop 0", v[0], v[1], v[2], v[3]);
    PROX_RQ_TIE4("", v[4], v[5], v[6], v[7]);
  }
  if constexpr (N == 16) {
    PROX_RQ_TIE4("s_waitcnt lgkmcnt(0)\n\ts_nop 0", v[0], v[1], v[2], v[3]);
    PROX_RQ_TIE4("", v[4], v[5], v[6], v[7]);
    PROX_RQ_TIE4("", v[8], v[9], v[10], v[11]);
    PROX_RQ_TIE4("", v[12], v[13], v[14], v[15]);
  }
}
// The last matrix instructions must have written their results before ordinary instructions read them (the
// compiler, which inserts these waits for instructions it knows, does not look into the assembly): 16 passes
// of the matrix pipe need 18 idle states, two s_nop 15 give 32.
template <int N, typename V>
__device__ __forceinline__ void regq_tie_matrix_done(V (&v)[N]) {
  static_assert(N == 2 || N == 4 || N == 8, "operand count");
  if constexpr (N == 2) PROX_RQ_TIE2("s_nop 15\n\ts_nop 15", v[0], v[1]);
  if constexpr (N == 4) PROX_RQ_TIE4("s_nop 15\n\ts_nop 15", v[0], v[1], v[2], v[3]);
  if constexpr (N == 8) {
    PROX_RQ_TIE4("s_nop 15\n\ts_nop 15", v[0], v[1], v[2], v[3]);
    PROX_RQ_TIE4("", v[4], v[5], v[6], v[7]);
  }
}
// The other direction: accumulators that ordinary instructions have just set (zeroes, copies) must have settled
// before a matrix instruction reads them -- two idle states -- and the compiler, left alone, is free to sink
// such moves down to right in front of the assembly statement that uses the registers.  Passing every
// accumulator through this statement pins the moves before it.
template <int N, typename V>
__device__ __forceinline__ void regq_tie_settled(V (&v)[N]) {
  static_assert(N == 2 || N == 4 || N == 8, "operand count");
  if constexpr (N == 2) PROX_RQ_TIE2("s_nop 1", v[0], v[1]);
  if constexpr (N == 4) PROX_RQ_TIE4("s_nop 1", v[0], v[1], v[2], v[3]);
  if constexpr (N == 8) {
    PROX_RQ_TIE4("", v[0], v[1], v[2], v[3]);
    PROX_RQ_TIE4("s_nop 1", v[4], v[5], v[6], v[7]);
  }
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
// two bfloat16 values in one register, each times -2 (exact: the product is formed in float32)
__device__ __forceinline__ uint32_t regq_bf16x2_times_minus2(uint32_t w) {
  const float lo = __uint_as_float(w << 16) * -2.f, hi = __uint_as_float(w & 0xffff0000u) * -2.f;
  return (__float_as_uint(lo) >> 16) | (__float_as_uint(hi) & 0xffff0000u);
}

// What the cache probe does with the kernel (MODE kRegqProbe): the "corpus" is the array of sources (slot keys, then the
// batch rows), the queries are batch rows, and instead of a running top-k every (row, source) pair whose score
// passes the row's bound is handed on: the candidates that the float64 distance then decides.
constexpr int kRegqScan = 0, kRegqProbe = 1, kRegqDump = 2;   // what the kernel does with its scores (MODE)
// kRegqScan with the first plane of the bfloat16 queries only: half the matrix work, which at 128 queries turns
// the scan from matrix-bound into HBM-bound.  Its scores are off by up to 2^-8 |q| |x| (coarse_score_error); they
// only pick the candidates whose float64 distances rank, the caller asks for a longer list than k + 8 and the
// exactness check of the ranking carries the term, so the ranked lists stay provably exact.
// On float32 rows the same mode rounds the rows to bfloat16 as well, on their way from LDS to the matrix
// instruction (two 16-byte reads and four v_cvt_pk_bf16_f32 per operand): sixteen times the float32 matrix rate
// for twice the rounding error, and a scan of up to 128 queries that is bound by HBM alone.  The rows' terms
// |x|^2 stay the exact float32 ones.
constexpr int kRegqCoarse = 3;
// The same scores, every one written out as a packed (score, row) key -- out[m * n_rows + row] for the m-th query
// of the miss list -- instead of filtered: the form in which the first rows of the corpus are scored as a sample
// one of whose best scores then starts the bounds of the scan proper (same instructions in the same order, so a row
// scores the same in both).
constexpr int kRegqCoarseKeys = 5;
__host__ __device__ constexpr bool regq_mode_rounds(int mode) { return mode == kRegqCoarse || mode == kRegqCoarseKeys; }
struct RegqRaw8 {   // eight consecutive float32 of a row, as two LDS reads return them
  f32x4 lo, hi;
};
__device__ __forceinline__ bf16x8 regq_round_bf16(const RegqRaw8& r) {   // round to nearest even
  typedef float f32x8 __attribute__((ext_vector_type(8)));
  const f32x8 v = __builtin_shufflevector(r.lo, r.hi, 0, 1, 2, 3, 4, 5, 6, 7);
  return __builtin_convertvector(v, bf16x8);
}

struct RegqEmit {
  int c;                 // cache slots: sources 0..c-1 are slot keys, c + j is batch row j
  const int* live_slots; // DEVICE: slots holding a key when the batch started; others are skipped
  double tau;            // tolerance; the bound of a row follows from it and the row's squared length
  int cap;               // entries a row's list holds
  int* cand_cnt;         // [batch rows] candidates found per row (may exceed cap), zero before the first launch
  int* cand_src;         // [batch rows][cap] the first cap of them, in no particular order,
  double* cand_d;        // ... and their float64 distances to the row
  int* ovf_cnt;          // number of rows whose list overflowed, zero before the launch
  int* ovf_list;         // those rows
  // kRegqDump only: every score is written out, S[m * ldS + row] for the m-th query from m_base on
  float* S;
  long ldS;
};

// Top-k scan (MODE kRegqScan).  The kernel serves the queries m_base .. m_base + QW WQ - 1 of the miss list when the
// number of queries from m_base on, M - m_base, lies in (rem_lo, rem_hi]; otherwise it returns at once, so the
// host can launch the shapes for few, some and many queries back to back without knowing M.
// float32: queries are rows qlist[m] (or m) of Qbase.  bfloat16: Qbase is not used; Qplanes[p][m][:] are the
// planes written by split_bf16x3_kernel.
// Output as scan_mfma_dma_kernel: out[((m) * gridDim.x + blockIdx.x) * kp ..], kp sorted keys per (query, block).
//
// Scores only (MODE kRegqDump): a handful of queries (at most QW; one query group), every score written to S --
// the form the selection kernels of single-query calls read.  With one to four queries the kernel is bound by
// HBM alone, and its loads (global->LDS, 80 KiB in flight per CU) stream a long corpus faster than the
// register loads of scores_stream_kernel do (6.95 against 6.6 TB/s at 1 M x 768).
//
// Cache probe (MODE kRegqProbe, float32 only).  The batch rows m_base .. m_limit - 1 in slices of QW WQ (rem_lo = the
// number of slices, at most the grid), each slice against the sources 0 .. c + (its last row): a row is only ever
// answered by a slot or an earlier row.  Row i's
// bound is the float32 pre-filter of "distance <= tau" (see below); xnrm holds the sources' squared lengths.
template <int DT, int DIM, int WQ, int MODE = kRegqScan>
__global__ __launch_bounds__(256, 1) void scan_regq_kernel(
    const void* __restrict__ Xv, const float* __restrict__ xnrm, long n_rows, const float* __restrict__ Qbase,
    const int* __restrict__ qlist, const uint16_t* __restrict__ Qplanes, long plane_stride,
    const int* __restrict__ m_count_ptr, int m_limit, int m_base, int rem_lo, int rem_hi, int kp,
    const uint64_t* __restrict__ seed, uint64_t* __restrict__ cand_buf, uint64_t* __restrict__ out, int cosine,
    RegqEmit emit) {
  constexpr bool ROWS32 = DT == kDtypeF32;         // float32 rows in memory and in LDS
  constexpr bool HYB = ROWS32 && regq_mode_rounds(MODE);   // ... multiplied as bfloat16
  constexpr bool F32 = ROWS32 && !HYB;             // the float32 matrix instruction
  constexpr int NW = 4;                            // waves per block
  constexpr int NT = NW * 64;
  constexpr int QW = regq_queries_per_wave(DT, HYB);   // queries per wave = rows per row block (square result tiles)
  constexpr int RB = QW;
  constexpr int AV = F32 ? 4 : 16;                 // result registers per row block
  constexpr int AG = AV / 4;                       // ... in groups of four consecutive rows
  constexpr int KS = ROWS32 ? 2 : 4;               // operands (16 columns each) per row block and slab
  constexpr int WR = NW / WQ;                      // row groups
  constexpr int TM = QW * WQ;                      // queries per block
  constexpr int TN = kRegqTileRows;
  constexpr int RPW = TN / WR;                     // rows of a tile one wave multiplies
  constexpr int NRB = RPW / RB;                    // row blocks of those
  constexpr int SLAB_COLS = ROWS32 ? 32 : 64;      // columns per slab (128 bytes per row)
  constexpr int SPT = DIM / SLAB_COLS;             // slabs per tile
  constexpr int NS = regq_stages(SPT);             // stages of the ring
  constexpr int NL = 16 / NW;                      // 1 KiB loads per wave per slab (a stage is 16 of them)
  static_assert(WQ >= 1 && NW % WQ == 0 && NRB >= 1, "bad shape");
  static_assert(NS >= 4 && NS <= SPT, "ring must not run more than one tile ahead (row terms are double-buffered)");
  static_assert(DIM % SLAB_COLS == 0, "whole slabs");

  constexpr bool EMIT = MODE == kRegqProbe, KEYS = MODE == kRegqCoarseKeys, DUMP = MODE == kRegqDump || KEYS;
  constexpr int PLANES = regq_mode_rounds(MODE) ? 1 : kRegqPlanes;
  static_assert(!EMIT || F32, "the probe's keys are float32");
  static_assert(!DUMP || KEYS || WQ == 1, "scores of one query group");
  const int M = m_count_ptr ? min(*m_count_ptr, m_limit) : m_limit;
  // probe: rem_lo is the number of row slices; block b serves slice b % slices and is part b / slices of the blocks
  // that share that slice's sources (the grid need not be a multiple of the slices: a grid of one block per
  // free CU is then used whole)
  const int slices = EMIT ? rem_lo : 1;
  const int slice = int(blockIdx.x) % slices, part = int(blockIdx.x) / slices;
  const int parts = EMIT ? int(gridDim.x) / slices + (slice < int(gridDim.x) % slices ? 1 : 0) : int(gridDim.x);
  const int m0 = EMIT ? m_base + slice * TM : m_base;
  const int rem = M - m0;
  if (EMIT ? rem <= 0 : (rem <= rem_lo || rem > rem_hi)) return;
  if (EMIT) {  // the sources that can answer this block's rows
    const long upto = long(emit.c) + (m0 + TM < M ? m0 + TM : M);
    n_rows = upto < n_rows ? upto : n_rows;
  }

  __shared__ __attribute__((aligned(1024))) float ring[NS][kRegqStageFloats];
  __shared__ __attribute__((aligned(16))) uint64_t wave_scratch[NW][kTopkCap];   // probe: the block's list of pairs
  constexpr int kPairCap = NW * kTopkCap;
  __shared__ int pair_count;
  __shared__ __attribute__((aligned(256))) float nrm_ring[2][TN];   // [tile parity][row], filled by DMA
  __shared__ float bound[TM];
  __shared__ int count[TM];

  const int tid = threadIdx.x, lane = tid & 63;
  const int wib = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform, so everything derived from it is scalar
  const int rl = lane & (RB - 1);                  // row within a row block for operand A, query within the group for B
  const int kg = lane / RB;                        // which 16 bytes of a 16-column step this lane holds
  const int qg = wib % WQ, rg = wib / WQ;          // this wave's query group and row group
  const int q_local = qg * QW + rl;                // this lane's query within the block's tile
  const int row_base = rg * RPW;                   // this wave's first row within a tile

  // ---- the wave's queries, times -2, into registers (queries past M repeat the last one; their results are
  // dropped) ----
  f32x4 bq_f[F32 ? DIM / 16 : 1];
  bf16x8 bq_h[F32 ? 1 : PLANES][F32 ? 1 : DIM / 16];
  {
    int m = m0 + q_local;
    m = m < M ? m : M - 1;
    if constexpr (F32) {
      const float* q = Qbase + long(!EMIT && qlist ? qlist[m] : m) * DIM;
#pragma unroll
      for (int t = 0; t < DIM / 16; ++t) {
        const float4 v = *reinterpret_cast<const float4*>(q + 16 * t + 4 * kg);
        bq_f[t] = f32x4{-2.f * v.x, -2.f * v.y, -2.f * v.z, -2.f * v.w};
      }
    } else {
#pragma unroll
      for (int p = 0; p < PLANES; ++p)
#pragma unroll
        for (int t = 0; t < DIM / 16; ++t) {
          uint4 w = *reinterpret_cast<const uint4*>(Qplanes + long(p) * plane_stride + long(m) * DIM + 16 * t + 8 * kg);
          w.x = regq_bf16x2_times_minus2(w.x);
          w.y = regq_bf16x2_times_minus2(w.y);
          w.z = regq_bf16x2_times_minus2(w.z);
          w.w = regq_bf16x2_times_minus2(w.w);
          bq_h[p][t] = __builtin_bit_cast(bf16x8, w);
        }
    }
  }

  // The query loads are waited for here, once: left to the compiler the wait would sit at the first use, inside
  // the tile loop, where on every later round it would drain the global->LDS loads in flight.
  __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0)

  for (int i = tid; i < TM; i += NT) {
    if constexpr (EMIT) {
      // Row i passes source s on to the float64 distance when |s|^2 - 2 q.s <= bound.  In exact arithmetic
      // "distance <= tau" is |s|^2 - 2 q.s <= tau^2 - |q|^2; the float32 score is off by less than
      // rel (|q|^2 + |s|^2) (prefilter_rel: every product and partial sum rounds once), and a source within
      // tau has |s| <= |q| + tau, which makes the bound independent of the source.  Rounded upwards.
      float b = -__builtin_inff();
      if (m0 + i < M) {
        const double qn = double(xnrm[emit.c + m0 + i]), rel = double(prefilter_rel(DIM));
        const double reach = sqrt(qn) + emit.tau;
        const double bd = emit.tau * emit.tau * (1.0 + 1e-3) + rel * (qn + reach * reach) - qn;
        b = bd > 3.0e38 ? 3.0e38f : __double2float_ru(bd);
      }
      bound[i] = b;
    } else {
      // starting bound: the last key of the caller's seed list, if it has one -- the kp-th best score of a
      // sample of the corpus, or a better-ranked one that cut_lists_kernel put there (a padding key gives +inf).
      // At least k + 8 rows of the corpus score at or below it, which is all the ranking needs; the exactness
      // check is told the bound for the case that fewer than kp do
      bound[i] = (seed && m0 + i < M) ? key_score(seed[long(m0 + i) * kp + kp - 1]) : __uint_as_float(0x7f800000u);
    }
    count[i] = 0;
  }
  if (tid == 0) pair_count = 0;
  const int live_slots = EMIT ? __builtin_amdgcn_readfirstlane(*emit.live_slots) : 0;

  // (the block's share of the tiles: values every lane holds alike; passing them through readfirstlane keeps
  // the loop control in scalar registers)
  auto uniform = [](long v) {
    const unsigned lo = unsigned(__builtin_amdgcn_readfirstlane(int(unsigned(v))));
    const unsigned hi = unsigned(__builtin_amdgcn_readfirstlane(int(unsigned((unsigned long)v >> 32))));
    return long(((unsigned long)hi << 32) | lo);
  };
  const long n_tiles = (n_rows + TN - 1) / TN;
  const long t_begin = uniform(n_tiles * part / parts);
  const long t_end = uniform(n_tiles * (part + 1) / parts);
  uint64_t* my_buf = cand_buf + long(blockIdx.x) * long(TM) * kTopkCap;
  const char* X = static_cast<const char*>(Xv);
  constexpr long ROW_BYTES = long(DIM) * (ROWS32 ? 4 : 2);

  // ---- load duty of this lane: load i of the wave covers stage rows 8 (wib NL + i) .. +7 ----
  // A load's address is a wave-uniform base (tile and slab: scalar registers, scalar arithmetic) plus a 32-bit
  // per-lane offset (row within the tile and 16-byte piece) that changes only where a tile is cut by the end of
  // the corpus.  Loads are issued NS - 1 slabs ahead unconditionally: past the block's last tile they fetch
  // rows of the following tiles (clamped to the corpus) into stages nobody reads any more -- a few dozen KiB
  // per block -- which keeps every branch out of the slab loop.
  int my_row[NL], my_chunk[NL];
#pragma unroll
  for (int i = 0; i < NL; ++i) {
    my_row[i] = 8 * (wib * NL + i) + (lane >> 3);
    my_chunk[i] = (lane & 7) ^ ((my_row[i] >> 1) & 7);
  }
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
    if (wib < 2) {  // the tile's 128 row terms, 64 per wave, parked in LDS until the tile's accumulators start from them
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
    asm volatile("" : "+s"(x_slab));   // (... and the scalar base is kept whole: no re-association with the offset)
#pragma unroll
    for (int i = 0; i < NL; ++i) {
      // (the offset passes through an empty statement so that its widening to 64 bits is not hoisted out of
      // the loop: next to the load, the compiler folds it into the scalar-base form of the instruction)
      asm volatile("" : "+v"(voff[i]));
      // corpus rows are read once: nontemporal (aux bit 1)
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(x_slab + size_t(voff[i])),
                                       (__attribute__((address_space(3))) void*)(base + i * 256), 16, 0, 2);
    }
    if (islab == SPT - 1) ++itile;
  };

  // ---- accumulators: NRB row blocks, each in NSPLIT partial sums so that at least two (usually four)
  // independent chains of matrix instructions are interleaved ----
  using Acc = typename std::conditional<F32, f32x4, f32x16>::type;
  constexpr int GB = NRB < 4 ? NRB : 4;            // row blocks multiplied side by side
  constexpr int NSPLIT = GB == 4 ? 1 : 2;
  constexpr int NACC = NRB * NSPLIT;
  static_assert(GB == 1 || GB == 2 || GB == 4, "one, two or four row blocks per chunk");
  Acc acc[NACC];                                   // [row block][partial sum]
  const uint32_t nrm_lds = regq_lds_addr(&nrm_ring[0][0]);
  // The first partial sum of every row block starts from the rows' terms (register 4 g + v of block b is row
  // RB b + 8 g + 4 kg + v of the wave's rows: four consecutive floats per read), the others from zero.  The
  // cosine distance multiplies by its row term at the end instead and starts from zero throughout.
  // (The candidate count of the lane's query comes along with the same wait: `my_count` afterwards.)
  const uint32_t my_count_lds = regq_lds_addr(&count[0]) + 4u * uint32_t(q_local);
  int my_count = 0;
  auto start_accumulators = [&](long tile) {
    if (cosine) {
#pragma unroll
      for (int i = 0; i < NACC; ++i)
#pragma unroll
        for (int v = 0; v < AV; ++v) acc[i][v] = 0.f;
      my_count = regq_lds_read_i32(my_count_lds);
      regq_tie_settled(acc);
      return;
    }
    const uint32_t nr_addr = nrm_lds + uint32_t((int(tile & 1) * TN + row_base + 4 * kg) * 4);
    f32x4 term[NRB * AG];
    asm volatile("ds_read_b32 %0, %1" : "=v"(my_count) : "v"(my_count_lds));
#pragma unroll
    for (int b = 0; b < NRB; ++b)
#pragma unroll
      for (int g = 0; g < AG; ++g) term[b * AG + g] = regq_lds_read128<f32x4>(nr_addr, (RB * b + 8 * g) * 4);
    regq_tie_wait_all(term);
    asm volatile("" : "+v"(my_count));   // (read before the terms: returned before them)
#pragma unroll
    for (int b = 0; b < NRB; ++b) {
#pragma unroll
      for (int v = 0; v < AV; ++v) acc[b * NSPLIT][v] = term[b * AG + v / 4][v % 4];
#pragma unroll
      for (int h = 1; h < NSPLIT; ++h)
#pragma unroll
        for (int v = 0; v < AV; ++v) acc[b * NSPLIT + h][v] = 0.f;
    }
    regq_tie_settled(acc);
  };

  // One slab (number S within its tile) = KS NRB operand reads, each feeding one group of matrix instructions.
  // Reads go in chunks of GB row blocks (same 16-column step); the instructions of a chunk are issued
  // column-major over its row blocks, so that consecutive instructions accumulate into different registers.
  // The next chunk's reads are in flight while a chunk is multiplied.
  // Address of a read: stage + (row_base + RB b + rl) * 128 bytes + the lane's swizzled 16 bytes.  Step ks
  // covers the 16-byte chunks ks (8 / KS) .. of the row, so chunk = ks (8 / KS) + kg, xor the swizzle
  // (row / 2) % 8 = (rl / 2) % 8 (row_base and RB b are multiples of 16); the step enters by xor as well
  // because kg < 8 / KS.  The address is a per-lane register plus an immediate: stage * 16 KiB + row block
  // offset must stay below 64 KiB, so stages 4.. use registers 64 KiB up.
  using AFrag = typename std::conditional<F32, f32x4, typename std::conditional<HYB, RegqRaw8, bf16x8>::type>::type;
  constexpr int NCHUNK = KS * NRB / GB;            // chunk c: row blocks (c / KS) * GB .., step c % KS
  const uint32_t ring_lds = regq_lds_addr(&ring[0][0]);
  // (float32 rows multiplied as bfloat16: a lane's eight columns of a step are the two chunks 2 kg and 2 kg + 1 of
  // the step's four; the second sits 16 bytes from the first, before or after it as the swizzle has it)
  uint32_t lane_lo[KS], lane_hi[KS], lane_lo2[HYB ? KS : 1], lane_hi2[HYB ? KS : 1];
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) {
    const int first_chunk = HYB ? 2 * kg : kg;
    lane_lo[ks] = ring_lds + (uint32_t((row_base + rl) * 128 + ((first_chunk ^ ((rl >> 1) & 7)) * 16)) ^ uint32_t(ks * (128 / KS)));
    lane_hi[ks] = lane_lo[ks] + 65536u;
    if constexpr (HYB) {
      lane_lo2[ks] = lane_lo[ks] ^ 16u;
      lane_hi2[ks] = lane_lo2[ks] + 65536u;
    }
  }
  auto read_chunk = [&](AFrag(&dst)[GB], const int stage, const int c) {
#pragma unroll
    for (int bb = 0; bb < GB; ++bb) {
      const int off = (stage & 3) * (kRegqStageFloats * 4) + ((c / KS) * GB + bb) * (RB * 128);
      if constexpr (HYB) {
        dst[bb].lo = regq_lds_read128<f32x4>(stage < 4 ? lane_lo[c % KS] : lane_hi[c % KS], off);
        dst[bb].hi = regq_lds_read128<f32x4>(stage < 4 ? lane_lo2[c % KS] : lane_hi2[c % KS], off);
      } else {
        dst[bb] = regq_lds_read128<AFrag>(stage < 4 ? lane_lo[c % KS] : lane_hi[c % KS], off);
      }
    }
  };
  // the chunk is complete once at most GB (or no) later reads are outstanding: LDS reads return in order
  auto wait_chunk = [&](AFrag(&f)[GB], const bool later_reads) {
    if constexpr (HYB) {   // two reads per operand
      if constexpr (GB == 4) {
        if (later_reads)
          PROX_RQ_TIE4("s_waitcnt lgkmcnt(8)\n\ts_nop 0", f[0].lo, f[0].hi, f[1].lo, f[1].hi);
        else
          PROX_RQ_TIE4("s_waitcnt lgkmcnt(0)\n\ts_nop 0", f[0].lo, f[0].hi, f[1].lo, f[1].hi);
        PROX_RQ_TIE4("", f[2].lo, f[2].hi, f[3].lo, f[3].hi);
      } else if constexpr (GB == 2) {
        if (later_reads)
          PROX_RQ_TIE4("s_waitcnt lgkmcnt(4)\n\ts_nop 0", f[0].lo, f[0].hi, f[1].lo, f[1].hi);
        else
          PROX_RQ_TIE4("s_waitcnt lgkmcnt(0)\n\ts_nop 0", f[0].lo, f[0].hi, f[1].lo, f[1].hi);
      } else {
        if (later_reads)
          PROX_RQ_TIE2("s_waitcnt lgkmcnt(2)\n\ts_nop 0", f[0].lo, f[0].hi);
        else
          PROX_RQ_TIE2("s_waitcnt lgkmcnt(0)\n\ts_nop 0", f[0].lo, f[0].hi);
      }
    } else if constexpr (GB == 4) {
      if (later_reads)
        PROX_RQ_TIE4("s_waitcnt lgkmcnt(4)\n\ts_nop 0", f[0], f[1], f[2], f[3]);
      else
        PROX_RQ_TIE4("s_waitcnt lgkmcnt(0)\n\ts_nop 0", f[0], f[1], f[2], f[3]);
    } else if constexpr (GB == 2) {
      if (later_reads)
        PROX_RQ_TIE2("s_waitcnt lgkmcnt(2)\n\ts_nop 0", f[0], f[1]);
      else
        PROX_RQ_TIE2("s_waitcnt lgkmcnt(0)\n\ts_nop 0", f[0], f[1]);
    } else {
      if (later_reads)
        PROX_RQ_TIE1("s_waitcnt lgkmcnt(1)\n\ts_nop 0", f[0]);
      else
        PROX_RQ_TIE1("s_waitcnt lgkmcnt(0)\n\ts_nop 0", f[0]);
    }
  };
  AFrag a_first[GB];   // first chunk of the slab that is multiplied next, read ahead across the slab boundary
  // Slab S of a tile sits in `stage`.  Half way through, `mid_slab` publishes the next slab (see the main loop);
  // the last chunk's wait is overlapped with the first reads of that next slab.
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
      const int b0 = (c / KS) * GB, t = KS * S + c % KS;
      if constexpr (F32) {
#pragma unroll
        for (int e = 0; e < 4; ++e)
#pragma unroll
          for (int bb = 0; bb < GB; ++bb) regq_mfma(acc[(b0 + bb) * NSPLIT + e % NSPLIT], a[c][bb][e], bq_f[t][e]);
      } else if constexpr (HYB) {
        // the chunk's rows rounded to bfloat16 (ordinary instructions; the empty statement keeps two idle
        // states between the last of them and the matrix instructions that read their results)
        bf16x8 rounded[GB];
#pragma unroll
        for (int bb = 0; bb < GB; ++bb) rounded[bb] = regq_round_bf16(a[c][bb]);
        if constexpr (GB == 4) PROX_RQ_TIE4("s_nop 1", rounded[0], rounded[1], rounded[2], rounded[3]);
        if constexpr (GB == 2) PROX_RQ_TIE2("s_nop 1", rounded[0], rounded[1]);
        if constexpr (GB == 1) PROX_RQ_TIE1("s_nop 1", rounded[0]);
#pragma unroll
        for (int bb = 0; bb < GB; ++bb) regq_mfma(acc[(b0 + bb) * NSPLIT + c % NSPLIT], rounded[bb], bq_h[0][t]);
      } else {
#pragma unroll
        for (int p = 0; p < PLANES; ++p)
#pragma unroll
          for (int bb = 0; bb < GB; ++bb)
            regq_mfma(acc[(b0 + bb) * NSPLIT + (PLANES == 1 ? c : p) % NSPLIT], a[c][bb], bq_h[p][t]);
      }
      if (c == NCHUNK / 2 - 1) {
        if (c + 1 < NCHUNK) wait_chunk(a[c + 1], false);  // nothing in flight across the barrier and the loads
        mid_slab();
      }
      if (c == NCHUNK - 1) wait_chunk(a_first, false);     // ... nor across the end of the slab
    }
  };

  // A buffer is cut back as soon as it holds clearly more than kp entries (so that the bound
  // tightens early), and in any case before the next tile could overflow it.
  const int trigger = min(kTopkCap - TN, max(2 * kp, 64));
  const uint32_t count_lds = regq_lds_addr(&count[0]);
  uint64_t* scratch = wave_scratch[wib];
  const bool q_real = m0 + q_local < M;
  uint64_t* my_q_buf = my_buf + long(q_local) * kTopkCap;

  float T = -__builtin_inff();   // this lane's query's bound, refreshed from LDS only when a buffer was cut back
  bool T_stale = true;
  // One candidate: room from the query's counter (written in assembly so that the compiler does not guard it
  // with a wait for the global->LDS loads in flight, which never touch the counters), then a plain store.
  const uint32_t pair_count_lds = regq_lds_addr(&pair_count), pair_lds = regq_lds_addr(&wave_scratch[0][0]);
  // probe, the block's LDS list is full (hundreds of candidates per row: a tolerance far above the distances
  // between keys): the row is marked as overflowed, which sends it to the dense probe row and the resolver's
  // search over it.  (A row's count is above cap from the first time an addition crosses cap; that addition
  // puts the row on the overflow list.)
  auto overflow_row = [&](int i) {
    const int before = atomicAdd(&emit.cand_cnt[i], emit.cap + 1);
    if (before <= emit.cap) emit.ovf_list[atomicAdd(emit.ovf_cnt, 1)] = i;
  };
  auto append = [&](float sc, uint32_t row) {
    if constexpr (EMIT) {
      // a slot that held no key, the row itself or a later row: not a source of this row
      const int i = m0 + q_local, src = int(row);
      if (!(src < live_slots || (src >= emit.c && src < emit.c + i))) return;
      // Pairs collect in LDS and go out once at the end of the block (an atomic on device memory here would
      // wait for every load in flight); a full list falls back to the direct way.
      uint32_t pos;
      asm volatile("ds_add_rtn_u32 %0, %1, %2\n\ts_waitcnt lgkmcnt(0)" : "=v"(pos) : "v"(pair_count_lds), "v"(1u) : "memory");
      if (pos < uint32_t(kPairCap)) {
        const uint64_t pr = (uint64_t(uint32_t(i)) << 32) | uint32_t(src);
        asm volatile("ds_write_b64 %0, %1" ::"v"(pair_lds + 8u * pos), "v"(pr) : "memory");
      } else {
        overflow_row(i);
      }
    } else {
      uint32_t pos;
      asm volatile("ds_add_rtn_u32 %0, %1, %2\n\ts_waitcnt lgkmcnt(0)" : "=v"(pos) : "v"(my_count_lds), "v"(1u) : "memory");
      my_q_buf[pos] = pack_key(sc, row);
    }
  };
  auto end_of_tile = [&](long tile) {
    regq_tie_matrix_done(acc);
    const uint32_t row0 = uint32_t(tile * TN + row_base + 4 * kg);   // register 4 g + v of row block b: row0 + RB b + 8 g + v
    if (T_stale) {
      T = q_real ? bound[q_local] : -__builtin_inff();
      T_stale = false;
    }
    // (four copies of the comparison code -- cosine or not, last tile of the corpus or not -- so that the usual
    // one carries neither the multiplication nor the test against the number of rows)
    // Per row block: the smallest score first (v_min3: half an instruction per score), and only a lane whose
    // smallest passes looks at its scores one by one -- with the bounds the samples give, most blocks pass nothing.
    auto sift = [&](auto cosine_c, auto cut_c) {
      constexpr bool kCosine = decltype(cosine_c)::value, kCut = decltype(cut_c)::value;
      const uint32_t nr_addr = nrm_lds + uint32_t((int(tile & 1) * TN + row_base + 4 * kg) * 4);
#pragma unroll
      for (int b = 0; b < NRB; ++b) {
        Acc& sc = acc[b * NSPLIT];
        if constexpr (NSPLIT == 2) {
#pragma unroll
          for (int v = 0; v < AV; ++v) sc[v] += acc[b * NSPLIT + 1][v];
        }
        if constexpr (kCosine) {   // score = (-2 q.x) / |x|: the row terms hold 1 / |x|
#pragma unroll
          for (int g = 0; g < AG; ++g) {
            f32x4 term[1] = {regq_lds_read128<f32x4>(nr_addr, (RB * b + 8 * g) * 4)};
            regq_tie_wait_all(term);
#pragma unroll
            for (int v = 0; v < 4; ++v) sc[4 * g + v] *= term[0][v];
          }
        }
        if constexpr (KEYS) {   // every score of a real query goes out as a key
          if (q_real) {
            uint64_t* dst = out + long(m0 + q_local) * n_rows;
#pragma unroll
            for (int v = 0; v < AV; ++v) {
              const uint32_t row = row0 + uint32_t(RB * b + 8 * (v / 4) + v % 4);
              if (!kCut || row < uint32_t(n_rows)) dst[row] = pack_key(sc[v], row);
            }
          }
          continue;
        } else if constexpr (DUMP) {   // every score of a real query goes out: four consecutive rows per store
          if (q_real) {
            float* dst = emit.S + long(q_local) * emit.ldS;
#pragma unroll
            for (int g = 0; g < AG; ++g) {
              const uint32_t row = row0 + uint32_t(RB * b + 8 * g);
              if (!kCut || row + 3 < uint32_t(n_rows)) {
                *reinterpret_cast<float4*>(dst + row) = make_float4(sc[4 * g], sc[4 * g + 1], sc[4 * g + 2], sc[4 * g + 3]);
              } else {
#pragma unroll
                for (int v = 0; v < 4; ++v)
                  if (row + v < uint32_t(n_rows)) dst[row + v] = sc[4 * g + v];
              }
            }
          }
          continue;
        }
        // (sixteen scores per lane: by groups of four, so that a lane with one score to hand on looks at eight
        // values instead of sixteen -- with one wave per SIMD every compare-and-branch is paid in full, and at
        // the usual one candidate per two row blocks that walk was a seventh of the low-reuse scan)
        float least_of[AG];
#pragma unroll
        for (int g = 0; g < AG; ++g)
          least_of[g] = fminf(fminf(sc[4 * g], fminf(sc[4 * g + 1], sc[4 * g + 2])), sc[4 * g + 3]);
        float least = least_of[0];
#pragma unroll
        for (int g = 1; g + 1 < AG; g += 2) least = fminf(least, fminf(least_of[g], least_of[g + 1]));
        if constexpr (AG > 1 && AG % 2 == 0) least = fminf(least, least_of[AG - 1]);
        if (least <= T) {
#pragma unroll
          for (int g = 0; g < AG; ++g) {
            if (AG > 1 && !(least_of[g] <= T)) continue;
#pragma unroll
            for (int v = 4 * g; v < 4 * g + 4; ++v)
              if (sc[v] <= T) {
                const uint32_t row = row0 + uint32_t(RB * b + 8 * (v / 4) + v % 4);
                if (!kCut || row < uint32_t(n_rows)) append(sc[v], row);
              }
          }
        }
      }
    };
    const bool cut = (tile + 1) * TN > n_rows;   // the corpus ends inside this tile
    if (cosine) {
      if (cut) sift(std::true_type{}, std::true_type{}); else sift(std::true_type{}, std::false_type{});
    } else {
      if (cut) sift(std::false_type{}, std::true_type{}); else sift(std::false_type{}, std::false_type{});
    }
    start_accumulators(tile + 1);
    if constexpr (EMIT || DUMP) return;
    if constexpr (WQ == NW) {
      // Four query groups: every query is one wave's alone, and so are its buffer, count and bound.  The wave
      // cuts its own buffers back when one has grown past the trigger, without a word to the others.
      const bool over = my_count > trigger && kg == 0;   // (one lane per query speaks)
      if (__any(over)) {
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // the wave's own appends have reached memory
        unsigned long long todo = __ballot(over);
        while (todo) {
          const int l = __ffsll((long long)todo) - 1;
          todo &= todo - 1;
          const int q = qg * QW + l;                       // kg == 0: lane l holds query l of the group
          const int n = __builtin_amdgcn_readlane(my_count, l);
          const int keep = wave_compact_topk(my_buf + long(q) * kTopkCap, n, kp, scratch, &bound[q], lane);
          if (lane == 0) count[q] = keep;
        }
        T_stale = true;
      }
      return;
    }
    // Fewer query groups: waves share queries.  Do any buffers have to be cut back before the next tile?  Every
    // wave reads the same counts after a plain barrier (no memory fence: loads in flight stay in flight), so all agree.
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
    // the barrier in the middle of the next slab orders these LDS writes
  };

  // ---- main loop ----
  // NS - 1 slabs are issued ahead.  Slab s + 1 is published (its loads waited for, then a plain barrier) half
  // way through the multiplication of slab s, with that slab's remaining operand reads already in flight, so
  // no wave ever sits at a barrier with nothing queued behind it; the same barrier retires the stage of slab
  // s - 1, which every wave has left by then, and slab s + NS - 1 is issued into it.
#pragma unroll
  for (int s = 0; s < NS - 1; ++s) issue(ring[s], s);
  asm volatile("s_waitcnt vmcnt(%0)\n\ts_barrier" ::"n"((NS - 2) * NL) : "memory");
  start_accumulators(t_begin);
  read_chunk(a_first, 0, 0);
  wait_chunk(a_first, false);
  for (long tile = t_begin; tile < t_end; ++tile) {
    // (fully unrolled: the slab number indexes the query registers and names the stages at compile time)
#pragma unroll
    for (int S = 0; S < SPT; ++S) {
      multiply(S % NS, S, (S + 1) % NS, [&]() {
        // slab S + 1 must have landed; the NS - 3 groups issued after it may stay in flight
        asm volatile("s_waitcnt vmcnt(%0)\n\ts_barrier" ::"n"((NS - 3) * NL) : "memory");
        issue(ring[(S + NS - 1) % NS], (S + NS - 1) % SPT);
      });
    }
    end_of_tile(tile);
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // the loads issued past the last tile

  if constexpr (EMIT) {
    // ---- the block's pairs to the rows' lists, each with its float64 distance: one wave per pair ----
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    __syncthreads();
    const int n_pairs = pair_count < kPairCap ? pair_count : kPairCap;
    const uint64_t* pairs = &wave_scratch[0][0];
    const float* keys = static_cast<const float*>(Xv);
    for (int e = wib; e < n_pairs; e += NW) {
      const int i = int(pairs[e] >> 32), src = int(uint32_t(pairs[e]));
      int pos = 0;
      if (lane == 0) {
        pos = atomicAdd(&emit.cand_cnt[i], 1);
        if (pos == emit.cap) emit.ovf_list[atomicAdd(emit.ovf_cnt, 1)] = i;
      }
      pos = __builtin_amdgcn_readfirstlane(pos);
      if (pos >= emit.cap) continue;
      const double d = wave_keydist64(keys + long(emit.c + i) * DIM, keys + long(src) * DIM, DIM, lane, 0);
      if (lane == 0) {
        emit.cand_src[long(i) * emit.cap + pos] = src;
        emit.cand_d[long(i) * emit.cap + pos] = d;
      }
    }
    return;
  }
  if constexpr (DUMP) return;
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
}

#undef PROX_RQ_TIE1
#undef PROX_RQ_TIE2
#undef PROX_RQ_TIE4

}  // namespace prox
