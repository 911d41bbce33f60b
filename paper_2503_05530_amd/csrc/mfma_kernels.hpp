// Batched query-by-rows contraction on the float32 matrix cores (v_mfma_f32_32x32x2_f32).
//
// The batched form of the distance step really is a dense GEMM:
//   score[m][j] = |x_j|^2 - 2 * sum_k q_m[k] x_j[k]
// for M queries against N stored rows.  Two kernels share one tiled main loop:
//
//   scan_mfma_topk_kernel   corpus scan fused with a running per-query top-k, so
//                           the M x N score matrix is never written (Section 2.2's
//                           search for many queries at once);
//   probe_mfma_dense_kernel cache probe: batch rows against [slot keys ; batch
//                           rows], scores written densely for the resolver
//                           (Algorithm 1, distances to every key).
//
// Tiling.  A block of 256 threads (4 waves) computes a TR x TC tile of the
// product A[TR x d] * B[TC x d]^T, both operands row-major with the contraction
// along rows.  The contraction runs in slabs of 32: the 256 threads copy the
// slab of both operands from global memory to registers (16-byte loads, eight
// lanes cover 128 contiguous bytes of one row), then to LDS with a row stride
// of 36 floats, which makes the 16-byte fragment reads below conflict-free.
// Global loads for slab s+1 are issued before the matrix instructions of slab s.
//
// Fragment order.  v_mfma_f32_32x32x2_f32 takes A[i][k] from lane (i + 32k) and
// B[k][j] from lane (j + 32k), k in {0,1}.  A lane reads four consecutive floats
// of "its" row with one ds_read_b128: lanes 0-31 at slab columns 8t..8t+3, lanes
// 32-63 at 8t+4..8t+7.  Register e of both fragments then pairs column 8t+e with
// 8t+4+e; a dot product does not care in which order its terms are added, so
// four matrix instructions consume the eight columns.  Result element v of lane
// l is row 8*(v/4) + 4*(l/32) + v%4, column l%32 of the 32 x 32 block.
#pragma once

#include <type_traits>

#include "device_utils.hpp"

namespace prox {

typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kSlabK = 32;   // contraction columns per slab
constexpr int kLdsK = 36;    // LDS row stride in floats
constexpr int kTopkCap = 512;  // per (block, query) candidate buffer entries

// ---- operand slab movement ------------------------------------------------------
// T rows x 32 columns of float32 = T*8 chunks of 16 bytes; thread t takes chunks
// t, t+256, ...  Chunk c is row c/8, columns 4*(c%8)..+3.
template <int T>
struct SlabF32 {
  static constexpr int NCH = T * 8 / 256;
  float4 v[NCH];
  // rows[i] points at column 0 of the row of chunk i (nullptr: row absent -> zeros)
  __device__ __forceinline__ void load(const float* const (&rows)[NCH], int k0, int tid) {
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
      const int c4 = (tid + 256 * i) & 7;
      v[i] = rows[i] ? *reinterpret_cast<const float4*>(rows[i] + k0 + 4 * c4) : make_float4(0.f, 0.f, 0.f, 0.f);
    }
  }
  __device__ __forceinline__ void store(float* lds, int tid) const {
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
      const int c = tid + 256 * i;
      *reinterpret_cast<float4*>(lds + (c >> 3) * kLdsK + 4 * (c & 7)) = v[i];
    }
  }
};

// T rows x 32 columns of bfloat16 = T*4 chunks of 16 bytes (8 values); chunk c is
// row c/4, columns 8*(c%4)..+7.  Widened to float32 on the way into LDS.
template <int T>
struct SlabBF16 {
  static constexpr int NCH = (T * 4 + 255) / 256;
  uint4 v[NCH];
  __device__ __forceinline__ void load(const uint16_t* const (&rows)[NCH], int k0, int tid) {
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
      const int c8 = (tid + 256 * i) & 3;
      v[i] = rows[i] ? *reinterpret_cast<const uint4*>(rows[i] + k0 + 8 * c8) : make_uint4(0, 0, 0, 0);
    }
  }
  __device__ __forceinline__ void store(float* lds, int tid) const {
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
      const int c = tid + 256 * i;
      if (c < T * 4) {
        float* p = lds + (c >> 2) * kLdsK + 8 * (c & 3);
        const uint32_t w[4] = {v[i].x, v[i].y, v[i].z, v[i].w};
        *reinterpret_cast<float4*>(p) =
            make_float4(__uint_as_float(w[0] << 16), __uint_as_float(w[0] & 0xffff0000u),
                        __uint_as_float(w[1] << 16), __uint_as_float(w[1] & 0xffff0000u));
        *reinterpret_cast<float4*>(p + 4) =
            make_float4(__uint_as_float(w[2] << 16), __uint_as_float(w[2] & 0xffff0000u),
                        __uint_as_float(w[3] << 16), __uint_as_float(w[3] & 0xffff0000u));
      }
    }
  }
};

// ---- one slab of matrix instructions -------------------------------------------
// The wave's RB x CB blocks of 32 x 32: rows from As starting at a_row0, columns
// from Bs starting at b_row0.
template <int RB, int CB>
__device__ __forceinline__ void mfma_slab(const float* __restrict__ As, const float* __restrict__ Bs, int a_row0,
                                          int b_row0, int lane, f32x16 (&acc)[RB][CB]) {
  const int r = lane & 31, half = lane >> 5;
#pragma unroll
  for (int t = 0; t < kSlabK / 8; ++t) {
    float4 a[RB], b[CB];
#pragma unroll
    for (int i = 0; i < RB; ++i)
      a[i] = *reinterpret_cast<const float4*>(As + (a_row0 + 32 * i + r) * kLdsK + 8 * t + 4 * half);
#pragma unroll
    for (int j = 0; j < CB; ++j)
      b[j] = *reinterpret_cast<const float4*>(Bs + (b_row0 + 32 * j + r) * kLdsK + 8 * t + 4 * half);
#pragma unroll
    for (int e = 0; e < 4; ++e) {
#pragma unroll
      for (int i = 0; i < RB; ++i)
#pragma unroll
        for (int j = 0; j < CB; ++j) {
          const float av = e == 0 ? a[i].x : e == 1 ? a[i].y : e == 2 ? a[i].z : a[i].w;
          const float bv = e == 0 ? b[j].x : e == 1 ? b[j].y : e == 2 ? b[j].z : b[j].w;
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(av, bv, acc[i][j], 0, 0, 0);
        }
    }
  }
}

// Wave-private ascending sort of P (power of two, <= 512) keys in LDS.
__device__ __forceinline__ void wave_bitonic_sort_lds(uint64_t* keys, int P, int lane) {
  for (int k = 2; k <= P; k <<= 1) {
    for (int j = k >> 1; j > 0; j >>= 1) {
      for (int t = lane; t < (P >> 1); t += 64) {
        const int i = ((t & ~(j - 1)) << 1) | (t & (j - 1));
        const int p = i | j;
        const bool asc = (i & k) == 0;
        const uint64_t a = keys[i], b = keys[p];
        if ((a > b) == asc) {
          keys[i] = b;
          keys[p] = a;
        }
      }
      __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
      __builtin_amdgcn_wave_barrier();
    }
  }
}

// Reduce the candidate buffer of one query to its kp best, by one wave:
// buf[0..n) -> sorted buf[0..min(n,kp)); returns the new count and updates the
// query's bound when at least kp candidates exist.
__device__ __forceinline__ int wave_compact_topk(uint64_t* buf, int n, int kp, uint64_t* scratch, float* bound,
                                                 int lane) {
  const int P = next_pow2(n < 2 ? 2 : n);
  for (int i = lane; i < P; i += 64) scratch[i] = i < n ? buf[i] : kPadKey;
  __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
  __builtin_amdgcn_wave_barrier();
  wave_bitonic_sort_lds(scratch, P, lane);
  const int keep = n < kp ? n : kp;
  for (int i = lane; i < keep; i += 64) buf[i] = scratch[i];
  if (n >= kp && lane == 0) *bound = key_score(scratch[kp - 1]);
  return keep;
}

// ---------------------------------------------------------------------------
// Corpus scan fused with top-k.
//
// Operand A = corpus rows (TN per tile), operand B = the query tile (TM rows,
// fixed for the block).  Grid: x = blocks sharing the corpus (each owns a
// contiguous range of tiles), y = query tiles.  The kernel serves miss counts
// M with m_lo < M <= m_hi and returns at once otherwise, so the host can launch
// the tile shapes for small, medium and large M back to back without knowing M.
//
// A launch covers the queries m_base + blockIdx.y*TM + (0..TM-1) of the miss list.
//
// Running top-k per (block, query): a bound T (the kp-th best score seen by this
// block, +inf until kp rows were seen) and a buffer of kTopkCap packed keys in
// global memory.  After each tile every score at or below T is appended; when a
// buffer could overflow on the next tile it is sorted and cut back to kp
// entries by one wave, which also tightens T.  T never drops below the true
// kp-th best score, so no row of the final answer is ever filtered out; the
// bound may start from the kp-th best score of a sample (`seed`: one sorted
// kp-entry list per query, or null).  At the end each query's
// buffer is cut to kp sorted entries and written to
//   out[((m0 + q) * gridDim.x + blockIdx.x) * kp ..]   (padded with kPadKey).
// ---------------------------------------------------------------------------
template <int TM, int TN, int DT>
__global__ __launch_bounds__(256, 2) void scan_mfma_topk_kernel(
    const void* __restrict__ X, const float* __restrict__ xnrm, long n_rows, int dim,
    const float* __restrict__ Qbase, const int* __restrict__ qlist, const int* __restrict__ m_count_ptr,
    int m_limit, int m_base, int m_lo, int m_hi, int kp, const uint64_t* __restrict__ seed,
    uint64_t* __restrict__ cand_buf, uint64_t* __restrict__ out, int cosine) {
  constexpr int WR = TM >= 128 ? 2 : 4;        // waves along corpus rows
  constexpr int WC = 4 / WR;                   // waves along queries
  constexpr int RB = TN / WR / 32;             // 32-row blocks per wave
  constexpr int CB = TM / WC / 32;             // 32-query blocks per wave
  static_assert(RB >= 1 && CB >= 1, "tile too small for four waves");

  const int M = m_count_ptr ? min(*m_count_ptr, m_limit) : m_limit;
  if (M <= m_lo || M > m_hi) return;
  const int m0 = m_base + blockIdx.y * TM;
  if (m0 >= M) return;

  __shared__ __attribute__((aligned(16))) float As[TN * kLdsK];
  __shared__ __attribute__((aligned(16))) float Bs[TM * kLdsK];
  __shared__ uint64_t sort_scratch[4][kTopkCap];
  __shared__ float bound[TM];
  __shared__ int count[TM];
  __shared__ float tile_nrm[TN];

  const int tid = threadIdx.x, lane = tid & 63, wib = tid >> 6;
  const int wr = wib % WR, wc = wib / WR;
  const int a_row0 = wr * (TN / WR), b_row0 = wc * (TM / WC);

  for (int i = tid; i < TM; i += 256) {
    // starting bound: the kp-th best score of a sample of the corpus, if the caller has one
    // (a padding key gives +inf); any value at or above the true kp-th best score is valid
    bound[i] = (seed && m0 + i < M) ? key_score(seed[long(m0 + i) * kp + kp - 1]) : __uint_as_float(0x7f800000u);
    count[i] = 0;
  }

  // this block's share of the corpus tiles
  const long n_tiles = (n_rows + TN - 1) / TN;
  const long t_begin = n_tiles * blockIdx.x / gridDim.x;
  const long t_end = n_tiles * (blockIdx.x + 1) / gridDim.x;
  uint64_t* my_buf = cand_buf + (long(blockIdx.y) * gridDim.x + blockIdx.x) * long(TM) * kTopkCap;

  // query rows of this block (operand B)
  SlabF32<TM> qs;
  const float* qrows[SlabF32<TM>::NCH];
#pragma unroll
  for (int i = 0; i < SlabF32<TM>::NCH; ++i) {
    const int r = (tid + 256 * i) >> 3;
    const int m = m0 + r;
    qrows[i] = m < M ? Qbase + long(qlist ? qlist[m] : m) * dim : nullptr;
  }

  using SlabX = typename std::conditional<DT == kDtypeF32, SlabF32<TN>, SlabBF16<TN>>::type;
  using XElem = typename std::conditional<DT == kDtypeF32, float, uint16_t>::type;
  constexpr int XCH = SlabX::NCH;
  constexpr int XCPR = DT == kDtypeF32 ? 8 : 4;  // chunks per row
  SlabX xs;
  const int n_slabs = dim / kSlabK;

  for (long tile = t_begin; tile < t_end; ++tile) {
    const long row0 = tile * TN;
    const XElem* xrows[XCH];
#pragma unroll
    for (int i = 0; i < XCH; ++i) {
      const long r = row0 + (tid + 256 * i) / XCPR;
      xrows[i] = (r < n_rows && (tid + 256 * i) < TN * XCPR) ? static_cast<const XElem*>(X) + r * dim : nullptr;
    }
    for (int i = tid; i < TN; i += 256) tile_nrm[i] = row0 + i < n_rows ? xnrm[row0 + i] : 0.f;

    f32x16 acc[RB][CB];
#pragma unroll
    for (int i = 0; i < RB; ++i)
#pragma unroll
      for (int j = 0; j < CB; ++j)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    xs.load(xrows, 0, tid);
    qs.load(qrows, 0, tid);
    for (int s = 0; s < n_slabs; ++s) {
      __syncthreads();  // everyone is done reading the previous slab
      xs.store(As, tid);
      qs.store(Bs, tid);
      __syncthreads();
      if (s + 1 < n_slabs) {
        xs.load(xrows, (s + 1) * kSlabK, tid);
        qs.load(qrows, (s + 1) * kSlabK, tid);
      }
      mfma_slab<RB, CB>(As, Bs, a_row0, b_row0, lane, acc);
    }

    // epilogue: scores below the query's bound go to its buffer
    float T[CB];
#pragma unroll
    for (int j = 0; j < CB; ++j) T[j] = bound[b_row0 + 32 * j + (lane & 31)];
#pragma unroll
    for (int i = 0; i < RB; ++i) {
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int lr = a_row0 + 32 * i + 8 * (e >> 2) + 4 * (lane >> 5) + (e & 3);
        const long row = row0 + lr;
        const float nr = tile_nrm[lr];
#pragma unroll
        for (int j = 0; j < CB; ++j) {
          const int q = b_row0 + 32 * j + (lane & 31);
          const float sc = row_score(nr, acc[i][j][e], cosine);
          if (sc <= T[j] && row < n_rows && m0 + q < M) {
            const int pos = atomicAdd(&count[q], 1);
            my_buf[long(q) * kTopkCap + pos] = pack_key(sc, uint32_t(row));
          }
        }
      }
    }
    __syncthreads();
    // cut back buffers that the next tile could overflow
    for (int q = wib; q < TM; q += 4) {
      const int n = count[q];
      if (n > kTopkCap - TN) {
        const int keep = wave_compact_topk(my_buf + long(q) * kTopkCap, n, kp, sort_scratch[wib], &bound[q], lane);
        if (lane == 0) count[q] = keep;
      }
    }
    // (the barrier at the top of the next slab loop orders these LDS writes before the next epilogue)
  }

  __syncthreads();
  for (int q = wib; q < TM; q += 4) {
    if (m0 + q >= M) continue;
    const int n = count[q];
    uint64_t* buf = my_buf + long(q) * kTopkCap;
    const int keep = wave_compact_topk(buf, n, kp, sort_scratch[wib], &bound[q], lane);
    uint64_t* o = out + (long(m0 + q) * gridDim.x + blockIdx.x) * kp;
    for (int i = lane; i < kp; i += 64) o[i] = i < keep ? sort_scratch[wib][i] : kPadKey;
  }
}

__device__ __forceinline__ float f4_get(const float4& v, int e) {
  return e == 0 ? v.x : e == 1 ? v.y : e == 2 ? v.z : v.w;
}

// ---------------------------------------------------------------------------
// Corpus scan fused with top-k, operands moved global -> LDS by the load unit
// itself (global_load_lds_dwordx4, gfx950), three slabs deep.
//
// Same contract and running top-k as scan_mfma_topk_kernel.  Differences:
//  * no register staging: each wave issues NL loads per slab whose 64 lanes
//    write 1 KiB = 8 rows x 128 bytes straight into the slab's LDS stage;
//  * LDS rows are 128 bytes with no padding; instead lane l of a load fetches
//    the 16-byte column chunk (l%8) xor ((r/2)%8) of its stage row r, so chunk c of
//    row r sits at position c xor ((r/2)%8).  A 16-byte LDS read is served 16 lanes
//    at a time; the sixteen lanes that read the same chunk of sixteen consecutive
//    rows for the matrix instruction then cover all 64 banks exactly once (with
//    c xor (r%8) rows r and r+8 collide and every read takes twice as long);
//  * a ring of three stages: while slab s is multiplied, slabs s+1 and s+2 are
//    in flight, and one barrier per slab suffices (it both publishes slab s and
//    retires the stage that slab s+2 will overwrite);
//  * a stage is (TN + TM) x 128 bytes = 24 KiB, so two blocks fit a CU and hide each
//    other's barriers (TM = 96: 28 KiB, one block per CU; still quicker than padding
//    65..96 queries to the 128-query shape).
// The compaction scratch is the stage that was consumed last, which stays free
// until the next slab's loads are issued.
// DUMP = true turns the selection off: every score is written as a key to
// out[query * n_rows + row] (used on a short head of the corpus, whose merged
// kp-th best score then seeds the bounds of the full scan).
// ---------------------------------------------------------------------------
__device__ __forceinline__ void lds_dma16(const float* gptr, float* lds_wave_base) {
  __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)gptr,
                                   (__attribute__((address_space(3))) void*)lds_wave_base, 16, 0, 0);
}
// the same with the nontemporal cache policy (aux bit 1), for rows that are read once
__device__ __forceinline__ void lds_dma16_once(const float* gptr, float* lds_wave_base) {
  __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)gptr,
                                   (__attribute__((address_space(3))) void*)lds_wave_base, 16, 0, 2);
}

template <int TM, bool DUMP>
__global__ __launch_bounds__(256, TM == 96 ? 1 : 2) void scan_mfma_dma_kernel(
    const float* __restrict__ X, const float* __restrict__ xnrm, long n_rows, int dim,
    const float* __restrict__ Qbase, const int* __restrict__ qlist, const int* __restrict__ m_count_ptr,
    int m_limit, int m_base, int m_lo, int m_hi, int kp, const uint64_t* __restrict__ seed,
    uint64_t* __restrict__ cand_buf, uint64_t* __restrict__ out, int cosine) {
  constexpr int TN = TM >= 128 ? 64 : 128;      // corpus rows per tile
  constexpr int WR = TN / 32;                   // waves along corpus rows (32 rows each)
  constexpr int WC = 4 / WR;                    // waves along queries
  constexpr int CB = TM / WC / 32;              // 32-query blocks per wave
  constexpr int ROWS = TN + TM;                 // rows of one stage: corpus tile, then query tile
  constexpr int NL = ROWS / 8 / 4;              // loads per wave per slab
  constexpr int STAGE = ROWS * 32;              // floats per stage
  static_assert(ROWS % 32 == 0 && STAGE * 4 >= 4 * kTopkCap * 8, "stage must hold the compaction scratch");

  const int M = m_count_ptr ? min(*m_count_ptr, m_limit) : m_limit;
  if (M <= m_lo || M > m_hi) return;
  const int m0 = m_base + blockIdx.y * TM;
  if (m0 >= M) return;

  // three stages as three objects, so that the compiler can tell that reading one stage does not
  // depend on the loads in flight into another (it then adds no vmcnt wait of its own)
  __shared__ __attribute__((aligned(1024))) float ring0[STAGE];
  __shared__ __attribute__((aligned(1024))) float ring1[STAGE];
  __shared__ __attribute__((aligned(1024))) float ring2[STAGE];
#define PROX_RING(s) ((s) == 0 ? ring0 : (s) == 1 ? ring1 : ring2)
  __shared__ float bound[TM];
  __shared__ int count[TM];
  __shared__ __attribute__((aligned(256))) float nrm_ring[2][4][64];  // [tile parity][wave][row], filled by DMA

  const int tid = threadIdx.x, lane = tid & 63, wib = tid >> 6;
  const int r32 = lane & 31, half = lane >> 5;
  const int a_row0 = (wib % WR) * 32;                   // this wave's corpus rows within the tile
  const int b_row0 = TN + (wib / WR) * (TM / WC);       // this wave's query rows within the stage

  for (int i = tid; i < TM; i += 256) {
    // starting bound: the kp-th best score of a sample of the corpus, if the caller has one
    // (a padding key gives +inf); any value at or above the true kp-th best score is valid
    bound[i] = (seed && m0 + i < M) ? key_score(seed[long(m0 + i) * kp + kp - 1]) : __uint_as_float(0x7f800000u);
    count[i] = 0;
  }

  const long n_tiles = (n_rows + TN - 1) / TN;
  const long t_begin = n_tiles * blockIdx.x / gridDim.x;
  const long t_end = n_tiles * (blockIdx.x + 1) / gridDim.x;
  const long total = (t_end - t_begin) * (dim / kSlabK);  // slabs this block multiplies
  uint64_t* my_buf = cand_buf + (long(blockIdx.y) * gridDim.x + blockIdx.x) * long(TM) * kTopkCap;
  const int n_slabs = dim / kSlabK;

  // load duty of this lane: NL loads per slab, load i covers stage rows 8*(wib*NL+i) .. +7;
  // the lane fetches column chunk (l%8) xor swizzle(stage row) of its row
  const float* src[NL];
  bool is_x[NL];
  int my_chunk[NL];
#pragma unroll
  for (int i = 0; i < NL; ++i) {
    const int srow = 8 * (wib * NL + i) + (lane >> 3);
    my_chunk[i] = (lane & 7) ^ ((srow >> 1) & 7);
    is_x[i] = srow < TN;
    if (!is_x[i]) {
      int m = m0 + srow - TN;
      m = m < M ? m : M - 1;
      src[i] = Qbase + long(qlist ? qlist[m] : m) * dim + 4 * my_chunk[i];
    }
  }
  auto point_at_tile = [&](long tile) {
#pragma unroll
    for (int i = 0; i < NL; ++i)
      if (is_x[i]) {
        long r = tile * TN + 8 * (wib * NL + i) + (lane >> 3);
        r = r < n_rows ? r : n_rows - 1;
        src[i] = X + r * dim + 4 * my_chunk[i];
      }
  };
  // issue stream: slab number `is` (flat over this block's tiles), one group of NL loads per call
  long is = 0;
  long itile = t_begin;
  int islab = 0;
  auto issue = [&](float* stage) {
    if (is >= total) return;
    if (islab == 0) {
      point_at_tile(itile);
      // norms of this wave's 32 rows of the tile, parked in LDS until the tile's scores are filtered
      // (with at least two slabs per tile only two tiles are ever live: the one multiplied and the next)
      long rn = itile * TN + a_row0 + r32;
      rn = rn < n_rows ? rn : n_rows - 1;
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(xnrm + rn),
                                       (__attribute__((address_space(3))) void*)&nrm_ring[itile & 1][wib][0], 4, 0,
                                       0);
    }
    float* base = stage + (wib * NL) * 256;
#pragma unroll
    for (int i = 0; i < NL; ++i) {
      if (is_x[i])
        lds_dma16_once(src[i] + islab * kSlabK, base + i * 256);  // corpus rows: streamed once
      else
        lds_dma16(src[i] + islab * kSlabK, base + i * 256);       // query rows: re-read by every block
    }
    ++is;
    if (++islab == n_slabs) {
      islab = 0;
      ++itile;
    }
  };

  f32x16 acc[CB];
#pragma unroll
  for (int j = 0; j < CB; ++j)
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[j][e] = 0.f;

  auto multiply = [&](const float* st) {
    const int sw = (r32 >> 1) & 7;  // swizzle of every row this lane reads: row offsets are multiples of 32
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      const int pos = ((2 * t + half) ^ sw) * 4;
      const float4 a = *reinterpret_cast<const float4*>(st + (a_row0 + r32) * 32 + pos);
      float4 b[CB];
#pragma unroll
      for (int j = 0; j < CB; ++j) b[j] = *reinterpret_cast<const float4*>(st + (b_row0 + 32 * j + r32) * 32 + pos);
#pragma unroll
      for (int e = 0; e < 4; ++e)
#pragma unroll
        for (int j = 0; j < CB; ++j)
          acc[j] = __builtin_amdgcn_mfma_f32_32x32x2f32(f4_get(a, e), f4_get(b[j], e), acc[j], 0, 0, 0);
    }
  };

  long ctile = t_begin;
  int cslab = 0;
  // A buffer is cut back as soon as it holds clearly more than kp entries (so that the bound
  // tightens early), and in any case before the next tile could overflow it.
  const int trigger = min(kTopkCap - TN, max(2 * kp, 64));
  const uint32_t count_lds = uint32_t(uintptr_t((__attribute__((address_space(3))) int*)&count[0]));
  auto end_of_tile = [&](float* consumed_stage) {
    const long row0 = ctile * TN + a_row0;
    const int qb0 = b_row0 - TN;
    if (DUMP) {
      // no selection here: every score goes out as a key, out[query][row], for the merge kernels
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int lr = 8 * (e >> 2) + 4 * half + (e & 3);
        const float nr = nrm_ring[ctile & 1][wib][lr];
#pragma unroll
        for (int j = 0; j < CB; ++j) {
          const int q = m0 + qb0 + 32 * j + r32;
          if (q < M && row0 + lr < n_rows) out[long(q) * n_rows + row0 + lr] = pack_key(row_score(nr, acc[j][e], cosine), uint32_t(row0 + lr));
          acc[j][e] = 0.f;
        }
      }
      return;
    }
    // pass 1: turn accumulators into scores and note which ones beat the query's bound
    uint32_t pass[CB];
#pragma unroll
    for (int j = 0; j < CB; ++j) pass[j] = 0;
    float T[CB];
#pragma unroll
    for (int j = 0; j < CB; ++j) T[j] = (m0 + qb0 + 32 * j + r32 < M) ? bound[qb0 + 32 * j + r32] : -__builtin_inff();
#pragma unroll
    for (int e = 0; e < 16; ++e) {
      const int lr = 8 * (e >> 2) + 4 * half + (e & 3);
      const float nr = nrm_ring[ctile & 1][wib][lr];
      const bool row_ok = row0 + lr < n_rows;
#pragma unroll
      for (int j = 0; j < CB; ++j) {
        const float sc = row_score(nr, acc[j][e], cosine);
        acc[j][e] = sc;
        pass[j] |= (sc <= T[j] && row_ok) ? (1u << e) : 0u;
      }
    }
    // pass 2: one LDS counter update per (lane, query) reserves room, then plain stores.
    // The counter update is written in assembly so that the compiler does not guard it with a
    // wait for the global->LDS loads in flight (they never touch the counters).
#pragma unroll
    for (int j = 0; j < CB; ++j) {
      if (pass[j]) {
        const int q = qb0 + 32 * j + r32;
        uint32_t pos;
        asm volatile("ds_add_rtn_u32 %0, %1, %2\n\ts_waitcnt lgkmcnt(0)"
                     : "=v"(pos)
                     : "v"(count_lds + 4u * uint32_t(q)), "v"(uint32_t(__builtin_popcount(pass[j])))
                     : "memory");
        uint64_t* dst = my_buf + long(q) * kTopkCap;
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          if (pass[j] & (1u << e)) {
            const int lr = 8 * (e >> 2) + 4 * half + (e & 3);
            dst[pos++] = pack_key(acc[j][e], uint32_t(row0 + lr));
          }
        }
      }
    }
#pragma unroll
    for (int j = 0; j < CB; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[j][e] = 0.f;
    // Do any buffers have to be cut back before the next tile?  Every wave reads the same counts
    // after a plain barrier (no memory fence: loads in flight stay in flight), so all agree.
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
    bool mine = false;
    for (int q = lane; q < TM; q += 64) mine |= count[q] > trigger;
    if (__any(mine)) {
      __syncthreads();  // full fence: the candidates other waves appended must be visible
      uint64_t* scratch = reinterpret_cast<uint64_t*>(consumed_stage) + wib * kTopkCap;
      for (int q = wib; q < TM; q += 4) {
        const int n = count[q];
        if (n > trigger) {
          const int keep = wave_compact_topk(my_buf + long(q) * kTopkCap, n, kp, scratch, &bound[q], lane);
          if (lane == 0) count[q] = keep;
        }
      }
    }
    // the barrier at the top of the next slab orders these LDS writes
  };

  issue(ring0);
  issue(ring1);
  for (long it = 0; it < total;) {
#pragma unroll
    for (int stage = 0; stage < 3; ++stage) {
      if (it < total) {
        // slab `it` must have landed; the group issued after it (slab it+1) may stay in flight.
        // Plain barrier: it publishes slab `it` to all waves and retires the stage that slab
        // it+2 is about to overwrite.
        if (it + 1 < total)
          asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" ::"n"(NL) : "memory");
        else
          asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)\n\ts_barrier" ::: "memory");
        issue(PROX_RING((stage + 2) % 3));
        multiply(PROX_RING(stage));
        if (++cslab == n_slabs) {
          end_of_tile(PROX_RING(stage));
          cslab = 0;
          ++ctile;
        }
        ++it;
      }
    }
  }

  if (DUMP) return;
  __syncthreads();
  uint64_t* scratch = reinterpret_cast<uint64_t*>(ring0) + wib * kTopkCap;
  for (int q = wib; q < TM; q += 4) {
    if (m0 + q >= M) continue;
    const int n = count[q];
    uint64_t* buf = my_buf + long(q) * kTopkCap;
    const int keep = wave_compact_topk(buf, n, kp, scratch, &bound[q], lane);
    uint64_t* o = out + (long(m0 + q) * gridDim.x + blockIdx.x) * kp;
    for (int i = lane; i < kp; i += 64) o[i] = i < keep ? scratch[i] : kPadKey;
  }
#undef PROX_RING
}

// One 128 x 128 tile of the dense probe (see probe_mfma_dense_kernel): source tile tile_x, query tile tile_y.
// With row_list, query m is row row_list[m] of Q and its scores go to row row_list[m] - row_origin of D.
__device__ __forceinline__ void probe_mfma_dense_tile(const float* __restrict__ srcs, const float* __restrict__ srcnrm,
                                                      int n_src, const float* __restrict__ Q, int n_q, int dim,
                                                      float* __restrict__ D, long ldD, const int* __restrict__ row_list,
                                                      int row_origin, int tile_x, int tile_y) {
  constexpr int T = 128, RB = 2, CB = 2;
  __shared__ __attribute__((aligned(16))) float As[T * kLdsK];
  __shared__ __attribute__((aligned(16))) float Bs[T * kLdsK];
  const int tid = threadIdx.x, lane = tid & 63, wib = tid >> 6;
  const int a_row0 = (wib & 1) * 64, b_row0 = (wib >> 1) * 64;
  const int q0 = tile_y * T, s0 = tile_x * T;

  SlabF32<T> qa, sb;
  const float* qrows[SlabF32<T>::NCH];
  const float* srows[SlabF32<T>::NCH];
#pragma unroll
  for (int i = 0; i < SlabF32<T>::NCH; ++i) {
    const int r = (tid + 256 * i) >> 3;
    qrows[i] = q0 + r < n_q ? Q + long(row_list ? row_list[q0 + r] : q0 + r) * dim : nullptr;
    srows[i] = s0 + r < n_src ? srcs + long(s0 + r) * dim : nullptr;
  }
  f32x16 acc[RB][CB];
#pragma unroll
  for (int i = 0; i < RB; ++i)
#pragma unroll
    for (int j = 0; j < CB; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  const int n_slabs = dim / kSlabK;
  qa.load(qrows, 0, tid);
  sb.load(srows, 0, tid);
  for (int s = 0; s < n_slabs; ++s) {
    __syncthreads();
    qa.store(As, tid);
    sb.store(Bs, tid);
    __syncthreads();
    if (s + 1 < n_slabs) {
      qa.load(qrows, (s + 1) * kSlabK, tid);
      sb.load(srows, (s + 1) * kSlabK, tid);
    }
    mfma_slab<RB, CB>(As, Bs, a_row0, b_row0, lane, acc);
  }
#pragma unroll
  for (int j = 0; j < CB; ++j) {
    const int sidx = s0 + b_row0 + 32 * j + (lane & 31);
    const float sn = sidx < n_src ? srcnrm[sidx] : 0.f;
#pragma unroll
    for (int i = 0; i < RB; ++i)
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int q = q0 + a_row0 + 32 * i + 8 * (e >> 2) + 4 * (lane >> 5) + (e & 3);
        if (q < n_q && sidx < n_src) D[long(row_list ? row_list[q] - row_origin : q) * ldD + sidx] = sn - 2.f * acc[i][j][e];
      }
  }
}


// ---------------------------------------------------------------------------
// Cache probe, dense output.  Operand A = batch rows (queries), operand B =
// sources [slot keys ; batch rows]; D[(m) * ldD + s] = |s|^2 - 2 q_m . s.
// Grid: x = source tiles of 128, y = query tiles of 128.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256, 2) void probe_mfma_dense_kernel(const float* __restrict__ srcs,
                                                                  const float* __restrict__ srcnrm, int n_src,
                                                                  const float* __restrict__ Q, int n_q, int dim,
                                                                  float* __restrict__ D, long ldD) {
  probe_mfma_dense_tile(srcs, srcnrm, n_src, Q, n_q, dim, D, ldD, nullptr, 0, blockIdx.x, blockIdx.y);
}

// The same for the rows row_list[0 .. *row_count) of Q, whose scores go to row row_list[m] - row_origin of D: the
// dense rows of just those batch rows whose candidate list overflowed.  The grid does not depend on their number
// (which the host does not know, and which is zero as a rule): blocks share the tiles round robin.
__global__ __launch_bounds__(256, 2) void probe_mfma_dense_listed_kernel(
    const float* __restrict__ srcs, const float* __restrict__ srcnrm, int n_src, const float* __restrict__ Q, int dim,
    float* __restrict__ D, long ldD, const int* __restrict__ row_list, const int* __restrict__ row_count,
    int row_origin) {
  const int n_q = *row_count;
  if (n_q == 0) return;
  const int tx = (n_src + 127) / 128, ty = (n_q + 127) / 128;
  for (int t = blockIdx.x; t < tx * ty; t += gridDim.x) {
    __syncthreads();  // the tile before has been read out of LDS
    probe_mfma_dense_tile(srcs, srcnrm, n_src, Q, n_q, dim, D, ldD, row_list, row_origin, t % tx, t / tx);
  }
}

// ---------------------------------------------------------------------------
// The same probe for shapes too small to fill the chip with 128 x 128 tiles, where the time
// of the kernel above is the latency of one block walking the whole contraction.
// A block owns 32 sources x 32 queries; its four waves each take a quarter of the columns
// (dim must be a multiple of 32) and feed the matrix instruction straight from global memory:
// per step of 8 columns a lane reads 16 bytes of its source row and of its query row (lanes
// 0-31 columns 8t..8t+3, lanes 32-63 columns 8t+4..8t+7; register e of both operands pairs
// column 8t+e with 8t+4+e).  The four partial tiles are added through LDS.
// Grid: x = source tiles of 32, y = query tiles of 32.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void probe_mfma_small_kernel(const float* __restrict__ srcs,
                                                               const float* __restrict__ srcnrm, int n_src,
                                                               const float* __restrict__ Q, int n_q, int dim,
                                                               float* __restrict__ D, long ldD) {
  constexpr int U = 8;  // steps whose loads are issued together
  __shared__ float part[4][16][64];
  const int tid = threadIdx.x, lane = tid & 63, wib = tid >> 6;
  const int r32 = lane & 31, half = lane >> 5;
  const int s0 = blockIdx.x * 32, q0 = blockIdx.y * 32;
  const int steps = dim / 32;  // steps of 8 columns per wave
  const int srow = s0 + r32 < n_src ? s0 + r32 : n_src - 1;   // rows past the end repeat the last one;
  const int qrow = q0 + r32 < n_q ? q0 + r32 : n_q - 1;       // their results are not written
  const float* ps = srcs + long(srow) * dim + wib * (dim / 4) + 4 * half;
  const float* pq = Q + long(qrow) * dim + wib * (dim / 4) + 4 * half;

  f32x16 acc;
#pragma unroll
  for (int e = 0; e < 16; ++e) acc[e] = 0.f;
  for (int t0 = 0; t0 < steps; t0 += U) {
    float4 a[U], b[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      if (t0 + u < steps) {
        a[u] = *reinterpret_cast<const float4*>(pq + 8 * (t0 + u));
        b[u] = *reinterpret_cast<const float4*>(ps + 8 * (t0 + u));
      } else {
        a[u] = make_float4(0.f, 0.f, 0.f, 0.f);
        b[u] = a[u];
      }
    }
#pragma unroll
    for (int u = 0; u < U; ++u)
#pragma unroll
      for (int e = 0; e < 4; ++e)
        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(f4_get(a[u], e), f4_get(b[u], e), acc, 0, 0, 0);
  }
#pragma unroll
  for (int e = 0; e < 16; ++e) part[wib][e][lane] = acc[e];
  __syncthreads();
  // element e of lane l is query 8*(e/4) + 4*(l/32) + e%4 against source l%32
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int e = wib + 4 * i;
    const float dot = part[0][e][lane] + part[1][e][lane] + part[2][e][lane] + part[3][e][lane];
    const int q = q0 + 8 * (e >> 2) + 4 * half + (e & 3);
    const int sidx = s0 + r32;
    if (q < n_q && sidx < n_src) D[long(q) * ldD + sidx] = srcnrm[sidx] - 2.f * dot;
  }
}

}  // namespace prox
