// Corpus scan for a bfloat16 corpus on the bfloat16 matrix cores, exact to float32 accuracy.
//
// A float32 query value q splits into three bfloat16 terms q = hi + mid + lo (each the rounding
// of what the previous ones leave; the remainder is below 2^-27 |q|).  A product of two bfloat16
// values is exact in float32, so  q . x = hi . x + mid . x + lo . x  with x in bfloat16 and
// float32 accumulation carries the same rounding as the float32 contraction: only sums round.
// v_mfma_f32_32x32x16_bf16 does sixteen columns per instruction at sixteen times the float32
// matrix rate, so three of them per query beat one float32 pass by more than five to one.
//
// split_bf16x3_kernel writes the three planes of the queries of a call; scan_bf16x3_kernel is
// scan_mfma_dma_kernel with 2-byte values: slabs of 32 columns (64-byte rows), a stage holds the
// corpus tile (128 rows) and the three planes of the query tile (3 x 64 rows), every wave takes
// 32 corpus rows against all 64 queries, and each step of 16 columns issues one matrix
// instruction per plane and query block.  Loads, ring, barriers, running top-k and seeding are the same.
#pragma once

#include "mfma_kernels.hpp"

namespace prox {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
constexpr int kSlabBf16 = 32;  // columns per slab of the bfloat16 scan

__device__ __forceinline__ uint16_t bf16_round(float f) {  // round to nearest even; finite inputs
  const uint32_t u = __float_as_uint(f);
  return uint16_t((u + 0x7fffu + ((u >> 16) & 1u)) >> 16);
}

// planes[p][m][:] (p = 0,1,2: hi, mid, lo) for the queries m < M of the miss list; one block per query.
__global__ __launch_bounds__(256) void split_bf16x3_kernel(const float* __restrict__ Qbase,
                                                           const int* __restrict__ qlist,
                                                           const int* __restrict__ m_count_ptr, int m_limit, int dim,
                                                           uint16_t* __restrict__ planes, long plane_stride) {
  const int m = blockIdx.x;
  const int M = m_count_ptr ? min(*m_count_ptr, m_limit) : m_limit;
  if (m >= M) return;
  const float* q = Qbase + long(qlist ? qlist[m] : m) * dim;
  for (int x = threadIdx.x; x < dim; x += 256) {
    const float v = q[x];
    const uint16_t hi = bf16_round(v);
    const float r1 = v - bf16_to_float(hi);
    const uint16_t mid = bf16_round(r1);
    const float r2 = r1 - bf16_to_float(mid);
    const uint16_t lo = bf16_round(r2);
    planes[long(m) * dim + x] = hi;
    planes[plane_stride + long(m) * dim + x] = mid;
    planes[2 * plane_stride + long(m) * dim + x] = lo;
  }
}

// TM = 64: four waves, 128 corpus rows per tile, two blocks per CU (query counts up to 64);
// TM = 128: eight waves, 256 corpus rows per tile, one block per CU.  The planes of the query tile are
// fetched again for every corpus tile and slab, so per multiply-add a block moves (TN + 3 TM) / (TN TM)
// operand bytes from L2: the larger shape halves that, and for more than 64 queries the corpus is
// streamed once instead of twice.
template <int TM, bool DUMP>
__global__ __launch_bounds__(TM * 4, TM == 128 ? 1 : 2) void scan_bf16x3_kernel(
    const uint16_t* __restrict__ X, const float* __restrict__ xnrm, long n_rows, int dim,
    const uint16_t* __restrict__ Qplanes, long plane_stride, const int* __restrict__ m_count_ptr,
    int m_limit, int m_base, int m_lo, int m_hi, int kp, const uint64_t* __restrict__ seed,
    uint64_t* __restrict__ cand_buf, uint64_t* __restrict__ out, int cosine) {
  constexpr int NW = TM / 16;                   // waves per block
  constexpr int NT = NW * 64;                   // threads per block
  constexpr int TN = 32 * NW;                   // corpus rows per tile (32 per wave)
  constexpr int CB = TM / 32;                   // 32-query blocks per wave (every wave takes all queries)
  constexpr int ROWS = TN + 3 * TM;             // rows of one stage: corpus tile, then the three query planes
  constexpr int NL = ROWS / 16 / NW;            // loads per wave per slab (a load covers 16 rows of 64 bytes)
  constexpr int STAGE = ROWS * 16;              // floats (4-byte units) per stage
  static_assert(ROWS % (16 * NW) == 0 && STAGE * 4 >= NW * kTopkCap * 8, "stage must hold the compaction scratch");

  const int M = m_count_ptr ? min(*m_count_ptr, m_limit) : m_limit;
  if (M <= m_lo || M > m_hi) return;
  const int m0 = m_base + blockIdx.y * TM;
  if (m0 >= M) return;

  // three stages as three objects, so that the compiler can tell that reading one stage does not
  // depend on the loads in flight into another (it then adds no vmcnt wait of its own)
  __shared__ __attribute__((aligned(1024))) float ring0[STAGE];
  __shared__ __attribute__((aligned(1024))) float ring1[STAGE];
  __shared__ __attribute__((aligned(1024))) float ring2[STAGE];
#define PROX_RING3(s) ((s) == 0 ? ring0 : (s) == 1 ? ring1 : ring2)
  __shared__ float bound[TM];
  __shared__ int count[TM];
  __shared__ __attribute__((aligned(256))) float nrm_ring[2][NW][64];  // [tile parity][wave][row], filled by DMA

  const int tid = threadIdx.x, lane = tid & 63, wib = tid >> 6;
  const int r32 = lane & 31, half = lane >> 5;
  const int a_row0 = wib * 32;                          // this wave's corpus rows within the tile
  const int b_row0 = TN;                                // plane p of the query tile starts at stage row TN + p*TM

  for (int i = tid; i < TM; i += NT) {
    // starting bound: the kp-th best score of a sample of the corpus, if the caller has one
    // (a padding key gives +inf); any value at or above the true kp-th best score is valid
    bound[i] = (seed && m0 + i < M) ? key_score(seed[long(m0 + i) * kp + kp - 1]) : __uint_as_float(0x7f800000u);
    count[i] = 0;
  }

  const long n_tiles = (n_rows + TN - 1) / TN;
  const long t_begin = n_tiles * blockIdx.x / gridDim.x;
  const long t_end = n_tiles * (blockIdx.x + 1) / gridDim.x;
  const long total = (t_end - t_begin) * (dim / kSlabBf16);  // slabs this block multiplies
  uint64_t* my_buf = cand_buf + (long(blockIdx.y) * gridDim.x + blockIdx.x) * long(TM) * kTopkCap;
  const int n_slabs = dim / kSlabBf16;

  // load duty of this lane: NL loads per slab, load i covers stage rows 16*(wib*NL+i) .. +15
  // (64 bytes = 32 values each); the lane fetches the 16-byte chunk (l%4) xor swizzle(stage row) of its row
  const uint16_t* src[NL];
  bool is_x[NL];
  int my_chunk[NL];
#pragma unroll
  for (int i = 0; i < NL; ++i) {
    const int srow = 16 * (wib * NL + i) + (lane >> 2);
    my_chunk[i] = (lane & 3) ^ ((srow >> 2) & 3);
    is_x[i] = srow < TN;
    if (!is_x[i]) {
      const int plane = (srow - TN) / TM;
      int m = m0 + (srow - TN) % TM;
      m = m < M ? m : M - 1;
      src[i] = Qplanes + long(plane) * plane_stride + long(m) * dim + 8 * my_chunk[i];
    }
  }
  auto point_at_tile = [&](long tile) {
#pragma unroll
    for (int i = 0; i < NL; ++i)
      if (is_x[i]) {
        long r = tile * TN + 16 * (wib * NL + i) + (lane >> 2);
        r = r < n_rows ? r : n_rows - 1;
        src[i] = X + r * dim + 8 * my_chunk[i];
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
      const float* g = reinterpret_cast<const float*>(src[i] + islab * kSlabBf16);
      // A slab takes 64 bytes of a row, half a cache line: the other half is wanted by the next slab,
      // so corpus rows are not marked read-once here (that would drop the line in between and fetch it twice).
      lds_dma16(g, base + i * 256);
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

  // One slab = two steps of 16 columns.  A lane reads the 8 values (16 bytes) of "its" row that the
  // instruction expects from it: lanes 0-31 columns 16s..16s+7, lanes 32-63 columns 16s+8..16s+15.
  auto multiply = [&](const float* st) {
    const int sw = (r32 >> 2) & 3;  // swizzle of every row this lane reads: row offsets are multiples of 32
#pragma unroll
    for (int s2 = 0; s2 < 2; ++s2) {
      const int pos = ((2 * s2 + half) ^ sw) * 4;
      const bf16x8 a = *reinterpret_cast<const bf16x8*>(st + (a_row0 + r32) * 16 + pos);
      bf16x8 b[3][CB];
#pragma unroll
      for (int p = 0; p < 3; ++p)
#pragma unroll
        for (int j = 0; j < CB; ++j)
          b[p][j] = *reinterpret_cast<const bf16x8*>(st + (b_row0 + p * TM + 32 * j + r32) * 16 + pos);
#pragma unroll
      for (int p = 0; p < 3; ++p)
#pragma unroll
        for (int j = 0; j < CB; ++j) acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b[p][j], acc[j], 0, 0, 0);
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
    const int qb0 = 0;
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
      for (int q = wib; q < TM; q += NW) {
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
        issue(PROX_RING3((stage + 2) % 3));
        multiply(PROX_RING3(stage));
        if (++cslab == n_slabs) {
          end_of_tile(PROX_RING3(stage));
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
  for (int q = wib; q < TM; q += NW) {
    if (m0 + q >= M) continue;
    const int n = count[q];
    uint64_t* buf = my_buf + long(q) * kTopkCap;
    const int keep = wave_compact_topk(buf, n, kp, scratch, &bound[q], lane);
    uint64_t* o = out + (long(m0 + q) * gridDim.x + blockIdx.x) * kp;
    for (int i = lane; i < kp; i += 64) o[i] = i < keep ? scratch[i] : kPadKey;
  }
#undef PROX_RING3
}

}  // namespace prox
