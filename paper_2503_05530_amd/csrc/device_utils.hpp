// Small device-side helpers shared by the kernels of this library (gfx950, wave64).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace prox {

constexpr int kWave = 64;
constexpr int kDtypeF32 = 0;
constexpr int kDtypeBF16 = 1;

// A candidate neighbour is a (score, id) pair packed into one 64-bit key whose
// unsigned order is "ascending score, then ascending id".  The float is mapped
// to an unsigned integer with the same order (sign bit flipped for
// non-negatives, all bits flipped for negatives).
__device__ __forceinline__ uint32_t float_to_ordered(float f) {
  uint32_t u = __float_as_uint(f);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
__device__ __forceinline__ float ordered_to_float(uint32_t o) {
  uint32_t u = (o & 0x80000000u) ? (o & 0x7fffffffu) : ~o;
  return __uint_as_float(u);
}
__device__ __forceinline__ uint64_t pack_key(float score, uint32_t id) {
  return (uint64_t(float_to_ordered(score)) << 32) | uint64_t(id);
}
__device__ __forceinline__ float key_score(uint64_t key) { return ordered_to_float(uint32_t(key >> 32)); }
__device__ __forceinline__ int32_t key_id(uint64_t key) { return int32_t(uint32_t(key)); }

// Padding entry: score +inf, id -1.  Sorts after every real entry.
constexpr uint64_t kPadKey = 0xFF800000FFFFFFFFull;

__device__ __forceinline__ float bf16_to_float(uint16_t b) { return __uint_as_float(uint32_t(b) << 16); }

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int m = 32; m >= 1; m >>= 1) v += __shfl_xor(v, m, kWave);
  return v;
}
// v + (v moved across lanes by the data-parallel-primitive control CTRL); lanes the move does not
// reach (outside ROW_MASK, or shifted in from beyond a row of 16) add zero.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ double dpp_move_add(double v) {
  const unsigned long long bits = (unsigned long long)__double_as_longlong(v);
  const int lo = __builtin_amdgcn_update_dpp(0, int(unsigned(bits)), CTRL, ROW_MASK, 0xf, false);
  const int hi = __builtin_amdgcn_update_dpp(0, int(unsigned(bits >> 32)), CTRL, ROW_MASK, 0xf, false);
  return v + __longlong_as_double((long long)(((unsigned long long)unsigned(hi) << 32) | unsigned(lo)));
}
// Sum of a float64 over the wave, the same value in every lane.  The shuffle form costs twelve
// trips through the LDS crossbar; this one stays in the vector unit: a running sum inside every
// row of 16 lanes (shifts by 1, 2, 4, 8), then the row totals are handed on (lane 15 to the
// next row for rows 1 and 3, lane 31 to rows 2 and 3), and lane 63 holds the total.
__device__ __forceinline__ double wave_sum(double v) {
  v = dpp_move_add<0x111, 0xf>(v);  // row_shr:1
  v = dpp_move_add<0x112, 0xf>(v);  // row_shr:2
  v = dpp_move_add<0x114, 0xf>(v);  // row_shr:4
  v = dpp_move_add<0x118, 0xf>(v);  // row_shr:8
  v = dpp_move_add<0x142, 0xa>(v);  // row_bcast:15 into rows 1 and 3
  v = dpp_move_add<0x143, 0xc>(v);  // row_bcast:31 into rows 2 and 3
  const unsigned long long bits = (unsigned long long)__double_as_longlong(v);
  const unsigned lo = unsigned(__builtin_amdgcn_readlane(int(unsigned(bits)), 63));
  const unsigned hi = unsigned(__builtin_amdgcn_readlane(int(unsigned(bits >> 32)), 63));
  return __longlong_as_double((long long)(((unsigned long long)hi << 32) | lo));
}

// Sum NV per-lane values across the 64 lanes of a wave with NV-1 + log2(64/NV)
// exchanges instead of 6*NV.  Each exchange step halves the number of values a
// lane carries: the lane whose bit `mask` is clear keeps the lower half of its
// values and receives its partner's lower half, the other lane keeps the upper
// half.  On return v[0] of lane l is the wave-wide sum of the input value with
// index value_index_of_lane<NV>(l).
template <int NV>
__device__ __forceinline__ void wave_sum_transposed(float (&v)[NV], int lane) {
  static_assert((NV & (NV - 1)) == 0 && NV >= 1 && NV <= 64, "NV must be a power of two");
  int mask = 1;
#pragma unroll
  for (int n = NV; n > 1; n >>= 1) {
    const bool upper = (lane & mask) != 0;
#pragma unroll
    for (int i = 0; i < n / 2; ++i) {
      const float send = upper ? v[i] : v[i + n / 2];
      const float keep = upper ? v[i + n / 2] : v[i];
      v[i] = keep + __shfl_xor(send, mask, kWave);
    }
    mask <<= 1;
  }
#pragma unroll
  for (int m = NV; m < kWave; m <<= 1) v[0] += __shfl_xor(v[0], m, kWave);
}

// Index of the input value whose total lane l holds after wave_sum_transposed<NV>.
template <int NV>
__device__ __forceinline__ int value_index_of_lane(int lane) {
  int idx = 0;
  int bit = 0;
#pragma unroll
  for (int n = NV; n > 1; n >>= 1) {
    idx += ((lane >> bit) & 1) * (n / 2);
    ++bit;
  }
  return idx;
}

// Ascending bitonic sort of P (power of two) 64-bit keys in LDS by all threads
// of the block.  Ends with a barrier.
__device__ __forceinline__ void block_bitonic_sort(uint64_t* keys, int P, int tid, int nthreads) {
  for (int k = 2; k <= P; k <<= 1) {
    for (int j = k >> 1; j > 0; j >>= 1) {
      for (int t = tid; t < (P >> 1); t += nthreads) {
        const int i = ((t & ~(j - 1)) << 1) | (t & (j - 1));
        const int p = i | j;
        const bool asc = (i & k) == 0;
        const uint64_t a = keys[i], b = keys[p];
        if ((a > b) == asc) {
          keys[i] = b;
          keys[p] = a;
        }
      }
      __syncthreads();
    }
  }
}

// Ascending sort of one 64-bit key per lane across a wave (bitonic network on shuffles, no LDS,
// no barrier).  On return lane l holds the (l+1)-th smallest key.
__device__ __forceinline__ uint64_t wave_sort64(uint64_t v, int lane) {
#pragma unroll
  for (int k = 2; k <= kWave; k <<= 1) {
#pragma unroll
    for (int j = k >> 1; j > 0; j >>= 1) {
      const uint64_t other = __shfl_xor(v, j, kWave);
      const bool keep_small = ((lane & k) == 0) == ((lane & j) == 0);
      const uint64_t lo = v < other ? v : other, hi = v < other ? other : v;
      v = keep_small ? lo : hi;
    }
  }
  return v;
}

// A bound B with at least kp of the block's per-thread keys at or below it (kp <= 4 * 64):
// every wave sorts its 64 keys in registers and offers its ceil(kp/NW)-th smallest; the largest
// offer qualifies.  Close to the exact kp-th smallest at a fraction of a block-wide sort.
// `slots` is NW words of LDS; one barrier inside.
template <int NW>
__device__ __forceinline__ uint64_t block_bound_for_kp(uint64_t thread_key, int kp, uint64_t* slots, int tid) {
  const int lane = tid & 63, wib = tid >> 6;
  const uint64_t sorted = wave_sort64(thread_key, lane);
  const int r = (kp + NW - 1) / NW;
  const uint64_t offer = __shfl(sorted, r - 1, kWave);
  if (lane == 0) slots[wib] = offer;
  __syncthreads();
  uint64_t b = slots[0];
#pragma unroll
  for (int w = 1; w < NW; ++w) b = slots[w] > b ? slots[w] : b;
  return b;
}

// Ascending sort of P <= 64 keys held in LDS, done by the first wave in registers; all threads
// of the block must call it.  Ends with a barrier.
__device__ __forceinline__ void block_sort_upto64(uint64_t* keys, int tid) {
  if (tid < kWave) keys[tid] = wave_sort64(keys[tid], tid);
  __syncthreads();
}

__device__ __forceinline__ int next_pow2(int v) {
  int p = 1;
  while (p < v) p <<= 1;
  return p;
}

// Score of a corpus row from its inner product with the query; smaller is closer, and per query
// the order of the scores is the order of the distances (Section 2.2's three distance functions):
//   Euclidean:      |x|^2 - 2 q.x    (row_term = |x|^2; the query's own |q|^2 is the same for every row)
//   inner product:  -2 q.x           (row_term = 0)
//   cosine:         -2 q.x / |x|     (row_term = 1/|x|, `cosine` set)
__device__ __forceinline__ float row_score(float row_term, float dot, int cosine) {
  const float mul = cosine ? -2.f * row_term : -2.f;
  const float add = cosine ? 0.f : row_term;
  return fmaf(dot, mul, add);
}

}  // namespace prox
