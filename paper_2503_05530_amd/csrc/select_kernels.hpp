// Top-k selection: the ranking step of the index search (Section 2.2 returns a
// *ranked* list of the k closest rows).  Order is ascending (score, id), so equal
// scores rank by ascending document index.
//
// Selection is hierarchical.  A first level turns slices of a dense score row
// into kp-entry sorted lists of packed (score,id) keys; further levels merge
// groups of such lists until one list of kp entries per query is left.  kp is
// k plus a small slack: the final ranking is redone in float64 on those kp rows
// (rerank_f64_kernel) so float32 rounding cannot reorder the k winners.
#pragma once

#include "device_utils.hpp"

namespace prox {

constexpr int kSelThreads = 256;

// One block reduces one segment of one query to its kp smallest keys, sorted.
//
//   DENSE  : input is float scores in[q * in_ld + j], j < len, id = id_base + j
//   !DENSE : input is packed keys   in[q * in_ld + j], j < len
// Segment g covers elements [g*E*256, (g+1)*E*256).  Output out[(q*n_seg+g)*kp ..+kp),
// padded with kPadKey when the segment holds fewer than kp elements.
//
// Method: every thread keeps its E elements in registers and finds its own
// minimum; the kp-th smallest of the 256 thread minima bounds the kp-th smallest
// element from above (kp distinct elements lie at or below it), so only
// elements at or below that bound are compacted into LDS and sorted.  With kp
// up to 256 the expected number of survivors is about 2*kp; exact ties can make
// it as large as the segment, which the LDS list is sized for.
template <bool DENSE, int E>
__global__ __launch_bounds__(kSelThreads) void select_kernel(const void* __restrict__ in, long in_ld, long len,
                                                             long id_base, int kp, uint64_t* __restrict__ out,
                                                             int n_seg, const int* __restrict__ m_count_ptr,
                                                             int m_limit, int m_begin) {
  constexpr int SEG = E * kSelThreads;
  const int q = blockIdx.y;  // query index relative to m_begin; in/out are relative too
  const int m_total = m_count_ptr ? min(*m_count_ptr, m_limit) : m_limit;
  if (m_begin + q >= m_total) return;
  const int g = blockIdx.x;
  const int tid = threadIdx.x;

  __shared__ uint64_t list[SEG];
  __shared__ uint64_t mins[kSelThreads];
  __shared__ int count;

  const long seg0 = long(g) * SEG;
  uint64_t key[E];
  uint64_t tmin = ~0ull;
#pragma unroll
  for (int e = 0; e < E; ++e) {
    const long j = seg0 + e * kSelThreads + tid;
    uint64_t kv = ~0ull;
    if (j < len) {
      if (DENSE)
        kv = pack_key(static_cast<const float*>(in)[long(q) * in_ld + j], uint32_t(id_base + j));
      else
        kv = static_cast<const uint64_t*>(in)[long(q) * in_ld + j];
    }
    key[e] = kv;
    tmin = kv < tmin ? kv : tmin;
  }
  mins[tid] = tmin;
  if (tid == 0) count = 0;
  __syncthreads();
  block_bitonic_sort(mins, kSelThreads, tid, kSelThreads);
  const uint64_t bound = mins[kp - 1];  // kp <= 256
#pragma unroll
  for (int e = 0; e < E; ++e) {
    const long j = seg0 + e * kSelThreads + tid;
    if (j < len && key[e] <= bound) {
      const int pos = atomicAdd(&count, 1);
      list[pos] = key[e];
    }
  }
  __syncthreads();
  const int cnt = count;
  const int P = next_pow2(cnt > kp ? cnt : kp);  // <= SEG because kp <= 256 <= SEG
  for (int i = cnt + tid; i < P; i += kSelThreads) list[i] = kPadKey;
  __syncthreads();
  block_bitonic_sort(list, P, tid, kSelThreads);
  uint64_t* o = out + (long(q) * n_seg + g) * kp;
  for (int i = tid; i < kp; i += kSelThreads) o[i] = list[i];
}

// Final ranking in float64.  One block of 16 waves per query: for each of the kp
// float32 candidates recompute the Euclidean distance to the query in direct-difference
// form in float64 (one wave per candidate row, rows fetched concurrently), rank the candidates by
// (distance, id) and write the first k ids and distances to row `qrow` of the
// result arrays.  Padding candidates (id -1) get distance +inf and id -1.
constexpr int kRerankThreads = 1024;
template <int DT>
__global__ __launch_bounds__(kRerankThreads) void rerank_f64_kernel(const uint64_t* __restrict__ cand, int kp, int k,
                                                         const void* __restrict__ X, int dim,
                                                         const float* __restrict__ Qbase,
                                                         const int* __restrict__ qlist,
                                                         const int* __restrict__ m_count_ptr, int m_limit,
                                                         int64_t* __restrict__ res_ids,
                                                         float* __restrict__ res_dists) {
  const int m = blockIdx.x;
  const int m_total = m_count_ptr ? min(*m_count_ptr, m_limit) : m_limit;
  if (m >= m_total) return;
  const int qrow = qlist ? qlist[m] : m;
  const float* q = Qbase + long(qrow) * dim;
  const int lane = threadIdx.x & 63, wib = threadIdx.x >> 6;

  __shared__ double d64[256];
  __shared__ int ids[256];

  for (int c = wib; c < kp; c += kRerankThreads / 64) {
    const int id = key_id(cand[long(m) * kp + c]);
    double acc = 0.0;
    if (id >= 0) {
      if (DT == kDtypeF32) {
        const float* x = static_cast<const float*>(X) + long(id) * dim;
        for (int i = lane; i < dim; i += 64) {
          const double diff = double(q[i]) - double(x[i]);
          acc += diff * diff;
        }
      } else {
        const uint16_t* x = static_cast<const uint16_t*>(X) + long(id) * dim;
        for (int i = lane; i < dim; i += 64) {
          const double diff = double(q[i]) - double(bf16_to_float(x[i]));
          acc += diff * diff;
        }
      }
      acc = wave_sum(acc);
    }
    if (lane == 0) {
      d64[c] = id >= 0 ? sqrt(acc) : __longlong_as_double(0x7ff0000000000000ll);
      ids[c] = id >= 0 ? id : 0x7fffffff;
    }
  }
  __syncthreads();
  for (int c = threadIdx.x; c < kp; c += kRerankThreads) {
    const double d = d64[c];
    const int id = ids[c];
    int rank = 0;
    for (int o = 0; o < kp; ++o) {
      const double od = d64[o];
      const int oid = ids[o];
      rank += (od < d || (od == d && oid < id) || (od == d && oid == id && o < c)) ? 1 : 0;
    }
    if (rank < k) {
      res_ids[long(qrow) * k + rank] = id == 0x7fffffff ? -1ll : int64_t(id);
      res_dists[long(qrow) * k + rank] = float(d);
    }
  }
}

// Fills result rows of the listed queries with "no document" (used when the
// instance has no corpus): ids -1, distances +inf.
__global__ void fill_empty_results_kernel(const int* __restrict__ qlist, const int* __restrict__ m_count_ptr,
                                          int m_limit, int k, int64_t* __restrict__ res_ids,
                                          float* __restrict__ res_dists) {
  const int m = blockIdx.x;
  const int m_total = m_count_ptr ? min(*m_count_ptr, m_limit) : m_limit;
  if (m >= m_total) return;
  const int qrow = qlist ? qlist[m] : m;
  for (int i = threadIdx.x; i < k; i += blockDim.x) {
    res_ids[long(qrow) * k + i] = -1;
    res_dists[long(qrow) * k + i] = __uint_as_float(0x7f800000u);
  }
}

}  // namespace prox
