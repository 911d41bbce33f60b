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

// ---------------------------------------------------------------------------
// Calls with a handful of queries: the whole ranking side in one launch.
//
// Every block does what select_kernel<true> does for its segment of the dense
// score row.  The block that finishes last for a query (ticket counter per
// query) then merges the per-segment lists, re-ranks the kp survivors in
// float64 like rerank_f64_kernel, and routes the result like finalize_kernel:
// the query's own row, the rows of the same call that hit it, and its cache slot
// if it still owns one.  With hit == nullptr there is no cache (plain k-NN call).
// ---------------------------------------------------------------------------
struct SmallRouting {
  const uint8_t* hit;        // per row of the call: 1 = hit (nullptr: no cache involved)
  const int* src;            // answering source of hit rows (>= c: row src-c of this call)
  const int* row_slot;       // slot a missing row took, -1 if none
  const long long* slot_seq; // inserting stream position per slot
  int64_t* val_ids;          // cache values
  float* val_d;
  long long base_seq;
  int n, c;
};

// kp smallest of `len` keys in global memory -> sorted list[0..kp) in LDS, by one block of 256.
__device__ __forceinline__ void block_topk_of_keys(const uint64_t* __restrict__ in, long len, int kp, uint64_t* list,
                                                   int list_cap, uint64_t* mins, int* count, int tid) {
  uint64_t tmin = ~0ull;
  for (long j = tid; j < len; j += kSelThreads) {
    const uint64_t kv = in[j];
    tmin = kv < tmin ? kv : tmin;
  }
  mins[tid] = tmin;
  if (tid == 0) *count = 0;
  __syncthreads();
  block_bitonic_sort(mins, kSelThreads, tid, kSelThreads);
  const uint64_t bound = mins[kp - 1];
  for (long j = tid; j < len; j += kSelThreads) {
    const uint64_t kv = in[j];
    if (kv <= bound) {
      const int pos = atomicAdd(count, 1);
      if (pos < list_cap) list[pos] = kv;
    }
  }
  __syncthreads();
  const int cnt = *count;
  if (cnt <= list_cap) {
    const int P = next_pow2(cnt > kp ? cnt : kp);
    for (int i = cnt + tid; i < P; i += kSelThreads) list[i] = kPadKey;
    __syncthreads();
    block_bitonic_sort(list, P, tid, kSelThreads);
    return;
  }
  // exact ties made the survivor set larger than the list: keep a running best-kp list and
  // fold the input in, half a list at a time
  const int chunk = list_cap / 2;
  for (int i = tid; i < kp; i += kSelThreads) list[i] = kPadKey;
  __syncthreads();
  for (long c0 = 0; c0 < len; c0 += chunk) {
    for (int i = tid; i < chunk; i += kSelThreads) list[kp + i] = c0 + i < len ? in[c0 + i] : kPadKey;
    const int P = next_pow2(kp + chunk);
    for (int i = kp + chunk + tid; i < P; i += kSelThreads) list[i] = kPadKey;
    __syncthreads();
    block_bitonic_sort(list, P, tid, kSelThreads);
  }
}

template <int DT, int E>
__global__ __launch_bounds__(kSelThreads) void select_finish_small_kernel(
    const float* __restrict__ S, long ldS, long len, int kp, int k, uint64_t* __restrict__ lists, int n_seg,
    unsigned* tickets, const void* __restrict__ X, int dim, const float* __restrict__ Qbase,
    const int* __restrict__ qlist, const int* __restrict__ m_count_ptr, int m_limit, int m_begin, SmallRouting rt,
    int64_t* __restrict__ out_ids, float* __restrict__ out_d) {
  constexpr int SEG = E * kSelThreads;
  const int q = m_begin + blockIdx.y;   // position in the miss list; S rows are relative to m_begin
  const int m_total = m_count_ptr ? min(*m_count_ptr, m_limit) : m_limit;
  if (q >= m_total) return;
  const int g = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wib = tid >> 6;

  __shared__ uint64_t list[SEG];
  __shared__ uint64_t mins[kSelThreads];
  __shared__ int count;
  __shared__ bool is_last;
  __shared__ double d64[256];
  __shared__ int cid[256];
  __shared__ int64_t fin_ids[256];
  __shared__ float fin_d[256];

  // ---- this block's segment of the dense scores -> kp sorted keys (as select_kernel<true>) ----
  const long seg0 = long(g) * SEG;
  uint64_t key[E];
  uint64_t tmin = ~0ull;
#pragma unroll
  for (int e = 0; e < E; ++e) {
    const long j = seg0 + e * kSelThreads + tid;
    uint64_t kv = ~0ull;
    if (j < len) kv = pack_key(S[long(blockIdx.y) * ldS + j], uint32_t(j));
    key[e] = kv;
    tmin = kv < tmin ? kv : tmin;
  }
  mins[tid] = tmin;
  if (tid == 0) count = 0;
  __syncthreads();
  block_bitonic_sort(mins, kSelThreads, tid, kSelThreads);
  const uint64_t bound = mins[kp - 1];
#pragma unroll
  for (int e = 0; e < E; ++e) {
    const long j = seg0 + e * kSelThreads + tid;
    if (j < len && key[e] <= bound) list[atomicAdd(&count, 1)] = key[e];
  }
  __syncthreads();
  {
    const int cnt = count;
    const int P = next_pow2(cnt > kp ? cnt : kp);
    for (int i = cnt + tid; i < P; i += kSelThreads) list[i] = kPadKey;
    __syncthreads();
    block_bitonic_sort(list, P, tid, kSelThreads);
    uint64_t* o = lists + (long(q) * n_seg + g) * kp;
    for (int i = tid; i < kp; i += kSelThreads) o[i] = list[i];
  }
  __threadfence();
  __syncthreads();
  if (tid == 0) {
    const unsigned t = atomicAdd(&tickets[q], 1u);
    is_last = t == unsigned(n_seg) - 1;
    if (is_last) tickets[q] = 0;
  }
  __syncthreads();
  if (!is_last) return;
  __threadfence();

  // ---- merge all segments' lists ----
  block_topk_of_keys(lists + long(q) * n_seg * kp, long(n_seg) * kp, kp, list, SEG, mins, &count, tid);

  // ---- float64 ranking of the kp survivors (as rerank_f64_kernel) ----
  const int qrow = qlist ? qlist[q] : q;
  const float* qv = Qbase + long(qrow) * dim;
  for (int c = wib; c < kp; c += kSelThreads / 64) {
    const int id = key_id(list[c]);
    double acc = 0.0;
    if (id >= 0) {
      if (DT == kDtypeF32) {
        const float* x = static_cast<const float*>(X) + long(id) * dim;
        for (int i = lane; i < dim; i += 64) {
          const double diff = double(qv[i]) - double(x[i]);
          acc += diff * diff;
        }
      } else {
        const uint16_t* x = static_cast<const uint16_t*>(X) + long(id) * dim;
        for (int i = lane; i < dim; i += 64) {
          const double diff = double(qv[i]) - double(bf16_to_float(x[i]));
          acc += diff * diff;
        }
      }
      acc = wave_sum(acc);
    }
    if (lane == 0) {
      d64[c] = id >= 0 ? sqrt(acc) : __longlong_as_double(0x7ff0000000000000ll);
      cid[c] = id >= 0 ? id : 0x7fffffff;
    }
  }
  __syncthreads();
  for (int c = tid; c < kp; c += kSelThreads) {
    const double d = d64[c];
    const int id = cid[c];
    int rank = 0;
    for (int o = 0; o < kp; ++o) {
      const double od = d64[o];
      const int oid = cid[o];
      rank += (od < d || (od == d && oid < id) || (od == d && oid == id && o < c)) ? 1 : 0;
    }
    if (rank < k) {
      fin_ids[rank] = id == 0x7fffffff ? -1ll : int64_t(id);
      fin_d[rank] = float(d);
    }
  }
  __syncthreads();

  // ---- routing (as finalize_kernel) ----
  for (int e = tid; e < k; e += kSelThreads) {
    out_ids[long(qrow) * k + e] = fin_ids[e];
    if (out_d) out_d[long(qrow) * k + e] = fin_d[e];
  }
  if (rt.hit) {
    const int t = rt.row_slot[qrow];
    if (t >= 0 && rt.slot_seq[t] == rt.base_seq + qrow)
      for (int e = tid; e < k; e += kSelThreads) {
        rt.val_ids[long(t) * k + e] = fin_ids[e];
        rt.val_d[long(t) * k + e] = fin_d[e];
      }
    for (int i = qrow + 1; i < rt.n; ++i)
      if (rt.hit[i] && rt.src[i] == rt.c + qrow)
        for (int e = tid; e < k; e += kSelThreads) {
          out_ids[long(i) * k + e] = fin_ids[e];
          if (out_d) out_d[long(i) * k + e] = fin_d[e];
        }
  }
}

}  // namespace prox
