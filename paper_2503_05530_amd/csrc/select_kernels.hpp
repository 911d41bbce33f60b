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

#include <type_traits>

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
// minimum; a value with at least kp of the 256 thread minima at or below it
// bounds the kp-th smallest element from above (kp distinct elements lie at or
// below it), so only elements at or below that bound are compacted into LDS and
// sorted.  The expected number of survivors is a few times kp; exact ties can
// make it as large as the segment, which the LDS list is sized for.
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
  if (tid == 0) count = 0;
  const uint64_t bound = block_bound_for_kp<kSelThreads / 64>(tmin, kp, mins, tid);  // kp <= 256
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
  for (int i = cnt + tid; i < (P < 64 ? 64 : P); i += kSelThreads) list[i] = kPadKey;
  __syncthreads();
  if (P <= 64)
    block_sort_upto64(list, tid);
  else
    block_bitonic_sort(list, P, tid, kSelThreads);
  uint64_t* o = out + (long(q) * n_seg + g) * kp;
  for (int i = tid; i < kp; i += kSelThreads) o[i] = list[i];
}


// The distance functions of Section 2.2, as numbered at the C boundary.
constexpr int kMetricL2 = 0, kMetricIP = 1, kMetricCosine = 2;
// How kernels that only pass the corpus through are told what it is: element type in the low
// four bits, distance function above them.
__host__ __device__ constexpr int corpus_kind(int dtype, int metric) { return dtype | (metric << 4); }
__host__ __device__ constexpr int kind_dtype(int kind) { return kind & 15; }
__host__ __device__ constexpr int kind_metric(int kind) { return kind >> 4; }

// Float64 distance from query q to each of the kp candidate rows named by `keys`, by the NW waves
// of a block; four candidates per wave are in flight at once so that their row fetches overlap.
// Euclidean: direct-difference form, sqrt(sum (q_i - x_i)^2); inner product: -(q.x); cosine:
// 1 - q.x / sqrt((q.q)(x.x)), all sums in float64.  d64[c] / cid[c] receive distance and id of candidate
// c (padding candidates: +inf and INT_MAX).  The caller synchronises afterwards.
template <int DT, int NW>
__device__ __forceinline__ void block_candidate_distances(const uint64_t* keys, int kp, const float* __restrict__ q,
                                                          const void* __restrict__ X, int dim, double* d64, int* cid,
                                                          int tid, int metric = kMetricL2) {
  using Elem = typename std::conditional<DT == kDtypeF32, float, uint16_t>::type;
  const int lane = tid & 63, wib = tid >> 6;
  // Candidates in flight per wave: enough that the usual k + 8 candidates of a query take one round
  // (four waves: 8 each; sixteen waves: 4 each).
  constexpr int G = NW >= 16 ? 4 : 8;
  constexpr int V = DT == kDtypeF32 ? 4 : 8;  // elements per 16-byte load
  const int n_vec = dim / V;                  // dim is a multiple of 32
  // element e of a 16-byte piece of a row / of the matching piece(s) of the query, as float64
  auto row_elem = [](const uint4& t, int e) -> double {
    const uint32_t w[4] = {t.x, t.y, t.z, t.w};
    if (DT == kDtypeF32) return double(__uint_as_float(w[e & 3]));
    const uint32_t pair = w[(e >> 1) & 3];
    return double(__uint_as_float((e & 1) ? (pair & 0xffff0000u) : (pair << 16)));
  };
  auto query_elem = [](const float4 (&t)[V / 4], int e) -> double {
    const float4& f = t[e >> 2];
    return double((e & 3) == 0 ? f.x : (e & 3) == 1 ? f.y : (e & 3) == 2 ? f.z : f.w);
  };
  for (int c0 = wib; c0 < kp; c0 += NW * G) {
    int id[G];
    const uint4* row[G];
    double acc[G], xx[G], qq = 0.0;
#pragma unroll
    for (int g = 0; g < G; ++g) {
      const int c = c0 + g * NW;
      id[g] = c < kp ? key_id(keys[c]) : -1;
      row[g] = reinterpret_cast<const uint4*>(static_cast<const Elem*>(X) + long(id[g] >= 0 ? id[g] : 0) * dim);
      acc[g] = 0.0;
      xx[g] = 0.0;
    }
    // Rows are fetched 16 bytes per lane, two steps of all G rows issued before anything is used, so
    // that a row of 768 floats costs two memory round trips.
    for (int iv0 = lane; iv0 < n_vec; iv0 += 128) {
      uint4 raw[2][G];
      float4 qraw[2][V / 4];
      const bool two = iv0 + 64 < n_vec;
#pragma unroll
      for (int st = 0; st < 2; ++st) {
        if (st == 1 && !two) break;
        const int iv = iv0 + 64 * st;
#pragma unroll
        for (int h = 0; h < V / 4; ++h) qraw[st][h] = reinterpret_cast<const float4*>(q)[iv * (V / 4) + h];
#pragma unroll
        for (int g = 0; g < G; ++g) raw[st][g] = row[g][iv];
      }
#pragma unroll
      for (int st = 0; st < 2; ++st) {
        if (st == 1 && !two) break;
#pragma unroll
        for (int e = 0; e < V; ++e) {
          const double qv = query_elem(qraw[st], e);
          if (metric != kMetricL2) qq += qv * qv;
#pragma unroll
          for (int g = 0; g < G; ++g) {
            const double xv = row_elem(raw[st][g], e);
            if (metric == kMetricL2) {
              const double diff = qv - xv;
              acc[g] += diff * diff;
            } else {
              // inner product, and for cosine the two squared lengths as well
              acc[g] += qv * xv;
              xx[g] += xv * xv;
            }
          }
        }
      }
    }
    if (metric != kMetricL2) qq = wave_sum(qq);
#pragma unroll
    for (int g = 0; g < G; ++g) {
      const int c = c0 + g * NW;
      if (c0 + g * NW >= kp && g > 0) break;  // wave-uniform: nothing left in this round
      const double total = wave_sum(acc[g]);
      double d;
      if (metric == kMetricL2) {
        d = sqrt(total);
      } else if (metric == kMetricIP) {
        d = -total;
      } else {
        d = 1.0 - total / sqrt(wave_sum(xx[g]) * qq);  // (one root over the product: exactly 0 for a row equal to q)
      }
      if (lane == 0 && c < kp) {
        d64[c] = id[g] >= 0 ? d : __longlong_as_double(0x7ff0000000000000ll);
        cid[c] = id[g] >= 0 ? id[g] : 0x7fffffff;
      }
    }
  }
}

// Ranks n (distance, id) pairs held in LDS by (distance, id) and writes the first k ids and
// distances (id INT_MAX stands for "no document": id -1, distance +inf).  out_d may be null.
// kth (LDS, may be null) receives the distance of rank k-1 when n >= k.
__device__ __forceinline__ void block_write_ranked(const double* d64, const int* ids, int n, int k,
                                                   int64_t* __restrict__ out_ids, float* __restrict__ out_d, int tid,
                                                   int nthreads, double* kth = nullptr) {
  for (int c = tid; c < n; c += nthreads) {
    const double d = d64[c];
    const int id = ids[c];
    int rank = 0;
    for (int o = 0; o < n; ++o) {
      const double od = d64[o];
      const int oid = ids[o];
      rank += (od < d || (od == d && oid < id) || (od == d && oid == id && o < c)) ? 1 : 0;
    }
    if (rank < k) {
      out_ids[rank] = id == 0x7fffffff ? -1ll : int64_t(id);
      if (out_d) out_d[rank] = float(d);
    }
    if (kth && rank == k - 1) *kth = d;
  }
  for (int r = n + tid; r < k; r += nthreads) {  // fewer entries than k: pad
    out_ids[r] = -1ll;
    if (out_d) out_d[r] = __uint_as_float(0x7f800000u);
  }
}

// The hit side of the re-ranking factor (Section 3.3.4): of the K documents stored with the
// matched key, the k nearest to the current query q, by float64 direct-difference distance,
// equal distances by index.  Stored ids below 0 are padding.  One block of NT threads;
// keys / d64 / cid are LDS arrays of at least K entries.  Ends with the writes issued, no barrier.
template <int DT, int NT>
__device__ __forceinline__ void block_rerank_stored(const int64_t* __restrict__ stored, int K, int k,
                                                    const float* __restrict__ q, const void* __restrict__ X, int dim,
                                                    int64_t* __restrict__ out_ids, float* __restrict__ out_d,
                                                    uint64_t* keys, double* d64, int* cid, int tid,
                                                    int metric = kMetricL2) {
  for (int e = tid; e < K; e += NT) {
    const int64_t id = stored[e];
    keys[e] = id >= 0 ? pack_key(0.f, uint32_t(id)) : kPadKey;
  }
  __syncthreads();
  block_candidate_distances<DT, NT / 64>(keys, K, q, X, dim, d64, cid, tid, metric);
  __syncthreads();
  block_write_ranked(d64, cid, K, k, out_ids, out_d, tid, NT);
}
// the same with the corpus type and the distance function chosen at run time (see corpus_kind)
template <int NT>
__device__ __forceinline__ void block_rerank_stored_any(int kind, const int64_t* __restrict__ stored, int K,
                                                        int k, const float* __restrict__ q,
                                                        const void* __restrict__ X, int dim,
                                                        int64_t* __restrict__ out_ids, float* __restrict__ out_d,
                                                        uint64_t* keys, double* d64, int* cid, int tid) {
  if (kind_dtype(kind) == kDtypeBF16)
    block_rerank_stored<kDtypeBF16, NT>(stored, K, k, q, X, dim, out_ids, out_d, keys, d64, cid, tid, kind_metric(kind));
  else
    block_rerank_stored<kDtypeF32, NT>(stored, K, k, q, X, dim, out_ids, out_d, keys, d64, cid, tid, kind_metric(kind));
}

// ---------------------------------------------------------------------------
// Is the float32 candidate list long enough?
//
// The scan ranks rows by float32 scores and hands the kp = k + slack best to the float64 ranking.  The
// answer is the exact ranked list of Section 2.2 only if no row outside the list belongs to the true k
// nearest.  A float32 score differs from the exact score of its row by at most E (below), every row
// outside the list has a float32 score of at least W, the list's worst, and the k-th smallest exact score
// inside the list, t_k, bounds the true k-th smallest from above.  So  W - E > t_k  proves the list
// sufficient.  Where the proof fails (many rows within rounding error of the k-th, e.g. duplicated
// documents) the query is ranked again from every row whose float32 score is at most t_k + E -- a set that
// provably holds the true k nearest -- and counted in `exhausted`; if that set outgrows its buffer
// (kWideCap rows) the query keeps the float64 ranking of its kp candidates and is counted in `unresolved`.
//
// E: a float32 inner product of dim terms, summed in any order, is within (terms + 2) 2^-24 |q| |x| of the
// exact one (each product and each partial sum rounds once); a bfloat16 corpus is scanned with the query split
// into bfloat16 planes: up to 3 dim exact products, and where only two planes are multiplied a remainder below
// 2^-18 |q_i| per element, 2^-17 |q| |x| in a score.  g = (3 dim + 16) 2^-24 + 2^-17 covers every scan kernel.
// The squared length of a row carries the same relative error; the final multiply-add rounds once more.
// With X the largest row length:
//   Euclidean      score = |x|^2 - 2 q.x          E = g (X^2 + 2 |q| X)
//   inner product  score = -2 q.x                 E = g 2 |q| X
//   cosine         score = -2 q.x / |x|           E = g 4 |q|     (the reciprocal length rounds as well)
// ---------------------------------------------------------------------------
constexpr int kWideCap = 2048;   // rows the second ranking of a query can hold

struct SlackState {
  unsigned xmax2_bits;      // largest squared row length of the corpus, as float bits (non-negative floats order as unsigned)
  int redo_count;           // queries of the current call whose list could not be proven sufficient
  int redo_ticket;          // blocks of the second ranking that have finished
  int coarse_fails;         // lists of a one-plane scan (regq_kernels.hpp) that could not be proven sufficient, ever
  unsigned long long exhausted, unresolved;
};
// The queries noted for the second ranking of the batched scan, one entry per row a call can carry.
struct RedoBuffers {
  int* list;        // [max_batch] their positions in the call's miss list
  float* thr;       // [max_batch] t_k + E of each, rounded up
  int* cnt;         // [max_batch] rows collected for each; zero between calls
  uint64_t* wide;   // [max_batch][kWideCap] the collected rows as packed (score, row) keys
  int* coarse_note; // HOST memory the device can write (or null): receives coarse_fails whenever it grows, for the
                    // host to read, without waiting for anything, when it picks the next call's scan
};

__host__ __device__ inline double score_error_bound(int metric, int dim, double q_len, double x_max) {
  const double g = (3.0 * double(dim) + 16.0) * 5.9604644775390625e-08 + 7.62939453125e-06;
  if (metric == kMetricL2) return g * (x_max * x_max + 2.0 * q_len * x_max);
  if (metric == kMetricIP) return g * 2.0 * q_len * x_max;
  return g * 4.0 * q_len;
}
// What a scan that multiplies only the first bfloat16 plane of the queries adds to that (level 1): the plane is
// the query rounded to nearest, |q_i - hi_i| <= 2^-9 |q_i|, so the inner product moves by at most 2^-9 |q| |x| and
// the score by twice that (a thousandth on top for the roundings that follow).  Level 2: float32 rows rounded to
// bfloat16 as well, |q.x - hi(q).hi(x)| <= |q - hi(q)| |x| + |hi(q)| |x - hi(x)| <= (2 + 2^-9) 2^-9 |q| |x|.
__host__ __device__ inline double coarse_score_error(int metric, double q_len, double x_max, int level = 1) {
  const double u = 0.00390625 * 1.001 * (level >= 2 ? 2.002 : 1.0);
  return metric == kMetricCosine ? u * q_len : u * q_len * x_max;
}
// the exact score that goes with a float64 distance (qq = |q|^2)
__device__ __forceinline__ double score_of_distance(int metric, double d, double qq) {
  if (metric == kMetricL2) return d * d - qq;
  if (metric == kMetricIP) return 2.0 * d;
  return 2.0 * (d - 1.0) * sqrt(qq);
}

// Block-uniform verdict on a sorted list of kp float32 candidates whose k-th smallest float64 distance is
// kth_d: true when the list provably holds the k nearest rows.  *thr receives t_k + E (rounded up), the
// score bound of the second ranking (which scores with the whole query: its bound never carries the coarse
// term).  `coarse`: the list was ranked by scores of rounded operands (level of coarse_score_error, 0: no).
// `red` is 2 doubles of LDS.  Ends with a barrier.
__device__ __forceinline__ bool block_list_sufficient(const uint64_t* keys, int kp, double kth_d,
                                                      const float* __restrict__ q, int dim, int metric,
                                                      const SlackState* __restrict__ slack, double* red, float* thr,
                                                      int tid, int coarse = 0,
                                                      float seed_bound = __builtin_inff()) {
  // (seed_bound: the score bound the scan started from, +inf if it started from none; a row the scan turned away
  // scores above it.  A value, not a pointer: a load through a pointer that may be null, placed under a
  // condition that differs from lane to lane, is issued as a scalar load whatever the lanes decide -- scalar
  // instructions ignore the execution mask -- and faults.)
  if (tid < 64) {
    double qq = 0.0;
    for (int x = tid; x < dim; x += 64) qq += double(q[x]) * double(q[x]);
    qq = wave_sum(qq);
    if (tid == 0) {
      const uint64_t worst = keys[kp - 1];
      bool ok = true;
      float t = __uint_as_float(0x7f800000u);
      // A list with a padding entry holds every row the scan did not turn away at its starting bound (bounds
      // tighten only where a buffer has filled, and merges cut only full lists): without a starting bound that is
      // every row of the corpus, with one the rows outside score above that bound, which then stands in for the
      // worst kept score.
      const bool full = key_id(worst) >= 0;
      const bool bounded = !full && seed_bound < __uint_as_float(0x7f800000u);
      if (full || bounded) {
        const double worst_kept = full ? double(key_score(worst)) : double(seed_bound);
        const double x_max = sqrt(double(__uint_as_float(slack->xmax2_bits)));
        const double e = score_error_bound(metric, dim, sqrt(qq), x_max) * (1.0 + 1e-6);
        const double e_list = coarse ? e + coarse_score_error(metric, sqrt(qq), x_max, coarse) : e;
        const double t_k = score_of_distance(metric, kth_d, qq);
        ok = worst_kept - e_list > t_k;
        t = __double2float_ru(t_k + e);
      }
      red[0] = ok ? 1.0 : 0.0;
      *thr = t;
    }
  }
  __syncthreads();
  return red[0] != 0.0;
}

// The second ranking: exact k nearest among n candidate rows named by `keys` (LDS, any order, ids >= 0), by
// float64 distance and index, 256 candidates at a time against a running best list.  Work arrays in LDS:
// d64 / cid [256] for a chunk, best_d / best_id [2][256].  Result: ids (or -1) and distances of rank 0..k-1
// through `emit(rank, id, distance)`.  All threads of the block call it; ends with a barrier.
template <int DT, int NT, typename Emit>
__device__ __forceinline__ void block_exact_topk_of_rows(const uint64_t* keys, int n, int k,
                                                         const float* __restrict__ q, const void* __restrict__ X,
                                                         int dim, int metric, double* d64, int* cid,
                                                         double (*best_d)[256], int (*best_id)[256], int tid,
                                                         Emit emit) {
  const double kInf = __longlong_as_double(0x7ff0000000000000ll);
  int nb = 0, cur = 0;   // entries of the running list, and which of the two buffers holds it
  for (int c0 = 0; c0 < n; c0 += 256) {
    const int nc = n - c0 < 256 ? n - c0 : 256;
    block_candidate_distances<DT, NT / 64>(keys + c0, nc, q, X, dim, d64, cid, tid, metric);
    __syncthreads();
    // rank the union of the running list and the chunk; the best k go to the other buffer in rank order
    const int total = nb + nc;
    for (int e = tid; e < total; e += NT) {
      const double d = e < nb ? best_d[cur][e] : d64[e - nb];
      const int id = e < nb ? best_id[cur][e] : cid[e - nb];
      int rank = 0;
      for (int o = 0; o < total; ++o) {
        const double od = o < nb ? best_d[cur][o] : d64[o - nb];
        const int oid = o < nb ? best_id[cur][o] : cid[o - nb];
        rank += (od < d || (od == d && oid < id) || (od == d && oid == id && o < e)) ? 1 : 0;
      }
      if (rank < k) {
        best_d[cur ^ 1][rank] = d;
        best_id[cur ^ 1][rank] = id;
      }
    }
    __syncthreads();
    nb = total < k ? total : k;
    cur ^= 1;
  }
  for (int r = tid; r < k; r += NT) {
    if (r < nb && best_id[cur][r] != 0x7fffffff)
      emit(r, int64_t(best_id[cur][r]), best_d[cur][r]);
    else
      emit(r, -1ll, kInf);
  }
  __syncthreads();
}

// Fills result rows of the listed queries with "no document" (used when the
// instance has no corpus): ids -1, distances +inf (res_dists may be null).
__global__ void fill_empty_results_kernel(const int* __restrict__ qlist, const int* __restrict__ m_count_ptr,
                                          int m_limit, int k, int64_t* __restrict__ res_ids,
                                          float* __restrict__ res_dists) {
  const int m = blockIdx.x;
  const int m_total = m_count_ptr ? min(*m_count_ptr, m_limit) : m_limit;
  if (m >= m_total) return;
  const int qrow = qlist ? qlist[m] : m;
  for (int i = threadIdx.x; i < k; i += blockDim.x) {
    res_ids[long(qrow) * k + i] = -1;
    if (res_dists) res_dists[long(qrow) * k + i] = __uint_as_float(0x7f800000u);
  }
}

// ---------------------------------------------------------------------------
// Calls with a handful of queries: the whole ranking side in two launches of this kernel.
//
// phase == 1, grid (segments, queries): every block does what select_kernel<true> does
// for its segment of the dense score row.  phase == 2, grid (1, queries): one block per
// query merges the per-segment lists, re-ranks the kp survivors in
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

// kp smallest of `len` keys in global memory -> sorted list[0..kp) in LDS, by one block of NT threads
// (mins: NT / 64 entries at least; list: list_cap >= 64 entries).
template <int NT>
__device__ __forceinline__ void block_topk_of_keys(const uint64_t* __restrict__ in, long len, int kp, uint64_t* list,
                                                   int list_cap, uint64_t* mins, int* count, int tid) {
  // both passes read eight keys per thread at a time, all loads issued before the first is used
  constexpr int U = 8;
  uint64_t tmin = ~0ull;
  for (long j0 = tid; j0 < len; j0 += long(U) * NT) {
    uint64_t kv[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const long j = j0 + long(u) * NT;
      kv[u] = j < len ? in[j] : ~0ull;
    }
#pragma unroll
    for (int u = 0; u < U; ++u) tmin = kv[u] < tmin ? kv[u] : tmin;
  }
  if (tid == 0) *count = 0;
  const uint64_t bound = block_bound_for_kp<NT / 64>(tmin, kp, mins, tid);
  for (long j0 = tid; j0 < len; j0 += long(U) * NT) {
    uint64_t kv[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const long j = j0 + long(u) * NT;
      kv[u] = j < len ? in[j] : ~0ull;
    }
#pragma unroll
    for (int u = 0; u < U; ++u)
      if (kv[u] <= bound && j0 + long(u) * NT < len) {
        const int pos = atomicAdd(count, 1);
        if (pos < list_cap) list[pos] = kv[u];
      }
  }
  __syncthreads();
  const int cnt = *count;
  if (cnt <= list_cap) {
    const int P = next_pow2(cnt > kp ? cnt : kp);
    for (int i = cnt + tid; i < (P < 64 ? 64 : P); i += NT) list[i] = kPadKey;
    __syncthreads();
    if (P <= 64)
      block_sort_upto64(list, tid);
    else
      block_bitonic_sort(list, P, tid, NT);
    return;
  }
  // exact ties made the survivor set larger than the list: keep a running best-kp list and
  // fold the input in, half a list at a time
  const int chunk = list_cap / 2;
  for (int i = tid; i < kp; i += NT) list[i] = kPadKey;
  __syncthreads();
  for (long c0 = 0; c0 < len; c0 += chunk) {
    for (int i = tid; i < chunk; i += NT) list[kp + i] = c0 + i < len ? in[c0 + i] : kPadKey;
    const int P = next_pow2(kp + chunk);
    for (int i = kp + chunk + tid; i < P; i += NT) list[i] = kPadKey;
    __syncthreads();
    block_bitonic_sort(list, P, tid, NT);
  }
}

// Final ranking in float64.  One block of 16 waves per query.  The query's float32 candidates arrive
// as n_lists sorted lists of kp keys each (what the last merge level would have read); the block
// first cuts them to the kp best (n_lists = 1: nothing to do), then recomputes for each of those the
// distance to the query in float64 (direct-difference form for the Euclidean distance; one wave per
// candidate row, rows fetched concurrently), ranks them by
// (distance, id) and writes the first k ids and distances to row `qrow` of the
// result arrays.  Padding candidates (id -1) get distance +inf and id -1.  Last it checks that the
// list was long enough for the result to be exact (block_list_sufficient).
constexpr int kRerankThreads = 1024;
constexpr int kRerankMergeKeys = 2048;  // LDS list of a cut: the keys at or below the block's bound (more: exact ties, folded in)
template <int DT>
__global__ __launch_bounds__(kRerankThreads) void rerank_f64_kernel(const uint64_t* __restrict__ cand, int n_lists,
                                                         int kp, int k,
                                                         const void* __restrict__ X, int dim,
                                                         const float* __restrict__ Qbase,
                                                         const int* __restrict__ qlist,
                                                         const int* __restrict__ m_count_ptr, int m_limit,
                                                         int64_t* __restrict__ res_ids,
                                                         float* __restrict__ res_dists, int metric,
                                                         SlackState* __restrict__ slack, RedoBuffers redo,
                                                         int coarse, const float* __restrict__ seed_bound,
                                                         int seeded) {
  // (seed_bound: an array of a float per query, always readable; it holds the scans' starting bounds if `seeded`)
  const int m = blockIdx.x;
  const int m_total = m_count_ptr ? min(*m_count_ptr, m_limit) : m_limit;
  if (m >= m_total) return;
  const float started_from = seeded ? seed_bound[m] : __builtin_inff();
  const int qrow = qlist ? qlist[m] : m;
  const float* q = Qbase + long(qrow) * dim;

  __shared__ double d64[256];
  __shared__ int ids[256];
  __shared__ uint64_t list[kRerankMergeKeys];
  __shared__ uint64_t mins[kRerankThreads / 64];
  __shared__ int count;
  __shared__ double kth_d, red[2];
  __shared__ float thr;

  const uint64_t* mine = cand + long(m) * n_lists * kp;
  if (n_lists > 1) {
    block_topk_of_keys<kRerankThreads>(mine, long(n_lists) * kp, kp, list, kRerankMergeKeys, mins, &count, threadIdx.x);
    __syncthreads();
    mine = list;
  }
  block_candidate_distances<DT, kRerankThreads / 64>(mine, kp, q, X, dim, d64, ids, threadIdx.x, metric);
  __syncthreads();
  block_write_ranked(d64, ids, kp, k, res_ids + long(qrow) * k, res_dists + long(qrow) * k, threadIdx.x,
                     kRerankThreads, &kth_d);
  __syncthreads();
  // Was the list long enough?  If that cannot be shown the query is noted for the second ranking
  // (redo_collect_kernel / redo_rank_kernel), which overwrites this row of the result.
  if (!block_list_sufficient(mine, kp, kth_d, q, dim, metric, slack, red, &thr, threadIdx.x, coarse, started_from) &&
      threadIdx.x == 0) {
    atomicAdd(&slack->exhausted, 1ull);
    const int pos = atomicAdd(&slack->redo_count, 1);   // below the call's row count: one note per query
    redo.list[pos] = m;
    redo.thr[pos] = thr;
    if (coarse) {
      const int fails = atomicAdd(&slack->coarse_fails, 1) + 1;
      if (redo.coarse_note) {   // (concurrent notes may land out of order: the host only asks "how many, roughly")
        *reinterpret_cast<volatile int*>(redo.coarse_note) = fails;
        __threadfence_system();
      }
    }
  }
}

// Per-query lists of `len` keys (sorted runs or not) cut to the kp best, sorted: out[m * kp ..].  One block of
// sixteen waves per query; what the merge levels do for lists too long for one block, in one launch.
//
// With `margin` set the list is a sample's and seeds the bound of a scan by another kernel than the one that
// scored the sample (another order of summation, other planes of the query): a sample row's score in that scan
// can lie above its score here by both kernels' errors, and the bound taken as it stands could turn away, by a
// rounding, rows that belong in the list.  The kp-th key (the only one the scans read) then gets that margin
// added: twice the float32 bound, plus the rounding term of a scan on rounded operands (margin = 1 + level of
// coarse_score_error).
// The key published in the list's last place -- the one that seeds a scan's bound -- is the list's entry number
// bound_rank (counting from 1; kp: the last entry itself).  Any rank from k on keeps the ranking sound: that many
// rows of the corpus score at or below the bound, so the scan's list holds at least so many rows, and the
// exactness check knows the bound (bound_out) for the case that the list does not fill.  A scan that keeps a long
// list because its scores are coarse starts from rank k + 8 all the same: its candidates are a matter of time, not
// of correctness.  Where the list is shorter than bound_rank (a second sample that the first one's bound let few
// rows of through) the earlier bound is passed on instead.
constexpr long kCutMaxKeys = 65536;
__global__ __launch_bounds__(kRerankThreads) void cut_lists_kernel(const uint64_t* __restrict__ in, long len, int kp,
                                                                   uint64_t* __restrict__ out,
                                                                   const int* __restrict__ m_count_ptr, int m_limit,
                                                                   int margin, const float* __restrict__ Qbase,
                                                                   const int* __restrict__ qlist, int dim, int metric,
                                                                   const SlackState* __restrict__ slack, int bound_rank,
                                                                   float* bound_io, int first) {
  // (bound_io: a float per query, always readable -- see block_list_sufficient on loads through pointers that may
  // be null; unless `first`, it holds the bound of the sample before this one on entry; the bound published here
  // on exit)
  const int m = blockIdx.x, tid = threadIdx.x;
  const int m_total = m_count_ptr ? min(*m_count_ptr, m_limit) : m_limit;
  if (m >= m_total) return;
  const float earlier_bound = first ? __builtin_inff() : bound_io[m];
  __shared__ uint64_t list[kRerankMergeKeys];
  __shared__ uint64_t mins[kRerankThreads / 64];
  __shared__ int count;
  block_topk_of_keys<kRerankThreads>(in + long(m) * len, len, kp, list, kRerankMergeKeys, mins, &count, tid);
  __syncthreads();
  uint64_t* o = out + long(m) * kp;
  for (int i = tid; i < kp - 1; i += kRerankThreads) o[i] = list[i];
  if (tid < 64) {
    uint64_t key = list[bound_rank - 1];
    if (key_id(key) < 0) {
      key = pack_key(earlier_bound, 0u);   // (margin and all; +inf when there was none)
    } else if (margin && key_id(key) >= 0) {   // (a padding key is +inf already)
      const float* q = Qbase + long(qlist ? qlist[m] : m) * dim;
      double qq = 0.0;
      for (int x = tid; x < dim; x += 64) qq += double(q[x]) * double(q[x]);
      qq = wave_sum(qq);
      const double x_max = sqrt(double(__uint_as_float(slack->xmax2_bits)));
      double e = 2.0 * score_error_bound(metric, dim, sqrt(qq), x_max);
      if (margin >= 2) e += coarse_score_error(metric, sqrt(qq), x_max, margin - 1);
      key = pack_key(__double2float_ru(double(key_score(key)) + e * (1.0 + 1e-6)), uint32_t(key_id(key)));
    }
    if (tid == 0) {
      o[kp - 1] = key;
      bound_io[m] = key_score(key);
    }
  }
}

template <int DT, int E, int NT>
__global__ __launch_bounds__(NT) void select_finish_small_kernel(
    const float* __restrict__ S, long ldS, long len, int kp, int k, int k_out, uint64_t* __restrict__ lists,
    int n_seg, int phase, const void* __restrict__ X, int dim, const float* __restrict__ Qbase,
    const int* __restrict__ qlist, const int* __restrict__ m_count_ptr, int m_limit, int m_begin, SmallRouting rt,
    int64_t* __restrict__ out_ids, float* __restrict__ out_d, int metric, SlackState* __restrict__ slack) {
  constexpr int SEG = E * NT;
  const int q = m_begin + blockIdx.y;   // position in the miss list; S rows are relative to m_begin
  const int m_total = m_count_ptr ? min(*m_count_ptr, m_limit) : m_limit;
  if (q >= m_total) return;
  const int g = blockIdx.x, tid = threadIdx.x;

  __shared__ uint64_t list[SEG];
  __shared__ uint64_t mins[NT];
  __shared__ int count;
  __shared__ double d64[256];
  __shared__ int cid[256];
  __shared__ int64_t fin_ids[256];
  __shared__ float fin_d[256];
  __shared__ double best_d[2][256];
  __shared__ int best_id[2][256];
  __shared__ double kth_d, red[2];
  __shared__ float thr;

  if (phase != 2) {
  // ---- this block's segment of the dense scores -> kp sorted keys (as select_kernel<true>) ----
  const long seg0 = long(g) * SEG;
  uint64_t key[E];
  uint64_t tmin = ~0ull;
#pragma unroll
  for (int e = 0; e < E; ++e) {
    const long j = seg0 + e * NT + tid;
    uint64_t kv = ~0ull;
    if (j < len) kv = pack_key(S[long(blockIdx.y) * ldS + j], uint32_t(j));
    key[e] = kv;
    tmin = kv < tmin ? kv : tmin;
  }
  if (tid == 0) count = 0;
  const uint64_t bound = block_bound_for_kp<NT / 64>(tmin, kp, mins, tid);
#pragma unroll
  for (int e = 0; e < E; ++e) {
    const long j = seg0 + e * NT + tid;
    if (j < len && key[e] <= bound) list[atomicAdd(&count, 1)] = key[e];
  }
  __syncthreads();
  {
    const int cnt = count;
    const int P = next_pow2(cnt > kp ? cnt : kp);
    for (int i = cnt + tid; i < (P < 64 ? 64 : P); i += NT) list[i] = kPadKey;
    __syncthreads();
    if (P <= 64)
      block_sort_upto64(list, tid);
    else
      block_bitonic_sort(list, P, tid, NT);
    uint64_t* o = lists + (long(q) * n_seg + g) * kp;
    for (int i = tid; i < kp; i += NT) o[i] = list[i];
  }
  }
  if (phase == 1) return;

  // ---- merge all segments' lists ----
  block_topk_of_keys<NT>(lists + long(q) * n_seg * kp, long(n_seg) * kp, kp, list, SEG, mins, &count, tid);

  // ---- float64 ranking of the kp survivors (as rerank_f64_kernel) ----
  const int qrow = qlist ? qlist[q] : q;
  const float* qv = Qbase + long(qrow) * dim;
  block_candidate_distances<DT, NT / 64>(list, kp, qv, X, dim, d64, cid, tid, metric);
  __syncthreads();
  for (int c = tid; c < kp; c += NT) {
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
    if (rank == k - 1) kth_d = d;
  }
  __syncthreads();

  // ---- was the list long enough?  If that cannot be shown, rank again from every row whose float32 score
  // (still at hand: the dense score row) is at most t_k + E ----
  if (!block_list_sufficient(list, kp, kth_d, qv, dim, metric, slack, red, &thr, tid)) {
    if (tid == 0) {
      atomicAdd(&slack->exhausted, 1ull);
      count = 0;
    }
    __syncthreads();
    const float bound_sc = thr;
    for (long j = tid; j < len; j += NT) {
      const float sc = S[long(blockIdx.y) * ldS + j];
      if (sc <= bound_sc) {
        const int pos = atomicAdd(&count, 1);
        if (pos < kWideCap) list[pos] = pack_key(sc, uint32_t(j));
      }
    }
    __syncthreads();
    const int cnt = count;
    if (cnt > kWideCap) {
      if (tid == 0) atomicAdd(&slack->unresolved, 1ull);
    } else {
      block_exact_topk_of_rows<DT, NT>(list, cnt, k, qv, X, dim, metric, d64, cid, best_d, best_id, tid,
                                       [&](int r, int64_t id, double d) {
                                         fin_ids[r] = id;
                                         fin_d[r] = float(d);
                                       });
    }
    __syncthreads();
  }

  // ---- routing (as finalize_kernel): k ranked entries are this query's result; the caller gets
  // the first k_out, the cache slot all k (k > k_out with a re-ranking factor, Section 3.3.4) ----
  for (int e = tid; e < k_out; e += NT) {
    out_ids[long(qrow) * k_out + e] = fin_ids[e];
    if (out_d) out_d[long(qrow) * k_out + e] = fin_d[e];
  }
  if (rt.hit) {
    const int t = rt.row_slot[qrow];
    if (t >= 0 && rt.slot_seq[t] == rt.base_seq + qrow)
      for (int e = tid; e < k; e += NT) {
        rt.val_ids[long(t) * k + e] = fin_ids[e];
        rt.val_d[long(t) * k + e] = fin_d[e];
      }
    for (int i = qrow + 1; i < rt.n; ++i)
      if (rt.hit[i] && rt.src[i] == rt.c + qrow) {
        if (k == k_out) {
          for (int e = tid; e < k; e += NT) {
            out_ids[long(i) * k + e] = fin_ids[e];
            if (out_d) out_d[long(i) * k + e] = fin_d[e];
          }
        } else {
          // a later row of the call hit this one: the stored documents nearest to that row's query
          __syncthreads();
          block_rerank_stored<DT, NT>(fin_ids, k, k_out, Qbase + long(i) * dim, X, dim,
                                               out_ids + long(i) * k_out, out_d ? out_d + long(i) * k_out : nullptr,
                                               list, d64, cid, tid, metric);
        }
      }
  }
}

}  // namespace prox
