// Cache-side kernels: candidate extraction after the probe, the order-preserving
// hit/miss/evict resolver, key insertion and result routing.
//
// Terms.  The cache has `c` slots.  A *source* that may answer row i of a batch
// is either a slot that held a key when the batch started (source id = slot,
// 0..c-1) or an earlier row j < i of the same batch that missed and was stored
// (source id = c + j).  Every key carries the stream position ("seq") of the
// query that inserted it; rows of the current batch have seq = base_seq + row.
// A slot whose seq is >= base_seq was overwritten during this batch, by row
// seq - base_seq.  Slots fill in index order and are never freed individually,
// so the live slots are always 0..size-1.
#pragma once

#include "device_utils.hpp"
#include "select_kernels.hpp"

namespace prox {

struct CacheState {
  int size;   // live keys
  int head;   // next victim (front of the eviction order), -1 when empty
  int tail;   // most recently inserted (FIFO) / used (LRU), -1 when empty
  int pad;
  unsigned long long queries, hits, misses, inserts, evictions, inbatch_hits, dense_resolves, pad2;
};

// Distance between a query and a key in float64, computed by one wave: the one routine every float64
// decision in this file goes through.  cosine == 0: Euclidean, direct-difference form,
// sqrt(sum (a_i - b_i)^2).  cosine == 1: 1 - a.b / sqrt((a.a)(b.b)); the three sums run over the same
// elements in the same order, so a vector against a bit-identical copy of itself gives exactly 0
// (a.b, a.a and b.b are then the same number s, and sqrt(s*s) == s in binary floating point), which is
// what makes a tolerance of zero an exact-match cache under this distance too (Section 3.3.3).
__device__ __forceinline__ double wave_keydist64(const float* __restrict__ a, const float* __restrict__ b, int dim,
                                                 int lane, int cosine) {
  // 16 bytes per lane and two steps in flight (rows are 128-byte aligned: dim is a multiple of 32)
  const float4* a4 = reinterpret_cast<const float4*>(a);
  const float4* b4 = reinterpret_cast<const float4*>(b);
  const int n_vec = dim / 4;
  double acc = 0.0, aa = 0.0, bb = 0.0;
  for (int iv = lane; iv < n_vec; iv += 128) {
    const bool two = iv + 64 < n_vec;
    const float4 x0 = a4[iv], y0 = b4[iv];
    float4 x1 = x0, y1 = y0;
    if (two) {
      x1 = a4[iv + 64];
      y1 = b4[iv + 64];
    }
    const float xs[8] = {x0.x, x0.y, x0.z, x0.w, x1.x, x1.y, x1.z, x1.w};
    const float ys[8] = {y0.x, y0.y, y0.z, y0.w, y1.x, y1.y, y1.z, y1.w};
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      if (e >= 4 && !two) break;
      const double x = double(xs[e]), y = double(ys[e]);
      if (cosine) {
        acc += x * y;
        aa += x * x;
        bb += y * y;
      } else {
        const double df = x - y;
        acc += df * df;
      }
    }
  }
  if (cosine) return 1.0 - wave_sum(acc) / sqrt(wave_sum(aa) * wave_sum(bb));
  return sqrt(wave_sum(acc));
}

// The float32 probe value of a source, from the probe's score  score = |s|^2 - 2 q.s  and the two squared
// lengths: the squared Euclidean distance, or (cosine) the cosine distance 1 - q.s / (|q| |s|).
__device__ __forceinline__ float probe_value(float score, float qn, float sn, int cosine) {
  if (cosine) return 1.f - 0.5f * (sn - score) / sqrtf(qn * sn);
  return score + qn;
}

// Float32 pre-filter bound for "distance <= tau" on probe_value.  The float32 inner product behind the
// probe value carries an absolute error of at most (dim + 8) * 2^-24 * |q| |s| (every product and every
// partial sum rounds once), so the squared distance is off by at most twice that plus the roundings of
// the two squared lengths, i.e. by less than `rel` * (|q|^2 + |s|^2), and the cosine distance by less
// than `rel`; anything that could be within tau in exact arithmetic passes the bound and is then decided
// in float64.  (The factor 1 + 1e-3 covers the float32 rounding of tau^2 itself.)
__device__ __forceinline__ float prefilter_rel(int dim) { return 2.5f * float(dim + 8) * 5.9604645e-8f; }
__device__ __forceinline__ float dense_slack(float qn, float sn_max, int dim, int cosine) {
  return 2.f * (cosine ? prefilter_rel(dim) + 1e-6f : prefilter_rel(dim) * (qn + sn_max));
}
__device__ __forceinline__ float prefilter_bound(double tau, float qn, float sn, int dim, int cosine) {
  const double rel = double(prefilter_rel(dim));
  const double b = cosine ? tau * (1.0 + 1e-3) + rel + 1e-6 : tau * tau * (1.0 + 1e-3) + rel * (double(qn) + double(sn));
  return b > 3.0e38 ? 3.0e38f : float(b);
}

// ---------------------------------------------------------------------------
// Step "distances to all keys" of Algorithm 1, second half: from the dense
// float32 probe row of each query keep the sources that can lie within tau, and
// evaluate those in float64.  One block per batch row.
//   D32[i*ldD + s]     score of row i against source s (slots 0..c-1, batch rows c..c+n-1)
//   srcs[(s)*dim ..]   the source vectors (slot keys, then the batch rows)
//   cand_cnt[i]        number of sources that passed (may exceed cap)
//   cand_src/cand_d    first min(cnt,cap) of them, unordered, with float64 distances
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void probe_candidates_kernel(
    const float* __restrict__ D32, long ldD, const float* __restrict__ srcs, const float* __restrict__ srcnrm,
    int dim, int c, int n, const CacheState* __restrict__ st, double tau, int cosine, int cap,
    int* __restrict__ cand_cnt, int* __restrict__ cand_src, double* __restrict__ cand_d, int row_begin) {
  // block b: batch row row_begin + b, whose probe row is D32 + b * ldD
  const int i = row_begin + blockIdx.x;
  if (i >= n) return;
  __shared__ int count;
  __shared__ int list[256];  // cap <= 256
  if (threadIdx.x == 0) count = 0;
  __syncthreads();
  const int size0 = st->size;
  const float qn = srcnrm[c + i];
  const float* row = D32 + long(blockIdx.x) * ldD;
  for (int s = threadIdx.x; s < size0; s += blockDim.x) {
    const float sn = srcnrm[s];
    if (probe_value(row[s], qn, sn, cosine) <= prefilter_bound(tau, qn, sn, dim, cosine)) {
      const int pos = atomicAdd(&count, 1);
      if (pos < cap) list[pos] = s;
    }
  }
  for (int j = threadIdx.x; j < i; j += blockDim.x) {
    const int s = c + j;
    const float sn = srcnrm[s];
    if (probe_value(row[s], qn, sn, cosine) <= prefilter_bound(tau, qn, sn, dim, cosine)) {
      const int pos = atomicAdd(&count, 1);
      if (pos < cap) list[pos] = s;
    }
  }
  __syncthreads();
  const int cnt = count;
  if (threadIdx.x == 0) cand_cnt[i] = cnt;
  const int lane = threadIdx.x & 63, wib = threadIdx.x >> 6;
  const float* q = srcs + long(c + i) * dim;
  const int m = cnt < cap ? cnt : cap;
  for (int p = wib; p < m; p += 4) {
    const int s = list[p];
    const double d = wave_keydist64(q, srcs + long(s) * dim, dim, lane, cosine);
    if (lane == 0) {
      cand_src[long(i) * cap + p] = s;
      cand_d[long(i) * cap + p] = d;
    }
  }
}

// Before the first probe of a batch: empty candidate lists and overflow lists, and the number of live
// slots as it is now (the resolver of an early range may change the state while a later range is probed).
__global__ __launch_bounds__(256) void probe_prepare_kernel(int n, int* __restrict__ cand_cnt, int n_ranges,
                                                            int* __restrict__ ovf_cnt, const CacheState* __restrict__ st,
                                                            int* __restrict__ live_slots) {
  const int t = blockIdx.x * 256 + threadIdx.x;
  if (t < n) cand_cnt[t] = 0;
  if (t < n_ranges) ovf_cnt[t] = 0;
  if (t == 0) *live_slots = st->size;
}

// ---------------------------------------------------------------------------
// Order-preserving resolver: Algorithm 1 after the distances (nearest key, tolerance test,
// eviction, insertion) for rows 0..n-1 in order,
// given every row's candidate sources.  One wave walks the rows; the only
// sequential state is which sources are live and the eviction order (a doubly
// linked list over slots: FIFO appends on insert, LRU also moves a slot to the
// back when it answers a query; Section 3.3.2).
//
// Per row: the nearest live source (ties: smaller seq) with float64 distance
// <= tau is a hit.  Otherwise the row misses, takes the next free slot or the
// slot at the front of the eviction order, and becomes a live source itself.
// Rows with more candidates than the list holds are resolved from the dense
// probe row over the live slots instead (float32 minimum, then float64 on the
// near-minimal ones).
//
// Outputs per row: hit flag, answering source (or -1), slot taken (or -1);
// the list of missing rows in row order and its length.
// ---------------------------------------------------------------------------
struct ResolverBest {
  double d;
  long long seq;
  int src;
};

__device__ __forceinline__ void best_take(ResolverBest& b, double d, long long seq, int src) {
  if (d < b.d || (d == b.d && seq < b.seq)) {
    b.d = d;
    b.seq = seq;
    b.src = src;
  }
}

__device__ __forceinline__ void best_wave_reduce(ResolverBest& b) {
#pragma unroll
  for (int m = 32; m >= 1; m >>= 1) {
    const double od = __shfl_xor(b.d, m, kWave);
    const long long os = __shfl_xor(b.seq, m, kWave);
    const int osrc = __shfl_xor(b.src, m, kWave);
    best_take(b, od, os, osrc);
  }
}

__global__ __launch_bounds__(64) void resolver_kernel(
    int n, int c, int dim, int policy_lru, long long base_seq, double tau, int cosine, CacheState* __restrict__ st,
    long long* slot_seq, int* slot_next, int* slot_prev, const int* __restrict__ cand_cnt,
    const int* __restrict__ cand_src, const double* __restrict__ cand_d, int cap, const float* __restrict__ D32,
    long ldD, const float* __restrict__ srcs, const float* __restrict__ srcnrm, uint8_t* __restrict__ hit_out,
    int* __restrict__ src_out, int* row_slot, int* __restrict__ miss_list, int* __restrict__ miss_count,
    int row_begin, int row_end) {
  // Rows row_begin .. row_end - 1 of the batch (a batch may take several launches, in row order: all state is
  // in device memory, and the list of missing rows grows from launch to launch); D32 holds the dense probe
  // rows of this range, row i at D32 + (i - row_begin) * ldD.
  (void)n;
  const int lane = threadIdx.x;
  int size = st->size, head = st->head, tail = st->tail;
  unsigned long long hits = 0, misses = 0, inserts = 0, evictions = 0, inbatch = 0, dense = 0;
  int M = row_begin > 0 ? *miss_count : 0;
  const double kInf = __longlong_as_double(0x7ff0000000000000ll);

  for (int i = row_begin; i < row_end; ++i) {
    const int cnt = cand_cnt ? cand_cnt[i] : 0;  // no probe ran when the cache is disabled
    ResolverBest best{kInf, 0x7fffffffffffffffll, -1};
    if (cnt > 0 && cnt <= cap) {
      for (int p0 = 0; p0 < cnt; p0 += 64) {
        const int p = p0 + lane;
        if (p < cnt) {
          const int s = cand_src[long(i) * cap + p];
          const double d = cand_d[long(i) * cap + p];
          long long seq;
          bool live;
          if (s < c) {
            seq = slot_seq[s];
            live = seq < base_seq;  // still holds the key it had when the batch began
          } else {
            const int t = row_slot[s - c];
            seq = base_seq + (s - c);
            live = t >= 0 && slot_seq[t] == seq;  // that row missed, was stored, and is still there
          }
          if (live && d <= tau) best_take(best, d, seq, s);
        }
      }
      best_wave_reduce(best);
    } else if (cnt > cap) {
      ++dense;
      const float qn = srcnrm[c + i];
      const float* row = D32 + long(i - row_begin) * ldD;
      float mn = 3.4e38f, snmax = 0.f;
      for (int t = lane; t < size; t += 64) {
        const long long sq = slot_seq[t];
        const int s = sq >= base_seq ? c + int(sq - base_seq) : t;
        mn = fminf(mn, probe_value(row[s], qn, srcnrm[s], cosine));
        snmax = fmaxf(snmax, srcnrm[s]);
      }
#pragma unroll
      for (int m = 32; m >= 1; m >>= 1) {
        mn = fminf(mn, __shfl_xor(mn, m, kWave));
        snmax = fmaxf(snmax, __shfl_xor(snmax, m, kWave));
      }
      // twice the error bound of a probe value: a source beyond minimum + slack cannot be the nearest
      const float slack = dense_slack(qn, snmax, dim, cosine);
      if (mn <= prefilter_bound(tau, qn, snmax, dim, cosine) + slack) {
        const float near = mn + slack;
        for (int t0 = 0; t0 < size; t0 += 64) {
          const int t = t0 + lane;
          int s = -1;
          long long sq = 0;
          bool is_near = false;
          if (t < size) {
            sq = slot_seq[t];
            s = sq >= base_seq ? c + int(sq - base_seq) : t;
            is_near = probe_value(row[s], qn, srcnrm[s], cosine) <= near;
          }
          unsigned long long mask = __ballot(is_near);
          while (mask) {
            const int b = __ffsll((long long)mask) - 1;
            mask &= mask - 1;
            const int sb = __shfl(s, b, kWave);
            const long long sqb = __shfl(sq, b, kWave);
            const double d = wave_keydist64(srcs + long(c + i) * dim, srcs + long(sb) * dim, dim, lane, cosine);
            if (d <= tau) best_take(best, d, sqb, sb);
          }
        }
      }
    }

    if (best.src >= 0) {
      ++hits;
      if (best.src >= c) ++inbatch;
      const int t = best.src < c ? best.src : row_slot[best.src - c];
      if (policy_lru && t != tail) {
        const int p = slot_prev[t], nx = slot_next[t];  // nx >= 0 because t is not the tail
        if (lane == 0) {
          if (p >= 0) slot_next[p] = nx;
          slot_prev[nx] = p;
          slot_prev[t] = tail;
          slot_next[t] = -1;
          slot_next[tail] = t;
        }
        if (p < 0) head = nx;
        tail = t;
      }
      if (lane == 0) {
        hit_out[i] = 1;
        src_out[i] = best.src;
        row_slot[i] = -1;
      }
    } else {
      ++misses;
      int t = -1;
      if (c > 0) {
        if (size < c) {
          t = size++;
        } else {
          t = head;
          head = slot_next[t];
          if (lane == 0 && head >= 0) slot_prev[head] = -1;
          if (head < 0) tail = -1;
          ++evictions;
        }
        if (lane == 0) {
          slot_seq[t] = base_seq + i;
          slot_prev[t] = tail;
          slot_next[t] = -1;
          if (tail >= 0) slot_next[tail] = t;
        }
        if (tail < 0) head = t;
        tail = t;
        ++inserts;
      }
      if (lane == 0) {
        hit_out[i] = 0;
        src_out[i] = -1;
        row_slot[i] = t;
        miss_list[M] = i;
      }
      ++M;
    }
  }
  if (lane == 0) {
    st->size = size;
    st->head = head;
    st->tail = tail;
    st->queries += (unsigned long long)(row_end - row_begin);
    st->hits += hits;
    st->misses += misses;
    st->inserts += inserts;
    st->evictions += evictions;
    st->inbatch_hits += inbatch;
    st->dense_resolves += dense;
    *miss_count = M;
  }
}

// ---------------------------------------------------------------------------
// After the resolver, before the scan.  One block per batch row.
//   - a row that missed and still owns its slot at the end of the batch copies
//     its vector and squared norm into the slot (Algorithm 1, "C[q] <- I", key part;
//     copy_keys == 0: the resolver has already written the keys);
//   - a row that hit a key resident since before the batch answers from that key's
//     stored list now, before any list is overwritten: the list itself (K == k), or
//     with a re-ranking factor above 1 (K = rho * k stored per key, Section 3.3.4) the
//     k stored documents nearest to the row's own query.
// X / corpus_kind: the corpus with its element type and distance function (see corpus_kind), read only for re-ranking.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void post_resolve_kernel(
    int n, int c, int dim, int k, int K, int copy_keys, long long base_seq, float* srcs, float* srcnrm,
    const long long* __restrict__ slot_seq, const uint8_t* __restrict__ hit, const int* __restrict__ src,
    const int* __restrict__ row_slot, const int64_t* __restrict__ val_ids, const float* __restrict__ val_d,
    const void* __restrict__ X, int corpus_kind, int64_t* __restrict__ out_ids, float* __restrict__ out_d) {
  const int i = blockIdx.x;
  if (i >= n) return;
  if (hit[i]) {
    const int s = src[i];
    if (s < c) {
      if (K == k || X == nullptr) {  // nothing to re-rank, or no corpus (every stored id is padding)
        for (int e = threadIdx.x; e < k; e += blockDim.x) {
          out_ids[long(i) * k + e] = val_ids[long(s) * K + e];
          if (out_d) out_d[long(i) * k + e] = val_d[long(s) * K + e];
        }
      } else {
        __shared__ uint64_t keys[256];
        __shared__ double d64[256];
        __shared__ int cid[256];
        const float* q = srcs + long(c + i) * dim;
        float* od = out_d ? out_d + long(i) * k : nullptr;
        block_rerank_stored_any<256>(corpus_kind, val_ids + long(s) * K, K, k, q, X, dim, out_ids + long(i) * k, od,
                                     keys, d64, cid, threadIdx.x);
      }
    }
  } else if (copy_keys) {
    const int t = row_slot[i];
    if (t >= 0 && slot_seq[t] == base_seq + i) {
      const float4* from = reinterpret_cast<const float4*>(srcs + long(c + i) * dim);
      float4* to = reinterpret_cast<float4*>(srcs + long(t) * dim);
      for (int e = threadIdx.x; e < dim / 4; e += blockDim.x) to[e] = from[e];
      if (threadIdx.x == 0) srcnrm[t] = srcnrm[c + i];
    }
  }
}

// ---------------------------------------------------------------------------
// After the scan.  One block per batch row.
//   - a row that missed returns its scan result, and stores it as its key's
//     value if the key is still resident (Algorithm 1, "C[q] <- I", value part);
//   - a row that hit an earlier row of the same batch answers from that row's result.
// A scan result has K entries (K = rho * k with a re-ranking factor rho, Section 3.3.4): the
// row that missed returns the first k and stores all K; a hit returns the stored list itself
// when K == k, else the k stored documents nearest to its own query (batch_rows[i]).
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void finalize_kernel(int n, int c, int k, int K, long long base_seq,
                                                       const long long* __restrict__ slot_seq,
                                                       const uint8_t* __restrict__ hit,
                                                       const int* __restrict__ src,
                                                       const int* __restrict__ row_slot,
                                                       const int64_t* __restrict__ res_ids,
                                                       const float* __restrict__ res_d, int64_t* val_ids,
                                                       float* val_d, const float* __restrict__ batch_rows, int dim,
                                                       const void* __restrict__ X, int corpus_kind,
                                                       int64_t* __restrict__ out_ids, float* __restrict__ out_d) {
  const int i = blockIdx.x;
  if (i >= n) return;
  if (hit[i]) {
    if (src[i] < c) return;
    const int from = src[i] - c;
    if (K == k || X == nullptr) {  // nothing to re-rank, or no corpus (every stored id is padding)
      for (int e = threadIdx.x; e < k; e += blockDim.x) {
        out_ids[long(i) * k + e] = res_ids[long(from) * K + e];
        if (out_d) out_d[long(i) * k + e] = res_d[long(from) * K + e];
      }
    } else {
      __shared__ uint64_t keys[256];
      __shared__ double d64[256];
      __shared__ int cid[256];
      const float* q = batch_rows + long(i) * dim;
      float* od = out_d ? out_d + long(i) * k : nullptr;
      block_rerank_stored_any<256>(corpus_kind, res_ids + long(from) * K, K, k, q, X, dim, out_ids + long(i) * k, od,
                                   keys, d64, cid, threadIdx.x);
    }
    return;
  }
  const int t = row_slot[i];
  const bool store = t >= 0 && slot_seq[t] == base_seq + i;
  for (int e = threadIdx.x; e < K; e += blockDim.x) {
    const int64_t id = res_ids[long(i) * K + e];
    const float d = res_d[long(i) * K + e];
    if (e < k) {
      out_ids[long(i) * k + e] = id;
      if (out_d) out_d[long(i) * k + e] = d;
    }
    if (store) {
      val_ids[long(t) * K + e] = id;
      val_d[long(t) * K + e] = d;
    }
  }
}

// ---------------------------------------------------------------------------
// Calls with a handful of rows (n <= kSmallRows): the whole cache side in two launches of
// this kernel.
//
// phase == 1, a grid of blocks: distance (Euclidean, or cosine when `cosine` is set) from every row of
// the call to every resident key, directly in float64 (one wave per key):
// with so few rows there is nothing to pre-filter.  D64[i * c + s].
// phase == 2, one block: rows in order, exactly as resolver_kernel does -- nearest live
// source within tau (ties: smaller seq) is a hit, otherwise evict/insert -- with distances
// between rows of the call evaluated on the spot.  The same block then copies the keys of
// rows that missed and still own their slot, and answers hits on resident keys from the
// stored lists (what post_resolve_kernel does for large calls).
// The rows are read from the caller's buffer; nothing is staged.
// (A single launch whose last block does phase 2 was slower: the device-wide fences that
// hand the distances from block to block cost more than a second launch.)
// ---------------------------------------------------------------------------
constexpr int kSmallRows = 4;

__global__ __launch_bounds__(1024) void probe_resolve_small_kernel(
    const float* __restrict__ queries, int n, int c, int dim, int k, int K, int policy_lru, long long base_seq,
    double tau, int cosine, CacheState* st, long long* slot_seq, int* slot_next, int* slot_prev, float* srcs,
    float* srcnrm,
    const int64_t* __restrict__ val_ids, const float* __restrict__ val_d, const void* __restrict__ X,
    int corpus_kind, double* D64, int phase,
    uint8_t* hit_out, int* src_out, int* row_slot, int* __restrict__ miss_list,
    int* __restrict__ miss_count, int64_t* __restrict__ out_ids, float* __restrict__ out_d) {
  const int tid = threadIdx.x, lane = tid & 63, wib = tid >> 6;
  constexpr int NW = 16;
  __shared__ uint64_t rr_keys[256];  // re-ranking of a stored list
  __shared__ double rr_d[256];
  __shared__ int rr_id[256];
  __shared__ double red_d[NW];
  __shared__ long long red_seq[NW];
  __shared__ int red_src[NW];
  __shared__ double pair_d[kSmallRows];
  // the decisions of this call, kept on chip for the routing below (reading them back from global
  // memory would put two more round trips on the path of every call)
  __shared__ int dec_hit[kSmallRows], dec_src[kSmallRows], dec_slot[kSmallRows];

  const int size0 = st->size;
  // phase 1
  if (phase != 2)
  for (int s = blockIdx.x * NW + wib; s < size0; s += gridDim.x * NW) {
    // 16 bytes per lane, two steps of the key and of every row issued before anything is used
    const float4* key = reinterpret_cast<const float4*>(srcs + long(s) * dim);
    const int n_vec = dim / 4;
    double acc[kSmallRows], qq[kSmallRows], kk = 0.0;   // cosine: inner products and the squared lengths
#pragma unroll
    for (int i = 0; i < kSmallRows; ++i) acc[i] = qq[i] = 0.0;
    for (int iv0 = lane; iv0 < n_vec; iv0 += 128) {
      const bool two = iv0 + 64 < n_vec;
      float4 kv[2], qv[2][kSmallRows];
#pragma unroll
      for (int st = 0; st < 2; ++st) {
        if (st == 1 && !two) break;
        kv[st] = key[iv0 + 64 * st];
#pragma unroll
        for (int i = 0; i < kSmallRows; ++i)
          if (i < n) qv[st][i] = reinterpret_cast<const float4*>(queries + long(i) * dim)[iv0 + 64 * st];
      }
#pragma unroll
      for (int st = 0; st < 2; ++st) {
        if (st == 1 && !two) break;
        const double kx = double(kv[st].x), ky = double(kv[st].y), kz = double(kv[st].z), kw = double(kv[st].w);
        if (cosine) kk += kx * kx + ky * ky + kz * kz + kw * kw;
#pragma unroll
        for (int i = 0; i < kSmallRows; ++i)
          if (i < n) {
            const double qx = double(qv[st][i].x), qy = double(qv[st][i].y), qz = double(qv[st][i].z),
                         qw = double(qv[st][i].w);
            if (cosine) {
              // (each sum takes its four products in the same order, so identical vectors give identical sums)
              acc[i] += qx * kx + qy * ky + qz * kz + qw * kw;
              qq[i] += qx * qx + qy * qy + qz * qz + qw * qw;
            } else {
              const double dx = qx - kx, dy = qy - ky, dz = qz - kz, dw = qw - kw;
              acc[i] += dx * dx + dy * dy + dz * dz + dw * dw;
            }
          }
      }
    }
    if (cosine) kk = wave_sum(kk);
#pragma unroll
    for (int i = 0; i < kSmallRows; ++i)
      if (i < n) {
        const double total = wave_sum(acc[i]);
        const double d = cosine ? 1.0 - total / sqrt(wave_sum(qq[i]) * kk) : sqrt(total);
        if (lane == 0) D64[long(i) * c + s] = d;
      }
  }
  if (phase == 1) return;

  // phase 2
  int size = size0, head = st->head, tail = st->tail;
  unsigned long long hits = 0, misses = 0, inserts = 0, evictions = 0, inbatch = 0;
  int M = 0;
  const double kInf = __longlong_as_double(0x7ff0000000000000ll);
  for (int i = 0; i < n; ++i) {
    // distances to earlier rows of this call (at most three), one wave each
    if (wib < i) {
      const double d = wave_keydist64(queries + long(i) * dim, queries + long(wib) * dim, dim, lane, cosine);
      if (lane == 0) pair_d[wib] = d;
    }
    __syncthreads();
    ResolverBest best{kInf, 0x7fffffffffffffffll, -1};
    for (int s = tid; s < c; s += 1024) {
      // (both read whether or not they are needed, and over all c slots rather than the size0 in use:
      // the loads then wait neither for each other nor for the cache state to arrive)
      const long long seq = slot_seq[s];
      const double d = D64[long(i) * c + s];
      // seq < base_seq: still the key it held when the call began
      if (s < size0 && seq < base_seq && d <= tau) best_take(best, d, seq, s);
    }
    if (tid < i) {
      const int t = dec_slot[tid];
      const long long seq = base_seq + tid;
      if (t >= 0 && slot_seq[t] == seq && pair_d[tid] <= tau) best_take(best, pair_d[tid], seq, c + tid);
    }
    best_wave_reduce(best);
    if (lane == 0) {
      red_d[wib] = best.d;
      red_seq[wib] = best.seq;
      red_src[wib] = best.src;
    }
    __syncthreads();
    if (tid == 0) {
      ResolverBest b{kInf, 0x7fffffffffffffffll, -1};
      for (int w = 0; w < NW; ++w)
        if (red_src[w] >= 0) best_take(b, red_d[w], red_seq[w], red_src[w]);
      if (b.src >= 0) {
        ++hits;
        if (b.src >= c) ++inbatch;
        const int t = b.src < c ? b.src : dec_slot[b.src - c];
        dec_hit[i] = 1;
        dec_src[i] = b.src;
        dec_slot[i] = -1;
        if (policy_lru && t != tail) {
          const int p = slot_prev[t], nx = slot_next[t];
          if (p >= 0) slot_next[p] = nx; else head = nx;
          slot_prev[nx] = p;
          slot_prev[t] = tail;
          slot_next[t] = -1;
          slot_next[tail] = t;
          tail = t;
        }
        hit_out[i] = 1;
        src_out[i] = b.src;
        row_slot[i] = -1;
      } else {
        ++misses;
        int t = -1;
        if (c > 0) {
          if (size < c) {
            t = size++;
          } else {
            t = head;
            head = slot_next[t];
            if (head >= 0) slot_prev[head] = -1; else tail = -1;
            ++evictions;
          }
          slot_seq[t] = base_seq + i;
          slot_prev[t] = tail;
          slot_next[t] = -1;
          if (tail >= 0) slot_next[tail] = t; else head = t;
          tail = t;
          ++inserts;
        }
        dec_hit[i] = 0;
        dec_src[i] = -1;
        dec_slot[i] = t;
        hit_out[i] = 0;
        src_out[i] = -1;
        row_slot[i] = t;
        miss_list[M++] = i;
      }
    }
    __syncthreads();   // (also a memory fence: the state written by thread 0 is visible to the next row)
  }
  if (tid == 0) {
    st->size = size;
    st->head = head;
    st->tail = tail;
    st->queries += (unsigned long long)n;
    st->hits += hits;
    st->misses += misses;
    st->inserts += inserts;
    st->evictions += evictions;
    st->inbatch_hits += inbatch;
    *miss_count = M;
  }
  // (no barrier: what follows reads only the decisions in LDS and the slot state of the row loop,
  // both behind that loop's last barrier, so it overlaps with the first thread's bookkeeping)
  // keys of rows that missed and still own their slot; hits on keys resident before the call
  for (int i = 0; i < n; ++i) {
    if (dec_hit[i]) {
      const int s = dec_src[i];
      if (s < c) {
        if (K == k) {
          for (int e = tid; e < k; e += 1024) {
            out_ids[long(i) * k + e] = val_ids[long(s) * k + e];
            if (out_d) out_d[long(i) * k + e] = val_d[long(s) * k + e];
          }
        } else {
          // re-ranking factor above 1 (Section 3.3.4): the stored documents nearest to this row's query
          block_rerank_stored_any<1024>(corpus_kind, val_ids + long(s) * K, K, k, queries + long(i) * dim, X, dim,
                                        out_ids + long(i) * k, out_d ? out_d + long(i) * k : nullptr, rr_keys, rr_d,
                                        rr_id, tid);
          __syncthreads();  // the LDS arrays serve the next row
        }
      }
    } else {
      const int t = dec_slot[i];
      if (t >= 0 && slot_seq[t] == base_seq + i) {
        float sq = 0.f;
        for (int e = tid; e < dim; e += 1024) {
          const float v = queries[long(i) * dim + e];
          srcs[long(t) * dim + e] = v;
          sq += v * v;
        }
        sq = wave_sum(sq);
        __syncthreads();
        if (lane == 0) red_d[wib] = double(sq);
        __syncthreads();
        if (tid == 0) {
          float total = 0.f;
          for (int w = 0; w < NW; ++w) total += float(red_d[w]);
          srcnrm[t] = total;
        }
      }
    }
  }
}

}  // namespace prox
