// The bucketed cache of Section 3.2: an L-bit code from the signs of the query's inner products
// with L hyperplane normals names a bucket; every bucket is a cache of capacity b with its own
// FIFO/LRU order, and a query is looked up (and on a miss stored) only in its bucket.
//
// Slots are laid out bucket by bucket: bucket g owns slots g*b .. g*b+b-1 and fills them in
// index order, so its live slots are always the first `size[g]`.  Buckets do not interact, so a
// batch is regrouped by code (keeping row order inside a code) and every bucket that occurs is
// walked by its own block, rows in order, exactly as Algorithm 1 prescribes for one cache (nearest
// key, tolerance test, eviction, insertion); different buckets run side by side.  A bucket holds a few dozen keys, so the block
// computes the distances to all of them directly in float64 (direct-difference form) and there is
// no pre-filter.  A key is written into its slot at once (the block owns the bucket), so later
// rows of the batch simply find it there; its value arrives after the scan, which is why a hit on
// such a key is reported as "row j of this call" like in the flat cache.
#pragma once

#include "cache_kernels.hpp"

namespace prox {

constexpr int kLshMaxBits = 16;
constexpr int kLshMaxBucket = 256;   // keys per bucket the resolver's LDS arrays hold
constexpr int kLshRowBits = 13;      // batch rows are numbered below 2^13 (the largest batch)

// ---------------------------------------------------------------------------
// Hash codes.  One wave per four rows: bit i of code[row] is 1 exactly when q . r_i >= 0, with the
// inner product accumulated in float64 (the sign is the decision here).  The normals are read
// once per four rows and four of them are in flight together with the four rows' values.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void lsh_codes_kernel(const float* __restrict__ Q, int n, int dim,
                                                        const float* __restrict__ planes, int n_bits,
                                                        int* __restrict__ code) {
  constexpr int R = 4;  // rows per wave
  const int lane = threadIdx.x & 63;
  const int row0 = (blockIdx.x * 4 + (threadIdx.x >> 6)) * R;
  if (row0 >= n) return;
  const float* q[R];
#pragma unroll
  for (int r = 0; r < R; ++r) q[r] = Q + long(row0 + r < n ? row0 + r : n - 1) * dim;
  int c[R] = {0, 0, 0, 0};
  for (int b0 = 0; b0 < n_bits; b0 += 4) {
    double acc[4][R];
#pragma unroll
    for (int u = 0; u < 4; ++u)
#pragma unroll
      for (int r = 0; r < R; ++r) acc[u][r] = 0.0;
    for (int x = lane; x < dim; x += 64) {
      float qv[R], pv[4];
#pragma unroll
      for (int r = 0; r < R; ++r) qv[r] = q[r][x];
#pragma unroll
      for (int u = 0; u < 4; ++u) pv[u] = b0 + u < n_bits ? planes[long(b0 + u) * dim + x] : 0.f;
#pragma unroll
      for (int u = 0; u < 4; ++u)
#pragma unroll
        for (int r = 0; r < R; ++r) acc[u][r] += double(qv[r]) * double(pv[u]);
    }
#pragma unroll
    for (int u = 0; u < 4; ++u)
#pragma unroll
      for (int r = 0; r < R; ++r)
        if (b0 + u < n_bits && wave_sum(acc[u][r]) >= 0.0) c[r] |= 1 << (b0 + u);
  }
  if (lane < R && row0 + lane < n) {
    int mine = c[0];
#pragma unroll
    for (int r = 1; r < R; ++r) mine = lane == r ? c[r] : mine;
    code[row0 + lane] = mine;
  }
}

// ---------------------------------------------------------------------------
// Regroup the batch by code, rows of one code in row order: sorts (code, row) pairs.
// One block of 1024 threads; n <= 2^13.  sorted[j] = (code << 13) | row; seg_start[g] is the
// position in `sorted` where the g-th distinct code begins, *n_segs the number of distinct codes.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(1024) void lsh_group_kernel(const int* __restrict__ code, int n,
                                                         uint32_t* __restrict__ sorted, int* __restrict__ seg_start,
                                                         int* __restrict__ n_segs) {
  __shared__ uint32_t keys[1 << kLshRowBits];
  __shared__ int counts[1024];
  const int tid = threadIdx.x;
  const int P = next_pow2(n < 2 ? 2 : n);
  for (int i = tid; i < P; i += 1024) keys[i] = i < n ? (uint32_t(code[i]) << kLshRowBits) | uint32_t(i) : 0xffffffffu;
  __syncthreads();
  for (int k = 2; k <= P; k <<= 1) {
    for (int j = k >> 1; j > 0; j >>= 1) {
      for (int t = tid; t < (P >> 1); t += 1024) {
        const int i = ((t & ~(j - 1)) << 1) | (t & (j - 1));
        const int p = i | j;
        const bool asc = (i & k) == 0;
        const uint32_t a = keys[i], b = keys[p];
        if ((a > b) == asc) {
          keys[i] = b;
          keys[p] = a;
        }
      }
      __syncthreads();
    }
  }
  for (int i = tid; i < n; i += 1024) sorted[i] = keys[i];
  // positions where a new code begins, in order
  constexpr int PER = (1 << kLshRowBits) / 1024;
  int mine = 0;
  for (int r = 0; r < PER; ++r) {
    const int i = tid * PER + r;
    if (i < n && (i == 0 || (keys[i] >> kLshRowBits) != (keys[i - 1] >> kLshRowBits))) ++mine;
  }
  counts[tid] = mine;
  __syncthreads();
  for (int off = 1; off < 1024; off <<= 1) {  // inclusive scan
    const int v = tid >= off ? counts[tid - off] : 0;
    __syncthreads();
    counts[tid] += v;
    __syncthreads();
  }
  int pos = counts[tid] - mine;
  for (int r = 0; r < PER; ++r) {
    const int i = tid * PER + r;
    if (i < n && (i == 0 || (keys[i] >> kLshRowBits) != (keys[i - 1] >> kLshRowBits))) seg_start[pos++] = i;
  }
  if (tid == 1023) *n_segs = counts[1023];
}

// ---------------------------------------------------------------------------
// One block per distinct code of the regrouped batch (blocks beyond *n_segs return at once);
// the block walks that bucket's rows in order.
//
// Per row: float64 distance (Euclidean, or cosine when `cosine` is set) to each live key of the bucket, nearest key (ties: smaller seq),
// hit if within tau (LRU: the key moves to the back of the bucket's order); otherwise the row
// takes the bucket's next free slot or evicts the front of its order, and its vector is written
// into the slot.  Outputs per row as resolver_kernel: hit flag, answering source (slot, or
// c_total + j when the key was stored by row j of this call), slot taken.
//
// The bucket's state lives in LDS while the block walks: inserting positions, the order as
// local links, the current query, and -- when keys_in_lds -- the bucket's keys themselves
// (b * dim floats), so that a row costs one fetch of its vector plus on-chip work.  Dynamic
// LDS: (1 + (keys_in_lds ? b : 0)) * dim floats.
// ---------------------------------------------------------------------------
constexpr int kLshThreads = 1024;
__global__ __launch_bounds__(kLshThreads) void lsh_resolve_kernel(
    const uint32_t* __restrict__ sorted, const int* __restrict__ seg_start, const int* __restrict__ n_segs, int n,
    int b, int c_total, int dim, int policy_lru, long long base_seq, double tau, int cosine, int keys_in_lds,
    const float* batch_rows, float* srcs, long long* slot_seq, int* slot_next,
    int* slot_prev, int* bkt_size, int* bkt_head, int* bkt_tail, CacheState* st, uint8_t* __restrict__ hit_out,
    int* __restrict__ src_out, int* __restrict__ row_slot) {
  if (int(blockIdx.x) >= *n_segs) return;
  const int j0 = seg_start[blockIdx.x];
  const int code = int(sorted[j0] >> kLshRowBits);

  extern __shared__ float lds_rows[];          // [dim] the current query, then [b][dim] keys if they fit
  float* lq = lds_rows;
  float* lkeys = lds_rows + dim;
  __shared__ double d64[kLshMaxBucket];
  __shared__ long long lseq[kLshMaxBucket];
  __shared__ int lnext[kLshMaxBucket];         // the bucket's order, local slot numbers, -1 = none
  __shared__ int lprev[kLshMaxBucket];
  __shared__ int s_best;                       // local slot of the answering key, -1: miss
  __shared__ int s_size;                       // live keys of the bucket
  __shared__ int s_slot;                       // local slot the current row takes when it misses
  const int tid = threadIdx.x, lane = tid & 63, wib = tid >> 6;
  // Inside the row loop only LDS traffic has to be ordered between the waves when the keys live in
  // LDS; a full __syncthreads() would also wait for the next row's vector, which is fetched ahead on purpose.
  auto row_barrier = [&]() {
    if (keys_in_lds)
      asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
    else
      __syncthreads();
  };

  const int slot0 = code * b;
  float* bucket_keys = srcs + long(slot0) * dim;
  const int size0 = bkt_size[code];
  for (int s = tid; s < size0; s += kLshThreads) {
    lseq[s] = slot_seq[slot0 + s];
    const int nx = slot_next[slot0 + s], pv = slot_prev[slot0 + s];
    lnext[s] = nx >= 0 ? nx - slot0 : -1;
    lprev[s] = pv >= 0 ? pv - slot0 : -1;
  }
  if (keys_in_lds)
    for (int x = tid; x < size0 * dim; x += kLshThreads) lkeys[x] = bucket_keys[x];
  // the order is walked by thread 0 alone
  int head = -1, tail = -1;
  int hits = 0, misses = 0, inserts = 0, evictions = 0, inbatch = 0;
  if (tid == 0) {
    s_size = size0;
    const int h = bkt_head[code], tl = bkt_tail[code];
    head = h >= 0 ? h - slot0 : -1;
    tail = tl >= 0 ? tl - slot0 : -1;
  }
  // the row being resolved sits in LDS; the bucket's next row is fetched into registers meanwhile
  constexpr int QR = 4096 / kLshThreads;  // values of a row per thread, at the largest dimension
  constexpr uint32_t kNone = 0xffffffffu;
  constexpr uint32_t kRowMask = (1u << kLshRowBits) - 1;
  uint32_t e_cur = sorted[j0];
  uint32_t e_nxt = j0 + 1 < n ? sorted[j0 + 1] : kNone;
  float qreg[QR];
#pragma unroll
  for (int u = 0; u < QR; ++u) {
    const int x = tid + u * kLshThreads;
    qreg[u] = x < dim ? batch_rows[long(e_cur & kRowMask) * dim + x] : 0.f;
  }
  __syncthreads();

  for (int j = j0;; ++j) {
    const int i = int(e_cur & kRowMask);
#pragma unroll
    for (int u = 0; u < QR; ++u) {
      const int x = tid + u * kLshThreads;
      if (x < dim) lq[x] = qreg[u];
    }
    const int size = s_size;
    row_barrier();
    const bool more = e_nxt != kNone && int(e_nxt >> kLshRowBits) == code;
    uint32_t e_nn = kNone;
    if (more) {
#pragma unroll
      for (int u = 0; u < QR; ++u) {
        const int x = tid + u * kLshThreads;
        if (x < dim) qreg[u] = batch_rows[long(e_nxt & kRowMask) * dim + x];
      }
      if (j + 2 < n) e_nn = sorted[j + 2];
    }

    for (int s = wib; s < size; s += kLshThreads / 64) {
      const float* key = keys_in_lds ? lkeys + s * dim : bucket_keys + long(s) * dim;
      // Euclidean: direct-difference form; cosine: 1 - q.k / sqrt((q.q)(k.k)), the three sums over the same
      // elements in the same order (so a key equal to the query is at distance exactly 0)
      double acc = 0.0, qq = 0.0, kk = 0.0;
      for (int x = lane; x < dim; x += 64) {
        const double qv = double(lq[x]), kv = double(key[x]);
        if (cosine) {
          acc += qv * kv;
          qq += qv * qv;
          kk += kv * kv;
        } else {
          const double diff = qv - kv;
          acc += diff * diff;
        }
      }
      acc = wave_sum(acc);
      if (cosine) acc = 1.0 - acc / sqrt(wave_sum(qq) * wave_sum(kk));
      if (lane == 0) d64[s] = cosine ? acc : sqrt(acc);
    }
    row_barrier();
    if (tid < 64) {
      ResolverBest best{__longlong_as_double(0x7ff0000000000000ll), 0x7fffffffffffffffll, -1};
      for (int s = lane; s < size; s += 64) {
        const double d = d64[s];
        if (d <= tau) best_take(best, d, lseq[s], s);
      }
      best_wave_reduce(best);
      if (lane == 0) {
        const int sb = best.src;
        s_best = sb;
        if (sb >= 0) {
          ++hits;
          const long long sq = lseq[sb];
          if (sq >= base_seq) ++inbatch;
          if (policy_lru && sb != tail) {
            const int p = lprev[sb], nx = lnext[sb];  // nx >= 0 because sb is not the tail
            if (p >= 0) lnext[p] = nx;
            lprev[nx] = p;
            lprev[sb] = tail;
            lnext[sb] = -1;
            lnext[tail] = sb;
            if (p < 0) head = nx;
            tail = sb;
          }
          hit_out[i] = 1;
          src_out[i] = sq >= base_seq ? c_total + int(sq - base_seq) : slot0 + sb;
          row_slot[i] = -1;
        } else {
          ++misses;
          int t;
          if (size < b) {
            t = size;
            s_size = size + 1;
          } else {
            t = head;
            head = lnext[t];
            if (head >= 0) lprev[head] = -1;
            if (head < 0) tail = -1;
            ++evictions;
          }
          lseq[t] = base_seq + i;
          lprev[t] = tail;
          lnext[t] = -1;
          if (tail >= 0) lnext[tail] = t;
          if (tail < 0) head = t;
          tail = t;
          ++inserts;
          hit_out[i] = 0;
          src_out[i] = -1;
          row_slot[i] = slot0 + t;
          s_slot = t;
        }
      }
    }
    row_barrier();
    if (s_best < 0) {  // the new key goes into its slot at once: later rows of the bucket compare against it
      const int t = s_slot;
      float* dst = bucket_keys + long(t) * dim;
      for (int x = tid; x < dim; x += kLshThreads) {
        const float v = lq[x];
        dst[x] = v;
        if (keys_in_lds) lkeys[t * dim + x] = v;
      }
    }
    row_barrier();  // the new key is in place, and lq may be overwritten by the next row
    if (!more) break;
    e_cur = e_nxt;
    e_nxt = e_nn;
  }

  __syncthreads();
  const int size1 = s_size;
  for (int s = tid; s < size1; s += kLshThreads) {
    slot_seq[slot0 + s] = lseq[s];
    slot_next[slot0 + s] = lnext[s] >= 0 ? slot0 + lnext[s] : -1;
    slot_prev[slot0 + s] = lprev[s] >= 0 ? slot0 + lprev[s] : -1;
  }
  if (tid == 0) {
    bkt_size[code] = size1;
    bkt_head[code] = head >= 0 ? slot0 + head : -1;
    bkt_tail[code] = tail >= 0 ? slot0 + tail : -1;
    atomicAdd(&st->size, inserts - evictions);
    atomicAdd(&st->hits, (unsigned long long)hits);
    atomicAdd(&st->misses, (unsigned long long)misses);
    atomicAdd(&st->inserts, (unsigned long long)inserts);
    atomicAdd(&st->evictions, (unsigned long long)evictions);
    atomicAdd(&st->inbatch_hits, (unsigned long long)inbatch);
  }
}

// ---------------------------------------------------------------------------
// Calls with a handful of rows (n <= kSmallRows): the whole cache side of the bucketed cache in
// one launch of one block.  Rows in order; per row the code (one wave per hyperplane), the
// float64 distances to the keys of its bucket, the decision and the update of that bucket, all
// in device memory (the block is alone, a barrier orders its own writes and reads).  Rows that
// hit a key stored before the call are answered from the stored lists at the end, as
// probe_resolve_small_kernel does; hits on rows of the same call and misses are routed by the
// selection kernel.  Rows are read from the caller's buffer.  b <= kLshMaxBucket.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(1024) void lsh_small_kernel(
    const float* __restrict__ queries, int n, int b, int c_total, int dim, int k, int K, int n_bits,
    const float* __restrict__ planes, int policy_lru, long long base_seq, double tau, int cosine, float* srcs,
    long long* slot_seq, int* slot_next, int* slot_prev, int* bkt_size, int* bkt_head, int* bkt_tail, CacheState* st,
    const int64_t* __restrict__ val_ids, const float* __restrict__ val_d, const void* __restrict__ X,
    int corpus_kind, uint8_t* hit_out, int* src_out, int* row_slot, int* __restrict__ miss_list,
    int* __restrict__ miss_count, int64_t* __restrict__ out_ids, float* __restrict__ out_d) {
  __shared__ uint64_t keys[kLshMaxBucket];
  __shared__ double d64[kLshMaxBucket];
  __shared__ int cid[kLshMaxBucket];
  __shared__ int s_bits[kLshMaxBits];
  __shared__ int s_best, s_slot;
  const int tid = threadIdx.x, lane = tid & 63, wib = tid >> 6;
  for (int s = tid; s < b; s += 1024) keys[s] = pack_key(0.f, uint32_t(s));
  int hits = 0, misses = 0, inserts = 0, evictions = 0, inbatch = 0, M = 0;  // kept by thread 0

  for (int i = 0; i < n; ++i) {
    const float* q = queries + long(i) * dim;
    // code: wave w takes hyperplane w
    if (wib < n_bits) {
      double acc = 0.0;
      for (int x = lane; x < dim; x += 64) acc += double(q[x]) * double(planes[long(wib) * dim + x]);
      acc = wave_sum(acc);
      if (lane == 0) s_bits[wib] = acc >= 0.0 ? 1 << wib : 0;
    }
    __syncthreads();
    int code = 0;
    for (int w = 0; w < n_bits; ++w) code |= s_bits[w];
    const int slot0 = code * b;
    float* bucket_keys = srcs + long(slot0) * dim;
    const int size = bkt_size[code];
    block_candidate_distances<kDtypeF32, 16>(keys, size, q, bucket_keys, dim, d64, cid, tid,
                                             cosine ? kMetricCosine : kMetricL2);
    __syncthreads();
    if (tid < 64) {
      ResolverBest best{__longlong_as_double(0x7ff0000000000000ll), 0x7fffffffffffffffll, -1};
      for (int s = lane; s < size; s += 64) {
        const double d = d64[s];
        if (d <= tau) best_take(best, d, slot_seq[slot0 + s], s);
      }
      best_wave_reduce(best);
      if (lane == 0) {
        int head = bkt_head[code], tail = bkt_tail[code];
        const int sb = best.src;
        s_best = sb;
        if (sb >= 0) {
          const int t = slot0 + sb;
          ++hits;
          const long long sq = slot_seq[t];
          if (sq >= base_seq) ++inbatch;
          if (policy_lru && t != tail) {
            const int p = slot_prev[t], nx = slot_next[t];  // nx >= 0 because t is not the tail
            if (p >= 0) slot_next[p] = nx;
            slot_prev[nx] = p;
            slot_prev[t] = tail;
            slot_next[t] = -1;
            slot_next[tail] = t;
            if (p < 0) head = nx;
            tail = t;
          }
          hit_out[i] = 1;
          src_out[i] = sq >= base_seq ? c_total + int(sq - base_seq) : t;
          row_slot[i] = -1;
        } else {
          ++misses;
          int t;
          if (size < b) {
            t = slot0 + size;
            bkt_size[code] = size + 1;
          } else {
            t = head;
            head = slot_next[t];
            if (head >= 0) slot_prev[head] = -1;
            if (head < 0) tail = -1;
            ++evictions;
          }
          slot_seq[t] = base_seq + i;
          slot_prev[t] = tail;
          slot_next[t] = -1;
          if (tail >= 0) slot_next[tail] = t;
          if (tail < 0) head = t;
          tail = t;
          ++inserts;
          hit_out[i] = 0;
          src_out[i] = -1;
          row_slot[i] = t;
          miss_list[M++] = i;
          s_slot = t;
        }
        bkt_head[code] = head;
        bkt_tail[code] = tail;
      }
    }
    __syncthreads();
    if (s_best < 0) {
      float* dst = srcs + long(s_slot) * dim;
      for (int x = tid; x < dim; x += 1024) dst[x] = q[x];
    }
    __syncthreads();  // this row's key, links and counts are in place for the next row
  }
  if (tid == 0) {
    st->size += inserts - evictions;
    st->queries += (unsigned long long)n;
    st->hits += (unsigned long long)hits;
    st->misses += (unsigned long long)misses;
    st->inserts += (unsigned long long)inserts;
    st->evictions += (unsigned long long)evictions;
    st->inbatch_hits += (unsigned long long)inbatch;
    *miss_count = M;
  }
  // hits on keys stored before the call: the stored list, or (re-ranking factor above 1) the stored
  // documents nearest to the row's own query
  for (int i = 0; i < n; ++i) {
    if (!hit_out[i]) continue;
    const int s = src_out[i];
    if (s >= c_total) continue;
    if (K == k || X == nullptr) {
      for (int e = tid; e < k; e += 1024) {
        out_ids[long(i) * k + e] = val_ids[long(s) * K + e];
        if (out_d) out_d[long(i) * k + e] = val_d[long(s) * K + e];
      }
    } else {
      __syncthreads();
      block_rerank_stored_any<1024>(corpus_kind, val_ids + long(s) * K, K, k, queries + long(i) * dim, X, dim,
                                    out_ids + long(i) * k, out_d ? out_d + long(i) * k : nullptr, keys, d64, cid, tid);
    }
  }
}

// ---------------------------------------------------------------------------
// The rows that missed, in row order, and their number.  One block of 1024 threads, n <= 2^13.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(1024) void lsh_miss_list_kernel(const uint8_t* __restrict__ hit, int n,
                                                             int* __restrict__ miss_list,
                                                             int* __restrict__ miss_count, CacheState* st) {
  __shared__ int counts[1024];
  const int tid = threadIdx.x;
  constexpr int PER = (1 << kLshRowBits) / 1024;  // rows per thread
  int mine = 0;
  for (int r = 0; r < PER; ++r) {
    const int i = tid * PER + r;
    if (i < n && !hit[i]) ++mine;
  }
  counts[tid] = mine;
  __syncthreads();
  for (int off = 1; off < 1024; off <<= 1) {  // inclusive scan
    const int v = tid >= off ? counts[tid - off] : 0;
    __syncthreads();
    counts[tid] += v;
    __syncthreads();
  }
  int pos = counts[tid] - mine;
  for (int r = 0; r < PER; ++r) {
    const int i = tid * PER + r;
    if (i < n && !hit[i]) miss_list[pos++] = i;
  }
  if (tid == 1023) {
    *miss_count = counts[1023];
    st->queries += (unsigned long long)n;
  }
}

}  // namespace prox
