// The bucketed cache of Section 3.2: an L-bit code from the signs of the query's inner products
// with L hyperplane normals names a bucket; every bucket is a cache of capacity b with its own
// FIFO/LRU order, and a query is looked up (and on a miss stored) only in its bucket.
//
// Slots are laid out bucket by bucket: bucket g owns slots g*b .. g*b+b-1 and fills them in
// index order, so its live slots are always the first `size[g]`.  Buckets do not interact, so a
// batch is regrouped by code (keeping row order inside a code) and every bucket that occurs is
// walked by its own block, rows in order, exactly as lines 2-9 of Algorithm 1 prescribe for one
// cache; different buckets run side by side.  A bucket holds a few dozen keys, so the block
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
// Hash codes.  One wave per row: bit i of code[row] is 1 exactly when q . r_i >= 0, with the
// inner product accumulated in float64 (the sign is the decision here).
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void lsh_codes_kernel(const float* __restrict__ Q, int n, int dim,
                                                        const float* __restrict__ planes, int n_bits,
                                                        int* __restrict__ code) {
  const int lane = threadIdx.x & 63;
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= n) return;
  const float* q = Q + long(row) * dim;
  int c = 0;
  for (int b = 0; b < n_bits; ++b) {
    const float* r = planes + long(b) * dim;
    double acc = 0.0;
    for (int i = lane; i < dim; i += 64) acc += double(q[i]) * double(r[i]);
    acc = wave_sum(acc);
    if (acc >= 0.0) c |= 1 << b;
  }
  if (lane == 0) code[row] = c;
}

// ---------------------------------------------------------------------------
// Regroup the batch by code, rows of one code in row order: sorts (code, row) pairs.
// One block of 1024 threads; n <= 2^13.  sorted[j] = (code << 13) | row.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(1024) void lsh_group_kernel(const int* __restrict__ code, int n,
                                                         uint32_t* __restrict__ sorted) {
  __shared__ uint32_t keys[1 << kLshRowBits];
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
}

// ---------------------------------------------------------------------------
// One block per position of the regrouped batch; the block at the first row of a code walks
// that bucket's rows in order, the others return at once.
//
// Per row: float64 distance to each live key of the bucket, nearest key (ties: smaller seq),
// hit if within tau (LRU: the key moves to the back of the bucket's order); otherwise the row
// takes the bucket's next free slot or evicts the front of its order, and its vector is written
// into the slot.  Outputs per row as resolver_kernel: hit flag, answering source (slot, or
// c_total + j when the key was stored by row j of this call), slot taken.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void lsh_resolve_kernel(
    const uint32_t* __restrict__ sorted, int n, int b, int c_total, int dim, int policy_lru, long long base_seq,
    double tau, const float* batch_rows, float* srcs, long long* slot_seq, int* slot_next,
    int* slot_prev, int* bkt_size, int* bkt_head, int* bkt_tail, CacheState* st, uint8_t* __restrict__ hit_out,
    int* __restrict__ src_out, int* __restrict__ row_slot) {
  const int j0 = blockIdx.x;
  if (j0 >= n) return;
  const uint32_t first = sorted[j0];
  const int code = int(first >> kLshRowBits);
  if (j0 > 0 && int(sorted[j0 - 1] >> kLshRowBits) == code) return;

  __shared__ uint64_t keys[kLshMaxBucket];
  __shared__ double d64[kLshMaxBucket];
  __shared__ int cid[kLshMaxBucket];
  __shared__ int s_best;  // local index of the answering key, -1: miss
  __shared__ int s_size;  // live keys of the bucket (read by every thread for the distances)
  __shared__ int s_slot;  // slot the current row takes when it misses
  const int tid = threadIdx.x, lane = tid & 63;
  for (int s = tid; s < b; s += 256) keys[s] = pack_key(0.f, uint32_t(s));

  const int slot0 = code * b;
  float* bucket_keys = srcs + long(slot0) * dim;
  // the bucket's order is walked by thread 0 alone; head/tail are global slot ids
  int head = 0, tail = 0;
  int hits = 0, misses = 0, inserts = 0, evictions = 0, inbatch = 0;
  if (tid == 0) {
    s_size = bkt_size[code];
    head = bkt_head[code];
    tail = bkt_tail[code];
  }
  __syncthreads();

  for (int j = j0; j < n; ++j) {
    const uint32_t e = sorted[j];
    if (int(e >> kLshRowBits) != code) break;
    const int i = int(e & ((1u << kLshRowBits) - 1));
    const float* q = batch_rows + long(i) * dim;
    const int size = s_size;

    block_candidate_distances<kDtypeF32, 4>(keys, size, q, bucket_keys, dim, d64, cid, tid);
    __syncthreads();
    if (tid < 64) {
      ResolverBest best{__longlong_as_double(0x7ff0000000000000ll), 0x7fffffffffffffffll, -1};
      for (int s = lane; s < size; s += 64) {
        const double d = d64[s];
        if (d <= tau) best_take(best, d, slot_seq[slot0 + s], s);
      }
      best_wave_reduce(best);
      if (lane == 0) {
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
            s_size = size + 1;
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
          s_slot = t;
        }
      }
    }
    __syncthreads();
    if (s_best < 0) {  // the new key goes into its slot at once: later rows of the bucket compare against it
      float* dst = srcs + long(s_slot) * dim;
      for (int x = tid; x < dim; x += 256) dst[x] = q[x];
    }
    __syncthreads();  // the seq and the new key are visible to the whole block for the next row
  }
  if (tid == 0) {
    bkt_size[code] = s_size;
    bkt_head[code] = head;
    bkt_tail[code] = tail;
    atomicAdd(&st->size, inserts - evictions);
    atomicAdd(&st->hits, (unsigned long long)hits);
    atomicAdd(&st->misses, (unsigned long long)misses);
    atomicAdd(&st->inserts, (unsigned long long)inserts);
    atomicAdd(&st->evictions, (unsigned long long)evictions);
    atomicAdd(&st->inbatch_hits, (unsigned long long)inbatch);
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
