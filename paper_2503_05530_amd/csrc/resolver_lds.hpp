// The order-preserving resolver (Algorithm 1 after the distances: nearest key, tolerance test,
// eviction, insertion; rows in order) with its
// sequential state in LDS.  Same inputs, outputs and decisions as resolver_kernel.
//
// Walking thousands of rows one after the other, every dependent memory access is
// on the critical path: a microsecond in global memory, some sixty nanoseconds in
// LDS.  This kernel therefore keeps the eviction order in a form whose updates need
// no dependent reads at all:
//
//   * The order is a queue of slot numbers in LDS, oldest use first.  Every use of a
//     slot (its insertion; under LRU also every hit on it, Section 3.3.2) appends the
//     slot to the queue and notes the position in qpos[slot].  An entry is current
//     iff qpos[queue[j]] == j; older entries of a slot that was used again are stale
//     and skipped.  The next victim is the first current entry, which is exactly the
//     least recently used (FIFO: first inserted) slot.
//   * The walking wave holds the next 64 queue entries in registers (one per lane)
//     with a mask of those still current.  A hit clears the bit of the slot it
//     touched with one compare; an eviction takes the lowest set bit.  The window is
//     refilled 64 entries at a time, so a miss costs no LDS round trip either.
//
// The linked list in global memory stays the representation between calls.  At entry
// the block turns it into the queue by list ranking (pointer jumping, log2(size)
// rounds over packed (next, distance-to-tail) words); at exit it compacts the current
// queue entries and writes the links back.
//
// Besides the order the LDS state holds "which row of this batch overwrote slot t"
// (-1: none), "which slot row j took" and "which source answered row j" (none: 0xffff),
// all 16 bits wide.  The walk itself issues no access to global memory on its usual
// paths (a store would be waited for at the next loop merge, a microsecond each
// time); flags, sources and the list of missing rows are written out at the end.
//
// Rows are taken in chunks of 64.  While the first wave resolves chunk k, the other
// waves stage chunk k+1: every row's candidate count and its first
// kStageCands candidates go to LDS, so that the walk touches global memory only
// for rows with longer lists.  A short loop handles the two common row kinds:
//   * runs of consecutive rows that miss whatever the state (no candidate, or a
//     single one beyond tau): their victims are the next current window entries,
//     one lane each does the bookkeeping of one row;
//   * one candidate within tau: a hit iff that source is live (one or two LDS reads).
// Rows with several candidates leave the short loop: one lane per candidate; the
// usual outcome (none or exactly one live candidate within tau) needs no reduction.
//
// One wave issues at most one instruction every four cycles, so after the memory
// waits are gone the instruction count per row is what is left to pay for; the loop
// state is kept in scalar registers for that reason (see the notes at `uniform`).
#pragma once

#include <type_traits>

#include "cache_kernels.hpp"

namespace prox {

constexpr int kStageCands = 8;
constexpr int kResolverThreads = 1024;
constexpr int kRankPerThread = 20;  // list-ranking results one thread carries over the buffer switch

struct ResolverChunk {
  int cnt[64];
  int src[64][kStageCands];
  double d[64][kStageCands];
};

constexpr size_t kResolverStaticLds = 2 * sizeof(ResolverChunk) + 256;

// A batch may be resolved in several launches, each over a range of rows (the probe of later rows then runs
// beside the walk of earlier ones, and the dense probe rows need to exist for one range at a time only).
// Between the launches the LDS state lives in device memory as it is (an image of the dynamic LDS) together
// with the walk's scalars; the linked list is read by the first launch and rewritten by the last.
struct ResolverCarry {
  int size, qnext, qtail, hits, evictions, inbatch, dense, M;
};

// Dynamic LDS of the kernel: queue [c + n], qpos [c], row-of-slot [c], slot-of-row [n], source-of-row [n],
// 16 bits each; the list ranking at entry uses the same memory as two buffers of c packed words.
__host__ __device__ inline size_t resolver_lds_bytes(size_t c, size_t n) {
  const size_t state = 2 * (c + n) + 2 * c + 2 * c + 2 * n + 2 * n;
  const size_t rank = 8 * c;
  return ((state > rank ? state : rank) + 15) & ~size_t(15);
}
// Can the kernel hold this cache and batch?  (16-bit positions; ranking results per thread.)
inline bool resolver_lds_fits(size_t c, size_t n, size_t lds_max) {
  return c >= 1 && c + n <= 65534 && c <= size_t(kResolverThreads) * kRankPerThread &&
         resolver_lds_bytes(c, n) <= lds_max;
}

// Exclusive prefix sum of one int per thread over the block (all threads call it; `wave_total`
// holds one int per wave and may be reused after the next barrier).
__device__ __forceinline__ int block_exclusive_sum(int mine, int* wave_total, int lane, int wib) {
  int incl = mine;
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    const int o = __shfl_up(incl, off, kWave);
    if (lane >= off) incl += o;
  }
  __syncthreads();  // earlier readers of wave_total are done
  if (lane == 63) wave_total[wib] = incl;
  __syncthreads();
  int at = incl - mine;
  for (int w = 0; w < wib; ++w) at += wave_total[w];
  return at;
}

__global__ __launch_bounds__(kResolverThreads) void resolver_lds_kernel(
    int n, int c, int dim, int policy_lru, long long base_seq, double tau, int cosine, CacheState* __restrict__ st,
    long long* slot_seq, int* slot_next, int* slot_prev, const int* __restrict__ cand_cnt,
    const int* __restrict__ cand_src, const double* __restrict__ cand_d, int cap, const float* __restrict__ D32,
    long ldD, const float* __restrict__ srcs, const float* __restrict__ srcnrm, uint8_t* __restrict__ hit_out,
    int* __restrict__ src_out, int* __restrict__ row_slot, int* __restrict__ miss_list,
    int* __restrict__ miss_count, int row_begin, int row_end, int first, int last, int* __restrict__ image,
    ResolverCarry* __restrict__ carry) {
  // rows row_begin .. row_end - 1 (row_begin a multiple of 64); D32 holds the dense probe rows of this range,
  // row i at D32 + (i - row_begin) * ldD
  extern __shared__ int lds_raw[];
  __shared__ ResolverChunk chunk[2];
  __shared__ int wave_total[kResolverThreads / 64];
  unsigned short* queue = reinterpret_cast<unsigned short*>(lds_raw);  // [c + n]
  unsigned short* qpos = queue + (c + n);                              // [c]
  short* lrow = reinterpret_cast<short*>(qpos + c);                    // [c]
  unsigned short* lslot = reinterpret_cast<unsigned short*>(lrow + c); // [n]
  unsigned short* lsrc = lslot + n;                                    // [n]
  constexpr unsigned kNone = 0xffffu;
  const int tid = threadIdx.x, lane = tid & 63, wib = tid >> 6;
  constexpr int NT = kResolverThreads;

  auto stage_chunk = [&](int i0, ResolverChunk& ch, int t, int nt) {
    for (int e = t; e < 64 * kStageCands; e += nt) {
      const int r = e / kStageCands, p = e % kStageCands;
      const int i = i0 + r;
      // (count and entry are fetched side by side, not the entry after the count: beside a probe that keeps the
      // memory system busy a dependent pair of loads takes about as long as the walk of a chunk; the entries
      // exist in memory whatever the count, kStageCands <= cap)
      const bool real = i < row_end;
      const int cn = real ? cand_cnt[i] : -1;  // rows past the end: neither empty nor a list
      const int sv = real ? cand_src[long(i) * cap + p] : 0;
      const double dv = real ? cand_d[long(i) * cap + p] : 0.0;
      if (p == 0) ch.cnt[r] = cn;
      if (cn <= cap && p < cn) {
        ch.src[r][p] = sv;
        ch.d[r][p] = dv;
      }
    }
  };

  // ---- the eviction order: linked list -> queue (position = size - 1 - distance to the tail) ----
  const int size0 = __builtin_amdgcn_readfirstlane(st->size);
  const int image_words = int(resolver_lds_bytes(size_t(c), size_t(n)) / 4);
  if (first) {
    unsigned* from = reinterpret_cast<unsigned*>(lds_raw);  // packed: next slot << 16 | distance to the tail so far
    unsigned* to = from + c;
    for (int s = tid; s < size0; s += NT) {
      const int nx = slot_next[s];
      from[s] = nx < 0 ? (kNone << 16) : (unsigned(nx) << 16 | 1u);
    }
    __syncthreads();
    for (int span = 1; span < size0; span <<= 1) {
      for (int s = tid; s < size0; s += NT) {
        unsigned a = from[s];
        const unsigned nx = a >> 16;
        if (nx != kNone) {
          const unsigned b = from[nx];
          a = (b & 0xffff0000u) | ((a & 0xffffu) + (b & 0xffffu));
        }
        to[s] = a;
      }
      __syncthreads();
      unsigned* t = from;
      from = to;
      to = t;
    }
    int dist[kRankPerThread];
#pragma unroll
    for (int j = 0; j < kRankPerThread; ++j) {
      const int s = tid + NT * j;
      dist[j] = s < size0 ? int(from[s] & 0xffffu) : 0;
    }
    __syncthreads();  // the ranking buffers are dead from here on; the state arrays take their place
#pragma unroll
    for (int j = 0; j < kRankPerThread; ++j) {
      const int s = tid + NT * j;
      if (s < size0) {
        const int pos = size0 - 1 - dist[j];
        queue[pos] = (unsigned short)s;
        qpos[s] = (unsigned short)pos;
      }
    }
  }
  if (first) {
    for (int s = tid; s < c; s += NT) lrow[s] = -1;
    for (int i = tid; i < n; i += NT) lslot[i] = (unsigned short)kNone;
  } else {
    for (int w = tid; w < image_words; w += NT) lds_raw[w] = image[w];
  }
  stage_chunk(row_begin, chunk[0], tid, NT);
  __syncthreads();

  // walked by the first wave only
  // (a later launch of the batch takes the scalars up where the one before left them; the window is loaded
  // again from the position it was last loaded from: which of its entries are still current follows from qpos)
  const bool resume = !first;
  int size = resume ? __builtin_amdgcn_readfirstlane(carry->size) : size0;
  int qnext = resume ? __builtin_amdgcn_readfirstlane(carry->qnext) : 0;       // queue positions: next one the window has not seen,
  int qtail = resume ? __builtin_amdgcn_readfirstlane(carry->qtail) : size0;   // end
  int qwin = qnext;             // where the window in registers was loaded from
  int wslot = int(kNone);       // window: this lane's queue entry
  unsigned long long wmask = 0; //         lanes whose entry is still current and not taken
  // counters of this batch; every miss inserts, so misses and insertions both equal M
  int hits = resume ? __builtin_amdgcn_readfirstlane(carry->hits) : 0;
  int evictions = resume ? __builtin_amdgcn_readfirstlane(carry->evictions) : 0;
  int inbatch = resume ? __builtin_amdgcn_readfirstlane(carry->inbatch) : 0;
  int dense = resume ? __builtin_amdgcn_readfirstlane(carry->dense) : 0;
  int M = resume ? __builtin_amdgcn_readfirstlane(carry->M) : 0;
  const double kInf = __longlong_as_double(0x7ff0000000000000ll);
  const int ck_begin = row_begin / 64, ck_end = (row_end + 63) / 64;

  auto window_load = [&]() {
    qwin = qnext;
    const int pos = qnext + lane;
    int sl = int(kNone);
    bool cur = false;
    if (pos < qtail) {
      sl = queue[pos];
      cur = qpos[sl] == pos;
    }
    wslot = sl;
    wmask = __ballot(cur);
    qnext = qnext + 64 < qtail ? qnext + 64 : qtail;
  };
  // slot t was used just now: it goes to the back of the order
  auto touch = [&](int t) {
    if (lane == 0) {
      queue[qtail] = (unsigned short)t;
      qpos[t] = (unsigned short)qtail;
    }
    ++qtail;
    wmask &= ~__ballot(wslot == t);  // an entry of t in the window is stale now
  };
  auto is_live = [&](int s) -> bool {
    if (s < c) return lrow[s] < 0;
    const unsigned t = lslot[s - c];
    return t != kNone && lrow[t] == s - c;
  };
  // The walking wave's control flow depends only on values every lane holds alike.  Values read
  // from LDS at a common address are such values, but the compiler cannot know; passing them
  // through readfirstlane keeps the loop state in scalar registers and the branches scalar.
  auto uniform = [](int v) { return __builtin_amdgcn_readfirstlane(v); };
  auto is_live_uniform = [&](int s) -> bool {
    if (s < c) return uniform(lrow[s]) < 0;
    const int t = uniform(lslot[s - c]);
    return t != int(kNone) && uniform(lrow[t]) == s - c;
  };

  // a run of m consecutive rows from row i on that all miss
  auto miss_run = [&](int i, int m) {
    int done = 0;
    if (size < c) {
      // free slots are taken in index order
      done = m < c - size ? m : c - size;
      if (lane < done) {
        const int t = size + lane;
        lrow[t] = short(i + lane);
        lslot[i + lane] = (unsigned short)t;
        queue[qtail + lane] = (unsigned short)t;
        qpos[t] = (unsigned short)(qtail + lane);
      }
      qtail += done;
      size += done;
    }
    // the other victims are the next current entries of the order; window lane number `rank` among
    // the current ones serves row i + done + rank
    while (done < m) {
      while (wmask == 0 && qnext < qtail) window_load();
      const int avail = __popcll(wmask);
      if (avail == 0) break;  // no live key: cannot happen with size == c >= 1
      const int g = m - done < avail ? m - done : avail;
      const int rank = __builtin_amdgcn_mbcnt_hi(unsigned(wmask >> 32), __builtin_amdgcn_mbcnt_lo(unsigned(wmask), 0u));
      const bool chosen = ((wmask >> lane) & 1ull) && rank < g;
      if (chosen) {
        const int t = wslot, row = i + done + rank;
        lrow[t] = short(row);
        lslot[row] = (unsigned short)t;
        queue[qtail + rank] = (unsigned short)t;
        qpos[t] = (unsigned short)(qtail + rank);
      }
      wmask &= ~__ballot(chosen);
      qtail += g;
      done += g;
      evictions += g;
    }
    M += m;
  };
  // row i hits on source s
  auto hit_row = [&](int s) {
    ++hits;
    if (s >= c) ++inbatch;
    if (policy_lru) touch(s < c ? s : uniform(lslot[s - c]));  // also when it is at the back already
  };

  for (int ck = ck_begin; ck < ck_end; ++ck) {
    const int i0 = ck * 64;
    // (the wave number as a scalar: the compiler then sees that whole waves take one side, and
    // the walk's state does not pass through the join of a divergent branch)
    if (__builtin_amdgcn_readfirstlane(wib) != 0) {
      if (ck + 1 < ck_end) stage_chunk(i0 + 64, chunk[(ck + 1 - ck_begin) & 1], tid - 64, NT - 64);
    } else {
      const ResolverChunk& ch = chunk[(ck - ck_begin) & 1];
      const int rows = row_end - i0 < 64 ? row_end - i0 : 64;
      const int my_cnt = ch.cnt[lane];
      int my_s0 = -1;
      bool my_within = false;
      if (my_cnt == 1) {
        my_s0 = ch.src[lane][0];
        my_within = ch.d[lane][0] <= tau;
      }
      // rows that miss whatever the state: no candidate, or a single one beyond tau
      const unsigned long long miss_mask = __ballot(my_cnt == 0 || (my_cnt == 1 && !my_within));
      // rows with one candidate within tau: a hit iff that source is live
      const unsigned long long one_mask = __ballot(my_cnt == 1 && my_within);
      int my_src = int(kNone);
      int r = 0;
      while (r < rows) {
        // ---- the short loop: runs of sure misses and single-candidate rows ----
        while (r < rows) {
          const unsigned long long mm = miss_mask >> r;
          if (mm & 1ull) {
            const unsigned long long rest = ~mm;  // rows past the end are in neither mask: a run ends there
            const int m = rest ? __ffsll((long long)rest) - 1 : 64;
            miss_run(i0 + r, m);
            r += m;
            continue;
          }
          if (!((one_mask >> r) & 1ull)) break;
          // r is wave-uniform: readlane moves the staged value without another trip through LDS
          const int s = __builtin_amdgcn_readlane(my_s0, r);
          if (is_live_uniform(s)) {
            hit_row(s);
            if (lane == r) my_src = s;
          } else {
            miss_run(i0 + r, 1);
          }
          ++r;
        }
        if (r >= rows) break;

        // ---- a row with several candidates ----
        const int i = i0 + r;
        const int cnt = __builtin_amdgcn_readlane(my_cnt, r);
        int best_src = -1;
        if (cnt <= cap) {
          // One lane per candidate.  The staged part of the list is read from LDS; longer lists come
          // from global memory.  (Two instances of the code rather than one that picks the address:
          // a load whose address may be in either memory goes through the slower generic path.)
          auto decide = [&](auto staged_tag) {
            constexpr bool kStaged = decltype(staged_tag)::value;
            // candidate p of this row: is it live and within tau?
            auto within = [&](int p, int& s, double& d) {
              if (kStaged) {
                s = ch.src[r][p];
                d = ch.d[r][p];
              } else {
                s = cand_src[long(i) * cap + p];
                d = cand_d[long(i) * cap + p];
              }
              return is_live(s) && d <= tau;
            };
            int my_ok_s = -1, total = 0;
            for (int p0 = 0; p0 < cnt; p0 += 64) {
              int s;
              double d;
              const bool ok = p0 + lane < cnt && within(p0 + lane, s, d);
              if (ok) my_ok_s = s;
              total += __popcll(__ballot(ok));
            }
            if (total == 1) {
              // the usual outcome: nothing to compare
              best_src = __builtin_amdgcn_readlane(my_ok_s, __ffsll((long long)__ballot(my_ok_s >= 0)) - 1);
            } else if (total >= 2) {
              // nearest wins, equal distances go to the older key: a key untouched in this batch still
              // carries its own seq, a row of this batch has base_seq + row
              ResolverBest best{kInf, 0x7fffffffffffffffll, -1};
              for (int p0 = 0; p0 < cnt; p0 += 64) {
                int s;
                double d;
                if (p0 + lane < cnt && within(p0 + lane, s, d))
                  best_take(best, d, s < c ? slot_seq[s] : base_seq + (s - c), s);
              }
              best_wave_reduce(best);
              best_src = best.src;
            }
          };
          if (cnt <= kStageCands)
            decide(std::true_type{});
          else
            decide(std::false_type{});
        } else {
          ++dense;
          ResolverBest best{kInf, 0x7fffffffffffffffll, -1};
          const float qn = srcnrm[c + i];
          const float* row = D32 + long(i - row_begin) * ldD;
          float mn = 3.4e38f, snmax = 0.f;
          for (int t = lane; t < size; t += 64) {
            const int s = lrow[t] >= 0 ? c + lrow[t] : t;
            mn = fminf(mn, probe_value(row[s], qn, srcnrm[s], cosine));
            snmax = fmaxf(snmax, srcnrm[s]);
          }
#pragma unroll
          for (int mm = 32; mm >= 1; mm >>= 1) {
            mn = fminf(mn, __shfl_xor(mn, mm, kWave));
            snmax = fmaxf(snmax, __shfl_xor(snmax, mm, kWave));
          }
          const float slack = dense_slack(qn, snmax, dim, cosine);
          if (mn <= prefilter_bound(tau, qn, snmax, dim, cosine) + slack) {
            const float near = mn + slack;
            for (int t0 = 0; t0 < size; t0 += 64) {
              const int t = t0 + lane;
              int s = -1;
              bool is_near = false;
              if (t < size) {
                s = lrow[t] >= 0 ? c + lrow[t] : t;
                is_near = probe_value(row[s], qn, srcnrm[s], cosine) <= near;
              }
              unsigned long long mask = __ballot(is_near);
              while (mask) {
                const int b = __ffsll((long long)mask) - 1;
                mask &= mask - 1;
                const int sb = __shfl(s, b, kWave);
                const long long sqb = sb < c ? slot_seq[sb] : base_seq + (sb - c);
                const double d = wave_keydist64(srcs + long(c + i) * dim, srcs + long(sb) * dim, dim, lane, cosine);
                if (d <= tau) best_take(best, d, sqb, sb);
              }
            }
          }
          best_src = best.src;
        }
        best_src = uniform(best_src);
        if (best_src >= 0) {
          hit_row(best_src);
          if (lane == r) my_src = best_src;
        } else {
          miss_run(i, 1);
        }
        ++r;
      }
      if (lane < rows) lsrc[i0 + lane] = (unsigned short)my_src;
    }
    __syncthreads();
  }

  // the walking wave hands the scalars the whole block needs through LDS
  __shared__ int walk_out[2];
  if (tid == 0) {
    walk_out[0] = size;
    walk_out[1] = qtail;
    if (last) {
      st->queries += (unsigned long long)n;
      st->hits += (unsigned long long)hits;
      st->misses += (unsigned long long)M;
      st->inserts += (unsigned long long)M;
      st->evictions += (unsigned long long)evictions;
      st->inbatch_hits += (unsigned long long)inbatch;
      st->dense_resolves += (unsigned long long)dense;
      *miss_count = M;
    } else {
      const ResolverCarry out{size, wmask ? qwin : qnext, qtail, hits, evictions, inbatch, dense, M};
      *carry = out;
    }
  }
  __syncthreads();
  if (!last) {
    for (int w = tid; w < image_words; w += NT) image[w] = lds_raw[w];
    return;
  }
  const int size_end = walk_out[0], q_end = walk_out[1];
  for (int s = tid; s < c; s += NT)
    if (lrow[s] >= 0) slot_seq[s] = base_seq + lrow[s];
  for (int i = tid; i < n; i += NT) {
    const unsigned t = lslot[i], src = lsrc[i];
    row_slot[i] = t == kNone ? -1 : int(t);
    hit_out[i] = uint8_t(src != kNone);
    src_out[i] = src == kNone ? -1 : int(src);
  }
  // the rows that missed, in row order: exactly those that took a slot
  {
    const int per = (n + NT - 1) / NT;
    const int a0 = tid * per < n ? tid * per : n;
    const int a1 = a0 + per < n ? a0 + per : n;
    int mine = 0;
    for (int i = a0; i < a1; ++i) mine += lslot[i] != kNone ? 1 : 0;
    int at = block_exclusive_sum(mine, wave_total, lane, wib);
    for (int i = a0; i < a1; ++i)
      if (lslot[i] != kNone) miss_list[at++] = i;
  }
  __syncthreads();  // lrow is free now: it takes the compacted order

  // ---- queue -> linked list: the current entries, in queue order ----
  unsigned short* order = reinterpret_cast<unsigned short*>(lrow);  // [size_end]
  const int per = (q_end + NT - 1) / NT;
  const int j0 = tid * per < q_end ? tid * per : q_end;
  const int j1 = j0 + per < q_end ? j0 + per : q_end;
  int mine = 0;
  for (int j = j0; j < j1; ++j) mine += qpos[queue[j]] == j ? 1 : 0;
  int at = block_exclusive_sum(mine, wave_total, lane, wib);
  for (int j = j0; j < j1; ++j) {
    const unsigned short s = queue[j];
    if (qpos[s] == j) order[at++] = s;
  }
  __syncthreads();
  for (int p = tid; p < size_end; p += NT) {
    const int s = order[p];
    slot_next[s] = p + 1 < size_end ? int(order[p + 1]) : -1;
    slot_prev[s] = p > 0 ? int(order[p - 1]) : -1;
  }
  if (tid == 0) {
    st->size = size_end;
    st->head = size_end > 0 ? int(order[0]) : -1;
    st->tail = size_end > 0 ? int(order[size_end - 1]) : -1;
  }
}

}  // namespace prox
