// The order-preserving resolver (Algorithm 1 after the distances: nearest key, tolerance test,
// eviction, insertion; rows in order) with its
// sequential state in LDS.  Same inputs, outputs and decisions as resolver_kernel.
//
// Walking thousands of rows one after the other, every dependent access to global
// memory costs a microsecond.  Here the block copies the eviction order (next/prev
// per slot) into LDS, keeps "which row of this batch overwrote slot t" (-1: none)
// and "which slot row j took" (-1: none) there as well, lets its first wave walk
// the rows, and writes the state back at the end.
//
// Rows are taken in chunks of 64.  While the first wave resolves chunk k, the other
// three waves stage chunk k+1: every row's candidate count and its first
// kStageCands candidates go to LDS, so that the walk touches global memory only
// for rows with longer lists.  Three row kinds get a short path:
//   * runs of consecutive rows without any candidate all miss; their victims are the
//     next slots along the eviction order, which keep their relative order when they
//     are appended again, so a run costs one pointer chase plus a constant number of
//     link updates, and the per-row bookkeeping is done by one lane per row;
//   * one candidate: liveness and threshold test on registers and LDS;
//   * up to kStageCands candidates: one lane per candidate; the usual outcome (none
//     or exactly one live candidate within tau) needs no reduction.
// Needs (3c + n) * 4 bytes of dynamic LDS on top of the static staging buffers.
#pragma once

#include "cache_kernels.hpp"

namespace prox {

constexpr int kStageCands = 8;

struct ResolverChunk {
  int cnt[64];
  int src[64][kStageCands];
  double d[64][kStageCands];
};

constexpr size_t kResolverStaticLds = 2 * sizeof(ResolverChunk);

__global__ __launch_bounds__(256) void resolver_lds_kernel(
    int n, int c, int dim, int policy_lru, long long base_seq, double tau, CacheState* __restrict__ st,
    long long* slot_seq, int* slot_next, int* slot_prev, const int* __restrict__ cand_cnt,
    const int* __restrict__ cand_src, const double* __restrict__ cand_d, int cap, const float* __restrict__ D32,
    long ldD, const float* __restrict__ srcs, const float* __restrict__ srcnrm, uint8_t* __restrict__ hit_out,
    int* __restrict__ src_out, int* __restrict__ row_slot, int* __restrict__ miss_list,
    int* __restrict__ miss_count) {
  extern __shared__ int lds_state[];
  __shared__ ResolverChunk chunk[2];
  int* lnext = lds_state;          // [c]
  int* lprev = lds_state + c;      // [c]
  int* lrow = lds_state + 2 * c;   // [c]  row of this batch that overwrote the slot, -1 if none
  int* lslot = lds_state + 3 * c;  // [n]  slot taken by a row that missed, -1 otherwise
  const int tid = threadIdx.x, lane = tid & 63;

  auto stage_chunk = [&](int i0, ResolverChunk& ch, int t, int nt) {
    for (int e = t; e < 64 * kStageCands; e += nt) {
      const int r = e / kStageCands, p = e % kStageCands;
      const int i = i0 + r;
      const int cn = i < n ? cand_cnt[i] : -1;  // rows past the end: neither empty nor a list
      if (p == 0) ch.cnt[r] = cn;
      if (cn <= cap && p < cn) {
        ch.src[r][p] = cand_src[long(i) * cap + p];
        ch.d[r][p] = cand_d[long(i) * cap + p];
      }
    }
  };

  for (int s = tid; s < c; s += 256) {
    lnext[s] = slot_next[s];
    lprev[s] = slot_prev[s];
    lrow[s] = -1;
  }
  for (int i = tid; i < n; i += 256) lslot[i] = -1;
  stage_chunk(0, chunk[0], tid, 256);
  __syncthreads();

  int size = st->size, head = st->head, tail = st->tail;  // walked by the first wave only
  unsigned long long hits = 0, misses = 0, inserts = 0, evictions = 0, inbatch = 0, dense = 0;
  int M = 0;
  const double kInf = __longlong_as_double(0x7ff0000000000000ll);
  const int n_chunks = (n + 63) / 64;

  for (int ck = 0; ck < n_chunks; ++ck) {
    const int i0 = ck * 64;
    if (tid >= 64) {
      if (ck + 1 < n_chunks) stage_chunk(i0 + 64, chunk[(ck + 1) & 1], tid - 64, 192);
    } else {
      const ResolverChunk& ch = chunk[ck & 1];
      const int rows = n - i0 < 64 ? n - i0 : 64;
      const int my_cnt = ch.cnt[lane];
      int my_s0 = -1;
      double my_d0 = kInf;
      if (my_cnt >= 1 && my_cnt <= cap) {
        my_s0 = ch.src[lane][0];
        my_d0 = ch.d[lane][0];
      }
      const unsigned long long zero_mask = __ballot(my_cnt == 0);
      int my_hit = 0, my_src = -1;
      int r = 0;
      while (r < rows) {
        const int i = i0 + r;
        // r is wave-uniform: readlane moves the staged values without another trip through LDS
        const int cnt = __builtin_amdgcn_readlane(my_cnt, r);
        if (cnt == 0) {
          // a run of rows without candidates: all miss
          const unsigned long long rest = ~(zero_mask >> r);
          int m = rest ? __ffsll((long long)rest) - 1 : 64;
          if (size < c) {
            // free slots are taken in index order
            m = m < c - size ? m : c - size;
            if (lane < m) {
              const int t = size + lane;
              lrow[t] = i + lane;
              lprev[t] = lane == 0 ? tail : t - 1;
              lnext[t] = lane == m - 1 ? -1 : t + 1;
              lslot[i + lane] = t;
              miss_list[M + lane] = i + lane;
            }
            if (tail >= 0) {
              if (lane == 0) lnext[tail] = size;
            } else {
              head = size;
            }
            tail = size + m - 1;
            size += m;
            inserts += m;
          } else {
            // victims are the first m slots of the eviction order; appended again in the same
            // order they keep the links among themselves
            m = m < c ? m : c;
            int my_t = -1, cur = head;
            for (int j = 0; j < m; ++j) {
              if (lane == j) my_t = cur;
              cur = lnext[cur];
            }
            if (lane < m) {
              lrow[my_t] = i + lane;
              lslot[i + lane] = my_t;
              miss_list[M + lane] = i + lane;
            }
            if (m < c) {  // otherwise the whole order was replaced by itself
              const int t_last = __builtin_amdgcn_readlane(my_t, m - 1);
              if (lane == 0) {
                lprev[cur] = -1;
                lnext[tail] = head;
                lprev[head] = tail;
                lnext[t_last] = -1;
              }
              head = cur;
              tail = t_last;
            }
            evictions += m;
            inserts += m;
          }
          misses += m;
          M += m;
          r += m;
          continue;
        }

        int best_src = -1;
        if (cnt == 1) {
          const int s = __builtin_amdgcn_readlane(my_s0, r);
          const long long dbits = __double_as_longlong(my_d0);
          const unsigned dlo = unsigned(__builtin_amdgcn_readlane(int(dbits & 0xffffffffll), r));
          const unsigned dhi = unsigned(__builtin_amdgcn_readlane(int(dbits >> 32), r));
          const double d = __longlong_as_double((long long)((unsigned long long)dhi << 32 | dlo));
          bool live;
          if (s < c) {
            live = lrow[s] < 0;
          } else {
            const int t = lslot[s - c];
            live = t >= 0 && lrow[t] == s - c;
          }
          if (live && d <= tau) best_src = s;
        } else if (cnt <= cap) {
          // several candidates, one lane each: from LDS when the staged part holds them all
          const bool staged = cnt <= kStageCands;
          // candidate p of this row: is it live and within tau?
          auto within = [&](int p, int& s, double& d) {
            s = staged ? ch.src[r][p] : cand_src[long(i) * cap + p];
            d = staged ? ch.d[r][p] : cand_d[long(i) * cap + p];
            bool live;
            if (s < c) {
              live = lrow[s] < 0;
            } else {
              const int t = lslot[s - c];
              live = t >= 0 && lrow[t] == s - c;
            }
            return live && d <= tau;
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
            best_src = __shfl(my_ok_s, __ffsll((long long)__ballot(my_ok_s >= 0)) - 1, kWave);
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
        } else {
          ++dense;
          ResolverBest best{kInf, 0x7fffffffffffffffll, -1};
          const float qn = srcnrm[c + i];
          const float* row = D32 + long(i) * ldD;
          float mn = 3.4e38f, snmax = 0.f;
          for (int t = lane; t < size; t += 64) {
            const int s = lrow[t] >= 0 ? c + lrow[t] : t;
            mn = fminf(mn, row[s] + qn);
            snmax = fmaxf(snmax, srcnrm[s]);
          }
#pragma unroll
          for (int mm = 32; mm >= 1; mm >>= 1) {
            mn = fminf(mn, __shfl_xor(mn, mm, kWave));
            snmax = fmaxf(snmax, __shfl_xor(snmax, mm, kWave));
          }
          const float slack = 2e-4f * (qn + snmax);
          if (mn <= prefilter_bound(tau, qn, snmax) + slack) {
            const float near = mn + slack;
            for (int t0 = 0; t0 < size; t0 += 64) {
              const int t = t0 + lane;
              int s = -1;
              bool is_near = false;
              if (t < size) {
                s = lrow[t] >= 0 ? c + lrow[t] : t;
                is_near = row[s] + qn <= near;
              }
              unsigned long long mask = __ballot(is_near);
              while (mask) {
                const int b = __ffsll((long long)mask) - 1;
                mask &= mask - 1;
                const int sb = __shfl(s, b, kWave);
                const long long sqb = sb < c ? slot_seq[sb] : base_seq + (sb - c);
                const double d = wave_dist64(srcs + long(c + i) * dim, srcs + long(sb) * dim, dim, lane);
                if (d <= tau) best_take(best, d, sqb, sb);
              }
            }
          }
          best_src = best.src;
        }

        if (best_src >= 0) {
          ++hits;
          if (best_src >= c) ++inbatch;
          const int t = best_src < c ? best_src : lslot[best_src - c];
          if (policy_lru && t != tail) {
            const int p = lprev[t], nx = lnext[t];  // nx >= 0 because t is not the tail
            if (lane == 0) {
              if (p >= 0) lnext[p] = nx;
              lprev[nx] = p;
              lprev[t] = tail;
              lnext[t] = -1;
              lnext[tail] = t;
            }
            if (p < 0) head = nx;
            tail = t;
          }
          if (lane == r) {
            my_hit = 1;
            my_src = best_src;
          }
        } else {
          ++misses;
          int t;
          if (size < c) {
            t = size++;
          } else {
            t = head;
            head = lnext[t];
            if (lane == 0 && head >= 0) lprev[head] = -1;
            if (head < 0) tail = -1;
            ++evictions;
          }
          if (lane == 0) {
            lrow[t] = i;
            lprev[t] = tail;
            lnext[t] = -1;
            if (tail >= 0) lnext[tail] = t;
            lslot[i] = t;
            miss_list[M] = i;
          }
          if (tail < 0) head = t;
          tail = t;
          ++inserts;
          ++M;
        }
        ++r;
      }
      if (lane < rows) {
        hit_out[i0 + lane] = uint8_t(my_hit);
        src_out[i0 + lane] = my_src;
      }
    }
    __syncthreads();
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
    st->dense_resolves += dense;
    *miss_count = M;
  }
  for (int s = tid; s < c; s += 256) {
    slot_next[s] = lnext[s];
    slot_prev[s] = lprev[s];
    if (lrow[s] >= 0) slot_seq[s] = base_seq + lrow[s];
  }
  for (int i = tid; i < n; i += 256) row_slot[i] = lslot[i];
}

}  // namespace prox
