// The second ranking of queries whose float32 candidate list could not be proven long enough
// (see block_list_sufficient in select_kernels.hpp), for the batched scan, which keeps no dense scores:
// the corpus is scored again for just those queries, every row at or below the query's bound t_k + E is
// collected, and the exact k nearest are taken from the collected rows in float64.  Both kernels are
// enqueued after every batched ranking and return at once when no query was noted, which is the usual case.
#pragma once

#include "scan_kernels.hpp"
#include "select_kernels.hpp"

namespace prox {

// The largest squared row length, for the error bound.  nrm holds the squared lengths.
__global__ __launch_bounds__(256) void max_norm_kernel(const float* __restrict__ nrm, long n_rows,
                                                       SlackState* __restrict__ slack) {
  float m = 0.f;
  const long stride = long(gridDim.x) * 256;
  for (long r = long(blockIdx.x) * 256 + threadIdx.x; r < n_rows; r += stride) m = fmaxf(m, nrm[r]);
#pragma unroll
  for (int s = 32; s >= 1; s >>= 1) m = fmaxf(m, __shfl_xor(m, s, kWave));
  if ((threadIdx.x & 63) == 0) atomicMax(&slack->xmax2_bits, __float_as_uint(m));
}

// Zeroes the whole state (a kernel rather than a memset so that callers may capture the launch).
__global__ void slack_reset_kernel(SlackState* __restrict__ slack) {
  int* w = reinterpret_cast<int*>(slack);
  for (int i = threadIdx.x; i < int(sizeof(SlackState) / sizeof(int)); i += blockDim.x) w[i] = 0;
}

// One wave per corpus row at a time; per noted query the float32 score of the row, kept when it is at most
// the query's bound.  redo.wide[f * kWideCap ..] receives the packed (score, row) keys of noted query f.
template <int DT>
__global__ __launch_bounds__(256) void redo_collect_kernel(const void* __restrict__ X, const float* __restrict__ xnrm,
                                                           long n_rows, int dim, const float* __restrict__ Qbase,
                                                           const int* __restrict__ qlist,
                                                           const SlackState* __restrict__ slack, RedoBuffers redo,
                                                           int cosine) {
  const int n = slack->redo_count;
  if (n == 0) return;
  constexpr int COLS = RowChunk<DT>::kCols;
  const int lane = threadIdx.x & 63;
  const long wave = long(blockIdx.x) * 4 + (threadIdx.x >> 6);
  const long n_waves = long(gridDim.x) * 4;
  for (long row = wave; row < n_rows; row += n_waves) {
    const float nr = xnrm[row];
    for (int f = 0; f < n; ++f) {
      const int m = redo.list[f];
      const float* q = Qbase + long(qlist ? qlist[m] : m) * dim;
      float acc = 0.f;
      for (int col = lane * COLS; col < dim; col += 64 * COLS) {
        RowChunk<DT> x;
        x.load(X, row * long(dim) + col);
        acc += x.dot(q + col);
      }
      acc = wave_sum(acc);
      if (lane == 0) {
        const float sc = row_score(nr, acc, cosine);
        if (sc <= redo.thr[f]) {
          const int pos = atomicAdd(&redo.cnt[f], 1);
          if (pos < kWideCap) redo.wide[long(f) * kWideCap + pos] = pack_key(sc, uint32_t(row));
        }
      }
    }
  }
}

// One block per noted query: exact k nearest of the collected rows into the query's result row.  The last
// block to finish clears the list of noted queries for the next call.  Grid: one block per row of the call.
template <int DT>
__global__ __launch_bounds__(1024) void redo_rank_kernel(const void* __restrict__ X, int dim,
                                                         const float* __restrict__ Qbase,
                                                         const int* __restrict__ qlist, SlackState* slack,
                                                         RedoBuffers redo, int k, int64_t* __restrict__ res_ids,
                                                         float* __restrict__ res_dists, int metric) {
  const int n = slack->redo_count;
  if (n == 0) return;
  const int f = blockIdx.x, tid = threadIdx.x;
  __shared__ uint64_t list[kWideCap];
  __shared__ double d64[256];
  __shared__ int cid[256];
  __shared__ double best_d[2][256];
  __shared__ int best_id[2][256];
  if (f < n) {
    const int cnt = redo.cnt[f];
    const int m = redo.list[f];
    const int qrow = qlist ? qlist[m] : m;
    if (cnt > kWideCap) {
      if (tid == 0) atomicAdd(&slack->unresolved, 1ull);   // the float64 ranking of the kp candidates stands
    } else {
      for (int i = tid; i < cnt; i += 1024) list[i] = redo.wide[long(f) * kWideCap + i];
      __syncthreads();
      int64_t* o_ids = res_ids + long(qrow) * k;
      float* o_d = res_dists + long(qrow) * k;
      block_exact_topk_of_rows<DT, 1024>(list, cnt, k, Qbase + long(qrow) * dim, X, dim, metric, d64, cid, best_d,
                                         best_id, tid, [&](int r, int64_t id, double d) {
                                           o_ids[r] = id;
                                           o_d[r] = float(d);
                                         });
    }
    __syncthreads();
    if (tid == 0) redo.cnt[f] = 0;
  }
  // every block has read the count by now; the last one to get here resets it
  if (tid == 0) {
    __threadfence();
    if (atomicAdd(&slack->redo_ticket, 1) == int(gridDim.x) - 1) {
      slack->redo_count = 0;
      slack->redo_ticket = 0;
    }
  }
}

}  // namespace prox
