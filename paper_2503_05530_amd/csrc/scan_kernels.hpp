// Distance kernels: squared row norms and the query-by-rows score contraction.
//
// A "score" of query q against stored row x is  |x|^2 - 2 q.x ; adding |q|^2
// gives the squared Euclidean distance |q - x|^2 (the distance of Algorithm 1's
// first line and of the nearest-neighbour search in Section 2.2).  For a fixed
// query the score orders rows exactly as the distance does.
//
// The same kernels serve the corpus scan (rows = documents) and the cache probe
// (rows = cached keys followed by the rows of the current batch).
#pragma once

#include "device_utils.hpp"

namespace prox {

// ---------------------------------------------------------------------------
// Squared L2 norm of every row.  One wave per row, 16-byte loads per lane.
// HBM-bound: reads the matrix once, writes 4 bytes per row.
// ---------------------------------------------------------------------------
template <int DT>
__global__ __launch_bounds__(256) void row_norms_kernel(const void* __restrict__ X, long n_rows, int dim,
                                                        float* __restrict__ nrm) {
  const int lane = threadIdx.x & 63;
  const long wave = long(blockIdx.x) * 4 + (threadIdx.x >> 6);
  const long n_waves = long(gridDim.x) * 4;
  for (long row = wave; row < n_rows; row += n_waves) {
    float acc = 0.f;
    if (DT == kDtypeF32) {
      const float4* p = reinterpret_cast<const float4*>(static_cast<const float*>(X) + row * dim);
      for (int c = lane; c < dim / 4; c += 64) {
        const float4 v = p[c];
        acc += v.x * v.x + v.y * v.y + v.z * v.z + v.w * v.w;
      }
    } else {
      const uint4* p = reinterpret_cast<const uint4*>(static_cast<const uint16_t*>(X) + row * dim);
      for (int c = lane; c < dim / 8; c += 64) {
        const uint4 v = p[c];
        const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const float lo = __uint_as_float(w[i] << 16);
          const float hi = __uint_as_float(w[i] & 0xffff0000u);
          acc += lo * lo + hi * hi;
        }
      }
    }
    acc = wave_sum(acc);
    if (lane == 0) nrm[row] = acc;
  }
}

// ---------------------------------------------------------------------------
// Streaming scores for a few queries (MQ <= 8): the HBM-bound form of the scan.
//
// Each wave owns blocks of 64 consecutive rows.  Per step it loads RPI rows,
// every lane taking 16 contiguous bytes per 1 KiB (f32: 256 columns, bf16: 512
// columns) segment of a row, so a row is read by fully coalesced 1 KiB wave
// loads; the query values for a lane's columns stay in registers.  Partial dot
// products are summed across the wave with the transposed reduction, parked
// in LDS, and written out as one coalesced 256-byte store per query per block.
//
// Queries are rows qlist[m_begin + m] of Qbase (qlist == nullptr: row m_begin+m);
// only the first *m_count_ptr list entries exist (m_count_ptr == nullptr: m_limit).
// ONCE = true marks the rows as read-once (the corpus); false keeps them cacheable (cached keys).
// Output S[m * ldS + (row - row_begin)] for m < MQ; queries past the count give
// unspecified values in their rows of S and are never read.
// ---------------------------------------------------------------------------
template <int DT>
struct RowChunk;  // the 16 bytes of a row one lane loads per segment
template <>
struct RowChunk<kDtypeF32> {
  static constexpr int kCols = 4;
  float4 v;
  __device__ __forceinline__ void load(const void* X, long elem) {
    v = *reinterpret_cast<const float4*>(static_cast<const float*>(X) + elem);
  }
  // read-once data: a nontemporal load keeps the row from displacing what the caches hold
  __device__ __forceinline__ void load_once(const void* X, long elem) {
    typedef float vf4 __attribute__((ext_vector_type(4)));
    const vf4 t = __builtin_nontemporal_load(reinterpret_cast<const vf4*>(static_cast<const float*>(X) + elem));
    v = make_float4(t.x, t.y, t.z, t.w);
  }
  __device__ __forceinline__ void zero() { v = make_float4(0.f, 0.f, 0.f, 0.f); }
  __device__ __forceinline__ float dot(const float* q) const {
    return v.x * q[0] + v.y * q[1] + v.z * q[2] + v.w * q[3];
  }
};
template <>
struct RowChunk<kDtypeBF16> {
  static constexpr int kCols = 8;
  uint4 v;
  __device__ __forceinline__ void load(const void* X, long elem) {
    v = *reinterpret_cast<const uint4*>(static_cast<const uint16_t*>(X) + elem);
  }
  __device__ __forceinline__ void load_once(const void* X, long elem) {
    typedef unsigned vu4 __attribute__((ext_vector_type(4)));
    const vu4 t = __builtin_nontemporal_load(reinterpret_cast<const vu4*>(static_cast<const uint16_t*>(X) + elem));
    v = make_uint4(t.x, t.y, t.z, t.w);
  }
  __device__ __forceinline__ void zero() { v = make_uint4(0, 0, 0, 0); }
  __device__ __forceinline__ float dot(const float* q) const {
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      s += __uint_as_float(w[i] << 16) * q[2 * i];
      s += __uint_as_float(w[i] & 0xffff0000u) * q[2 * i + 1];
    }
    return s;
  }
};

template <int DIM, int MQ, int DT, bool ONCE>
__global__ __launch_bounds__(256) void scores_stream_kernel(
    const void* __restrict__ X, const float* __restrict__ xnrm, long row_begin, long n_rows,
    const float* __restrict__ Qbase, const int* __restrict__ qlist, const int* __restrict__ m_count_ptr,
    int m_limit, int m_begin, float* __restrict__ S, long ldS, int cosine) {
  constexpr int COLS = RowChunk<DT>::kCols;       // columns per lane per segment
  constexpr int SEG = 64 * COLS;                  // columns per wave-wide load
  constexpr int NSEG = (DIM + SEG - 1) / SEG;     // segments per row
  constexpr int RPI = 4;                          // rows per step
  constexpr int NV = RPI * MQ;

  const int m_total = m_count_ptr ? min(*m_count_ptr, m_limit) : m_limit;
  const int m_here = min(MQ, m_total - m_begin);
  if (m_here <= 0) return;

  const int lane = threadIdx.x & 63;
  const int wib = threadIdx.x >> 6;
  __shared__ float stage[4][MQ][64];

  // query values for this lane's columns
  float q[MQ][NSEG][COLS];
#pragma unroll
  for (int m = 0; m < MQ; ++m) {
    const bool have = m < m_here;
    const int qrow = have ? (qlist ? qlist[m_begin + m] : m_begin + m) : 0;
#pragma unroll
    for (int s = 0; s < NSEG; ++s) {
      const int col = s * SEG + lane * COLS;
#pragma unroll
      for (int c = 0; c < COLS; ++c)
        q[m][s][c] = (have && col < DIM) ? Qbase[long(qrow) * DIM + col + c] : 0.f;
    }
  }

  const long n_blocks = (n_rows + 63) / 64;
  const long wave = long(blockIdx.x) * 4 + wib;
  const long n_waves = long(gridDim.x) * 4;
  const int my_idx = value_index_of_lane<NV>(lane);

  for (long blk = wave; blk < n_blocks; blk += n_waves) {
    const long blk_row0 = blk * 64;
#pragma unroll 1
    for (int it = 0; it < 64 / RPI; ++it) {
      RowChunk<DT> x[RPI][NSEG];
#pragma unroll
      for (int r = 0; r < RPI; ++r) {
        const long row = blk_row0 + it * RPI + r;
#pragma unroll
        for (int s = 0; s < NSEG; ++s) {
          const int col = s * SEG + lane * COLS;
          if (row < n_rows && col < DIM)
          {
            if (ONCE)
              x[r][s].load_once(X, (row_begin + row) * long(DIM) + col);
            else
              x[r][s].load(X, (row_begin + row) * long(DIM) + col);
          }
          else
            x[r][s].zero();
        }
      }
      float acc[NV];
#pragma unroll
      for (int r = 0; r < RPI; ++r)
#pragma unroll
        for (int m = 0; m < MQ; ++m) {
          float a = 0.f;
#pragma unroll
          for (int s = 0; s < NSEG; ++s) a += x[r][s].dot(q[m][s]);
          acc[r * MQ + m] = a;
        }
      wave_sum_transposed<NV>(acc, lane);
      if (lane < NV) {
        const int r = my_idx / MQ, m = my_idx % MQ;
        stage[wib][m][it * RPI + r] = acc[0];
      }
    }
    // LDS traffic of one wave is ordered; no barrier needed between a wave's own write and read
    const long row = blk_row0 + lane;
    if (row < n_rows) {
      const float nr = xnrm[row_begin + row];
#pragma unroll
      for (int m = 0; m < MQ; ++m)
        if (m < m_here) S[long(m) * ldS + row] = row_score(nr, stage[wib][m][lane], cosine);
    }
  }
}

// Same contract, any dimension that is a multiple of 32: query values are read
// from LDS instead of registers.  Used for dimensions without a specialised
// instance.
template <int MQ, int DT>
__global__ __launch_bounds__(256) void scores_stream_generic_kernel(
    const void* __restrict__ X, const float* __restrict__ xnrm, long row_begin, long n_rows, int dim,
    const float* __restrict__ Qbase, const int* __restrict__ qlist, const int* __restrict__ m_count_ptr,
    int m_limit, int m_begin, float* __restrict__ S, long ldS, int cosine) {
  constexpr int COLS = RowChunk<DT>::kCols;
  constexpr int SEG = 64 * COLS;
  extern __shared__ float qs[];  // [MQ][dim]

  const int m_total = m_count_ptr ? min(*m_count_ptr, m_limit) : m_limit;
  const int m_here = min(MQ, m_total - m_begin);
  if (m_here <= 0) return;

  for (int i = threadIdx.x; i < MQ * dim; i += blockDim.x) {
    const int m = i / dim, c = i % dim;
    float v = 0.f;
    if (m < m_here) {
      const int qrow = qlist ? qlist[m_begin + m] : m_begin + m;
      v = Qbase[long(qrow) * dim + c];
    }
    qs[i] = v;
  }
  __syncthreads();

  const int lane = threadIdx.x & 63;
  const long wave = long(blockIdx.x) * 4 + (threadIdx.x >> 6);
  const long n_waves = long(gridDim.x) * 4;
  for (long row = wave; row < n_rows; row += n_waves) {
    float acc[MQ];
#pragma unroll
    for (int m = 0; m < MQ; ++m) acc[m] = 0.f;
    for (int col = lane * COLS; col < dim; col += SEG) {
      RowChunk<DT> x;
      x.load(X, (row_begin + row) * long(dim) + col);
#pragma unroll
      for (int m = 0; m < MQ; ++m) acc[m] += x.dot(&qs[m * dim + col]);
    }
#pragma unroll
    for (int m = 0; m < MQ; ++m) acc[m] = wave_sum(acc[m]);
    if (lane == 0) {
      const float nr = xnrm[row_begin + row];
#pragma unroll
      for (int m = 0; m < MQ; ++m)
        if (m < m_here) S[long(m) * ldS + row] = row_score(nr, acc[m], cosine);
    }
  }
}

// A call's rows copied into the instance's batch buffer together with their squared norms
// (row_norms_kernel's arithmetic), in one launch.  One wave per row.
__global__ __launch_bounds__(256) void copy_rows_norms_kernel(const float* __restrict__ in, int n_rows, int dim,
                                                              float* __restrict__ out, float* __restrict__ nrm) {
  const int lane = threadIdx.x & 63;
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= n_rows) return;
  const float4* src = reinterpret_cast<const float4*>(in + long(row) * dim);
  float4* dst = reinterpret_cast<float4*>(out + long(row) * dim);
  float acc = 0.f;
  for (int c = lane; c < dim / 4; c += 64) {
    const float4 v = src[c];
    dst[c] = v;
    acc += v.x * v.x + v.y * v.y + v.z * v.z + v.w * v.w;
  }
  acc = wave_sum(acc);
  if (lane == 0) nrm[row] = acc;
}

// The per-row term of row_score for the distance functions other than Euclidean, made in place
// from the squared lengths: inner product 0, cosine 1/|x|.
__global__ __launch_bounds__(256) void row_terms_kernel(float* __restrict__ nrm, long n_rows, int cosine) {
  const long stride = long(gridDim.x) * 256;
  for (long r = long(blockIdx.x) * 256 + threadIdx.x; r < n_rows; r += stride)
    nrm[r] = cosine ? 1.f / sqrtf(nrm[r]) : 0.f;
}

}  // namespace prox
