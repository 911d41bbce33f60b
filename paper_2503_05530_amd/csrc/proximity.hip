// Host runtime and C ABI of the Proximity-FLAT retrieval step (see include/proximity.h).
//
// One instance owns: the squared norms of the corpus rows, the cache (slot
// arrays for keys, values and eviction order, all resident on the device) and
// the per-batch workspaces.  A call enqueues, on the caller's stream and
// without waiting for the device:
//
//   copy batch rows behind the slot keys -> row norms of the batch
//   -> probe scores (batch rows x [slot keys, batch rows])      Algorithm 1, distances to all keys
//   -> candidate extraction + float64 evaluation
//   -> resolver (sequential semantics, hit / miss / evict)        Algorithm 1, nearest key, test, evict
//   -> key insertion and hits answered from resident keys
//   -> corpus scan for the rows that missed (scores, top-k, float64 ranking)   Algorithm 1, database call
//   -> result routing and value insertion.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <new>
#include <string>
#include <vector>

#include "../../include/proximity.h"
#include "cache_kernels.hpp"
#include "lsh_kernels.hpp"
#include "mfma_kernels.hpp"
#include "regq_kernels.hpp"
#include "bf16x3_kernels.hpp"
#include "resolver_lds.hpp"
#include "scan_kernels.hpp"
#include "select_kernels.hpp"
#include "slack_kernels.hpp"

using namespace prox;

namespace {

constexpr int kSlack = 8;          // extra float32 candidates handed to the float64 ranking
constexpr int kCandCap = 64;       // per-row candidate list length of the probe
constexpr int kSelE = 16;          // elements per thread in a selection segment
constexpr int kSelSeg = kSelE * kSelThreads;
constexpr int kMaxProfiled = 8192;
constexpr int kStreamMaxQueries = 4;   // calls with at most this many rows use the streaming kernels
static_assert(kStreamMaxQueries == kSmallRows, "the fused small-call kernels pair with the streaming scan");
constexpr int kScanPassQueries = 1024; // queries one launch of the batched scan covers
constexpr size_t kResolverLdsMax = 147 * 1024;  // dynamic LDS the LDS-state resolver may ask for
static_assert(kResolverLdsMax + kResolverStaticLds <= 160 * 1024 - 256, "the resolver block must fit the LDS of one CU");
constexpr size_t kProbeRangeRows = 1536;             // rows of a batch probed and resolved together, at most
constexpr size_t kProbeScoreBudget = size_t(512) << 20;  // bytes the dense probe scores may take (two ranges)
constexpr long kProbeSmallBlocks = 1536;  // probes of at most this many 32 x 32 tiles use the split-column kernel
constexpr size_t kLshLdsMax = 144 * 1024;  // dynamic LDS the bucket resolver may ask for (query + bucket keys)
constexpr int kSeedRows = 16384;       // head of the corpus scanned first to seed the top-k bounds
constexpr long kRegqDumpMinRows = 500000;  // single-query calls: corpora from here on are scored by the register-resident kernel
constexpr long kSeedRows2 = 262144;    // second sample of a long corpus (register-resident scan)

static_assert(sizeof(proximity_config) == 72, "proximity_config layout is part of the ABI");
static_assert(sizeof(proximity_stats_t) == 128, "proximity_stats_t layout is part of the ABI");
static_assert(sizeof(proximity_launch_t) == 20, "proximity_launch_t layout is part of the ABI");

thread_local std::string g_create_error;

// ---- proximity_knn_static: workspace that is part of the loaded library, not of any allocation ----
// Layout (all offsets multiples of 256 bytes): the state of the exactness check (1 KiB); row terms
// [kStaticMaxDocs] float32; dense scores
// [kStaticMaxQueries][kStaticMaxDocs] float32; per-segment top-k lists
// [kStaticMaxQueries][kStaticMaxDocs / kSelSeg][256] packed keys.
constexpr size_t kStaticMaxDocs = PROXIMITY_STATIC_MAX_DOCS;
constexpr size_t kStaticMaxQueries = PROXIMITY_STATIC_MAX_QUERIES;
static_assert(kStaticMaxQueries == size_t(kStreamMaxQueries), "the static search runs the streaming kernels");
static_assert(kStaticMaxDocs % kSelSeg == 0 && kStaticMaxDocs % 64 == 0, "whole selection segments");
constexpr size_t kStaticOffSlack = 0;   // SlackState (the largest row length, the counters of the exactness check)
static_assert(sizeof(SlackState) <= 1024, "the state must fit the first KiB of the workspace");
constexpr size_t kStaticOffNorms = 1024;
constexpr size_t kStaticOffScores = kStaticOffNorms + kStaticMaxDocs * sizeof(float);
constexpr size_t kStaticOffLists = kStaticOffScores + kStaticMaxQueries * kStaticMaxDocs * sizeof(float);
constexpr size_t kStaticScratchBytes =
    kStaticOffLists + kStaticMaxQueries * (kStaticMaxDocs / kSelSeg) * 256 * sizeof(uint64_t);
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

// Every device holds its own copy of `scratch` at its own address.  In host code the array's name is
// only a handle for hipGetSymbolAddress: the address a kernel may use is looked up once per device,
// with that device current, and kept here.
constexpr int kStaticMaxDevices = 64;
struct StaticDevice {
  unsigned char* ptr = nullptr;
  int n_cu = 0;
};
StaticDevice g_static_dev[kStaticMaxDevices];
std::mutex g_static_mutex;

struct DeviceGuard {
  int prev = -1;
  bool ok = true;
  explicit DeviceGuard(int dev) {
    if (hipGetDevice(&prev) != hipSuccess) ok = false;
    if (ok && prev != dev && hipSetDevice(dev) != hipSuccess) ok = false;
  }
  ~DeviceGuard() {
    if (prev >= 0) (void)hipSetDevice(prev);
  }
};

}  // namespace

struct proximity {
  proximity_config cfg{};
  int K = 0;  // neighbours asked of the index and stored per key: rerank_factor * k (Section 3.3.4)
  // bucketed cache (Section 3.2): lsh_bits > 0; slots = capacity << lsh_bits, bucket g owns g*b .. g*b+b-1
  int lsh_bits = 0;
  int slots = 0;               // all key slots: capacity, or capacity << lsh_bits
  float* lsh_planes = nullptr; // [lsh_bits][dim], the library's own copy
  int* lsh_code = nullptr;     // [max_batch] code of each batch row
  uint32_t* lsh_sorted = nullptr;  // [max_batch] (code, row) pairs grouped by code
  int* lsh_seg_start = nullptr;    // [max_batch] where each distinct code of the batch begins in lsh_sorted
  int* lsh_n_segs = nullptr;       // number of distinct codes in the batch
  int* bkt_size = nullptr;     // per bucket: live keys, front and back of its eviction order (-1: empty)
  int* bkt_head = nullptr;
  int* bkt_tail = nullptr;
  int n_cu = 256;
  uint64_t next_seq = 0;
  hipStream_t last_stream = nullptr;
  std::string err;
  std::vector<void*> allocs;

  // corpus side
  float* xnrm = nullptr;
  float* S = nullptr;  // dense scan scores [8][ldS]
  long ldS = 0;
  uint64_t* pairs[2] = {nullptr, nullptr};
  long pairs_elems = 0;
  uint64_t* topk_buf = nullptr;  // batched scan: [query tiles][scan blocks][tile queries][kTopkCap]
  uint16_t* qplanes = nullptr;   // bfloat16 corpus: the three bfloat16 planes of a call's queries, [3][max_batch][dim]
  int scan_blocks = 1;           // blocks that share the corpus in the batched scan
  int scan_blocks_regq = 1;      // the same for the scan that keeps its queries in registers (one block per CU)
  int64_t* res_ids = nullptr;
  float* res_d = nullptr;
  SlackState* slack = nullptr;   // is the float32 candidate list long enough? (select_kernels.hpp)
  float* seed_bound = nullptr;   // [max_batch] the score bound a batched scan of the current call started from
  RedoBuffers redo{};            // queries noted for the second ranking of the batched scan, and their rows
  // One-plane scans of a bfloat16 corpus (kRegqCoarse): whether this instance may run them, the list length
  // they ask for, the host word the ranking kernel notes its failures in, and what the host has launched so far.
  bool coarse_capable = false;
  int coarse_level = 0;          // 1: queries rounded (bfloat16 corpus); 2: rows rounded too (float32 corpus)
  int* coarse_note = nullptr;
  uint64_t coarse_calls = 0, coarse_queries = 0;

  // cache side
  float* srcs = nullptr;     // [capacity + max_batch][dim]: slot keys, then the current batch
  float* srcnrm = nullptr;   // their squared norms
  int64_t* val_ids = nullptr;
  float* val_d = nullptr;
  long long* slot_seq = nullptr;
  int* slot_next = nullptr;
  int* slot_prev = nullptr;
  CacheState* state = nullptr;
  float* D32 = nullptr;  // probe scores: [max_batch][ldD], or two buffers of [probe_rows][ldD] (see probe_rows)
  long ldD = 0;
  // A batch of more than probe_rows rows is probed and resolved in row ranges of that many: the probe of a
  // range runs on the caller's stream while the resolver walks the range before it on `side`, and the dense
  // probe scores exist for two ranges at a time.
  int probe_rows = 0;
  hipStream_t side = nullptr;
  std::vector<hipEvent_t> ev_probe, ev_go, ev_res;  // per range: candidates ready / resolver next in line / resolved
  int* ovf_cnt = nullptr;                    // per range: rows whose candidate list overflowed, and which
  int* ovf_list = nullptr;
  int* live_slots = nullptr;                 // keys resident when the batch started
  int* res_image = nullptr;                  // the LDS resolver's state between the ranges of a batch
  ResolverCarry* res_carry = nullptr;
  size_t probe_ws_bytes = 0;                 // device memory of the flat cache's probe (scores, lists, carry)
  int* cand_cnt = nullptr;
  int* cand_src = nullptr;
  double* cand_d = nullptr;
  uint8_t* hit = nullptr;
  int* src = nullptr;
  int* row_slot = nullptr;
  int* miss_list = nullptr;
  int* miss_count = nullptr;
  double* D64 = nullptr;        // small calls: float64 distances [kSmallRows][capacity]

  // kernel timing
  bool prof_on = false;
  std::vector<hipEvent_t> ev0, ev1;
  std::vector<proximity_launch_t> ev_info;
  size_t ev_used = 0;
  uint32_t prof_call = 0;
};

namespace {

int fail(proximity* h, int code, const char* fmt, ...) {
  char buf[512];
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(buf, sizeof buf, fmt, ap);
  va_end(ap);
  if (h)
    h->err = buf;
  else
    g_create_error = buf;
  return code;
}

#define HIP_TRY(h, expr)                                                                         \
  do {                                                                                           \
    hipError_t e_ = (expr);                                                                      \
    if (e_ != hipSuccess)                                                                        \
      return fail(h, e_ == hipErrorOutOfMemory ? PROXIMITY_ERR_OOM : PROXIMITY_ERR_HIP,          \
                  "%s failed: %s", #expr, hipGetErrorString(e_));                                \
  } while (0)

template <typename T>
int dev_alloc(proximity* h, T** p, size_t count, bool zero) {
  void* q = nullptr;
  size_t bytes = count * sizeof(T);
  if (bytes == 0) bytes = sizeof(T);
  HIP_TRY(h, hipMalloc(&q, bytes));
  h->allocs.push_back(q);
  if (zero) HIP_TRY(h, hipMemset(q, 0, bytes));
  *p = static_cast<T*>(q);
  return PROXIMITY_OK;
}

// ---- launch helpers --------------------------------------------------------

template <int DT>
void launch_row_norms(const proximity* h, const void* X, long n_rows, int dim, float* nrm, hipStream_t s) {
  if (n_rows <= 0) return;
  long blocks = (n_rows + 3) / 4;
  const long cap = long(h->n_cu) * 16;
  if (blocks > cap) blocks = cap;
  row_norms_kernel<DT><<<dim3((unsigned)blocks), dim3(256), 0, s>>>(X, n_rows, dim, nrm);
}

// Largest group of queries one streaming pass handles for this problem.
int stream_group(int dim, int n) {
  int mq = n <= 1 ? 1 : n <= 2 ? 2 : n <= 4 ? 4 : 8;
  const bool fast = dim == 768 || dim == 384 || dim == 1024;
  if (!fast)
    while (mq > 1 && size_t(mq) * dim * sizeof(float) > 48 * 1024) mq >>= 1;
  return mq;
}

template <int DT, int MQ, bool ONCE>
void launch_scores_stream_mq(const proximity* h, const void* X, const float* xnrm, long n_rows, int dim,
                             const float* Qbase, const int* qlist, const int* m_count_ptr, int m_limit,
                             int m_begin, float* S, long ldS, int cosine, hipStream_t s) {
  const long n_blocks64 = (n_rows + 63) / 64;
  long grid = (n_blocks64 + 3) / 4;
  const long cap = long(h->n_cu) * 8;
  if (grid > cap) grid = cap;
  if (grid < 1) grid = 1;
  const dim3 g((unsigned)grid), b(256);
#define PROX_STREAM_CASE(D)                                                                              \
  case D:                                                                                                \
    scores_stream_kernel<D, MQ, DT, ONCE><<<g, b, 0, s>>>(X, xnrm, 0, n_rows, Qbase, qlist, m_count_ptr,      \
                                                    m_limit, m_begin, S, ldS, cosine);                  \
    return;
  switch (dim) {
    PROX_STREAM_CASE(768)
    PROX_STREAM_CASE(384)
    PROX_STREAM_CASE(1024)
    default:
      break;
  }
#undef PROX_STREAM_CASE
  long ggrid = (n_rows + 3) / 4;
  if (ggrid > cap) ggrid = cap;
  if (ggrid < 1) ggrid = 1;
  scores_stream_generic_kernel<MQ, DT><<<dim3((unsigned)ggrid), b, size_t(MQ) * dim * sizeof(float), s>>>(
      X, xnrm, 0, n_rows, dim, Qbase, qlist, m_count_ptr, m_limit, m_begin, S, ldS, cosine);
}

template <int DT, bool ONCE>
void launch_scores_stream(const proximity* h, int mq, const void* X, const float* xnrm, long n_rows, int dim,
                          const float* Qbase, const int* qlist, const int* m_count_ptr, int m_limit,
                          int m_begin, float* S, long ldS, int cosine, hipStream_t s) {
  switch (mq) {
    case 1:
      launch_scores_stream_mq<DT, 1, ONCE>(h, X, xnrm, n_rows, dim, Qbase, qlist, m_count_ptr, m_limit, m_begin, S, ldS, cosine, s);
      break;
    case 2:
      launch_scores_stream_mq<DT, 2, ONCE>(h, X, xnrm, n_rows, dim, Qbase, qlist, m_count_ptr, m_limit, m_begin, S, ldS, cosine, s);
      break;
    case 4:
      launch_scores_stream_mq<DT, 4, ONCE>(h, X, xnrm, n_rows, dim, Qbase, qlist, m_count_ptr, m_limit, m_begin, S, ldS, cosine, s);
      break;
    default:
      launch_scores_stream_mq<DT, 8, ONCE>(h, X, xnrm, n_rows, dim, Qbase, qlist, m_count_ptr, m_limit, m_begin, S, ldS, cosine, s);
      break;
  }
}

void prof_begin(proximity* h, hipStream_t s) {
  if (h->prof_on && h->ev_used < h->ev0.size()) (void)hipEventRecord(h->ev0[h->ev_used], s);
}
void prof_end(proximity* h, hipStream_t s, int first_query, int n_queries, uint32_t kind = PROXIMITY_LAUNCH_SCAN) {
  if (h->prof_on && h->ev_used < h->ev0.size()) {
    (void)hipEventRecord(h->ev1[h->ev_used], s);
    h->ev_info[h->ev_used] = proximity_launch_t{h->prof_call, uint32_t(first_query), uint32_t(n_queries), 0.f, kind};
    ++h->ev_used;
  }
}

// One pass of the matrix-core scan over corpus rows [0, n_rows), shared by G blocks, for the
// queries base .. base+span-1 of the miss list.  The number of misses M is only known on the
// device: the tile shape for each range of M that this call can reach is launched, and the ones
// whose range does not contain M return at once.  Per-query lists of G*kp keys land in `out`.
void launch_batched_scan(proximity* h, long n_rows, int G, const float* Qbase, const int* qlist,
                         const int* m_count_ptr, int m_limit, int base, int span, int kp, const uint64_t* seed,
                         uint64_t* out, bool dump_all, hipStream_t s) {
  const int dim = int(h->cfg.dim);
  const int cosine = h->cfg.metric == PROXIMITY_METRIC_COSINE ? 1 : 0;
  const bool bf16 = h->cfg.corpus_dtype == PROXIMITY_DTYPE_BF16;
  const bool dma = !bf16 && dim >= 64;  // the global->LDS pipeline needs float32 rows and two slabs per tile
  if (bf16 && dim >= 64) {
    // bfloat16 rows: three-term split of the queries on the bfloat16 matrix cores (planes written by the
    // caller); the tile shape for up to 64 queries, and the one for more
    const long plane_stride = long(h->cfg.max_batch) * dim;
    const uint16_t* X16 = static_cast<const uint16_t*>(h->cfg.corpus);
    const bool known = m_count_ptr == nullptr;
#define PROX_SCAN16(TM, LO, HI)                                                                                 \
  do {                                                                                                          \
    const dim3 grid(G, (span + TM - 1) / TM);                                                                   \
    if (dump_all)                                                                                               \
      scan_bf16x3_kernel<TM, true><<<grid, dim3(TM * 4), 0, s>>>(X16, h->xnrm, n_rows, dim, h->qplanes,        \
                                                                  plane_stride, m_count_ptr, m_limit, base, LO, \
                                                                  HI, kp, seed, h->topk_buf, out, cosine);      \
    else                                                                                                        \
      scan_bf16x3_kernel<TM, false><<<grid, dim3(TM * 4), 0, s>>>(X16, h->xnrm, n_rows, dim, h->qplanes,       \
                                                                   plane_stride, m_count_ptr, m_limit, base,    \
                                                                   LO, HI, kp, seed, h->topk_buf, out, cosine); \
  } while (0)
    if (!known || m_limit <= 64) PROX_SCAN16(64, 0, 64);
    if (m_limit > 64) PROX_SCAN16(128, 64, 0x7fffffff);
#undef PROX_SCAN16
    return;
  }
#define PROX_SCAN(TM, TN, LO, HI)                                                                              \
  do {                                                                                                         \
    const dim3 grid(G, (span + TM - 1) / TM);                                                                  \
    if (dma && dump_all)                                                                                       \
      scan_mfma_dma_kernel<TM, true><<<grid, dim3(256), 0, s>>>(                                               \
          static_cast<const float*>(h->cfg.corpus), h->xnrm, n_rows, dim, Qbase, qlist, m_count_ptr, m_limit,  \
          base, LO, HI, kp, seed, h->topk_buf, out, cosine);                                                   \
    else if (dma)                                                                                              \
      scan_mfma_dma_kernel<TM, false><<<grid, dim3(256), 0, s>>>(                                              \
          static_cast<const float*>(h->cfg.corpus), h->xnrm, n_rows, dim, Qbase, qlist, m_count_ptr, m_limit,  \
          base, LO, HI, kp, seed, h->topk_buf, out, cosine);                                                   \
    else if (bf16)                                                                                             \
      scan_mfma_topk_kernel<TM, TN, kDtypeBF16><<<grid, dim3(256), 0, s>>>(                                    \
          h->cfg.corpus, h->xnrm, n_rows, dim, Qbase, qlist, m_count_ptr, m_limit, base, LO, HI, kp, seed,     \
          h->topk_buf, out, cosine);                                                                           \
    else                                                                                                       \
      scan_mfma_topk_kernel<TM, TN, kDtypeF32><<<grid, dim3(256), 0, s>>>(                                     \
          h->cfg.corpus, h->xnrm, n_rows, dim, Qbase, qlist, m_count_ptr, m_limit, base, LO, HI, kp, seed,     \
          h->topk_buf, out, cosine);                                                                           \
  } while (0)
  const bool known = m_count_ptr == nullptr;  // then M = m_limit and only its own shape is launched
  if (!known || m_limit <= 32) PROX_SCAN(32, 256, 0, 32);
  if (m_limit > 32 && (!known || m_limit <= 64)) PROX_SCAN(64, 256, 32, 64);
  if (dma) {  // 96 queries: three accumulator blocks per wave, one block per CU (84 KiB ring)
    if (m_limit > 64 && (!known || m_limit <= 96)) PROX_SCAN(96, 128, 64, 96);
    if (m_limit > 96) PROX_SCAN(128, 128, 96, 0x7fffffff);
  } else if (m_limit > 64) {
    PROX_SCAN(128, 128, 64, 0x7fffffff);
  }
#undef PROX_SCAN
}

// Candidates per query that a batched scan hands to the float64 ranking.  Scores of rounded operands order rows
// less finely than the error of a full score, so such a scan keeps more than k + 8: as many as a corpus of
// isotropic rows would put within the rounding error E of the k-th, and a margin.  There a score has standard
// deviation sigma = 2 |q| |x| / sqrt(d), so E = f 2^-8 |q| |x| is delta = f 2^-9 sqrt(d) of them (f = 1, or
// 2.002 when the rows are rounded too); the k-th of N rows sits z = sqrt(2 ln(N / k)) deviations out, where the
// density grows by e^z per deviation: k (e^(z delta) - 1) rows more on average, plus five times their spread,
// plus 16.  (Low-reuse workload: 159; 1 M x 768 float32, k = 10: 46; 24 M x 768, k = 32: 97.)  Rows that crowd
// more than that fail the exactness check and are ranked again, exactly; see coarse_now.
inline int coarse_list_length(int k, int level, int dim, double n_docs) {
  const double delta = std::sqrt(double(dim)) / 512.0 * (level >= 2 ? 2.002 : 1.0);
  const double ratio = n_docs / double(k) > 2.0 ? n_docs / double(k) : 2.0;
  const double more = double(k) * std::expm1(std::sqrt(2.0 * std::log(ratio)) * delta);
  return k + int(std::ceil(more + 5.0 * std::sqrt(more) + 16.0));
}
constexpr int kCoarseMaxList = 248;
inline int batched_list_length(const proximity* h, int k) {
  return h->coarse_capable ? coarse_list_length(k, h->coarse_level, int(h->cfg.dim), double(h->cfg.n_docs)) : k + kSlack;
}
// Does the next batched scan multiply one plane only?  Yes while lists that could not be proven sufficient stay
// rare: each one costs a second ranking from a rescan (more than the plane saves in a whole call), so past
// eight of them, and one per 1 024 queries scanned, the instance goes back to two planes for good.
inline bool coarse_now(const proximity* h) {
  if (!h->coarse_capable || !h->coarse_note) return false;
  const uint64_t fails = uint64_t(*reinterpret_cast<volatile int*>(h->coarse_note));
  return fails * 1024 <= h->coarse_queries + 8 * 1024;
}

// The same pass with the query tile resident in registers (regq_kernels.hpp), for the corpus types and
// dimensions that kernel is instantiated for.  The queries base .. base+span-1 go in slices of 64 (float32)
// or 128 (bfloat16); per slice the shape for every range of "queries from the slice's start on" that the
// call can reach is launched, and the ones whose range does not contain the device-side count return at once.
template <int DT, int DIM, int MODE = kRegqScan>
void launch_regq_dim(proximity* h, const void* X, const float* xnrm, long n_rows, int G, const float* Qbase, const int* qlist,
                     const int* m_count_ptr, int m_limit, int base, int span, int kp, const uint64_t* seed,
                     uint64_t* out, hipStream_t s) {
  constexpr int QW = regq_queries_per_wave(DT, regq_mode_rounds(MODE)), SLICE = 4 * QW;   // queries per wave and per block at most
  const int cosine = h->cfg.metric == PROXIMITY_METRIC_COSINE ? 1 : 0;
  const long plane_stride = long(h->cfg.max_batch) * DIM;
  const bool known = m_count_ptr == nullptr;  // then M = m_limit and only its own shape is launched
  for (int mb = base; mb < base + span; mb += SLICE) {
    const int rem_max = m_limit - mb;         // the most queries this slice can have to serve
    // (every shape is timed on its own: of the launches of one slice only the one whose range holds the number of
    // misses does the work, and proximity_profile_stop reports that one)
#define PROX_REGQ(WQ, LO, HI)                                                                                   \
  if (rem_max > (LO) && (!known || rem_max <= (HI))) {                                                           \
    prof_begin(h, s);                                                                                            \
    scan_regq_kernel<DT, DIM, WQ, MODE><<<dim3(G), dim3(256), 0, s>>>(X, xnrm, n_rows, Qbase, qlist, h->qplanes,       \
                                                                plane_stride, m_count_ptr, m_limit, mb, LO, HI, kp,    \
                                                                seed, h->topk_buf, out, cosine, RegqEmit{});           \
    prof_end(h, s, mb, rem_max < SLICE ? rem_max : SLICE);                                                       \
  }
    PROX_REGQ(1, 0, QW);
    PROX_REGQ(2, QW, 2 * QW);
    PROX_REGQ(4, 2 * QW, 0x7fffffff);
#undef PROX_REGQ
  }
}

void launch_regq_scan(proximity* h, const void* X, const float* xnrm, long n_rows, int G, const float* Qbase, const int* qlist,
                      const int* m_count_ptr, int m_limit, int base, int span, int kp, const uint64_t* seed,
                      uint64_t* out, bool coarse, hipStream_t s, bool keys = false) {
  // (keys: every score of the rows written out as a key, rounded operands only: the sample of a rounded scan)
  const int dim = int(h->cfg.dim);
#define PROX_REGQ_DIM(DT, D, MODE)                                                                                 \
  launch_regq_dim<DT, D, MODE>(h, X, xnrm, n_rows, G, Qbase, qlist, m_count_ptr, m_limit, base, span, kp, seed, out, s)
  if (keys) {
    if (h->cfg.corpus_dtype == PROXIMITY_DTYPE_BF16) {
      if (dim == 384) PROX_REGQ_DIM(kDtypeBF16, 384, kRegqCoarseKeys);
      else PROX_REGQ_DIM(kDtypeBF16, 256, kRegqCoarseKeys);
    } else {
      if (dim == 768) PROX_REGQ_DIM(kDtypeF32, 768, kRegqCoarseKeys);
      else PROX_REGQ_DIM(kDtypeF32, 384, kRegqCoarseKeys);
    }
  } else if (h->cfg.corpus_dtype == PROXIMITY_DTYPE_BF16) {
    if (coarse) {
      if (dim == 384) PROX_REGQ_DIM(kDtypeBF16, 384, kRegqCoarse);
      else PROX_REGQ_DIM(kDtypeBF16, 256, kRegqCoarse);
    } else {
      if (dim == 384) PROX_REGQ_DIM(kDtypeBF16, 384, kRegqScan);
      else PROX_REGQ_DIM(kDtypeBF16, 256, kRegqScan);
    }
  } else if (coarse) {
    if (dim == 768) PROX_REGQ_DIM(kDtypeF32, 768, kRegqCoarse);
    else PROX_REGQ_DIM(kDtypeF32, 384, kRegqCoarse);
  } else {
    if (dim == 768) PROX_REGQ_DIM(kDtypeF32, 768, kRegqScan);
    else PROX_REGQ_DIM(kDtypeF32, 384, kRegqScan);
  }
#undef PROX_REGQ_DIM
}

// Merge per-query lists of `len` keys in pairs[cur] down to one sorted list of kp keys per
// query, ping-ponging between the two key buffers.  Returns the index of the buffer that
// holds the result.
// Merge levels over per-query lists of `len` keys (sorted runs of kp) until at most stop_len keys are
// left per query (stop_len = kp: one list).  *len_out receives what is left.
int enqueue_merge_levels(proximity* h, int cur, long len, int kp, const int* m_count_ptr, int m_limit,
                         hipStream_t s, long stop_len, long* len_out = nullptr) {
  if (stop_len < kp) stop_len = kp;
  while (len > stop_len) {
    const int g = int((len + kSelSeg - 1) / kSelSeg);
    select_kernel<false, kSelE><<<dim3(g, m_limit), dim3(kSelThreads), 0, s>>>(
        h->pairs[cur], len, len, 0, kp, h->pairs[cur ^ 1], g, m_count_ptr, m_limit, 0);
    cur ^= 1;
    len = long(g) * kp;
  }
  if (len_out) *len_out = len;
  return cur;
}

// Per-query lists of `len` keys in pairs[cur] down to one sorted list of kp keys: merge levels while a query's
// keys are too many for one block, then one block per query.  `margin`: see cut_lists_kernel.
int enqueue_cut(proximity* h, int cur, long len, int kp, const float* Qbase, const int* qlist, const int* m_count_ptr,
                int m_limit, int margin, int bound_rank, bool first, hipStream_t s) {
  long left = len;
  cur = enqueue_merge_levels(h, cur, len, kp, m_count_ptr, m_limit, s, kCutMaxKeys, &left);
  // (always launched: it publishes the bound, also to the exactness check)
  cut_lists_kernel<<<dim3(m_limit), dim3(kRerankThreads), 0, s>>>(
      h->pairs[cur], left, kp, h->pairs[cur ^ 1], m_count_ptr, m_limit, margin, Qbase, qlist, int(h->cfg.dim),
      int(h->cfg.metric), h->slack, bound_rank, h->seed_bound, first ? 1 : 0);
  return cur ^ 1;
}

// The index search for the queries listed in qlist (or rows 0..m_limit-1 of
// Qbase when qlist is null): scores, hierarchical top-k, float64 ranking.
// Results (k entries per query, k <= the instance's K) land in row qlist[m] (or m) of res_ids / res_d.
// With small_routing (a handful of queries) res_ids / res_d are the caller's rows of k_out <= k entries
// and the k ranked entries go to the cache; otherwise k_out is not used.
int enqueue_scan(proximity* h, const float* Qbase, const int* qlist, const int* m_count_ptr, int m_limit, int k,
                 int k_out, int64_t* res_ids, float* res_d, const SmallRouting* small_routing, hipStream_t s) {
  const int dim = int(h->cfg.dim);
  const long N = long(h->cfg.n_docs);
  if (N == 0) {
    fill_empty_results_kernel<<<dim3(m_limit), dim3(64), 0, s>>>(qlist, m_count_ptr, m_limit, k, res_ids, res_d);
    return PROXIMITY_OK;
  }
  const bool batched = m_limit > kStreamMaxQueries;
  const int kp = batched ? batched_list_length(h, k) : k + kSlack;
  const bool bf16 = h->cfg.corpus_dtype == PROXIMITY_DTYPE_BF16;
  const int metric = int(h->cfg.metric), cosine = metric == PROXIMITY_METRIC_COSINE ? 1 : 0;
  int cur = 0;
  long left = kp;  // keys per query handed to the ranking kernel
  bool coarse = false, seeded = false;   // (seeded: the scan started from a sample's bound)
  if (!batched) {
    const int mq = stream_group(dim, m_limit);
    const int g1 = int((N + kSelSeg - 1) / kSelSeg);
    for (int m0 = 0; m0 < m_limit; m0 += mq) {
      prof_begin(h, s);
      if (!bf16 && N >= kRegqDumpMinRows && (dim == 768 || dim == 384)) {
        // a long float32 corpus of these dimensions: the register-resident kernel's loads stream it faster
        // (its per-block top-k lists instead of the first selection pass were tried: the scan lost what the
        // selection had cost)
        RegqEmit dump{};
        dump.S = h->S;
        dump.ldS = h->ldS;
        const int upto = m0 + mq < m_limit ? m0 + mq : m_limit;   // S has room for the mq queries of this pass
        if (dim == 768)
          scan_regq_kernel<kDtypeF32, 768, 1, kRegqDump><<<dim3(h->scan_blocks_regq), dim3(256), 0, s>>>(
              h->cfg.corpus, h->xnrm, N, Qbase, qlist, nullptr, 0, m_count_ptr, upto, m0, 0, 0x7fffffff, 0, nullptr, nullptr,
              nullptr, cosine, dump);
        else
          scan_regq_kernel<kDtypeF32, 384, 1, kRegqDump><<<dim3(h->scan_blocks_regq), dim3(256), 0, s>>>(
              h->cfg.corpus, h->xnrm, N, Qbase, qlist, nullptr, 0, m_count_ptr, upto, m0, 0, 0x7fffffff, 0, nullptr, nullptr,
              nullptr, cosine, dump);
      } else if (bf16) {
        launch_scores_stream<kDtypeBF16, true>(h, mq, h->cfg.corpus, h->xnrm, N, dim, Qbase, qlist, m_count_ptr, m_limit,
                                         m0, h->S, h->ldS, cosine, s);
      } else {
        launch_scores_stream<kDtypeF32, true>(h, mq, h->cfg.corpus, h->xnrm, N, dim, Qbase, qlist, m_count_ptr, m_limit,
                                        m0, h->S, h->ldS, cosine, s);
      }
      prof_end(h, s, m0, mq);
      if (small_routing) {
        // a handful of queries: selection, float64 ranking and routing in one launch;
        // res_ids / res_d are then the caller's output rows
        for (int phase = 1; phase <= 2; ++phase) {
          const dim3 grid(phase == 2 ? 1 : g1, mq);
          // (four waves for both phases: with sixteen the second phase, one block per query, was slower)
          if (bf16)
            select_finish_small_kernel<kDtypeBF16, kSelE, kSelThreads><<<grid, dim3(kSelThreads), 0, s>>>(
                h->S, h->ldS, N, kp, k, k_out, h->pairs[0], g1, phase, h->cfg.corpus, dim, Qbase, qlist,
                m_count_ptr, m_limit, m0, *small_routing, res_ids, res_d, metric, h->slack);
          else
            select_finish_small_kernel<kDtypeF32, kSelE, kSelThreads><<<grid, dim3(kSelThreads), 0, s>>>(
                h->S, h->ldS, N, kp, k, k_out, h->pairs[0], g1, phase, h->cfg.corpus, dim, Qbase, qlist,
                m_count_ptr, m_limit, m0, *small_routing, res_ids, res_d, metric, h->slack);
        }
      } else {
        select_kernel<true, kSelE><<<dim3(g1, mq), dim3(kSelThreads), 0, s>>>(
            h->S, h->ldS, N, 0, kp, h->pairs[0] + long(m0) * g1 * kp, g1, m_count_ptr, m_limit, m0);
      }
    }
    if (small_routing) return PROXIMITY_OK;
    cur = enqueue_merge_levels(h, 0, long(g1) * kp, kp, m_count_ptr, m_limit, s, kRerankMergeKeys, &left);
  } else {
    // (the kernels below write through these: never launch them on an instance that was not given the buffers)
    if (!h->topk_buf || !h->pairs[0] || !h->pairs[1] || !h->seed_bound ||
        (((bf16 && dim >= 64) || h->coarse_capable) && !h->qplanes))
      return fail(h, PROXIMITY_ERR_INVALID_ARG, "%d queries in one search on an instance without the batched scan's workspace",
                  m_limit);
    // Batched scan on the matrix cores, in two steps.  First the head of the corpus (kSeedRows rows) is scanned
    // and cut on its own: one of its best scores per query (bound_rank below) is a valid bound for the whole
    // corpus and lets the full scan drop almost every row at once instead of learning a bound block by block.
    // Then the full scan, then the merge.
    const uint64_t* seed = nullptr;
    // which entry of a sample's list bounds the scan: the last of a list of k + 8, the same rank of a longer one
    const int bound_rank = k + kSlack < kp ? k + kSlack : kp;
    const bool regq = regq_supported(int(h->cfg.corpus_dtype), dim);
    coarse = regq && coarse_now(h);
    if ((bf16 && dim >= 64) || coarse)
      split_bf16x3_kernel<<<dim3(m_limit), dim3(256), 0, s>>>(Qbase, qlist, m_count_ptr, m_limit, dim, h->qplanes,
                                                               long(h->cfg.max_batch) * dim);
    if (coarse) {
      ++h->coarse_calls;
      h->coarse_queries += uint64_t(m_limit);
    }
    if (N >= 8L * kSeedRows) {
      const int gs = kSeedRows / 128;
      // the head's scores are written out whole and merged; rows of 32 columns only: per-block lists
      const bool dump_seed = dim >= 64;
      const bool timing = h->prof_on;   // (the sample's launches are not among the timed scans)
      h->prof_on = false;
      for (int base = 0; base < m_limit; base += kScanPassQueries) {
        const int span = m_limit - base < kScanPassQueries ? m_limit - base : kScanPassQueries;
        if (coarse)   // the scan's own kernel and arithmetic, every score written out
          launch_regq_scan(h, h->cfg.corpus, h->xnrm, kSeedRows, gs, Qbase, qlist, m_count_ptr, m_limit, base, span, kp,
                           nullptr, h->pairs[0], true, s, true);
        else
          launch_batched_scan(h, kSeedRows, gs, Qbase, qlist, m_count_ptr, m_limit, base, span, kp, nullptr,
                              h->pairs[0], dump_seed, s);
      }
      h->prof_on = timing;
      // (the register-resident scan on the operands as stored is not the kernel that scored the head: its bound
      // gets the margin between the two; the rounded scan scored its own sample, the margin stays all the same)
      cur = enqueue_cut(h, 0, dump_seed ? long(kSeedRows) : long(gs) * kp, kp, Qbase, qlist, m_count_ptr, m_limit,
                        regq ? 1 : 0, bound_rank, true, s);
      seed = h->pairs[cur];
      seeded = true;
      cur ^= 1;  // the full scan writes into the other buffer
    }
    const int G = regq ? h->scan_blocks_regq : h->scan_blocks;
    if (regq && seed && N >= 128L * kSeedRows) {
      // A long corpus gets a second, longer sample (the next N / 32 rows, at most kSeedRows2), scanned with the
      // first sample's bound: the bound it yields lets through a sixteenth of the rows the first one would, and
      // with one wave per SIMD in the register-resident scan every candidate appended is matrix time lost.
      long rows2 = N / 32 < kSeedRows2 ? N / 32 : kSeedRows2;
      rows2 -= rows2 % 128;
      int g2 = int(rows2 / 1024);   // eight tiles per block
      if (g2 > G) g2 = G;
      const char* X2 = static_cast<const char*>(h->cfg.corpus) + size_t(kSeedRows) * dim * (bf16 ? 2 : 4);
      const bool timing = h->prof_on;   // (the sample's launches are not among the timed scans)
      h->prof_on = false;
      for (int base = 0; base < m_limit; base += kScanPassQueries) {
        const int span = m_limit - base < kScanPassQueries ? m_limit - base : kScanPassQueries;
        launch_regq_scan(h, X2, h->xnrm + kSeedRows, rows2, g2, Qbase, qlist, m_count_ptr, m_limit, base, span, kp, seed,
                         h->pairs[cur], coarse, s);
      }
      h->prof_on = timing;
      cur = enqueue_cut(h, cur, long(g2) * kp, kp, Qbase, qlist, m_count_ptr, m_limit, 0, bound_rank, false, s);
      seed = h->pairs[cur];   // (row numbers in these keys count from the sample's first row; only scores are used)
      cur ^= 1;
    }
    for (int base = 0; base < m_limit; base += kScanPassQueries) {
      const int span = m_limit - base < kScanPassQueries ? m_limit - base : kScanPassQueries;
      if (regq) {
        launch_regq_scan(h, h->cfg.corpus, h->xnrm, N, G, Qbase, qlist, m_count_ptr, m_limit, base, span, kp, seed,
                         h->pairs[cur], coarse, s);
      } else {
        prof_begin(h, s);
        launch_batched_scan(h, N, G, Qbase, qlist, m_count_ptr, m_limit, base, span, kp, seed, h->pairs[cur], false,
                            s);
        prof_end(h, s, base, span);
      }
    }
    // the last merge level happens inside the ranking kernel
    cur = enqueue_merge_levels(h, cur, long(G) * kp, kp, m_count_ptr, m_limit, s, kCutMaxKeys, &left);
  }
  const int n_lists = int(left / kp);
  // float64 ranking of the candidates, then -- for queries whose list could not be proven long enough, which
  // the ranking notes on the device -- a second ranking from a rescan; its two launches return at once otherwise
  long rg = (N + 3) / 4;
  if (rg > long(h->n_cu) * 8) rg = long(h->n_cu) * 8;
  if (bf16) {
    rerank_f64_kernel<kDtypeBF16><<<dim3(m_limit), dim3(kRerankThreads), 0, s>>>(
        h->pairs[cur], n_lists, kp, k, h->cfg.corpus, dim, Qbase, qlist, m_count_ptr, m_limit, res_ids, res_d, metric,
        h->slack, h->redo, coarse ? h->coarse_level : 0, h->seed_bound, seeded ? 1 : 0);
    redo_collect_kernel<kDtypeBF16><<<dim3((unsigned)rg), dim3(256), 0, s>>>(h->cfg.corpus, h->xnrm, N, dim, Qbase, qlist,
                                                                             h->slack, h->redo, cosine);
    redo_rank_kernel<kDtypeBF16><<<dim3(m_limit), dim3(1024), 0, s>>>(h->cfg.corpus, dim, Qbase, qlist, h->slack,
                                                                      h->redo, k, res_ids, res_d, metric);
  } else {
    rerank_f64_kernel<kDtypeF32><<<dim3(m_limit), dim3(kRerankThreads), 0, s>>>(
        h->pairs[cur], n_lists, kp, k, h->cfg.corpus, dim, Qbase, qlist, m_count_ptr, m_limit, res_ids, res_d, metric,
        h->slack, h->redo, coarse ? h->coarse_level : 0, h->seed_bound, seeded ? 1 : 0);
    redo_collect_kernel<kDtypeF32><<<dim3((unsigned)rg), dim3(256), 0, s>>>(h->cfg.corpus, h->xnrm, N, dim, Qbase, qlist,
                                                                            h->slack, h->redo, cosine);
    redo_rank_kernel<kDtypeF32><<<dim3(m_limit), dim3(1024), 0, s>>>(h->cfg.corpus, dim, Qbase, qlist, h->slack,
                                                                     h->redo, k, res_ids, res_d, metric);
  }
  return PROXIMITY_OK;
}

int check_launch(proximity* h, const char* what) {
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(h, PROXIMITY_ERR_HIP, "%s: %s", what, hipGetErrorString(e));
  return PROXIMITY_OK;
}

int validate_call(proximity* h, const float* queries, uint32_t n, uint32_t k, int64_t* out_ids) {
  if (!h) return fail(nullptr, PROXIMITY_ERR_INVALID_ARG, "handle is null");
  if (k != h->cfg.k) return fail(h, PROXIMITY_ERR_K_MISMATCH, "k=%u but the instance was created with k=%u", k, h->cfg.k);
  if (n > h->cfg.max_batch)
    return fail(h, PROXIMITY_ERR_BATCH_TOO_LARGE, "n=%u exceeds max_batch=%u", n, h->cfg.max_batch);
  if (n > 0 && (!queries || !out_ids)) return fail(h, PROXIMITY_ERR_INVALID_ARG, "queries or out_ids is null");
  if (reinterpret_cast<uintptr_t>(queries) % 16 != 0)
    return fail(h, PROXIMITY_ERR_INVALID_ARG, "queries must be 16-byte aligned (rows are read 16 bytes at a time)");
  return PROXIMITY_OK;
}

// Rows of a call whose dense float32 probe scores are held at a time: as many as two score buffers of that many
// rows fit the budget, a multiple of 64 between 64 and kProbeRangeRows.
size_t probe_range_rows(size_t capacity, size_t max_batch) {
  const size_t ld = (capacity + max_batch + 63) / 64 * 64;
  const size_t fit = kProbeScoreBudget / (2 * ld * sizeof(float)) / 64 * 64;
  return fit < 64 ? 64 : fit > kProbeRangeRows ? kProbeRangeRows : fit;
}

// The row ranges of a call of nn > R rows: cut[g] = row after the last of range g; returns their number.
// What is left when the last probe ends is the resolution of the last range, so the last rows go in two halves.
// The listing probe runs one block per CU, each over whole tiles of 128 sources for 64 rows: there the range size
// decides how evenly the tiles divide among the blocks (at 10 000 keys, ranges of 1 024 rows leave the slowest
// block with 6 tiles where the average is 5.5).  The size with the best rows x tiles per time of the slowest block
// is taken, half a tile's time counted as the fixed cost of a launch.
int probe_range_cuts(int nn, int R, int c, bool listing, int n_cu, int* cut) {
  int ranges = 0, r = 0;
  auto listing_rows = [&](int from) {
    int most = nn - from < R ? nn - from : R;
    if (nn - from - most < 512) most = nn - from - 512;   // (at least 512 rows stay for the two short last ranges)
    if (most < 512) return nn - from < R ? nn - from : R;
    const int nb = n_cu > 8 ? n_cu - 8 : 1;
    int best = most;
    double best_rate = 0.0;
    for (int rows = 512; rows <= most; rows += 64) {
      const int slices = rows / 64, tiles = (c + from + rows + 127) / 128;
      const int parts = nb / slices > 0 ? nb / slices : 1;
      const int per = (tiles + parts - 1) / parts;
      const double rate = double(rows) * tiles / (per + 0.5);
      if (rate >= best_rate) {
        best_rate = rate;
        best = rows;
      }
    }
    return best;
  };
  const int tail = listing && R > 1024 ? 1024 : R;   // rows left for the short last ranges, at most
  while (nn - r > tail) cut[ranges++] = (r += listing ? listing_rows(r) : R);
  if (nn - r >= 256) cut[ranges++] = (r += ((nn - r) / 2 + 63) / 64 * 64);
  if (r < nn) cut[ranges++] = nn;
  return ranges;
}

}  // namespace

extern "C" {

uint32_t proximity_abi_version(void) { return PROXIMITY_ABI_VERSION; }

double proximity_score_error_bound(uint32_t metric, uint32_t dim, double query_length, double max_row_length) {
  if (metric > PROXIMITY_METRIC_COSINE || dim == 0 || !(query_length >= 0.0) || !(max_row_length >= 0.0))
    return std::nan("");
  return score_error_bound(int(metric), int(dim), query_length, max_row_length);
}

uint32_t proximity_rounded_scan_list_length(uint32_t k, uint32_t corpus_dtype, uint32_t dim, uint64_t n_docs) {
  if (k == 0 || k > PROXIMITY_MAX_K || corpus_dtype > PROXIMITY_DTYPE_BF16 || dim == 0 || dim > PROXIMITY_MAX_DIM) return 0;
  return uint32_t(coarse_list_length(int(k), corpus_dtype == PROXIMITY_DTYPE_BF16 ? 1 : 2, int(dim), double(n_docs)));
}

double proximity_coarse_score_error(uint32_t metric, uint32_t corpus_dtype, double query_length, double max_row_length) {
  if (metric > PROXIMITY_METRIC_COSINE || corpus_dtype > PROXIMITY_DTYPE_BF16 || !(query_length >= 0.0) ||
      !(max_row_length >= 0.0))
    return std::nan("");
  return coarse_score_error(int(metric), query_length, max_row_length, corpus_dtype == PROXIMITY_DTYPE_BF16 ? 1 : 2);
}

uint32_t proximity_probe_row_ranges(uint32_t n, uint32_t capacity, uint32_t max_batch, uint32_t listing, uint32_t n_cu,
                                    uint32_t* ends, uint32_t max_ranges) {
  if (!ends || n == 0 || n > max_batch || max_batch > PROXIMITY_MAX_BATCH || capacity == 0 ||
      capacity > PROXIMITY_MAX_CAPACITY || n_cu == 0)
    return 0;
  const int R = int(probe_range_rows(capacity, max_batch));
  int cut[PROXIMITY_MAX_BATCH / 64 + 4];
  int ranges = 1;
  cut[0] = int(n);
  if (int(n) > R) ranges = probe_range_cuts(int(n), R, int(capacity), listing != 0, int(n_cu), cut);
  if (uint32_t(ranges) > max_ranges) return 0;
  for (int g = 0; g < ranges; ++g) ends[g] = uint32_t(cut[g]);
  return uint32_t(ranges);
}

const char* proximity_last_error(const proximity_t* h) { return h ? h->err.c_str() : g_create_error.c_str(); }

int proximity_create(const proximity_config* cfg, proximity_t** out) {
  if (out) *out = nullptr;
  if (!cfg || !out) return fail(nullptr, PROXIMITY_ERR_INVALID_ARG, "cfg or out is null");
  if (cfg->struct_size != sizeof(proximity_config))
    return fail(nullptr, PROXIMITY_ERR_INVALID_ARG, "struct_size=%u, expected %zu", cfg->struct_size,
                sizeof(proximity_config));
  if (cfg->dim == 0 || cfg->dim % 32 != 0 || cfg->dim > PROXIMITY_MAX_DIM)
    return fail(nullptr, PROXIMITY_ERR_INVALID_ARG, "dim=%u must be a multiple of 32 in 32..%u", cfg->dim,
                PROXIMITY_MAX_DIM);
  if (cfg->k == 0 || cfg->k > PROXIMITY_MAX_K)
    return fail(nullptr, PROXIMITY_ERR_INVALID_ARG, "k=%u must be in 1..%u", cfg->k, PROXIMITY_MAX_K);
  const uint32_t rho = cfg->rerank_factor == 0 ? 1u : cfg->rerank_factor;
  if (rho > PROXIMITY_MAX_K || rho * cfg->k > PROXIMITY_MAX_K)
    return fail(nullptr, PROXIMITY_ERR_INVALID_ARG, "rerank_factor * k = %u * %u exceeds %u", rho, cfg->k,
                PROXIMITY_MAX_K);
  if (cfg->lsh_bits > uint32_t(kLshMaxBits))
    return fail(nullptr, PROXIMITY_ERR_INVALID_ARG, "lsh_bits=%u exceeds %d", cfg->lsh_bits, kLshMaxBits);
  const bool lsh = cfg->lsh_bits > 0 && cfg->capacity > 0;
  if (lsh) {
    if (!cfg->lsh_planes) return fail(nullptr, PROXIMITY_ERR_INVALID_ARG, "lsh_planes is null but lsh_bits > 0");
    if (cfg->capacity > uint32_t(kLshMaxBucket))
      return fail(nullptr, PROXIMITY_ERR_INVALID_ARG, "capacity=%u per bucket exceeds %d", cfg->capacity, kLshMaxBucket);
    if ((uint64_t(cfg->capacity) << cfg->lsh_bits) > PROXIMITY_MAX_CAPACITY)
      return fail(nullptr, PROXIMITY_ERR_INVALID_ARG, "capacity << lsh_bits = %llu exceeds %u",
                  (unsigned long long)(uint64_t(cfg->capacity) << cfg->lsh_bits), PROXIMITY_MAX_CAPACITY);
  }
  if (cfg->max_batch == 0 || cfg->max_batch > PROXIMITY_MAX_BATCH)
    return fail(nullptr, PROXIMITY_ERR_INVALID_ARG, "max_batch=%u must be in 1..%u", cfg->max_batch,
                PROXIMITY_MAX_BATCH);
  if (cfg->capacity > PROXIMITY_MAX_CAPACITY)
    return fail(nullptr, PROXIMITY_ERR_INVALID_ARG, "capacity=%u exceeds %u", cfg->capacity, PROXIMITY_MAX_CAPACITY);
  if (cfg->n_docs >= (1ull << 31))
    return fail(nullptr, PROXIMITY_ERR_INVALID_ARG, "n_docs=%llu must be below 2^31", (unsigned long long)cfg->n_docs);
  if (cfg->n_docs > 0 && !cfg->corpus) return fail(nullptr, PROXIMITY_ERR_INVALID_ARG, "corpus is null but n_docs > 0");
  if (cfg->corpus_dtype != PROXIMITY_DTYPE_F32 && cfg->corpus_dtype != PROXIMITY_DTYPE_BF16)
    return fail(nullptr, PROXIMITY_ERR_INVALID_ARG, "unknown corpus_dtype %u", cfg->corpus_dtype);
  if (cfg->policy != PROXIMITY_POLICY_FIFO && cfg->policy != PROXIMITY_POLICY_LRU)
    return fail(nullptr, PROXIMITY_ERR_INVALID_ARG, "unknown policy %u", cfg->policy);
  if (reinterpret_cast<uintptr_t>(cfg->corpus) % 16 != 0)
    return fail(nullptr, PROXIMITY_ERR_INVALID_ARG, "corpus must be 16-byte aligned (rows are read 16 bytes at a time)");
  if (cfg->metric > PROXIMITY_METRIC_COSINE)
    return fail(nullptr, PROXIMITY_ERR_INVALID_ARG, "unknown metric %u", cfg->metric);
  if ((cfg->flags & ~PROXIMITY_FLAG_NO_ROUNDED_SCAN) != 0)
    return fail(nullptr, PROXIMITY_ERR_INVALID_ARG, "unknown flags %#x", cfg->flags);
  if (cfg->device < 0) return fail(nullptr, PROXIMITY_ERR_INVALID_ARG, "device=%d is negative", cfg->device);

  int n_dev = 0;
  if (hipGetDeviceCount(&n_dev) != hipSuccess || cfg->device >= n_dev)
    return fail(nullptr, PROXIMITY_ERR_HIP, "device %d is not available (%d devices visible)", cfg->device, n_dev);

  proximity* h = new (std::nothrow) proximity();
  if (!h) return fail(nullptr, PROXIMITY_ERR_OOM, "host allocation failed");
  h->cfg = *cfg;
  h->cfg.rerank_factor = rho;
  h->K = int(rho * cfg->k);
  h->lsh_bits = lsh ? int(cfg->lsh_bits) : 0;
  h->slots = int(cfg->capacity) << h->lsh_bits;
  DeviceGuard guard(cfg->device);
  auto bail = [&](int code) {
    g_create_error = h->err;
    for (hipEvent_t e : h->ev_probe) if (e) (void)hipEventDestroy(e);
    for (hipEvent_t e : h->ev_go) if (e) (void)hipEventDestroy(e);
    for (hipEvent_t e : h->ev_res) if (e) (void)hipEventDestroy(e);
    if (h->side) (void)hipStreamDestroy(h->side);
    for (void* p : h->allocs) (void)hipFree(p);
    if (h->coarse_note) (void)hipHostFree(h->coarse_note);
    delete h;
    return code;
  };
  if (!guard.ok) {
    h->err = "hipSetDevice failed";
    return bail(PROXIMITY_ERR_HIP);
  }
  hipDeviceProp_t prop;
  if (hipGetDeviceProperties(&prop, cfg->device) == hipSuccess && prop.multiProcessorCount > 0)
    h->n_cu = prop.multiProcessorCount;

  const size_t c = size_t(h->slots), B = cfg->max_batch, d = cfg->dim, k = size_t(h->K), N = cfg->n_docs;
  // Scans on rounded operands: a corpus of a type and dimension the register-resident scan has, calls of more than
  // a handful of rows, and a list length the ranking kernel holds.
  h->coarse_level = cfg->corpus_dtype == PROXIMITY_DTYPE_BF16 ? 1 : 2;
  h->coarse_capable = regq_supported(int(cfg->corpus_dtype), int(d)) && N > 0 && B > size_t(kStreamMaxQueries) &&
                      coarse_list_length(int(k), h->coarse_level, int(d), double(N)) <= kCoarseMaxList &&
                      (cfg->flags & PROXIMITY_FLAG_NO_ROUNDED_SCAN) == 0;
  // sized for the K = rerank_factor * k neighbours a search call asks for
  const int kp = h->coarse_capable ? coarse_list_length(int(k), h->coarse_level, int(d), double(N)) : int(k) + kSlack;
  int rc;
#define TRY_ALLOC(ptr, count, zero)                              \
  if ((rc = dev_alloc(h, &(ptr), (count), (zero))) != PROXIMITY_OK) return bail(rc)
  TRY_ALLOC(h->xnrm, N, false);
  h->ldS = long((N + 63) / 64 * 64);
  TRY_ALLOC(h->S, size_t(8) * size_t(h->ldS), false);
  const size_t g1 = (N + kSelSeg - 1) / kSelSeg;
  size_t lists = g1 > 0 ? g1 : 1;
  if (N > 0) {  // (also for instances of single-row calls: the scores-only form of that scan serves them)
    const size_t tiles128 = (N + kRegqTileRows - 1) / kRegqTileRows;
    h->scan_blocks_regq = int(tiles128 < size_t(h->n_cu) ? tiles128 : size_t(h->n_cu));
  }
  if (B > size_t(kStreamMaxQueries) && N > 0) {
    const size_t tiles256 = (N + 255) / 256;
    h->scan_blocks = int(tiles256 < size_t(2 * h->n_cu) ? tiles256 : size_t(2 * h->n_cu));
    if (size_t(h->scan_blocks) > lists) lists = size_t(h->scan_blocks);
    if (size_t(h->scan_blocks_regq) > lists) lists = size_t(h->scan_blocks_regq);
    if (size_t(kSeedRows + kp - 1) / kp > lists) lists = size_t(kSeedRows + kp - 1) / kp;  // dumped head scores
    const size_t pass_q = (B < size_t(kScanPassQueries) ? B : size_t(kScanPassQueries)) + 127;
    // candidate buffers: per (block, query of the launch's tile); the register-resident scan runs one slice
    // of at most 128 queries per launch
    size_t cand_sets = size_t(h->scan_blocks) * pass_q;
    if (size_t(h->scan_blocks_regq) * 128 > cand_sets) cand_sets = size_t(h->scan_blocks_regq) * 128;
    TRY_ALLOC(h->topk_buf, cand_sets * kTopkCap, false);
    if (cfg->corpus_dtype == PROXIMITY_DTYPE_BF16 || h->coarse_capable) TRY_ALLOC(h->qplanes, 3 * B * d, true);
  }
  h->pairs_elems = long(B * lists * kp);
  TRY_ALLOC(h->pairs[0], size_t(h->pairs_elems), false);
  TRY_ALLOC(h->pairs[1], size_t(h->pairs_elems), false);
  TRY_ALLOC(h->res_ids, B * k, true);
  TRY_ALLOC(h->res_d, B * k, true);
  TRY_ALLOC(h->slack, 1, true);
  TRY_ALLOC(h->seed_bound, B, true);
  if (N > 0) {
    TRY_ALLOC(h->redo.list, B, true);
    TRY_ALLOC(h->redo.thr, B, true);
    TRY_ALLOC(h->redo.cnt, B, true);
    TRY_ALLOC(h->redo.wide, B * size_t(kWideCap), false);
  }
  if (h->coarse_capable) {
    // (pinned host memory the device writes through; without it the instance simply scans with two planes)
    void* note = nullptr;
    if (hipHostMalloc(&note, 64, hipHostMallocDefault) == hipSuccess && note) {
      std::memset(note, 0, 64);
      void* dev_view = nullptr;
      if (hipHostGetDevicePointer(&dev_view, note, 0) == hipSuccess && dev_view) {
        h->coarse_note = static_cast<int*>(note);
        h->redo.coarse_note = static_cast<int*>(dev_view);
      } else {
        (void)hipHostFree(note);
      }
    } else {
      (void)hipGetLastError();
    }
  }
  TRY_ALLOC(h->srcs, (c + B) * d, true);
  TRY_ALLOC(h->srcnrm, c + B, true);
  TRY_ALLOC(h->val_ids, c * k, true);
  TRY_ALLOC(h->val_d, c * k, true);
  TRY_ALLOC(h->slot_seq, c, true);
  TRY_ALLOC(h->slot_next, c, true);
  TRY_ALLOC(h->slot_prev, c, true);
  TRY_ALLOC(h->state, 1, true);
  h->ldD = long((c + B + 63) / 64 * 64);
  if (!lsh) {  // the dense probe and its candidate lists belong to the flat cache
    // rows per range: as many as two score buffers of that many rows fit the budget, 64..kProbeRangeRows
    const size_t R = probe_range_rows(c, B);
    h->probe_rows = int(R);
    const size_t score_rows = B <= R ? B : 2 * R;
    TRY_ALLOC(h->D32, score_rows * size_t(h->ldD), true);
    TRY_ALLOC(h->cand_cnt, B, true);
    TRY_ALLOC(h->cand_src, B * kCandCap, true);
    TRY_ALLOC(h->cand_d, B * kCandCap, true);
    TRY_ALLOC(h->ovf_cnt, (B + 63) / 64 + 4, true);
    TRY_ALLOC(h->ovf_list, B, true);
    TRY_ALLOC(h->live_slots, 1, true);
    TRY_ALLOC(h->res_image, kResolverLdsMax / sizeof(int), false);
    TRY_ALLOC(h->res_carry, 1, true);
    h->probe_ws_bytes = score_rows * size_t(h->ldD) * sizeof(float) + 3 * B * sizeof(int) +
                        B * kCandCap * (sizeof(int) + sizeof(double)) + kResolverLdsMax + sizeof(ResolverCarry);
    if (B > R) {
      const size_t ranges = B / 64 + 4;
      if (hipStreamCreateWithFlags(&h->side, hipStreamNonBlocking) != hipSuccess) {
        h->side = nullptr;
        h->err = "could not create the resolver's stream";
        return bail(PROXIMITY_ERR_HIP);
      }
      h->ev_probe.assign(ranges, nullptr);
      h->ev_go.assign(ranges, nullptr);
      h->ev_res.assign(ranges, nullptr);
      for (size_t i = 0; i < ranges; ++i)
        if (hipEventCreateWithFlags(&h->ev_probe[i], hipEventDisableTiming) != hipSuccess ||
            hipEventCreateWithFlags(&h->ev_go[i], hipEventDisableTiming) != hipSuccess ||
            hipEventCreateWithFlags(&h->ev_res[i], hipEventDisableTiming) != hipSuccess) {
          h->err = "could not create the events that order probe and resolver";
          return bail(PROXIMITY_ERR_HIP);
        }
    }
  } else {
    const size_t nb = size_t(1) << h->lsh_bits;
    TRY_ALLOC(h->lsh_planes, size_t(h->lsh_bits) * d, false);
    TRY_ALLOC(h->lsh_code, B, true);
    TRY_ALLOC(h->lsh_sorted, B, true);
    TRY_ALLOC(h->lsh_seg_start, B, true);
    TRY_ALLOC(h->lsh_n_segs, 1, true);
    TRY_ALLOC(h->bkt_size, nb, true);
    TRY_ALLOC(h->bkt_head, nb, false);
    TRY_ALLOC(h->bkt_tail, nb, false);
    if (hipMemcpy(h->lsh_planes, cfg->lsh_planes, size_t(h->lsh_bits) * d * sizeof(float), hipMemcpyDeviceToDevice) !=
            hipSuccess ||
        hipMemset(h->bkt_head, 0xff, nb * sizeof(int)) != hipSuccess ||
        hipMemset(h->bkt_tail, 0xff, nb * sizeof(int)) != hipSuccess) {
      h->err = "could not set up the bucketed cache";
      return bail(PROXIMITY_ERR_HIP);
    }
    h->cfg.lsh_planes = h->lsh_planes;
  }
  TRY_ALLOC(h->hit, B, true);
  TRY_ALLOC(h->src, B, true);
  TRY_ALLOC(h->row_slot, B, true);
  TRY_ALLOC(h->miss_list, B, true);
  TRY_ALLOC(h->miss_count, 1, true);
  TRY_ALLOC(h->D64, size_t(kSmallRows) * (c > 0 && !lsh ? c : 1), false);
#undef TRY_ALLOC
  if (hipFuncSetAttribute(reinterpret_cast<const void*>(resolver_lds_kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                          int(kResolverLdsMax)) != hipSuccess) {
    h->err = "could not raise the dynamic LDS limit of the resolver";
    return bail(PROXIMITY_ERR_HIP);
  }
  if (hipFuncSetAttribute(reinterpret_cast<const void*>(lsh_resolve_kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                          int(kLshLdsMax)) != hipSuccess) {
    h->err = "could not raise the dynamic LDS limit of the bucket resolver";
    return bail(PROXIMITY_ERR_HIP);
  }
  CacheState init{};
  init.head = init.tail = -1;
  if (hipMemcpy(h->state, &init, sizeof init, hipMemcpyHostToDevice) != hipSuccess) {
    h->err = "state upload failed";
    return bail(PROXIMITY_ERR_HIP);
  }
  if (N > 0) {
    if (cfg->corpus_dtype == PROXIMITY_DTYPE_BF16)
      launch_row_norms<kDtypeBF16>(h, cfg->corpus, long(N), int(d), h->xnrm, nullptr);
    else
      launch_row_norms<kDtypeF32>(h, cfg->corpus, long(N), int(d), h->xnrm, nullptr);
    {  // the largest row length, for the error bound of the float32 scores
      long g = (long(N) + 255) / 256;
      if (g > long(h->n_cu) * 8) g = long(h->n_cu) * 8;
      max_norm_kernel<<<dim3((unsigned)g), dim3(256)>>>(h->xnrm, long(N), h->slack);
    }
    if (cfg->metric != PROXIMITY_METRIC_L2) {
      long g = (long(N) + 255) / 256;
      if (g > long(h->n_cu) * 8) g = long(h->n_cu) * 8;
      row_terms_kernel<<<dim3((unsigned)g), dim3(256)>>>(h->xnrm, long(N), cfg->metric == PROXIMITY_METRIC_COSINE ? 1 : 0);
    }
    hipError_t e = hipGetLastError();
    if (e == hipSuccess) e = hipDeviceSynchronize();
    if (e != hipSuccess) {
      h->err = std::string("corpus norm pass failed: ") + hipGetErrorString(e);
      return bail(PROXIMITY_ERR_HIP);
    }
  }
  *out = h;
  return PROXIMITY_OK;
}

void proximity_destroy(proximity_t* h) {
  if (!h) return;
  DeviceGuard guard(h->cfg.device);
  (void)hipDeviceSynchronize();
  for (hipEvent_t e : h->ev0) (void)hipEventDestroy(e);
  for (hipEvent_t e : h->ev1) (void)hipEventDestroy(e);
  for (hipEvent_t e : h->ev_probe) if (e) (void)hipEventDestroy(e);
  for (hipEvent_t e : h->ev_go) if (e) (void)hipEventDestroy(e);
  for (hipEvent_t e : h->ev_res) if (e) (void)hipEventDestroy(e);
  if (h->side) (void)hipStreamDestroy(h->side);
  for (void* p : h->allocs) (void)hipFree(p);
  if (h->coarse_note) (void)hipHostFree(h->coarse_note);
  delete h;
}

int proximity_knn_batch(proximity_t* h, const float* queries, uint32_t n, uint32_t k, int64_t* out_ids,
                        float* out_dists, void* hip_stream) {
  int rc = validate_call(h, queries, n, k, out_ids);
  if (rc != PROXIMITY_OK) return rc;
  if (n == 0) return PROXIMITY_OK;
  DeviceGuard guard(h->cfg.device);
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  h->last_stream = s;
  SmallRouting no_cache{};
  rc = enqueue_scan(h, queries, nullptr, nullptr, int(n), int(k), int(k), out_ids, out_dists ? out_dists : h->res_d,
                    int(n) <= kSmallRows ? &no_cache : nullptr, s);
  if (h->prof_on) ++h->prof_call;
  if (rc != PROXIMITY_OK) return rc;
  return check_launch(h, "proximity_knn_batch");
}

int proximity_knn_static(const void* corpus, uint64_t n_docs, uint32_t dim, uint32_t corpus_dtype, uint32_t metric,
                         const float* queries, uint32_t n, uint32_t k, int64_t* out_ids, float* out_dists,
                         int32_t device, void* hip_stream) {
  // argument checks first: nothing is enqueued and nothing on the device changes when one fails
  if (dim == 0 || dim % 32 != 0 || dim > PROXIMITY_MAX_DIM)
    return fail(nullptr, PROXIMITY_ERR_INVALID_ARG, "dim=%u must be a multiple of 32 in 32..%u", dim, PROXIMITY_MAX_DIM);
  if (k == 0 || k > PROXIMITY_MAX_K)
    return fail(nullptr, PROXIMITY_ERR_INVALID_ARG, "k=%u must be in 1..%u", k, PROXIMITY_MAX_K);
  if (n_docs > kStaticMaxDocs)
    return fail(nullptr, PROXIMITY_ERR_INVALID_ARG,
                "n_docs=%llu exceeds PROXIMITY_STATIC_MAX_DOCS=%zu, the corpus size the library's built-in "
                "workspace holds (use proximity_create / proximity_knn_batch for larger corpora)",
                (unsigned long long)n_docs, kStaticMaxDocs);
  if (n > kStaticMaxQueries)
    return fail(nullptr, PROXIMITY_ERR_BATCH_TOO_LARGE, "n=%u exceeds PROXIMITY_STATIC_MAX_QUERIES=%zu", n,
                kStaticMaxQueries);
  if (corpus_dtype != PROXIMITY_DTYPE_F32 && corpus_dtype != PROXIMITY_DTYPE_BF16)
    return fail(nullptr, PROXIMITY_ERR_INVALID_ARG, "unknown corpus_dtype %u", corpus_dtype);
  if (metric > PROXIMITY_METRIC_COSINE) return fail(nullptr, PROXIMITY_ERR_INVALID_ARG, "unknown metric %u", metric);
  if (n_docs > 0 && !corpus) return fail(nullptr, PROXIMITY_ERR_INVALID_ARG, "corpus is null but n_docs > 0");
  if (n > 0 && (!queries || !out_ids)) return fail(nullptr, PROXIMITY_ERR_INVALID_ARG, "queries or out_ids is null");
  if (reinterpret_cast<uintptr_t>(corpus) % 16 != 0 || reinterpret_cast<uintptr_t>(queries) % 16 != 0)
    return fail(nullptr, PROXIMITY_ERR_INVALID_ARG, "corpus and queries must be 16-byte aligned");
  if (device < 0 || device >= kStaticMaxDevices)
    return fail(nullptr, PROXIMITY_ERR_INVALID_ARG, "device=%d must be in 0..%d", device, kStaticMaxDevices - 1);
  DeviceGuard guard(device);
  if (!guard.ok) return fail(nullptr, PROXIMITY_ERR_HIP, "device %d cannot be made current", device);

  // once per device: where this device keeps its copy of the workspace, and its size in compute units
  StaticDevice dev;
  {
    std::lock_guard<std::mutex> lock(g_static_mutex);
    StaticDevice& slot = g_static_dev[device];
    if (!slot.ptr) {
      void* p = nullptr;
      hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
      if (e != hipSuccess || !p)
        return fail(nullptr, PROXIMITY_ERR_HIP, "hipGetSymbolAddress(scratch) on device %d failed: %s", device,
                    hipGetErrorString(e));
      int n_cu = 0;
      e = hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, device);
      if (e != hipSuccess || n_cu <= 0)
        return fail(nullptr, PROXIMITY_ERR_HIP, "could not read the compute-unit count of device %d", device);
      slot.n_cu = n_cu;
      slot.ptr = static_cast<unsigned char*>(p);
    }
    dev = slot;
  }
  if (n == 0) return PROXIMITY_OK;

  // The search itself is the one proximity_knn_batch runs for a handful of queries (row terms, streaming
  // scores, selection, float64 ranking), with every buffer of the instance replaced by a piece of the
  // workspace.
  proximity view;
  view.cfg.dim = dim;
  view.cfg.corpus = corpus;
  view.cfg.n_docs = n_docs;
  view.cfg.corpus_dtype = corpus_dtype;
  view.cfg.k = k;
  view.cfg.metric = metric;
  view.cfg.max_batch = uint32_t(kStaticMaxQueries);
  view.K = int(k);
  view.n_cu = dev.n_cu;
  view.slack = reinterpret_cast<SlackState*>(dev.ptr + kStaticOffSlack);
  view.xnrm = reinterpret_cast<float*>(dev.ptr + kStaticOffNorms);
  view.S = reinterpret_cast<float*>(dev.ptr + kStaticOffScores);
  view.ldS = long(kStaticMaxDocs);
  view.pairs[0] = reinterpret_cast<uint64_t*>(dev.ptr + kStaticOffLists);
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  if (n_docs > 0) {
    // the one piece of the workspace that must start at zero: the state of the exactness check (the largest
    // row length is gathered with an atomic maximum); cleared by a kernel, not a memset, so that the call
    // can be captured into a graph
    slack_reset_kernel<<<dim3(1), dim3(256), 0, s>>>(view.slack);
    if (corpus_dtype == PROXIMITY_DTYPE_BF16)
      launch_row_norms<kDtypeBF16>(&view, corpus, long(n_docs), int(dim), view.xnrm, s);
    else
      launch_row_norms<kDtypeF32>(&view, corpus, long(n_docs), int(dim), view.xnrm, s);
    {
      long g = (long(n_docs) + 255) / 256;
      if (g > long(dev.n_cu) * 8) g = long(dev.n_cu) * 8;
      max_norm_kernel<<<dim3((unsigned)g), dim3(256), 0, s>>>(view.xnrm, long(n_docs), view.slack);
    }
    if (metric != PROXIMITY_METRIC_L2) {
      long g = (long(n_docs) + 255) / 256;
      if (g > long(dev.n_cu) * 8) g = long(dev.n_cu) * 8;
      row_terms_kernel<<<dim3((unsigned)g), dim3(256), 0, s>>>(view.xnrm, long(n_docs),
                                                               metric == PROXIMITY_METRIC_COSINE ? 1 : 0);
    }
  }
  SmallRouting no_cache{};
  int rc = enqueue_scan(&view, queries, nullptr, nullptr, int(n), int(k), int(k), out_ids, out_dists, &no_cache, s);
  if (rc != PROXIMITY_OK) return fail(nullptr, rc, "%s", view.err.c_str());
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(nullptr, PROXIMITY_ERR_HIP, "proximity_knn_static: %s", hipGetErrorString(e));
  return PROXIMITY_OK;
}

int proximity_search_batch(proximity_t* h, const float* queries, uint32_t n, uint32_t k, float tau,
                           int64_t* out_ids, float* out_dists, uint8_t* out_hit, void* hip_stream) {
  int rc = validate_call(h, queries, n, k, out_ids);
  if (rc != PROXIMITY_OK) return rc;
  if (!(tau >= 0.f) || std::isinf(tau)) return fail(h, PROXIMITY_ERR_BAD_TAU, "tau must be finite and >= 0");
  if (n == 0) return PROXIMITY_OK;
  if (!out_hit) return fail(h, PROXIMITY_ERR_INVALID_ARG, "out_hit is null");
  DeviceGuard guard(h->cfg.device);
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  h->last_stream = s;

  const int c = h->slots, dim = int(h->cfg.dim), kk = int(h->cfg.k), nn = int(n);
  const bool lsh = h->lsh_bits > 0;
  const long long base_seq = (long long)h->next_seq;
  float* batch_rows = h->srcs + size_t(c) * dim;
  const int xkind = corpus_kind(int(h->cfg.corpus_dtype), int(h->cfg.metric));
  // The cache compares query and key by the index's own distance (Section 3.1), in float64 on the vectors as
  // the caller gave them: Euclidean for the Euclidean index and for the inner-product index (whose negated
  // inner product is no distance between two queries), cosine distance for the cosine index.  tau is in
  // that distance's units.
  const double tau_key = double(tau);
  const int cos_keys = h->cfg.metric == PROXIMITY_METRIC_COSINE ? 1 : 0;

  const int K = h->K;
  if (nn <= kSmallRows && h->cfg.n_docs > 0 && !lsh) {
    // A handful of rows: five launches in all.  Cache side (probe in float64; then resolver, key
    // insertion, hits on resident keys), streaming scan for the rows that missed, and
    // selection; then merge + float64 ranking + routing.  The rows are read from the caller's buffer.
    const int grid = c > 0 ? ((c + 15) / 16 < h->n_cu ? (c + 15) / 16 : h->n_cu) : 1;
    for (int phase = 1; phase <= 2; ++phase) {
      probe_resolve_small_kernel<<<dim3(phase == 2 ? 1 : grid), dim3(1024), 0, s>>>(
          queries, nn, c, dim, kk, K, h->cfg.policy == PROXIMITY_POLICY_LRU ? 1 : 0, base_seq, tau_key, cos_keys,
          h->state, h->slot_seq, h->slot_next, h->slot_prev, h->srcs, h->srcnrm, h->val_ids, h->val_d, h->cfg.corpus,
          xkind, h->D64, phase, out_hit, h->src, h->row_slot, h->miss_list, h->miss_count, out_ids,
          out_dists);
    }
    const SmallRouting rt{out_hit, h->src, h->row_slot, h->slot_seq, h->val_ids, h->val_d, base_seq, nn, c};
    rc = enqueue_scan(h, queries, h->miss_list, h->miss_count, nn, K, kk, out_ids, out_dists, &rt, s);
    if (rc != PROXIMITY_OK) return rc;
    h->next_seq += n;
    if (h->prof_on) ++h->prof_call;
    return check_launch(h, "proximity_search_batch");
  }

  if (lsh && nn <= kSmallRows && h->cfg.n_docs > 0) {
    // A handful of rows on the bucketed cache: the cache side in one launch, then the same scan,
    // selection and routing launches as for the flat cache.
    lsh_small_kernel<<<dim3(1), dim3(1024), 0, s>>>(
        queries, nn, int(h->cfg.capacity), c, dim, kk, K, h->lsh_bits, h->lsh_planes,
        h->cfg.policy == PROXIMITY_POLICY_LRU ? 1 : 0, base_seq, tau_key, cos_keys, h->srcs, h->slot_seq, h->slot_next,
        h->slot_prev, h->bkt_size, h->bkt_head, h->bkt_tail, h->state, h->val_ids, h->val_d, h->cfg.corpus,
        xkind, out_hit, h->src, h->row_slot, h->miss_list, h->miss_count, out_ids, out_dists);
    const SmallRouting rt{out_hit, h->src, h->row_slot, h->slot_seq, h->val_ids, h->val_d, base_seq, nn, c};
    rc = enqueue_scan(h, queries, h->miss_list, h->miss_count, nn, K, kk, out_ids, out_dists, &rt, s);
    if (rc != PROXIMITY_OK) return rc;
    h->next_seq += n;
    if (h->prof_on) ++h->prof_call;
    return check_launch(h, "proximity_search_batch");
  }

  if (lsh)
    HIP_TRY(h, hipMemcpyAsync(batch_rows, queries, size_t(n) * dim * sizeof(float), hipMemcpyDeviceToDevice, s));
  if (lsh) {
    // Section 3.2: codes, regrouping by code, one block per bucket that occurs, miss list in row order
    const int b = int(h->cfg.capacity);
    lsh_codes_kernel<<<dim3((nn + 15) / 16), dim3(256), 0, s>>>(batch_rows, nn, dim, h->lsh_planes, h->lsh_bits,
                                                              h->lsh_code);
    lsh_group_kernel<<<dim3(1), dim3(1024), 0, s>>>(h->lsh_code, nn, h->lsh_sorted, h->lsh_seg_start, h->lsh_n_segs);
    const int max_segs = nn < (1 << h->lsh_bits) ? nn : (1 << h->lsh_bits);  // distinct codes a batch can have
    // the bucket's keys stay in LDS while its block walks, when b * dim floats fit
    const size_t row_bytes = size_t(dim) * sizeof(float);
    const int keys_in_lds = (size_t(b) + 1) * row_bytes <= kLshLdsMax ? 1 : 0;
    lsh_resolve_kernel<<<dim3(max_segs), dim3(kLshThreads), (keys_in_lds ? size_t(b) + 1 : 1) * row_bytes, s>>>(
        h->lsh_sorted, h->lsh_seg_start, h->lsh_n_segs, nn, b, c, dim, h->cfg.policy == PROXIMITY_POLICY_LRU ? 1 : 0, base_seq, tau_key, cos_keys, keys_in_lds,
        batch_rows,
        h->srcs, h->slot_seq, h->slot_next, h->slot_prev, h->bkt_size, h->bkt_head, h->bkt_tail, h->state, out_hit,
        h->src, h->row_slot);
    lsh_miss_list_kernel<<<dim3(1), dim3(1024), 0, s>>>(out_hit, nn, h->miss_list, h->miss_count, h->state);
  } else {
  // the rows into the batch buffer and their norms, in one launch
  copy_rows_norms_kernel<<<dim3((nn + 3) / 4), dim3(256), 0, s>>>(queries, nn, dim, batch_rows, h->srcnrm + c);
  const int have_probe = c > 0 ? 1 : 0;
  const int lru = h->cfg.policy == PROXIMITY_POLICY_LRU ? 1 : 0;
  // Candidate lists of rows r0 .. r1-1 (range g) against the slots and the batch rows before them.
  // Euclidean keys of the dimensions the register-resident kernel is built for: that kernel lists the candidates
  // itself, and dense scores are made for the rows whose list overflowed only (worth its set-up from a couple
  // of thousand sources on).  Otherwise: dense scores of every row of the range, and the lists from those.
  const bool listing = have_probe && !cos_keys && regq_supported(kDtypeF32, dim) && nn >= 64 && long(c) + nn >= 2048;
  if (listing)
    probe_prepare_kernel<<<dim3((nn + 255) / 256), dim3(256), 0, s>>>(nn, h->cand_cnt, (nn + 63) / 64 + 4, h->ovf_cnt,
                                                                       h->state, h->live_slots);
  auto enqueue_probe = [&](int g, int r0, int r1, float* D, bool beside_resolver) {
    const int rows = r1 - r0, n_src = c + r1;
    const float* Q = batch_rows + size_t(r0) * dim;
    if (listing) {
      // Blocks: 64 rows each, a slice's sources shared by the blocks that serve it; one block per CU.  Beside the
      // resolver, whose block needs a CU to itself, eight CUs stay free: workgroups go to the eight XCDs in turn
      // whatever their load, so a free CU helps the resolver only if it is in the XCD its block is sent to
      // (with 255 blocks the resolver waited for most of a probe).
      const int slices = (rows + 63) / 64, tiles = (n_src + 127) / 128;
      long nb = h->n_cu - (beside_resolver ? 8 : 0);
      if (nb > long(slices) * tiles) nb = long(slices) * tiles;
      if (nb < slices) nb = slices;
      const RegqEmit em{c,         h->live_slots,  tau_key,         kCandCap, h->cand_cnt, h->cand_src,
                        h->cand_d, h->ovf_cnt + g, h->ovf_list + r0, nullptr,      0};
      prof_begin(h, s);
      if (dim == 768)
        scan_regq_kernel<kDtypeF32, 768, 4, kRegqProbe><<<dim3((unsigned)nb), dim3(256), 0, s>>>(
            h->srcs, h->srcnrm, n_src, batch_rows, nullptr, nullptr, 0, nullptr, r1, r0, slices, 0, 0, nullptr, nullptr,
            nullptr, 0, em);
      else
        scan_regq_kernel<kDtypeF32, 384, 4, kRegqProbe><<<dim3((unsigned)nb), dim3(256), 0, s>>>(
            h->srcs, h->srcnrm, n_src, batch_rows, nullptr, nullptr, 0, nullptr, r1, r0, slices, 0, 0, nullptr, nullptr,
            nullptr, 0, em);
      prof_end(h, s, r0, rows, PROXIMITY_LAUNCH_PROBE);
      return;   // (enqueue_lists follows, on the stream that resolves the range)
    }
    if (nn <= kStreamMaxQueries) {
      const int mq = stream_group(dim, nn);
      for (int m0 = 0; m0 < nn; m0 += mq)
        launch_scores_stream<kDtypeF32, false>(h, mq, h->srcs, h->srcnrm, long(c) + nn, dim, batch_rows, nullptr, nullptr,
                                        nn, m0, D + size_t(m0) * h->ldD, h->ldD, 0, s);
    } else if (long((n_src + 31) / 32) * ((rows + 31) / 32) <= kProbeSmallBlocks) {
      probe_mfma_small_kernel<<<dim3((n_src + 31) / 32, (rows + 31) / 32), dim3(256), 0, s>>>(
          h->srcs, h->srcnrm, n_src, Q, rows, dim, D, h->ldD);
    } else {
      probe_mfma_dense_kernel<<<dim3((n_src + 127) / 128, (rows + 127) / 128), dim3(256), 0, s>>>(
          h->srcs, h->srcnrm, n_src, Q, rows, dim, D, h->ldD);
    }
    probe_candidates_kernel<<<dim3(rows), dim3(256), 0, s>>>(D, h->ldD, h->srcs, h->srcnrm, dim, c, nn, h->state, tau_key,
                                                             cos_keys, kCandCap, h->cand_cnt, h->cand_src, h->cand_d, r0);
  };
  // After the listing probe: dense scores for the rows whose list overflowed (none, as a rule).
  auto enqueue_lists = [&](int g, int r0, int r1, float* D, hipStream_t rs) {
    probe_mfma_dense_listed_kernel<<<dim3(h->n_cu), dim3(256), 0, rs>>>(h->srcs, h->srcnrm, c + r1, batch_rows, dim, D, h->ldD,
                                                                         h->ovf_list + r0, h->ovf_cnt + g, r0);
  };
  // The sequential resolver over rows r0 .. r1-1, with its state in LDS whenever that fits.
  // Bringing the eviction order on chip costs about 2.5 ns per key; walking it in device memory about
  // 1.5 us per row.  A few rows against a large cache are cheaper in place.
  const bool few_rows = long(nn) * 600 < long(c);
  const bool in_lds = have_probe && !few_rows && resolver_lds_fits(size_t(c), size_t(nn), kResolverLdsMax);
  auto enqueue_resolver = [&](int r0, int r1, const float* D, hipStream_t rs) {
    // (beside a probe the block asks for all the LDS it may have: no block of the probe then shares its CU, whose
    // waves would otherwise take issue slots from the one wave that walks the rows)
    if (in_lds)
      resolver_lds_kernel<<<dim3(1), dim3(kResolverThreads),
                            rs == s ? resolver_lds_bytes(size_t(c), size_t(nn)) : kResolverLdsMax, rs>>>(
          nn, c, dim, lru, base_seq, tau_key, cos_keys, h->state, h->slot_seq, h->slot_next, h->slot_prev, h->cand_cnt,
          h->cand_src, h->cand_d, kCandCap, D, h->ldD, h->srcs, h->srcnrm, out_hit, h->src, h->row_slot, h->miss_list,
          h->miss_count, r0, r1, r0 == 0 ? 1 : 0, r1 == nn ? 1 : 0, h->res_image, h->res_carry);
    else
      resolver_kernel<<<dim3(1), dim3(64), 0, rs>>>(nn, c, dim, lru, base_seq, tau_key, cos_keys, h->state, h->slot_seq,
                                                    h->slot_next, h->slot_prev, have_probe ? h->cand_cnt : nullptr,
                                                    h->cand_src, h->cand_d, kCandCap, D, h->ldD, h->srcs, h->srcnrm,
                                                    out_hit, h->src, h->row_slot, h->miss_list, h->miss_count, r0, r1);
  };
  const int R = h->probe_rows;
  if (!have_probe || nn <= R) {
    if (have_probe) enqueue_probe(0, 0, nn, h->D32, false);
    if (listing) enqueue_lists(0, 0, nn, h->D32, s);
    enqueue_resolver(0, nn, h->D32, s);
  } else {
    // Row ranges: the probe of a range on the caller's stream, its resolution on the side stream, which so walks
    // a range while the next one is being multiplied.  What is left when the last probe ends is the resolution
    // of the last range, so the last rows go in two short ranges (probe_range_cuts).  The side stream joins the
    // caller's stream before anything else is enqueued.
    int cut[PROXIMITY_MAX_BATCH / 64 + 4];
    const int ranges = probe_range_cuts(nn, R, c, listing, h->n_cu, cut);
    for (int g = 0; g < ranges; ++g) {
      const int r0 = g ? cut[g - 1] : 0, r1 = cut[g];
      float* D = h->D32 + size_t(g & 1) * size_t(R) * size_t(h->ldD);
      if (listing) {
        // The listing kernel leaves one CU free (the resolver block needs one to itself), so the probes follow
        // each other without regard to the resolver.  The (as a rule empty) launch for overflowed rows stays on
        // this stream: beside a probe that holds every register of its CUs it would wait for room.  It writes a
        // score buffer, which the resolver of two ranges ago has left by now unless it is far behind.
        enqueue_probe(g, r0, r1, D, true);
        if (g >= 2) HIP_TRY(h, hipStreamWaitEvent(s, h->ev_res[g - 2], 0));
        enqueue_lists(g, r0, r1, D, s);
        HIP_TRY(h, hipEventRecord(h->ev_probe[g], s));
        HIP_TRY(h, hipStreamWaitEvent(h->side, h->ev_probe[g], 0));
        enqueue_resolver(r0, r1, D, h->side);
      } else {
        // A score buffer is written again two ranges later, once the resolver has left it.  The dense probe
        // fills every CU and the resolver block needs one to itself: the probe is held until the side stream has
        // reached the resolver of the range before, which so is dispatched first.
        if (g >= 2) HIP_TRY(h, hipStreamWaitEvent(s, h->ev_res[g - 2], 0));
        if (g >= 1) HIP_TRY(h, hipStreamWaitEvent(s, h->ev_go[g - 1], 0));
        enqueue_probe(g, r0, r1, D, g >= 1);
        HIP_TRY(h, hipEventRecord(h->ev_probe[g], s));
        HIP_TRY(h, hipStreamWaitEvent(h->side, h->ev_probe[g], 0));
        HIP_TRY(h, hipEventRecord(h->ev_go[g], h->side));
        enqueue_resolver(r0, r1, D, h->side);
      }
      HIP_TRY(h, hipEventRecord(h->ev_res[g], h->side));
    }
    HIP_TRY(h, hipStreamWaitEvent(s, h->ev_res[ranges - 1], 0));
  }
  }
  const void* X = h->cfg.n_docs > 0 ? h->cfg.corpus : nullptr;
  const int xdt = xkind;
  post_resolve_kernel<<<dim3(nn), dim3(256), 0, s>>>(nn, c, dim, kk, K, lsh ? 0 : 1, base_seq, h->srcs, h->srcnrm, h->slot_seq,
                                                     out_hit, h->src, h->row_slot, h->val_ids, h->val_d, X, xdt,
                                                     out_ids, out_dists);
  rc = enqueue_scan(h, batch_rows, h->miss_list, h->miss_count, nn, K, K, h->res_ids, h->res_d, nullptr, s);
  if (rc != PROXIMITY_OK) return rc;
  finalize_kernel<<<dim3(nn), dim3(256), 0, s>>>(nn, c, kk, K, base_seq, h->slot_seq, out_hit, h->src, h->row_slot,
                                                 h->res_ids, h->res_d, h->val_ids, h->val_d, batch_rows, dim, X, xdt,
                                                 out_ids, out_dists);
  h->next_seq += n;
  if (h->prof_on) ++h->prof_call;
  return check_launch(h, "proximity_search_batch");
}

int proximity_stats(const proximity_t* h, proximity_stats_t* out) {
  if (!h || !out) return fail(const_cast<proximity_t*>(h), PROXIMITY_ERR_INVALID_ARG, "handle or out is null");
  proximity* hh = const_cast<proximity*>(h);
  DeviceGuard guard(h->cfg.device);
  HIP_TRY(hh, hipStreamSynchronize(h->last_stream));
  CacheState st;
  HIP_TRY(hh, hipMemcpy(&st, h->state, sizeof st, hipMemcpyDeviceToHost));
  std::memset(out, 0, sizeof *out);
  out->queries = st.queries;
  out->hits = st.hits;
  out->misses = st.misses;
  out->inserts = st.inserts;
  out->evictions = st.evictions;
  out->size = uint64_t(st.size);
  out->inbatch_hits = st.inbatch_hits;
  out->dense_resolves = st.dense_resolves;
  SlackState sl;
  HIP_TRY(hh, hipMemcpy(&sl, h->slack, sizeof sl, hipMemcpyDeviceToHost));
  out->slack_exhausted = sl.exhausted;
  out->slack_unresolved = sl.unresolved;
  out->probe_workspace_bytes = h->probe_ws_bytes;
  out->coarse_scan_calls = h->coarse_calls;
  out->coarse_scan_fails = uint64_t(sl.coarse_fails);
  return PROXIMITY_OK;
}

int proximity_cache_dump(const proximity_t* h, uint64_t* seq, float* keys, int64_t* ids, uint32_t* n_live) {
  if (!h || !n_live) return fail(const_cast<proximity_t*>(h), PROXIMITY_ERR_INVALID_ARG, "handle or n_live is null");
  proximity* hh = const_cast<proximity*>(h);
  DeviceGuard guard(h->cfg.device);
  HIP_TRY(hh, hipStreamSynchronize(h->last_stream));
  const size_t c = size_t(h->slots), d = h->cfg.dim, k = size_t(h->K);  // K = rerank_factor * k ids per key
  CacheState st;
  HIP_TRY(hh, hipMemcpy(&st, h->state, sizeof st, hipMemcpyDeviceToHost));
  std::vector<long long> sseq(c);
  std::vector<int> snext(c);
  if (c) {
    HIP_TRY(hh, hipMemcpy(sseq.data(), h->slot_seq, c * sizeof(long long), hipMemcpyDeviceToHost));
    HIP_TRY(hh, hipMemcpy(snext.data(), h->slot_next, c * sizeof(int), hipMemcpyDeviceToHost));
  }
  // whole arrays in one copy each, then gathered in eviction order on the host
  std::vector<float> all_keys;
  std::vector<int64_t> all_ids;
  if (keys && c) {
    all_keys.resize(c * d);
    HIP_TRY(hh, hipMemcpy(all_keys.data(), h->srcs, c * d * sizeof(float), hipMemcpyDeviceToHost));
  }
  if (ids && c) {
    all_ids.resize(c * k);
    HIP_TRY(hh, hipMemcpy(all_ids.data(), h->val_ids, c * k * sizeof(int64_t), hipMemcpyDeviceToHost));
  }
  // one eviction order (flat cache), or one per bucket, buckets in ascending code
  std::vector<int> heads(1, st.head);
  if (h->lsh_bits > 0) {
    heads.resize(size_t(1) << h->lsh_bits);
    HIP_TRY(hh, hipMemcpy(heads.data(), h->bkt_head, heads.size() * sizeof(int), hipMemcpyDeviceToHost));
  }
  uint32_t count = 0;
  for (int first : heads)
    for (int t = first; t >= 0 && count < c; t = snext[size_t(t)]) {
      if (seq) seq[count] = uint64_t(sseq[size_t(t)]);
      if (keys) std::memcpy(keys + size_t(count) * d, all_keys.data() + size_t(t) * d, d * sizeof(float));
      if (ids) std::memcpy(ids + size_t(count) * k, all_ids.data() + size_t(t) * k, k * sizeof(int64_t));
      ++count;
    }
  *n_live = count;
  return PROXIMITY_OK;
}

int proximity_clear(proximity_t* h) {
  if (!h) return fail(nullptr, PROXIMITY_ERR_INVALID_ARG, "handle is null");
  DeviceGuard guard(h->cfg.device);
  HIP_TRY(h, hipDeviceSynchronize());
  CacheState init{};
  init.head = init.tail = -1;
  HIP_TRY(h, hipMemcpy(h->state, &init, sizeof init, hipMemcpyHostToDevice));
  if (h->lsh_bits > 0) {
    const size_t nb = size_t(1) << h->lsh_bits;
    HIP_TRY(h, hipMemset(h->bkt_size, 0, nb * sizeof(int)));
    HIP_TRY(h, hipMemset(h->bkt_head, 0xff, nb * sizeof(int)));
    HIP_TRY(h, hipMemset(h->bkt_tail, 0xff, nb * sizeof(int)));
  }
  HIP_TRY(h, hipMemset(&h->slack->exhausted, 0, 2 * sizeof(unsigned long long)));
  h->next_seq = 0;
  return PROXIMITY_OK;
}

int proximity_profile_start(proximity_t* h) {
  if (!h) return fail(nullptr, PROXIMITY_ERR_INVALID_ARG, "handle is null");
  DeviceGuard guard(h->cfg.device);
  if (h->ev0.empty()) {
    h->ev0.resize(kMaxProfiled);
    h->ev1.resize(kMaxProfiled);
    h->ev_info.resize(kMaxProfiled);
    for (int i = 0; i < kMaxProfiled; ++i) {
      HIP_TRY(h, hipEventCreate(&h->ev0[i]));
      HIP_TRY(h, hipEventCreate(&h->ev1[i]));
    }
  }
  h->ev_used = 0;
  h->prof_call = 0;
  h->prof_on = true;
  return PROXIMITY_OK;
}

int proximity_profile_stop(proximity_t* h, proximity_launch_t* records, uint32_t cap, uint32_t* n_records) {
  if (!h) return fail(nullptr, PROXIMITY_ERR_INVALID_ARG, "handle is null");
  if (n_records) *n_records = 0;
  if (cap > 0 && !records) return fail(h, PROXIMITY_ERR_INVALID_ARG, "records is null but cap > 0");
  DeviceGuard guard(h->cfg.device);
  h->prof_on = false;
  HIP_TRY(h, hipStreamSynchronize(h->last_stream));
  uint32_t w = 0;
  for (size_t i = 0; i < h->ev_used; ++i) {
    float ms = 0.f;
    HIP_TRY(h, hipEventElapsedTime(&ms, h->ev0[i], h->ev1[i]));
    // launches of one call for the same queries (one per tile shape): one record, that of the longest -- the
    // others returned at once
    if (w > 0 && records[w - 1].call == h->ev_info[i].call && records[w - 1].first_query == h->ev_info[i].first_query &&
        records[w - 1].kind == h->ev_info[i].kind) {
      if (ms > records[w - 1].ms) {
        records[w - 1] = h->ev_info[i];
        records[w - 1].ms = ms;
      }
      continue;
    }
    if (w >= cap) break;
    records[w] = h->ev_info[i];
    records[w].ms = ms;
    ++w;
  }
  if (n_records) *n_records = w;
  h->ev_used = 0;
  return PROXIMITY_OK;
}

}  // extern "C"
