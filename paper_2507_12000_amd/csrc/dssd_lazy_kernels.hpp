// Early-exit verification: the loop of Algorithm 2 ("while j <= gamma and Flag = 1") taken at its
// word.  Row i of a session decides position i, and nothing after the first rejection is ever
// looked at, so the rows are visited in a few rounds of growing blocks -- rows [0,k1) of every
// session, then rows [k1,k2) of the sessions still without a rejection, and so on -- and a
// session leaves as soon as one of its blocks holds a rejection or its bonus row.  On the
// benchmark workloads this reads a little over half of the logits.
//
// Each round is the streaming pair again (chunk statistics, then one workgroup per session for
// the accept scan), restricted to the block and to the sessions still open, which the accept
// launch of the round before has appended to a list.  Every value that is computed is computed
// by the same device functions in the same order as in the default path, so accepted_len,
// rejected, out_token and the statistics of visited rows are bit-identical to its results.
// Nothing waits on another workgroup; every launch has a grid fixed by the host and workgroups
// without work exit at once.
#pragma once
#include "dssd_kernels.hpp"

namespace dssd {

constexpr int kMaxRounds = 8;

// Lengths of a round's two lists in one word, so that a session is appended to both with a
// single atomic: sessions in the high half, rows in the low half.
using ListLengths = unsigned long long;
__device__ __forceinline__ int32_t listed_sessions(ListLengths n) { return (int32_t)(n >> 32); }
__device__ __forceinline__ int32_t listed_rows(ListLengths n) { return (int32_t)(n & 0xFFFFFFFFull); }

// Sessions of a round: all of them (list == nullptr) or the listed_sessions(*lengths) entries of `list`.
struct OpenSessions {
  const int32_t* list;
  const ListLengths* lengths;
};
// One logits row to take statistics of, with its session's log2(e)/T.
struct __attribute__((aligned(16))) RowTask {
  int64_t lrow;
  float c1;
  int32_t pad;
};

// Round 0: chunk statistics of rows [0, width) of every session, one wave per chunk.
// zero[0..n_zero) is cleared by the first threads (the list lengths of the rounds that follow).
template <bool BF16, bool ALIGNED, bool SUPPORT>
__global__ __launch_bounds__(256) void row_chunk_stats_head(const BatchView a, int32_t width, ListLengths* zero,
                                                            int32_t n_zero) {
  // wave-uniform 32-bit arithmetic up to the loads, as in row_chunk_stats (the host refuses
  // batches with 2^31 chunk tasks or more)
  const int lane = threadIdx.x & 63;
  const uint32_t wave = (uint32_t)__builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
  if (blockIdx.x == 0 && threadIdx.x < n_zero) zero[threadIdx.x] = 0;
  const uint32_t C = (uint32_t)a.C;
  const uint32_t per_session = (uint32_t)width * C;
  const uint32_t task = xcd_contiguous32(blockIdx.x, gridDim.x, a) * 4 + wave;
  if (task >= (uint32_t)a.B * per_session) return;
  const int32_t b = (int32_t)(task / per_session);
  const uint32_t rem = task - (uint32_t)b * per_session;
  const int32_t i = (int32_t)(rem / C), c = (int32_t)(rem - (rem / C) * C);
  const int64_t off0 = session_first_draft(a, b);
  const int64_t off1 = a.offsets ? (int64_t)a.offsets[b + 1] : off0 + a.gamma;
  if (off0 < 0 || off1 < off0 || off1 > a.R_Q) return;   // reported by the accept launch
  if (i > off1 - off0) return;                            // the session has fewer rows
  const int64_t lrow = off0 + b + i;
  SupportRow sup{};
  if constexpr (SUPPORT)
    sup = SupportRow{a.support_count + lrow, a.support_idx + lrow * kMaxSupport, a.support_z + lrow * kMaxSupport};
  auto c1_of = [&]() { return (a.inv_temp ? a.inv_temp[b] : 1.f) * kLog2e; };
  const float2 st = chunk_stats_of<BF16, ALIGNED, SUPPORT>(logits_row<BF16>(a, lrow), c, a.V, c1_of, lane, sup);
  if (lane == 0) a.chunk_stats[lrow * a.C + c] = st;
}

// Later rounds: chunk statistics of the rows the accept launch before has listed, one wave per
// chunk, grid-stride (the grid is fixed by the host, the list length is not known there).
template <bool BF16, bool ALIGNED, bool SUPPORT>
__global__ __launch_bounds__(256) void row_chunk_stats_list(const BatchView a, const RowTask* rows,
                                                            const ListLengths* lengths) {
  const int lane = threadIdx.x & 63;
  const uint32_t wave = (uint32_t)__builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
  const uint32_t C = (uint32_t)a.C;
  const uint32_t total = (uint32_t)listed_rows(*lengths) * C;   // below 2^31: the listed rows are rows of the batch
  // each XCD walks one contiguous share of the list (the grid is a multiple of the XCD count)
  const uint32_t xcds = (uint32_t)a.xcds;
  const uint32_t nblk = (total + 3) / 4, per = (nblk + xcds - 1) / xcds;
  const uint32_t first = (blockIdx.x % xcds) * per;
  for (uint32_t k = blockIdx.x / xcds; k < per; k += gridDim.x / xcds) {
    const uint32_t task = (first + k) * 4 + wave;
    if (task >= total) continue;
    const uint32_t e = task / C;
    const int32_t c = (int32_t)(task - e * C);
    const RowTask t = rows[e];
    SupportRow sup{};
    if constexpr (SUPPORT)
      sup = SupportRow{a.support_count + t.lrow, a.support_idx + t.lrow * kMaxSupport,
                       a.support_z + t.lrow * kMaxSupport};
    const float2 st = chunk_stats_of<BF16, ALIGNED, SUPPORT>(logits_row<BF16>(a, t.lrow), c, a.V, [=]() { return t.c1; }, lane, sup);
    if (lane == 0) a.chunk_stats[t.lrow * a.C + c] = st;
  }
}

// Accept scan of rows [row_begin, row_end) for every open session, one workgroup per session.
// A session that stays open is appended to next_list, and its next rows -- next_width of them,
// or all that are left -- to next_rows (one atomic on the packed lengths does both).  TAIL_BONUS: a session whose drafts were all accepted
// also gets its bonus token here.
template <bool BF16, bool ALIGNED, bool TAIL_BONUS>
__global__ __launch_bounds__(256) void accept_scan_block(const BatchView a, OpenSessions open, int32_t row_begin,
                                                         int32_t row_end, int32_t* next_list, RowTask* next_rows,
                                                         ListLengths* next_lengths, int32_t next_width) {
  __shared__ ListLengths sh_at;
  if (open.list && (int32_t)blockIdx.x >= listed_sessions(*open.lengths)) return;
  const int32_t b = open.list ? open.list[blockIdx.x] : (int32_t)blockIdx.x;
  Job job;
  const int32_t kind = accept_session<BF16>(a, b, &job, row_begin, row_end, true);
  if (kind == 3) {
    // still open: offsets were found consistent, and row_end <= gamma_b
    const int64_t off0 = session_first_draft(a, b);
    const int32_t g = (int32_t)((a.offsets ? (int64_t)a.offsets[b + 1] : off0 + a.gamma) - off0);
    const int32_t n = min(next_width, g + 1 - row_end);
    if (threadIdx.x == 0) sh_at = atomicAdd(next_lengths, (1ull << 32) | (ListLengths)n);
    __syncthreads();
    const ListLengths at = sh_at;
    if (threadIdx.x == 0) next_list[listed_sessions(at)] = b;
    const float c1 = (a.inv_temp ? a.inv_temp[b] : 1.f) * kLog2e;
    for (int32_t k = threadIdx.x; k < n; k += blockDim.x) {
      RowTask t;
      t.lrow = off0 + b + row_end + k; t.c1 = c1; t.pad = 0;
      next_rows[listed_rows(at) + k] = t;
    }
    return;
  }
  if constexpr (TAIL_BONUS)
    if (kind == 2 && threadIdx.x < kWave) pick_for_session<BF16, ALIGNED, false>(a, b, job, threadIdx.x);
}

}  // namespace dssd
