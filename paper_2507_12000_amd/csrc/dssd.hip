// C ABI of the DSSD verification library (see include/dssd.h, include/dssd_aux.h): argument checks, workspace,
// kernel launches, optional per-kernel event timing.  No step of the method runs on the host.
#include "../../include/dssd_aux.h"

#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <mutex>
#include <new>
#include <type_traits>

#include "dssd_fused_kernels.hpp"
#include "dssd_util_kernels.hpp"
#include "dssd_lazy_kernels.hpp"
#include "dssd_topk_kernels.hpp"
#include "dssd_split_kernels.hpp"

using namespace dssd;

static_assert(kMaxSupport == DSSD_MAX_SUPPORT, "header and kernels must agree on the support size");

// Workspace of dssd_step_static: one array per device, part of the loaded code object, so the
// call never has to allocate.  In host code this name is only a handle for
// hipGetSymbolAddress; the device address it yields (one per device) is what kernels and
// copies receive.
static __device__ __align__(256) unsigned char scratch[DSSD_STATIC_SCRATCH_BYTES];

namespace {
// What the launches need to know about a device; the defaults are the MI355X's.
struct DeviceFacts {
  int32_t xcds = 8;
  int32_t cus = 256;
  int64_t lds_per_cu = 160 << 10;
};
DeviceFacts read_device_facts(int device) {
  DeviceFacts f;
  int attr = 0;
  if (hipDeviceGetAttribute(&attr, hipDeviceAttributeNumberOfXccs, device) == hipSuccess && attr >= 1) f.xcds = attr;
  else (void)hipGetLastError();
  if (hipDeviceGetAttribute(&attr, hipDeviceAttributeMultiprocessorCount, device) == hipSuccess && attr >= 1) f.cus = attr;
  else (void)hipGetLastError();
  if (hipDeviceGetAttribute(&attr, hipDeviceAttributeMaxSharedMemoryPerMultiprocessor, device) == hipSuccess &&
      attr >= (64 << 10))
    f.lds_per_cu = attr;
  else (void)hipGetLastError();
  return f;
}

constexpr int kMaxDevices = 64;
std::mutex scratch_lock;
void* scratch_ptr[kMaxDevices] = {};       // device address of device d's copy of `scratch`, once resolved
DeviceFacts scratch_facts[kMaxDevices];    // and that device's facts

// Address of the CURRENT device's copy of `scratch`, resolved on the first request per device.
dssd_status current_scratch(void** ptr, DeviceFacts* facts) {
  int device = -1;
  if (hipGetDevice(&device) != hipSuccess) { (void)hipGetLastError(); return DSSD_EHIP; }
  if (device < 0 || device >= kMaxDevices) return DSSD_EUNSUPPORTED;
  std::lock_guard<std::mutex> hold(scratch_lock);
  if (!scratch_ptr[device]) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) { (void)hipGetLastError(); return DSSD_EHIP; }
    scratch_facts[device] = read_device_facts(device);
    scratch_ptr[device] = p;
  }
  *ptr = scratch_ptr[device];
  *facts = scratch_facts[device];
  return DSSD_OK;
}
}  // namespace

struct dssd_ctx {
  int device = 0;
  int32_t xcds = 8;                  // XCDs of the device, read at creation
  int32_t cus = 256;                 // compute units of the device
  int64_t lds_per_cu = 160 << 10;    // LDS bytes of one compute unit
  // Streaming kernels run fastest with a moderate number of bytes in flight per compute unit
  // (measured: read throughput peaks at 10 to 16 waves of 8 KiB and falls off by several percent
  // towards full occupancy).  The caps below are waves per compute unit, enforced by asking for
  // LDS the kernels never touch; 0 = whatever the registers allow.  Until the caller sets them the
  // statistics kernels run at 12 waves for bf16 logits and 10 for fp32, the residual masses at 12
  // and 16.
  int32_t stats_waves_per_cu = 12;
  int32_t resid_waves_per_cu = 16;
  bool stats_cap_auto = true;
  int64_t max_rows = 0;
  int32_t max_V = 0;
  int32_t max_C = 0;
  void* workspace = nullptr;
  float2* chunk_stats = nullptr;
  float2* row_tab = nullptr;
  float* resid_mass = nullptr;
  Job* resid_job = nullptr;
  Job* bonus_job = nullptr;
  int32_t* arrive_resid = nullptr;
  int32_t* arrive_stats = nullptr;
  int32_t* open_list[2] = {nullptr, nullptr};   // early exit: sessions open in odd / even rounds
  RowTask* open_rows[2] = {nullptr, nullptr};   // and the rows such a round takes statistics of
  int32_t ee_begin[kMaxRounds] = {0};           // early-exit schedule set by the caller (ee_rounds > 0)
  int ee_rounds = 0;
  ListLengths* open_count = nullptr;            // [kMaxRounds]: lengths of the lists of round r
  int32_t* support_count = nullptr;
  int32_t* support_idx = nullptr;
  float* support_z = nullptr;
  uint32_t profile_mask = 0;         // bit k: time kernel k
  bool fused_force = false;          // set by dssd_set_fused_limit with a negative limit: ignore the row-size rule
  int64_t fused_max_blocks = 512;    // dssd_step_fused: largest grid that runs as one launch
  int64_t pair_max_blocks = 512;     // dssd_step_fused: largest grid that runs as two launches
  // Timing brackets: a fixed pool of event pairs per kernel, created by dssd_profile_enable.
  hipEvent_t* ev_begin[DSSD_K_COUNT] = {};
  hipEvent_t* ev_end[DSSD_K_COUNT] = {};
  size_t ev_cap[DSSD_K_COUNT] = {};
  size_t ev_used[DSSD_K_COUNT] = {};
  size_t ev_dropped[DSSD_K_COUNT] = {};   // brackets skipped because the pool was exhausted
  bool ev_failed = false;                  // an event could not be recorded: the next hot call reports it
};
constexpr size_t kEventPool = 2048;        // brackets per kernel between two resets

static inline int32_t chunks_per_row(int32_t V, int32_t dtype) {
  const int32_t ce = dtype == DSSD_BF16 ? chunk_elems<true>() : chunk_elems<false>();
  return (V + ce - 1) / ce;
}
static inline size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

extern "C" size_t dssd_workspace_bytes(int64_t max_rows, int32_t max_V, int32_t logits_dtype) {
  if (max_rows < 1 || max_V < 1) return 0;
  const size_t C = (size_t)chunks_per_row(max_V, logits_dtype);
  const size_t rows = (size_t)max_rows;
  return align256(rows * C * sizeof(float2)) + align256(rows * sizeof(float2)) +
         align256(rows * C * sizeof(float)) + 2 * align256(rows * sizeof(Job)) +
         align256(2 * rows * sizeof(int32_t)) + align256(rows * sizeof(int32_t)) +
         2 * align256(rows * kMaxSupport * sizeof(int32_t)) + 2 * align256(rows * sizeof(int32_t)) + 2 * align256(rows * sizeof(RowTask)) + 256;
}

extern "C" const char* dssd_status_str(dssd_status s) {
  switch (s) {
    case DSSD_OK: return "ok";
    case DSSD_EINVAL: return "invalid argument";
    case DSSD_EALIGN: return "misaligned pointer";
    case DSSD_ENOMEM: return "batch exceeds workspace or allocation failed";
    case DSSD_EHIP: return "HIP runtime error";
    case DSSD_EUNSUPPORTED: return "unsupported";
  }
  return "unknown status";
}

extern "C" const char* dssd_kernel_name(int k) {
  static const char* names[DSSD_K_COUNT] = {"row_chunk_stats", "accept_scan", "resid_mass", "resid_pick",
                                            "bonus_pick", "export_p_rows", "device_resid_mass",
                                            "device_resid_pick", "fused_small_step", "read_probe",
                                            "row_chunk_stats_block", "topk_step"};
  return (k >= 0 && k < DSSD_K_COUNT) ? names[k] : "?";
}

extern "C" dssd_status dssd_create(dssd_ctx** out, int device, int64_t max_rows, int32_t max_V) {
  if (!out || max_rows < 1 || max_V < 1 || device < 0) return DSSD_EINVAL;
  *out = nullptr;
  int count = 0;
  if (hipGetDeviceCount(&count) != hipSuccess || device >= count) return DSSD_EHIP;
  int previous = -1;
  if (hipGetDevice(&previous) != hipSuccess) previous = -1;
  if (hipSetDevice(device) != hipSuccess) return DSSD_EHIP;
  // the caller's current device is put back on every way out
  struct Restore { int d; ~Restore() { if (d >= 0) (void)hipSetDevice(d); } } restore{previous};
  dssd_ctx* c = new (std::nothrow) dssd_ctx;
  if (!c) return DSSD_ENOMEM;
  c->device = device;
  const DeviceFacts facts = read_device_facts(device);
  c->xcds = facts.xcds; c->cus = facts.cus; c->lds_per_cu = facts.lds_per_cu;
  c->max_rows = max_rows;
  c->max_V = max_V;
  c->max_C = chunks_per_row(max_V, DSSD_F32);  // fp32 chunks hold fewer elements: the larger count
  const size_t bytes = dssd_workspace_bytes(max_rows, max_V, DSSD_F32);
  if (hipMalloc(&c->workspace, bytes) != hipSuccess) {
    (void)hipGetLastError();
    delete c;
    return DSSD_ENOMEM;
  }
  char* p = static_cast<char*>(c->workspace);
  const size_t rows = (size_t)max_rows, C = (size_t)c->max_C;
  c->chunk_stats = reinterpret_cast<float2*>(p); p += align256(rows * C * sizeof(float2));
  c->row_tab = reinterpret_cast<float2*>(p);     p += align256(rows * sizeof(float2));
  c->resid_mass = reinterpret_cast<float*>(p);   p += align256(rows * C * sizeof(float));
  c->resid_job = reinterpret_cast<Job*>(p);      p += align256(rows * sizeof(Job));
  c->bonus_job = reinterpret_cast<Job*>(p);      p += align256(rows * sizeof(Job));
  c->arrive_resid = reinterpret_cast<int32_t*>(p);
  c->arrive_stats = c->arrive_resid + rows;           p += align256(2 * rows * sizeof(int32_t));
  c->support_count = reinterpret_cast<int32_t*>(p);   p += align256(rows * sizeof(int32_t));
  c->support_idx = reinterpret_cast<int32_t*>(p);     p += align256(rows * kMaxSupport * sizeof(int32_t));
  c->support_z = reinterpret_cast<float*>(p);         p += align256(rows * kMaxSupport * sizeof(float));
  c->open_list[0] = reinterpret_cast<int32_t*>(p);    p += align256(rows * sizeof(int32_t));
  c->open_list[1] = reinterpret_cast<int32_t*>(p);    p += align256(rows * sizeof(int32_t));
  c->open_rows[0] = reinterpret_cast<RowTask*>(p);    p += align256(rows * sizeof(RowTask));
  c->open_rows[1] = reinterpret_cast<RowTask*>(p);    p += align256(rows * sizeof(RowTask));
  c->open_count = reinterpret_cast<ListLengths*>(p);
  // arrival counters start at zero; every kernel that uses them leaves them at zero
  if (hipMemset(c->arrive_resid, 0, 2 * rows * sizeof(int32_t)) != hipSuccess || hipDeviceSynchronize() != hipSuccess) {
    (void)hipFree(c->workspace);
    delete c;
    return DSSD_EHIP;
  }
  {   // the static scratch of this device is resolved here too, so that a later dssd_step_static
      // on it has nothing left to set up (a failure only matters to that call, which repeats it)
    void* p; DeviceFacts f;
    (void)current_scratch(&p, &f);
  }
  *out = c;
  return DSSD_OK;
}

extern "C" void dssd_destroy(dssd_ctx* c) {
  if (!c) return;
  for (int k = 0; k < DSSD_K_COUNT; ++k) {
    for (size_t i = 0; i < c->ev_cap[k]; ++i) {
      (void)hipEventDestroy(c->ev_begin[k][i]);
      (void)hipEventDestroy(c->ev_end[k][i]);
    }
    delete[] c->ev_begin[k];
    delete[] c->ev_end[k];
  }
  if (c->workspace) (void)hipFree(c->workspace);
  delete c;
}

// Host-side checks shared by the three hot calls.  Fills the kernel argument block.
static dssd_status check_and_view(const dssd_ctx* c, const dssd_batch* b, const dssd_out* o, BatchView* v,
                                  bool need_out = true) {
  static const dssd_out no_out = {};
  if (!need_out && !o) o = &no_out;
  if (!c || !b || !o) return DSSD_EINVAL;
  if (b->B < 0 || b->V < 1 || b->gamma < 0 || b->total_drafts < 0) return DSSD_EINVAL;
  if (b->logits_dtype != DSSD_F32 && b->logits_dtype != DSSD_BF16) return DSSD_EINVAL;
  if (b->flags & ~(uint32_t)(DSSD_FLAG_SPARSE_SUPPORT | DSSD_FLAG_EARLY_EXIT)) return DSSD_EINVAL;
  if (!b->draft_offsets && b->total_drafts != (int64_t)b->B * b->gamma) return DSSD_EINVAL;
  if (b->B > 0) {
    if (!b->logits) return DSSD_EINVAL;
    if (need_out && (!o->accepted_len || !o->rejected || !o->out_token)) return DSSD_EINVAL;
    if (b->total_drafts > 0 && (!b->draft_tokens || (!b->draft_probs && !b->draft_q_tok))) return DSSD_EINVAL;
  }
  const uintptr_t esz = b->logits_dtype == DSSD_BF16 ? 2 : 4;
  auto mis = [](const void* p, uintptr_t a) { return p && (reinterpret_cast<uintptr_t>(p) % a) != 0; };
  if (mis(b->logits, esz) || mis(b->draft_probs, 4) || mis(b->draft_q_tok, 4) || mis(b->draft_tokens, 4) || mis(b->draft_offsets, 4) ||
      mis(b->inv_temperature, 4) || mis(o->accepted_len, 4) || mis(o->rejected, 4) || mis(o->out_token, 4) ||
      mis(o->row_stats, 4) || mis(o->p_tok, 4) || mis(o->q_tok, 4) || mis(o->status, 4) ||
      mis(b->step_counter, 8))
    return DSSD_EALIGN;
  const int64_t R_L = b->total_drafts + b->B;
  const int32_t C = chunks_per_row(b->V, b->logits_dtype);
  if (R_L > c->max_rows || b->V > c->max_V || C > c->max_C) return DSSD_ENOMEM;
  v->B = b->B; v->V = b->V; v->gamma = b->gamma; v->C = C; v->xcds = c->xcds;
  v->xcd_shift = -1;
  for (int sh = 0; sh < 16; ++sh)
    if ((1 << sh) == c->xcds) v->xcd_shift = sh;
  v->R_L = R_L; v->R_Q = b->total_drafts;
  v->offsets = b->draft_offsets; v->logits = b->logits; v->draft_probs = b->draft_probs;
  v->q_scalars = b->draft_probs ? nullptr : b->draft_q_tok;   // Q rows win when both are given
  v->tokens = b->draft_tokens; v->inv_temp = b->inv_temperature;
  v->seed_lo = (uint32_t)b->seed; v->seed_hi = (uint32_t)(b->seed >> 32);
  v->step_lo = (uint32_t)b->step; v->step_hi = (uint32_t)(b->step >> 32);
  v->step_dev = b->step_counter;
  v->session_base = b->session_base;
  v->accepted_len = o->accepted_len; v->rejected = o->rejected; v->out_token = o->out_token;
  v->row_stats = o->row_stats; v->p_tok = o->p_tok; v->q_tok = o->q_tok; v->status = o->status;
  v->chunk_stats = c->chunk_stats; v->row_tab = c->row_tab; v->resid_mass = c->resid_mass;
  v->resid_job = c->resid_job; v->bonus_job = c->bonus_job; v->arrive_resid = c->arrive_resid;
  v->support_count = c->support_count; v->support_idx = c->support_idx; v->support_z = c->support_z;
  return DSSD_OK;
}

// 128-bit loads need 16-byte aligned rows: aligned bases and V a multiple of the vector width.
static bool vector_ok(const dssd_batch* b) {
  const int per_vec = b->logits_dtype == DSSD_BF16 ? 8 : 4;
  auto al16 = [](const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; };
  return (b->V % per_vec) == 0 && al16(b->logits) && al16(b->draft_probs);   // a null pointer counts as aligned
}

namespace {
// Brackets one launch with a pair of events from the kernel's pool.  Nothing is created here:
// a pool that is used up drops the bracket (dssd_profile_read then says so), a stream that is
// being captured into a graph is left alone, and a record that fails is reported by the hot
// call through launch_status(c).
struct Timed {
  dssd_ctx* c; int k; hipStream_t s; hipEvent_t end = nullptr;
  Timed(dssd_ctx* c_, int k_, hipStream_t s_) : c(c_), k(k_), s(s_) {
    if (!((c->profile_mask >> k) & 1u)) return;
    hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(s, &cap) != hipSuccess) { (void)hipGetLastError(); c->ev_failed = true; return; }
    if (cap != hipStreamCaptureStatusNone) return;
    if (c->ev_used[k] >= c->ev_cap[k]) { ++c->ev_dropped[k]; return; }
    const size_t i = c->ev_used[k];
    if (hipEventRecord(c->ev_begin[k][i], s) != hipSuccess) { (void)hipGetLastError(); c->ev_failed = true; return; }
    ++c->ev_used[k];
    end = c->ev_end[k][i];
  }
  ~Timed() {
    if (end && hipEventRecord(end, s) != hipSuccess) { (void)hipGetLastError(); c->ev_failed = true; }
  }
};
}  // namespace

#define DSSD_LAUNCH_WG(kernel, grid, threads, lds, stream, ...)                                        \
  do {                                                                                                 \
    hipLaunchKernelGGL(kernel, dim3((unsigned)(grid)), dim3((unsigned)(threads)), lds, stream, __VA_ARGS__); \
  } while (0)
#define DSSD_LAUNCH(kernel, grid, stream, ...) DSSD_LAUNCH_WG(kernel, grid, 256, 0, stream, __VA_ARGS__)

// Dynamic LDS (bytes per workgroup, never touched by the kernel) that lets at most
// waves_per_cu / wg_waves workgroups share a compute unit: just more than an (n+1)-th of the
// unit's LDS.  One workgroup per unit would need more than a launch may ask for: two is the floor.
// Small grids (under 64 waves per unit in all) are left alone: they are bound by latency, not by
// the memory system.
static unsigned occupancy_cap_lds(const dssd_ctx* c, int wg_waves, int waves_per_cu, int64_t grid) {
  if (waves_per_cu <= 0 || grid * wg_waves < (int64_t)64 * c->cus) return 0;
  const int64_t n = std::max(waves_per_cu / wg_waves, 2);
  const int64_t bytes = (c->lds_per_cu / (n + 1) / 512 + 1) * 512;
  return (unsigned)std::min<int64_t>(bytes, 64 << 10);
}

// Threads of a session's workgroup in the accept kernels: four waves (each merges rows of its own)
// while the chip can hold four waves for every session at once, fewer for larger batches, whose
// workgroups would otherwise queue up behind each other for work a single wave does in one pass.
static unsigned accept_threads(const dssd_ctx* c, int32_t B) {
  const int64_t resident = (int64_t)c->cus * 32;   // waves the chip holds at eight per SIMD
  return (unsigned)(kWave * std::min<int64_t>(4, std::max<int64_t>(1, resident / std::max(B, 1))));
}

// Waves per compute unit for a statistics launch, and for one of the residual masses.
static int32_t stats_waves_for(const dssd_ctx* c, bool bf16) {
  return c->stats_cap_auto && !bf16 ? 10 : c->stats_waves_per_cu;
}
static int32_t resid_waves_for(const dssd_ctx* c, bool bf16) {
  return c->stats_cap_auto && bf16 ? 12 : c->resid_waves_per_cu;
}

static dssd_status launch_status(const dssd_ctx* c) {
  const bool launched = hipGetLastError() == hipSuccess;
  return launched && !c->ev_failed ? DSSD_OK : DSSD_EHIP;
}

// Run-time booleans to template arguments: f receives one std::bool_constant per flag, in order.
// FLAG(x) is the compile-time value of such an argument.
template <class F> static void with_flags(F&& f) { f(); }
template <class F, class... Rest> static void with_flags(F&& f, bool first, Rest... rest) {
  if (first) with_flags([&](auto... r) { f(std::true_type{}, r...); }, rest...);
  else       with_flags([&](auto... r) { f(std::false_type{}, r...); }, rest...);
}
#define FLAG(x) decltype(x)::value

// Early exit: rounds of (chunk statistics of a block of rows, accept scan of that block) over the
// sessions that are still open.  `begin` holds the first row of every block; the last block is
// open-ended.  Blocks grow because the share of open sessions shrinks geometrically while every
// round costs two launches.
struct Schedule { int32_t begin[kMaxRounds]; int n; };

// Which blocks, if any.  The host does not know how the drafts will fare, so it prices the
// candidates with a fixed per-position acceptance of 0.8 (the middle of what speculative pairs
// reach): rows a schedule leaves unread, times the row size, against about 20 us of extra
// launches per round beyond the first, i.e. 140 MB of streaming.  Measured on the benchmark
// workloads and a sweep of shapes: {0,2,6} wins from a few GB of logits on, {0,3} below that,
// and small batches or short sessions are better off reading everything.
static Schedule early_exit_schedule(const dssd_ctx* c, const dssd_batch* b, const BatchView& v) {
  if (c->ee_rounds > 0) {
    Schedule s{}; s.n = c->ee_rounds;
    for (int r = 0; r < s.n; ++r) s.begin[r] = c->ee_begin[r];
    return s;
  }
  static const Schedule candidates[2] = {{{0, 3}, 2}, {{0, 2, 6}, 3}};
  const double rows = (double)v.R_L / std::max(b->B, 1);   // rows per session (mean, if ragged)
  const double row_bytes = (double)b->V * (b->logits_dtype == DSSD_BF16 ? 2 : 4);
  const double alpha = 0.8, round_cost_bytes = 140e6;
  Schedule best{{0}, 0};
  double best_gain = 0.0;
  for (const Schedule& s : candidates) {
    double read = 0.0, open = 1.0;   // open = share of sessions that reach the block
    int rounds = 0;
    for (int r = 0; r < s.n && s.begin[r] < rows; ++r) {
      const double end = r + 1 < s.n ? std::min<double>(s.begin[r + 1], rows) : rows;
      read += open * (end - s.begin[r]);
      open = std::pow(alpha, end);
      ++rounds;
    }
    const double gain = (rows - read) * b->B * row_bytes - (rounds - 1) * round_cost_bytes;
    if (rounds > 1 && gain > best_gain) { best_gain = gain; best = s; }
  }
  return best;
}

static dssd_status early_exit_launches(dssd_ctx* c, const dssd_batch* b, const BatchView& v, hipStream_t s,
                                       bool tail_bonus, const Schedule& sched) {
  const bool bf16 = b->logits_dtype == DSSD_BF16, al = vector_ok(b);
  const bool sparse = (b->flags & DSSD_FLAG_SPARSE_SUPPORT) != 0;
  if (sparse) {   // support lists start empty; the bonus draw comes from them, in dssd_bonus_sample
    hipLaunchKernelGGL(zero_i32, dim3((unsigned)((v.R_L + 255) / 256)), dim3(256), 0, s, v.support_count, v.R_L);
    tail_bonus = false;
  }
  const int32_t* kEarlyExitBegin = sched.begin;
  const int kEarlyExitRounds = sched.n;
  const int32_t known_rows = b->draft_offsets ? 0x7FFFFFFF : b->gamma + 1;   // rows per session, if uniform
  for (int r = 0; r < kEarlyExitRounds; ++r) {
    const int32_t begin = kEarlyExitBegin[r];
    if (begin >= known_rows) break;
    const bool last = r == kEarlyExitRounds - 1 || kEarlyExitBegin[r + 1] >= known_rows;
    const int32_t end = last ? 0x7FFFFFFF : kEarlyExitBegin[r + 1];
    {
      Timed t(c, DSSD_K_ROW_STATS_BLOCK, s);
      if (r == 0) {
        const int32_t w = std::min(end, known_rows);
        if ((int64_t)b->B * w * v.C > 0x7FFFFFFFll) return DSSD_EUNSUPPORTED;   // 32-bit chunk indices
        // (this kernel measured best in four-wave workgroups at 16 waves per unit: 0.5-2 % faster
        // for the whole mode than the two-wave workgroups of row_chunk_stats at any cap)
        const int64_t blocks = ((int64_t)b->B * w * v.C + 3) / 4;
        const int32_t waves_per_cu = c->stats_cap_auto ? 16 : c->stats_waves_per_cu;
        with_flags([&](auto BF, auto AL, auto SP) {
          DSSD_LAUNCH_WG((row_chunk_stats_head<FLAG(BF), FLAG(AL), FLAG(SP)>), blocks, 256,
                         occupancy_cap_lds(c, 4, waves_per_cu, blocks), s, v, w, c->open_count, kMaxRounds);
        }, bf16, al, sparse);
      } else {
        // the rows listed by the accept launch before: at most every row that is left
        const int64_t rows_left = b->draft_offsets ? v.R_L : (int64_t)b->B * (known_rows - begin);
        const int64_t worst = last ? rows_left : std::min<int64_t>(rows_left, (int64_t)b->B * (end - begin));
        const int64_t blocks = (std::min<int64_t>((worst * v.C + 3) / 4, 1 << 16) + c->xcds - 1) / c->xcds * c->xcds;
        const RowTask* rows = c->open_rows[r & 1];
        with_flags([&](auto BF, auto AL, auto SP) {
          DSSD_LAUNCH((row_chunk_stats_list<FLAG(BF), FLAG(AL), FLAG(SP)>), blocks, s, v, rows, c->open_count + r);
        }, bf16, al, sparse);
      }
    }
    {
      Timed t(c, DSSD_K_ACCEPT, s);
      const OpenSessions open{r ? c->open_list[r & 1] : nullptr, r ? c->open_count + r : nullptr};
      int32_t* next_list = last ? nullptr : c->open_list[(r + 1) & 1];
      RowTask* next_rows = last ? nullptr : c->open_rows[(r + 1) & 1];
      ListLengths* next_lengths = last ? nullptr : c->open_count + r + 1;
      // the round after next starts at begin[r + 2]: the next one takes the rows in between, or all
      const int32_t next_width = last ? 0 : (r + 2 < kEarlyExitRounds ? kEarlyExitBegin[r + 2] - end : 0x7FFFFFFF);
      with_flags([&](auto BF, auto AL, auto TB) {
        DSSD_LAUNCH_WG((accept_scan_block<FLAG(BF), FLAG(AL), FLAG(TB)>), b->B, accept_threads(c, b->B), 0, s, v, open,
                       begin, end, next_list, next_rows, next_lengths, next_width);
      }, bf16, al, tail_bonus);
    }
    if (last) break;
  }
  return launch_status(c);
}

// Row statistics, then accept / first-reject per session.  tail_bonus: the accept kernel also
// draws the bonus token of all-accepted sessions (dense rows only).
static dssd_status verify_launches(dssd_ctx* c, const dssd_batch* b, const BatchView& v, hipStream_t s,
                                   bool tail_bonus) {
  const bool bf16 = b->logits_dtype == DSSD_BF16, al = vector_ok(b);
  const int64_t tasks = v.R_L * v.C;
  if (tasks > 0x7FFFFFFFll) return DSSD_EUNSUPPORTED;   // the kernels index chunks with 32 bits
  const unsigned grid = (unsigned)((tasks + kStatsWaves - 1) / kStatsWaves);
  const bool sparse = (b->flags & DSSD_FLAG_SPARSE_SUPPORT) != 0;
  if (b->flags & DSSD_FLAG_EARLY_EXIT) {
    const Schedule sched = early_exit_schedule(c, b, v);
    if (sched.n > 0) return early_exit_launches(c, b, v, s, tail_bonus, sched);
  }
  if (sparse)   // the rows' support lists start empty (a fill kernel, so the call stays graph-capturable)
    hipLaunchKernelGGL(zero_i32, dim3((unsigned)((v.R_L + 255) / 256)), dim3(256), 0, s, v.support_count, v.R_L);
  {
    Timed t(c, DSSD_K_ROW_STATS, s);
    const int32_t waves_per_cu = stats_waves_for(c, bf16);
    with_flags([&](auto BF, auto AL, auto SP) {
      DSSD_LAUNCH_WG((row_chunk_stats<FLAG(BF), FLAG(AL), FLAG(SP)>), grid, kStatsWaves * kWave,
                     occupancy_cap_lds(c, kStatsWaves, waves_per_cu, grid), s, v);
    }, bf16, al, sparse);
  }
  {
    Timed t(c, DSSD_K_ACCEPT, s);
    const unsigned g2 = (unsigned)b->B;   // one workgroup per session
    if (tail_bonus && !sparse)
      with_flags([&](auto BF, auto AL) {
        DSSD_LAUNCH_WG((accept_scan_bonus<FLAG(BF), FLAG(AL)>), g2, accept_threads(c, b->B), 0, s, v);
      }, bf16, al);
    else
      with_flags([&](auto BF) { DSSD_LAUNCH_WG((accept_scan<FLAG(BF)>), g2, accept_threads(c, b->B), 0, s, v); }, bf16);
  }
  return launch_status(c);
}

extern "C" dssd_status dssd_verify_batch(dssd_ctx* c, const dssd_batch* b, dssd_out* o, void* hip_stream) {
  BatchView v;
  const dssd_status st = check_and_view(c, b, o, &v);
  if (st != DSSD_OK || b->B == 0) return st;
  return verify_launches(c, b, v, static_cast<hipStream_t>(hip_stream), false);
}

extern "C" dssd_status dssd_residual_sample(dssd_ctx* c, const dssd_batch* b, dssd_out* o, void* hip_stream) {
  BatchView v;
  const dssd_status st = check_and_view(c, b, o, &v);
  if (st != DSSD_OK || b->B == 0) return st;
  if (b->total_drafts == 0) return DSSD_OK;   // nothing can have been rejected
  if (!b->draft_probs) return DSSD_EINVAL;    // the residual needs the full Q rows
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  const bool bf16 = b->logits_dtype == DSSD_BF16, al = vector_ok(b);
  if (b->flags & DSSD_FLAG_SPARSE_SUPPORT) {   // draw from the recorded support: no pass over V
    Timed t(c, DSSD_K_RESID_PICK, s);
    const unsigned g2 = (unsigned)((b->B + 3) / 4);
    with_flags([&](auto BF) { DSSD_LAUNCH((pick_sparse<FLAG(BF), true>), g2, s, v); }, bf16);
    return launch_status(c);
  }
  const int32_t groups = (v.C + 3) / 4;
  if ((int64_t)groups * b->B > 0x7FFFFFFFll) return DSSD_EUNSUPPORTED;
  const unsigned grid = (unsigned)(groups * b->B);
  // Few workgroups: one launch, the last workgroup of each session to finish its chunk masses
  // draws the token.  Many: the arrival (a store that must be acknowledged, a barrier, an atomic
  // that must return) holds every workgroup's wave slots a few microseconds longer with nothing
  // in flight, which costs a streaming kernel more than the second launch does.
  // (swept on the benchmark workloads: folding wins up to about a thousand workgroups and loses
  // from two thousand on)
  constexpr int64_t kResidFuseLimit = 1024;
  const bool fuse = (int64_t)grid <= kResidFuseLimit;
  {
    Timed t(c, DSSD_K_RESID_MASS, s);
    with_flags([&](auto BF, auto AL, auto FP) {
      DSSD_LAUNCH_WG((resid_mass<FLAG(BF), FLAG(AL), FLAG(FP)>), grid, 256, occupancy_cap_lds(c, 4, resid_waves_for(c, bf16), grid), s, v, groups);
    }, bf16, al, fuse);
  }
  if (!fuse) {
    Timed t(c, DSSD_K_RESID_PICK, s);
    const unsigned g2 = (unsigned)((b->B + 3) / 4);
    with_flags([&](auto BF, auto AL) { DSSD_LAUNCH((pick_token<FLAG(BF), FLAG(AL), true>), g2, s, v); }, bf16, al);
  }
  return launch_status(c);
}

extern "C" dssd_status dssd_bonus_sample(dssd_ctx* c, const dssd_batch* b, dssd_out* o, void* hip_stream) {
  BatchView v;
  const dssd_status st = check_and_view(c, b, o, &v);
  if (st != DSSD_OK || b->B == 0) return st;
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  const bool bf16 = b->logits_dtype == DSSD_BF16, al = vector_ok(b);
  if (b->flags & DSSD_FLAG_SPARSE_SUPPORT) {
    Timed t(c, DSSD_K_BONUS_PICK, s);
    const unsigned g2 = (unsigned)((b->B + 3) / 4);
    with_flags([&](auto BF) { DSSD_LAUNCH((pick_sparse<FLAG(BF), false>), g2, s, v); }, bf16);
    return launch_status(c);
  }
  {
    Timed t(c, DSSD_K_BONUS_PICK, s);
    const unsigned g2 = (unsigned)((b->B + 3) / 4);
    with_flags([&](auto BF, auto AL) { DSSD_LAUNCH((pick_token<FLAG(BF), FLAG(AL), false>), g2, s, v); }, bf16, al);
  }
  return launch_status(c);
}

// The whole step in one call: what Algorithm 1 does at the edge (accept/reject, redraw on a
// rejection, bonus token otherwise).  Small batches with uniform gamma run as a single launch;
// everything else is the three calls in a row.
static dssd_status step_fused_launches(dssd_ctx* c, const dssd_batch* b, dssd_out* o, const BatchView& v,
                                       void* hip_stream);

extern "C" dssd_status dssd_step_fused(dssd_ctx* c, const dssd_batch* b, dssd_out* o, void* hip_stream) {
  BatchView v;
  const dssd_status st = check_and_view(c, b, o, &v);
  if (st != DSSD_OK || b->B == 0) return st;
  if (b->total_drafts > 0 && !b->draft_probs) return DSSD_EINVAL;
  return step_fused_launches(c, b, o, v, hip_stream);
}

static dssd_status step_fused_launches(dssd_ctx* c, const dssd_batch* b, dssd_out* o, const BatchView& v,
                                       void* hip_stream) {
  const int64_t groups = ((int64_t)(b->gamma + 1) * v.C + 3) / 4;
  // One launch pays only while the lone workgroup that finishes a session can stream the
  // rejected row (logits + Q) quickly: small grids and rows of a few hundred KiB.
  const int64_t resid_row_bytes = (int64_t)b->V * ((b->logits_dtype == DSSD_BF16 ? 2 : 4) + 4);
  const bool early_exit = (b->flags & DSSD_FLAG_EARLY_EXIT) && early_exit_schedule(c, b, v).n > 0;
  const bool fusable = !b->draft_offsets && !(b->flags & DSSD_FLAG_SPARSE_SUPPORT) && !early_exit;
  const bool single = fusable && groups * b->B <= c->fused_max_blocks &&
                      (c->fused_force || resid_row_bytes <= (384 << 10));
  // Longer rows, still a small grid: statistics + accept + bonus in one launch, the redraw of
  // rejected sessions in a second one that every workgroup of the chip can share.
  const bool pair = fusable && !single && groups * b->B <= c->pair_max_blocks;
  if (!single && !pair) {
    // The streaming kernels, with the bonus draw folded into the accept launch where the rows
    // are dense: one launch fewer than the three calls, the same device functions.
    const bool sparse = (b->flags & DSSD_FLAG_SPARSE_SUPPORT) != 0;
    dssd_status r = verify_launches(c, b, v, static_cast<hipStream_t>(hip_stream), true);
    if (r == DSSD_OK) r = dssd_residual_sample(c, b, o, hip_stream);
    if (r == DSSD_OK && sparse) r = dssd_bonus_sample(c, b, o, hip_stream);
    return r;
  }
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  const bool bf16 = b->logits_dtype == DSSD_BF16, al = vector_ok(b);
  {
    Timed t(c, DSSD_K_FUSED_STEP, s);
    const int32_t g32 = (int32_t)(((int64_t)(b->gamma + 1) * v.C + kFusedWaves - 1) / kFusedWaves);
    const unsigned grid = (unsigned)((int64_t)g32 * b->B);
    with_flags([&](auto BF, auto AL, auto TR) {
      DSSD_LAUNCH_WG((fused_small_step<FLAG(BF), FLAG(AL), FLAG(TR)>), grid, kFusedWaves * kWave, 0, s, v, g32,
                     c->arrive_stats);
    }, bf16, al, single);
  }
  if (pair && b->total_drafts > 0) {
    const dssd_status r = launch_status(c);
    return r == DSSD_OK ? dssd_residual_sample(c, b, o, hip_stream) : r;
  }
  return launch_status(c);
}

// The whole step on the static scratch array: no context, no allocation.
extern "C" dssd_status dssd_step_static(const dssd_batch* b, dssd_out* o, void* hip_stream) {
  if (!b || !o) return DSSD_EINVAL;
  if (b->B < 0 || b->V < 1 || b->gamma < 0 || b->total_drafts < 0) return DSSD_EINVAL;
  if (b->logits_dtype != DSSD_F32 && b->logits_dtype != DSSD_BF16) return DSSD_EINVAL;
  if (b->flags & ~(uint32_t)(DSSD_FLAG_SPARSE_SUPPORT | DSSD_FLAG_EARLY_EXIT)) return DSSD_EINVAL;
  if (b->flags) return DSSD_EUNSUPPORTED;   // both modes need lists beyond the static scratch
  // Carve the scratch for this batch; refuse what does not fit before anything touches the device.
  const int32_t C = chunks_per_row(b->V, b->logits_dtype);
  if (b->total_drafts > (int64_t)1 << 40) return DSSD_ENOMEM;
  const size_t rows = (size_t)(b->total_drafts + b->B), B = (size_t)b->B;
  if (rows * (size_t)C > DSSD_STATIC_SCRATCH_BYTES) return DSSD_ENOMEM;
  const size_t at_chunk_stats = 0;
  const size_t at_row_tab = at_chunk_stats + align256(rows * C * sizeof(float2));
  const size_t at_resid_mass = at_row_tab + align256(rows * sizeof(float2));
  const size_t at_resid_job = at_resid_mass + align256(B * C * sizeof(float));
  const size_t at_bonus_job = at_resid_job + align256(B * sizeof(Job));
  const size_t at_arrive = at_bonus_job + align256(B * sizeof(Job));
  const size_t end = at_arrive + align256(2 * B * sizeof(int32_t));
  if (end > DSSD_STATIC_SCRATCH_BYTES) return DSSD_ENOMEM;
  void* base = nullptr;
  DeviceFacts facts;
  const dssd_status got = current_scratch(&base, &facts);
  if (got != DSSD_OK) return got;
  char* p = static_cast<char*>(base);
  dssd_ctx c;   // a view of the scratch with the library's default settings; owns nothing
  c.xcds = facts.xcds; c.cus = facts.cus; c.lds_per_cu = facts.lds_per_cu;
  c.max_rows = (int64_t)rows; c.max_V = b->V; c.max_C = C;
  c.chunk_stats = reinterpret_cast<float2*>(p + at_chunk_stats);
  c.row_tab = reinterpret_cast<float2*>(p + at_row_tab);
  c.resid_mass = reinterpret_cast<float*>(p + at_resid_mass);
  c.resid_job = reinterpret_cast<Job*>(p + at_resid_job);
  c.bonus_job = reinterpret_cast<Job*>(p + at_bonus_job);
  c.arrive_resid = reinterpret_cast<int32_t*>(p + at_arrive);
  c.arrive_stats = c.arrive_resid + B;
  BatchView v;
  const dssd_status st = check_and_view(&c, b, o, &v);
  if (st != DSSD_OK || b->B == 0) return st;
  if (b->total_drafts > 0 && !b->draft_probs) return DSSD_EINVAL;
  // The array keeps whatever the last call left, carved for another batch: the arrival
  // counters must start at zero (a fill kernel, not a memset node, so the call can be captured).
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  hipLaunchKernelGGL(zero_i32, dim3((unsigned)((2 * B + 255) / 256)), dim3(256), 0, s, c.arrive_resid, (int64_t)(2 * B));
  return step_fused_launches(&c, b, o, v, hip_stream);
}

extern "C" dssd_status dssd_set_fused_limit(dssd_ctx* c, int64_t max_blocks) {
  if (!c) return DSSD_EINVAL;
  c->fused_force = max_blocks < 0;
  c->fused_max_blocks = max_blocks < 0 ? -max_blocks : max_blocks;
  return DSSD_OK;
}

extern "C" dssd_status dssd_set_early_exit_schedule(dssd_ctx* c, const int32_t* begin, int32_t n) {
  if (!c || n < 0 || n == 1 || n > kMaxRounds || (n > 0 && (!begin || begin[0] != 0))) return DSSD_EINVAL;
  for (int r = 1; r < n; ++r)
    if (begin[r] <= begin[r - 1]) return DSSD_EINVAL;
  for (int r = 0; r < n; ++r) c->ee_begin[r] = begin[r];
  c->ee_rounds = n;
  return DSSD_OK;
}

extern "C" dssd_status dssd_set_stream_occupancy(dssd_ctx* c, int32_t stats_waves_per_cu, int32_t resid_waves_per_cu) {
  if (!c || stats_waves_per_cu < 0 || resid_waves_per_cu < 0) return DSSD_EINVAL;
  c->stats_waves_per_cu = stats_waves_per_cu;
  c->resid_waves_per_cu = resid_waves_per_cu;
  c->stats_cap_auto = false;
  return DSSD_OK;
}

extern "C" dssd_status dssd_set_fused_pair_limit(dssd_ctx* c, int64_t max_blocks) {
  if (!c || max_blocks < 0) return DSSD_EINVAL;
  c->pair_max_blocks = max_blocks;
  return DSSD_OK;
}

extern "C" dssd_status dssd_export_p_rows(dssd_ctx* c, const dssd_batch* b, void* p_rows, int32_t p_dtype,
                                          void* hip_stream) {
  BatchView v;
  const dssd_status st = check_and_view(c, b, nullptr, &v, false);
  if (st != DSSD_OK || b->B == 0) return st;
  if (b->total_drafts == 0) return DSSD_OK;
  if (!p_rows || (p_dtype != DSSD_F32 && p_dtype != DSSD_F16)) return DSSD_EINVAL;
  const bool f16 = p_dtype == DSSD_F16;
  if (reinterpret_cast<uintptr_t>(p_rows) % (f16 ? 2 : 4)) return DSSD_EALIGN;
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  const bool bf16 = b->logits_dtype == DSSD_BF16;
  const bool al = vector_ok(b) && (reinterpret_cast<uintptr_t>(p_rows) & 15) == 0;
  const int32_t groups = (v.C + 3) / 4;
  if ((int64_t)groups * b->B > 0x7FFFFFFFll) return DSSD_EUNSUPPORTED;
  const unsigned grid = (unsigned)(groups * b->B);
  {
    Timed t(c, DSSD_K_EXPORT_P, s);
    with_flags([&](auto BF, auto AL, auto H) {
      // (read + write stream: 16 waves per unit measured 1-5 % faster than what the registers allow)
      DSSD_LAUNCH_WG((export_p_rows<FLAG(BF), FLAG(AL), FLAG(H)>), grid, 256,
                     occupancy_cap_lds(c, 4, c->resid_waves_per_cu, grid), s, v, groups, p_rows);
    }, bf16, al, f16);
  }
  return launch_status(c);
}

extern "C" dssd_status dssd_residual_sample_from_p(dssd_ctx* c, const dssd_device_batch* b, void* hip_stream) {
  if (!c || !b) return DSSD_EINVAL;
  if (b->B < 0 || b->V < 1 || b->gamma < 0 || b->total_drafts < 0) return DSSD_EINVAL;
  if (b->p_dtype != DSSD_F32 && b->p_dtype != DSSD_F16) return DSSD_EINVAL;
  if (!b->draft_offsets && b->total_drafts != (int64_t)b->B * b->gamma) return DSSD_EINVAL;
  if (b->B == 0 || b->total_drafts == 0) return DSSD_OK;
  if (!b->draft_probs || !b->p_rows || !b->accepted_len || !b->rejected || !b->out_token) return DSSD_EINVAL;
  const bool f16 = b->p_dtype == DSSD_F16;
  auto mis = [](const void* p, uintptr_t a) { return p && (reinterpret_cast<uintptr_t>(p) % a) != 0; };
  if (mis(b->draft_probs, 4) || mis(b->p_rows, f16 ? 2 : 4) || mis(b->draft_offsets, 4) || mis(b->accepted_len, 4) ||
      mis(b->rejected, 4) || mis(b->out_token, 4) || mis(b->status, 4) || mis(b->step_counter, 8))
    return DSSD_EALIGN;
  DeviceView d;
  d.B = b->B; d.V = b->V; d.gamma = b->gamma; d.C = (b->V + 4095) / 4096; d.R_Q = b->total_drafts;
  if (b->B > c->max_rows || b->V > c->max_V || d.C > c->max_C) return DSSD_ENOMEM;
  d.offsets = b->draft_offsets; d.draft_probs = b->draft_probs; d.p_rows = b->p_rows;
  d.accepted_len = b->accepted_len; d.rejected = b->rejected;
  d.seed_lo = (uint32_t)b->seed; d.seed_hi = (uint32_t)(b->seed >> 32);
  d.step_lo = (uint32_t)b->step; d.step_hi = (uint32_t)(b->step >> 32);
  d.step_dev = b->step_counter;
  d.session_base = b->session_base;
  d.out_token = b->out_token; d.status = b->status; d.resid_mass = c->resid_mass;
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  const bool al = (b->V % 8) == 0 && (reinterpret_cast<uintptr_t>(b->p_rows) & 15) == 0 &&
                  (reinterpret_cast<uintptr_t>(b->draft_probs) & 15) == 0;
  const int32_t groups = (d.C + 3) / 4;
  if ((int64_t)groups * b->B > 0x7FFFFFFFll) return DSSD_EUNSUPPORTED;
  {
    Timed t(c, DSSD_K_DEVICE_MASS, s);
    const unsigned grid = (unsigned)(groups * b->B);
    with_flags([&](auto H, auto AL) { DSSD_LAUNCH((device_resid_mass<FLAG(H), FLAG(AL)>), grid, s, d, groups); }, f16, al);
  }
  {
    Timed t(c, DSSD_K_DEVICE_PICK, s);
    const unsigned g2 = (unsigned)((b->B + 3) / 4);
    with_flags([&](auto H, auto AL) { DSSD_LAUNCH((device_pick<FLAG(H), FLAG(AL)>), g2, s, d); }, f16, al);
  }
  return launch_status(c);
}

extern "C" dssd_status dssd_probe_read(dssd_ctx* c, const void* buf, size_t bytes, int32_t loads_per_lane,
                                       int32_t waves_per_cu, void* hip_stream) {
  if (!c || !buf || waves_per_cu < 0) return DSSD_EINVAL;
  if (loads_per_lane != 1 && loads_per_lane != 2 && loads_per_lane != 4 && loads_per_lane != 8) return DSSD_EINVAL;
  if (reinterpret_cast<uintptr_t>(buf) & 15) return DSSD_EALIGN;
  const int64_t units = (int64_t)(bytes / ((size_t)kWave * 16 * loads_per_lane));
  if (units == 0) return DSSD_OK;
  if ((units + 3) / 4 > 0x7FFFFFFFll) return DSSD_EUNSUPPORTED;
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  const int64_t grid = (units + 3) / 4;
  const unsigned lds = occupancy_cap_lds(c, 4, waves_per_cu, grid);
  const u32x4* src = static_cast<const u32x4*>(buf);
  uint32_t* sink = reinterpret_cast<uint32_t*>(c->resid_mass);
  {
    Timed t(c, DSSD_K_READ_PROBE, s);
    switch (loads_per_lane) {
      case 1: DSSD_LAUNCH_WG(read_probe<1>, grid, 256, lds, s, src, units, sink, c->xcds); break;
      case 2: DSSD_LAUNCH_WG(read_probe<2>, grid, 256, lds, s, src, units, sink, c->xcds); break;
      case 4: DSSD_LAUNCH_WG(read_probe<4>, grid, 256, lds, s, src, units, sink, c->xcds); break;
      default: DSSD_LAUNCH_WG(read_probe<8>, grid, 256, lds, s, src, units, sink, c->xcds); break;
    }
  }
  return launch_status(c);
}

extern "C" dssd_status dssd_step_topk(dssd_ctx* c, const dssd_topk_batch* b, dssd_out* o, void* hip_stream) {
  if (!c || !b || !o) return DSSD_EINVAL;
  if (b->B < 0 || b->k < 1 || b->k > kWave || b->gamma < 0 || b->V < 0 || b->total_drafts < 0) return DSSD_EINVAL;
  if (!b->draft_offsets && b->total_drafts != (int64_t)b->B * b->gamma) return DSSD_EINVAL;
  if (b->B == 0) return DSSD_OK;
  if (!b->p_idx || !b->p_logit || !o->accepted_len || !o->rejected || !o->out_token) return DSSD_EINVAL;
  if (b->total_drafts > 0 && (!b->q_idx || !b->q_prob || !b->draft_tokens)) return DSSD_EINVAL;
  auto mis = [](const void* p, uintptr_t a) { return p && (reinterpret_cast<uintptr_t>(p) % a) != 0; };
  if (mis(b->draft_offsets, 4) || mis(b->p_idx, 4) || mis(b->p_logit, 4) || mis(b->q_idx, 4) || mis(b->q_prob, 4) ||
      mis(b->draft_tokens, 4) || mis(b->inv_temperature, 4) || mis(b->step_counter, 8) || mis(o->accepted_len, 4) ||
      mis(o->rejected, 4) || mis(o->out_token, 4) || mis(o->row_stats, 4) || mis(o->p_tok, 4) || mis(o->q_tok, 4) ||
      mis(o->status, 4))
    return DSSD_EALIGN;
  if ((b->B + 3) / 4 > 0x7FFFFFFF) return DSSD_EUNSUPPORTED;
  TopkView t;
  t.B = b->B; t.k = b->k; t.gamma = b->gamma; t.V = b->V; t.R_Q = b->total_drafts;
  t.offsets = b->draft_offsets; t.p_idx = b->p_idx; t.p_logit = b->p_logit; t.q_idx = b->q_idx; t.q_prob = b->q_prob;
  t.tokens = b->draft_tokens; t.inv_temp = b->inv_temperature;
  t.seed_lo = (uint32_t)b->seed; t.seed_hi = (uint32_t)(b->seed >> 32);
  t.step_lo = (uint32_t)b->step; t.step_hi = (uint32_t)(b->step >> 32);
  t.session_base = b->session_base; t.step_dev = b->step_counter;
  t.accepted_len = o->accepted_len; t.rejected = o->rejected; t.out_token = o->out_token;
  t.row_stats = o->row_stats; t.p_tok = o->p_tok; t.q_tok = o->q_tok; t.status = o->status;
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  {
    Timed tm(c, DSSD_K_TOPK_STEP, s);
    DSSD_LAUNCH(topk_step, (b->B + 3) / 4, s, t);
  }
  return launch_status(c);
}

extern "C" dssd_status dssd_random_words(dssd_ctx* c, uint64_t seed, uint64_t step, uint32_t session_first,
                                         uint32_t position_first, int32_t n_sessions, int32_t n_positions,
                                         uint32_t* words, void* hip_stream) {
  if (!c || n_sessions < 0 || n_positions < 0) return DSSD_EINVAL;
  const int64_t n = (int64_t)n_sessions * n_positions;
  if (n == 0) return DSSD_OK;
  if (!words) return DSSD_EINVAL;
  if (reinterpret_cast<uintptr_t>(words) & 3) return DSSD_EALIGN;
  if ((n + 255) / 256 > 0x7FFFFFFFll) return DSSD_EUNSUPPORTED;
  hipLaunchKernelGGL(random_words, dim3((unsigned)((n + 255) / 256)), dim3(256), 0,
                     static_cast<hipStream_t>(hip_stream), session_first, position_first, n_sessions,
                     n_positions, (uint32_t)step, (uint32_t)(step >> 32), (uint32_t)seed, (uint32_t)(seed >> 32),
                     words);
  return launch_status(c);
}

extern "C" dssd_status dssd_profile_enable(dssd_ctx* c, uint32_t kernel_mask) {
  if (!c) return DSSD_EINVAL;
  // the pools of the kernels asked for are created here, never inside a hot call
  for (int k = 0; k < DSSD_K_COUNT; ++k) {
    if (!((kernel_mask >> k) & 1u) || c->ev_cap[k]) continue;
    hipEvent_t* a = new (std::nothrow) hipEvent_t[kEventPool];
    hipEvent_t* b = new (std::nothrow) hipEvent_t[kEventPool];
    size_t made = 0;
    if (a && b)
      for (; made < kEventPool; ++made) {
        if (hipEventCreate(&a[made]) != hipSuccess) break;
        if (hipEventCreate(&b[made]) != hipSuccess) { (void)hipEventDestroy(a[made]); break; }
      }
    if (made < kEventPool) {
      (void)hipGetLastError();
      for (size_t i = 0; i < made; ++i) { (void)hipEventDestroy(a[i]); (void)hipEventDestroy(b[i]); }
      delete[] a;
      delete[] b;
      return a && b ? DSSD_EHIP : DSSD_ENOMEM;
    }
    c->ev_begin[k] = a; c->ev_end[k] = b; c->ev_cap[k] = kEventPool;
  }
  c->profile_mask = kernel_mask;
  return DSSD_OK;
}

extern "C" dssd_status dssd_profile_reset(dssd_ctx* c) {
  if (!c) return DSSD_EINVAL;
  for (int k = 0; k < DSSD_K_COUNT; ++k) c->ev_used[k] = c->ev_dropped[k] = 0;
  c->ev_failed = false;
  return DSSD_OK;
}

extern "C" dssd_status dssd_profile_read(dssd_ctx* c, int k, double* total_ms, int64_t* launches) {
  if (!c || k < 0 || k >= DSSD_K_COUNT || !total_ms || !launches) return DSSD_EINVAL;
  double sum = 0.0;
  for (size_t i = 0; i < c->ev_used[k]; ++i) {
    if (hipEventSynchronize(c->ev_end[k][i]) != hipSuccess) return DSSD_EHIP;
    float ms = 0.f;
    if (hipEventElapsedTime(&ms, c->ev_begin[k][i], c->ev_end[k][i]) != hipSuccess) return DSSD_EHIP;
    sum += ms;
  }
  *total_ms = sum;
  *launches = (int64_t)c->ev_used[k];
  if (c->ev_failed) return DSSD_EHIP;
  return c->ev_dropped[k] ? DSSD_ENOMEM : DSSD_OK;   // ENOMEM: launches beyond the pool went untimed
}
