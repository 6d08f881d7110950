// Host side of the QSAC C ABI (include/qsac.h): argument validation, workspace layout and the
// launch sequence of one step.  No device memory is allocated here; everything lives in the
// caller's workspace.
#include "qsac.h"

#include <hip/hip_runtime.h>

#include <immintrin.h>
#include <time.h>

#include <atomic>
#include <cmath>
#include <cstdlib>
#include <cstring>
#include <new>
#include <thread>
#include <vector>

#include "qsac_kernels.hip.h"

using namespace qsac;

namespace {

constexpr uint32_t kMagic = 0x51534143u;       // "QSAC"
constexpr uint32_t kGraphMagic = 0x51534147u;  // "QSAG"
constexpr int kStages = 6;
const char* const kStageNames[kStages] = {"gate", "score", "select", "fill", "attn", "combine"};

thread_local int g_last_hip = 0;

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

int check_config(const qsac_config* c) {
  if (!c) return QSAC_ENULL;
  if (c->head_dim != QSAC_HEAD_DIM) return QSAC_EINVAL;
  if (c->dtype != QSAC_F16 && c->dtype != QSAC_BF16) return QSAC_EINVAL;
  if (c->batch < 1 || c->n_q_heads < 1 || c->n_kv_heads < 1) return QSAC_ERANGE;
  if (c->n_kv_heads > QSAC_MAX_KV_HEADS) return QSAC_ERANGE;
  if (c->n_q_heads % c->n_kv_heads != 0) return QSAC_EINVAL;
  if (c->n_q_heads / c->n_kv_heads > QSAC_MAX_GROUP) return QSAC_ERANGE;
  if (c->n_ctx < 1 || c->n_ctx > (int64_t(1) << 20)) return QSAC_ERANGE;
  if (c->k_max < 1 || c->k_max > c->n_ctx) return QSAC_ERANGE;
  if ((int64_t)c->batch * c->n_kv_heads > 65535) return QSAC_ERANGE;  // grid.y
  if (c->append_capacity < 0 || c->append_capacity > (1 << 20)) return QSAC_ERANGE;
  if (c->n_sink < 0 || c->n_recent < 0 || (int64_t)c->n_sink + c->n_recent > c->k_max) return QSAC_ERANGE;
  if (c->flags & ~(QSAC_FLAG_DRY_RUN | QSAC_FLAG_SERIAL | QSAC_FLAG_SCORE_VALU | QSAC_FLAG_PROFILE | QSAC_FLAG_FILL_KERNEL |
                   QSAC_FLAG_PUSH_FILL | QSAC_FLAG_PUSH_HOLD | QSAC_FLAG_STAGGER))
    return QSAC_EINVAL;
  if ((c->flags & QSAC_FLAG_PUSH_HOLD) && !(c->flags & QSAC_FLAG_PUSH_FILL)) return QSAC_EINVAL;
  if ((c->flags & QSAC_FLAG_PUSH_FILL) && (c->flags & QSAC_FLAG_FILL_KERNEL)) return QSAC_EINVAL;  // one way to fill
  // the staggered schedule is two plain pull-mode steps on two streams
  if ((c->flags & QSAC_FLAG_STAGGER) &&
      ((c->flags & (QSAC_FLAG_SERIAL | QSAC_FLAG_PROFILE | QSAC_FLAG_FILL_KERNEL | QSAC_FLAG_PUSH_FILL)) || c->batch < 2 ||
       (int64_t)c->batch * c->n_kv_heads > 8192))  // (its fill kernel keeps a table of the slice's pairs in LDS)
    return QSAC_EINVAL;  // (qsac_init also asks for the second stream)
  if (c->push_threads < 0 || c->push_threads > 64 || c->push_wait_us < 0) return QSAC_ERANGE;
  if (c->q_head_importance)
    for (int i = 0; i < c->n_q_heads; ++i)
      if (!(c->q_head_importance[i] > 0.f) || !std::isfinite(c->q_head_importance[i])) return QSAC_EINVAL;
  return QSAC_OK;
}

// Attention split: rows of slots per workgroup for k slots in use.  The kernel keeps two waves per
// SIMD resident, i.e. two workgroups per compute unit, so about 512 workgroups fill the chip in one
// round (measured: 512 beats 256, 768, 1024 and 2048 at 64 pairs x 2048 slots); at least 64 rows,
// one 16-slot tile per wave, each.
int attn_rows(int P, int k) {
  int64_t rows = ((int64_t)P * k + 511) / 512;
  rows = (rows + 63) / 64 * 64;
  if (rows < 64) rows = 64;
  if (rows > 1024) rows = 1024;
  return (int)rows;
}

// Rank, within the select's sample of 4096 keys (one key in vpt), whose key bounds the candidates of the
// guided select from below: the count C of keys at or above it has mean vpt * r and a standard deviation
// below vpt * sqrt(r); r solves  vpt * (r - 6 sqrt(r)) = k, which puts k six deviations below the mean.
// 0 (no guided select) when the candidates might not fit the list, or the context is short.
int select_sample_rank(int k, int vpt) {
  if (vpt < 8) return 0;  // up to 16384 keys the three full passes are as quick (measured)
  const double x = 3.0 + std::sqrt(9.0 + (double)k / vpt);
  const int r = (int)std::ceil(x * x);
  const double upper = (double)vpt * (r + 6.0 * std::sqrt((double)r));
  // the bound is the lower edge of a histogram bin, which adds up to a bin's worth of keys: leave half the list
  if (r > 2048 || upper > 0.6 * kSelectListCap) return 0;
  return r;
}

void make_layout(const qsac_config* c, qsac_ws_layout* L) {
  const size_t P = (size_t)c->batch * c->n_kv_heads;
  const size_t G = (size_t)(c->n_q_heads / c->n_kv_heads);
  const size_t n_pad = align_up((size_t)c->n_ctx, kSelChunk);
  const size_t words = n_pad / 32;
  const size_t splits = ((size_t)c->k_max + (size_t)c->append_capacity + 63) / 64;  // rows per split >= 64
  size_t off = 0;
  auto take = [&](size_t bytes) {
    size_t o = off;
    off = align_up(off + bytes, 256);
    return o;
  };
  L->valid = take(P * 4);
  L->set_sorted = take(P * c->k_max * 4);
  L->keys = take(P * n_pad * 4);
  L->hist = take(P * 3 * kBins * 4);
  // (the mid-N select keeps the pairs' candidate lists where the grid-wide path has its first bitmap)
  const bool mid_n = (size_t)c->n_ctx > (size_t)kSmallMaxN && (size_t)c->n_ctx <= (size_t)kStreamMaxN;
  L->bm_new = take(mid_n ? std::max(P * words * 4, P * (size_t)kStreamListCap * 8) : P * words * 4);
  L->bm_eq = take(P * words * 4);
  L->bm_old = take(P * words * 4);
  L->miss_count = take(P * 4);
  L->miss_slot = take(P * c->k_max * 4);
  L->miss_tok = take(P * c->k_max * 4);
  L->part_ml = take(P * G * splits * 2 * 4);
  L->part_acc = take(P * G * splits * kD * 4);
  L->stats = take(8 * 8);
  L->importance = take((size_t)c->n_q_heads * 8);
  L->sel_r = take(P * kSelStride * 4);
  L->chunk_cnt = take(P * (n_pad / kSelChunk) * 2 * 4);
  L->fetch_tok = take(P * c->k_max * 4);
  L->push = take(4 * 4);
  L->total = off;
  L->n_pad = (int64_t)n_pad;
  L->words = (int32_t)words;
  L->max_splits = (int32_t)splits;
}

}  // namespace

// ---- push-mode transfer engine (Section 6.2 of the paper): host threads that copy the rows of a request's miss
// lists from the host K / V store straight into the cache slots, through the device memory window the host can
// write, and then raise the completion flag.
struct PushJob {
  const char* K_src;
  const char* V_src;
  char* K_slots;
  char* V_slots;
  int64_t N;
  int k_max, P;
};

struct PushEngine {
  static constexpr uint32_t kRing = 1024;  // requests the host may be ahead of the device
  uint32_t* box = nullptr;                 // mailbox in pinned host memory (layout: qsac_publish_kernel)
  volatile uint32_t* hdp_flush = nullptr;  // the device's host-data-path flush register, mapped into this process
  int T = 0;
  bool hold = false;
  std::vector<std::thread> threads;
  std::atomic<bool> stop{false};
  std::atomic<int> arrived{0};
  uint32_t submitted = 0;  // sequence number of the last request whose job is in the ring (host thread of the caller)
  const char *mapped_K = nullptr, *mapped_V = nullptr;  // slot tensors whose window pages have been touched
  PushJob ring[kRing];

  // The first host access to a page of the device memory window faults its mapping in, which costs tens of
  // microseconds per page here: touch every page of a slot tensor once (a read; the contents stay), with all
  // the threads, before the first request that writes into it, so that no polling kernel waits for page faults.
  void map_window(const char* base, size_t bytes) {
    std::vector<std::thread> th;
    const int n = T > 0 ? T : 1;
    for (int i = 0; i < n; ++i)
      th.emplace_back([=] {
        const size_t lo = bytes * i / n / 4096 * 4096, hi = bytes * (i + 1) / n;
        unsigned acc = 0;
        for (size_t off = lo; off < hi; off += 4096) acc += *reinterpret_cast<const volatile unsigned char*>(base + off);
        (void)acc;
      });
    for (auto& t : th) t.join();
  }

  void start(uint32_t seq_now) {
    stop.store(false);
    arrived.store(0);
    submitted = seq_now;
    for (int i = 0; i < T; ++i) threads.emplace_back([this, i, seq_now] { worker(i, seq_now); });
  }
  void halt() {
    stop.store(true);
    for (auto& t : threads) t.join();
    threads.clear();
  }
  void worker(int id, uint32_t seen) {
    int idle = 0;
    while (!stop.load(std::memory_order_relaxed)) {
      const uint32_t f1 = __atomic_load_n(box + qsac::kPushFlag1, __ATOMIC_ACQUIRE);
      if (hold || f1 == seen) {
        // spin while requests keep coming, doze once the device has been quiet for a while
        if (++idle < 200000) {
          _mm_pause();
        } else {
          timespec ts = {0, 50000};
          nanosleep(&ts, nullptr);
        }
        continue;
      }
      idle = 0;
      const uint32_t seq = seen + 1;
      const PushJob J = ring[seq % kRing];
      const int* count = reinterpret_cast<const int*>(box + qsac::kPushHeaderWords);
      const int* slot = count + J.P;
      const int* tok = slot + (size_t)J.P * J.k_max;
      long total = 0;
      for (int p = 0; p < J.P; ++p) total += count[p];
      // thread `id` takes the rows [lo, hi) of all pairs' lists laid end to end
      const long lo = total * id / T, hi = total * (id + 1) / T;
      long base = 0;
      for (int p = 0; p < J.P && base < hi; ++p) {
        const long c = count[p];
        if (base + c > lo) {
          const long e0 = lo > base ? lo - base : 0, e1 = hi - base < c ? hi - base : c;
          const int* sp = slot + (size_t)p * J.k_max;
          const int* tp = tok + (size_t)p * J.k_max;
          const char* Ks = J.K_src + (size_t)p * (size_t)J.N * 256;
          const char* Vs = J.V_src + (size_t)p * (size_t)J.N * 256;
          char* Kd = J.K_slots + (size_t)p * (size_t)J.k_max * 256;
          char* Vd = J.V_slots + (size_t)p * (size_t)J.k_max * 256;
          for (long e = e0; e < e1; ++e) {
            std::memcpy(Kd + (size_t)sp[e] * 256, Ks + (size_t)tp[e] * 256, 256);
            std::memcpy(Vd + (size_t)sp[e] * 256, Vs + (size_t)tp[e] * 256, 256);
          }
        }
        base += c;
      }
      _mm_sfence();  // this thread's write-combined stores have left the core
      if (arrived.fetch_add(1, std::memory_order_acq_rel) == T - 1) {
        // Last thread of the request.  Host writes travel through the device's host data path, which may hold them
        // back from device memory: flush it (the register write follows the row writes on the bus), then read
        // through the same window, which cannot return before the writes ahead of it have arrived.
        if (hdp_flush) *hdp_flush = 1u;
        _mm_sfence();
        (void)*reinterpret_cast<const volatile uint32_t*>(J.K_slots);
        arrived.store(0, std::memory_order_relaxed);
        __atomic_store_n(box + qsac::kPushFlag2, seq, __ATOMIC_RELEASE);  // the paper's Flag2
      }
      seen = seq;
    }
  }
};

constexpr int kStaggerSlices = 8;        // at most (a batch of 32 runs as 2 + 4 + 8 + 18)
constexpr int kTrickleWorkgroups = 64;  // of the staggered schedule's fill kernel (32: 3.32 ms, 48: 3.16, 64: 3.14,
                                        // 96: 3.23, 128: 3.19 per step of the largest workload)

struct qsac_ctx {
  uint32_t magic;
  qsac_config cfg;
  qsac_ws_layout L;
  int P, G;
  int k_bound;  // k of the steps since the last reset, 0 if none yet
  uint64_t steps;
  hipStream_t s_main, s_side;
  hipEvent_t ev_sel, ev_fill;
  hipEvent_t ev_selected[kStaggerSlices], ev_filled[kStaggerSlices];  // staggered schedule, per batch slice
  bool dry, overlap, profile, small, fill_kernel, stagger;
  hipEvent_t prof[kStages + 1];
  double stage_ms[kStages];
  uint64_t stage_calls;
  bool prof_pending;
  bool broken;  // a HIP call failed in the middle of a step: the caches may be half updated, only a reset clears this
  PushEngine* push;  // push-mode transfer engine, nullptr otherwise
  // where the fill sources of the last step live (looked up when the pointers change)
  const void *seen_K_src, *seen_V_src;
  bool K_src_host, V_src_host;
};

struct qsac_graph {
  uint32_t magic;
  qsac_ctx* ctx;
  hipGraphExec_t exec;
  int k;
  PushJob job;  // push mode: what the transfer threads need for a replay
};

// State and scratch of qsac_step_static(): one copy per GPU inside the library's device image.  In host code
// this name is only a handle for hipGetSymbolAddress(); the device address it resolves to (per device) is what
// kernels and the workspace layout use.
static __device__ __align__(256) unsigned char scratch[QSAC_STATIC_SCRATCH_BYTES];

namespace {

#define HIP_TRY(expr)                 \
  do {                                \
    hipError_t e_ = (expr);           \
    if (e_ != hipSuccess) {           \
      g_last_hip = (int)e_;           \
      return QSAC_EHIP;               \
    }                                 \
  } while (0)

#define HIP_TRY_OR(expr, cleanup)     \
  do {                                \
    hipError_t e_ = (expr);           \
    if (e_ != hipSuccess) {           \
      g_last_hip = (int)e_;           \
      cleanup;                        \
      return QSAC_EHIP;               \
    }                                 \
  } while (0)

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

int clear_state(qsac_ctx* c) {
  char* ws = static_cast<char*>(c->cfg.workspace);
  // bookkeeping that must start at zero: validity flags, counters (fill kernel, not a memset node)
  qsac_zero_kernel<<<1, 256, 0, c->s_main>>>(reinterpret_cast<u32*>(ws + c->L.valid), (size_t)c->P);
  qsac_zero_kernel<<<1, 256, 0, c->s_main>>>(reinterpret_cast<u32*>(ws + c->L.stats), (size_t)16);
  qsac_zero_kernel<<<1, 256, 0, c->s_main>>>(reinterpret_cast<u32*>(ws + c->L.miss_count), (size_t)c->P);
  qsac_zero_kernel<<<1, 256, 0, c->s_main>>>(reinterpret_cast<u32*>(ws + c->L.sel_r), (size_t)c->P * kSelStride);
  HIP_TRY(hipGetLastError());
  c->k_bound = 0;
  c->steps = 0;
  c->broken = false;
  for (int i = 0; i < kStages; ++i) c->stage_ms[i] = 0.0;
  c->stage_calls = 0;
  c->prof_pending = false;
  return QSAC_OK;
}

// True if `ptr` is host memory mapped into the device (hipHostMalloc); HBM and anything the runtime does not
// know count as device memory.
bool is_host_memory(const void* ptr) {
  hipPointerAttribute_t at;
  if (hipPointerGetAttributes(&at, ptr) != hipSuccess) {
    (void)hipGetLastError();
    return false;
  }
  return at.type == hipMemoryTypeHost;
}

// The one-workgroup select keeps its candidate list in LDS beyond the default 64 KiB (and the long-context
// diff its lists): raise the kernels' dynamic LDS limit.  Per device; harmless to repeat.
int raise_lds_limits() {
  const int lds_max = std::max((int)(((size_t)(kSmallMaxN / 32) * 3 + 2 * (size_t)kSelectListCap) * sizeof(u32)),
                               kDiffListMax * 13);
  const void* fns[] = {(const void*)qsac_select_small_kernel<2, 1024>, (const void*)qsac_select_small_kernel<4, 1024>,
                       (const void*)qsac_select_small_kernel<8, 1024>, (const void*)qsac_select_small_kernel<16, 1024>,
                       (const void*)qsac_diff_list_kernel};
  for (const void* fn : fns) HIP_TRY(hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, lds_max));
  HIP_TRY(hipFuncSetAttribute((const void*)qsac_select_stream_kernel<1024>, hipFuncAttributeMaxDynamicSharedMemorySize,
                              (int)(((size_t)(kStreamMaxN / 32) * 3 + 2 * (size_t)kSelectListCap) * sizeof(u32))));
  return QSAC_OK;
}

// Eq. (2) weights into the workspace (all 1 when none are given), by a kernel on stream_main.
int set_importance(qsac_ctx* c, const float* w) {
  ImportanceArg arg;
  for (int i = 0; i < c->cfg.n_q_heads; ++i) arg.v[i] = w ? w[i] : 1.f;
  qsac_set_importance_kernel<<<1, 256, 0, c->s_main>>>(
      reinterpret_cast<double*>(static_cast<char*>(c->cfg.workspace) + c->L.importance), arg, c->cfg.n_q_heads);
  HIP_TRY(hipGetLastError());
  return QSAC_OK;
}

int drain_profile(qsac_ctx* c) {
  if (!c->prof_pending) return QSAC_OK;
  HIP_TRY(hipEventSynchronize(c->prof[kStages]));
  for (int i = 0; i < kStages; ++i) {
    float ms = 0.f;
    HIP_TRY(hipEventElapsedTime(&ms, c->prof[i], c->prof[i + 1]));
    c->stage_ms[i] += ms;
  }
  c->stage_calls += 1;
  c->prof_pending = false;
  return QSAC_OK;
}

template <int DT, int G>
void launch_score(const qsac_ctx* c, const qsac_step_args* a, u32* keys, u32* hist, int P, hipStream_t sm) {
  auto q = static_cast<const uint16_t*>(a->q);
  auto K = static_cast<const uint16_t*>(a->K_dev);
  const int64_t N = c->cfg.n_ctx;
  const int Hq = c->cfg.n_q_heads, Hkv = c->cfg.n_kv_heads;
  const bool valu = (c->cfg.flags & QSAC_FLAG_SCORE_VALU) != 0;
  if (c->small) {
    dim3 grid((unsigned)((N + kScoreRowsSmall - 1) / kScoreRowsSmall), (unsigned)P);
    if (valu)
      qsac_score_valu_kernel<DT, G, kScoreRowsSmall, false><<<grid, 256, 0, sm>>>(q, K, a->reuse_flags, keys, hist, Hq, Hkv, N, c->L.n_pad, c->cfg.n_sink, c->cfg.n_recent);
    else
      qsac_score_mfma_kernel<DT, G, kScoreRowsSmall, false><<<grid, 256, 0, sm>>>(q, K, a->reuse_flags, keys, hist, Hq, Hkv, N, c->L.n_pad, c->cfg.n_sink, c->cfg.n_recent);
  } else {
    dim3 grid((unsigned)((N + kScoreRowsLarge - 1) / kScoreRowsLarge), (unsigned)P);
    if (valu)
      qsac_score_valu_kernel<DT, G, kScoreRowsLarge, true><<<grid, 256, 0, sm>>>(q, K, a->reuse_flags, keys, hist, Hq, Hkv, N, c->L.n_pad, c->cfg.n_sink, c->cfg.n_recent);
    else
      qsac_score_mfma_kernel<DT, G, kScoreRowsLarge, true><<<grid, 256, 0, sm>>>(q, K, a->reuse_flags, keys, hist, Hq, Hkv, N, c->L.n_pad, c->cfg.n_sink, c->cfg.n_recent);
  }
}

AttnArgs attn_args(const qsac_ctx* c, const qsac_step_args* a, const int* fetch_tok, const int* miss_count,
                   float* part_ml, float* part_acc, int rows, int n_splits, int which) {
  AttnArgs A;
  A.q = static_cast<const uint16_t*>(a->q);
  A.K_slots = static_cast<v4u*>(a->K_slots);
  A.V_slots = static_cast<v4u*>(a->V_slots);
  A.fetch_tok = fetch_tok;
  A.miss_count = miss_count;
  A.reuse_flags = a->reuse_flags;
  A.part_ml = part_ml;
  A.part_acc = part_acc;
  A.out = a->out;
  A.K_app = static_cast<const v4u*>(a->K_app);
  A.V_app = static_cast<const v4u*>(a->V_app);
  A.dp = reinterpret_cast<const DevParams*>(a->dev_params);
  A.N = c->cfg.n_ctx;
  A.n_app = a->n_app;
  A.app_cap = c->cfg.append_capacity;
  A.Hq = c->cfg.n_q_heads;
  A.Hkv = c->cfg.n_kv_heads;
  A.k = a->k;
  A.k_max = c->cfg.k_max;
  A.rows = rows;
  A.n_splits = n_splits;
  A.max_splits = c->L.max_splits;
  A.which = which;
  return A;
}

template <int DT, int G>
void launch_attn(const qsac_ctx* c, hipStream_t stream, const AttnArgs& A, const FillSrc& src, int P, bool filled) {
  dim3 grid((unsigned)A.n_splits, (unsigned)P);
  if (filled || c->fill_kernel || c->push)  // the rows are in their slots before the attention starts
    qsac_attn_kernel<DT, G, false><<<grid, 256, 0, stream>>>(A, src);
  else
    qsac_attn_kernel<DT, G, true><<<grid, 256, 0, stream>>>(A, src);
}

// Dispatch on (dtype, G) to the instantiated kernels.
#define QSAC_DISPATCH_G(FN, DT, ...)            \
  switch (c->G) {                               \
    case 1: FN<DT, 1>(__VA_ARGS__); break;      \
    case 2: FN<DT, 2>(__VA_ARGS__); break;      \
    case 3: FN<DT, 3>(__VA_ARGS__); break;      \
    case 4: FN<DT, 4>(__VA_ARGS__); break;      \
    case 5: FN<DT, 5>(__VA_ARGS__); break;      \
    case 6: FN<DT, 6>(__VA_ARGS__); break;      \
    case 7: FN<DT, 7>(__VA_ARGS__); break;      \
    default: FN<DT, 8>(__VA_ARGS__); break;     \
  }
#define QSAC_DISPATCH(FN, ...)                                  \
  do {                                                          \
    if (c->cfg.dtype == QSAC_F16) {                             \
      QSAC_DISPATCH_G(FN, 0, __VA_ARGS__)                       \
    } else {                                                    \
      QSAC_DISPATCH_G(FN, 1, __VA_ARGS__)                       \
    }                                                           \
  } while (0)

// The host-side fields of a context for `cfg` (no events yet, nothing enqueued).
void fill_ctx(qsac_ctx* c, const qsac_config* cfg, const qsac_ws_layout& L) {
  c->magic = kMagic;
  c->cfg = *cfg;
  c->cfg.q_head_importance = nullptr;  // handed to the device at set-up; the caller's array is not kept
  c->L = L;
  c->P = cfg->batch * cfg->n_kv_heads;
  c->G = cfg->n_q_heads / cfg->n_kv_heads;
  c->dry = (cfg->flags & QSAC_FLAG_DRY_RUN) != 0;
  c->small = cfg->n_ctx <= kSmallMaxN;
  c->s_main = static_cast<hipStream_t>(cfg->stream_main);
  c->s_side = static_cast<hipStream_t>(cfg->stream_side);
  c->fill_kernel = (cfg->flags & QSAC_FLAG_FILL_KERNEL) != 0;
  c->overlap = cfg->stream_side != nullptr && cfg->stream_side != cfg->stream_main && !(cfg->flags & QSAC_FLAG_SERIAL);
  c->profile = (cfg->flags & QSAC_FLAG_PROFILE) != 0;
  if (c->profile) c->overlap = false;  // stage times are taken on one stream
  c->stagger = (cfg->flags & QSAC_FLAG_STAGGER) != 0;
  c->k_bound = 0;
  c->steps = 0;
  c->broken = false;
  c->seen_K_src = c->seen_V_src = nullptr;
  c->K_src_host = c->V_src_host = false;
  c->ev_sel = c->ev_fill = nullptr;
  for (auto& e : c->ev_selected) e = nullptr;
  for (auto& e : c->ev_filled) e = nullptr;
  c->push = nullptr;
  for (auto& e : c->prof) e = nullptr;
  for (int i = 0; i < kStages; ++i) c->stage_ms[i] = 0.0;
  c->stage_calls = 0;
  c->prof_pending = false;
}

// Everything qsac_step checks before anything is enqueued.
int validate_step(const qsac_ctx* c, const qsac_step_args* a) {
  if (!c || c->magic != kMagic) return QSAC_ESTATE;
  if (!a) return QSAC_ENULL;
  if (!a->q || !a->K_dev || !a->K_src || !a->V_src || !a->K_slots || !a->V_slots || !a->slot_idx || !a->prev_q ||
      !a->out || !a->topk_idx || !a->hit_mask || !a->reuse_flags)
    return QSAC_ENULL;
  if (a->dev_params) {
    if (!aligned16(a->dev_params)) return QSAC_EALIGN;  // tau and n_app come from the device at run time
  } else {
    if (!a->tau) return QSAC_ENULL;
    if (a->n_tau != 1 && a->n_tau != c->cfg.n_kv_heads) return QSAC_EINVAL;
    for (int i = 0; i < a->n_tau; ++i)
      if (std::isnan(a->tau[i])) return QSAC_EINVAL;
  }
  if (a->k < 1 || a->k > c->cfg.k_max) return QSAC_ERANGE;
  if (c->k_bound != 0 && a->k != c->k_bound) return QSAC_ESTATE;
  const void* al[] = {a->q, a->K_dev, a->K_src, a->V_src, a->K_slots, a->V_slots, a->slot_idx, a->prev_q, a->out, a->topk_idx};
  for (const void* ptr : al)
    if (!aligned16(ptr)) return QSAC_EALIGN;
  if (a->n_app < 0 || a->n_app > c->cfg.append_capacity) return QSAC_ERANGE;
  if (a->n_app > 0) {
    if (!a->K_app || !a->V_app) return QSAC_ENULL;
    if (!aligned16(a->K_app) || !aligned16(a->V_app)) return QSAC_EALIGN;
  }
  if (a->k < c->cfg.n_sink + c->cfg.n_recent) return QSAC_ERANGE;
  if (a->res_slot) {
    if (!a->V_res) return QSAC_ENULL;
    if (a->n_res < 1 || a->n_res > c->cfg.n_kv_heads) return QSAC_ERANGE;
    if (!aligned16(a->V_res)) return QSAC_EALIGN;
    for (int h = 0; h < c->cfg.n_kv_heads; ++h)
      if (a->res_slot[h] < -1 || a->res_slot[h] >= a->n_res) return QSAC_ERANGE;
  }
  if (c->push && a->res_slot) return QSAC_EINVAL;  // the transfer threads cannot read HBM sources
  if (c->broken) return QSAC_ESTATE;
  return QSAC_OK;
}

// Looks up, when the pointers change, whether the fill sources are host memory (for the byte counters).
void note_fill_sources(qsac_ctx* c, const qsac_step_args* a) {
  if (a->K_src != c->seen_K_src) {
    c->K_src_host = is_host_memory(a->K_src);
    c->seen_K_src = a->K_src;
  }
  if (a->V_src != c->seen_V_src) {
    c->V_src_host = is_host_memory(a->V_src);
    c->seen_V_src = a->V_src;
  }
}

// Push mode, before a step is enqueued or replayed: both fill sources must be host memory; a poll that gave up
// earlier poisons the context; the job of the coming request goes into the ring the transfer threads read.
int push_submit(qsac_ctx* c, const PushJob& job, bool sources_on_host) {
  PushEngine* E = c->push;
  if (!sources_on_host) return QSAC_EINVAL;
  if (__atomic_load_n(E->box + kPushTimeouts, __ATOMIC_ACQUIRE) != 0) {
    c->broken = true;
    return QSAC_ETIMEOUT;
  }
  // at most kRing requests ahead of the answers
  for (int spins = 0; E->submitted + 1 - __atomic_load_n(E->box + kPushFlag2, __ATOMIC_ACQUIRE) >= PushEngine::kRing; ++spins) {
    if (spins > 100000) return QSAC_ETIMEOUT;  // ten seconds
    timespec ts = {0, 100000};
    nanosleep(&ts, nullptr);
  }
  const size_t slot_bytes = (size_t)job.P * (size_t)job.k_max * 256;
  if (job.K_slots != E->mapped_K) {
    E->map_window(job.K_slots, slot_bytes);
    E->mapped_K = job.K_slots;
  }
  if (job.V_slots != E->mapped_V) {
    E->map_window(job.V_slots, slot_bytes);
    E->mapped_V = job.V_slots;
  }
  E->ring[(E->submitted + 1) % PushEngine::kRing] = job;
  std::atomic_thread_fence(std::memory_order_release);
  E->submitted += 1;
  return QSAC_OK;
}

PushJob push_job_of(const qsac_ctx* c, const qsac_step_args* a) {
  PushJob J;
  J.K_src = static_cast<const char*>(a->K_src);
  J.V_src = static_cast<const char*>(a->V_src);
  J.K_slots = static_cast<char*>(a->K_slots);
  J.V_slots = static_cast<char*>(a->V_slots);
  J.N = c->cfg.n_ctx;
  J.k_max = c->cfg.k_max;
  J.P = c->P;
  return J;
}

// Push mode: zeroes the device-side request state and the mailbox flags (nothing may be in flight).
int push_rewind(qsac_ctx* c) {
  PushEngine* E = c->push;
  qsac_zero_kernel<<<1, 256, 0, c->s_main>>>(reinterpret_cast<u32*>(static_cast<char*>(c->cfg.workspace) + c->L.push), (size_t)4);
  HIP_TRY(hipGetLastError());
  HIP_TRY(hipStreamSynchronize(c->s_main));
  E->box[kPushFlag1] = 0;
  E->box[kPushFlag2] = 0;
  E->box[kPushTimeouts] = 0;
  std::atomic_thread_fence(std::memory_order_seq_cst);
  return QSAC_OK;
}

// Push mode: the mailbox in pinned host memory and the transfer threads.  The threads write the cache slots
// through the device's host-visible memory window, which must span device memory (a "large BAR").
int push_start(qsac_ctx* c) {
  int dev = 0, large_bar = 0;
  HIP_TRY(hipGetDevice(&dev));
  HIP_TRY(hipDeviceGetAttribute(&large_bar, hipDeviceAttributeIsLargeBar, dev));
  if (!large_bar) return QSAC_EINVAL;
  PushEngine* E = new (std::nothrow) PushEngine();
  if (!E) return QSAC_EINVAL;
  const size_t words = (size_t)kPushHeaderWords + (size_t)c->P + 2 * (size_t)c->P * (size_t)c->cfg.k_max;
  void* box = nullptr;
  hipError_t e = hipHostMalloc(&box, words * sizeof(uint32_t), hipHostMallocCoherent);
  if (e != hipSuccess) {
    g_last_hip = (int)e;
    delete E;
    return QSAC_EHIP;
  }
  std::memset(box, 0, words * sizeof(uint32_t));
  E->box = static_cast<uint32_t*>(box);
  {
    uint32_t* reg = nullptr;  // the attribute is pointer-sized: address of the HDP_MEM_COHERENCY_FLUSH_CNTL register
    if (hipDeviceGetAttribute(reinterpret_cast<int*>(&reg), hipDeviceAttributeHdpMemFlushCntl, dev) == hipSuccess)
      E->hdp_flush = reg;
    else
      (void)hipGetLastError();
  }
  E->T = c->cfg.push_threads ? c->cfg.push_threads : 4;
  E->hold = (c->cfg.flags & QSAC_FLAG_PUSH_HOLD) != 0;
  c->push = E;
  int rc = push_rewind(c);
  if (rc != QSAC_OK) return rc;  // qsac_free releases the engine
  E->start(0);
  return QSAC_OK;
}

// Enqueues the launches of one step (also what a graph capture records).  QSAC_EHIP if a HIP call fails,
// possibly after part of the step has been enqueued.
// The step arguments of the batch elements from b0 on: every tensor is [B, ...], so a slice of the batch is the
// same step on offset pointers.
qsac_step_args slice_args(const qsac_ctx* c, const qsac_step_args* a, int b0) {
  qsac_step_args s = *a;
  if (b0 == 0) return s;
  const size_t Hq = (size_t)c->cfg.n_q_heads, Hkv = (size_t)c->cfg.n_kv_heads, N = (size_t)c->cfg.n_ctx;
  const size_t k_max = (size_t)c->cfg.k_max, cap = (size_t)c->cfg.append_capacity, b = (size_t)b0, p0 = b * Hkv;
  auto e16 = [](const void* p, size_t elems) -> const void* {
    return p ? static_cast<const void*>(static_cast<const uint16_t*>(p) + elems) : nullptr;
  };
  s.q = e16(a->q, b * Hq * kD);
  s.prev_q = const_cast<void*>(e16(a->prev_q, b * Hq * kD));
  s.K_dev = e16(a->K_dev, p0 * N * kD);
  s.K_src = e16(a->K_src, p0 * N * kD);
  s.V_src = e16(a->V_src, p0 * N * kD);
  s.V_res = e16(a->V_res, b * (size_t)a->n_res * N * kD);
  s.K_slots = const_cast<void*>(e16(a->K_slots, p0 * k_max * kD));
  s.V_slots = const_cast<void*>(e16(a->V_slots, p0 * k_max * kD));
  s.K_app = e16(a->K_app, p0 * cap * kD);
  s.V_app = e16(a->V_app, p0 * cap * kD);
  s.slot_idx = a->slot_idx + p0 * k_max;
  s.out = a->out + b * Hq * kD;
  s.topk_idx = a->topk_idx + p0 * (size_t)a->k;
  s.hit_mask = a->hit_mask + p0 * (size_t)a->k;
  s.reuse_flags = a->reuse_flags + p0;
  s.sim = a->sim ? a->sim + b * Hq : nullptr;
  return s;
}

// What enqueue_range launches.  The whole step is gate, scoring + select (with the diff), and attention with
// the fill folded in or before it, as the context says; the staggered schedule asks for the pieces one by one,
// with the fill as the trickle kernel and the attention over slots that are already filled.
enum { kGate = 1, kScoreSelect = 2, kAttend = 4, kWholeStep = 7, kTrickleFill = 8, kAttendFilled = 16 };

// The step for the batch elements [b0, b0 + nb) on stream sm.  The modes that use both streams inside one range
// (and the stage timing) apply only to the whole batch on stream_main (`whole`).
int enqueue_range(qsac_ctx* c, const qsac_step_args* a_full, int b0, int nb, hipStream_t sm, int what, bool whole) {
  const qsac_step_args a_slice = slice_args(c, a_full, b0);
  const qsac_step_args* a = &a_slice;

  const qsac_ws_layout& L = c->L;
  char* ws = static_cast<char*>(c->cfg.workspace);
  u32* valid = reinterpret_cast<u32*>(ws + L.valid);
  int* set_sorted = reinterpret_cast<int*>(ws + L.set_sorted);
  u32* keys = reinterpret_cast<u32*>(ws + L.keys);
  u32* hist = reinterpret_cast<u32*>(ws + L.hist);
  u32* bm_new = reinterpret_cast<u32*>(ws + L.bm_new);
  u32* bm_eq = reinterpret_cast<u32*>(ws + L.bm_eq);
  u32* bm_old = reinterpret_cast<u32*>(ws + L.bm_old);
  int* miss_count = reinterpret_cast<int*>(ws + L.miss_count);
  int* miss_slot = reinterpret_cast<int*>(ws + L.miss_slot);
  int* miss_tok = reinterpret_cast<int*>(ws + L.miss_tok);
  float* part_ml = reinterpret_cast<float*>(ws + L.part_ml);
  float* part_acc = reinterpret_cast<float*>(ws + L.part_acc);
  u64* stats = reinterpret_cast<u64*>(ws + L.stats);
  const double* importance = reinterpret_cast<const double*>(ws + L.importance);
  int* sel_r = reinterpret_cast<int*>(ws + L.sel_r);
  int* fetch_tok = reinterpret_cast<int*>(ws + L.fetch_tok);

  const int G = c->G, k = a->k, k_max = c->cfg.k_max;
  const int Hq = c->cfg.n_q_heads, Hkv = c->cfg.n_kv_heads;
  const int P = nb * Hkv;
  const int64_t N = c->cfg.n_ctx;
  u64* glist = reinterpret_cast<u64*>(bm_new);  // (the list-building select keeps the pairs' lists there)
  int* chunk_cnt = reinterpret_cast<int*>(ws + L.chunk_cnt);
  {  // this range's part of every per-pair array of the workspace
    const size_t p0 = (size_t)b0 * (size_t)Hkv;
    valid += p0;
    set_sorted += p0 * (size_t)k_max;
    keys += p0 * (size_t)L.n_pad;
    hist += p0 * 3 * kBins;
    bm_new += p0 * (size_t)L.words;
    bm_eq += p0 * (size_t)L.words;
    bm_old += p0 * (size_t)L.words;
    miss_count += p0;
    miss_slot += p0 * (size_t)k_max;
    miss_tok += p0 * (size_t)k_max;
    part_ml += p0 * (size_t)G * (size_t)L.max_splits * 2;
    part_acc += p0 * (size_t)G * (size_t)L.max_splits * kD;
    sel_r += p0 * kSelStride;
    fetch_tok += p0 * (size_t)k_max;
    glist += p0 * (size_t)kStreamListCap;
    chunk_cnt += p0 * (size_t)(L.n_pad / kSelChunk) * 2;
  }
  const bool timed = whole && c->profile;

  if (timed) {
    int rc = drain_profile(c);
    if (rc != QSAC_OK) return rc;
  }
  auto mark = [&](int i) {
    if (timed) (void)hipEventRecord(c->prof[i], sm);
  };

  const DevParams* dp = reinterpret_cast<const DevParams*>(a->dev_params);
  TauArg tau;
  for (int h = 0; h < Hkv; ++h) tau.v[h] = dp ? 0.f : a->tau[a->n_tau == 1 ? 0 : h];
  FillSrc src;
  src.K_src = static_cast<const v4u*>(a->K_src);
  src.V_src = static_cast<const v4u*>(a->V_src);
  src.K_res = static_cast<const v4u*>(a->K_dev);
  src.V_res = static_cast<const v4u*>(a->V_res);
  src.n_res = a->res_slot ? a->n_res : 0;
  src.host_row_bytes = 256 * ((int)c->K_src_host + (int)c->V_src_host);
  for (int h = 0; h < 64; ++h) src.slot[h] = (a->res_slot && h < Hkv) ? a->res_slot[h] : -1;

  // 1. gate (+ label update on a miss)
  mark(0);
  if (!(what & kGate)) {
  } else if (c->cfg.dtype == QSAC_F16)
    qsac_gate_kernel<0><<<P, 256, 0, sm>>>(static_cast<const uint16_t*>(a->q), static_cast<uint16_t*>(a->prev_q),
                                           importance, tau, valid, set_sorted, a->topk_idx, a->hit_mask,
                                           a->reuse_flags, a->sim, miss_count, hist, stats, Hq, Hkv, G, k, k_max,
                                           !c->small, dp);
  else
    qsac_gate_kernel<1><<<P, 256, 0, sm>>>(static_cast<const uint16_t*>(a->q), static_cast<uint16_t*>(a->prev_q),
                                           importance, tau, valid, set_sorted, a->topk_idx, a->hit_mask,
                                           a->reuse_flags, a->sim, miss_count, hist, stats, Hq, Hkv, G, k, k_max,
                                           !c->small, dp);
  if (!(what & ~kGate)) {
    HIP_TRY(hipGetLastError());
    return QSAC_OK;
  }
  const int rows = attn_rows(P, k + a->n_app);
  const int n_splits = (k + a->n_app + rows - 1) / rows;
  dim3 fill_grid((unsigned)((k + kFillRows - 1) / kFillRows), (unsigned)P);
  auto fill_on = [&](hipStream_t s) {
    qsac_fill_kernel<<<fill_grid, 256, 0, s>>>(miss_count, miss_slot, miss_tok, src, static_cast<v4u*>(a->K_slots),
                                               static_cast<v4u*>(a->V_slots), Hkv, N, k_max);
  };
  auto attend = [&](hipStream_t s, int which) {
    const AttnArgs A = attn_args(c, a, fetch_tok, miss_count, part_ml, part_acc, rows, n_splits, which);
    QSAC_DISPATCH(launch_attn, c, s, A, src, P, (what & kAttendFilled) != 0);
  };
  auto combine = [&]() {
    if (n_splits > 1)
      qsac_combine_kernel<<<P * G, n_splits > 16 ? 512 : 128, 0, sm>>>(part_ml, part_acc, a->reuse_flags, a->out, Hq, Hkv, G, n_splits,
                                                 L.max_splits, 0);
  };
  const bool side_attn = whole && c->overlap && !c->fill_kernel && !c->push;  // reused heads are attended to beside the select
  const bool side_fill = whole && c->overlap && c->fill_kernel;               // the fill kernel runs beside their attention
  // push mode: the miss lists go to the host transfer threads, the polling kernel waits for their answer
  u32* push_state = reinterpret_cast<u32*>(ws + L.push);
  auto publish = [&]() {
    qsac_publish_kernel<<<P, 256, 0, sm>>>(miss_count, miss_slot, miss_tok, c->push->box, push_state, k_max, P);
  };
  auto poll = [&]() {
    const unsigned long long us = c->cfg.push_wait_us ? (unsigned long long)c->cfg.push_wait_us : 2000000ull;
    qsac_poll_kernel<<<1, 64, 0, sm>>>(c->push->box, push_state, us * 100ull);  // 100 ticks per microsecond
  };

  // 2. scores of the missing pairs
  mark(1);
  if (what & kScoreSelect) QSAC_DISPATCH(launch_score, c, a, keys, hist, P, sm);
  if (side_attn) {
    // The heads that reused need nothing from the miss path.  Their attention starts on the side stream once
    // the scoring pass has had the memory system to itself, and runs beside the select, which is latency
    // bound on a few compute units.
    HIP_TRY(hipEventRecord(c->ev_sel, sm));
    HIP_TRY(hipStreamWaitEvent(c->s_side, c->ev_sel, 0));
    attend(c->s_side, 1);
    HIP_TRY(hipEventRecord(c->ev_fill, c->s_side));
  }
  // 3. select the k best, diff against the cache slots
  mark(2);
  if (!(what & kScoreSelect)) {
  } else if (N <= kStreamMaxN) {
    // one workgroup per pair: the keys in its registers (vpt key vectors per thread), or streamed
    const int64_t nvec = (N + 3) / 4;
    const int vpt = nvec <= 2 * kDiffThreads ? 2 : nvec <= 4 * kDiffThreads ? 4 : nvec <= 8 * kDiffThreads ? 8 : 16;
    SelArgs S;
    S.reuse_flags = a->reuse_flags;
    S.keys = keys;
    S.valid = valid;
    S.slot_idx = a->slot_idx;
    S.set_sorted = set_sorted;
    S.topk_idx = a->topk_idx;
    S.hit_mask = a->hit_mask;
    S.miss_count = miss_count;
    S.miss_slot = miss_slot;
    S.miss_tok = miss_tok;
    S.fetch_tok = fetch_tok;
    S.stats = stats;
    S.N = N;
    S.n_pad = (int64_t)L.n_pad;
    S.Hkv = Hkv;
    S.k = k;
    S.k_max = k_max;
    S.bm_words = (int)((N + 63) / 64 * 2);
    S.list_cap = kSelectListCap;
    S.r_sample = c->small ? select_sample_rank(k, vpt) : 0;
    const size_t lds_sel = ((size_t)S.bm_words * 3 + 2 * (size_t)kSelectListCap) * sizeof(u32);
    if (!c->small) {
      // the first bitmap region of the grid-wide path (unused here, sized for this) holds the pairs' lists
      const dim3 grid((unsigned)((N + 4 * kStreamChunkVec * 1024 - 1) / (4 * kStreamChunkVec * 1024)), (unsigned)P);
      qsac_select_stream_kernel<1024><<<grid, 1024, lds_sel, sm>>>(S, hist, glist, kStreamListCap, sel_r, src);
    } else
    switch (vpt) {
      case 2: qsac_select_small_kernel<2, 1024><<<P, 1024, lds_sel, sm>>>(S, src); break;
      case 4: qsac_select_small_kernel<4, 1024><<<P, 1024, lds_sel, sm>>>(S, src); break;
      case 8: qsac_select_small_kernel<8, 1024><<<P, 1024, lds_sel, sm>>>(S, src); break;
      default: qsac_select_small_kernel<16, 1024><<<P, 1024, lds_sel, sm>>>(S, src); break;
    }
  } else {
    dim3 sel_grid((unsigned)(L.n_pad / kSelChunk), (unsigned)P);
    qsac_refine_kernel<1><<<sel_grid, 256, 0, sm>>>(a->reuse_flags, keys, hist, sel_r, N, L.n_pad, k);
    qsac_refine_kernel<2><<<sel_grid, 256, 0, sm>>>(a->reuse_flags, keys, hist, sel_r, N, L.n_pad, k);
    if (L.words > 8 * kDiffThreads && k <= kDiffListMax) {
      // Long contexts: the set becomes a token list written by the whole grid, and the one-workgroup diff works on
      // that list in LDS (one workgroup alone takes tens of microseconds to read bitmaps of this size).
      qsac_mark_kernel<<<sel_grid, 256, 0, sm>>>(a->reuse_flags, keys, hist, bm_new, bm_eq, bm_old, sel_r, chunk_cnt, N,
                                                L.n_pad, L.words, k);
      qsac_emit_kernel<<<sel_grid, 256, 0, sm>>>(a->reuse_flags, bm_new, bm_eq, chunk_cnt, sel_r, set_sorted,
                                                a->topk_idx, L.words, k, k_max);
      qsac_diff_list_kernel<<<P, kDiffThreads, (size_t)k * 13, sm>>>(a->reuse_flags, valid, a->slot_idx, set_sorted,
                                                                    a->topk_idx, a->hit_mask, miss_count, miss_slot,
                                                                    miss_tok, fetch_tok, stats, src, Hkv, k, k_max);
    } else {
      qsac_mark_kernel<<<sel_grid, 256, 0, sm>>>(a->reuse_flags, keys, hist, bm_new, bm_eq, bm_old, sel_r, nullptr, N,
                                                L.n_pad, L.words, k);
      // bitmap words per lane of the 1024-thread diff: 8 up to 262144 keys, 32 up to 2^20
#define QSAC_DIFF(WPL)                                                                                             \
  qsac_diff_kernel<WPL><<<P, kDiffThreads, 0, sm>>>(a->reuse_flags, valid, bm_new, bm_eq, bm_old, sel_r, a->slot_idx, \
                                                   set_sorted, a->topk_idx, a->hit_mask, miss_count, miss_slot,     \
                                                   miss_tok, fetch_tok, stats, src, Hkv, L.words, k, k_max)
      if (L.words <= 8 * kDiffThreads) QSAC_DIFF(8);
      else QSAC_DIFF(32);
#undef QSAC_DIFF
    }
  }
  if (what & kTrickleFill)
    qsac_fill_trickle_kernel<<<kTrickleWorkgroups, 256, (size_t)(P + 1) * sizeof(int), sm>>>(miss_count, miss_slot, miss_tok, src,
                                                               static_cast<v4u*>(a->K_slots),
                                                               static_cast<v4u*>(a->V_slots), Hkv, N, k_max, P);
  if (what & kAttendFilled) {
    attend(sm, 0);
    combine();
  }
  if (!(what & kAttend)) {
    HIP_TRY(hipGetLastError());
    return QSAC_OK;
  }
  // 4. fill the missing rows (own kernel, or folded into the attention kernel's loads); 5. attention
  if (side_attn) {
    attend(sm, 2);
    HIP_TRY(hipStreamWaitEvent(sm, c->ev_fill, 0));
    combine();
  } else if (side_fill) {
    // the fill runs on the side stream while the pairs that reused their cache are attended to
    HIP_TRY(hipEventRecord(c->ev_sel, sm));
    HIP_TRY(hipStreamWaitEvent(c->s_side, c->ev_sel, 0));
    fill_on(c->s_side);
    HIP_TRY(hipEventRecord(c->ev_fill, c->s_side));
    attend(sm, 1);
    HIP_TRY(hipStreamWaitEvent(sm, c->ev_fill, 0));
    attend(sm, 2);
    combine();
  } else if (c->push && !timed) {
    // the transfer runs beside the attention of the pairs that reused their cache
    publish();
    attend(sm, 1);
    poll();
    attend(sm, 2);
    combine();
  } else {
    mark(3);
    if (c->fill_kernel) fill_on(sm);
    if (c->push) {
      publish();
      poll();
    }
    mark(4);
    attend(sm, 0);
    mark(5);
    combine();
    mark(6);
    if (whole) c->prof_pending = c->profile;
  }
  HIP_TRY(hipGetLastError());
  return QSAC_OK;
}

// One step.  Staggered schedule (QSAC_FLAG_STAGGER): the gate for everybody, then the batch in up to
// kStaggerSlices slices, software-pipelined over the two streams: stream_main scores and selects slice i + 1,
// then attends to slice i; stream_side fills slice i's missing rows (trickle kernel) as soon as its select is
// through.  So the fetch of one slice (PCIe when the fill sources are host memory) runs beside the scoring of the
// next (HBM), the link waits for a scoring pass only once, at the start, and stream_side is joined back with the
// last slice's fill.
int enqueue_step(qsac_ctx* c, const qsac_step_args* a) {
  const int B = c->cfg.batch;
  if (!c->stagger) return enqueue_range(c, a, 0, B, c->s_main, kWholeStep, true);
  int rc = enqueue_range(c, a, 0, B, c->s_main, kGate, false);
  if (rc != QSAC_OK) return rc;
  // Slice sizes: a small first slice (B / 12), so that the link starts early, then each twice the one before:
  // beside the fill a scoring pass runs at a half to a third of its speed, and the scoring of slice i + 1 has to
  // be through before the fill of slice i is.  (First slice B/6 .. B/12, growth 1.5 or 2: 3.11 to 3.15 ms per step
  // of the largest workload.)
  int start[kStaggerSlices + 1];
  int n = 0;
  for (int at = 0, size = B / 12 > 0 ? B / 12 : 1; at < B; size *= 2) {
    start[n++] = at;
    at = (n == kStaggerSlices || B - at - size < size / 2) ? B : at + size;  // (a small rest joins the last slice)
  }
  start[n] = B;
  auto lo = [&](int i) { return start[i]; };
  for (int i = 0; i <= n; ++i) {
    if (i < n) {
      rc = enqueue_range(c, a, lo(i), lo(i + 1) - lo(i), c->s_main, kScoreSelect, false);
      if (rc != QSAC_OK) return rc;
      HIP_TRY(hipEventRecord(c->ev_selected[i], c->s_main));
      HIP_TRY(hipStreamWaitEvent(c->s_side, c->ev_selected[i], 0));
      rc = enqueue_range(c, a, lo(i), lo(i + 1) - lo(i), c->s_side, kTrickleFill, false);
      if (rc != QSAC_OK) return rc;
      HIP_TRY(hipEventRecord(c->ev_filled[i], c->s_side));
    }
    if (i > 0) {
      HIP_TRY(hipStreamWaitEvent(c->s_main, c->ev_filled[i - 1], 0));
      rc = enqueue_range(c, a, lo(i - 1), lo(i) - lo(i - 1), c->s_main, kAttendFilled, false);
      if (rc != QSAC_OK) return rc;
    }
  }
  return QSAC_OK;
}

}  // namespace

extern "C" {

size_t qsac_workspace_bytes(const qsac_config* cfg) {
  if (check_config(cfg) != QSAC_OK) return 0;
  qsac_ws_layout L;
  make_layout(cfg, &L);
  return L.total;
}

int qsac_workspace_layout(const qsac_config* cfg, qsac_ws_layout* out) {
  if (!out) return QSAC_ENULL;
  int rc = check_config(cfg);
  if (rc != QSAC_OK) return rc;
  make_layout(cfg, out);
  return QSAC_OK;
}

int qsac_init(const qsac_config* cfg, qsac_ctx** out) {
  if (!out) return QSAC_ENULL;
  *out = nullptr;
  int rc = check_config(cfg);
  if (rc != QSAC_OK) return rc;
  qsac_ws_layout L;
  make_layout(cfg, &L);
  const bool dry = (cfg->flags & QSAC_FLAG_DRY_RUN) != 0;
  if (!dry) {
    if ((cfg->flags & QSAC_FLAG_STAGGER) && (cfg->stream_side == nullptr || cfg->stream_side == cfg->stream_main))
      return QSAC_EINVAL;
    if (!cfg->workspace) return QSAC_EWORKSPACE;
    if (reinterpret_cast<uintptr_t>(cfg->workspace) & 255u) return QSAC_EWORKSPACE;
    if (cfg->workspace_bytes < L.total) return QSAC_EWORKSPACE;
  }
  qsac_ctx* c = new (std::nothrow) qsac_ctx();
  if (!c) return QSAC_EINVAL;
  fill_ctx(c, cfg, L);
  if (dry) {
    *out = c;
    return QSAC_OK;
  }
  auto fail = [&](int code) {
    qsac_free(c);
    return code;
  };
  if (hipEventCreateWithFlags(&c->ev_sel, hipEventDisableTiming) != hipSuccess ||
      hipEventCreateWithFlags(&c->ev_fill, hipEventDisableTiming) != hipSuccess) {
    g_last_hip = (int)hipGetLastError();
    return fail(QSAC_EHIP);
  }
  if (c->stagger)
    for (int i = 0; i < 2 * kStaggerSlices; ++i)
      if (hipEventCreateWithFlags(i < kStaggerSlices ? &c->ev_selected[i] : &c->ev_filled[i - kStaggerSlices],
                                  hipEventDisableTiming) != hipSuccess) {
        g_last_hip = (int)hipGetLastError();
        return fail(QSAC_EHIP);
      }
  if (c->profile)
    for (auto& e : c->prof)
      if (hipEventCreate(&e) != hipSuccess) {
        g_last_hip = (int)hipGetLastError();
        return fail(QSAC_EHIP);
      }
  rc = raise_lds_limits();
  if (rc != QSAC_OK) return fail(rc);
  rc = set_importance(c, cfg->q_head_importance);
  if (rc != QSAC_OK) return fail(rc);
  rc = clear_state(c);
  if (rc != QSAC_OK) return fail(rc);
  if (cfg->flags & QSAC_FLAG_PUSH_FILL) {
    rc = push_start(c);
    if (rc != QSAC_OK) return fail(rc);
  }
  *out = c;
  return QSAC_OK;
}

int qsac_reset(qsac_ctx* c) {
  if (!c || c->magic != kMagic) return QSAC_ESTATE;
  if (c->dry) {
    c->k_bound = 0;
    c->steps = 0;
    return QSAC_OK;
  }
  if (c->push) {
    // bring the device and the transfer threads back to a common starting point: nothing in flight, sequence 0
    HIP_TRY(hipStreamSynchronize(c->s_main));
    c->push->halt();
    int rc = push_rewind(c);
    if (rc != QSAC_OK) return rc;
    c->push->start(0);
  }
  return clear_state(c);
}

int qsac_step(qsac_ctx* c, const qsac_step_args* a) {
  if (!c || c->magic != kMagic) return QSAC_ESTATE;
  int rc = validate_step(c, a);
  if (rc != QSAC_OK) return rc;
  if (!c->dry) {
    note_fill_sources(c, a);
    if (c->push) {
      rc = push_submit(c, push_job_of(c, a), c->K_src_host && c->V_src_host);
      if (rc != QSAC_OK) return rc;
    }
    rc = enqueue_step(c, a);
    if (rc != QSAC_OK) {
      c->broken = true;  // part of the step may be enqueued: labels and slots can disagree until a reset
      return rc;
    }
  }
  c->k_bound = a->k;
  c->steps += 1;
  return QSAC_OK;
}

int qsac_graph_capture(qsac_ctx* c, const qsac_step_args* a, qsac_graph** out) {
  if (!out) return QSAC_ENULL;
  *out = nullptr;
  if (!c || c->magic != kMagic) return QSAC_ESTATE;
  if (c->dry || c->profile) return QSAC_ESTATE;
  int rc = validate_step(c, a);
  if (rc != QSAC_OK) return rc;
  if (!a->dev_params) return QSAC_ENULL;
  note_fill_sources(c, a);
  if (c->push && !(c->K_src_host && c->V_src_host)) return QSAC_EINVAL;
  qsac_graph* g = new (std::nothrow) qsac_graph();
  if (!g) return QSAC_EINVAL;
  HIP_TRY_OR(hipStreamBeginCapture(c->s_main, hipStreamCaptureModeThreadLocal), delete g);
  rc = enqueue_step(c, a);
  hipGraph_t graph = nullptr;
  const hipError_t e_end = hipStreamEndCapture(c->s_main, &graph);  // always leave capture mode
  if (rc == QSAC_OK && e_end != hipSuccess) {
    g_last_hip = (int)e_end;
    rc = QSAC_EHIP;
  }
  if (rc == QSAC_OK) {
    const hipError_t e_inst = hipGraphInstantiate(&g->exec, graph, nullptr, nullptr, 0);
    if (e_inst != hipSuccess) {
      g_last_hip = (int)e_inst;
      rc = QSAC_EHIP;
    }
  }
  if (graph) (void)hipGraphDestroy(graph);
  if (rc != QSAC_OK) {
    (void)hipGetLastError();
    delete g;
    return rc;  // nothing ran: the context is as it was
  }
  g->magic = kGraphMagic;
  g->ctx = c;
  g->k = a->k;
  g->job = push_job_of(c, a);
  *out = g;
  return QSAC_OK;
}

int qsac_graph_launch(qsac_graph* g) {
  if (!g || g->magic != kGraphMagic) return QSAC_ESTATE;
  qsac_ctx* c = g->ctx;
  if (!c || c->magic != kMagic || c->broken) return QSAC_ESTATE;
  if (c->k_bound != 0 && c->k_bound != g->k) return QSAC_ESTATE;
  if (c->push) {
    const int rc = push_submit(c, g->job, true);
    if (rc != QSAC_OK) return rc;
  }
  const hipError_t e = hipGraphLaunch(g->exec, c->s_main);
  if (e != hipSuccess) {
    g_last_hip = (int)e;
    c->broken = true;
    return QSAC_EHIP;
  }
  c->k_bound = g->k;
  c->steps += 1;
  return QSAC_OK;
}

int qsac_graph_free(qsac_graph* g) {
  if (!g || g->magic != kGraphMagic) return QSAC_ESTATE;
  (void)hipGraphExecDestroy(g->exec);
  g->magic = 0;
  delete g;
  return QSAC_OK;
}

namespace {

constexpr int kMaxStaticDevices = 64;
struct StaticSlot {
  bool ready;     // the device address of `scratch` is known and the LDS limits are raised on this device
  bool bound;     // a reset has bound a configuration
  void* ptr;      // device address of this GPU's copy of `scratch`
  qsac_ctx ctx;   // the layer context that lives in it (host fields; no events, no second stream)
};
StaticSlot g_static[kMaxStaticDevices];

bool same_shape(const qsac_config& a, const qsac_config& b) {
  return a.batch == b.batch && a.n_q_heads == b.n_q_heads && a.n_kv_heads == b.n_kv_heads && a.head_dim == b.head_dim &&
         a.n_ctx == b.n_ctx && a.k_max == b.k_max && a.dtype == b.dtype && a.flags == b.flags && a.n_sink == b.n_sink &&
         a.n_recent == b.n_recent && a.append_capacity == b.append_capacity && a.stream_main == b.stream_main;
}

}  // namespace

int qsac_step_static(const qsac_config* cfg, const qsac_step_args* a, int reset) {
  if (!cfg || !a) return QSAC_ENULL;
  int rc = check_config(cfg);
  if (rc != QSAC_OK) return rc;
  if (cfg->flags & ~(QSAC_FLAG_SCORE_VALU | QSAC_FLAG_FILL_KERNEL)) return QSAC_EINVAL;
  if (cfg->stream_side || (cfg->flags & QSAC_FLAG_STAGGER)) return QSAC_EINVAL;
  qsac_ws_layout L;
  make_layout(cfg, &L);
  if (L.total > (size_t)QSAC_STATIC_SCRATCH_BYTES) return QSAC_EWORKSPACE;
  int dev = -1;
  HIP_TRY(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxStaticDevices) return QSAC_ERANGE;
  StaticSlot& S = g_static[dev];
  if (!S.ready) {
    // once per device, with that device current: every GPU holds its own copy of the array at its own address
    void* ptr = nullptr;
    HIP_TRY(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
    if (!ptr || (reinterpret_cast<uintptr_t>(ptr) & 255u)) return QSAC_EWORKSPACE;
    rc = raise_lds_limits();
    if (rc != QSAC_OK) return rc;
    S.ptr = ptr;
    S.ready = true;
  }
  if (reset) {
    qsac_ctx fresh;
    fill_ctx(&fresh, cfg, L);
    fresh.cfg.workspace = S.ptr;
    fresh.cfg.workspace_bytes = QSAC_STATIC_SCRATCH_BYTES;
    rc = validate_step(&fresh, a);  // before anything is enqueued or the bound configuration changes
    if (rc != QSAC_OK) return rc;
    S.ctx = fresh;
    S.bound = true;
    // what must start at zero (validity flags, counters) is cleared by kernels on stream_main; everything else in
    // the array is written before it is read
    rc = set_importance(&S.ctx, cfg->q_head_importance);
    if (rc == QSAC_OK) rc = clear_state(&S.ctx);
    if (rc != QSAC_OK) {
      S.bound = false;
      return rc;
    }
  } else {
    if (!S.bound || !same_shape(S.ctx.cfg, *cfg)) return QSAC_ESTATE;
    rc = validate_step(&S.ctx, a);
    if (rc != QSAC_OK) return rc;
  }
  qsac_ctx* c = &S.ctx;
  note_fill_sources(c, a);
  rc = enqueue_step(c, a);
  if (rc != QSAC_OK) {
    c->broken = true;  // only a call with reset clears this
    return rc;
  }
  c->k_bound = a->k;
  c->steps += 1;
  return QSAC_OK;
}

int qsac_get_stats(qsac_ctx* c, qsac_stats* out) {
  if (!c || c->magic != kMagic) return QSAC_ESTATE;
  if (!out) return QSAC_ENULL;
  std::memset(out, 0, sizeof *out);
  out->steps = c->steps;
  if (c->dry) return QSAC_OK;
  unsigned long long dev[8];
  HIP_TRY(hipStreamSynchronize(c->s_main));
  HIP_TRY(hipMemcpy(dev, static_cast<char*>(c->cfg.workspace) + c->L.stats, sizeof dev, hipMemcpyDeviceToHost));
  if (c->push && __atomic_load_n(c->push->box + kPushTimeouts, __ATOMIC_ACQUIRE) != 0) {
    c->broken = true;
    return QSAC_ETIMEOUT;  // a polling kernel gave up: the steps since then attended to rows that were not there
  }
  out->reuse_heads = dev[1];
  out->miss_heads = dev[2];
  out->slot_hits = dev[3];
  out->slot_misses = dev[4];
  out->resident_rows = dev[5];
  out->guided_selects = dev[6];
  out->bytes_filled_host = dev[7];
  out->bytes_filled_dev = 512ull * dev[4] - dev[7];
  return QSAC_OK;
}

int qsac_get_stage_ms(qsac_ctx* c, double* ms_sum, uint64_t* n_steps) {
  if (!c || c->magic != kMagic) return QSAC_ESTATE;
  if (!ms_sum || !n_steps) return QSAC_ENULL;
  if (!c->profile) return QSAC_ESTATE;
  if (!c->dry) {
    int rc = drain_profile(c);
    if (rc != QSAC_OK) return rc;
  }
  for (int i = 0; i < kStages; ++i) ms_sum[i] = c->stage_ms[i];
  *n_steps = c->stage_calls;
  return QSAC_OK;
}

int qsac_free(qsac_ctx* c) {
  if (!c || c->magic != kMagic) return QSAC_ESTATE;
  if (c->push) {
    (void)hipStreamSynchronize(c->s_main);  // no polling kernel may still be waiting for the threads
    c->push->halt();
    if (c->push->box) (void)hipHostFree(c->push->box);
    delete c->push;
    c->push = nullptr;
  }
  if (!c->dry) {
    if (c->ev_sel) (void)hipEventDestroy(c->ev_sel);
    if (c->ev_fill) (void)hipEventDestroy(c->ev_fill);
    for (auto& e : c->ev_selected)
      if (e) (void)hipEventDestroy(e);
    for (auto& e : c->ev_filled)
      if (e) (void)hipEventDestroy(e);
    for (auto& e : c->prof)
      if (e) (void)hipEventDestroy(e);
  }
  c->magic = 0;
  delete c;
  return QSAC_OK;
}

const char* qsac_strerror(int code) {
  switch (code) {
    case QSAC_OK: return "ok";
    case QSAC_EINVAL: return "invalid value in an argument";
    case QSAC_ENULL: return "required pointer is NULL";
    case QSAC_ERANGE: return "size or count out of range (n_ctx is limited to 2^20, G to 8, n_kv_heads to 64)";
    case QSAC_EWORKSPACE: return "workspace missing, misaligned or too small";
    case QSAC_EHIP: return "HIP runtime call failed";
    case QSAC_ESTATE: return "bad handle, call out of order, or the context needs qsac_reset after a failed step";
    case QSAC_EALIGN: return "pointer is not 16-byte aligned";
    case QSAC_ETIMEOUT: return "push mode: a polling kernel gave up waiting for the host transfer threads";
    default: return "unknown error";
  }
}

int qsac_last_hip_error(void) { return g_last_hip; }

int qsac_adaptive_thresholds(const float* importance, int32_t n, float eta, float p, float* tau_out) {
  if (!importance || !tau_out) return QSAC_ENULL;
  if (n < 0) return QSAC_ERANGE;
  if (!(eta >= -1.f && eta <= 1.f) || !(p > 0.f) || !std::isfinite(p)) return QSAC_EINVAL;
  for (int i = 0; i < n; ++i)
    if (!(importance[i] >= 0.f && importance[i] <= 1.f)) return QSAC_EINVAL;
  const double pi = 3.14159265358979323846;
  const double theta_star = std::acos((double)eta);
  for (int i = 0; i < n; ++i) {
    const double lambda = std::pow((double)importance[i], (double)p);
    const double theta = lambda * theta_star + (1.0 - lambda) * pi;
    tau_out[i] = (float)std::cos(theta);
  }
  return QSAC_OK;
}

int qsac_reuse_difficulty(const float* tau, const float* avg_sim, int32_t n, float eps, float* d_out) {
  if (!tau || !avg_sim || !d_out) return QSAC_ENULL;
  if (n < 0) return QSAC_ERANGE;
  if (!(eps > 0.f) || !std::isfinite(eps)) return QSAC_EINVAL;
  for (int i = 0; i < n; ++i) d_out[i] = (float)((double)tau[i] - ((double)avg_sim[i] - (double)eps));
  return QSAC_OK;
}

int qsac_num_stages(void) { return kStages; }

const char* qsac_stage_name(int i) { return (i >= 0 && i < kStages) ? kStageNames[i] : nullptr; }

}  // extern "C"
