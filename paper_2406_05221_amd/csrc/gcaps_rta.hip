/*
 * gcaps_rta: C ABI and host logic of the batched response-time analysis for
 * gfx950 (see include/gcaps_rta.h for the contract of every entry point).
 *
 * Host side: argument checks, a grow-only pool of device scratch per context,
 * kernel launches on the context's stream.  Every step of the analysis runs in
 * the kernels; there is no host fallback.
 */
#include <hip/hip_runtime.h>

#include <cstdlib>
#include <mutex>
#include <new>
#include <utility>
#include <type_traits>

#include "gcaps_rta.h"

#include "rta_wide.hip.inc"
#include "rta_fast.hip.inc"
#include "rta_deep.hip.inc"
#include "rta_quad.hip.inc"
#include "rta_bin.hip.inc"
#include "gprio_wide.hip.inc"
#include "gprio_fast.hip.inc"
#include "gprio_tile.hip.inc"
#include "gprio_given.hip.inc"
#include "sim.hip.inc"
#include "taskgen_device.hip.inc"
#include "taskgen_table3.hip.inc"
#include "valu_probe.hip.inc"
#include "hbm_probe.hip.inc"

namespace {

typedef unsigned int u32;
typedef unsigned long long u64;

struct DeviceBuffer {
  void *ptr = nullptr;
  size_t bytes = 0;
  bool fixed = false; /* a slice of memory owned by someone else: never freed, never grown */
  /* grow-only: keeps the allocation when it is already large enough.  may_grow = false (the stream is
   * recording into a HIP graph, or the buffer is fixed): a larger request is refused and the
   * allocation is left as it is. */
  int reserve(size_t want, bool may_grow = true) {
    if (want <= bytes) return GCAPS_OK;
    if (fixed || !may_grow) return GCAPS_ESIZE;
    if (ptr) {
      if (hipFree(ptr) != hipSuccess) return GCAPS_EDEVICE;
      ptr = nullptr;
      bytes = 0;
    }
    if (hipMalloc(&ptr, want) != hipSuccess) {
      (void)hipGetLastError();
      ptr = nullptr;
      return GCAPS_ENOMEM;
    }
    bytes = want;
    return GCAPS_OK;
  }
  void release() {
    if (ptr && !fixed) (void)hipFree(ptr);
    ptr = nullptr;
    bytes = 0;
  }
};

/* the device scratch of the analysis launches */
struct Pool {
  DeviceBuffer status;       /* three blocks of fast::kStatusWords words: two used by alternate calls, the
                                third by calls that must not depend on their neighbours (recorded into a
                                HIP graph, or running in the static scratch) */
  DeviceBuffer wide_list;    /* taskset indices handed to the 64-bit kernel */
  DeviceBuffer deep_list;    /* taskset indices alive after the first fast launch */
  DeviceBuffer deep_sorted;  /* the same list, contiguous and ordered (binning) */
  DeviceBuffer deep_aux;     /* bucket and position inside the bucket of every list entry (binning) */
  DeviceBuffer wide_scratch; /* per-lane columns of the wide kernel */
  void release() {
    status.release();
    wide_list.release();
    deep_list.release();
    deep_sorted.release();
    deep_aux.release();
    wide_scratch.release();
  }
};

/*
 * Scratch of gcaps_rta_batch_device_static: one array per GPU that the library is loaded on,
 * held until the process ends.  Host code never uses the array's name as an address: the
 * address on a device is asked for once per device (scratch_on_device) and kept.
 */
constexpr size_t kStaticMaxTasksets = 65536; /* keep in step with include/gcaps_rta.h */
constexpr size_t kStaticMaxTasks = 32;
constexpr size_t kStaticWideSlots = 8192; /* lanes of the 64-bit kernel in a static call */
constexpr size_t kStaticRegionCap = ((kStaticMaxTasksets / 16 + 63) / 64) * 64;
constexpr size_t up256(size_t x) { return (x + 255) / 256 * 256; }
constexpr size_t kStaticStatusBytes = up256(3 * (size_t)fast::kStatusWords * sizeof(unsigned));
constexpr size_t kStaticListBytes = up256(kStaticMaxTasksets * sizeof(unsigned));
constexpr size_t kStaticDeepBytes = up256(kStaticRegionCap * 64 * sizeof(unsigned));
constexpr size_t kStaticColumnBytes = up256(kStaticWideSlots * kStaticMaxTasks * (4 * 4 + 3 * 8));
constexpr size_t kStaticScratchBytes =
    kStaticStatusBytes + 2 * kStaticListBytes + 3 * kStaticDeepBytes + kStaticColumnBytes;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

constexpr int kMaxDevices = 64;
void *g_scratch_of_device[kMaxDevices] = {};
std::mutex g_scratch_mutex;

/* address of `scratch` on device `dev`, which must be the current device; null on failure */
void *scratch_on_device(int dev) {
  if (dev < 0 || dev >= kMaxDevices) return nullptr;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_of_device[dev]) {
    void *p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess) {
      (void)hipGetLastError();
      return nullptr;
    }
    g_scratch_of_device[dev] = p;
  }
  return g_scratch_of_device[dev];
}

int npol(int policy) { return ((policy & 1) ? 1 : 0) + ((policy & 2) ? 1 : 0); }

}  // namespace

struct gcaps_ctx {
  int device = 0;
  hipStream_t stream = nullptr;
  int n_cu = 0;
  int binning = 0;
  int cont = 0;             /* continue-after-miss (gcaps_set_continue_after_miss) */
  u64 chunk_cap = 0;        /* GCAPS_CHUNK_TASKSETS: smaller chunks than the 32-bit limit needs (testing) */
  u32 sim_blocks_cap = 0;   /* GCAPS_SIM_BLOCKS: fewer workgroups per simulation launch than fit the GPU (testing:
                               every lane then takes many tasksets) */
  u32 screen_tasks = 4;     /* tasks per taskset analysed by the first fast launch (GCAPS_SCREEN_TASKS) */
  u32 deep_lanes = 4;       /* lanes per taskset in the second fast launch, 4 or 8 (GCAPS_DEEP_LANES) */
  bool gen_by_taskset = false; /* GCAPS_GEN_KERNEL=taskset: the generator with one lane per taskset */
  bool gprio_list = false;  /* GCAPS_GPRIO_KERNEL=list: the priority search as two launches with a list between them */
  bool legacy_deep = false; /* GCAPS_DEEP_KERNEL=lds: the second launch in its LDS-record form for every shape */
  size_t resp_stride = 0, sched_stride = 0; /* elements between the policies of the current call */
  u32 ts_offset = 0;                        /* first taskset of the current chunk */
  bool wide_only = false;   /* last call: shape outside the fast kernel, everything went 64-bit */
  u32 last_n_tasksets = 0;
  int lds_limit = 65536;     /* dynamic LDS a workgroup may ask for */
  Pool pool;                 /* device scratch of the analysis launches (grows on demand) */
  Pool static_pool;          /* the same buffers as fixed slices of the static scratch array */
  bool static_call = false;  /* the current call runs in the static scratch: no allocation */
  u32 *last_status = nullptr; /* status block of the most recent call */
  u32 status_parity = 0;     /* block of the most recent call that ran directly */
  u32 status_block = 0;      /* block of the current (most recent) call */
  bool next_prepared = false; /* the other block has been made ready by the last kernel of that call */
  u32 *next_status = nullptr; /* what the last kernel of the current chunk is to prepare, or null */
  bool capturing = false;     /* the stream is recording the current call into a HIP graph */
  u32 region_cap = 0;        /* slots per region of deep_list in the current chunk */
  size_t lds_total = 65536;  /* LDS of one CU */
  DeviceBuffer staging_in, staging_out; /* device copies for the host entry point */
  u32 *host_status = nullptr; /* pinned */
};

namespace {

u32 *status_of(const gcaps_ctx *ctx) {
  return (u32 *)ctx->pool.status.ptr + (size_t)ctx->status_block * fast::kStatusWords;
}

struct DeviceGuard {
  int prev = -1;
  bool ok = false;
  explicit DeviceGuard(int dev) {
    if (hipGetDevice(&prev) != hipSuccess) return;
    ok = (prev == dev) || (hipSetDevice(dev) == hipSuccess);
  }
  ~DeviceGuard() {
    if (ok && prev >= 0) (void)hipSetDevice(prev);
  }
};

int check_batch(const gcaps_batch *b, int policy, int wait_mode, const void *out_resp, const void *out_sched) {
  if (!b || !out_resp || !out_sched) return GCAPS_EINVAL;
  if (b->n_tasksets == 0 || b->n_tasks == 0 || b->n_tasks > 255 || b->max_gseg > 255) return GCAPS_EINVAL;
  if (!b->theta_us || !b->eps_us || !b->slice_us || !b->cpu_us || !b->period_us || !b->deadline_us ||
      !b->prio || !b->core || !b->n_gseg)
    return GCAPS_EINVAL;
  if (b->max_gseg > 0 && (!b->gm_us || !b->ge_us)) return GCAPS_EINVAL;
  if (policy < GCAPS_POLICY_GCAPS || policy > GCAPS_POLICY_BOTH) return GCAPS_EINVAL;
  if (wait_mode != GCAPS_WAIT_BUSY && wait_mode != GCAPS_WAIT_SUSPEND) return GCAPS_EINVAL;
  return GCAPS_OK;
}

/* lanes the wide kernel is launched with: enough to fill the chip, bounded so that
 * its scratch columns stay modest */
u32 wide_slots(const gcaps_ctx *ctx, u32 n_tasksets) {
  u32 cap = (u32)ctx->n_cu * 8u * 256u;
  if (ctx->static_call) cap = (u32)kStaticWideSlots; /* the kernel's lanes stride over the list */
  u32 want = (n_tasksets + 255u) / 256u * 256u;
  return want < cap ? want : cap;
}

/* the per-lane scratch columns of the one-lane-per-taskset kernels, for `slots` lanes */
int wide_columns(gcaps_ctx *ctx, u32 n_tasks, u32 slots, wide::Scratch *ws) {
  const size_t col = (size_t)slots * n_tasks;
  const size_t bytes = col * (4 * sizeof(u32) + 3 * sizeof(u64));
  int rc = ctx->pool.wide_scratch.reserve(bytes, !ctx->capturing);
  if (rc != GCAPS_OK) return rc;
  char *base = (char *)ctx->pool.wide_scratch.ptr;
  ws->CGm = (u64 *)base;
  ws->Ge = ws->CGm + col;
  ws->K = ws->Ge + col;
  ws->T = (u32 *)(ws->K + col);
  ws->D = ws->T + col;
  ws->meta = ws->D + col;
  ws->R = ws->meta + col;
  ws->n_slots = slots;
  return GCAPS_OK;
}

int launch_wide(gcaps_ctx *ctx, const gcaps_batch *b, int policy, int wait_mode, int64_t *d_resp,
                uint8_t *d_sched, const u32 *d_list, const u32 *d_list_count, u32 max_items) {
  const u32 slots = wide_slots(ctx, max_items);
  wide::Scratch ws;
  int rc = wide_columns(ctx, b->n_tasks, slots, &ws);
  if (rc != GCAPS_OK) return rc;
  hipLaunchKernelGGL(wide::rta_wide_kernel, dim3(slots / 256), dim3(256), 0, ctx->stream, *b, policy,
                     wait_mode, (long long *)d_resp, d_sched, status_of(ctx), ws, d_list, d_list_count,
                     ctx->resp_stride, ctx->sched_stride, ctx->ts_offset, ctx->cont != 0, ctx->next_status,
                     (u32)fast::kStatusWords);
  return hipGetLastError() == hipSuccess ? GCAPS_OK : GCAPS_EDEVICE;
}

/* Clears the per-call device words with a kernel (not a memset node) so that a caller
 * may capture the launches of one call into a HIP graph.  Outside a capture the first chunk of
 * a call does not need it (see begin_chunk). */
__global__ void reset_status_kernel(u32 *status, int first_chunk) {
  if (threadIdx.x == 0) {
    if (first_chunk) {
      status[0] = 0xffffffffu; /* smallest invalid taskset index of the call */
      status[3] = 0;           /* tasksets sent to the 64-bit kernel by earlier chunks */
      status[4] = 0;           /* steps of the schedule simulation, 64 bits */
      status[5] = 0;
    } else {
      status[3] += status[1];
    }
    status[1] = 0; /* length of the list for the 64-bit kernel */
    status[2] = 0; /* length of the ordered list for the second fast launch (binning only) */
  }
  status[fast::ST_DEEP_COUNTS + threadIdx.x] = 0; /* per-region lengths of the list for the second fast launch */
  for (u32 k = threadIdx.x; k < fast::kOrderBuckets; k += blockDim.x) status[fast::ST_ORDER_HIST + k] = 0;
  status[fast::ST_CLAIM + threadIdx.x] = 0; /* tiles handed out by the persistent launch (kClaimCounters = 64 words) */
}

/* Status words at the start of a chunk.  The first chunk of a call finds its block prepared by the
 * last kernel of the previous call (see wide::prepare_next_call); otherwise a small kernel does it. */
int begin_chunk(gcaps_ctx *ctx, bool first_chunk) {
  if (first_chunk && ctx->next_prepared && !ctx->capturing && !ctx->static_call) {
    ctx->next_prepared = false;
    return GCAPS_OK;
  }
  hipLaunchKernelGGL(reset_status_kernel, dim3(1), dim3(64), 0, ctx->stream, status_of(ctx), first_chunk ? 1 : 0);
  return hipGetLastError() == hipSuccess ? GCAPS_OK : GCAPS_EDEVICE;
}

/* the list between the two fast launches: regions filled by the first launch, or (binning) the
 * contiguous list ordered by bucket */
fast::ListSpec deep_list_spec(const gcaps_ctx *ctx, bool sorted) {
  u32 *status = status_of(ctx);
  if (sorted)
    return fast::ListSpec{(u32 *)ctx->pool.deep_sorted.ptr, status + fast::ST_DEEP_TOTAL, 1u, 0u, nullptr, nullptr, nullptr};
  fast::ListSpec dl{(u32 *)ctx->pool.deep_list.ptr, status + fast::ST_DEEP_COUNTS, fast::kListRegions, ctx->region_cap,
                    nullptr, nullptr, nullptr};
  if (ctx->binning) {
    dl.keys = (u32 *)ctx->pool.deep_aux.ptr;
    dl.positions = dl.keys + (size_t)ctx->region_cap * fast::kListRegions;
    dl.hist = status + fast::ST_ORDER_HIST;
  }
  return dl;
}

template <int TS, int NP>
int launch_fast_np(gcaps_ctx *ctx, const gcaps_batch *b, int policy, int wait_mode, int64_t *d_resp,
                   uint8_t *d_sched, u32 kr, u32 blocks) {
  const size_t lds = fast::lds_bytes(b->n_tasks, kr, TS, false);
  fast::ListSpec dl = deep_list_spec(ctx, false);
  hipLaunchKernelGGL((fast::rta_fast_kernel<TS, NP>), dim3(blocks), dim3(64), lds, ctx->stream, *b,
                     policy, wait_mode, (long long *)d_resp, d_sched, status_of(ctx),
                     (u32 *)ctx->pool.wide_list.ptr, dl, kr, ctx->resp_stride, ctx->sched_stride, ctx->ts_offset);
  return hipGetLastError() == hipSuccess ? GCAPS_OK : GCAPS_EDEVICE;
}

int launch_screen(gcaps_ctx *ctx, const gcaps_batch *b, int policy, int wait_mode, int64_t *d_resp,
                  uint8_t *d_sched, u32 kr, u32 blocks) {
  const size_t lds = fast::lds_bytes(b->n_tasks, kr, 64, true);
  const fast::ListSpec dl = deep_list_spec(ctx, false);
  if (wait_mode == GCAPS_WAIT_BUSY)
    hipLaunchKernelGGL(fast::rta_screen_kernel<true>, dim3(blocks), dim3(64), lds, ctx->stream, *b, policy,
                       (long long *)d_resp, d_sched, status_of(ctx), (u32 *)ctx->pool.wide_list.ptr, dl, kr,
                       ctx->resp_stride, ctx->sched_stride, ctx->ts_offset);
  else
    hipLaunchKernelGGL(fast::rta_screen_kernel<false>, dim3(blocks), dim3(64), lds, ctx->stream, *b, policy,
                       (long long *)d_resp, d_sched, status_of(ctx), (u32 *)ctx->pool.wide_list.ptr, dl, kr,
                       ctx->resp_stride, ctx->sched_stride, ctx->ts_offset);
  return hipGetLastError() == hipSuccess ? GCAPS_OK : GCAPS_EDEVICE;
}

/* NP: register slots for the terms of one task (ranks analysed in this launch, rounded up);
 * only the 64-wide tile has register variants, everything else loops over LDS */
template <int TS>
int launch_fast(gcaps_ctx *ctx, const gcaps_batch *b, int policy, int wait_mode, int64_t *d_resp,
                uint8_t *d_sched, u32 kr, u32 blocks) {
  if constexpr (TS == 64) {
    if (kr <= (u32)fast::kCacheRanks && b->max_gseg <= (u32)fast::kCacheSegs && b->n_tasks <= 255)
        return launch_screen(ctx, b, policy, wait_mode, d_resp, d_sched, kr, blocks);
    if (kr <= 4) return launch_fast_np<TS, 4>(ctx, b, policy, wait_mode, d_resp, d_sched, kr, blocks);
    if (kr <= 8) return launch_fast_np<TS, 8>(ctx, b, policy, wait_mode, d_resp, d_sched, kr, blocks);
    if (kr <= 16) return launch_fast_np<TS, 16>(ctx, b, policy, wait_mode, d_resp, d_sched, kr, blocks);
    if (kr <= 24) return launch_fast_np<TS, 24>(ctx, b, policy, wait_mode, d_resp, d_sched, kr, blocks);
    if (kr <= 32) return launch_fast_np<TS, 32>(ctx, b, policy, wait_mode, d_resp, d_sched, kr, blocks);
  }
  return launch_fast_np<TS, 0>(ctx, b, policy, wait_mode, d_resp, d_sched, kr, blocks);
}

/* second launch: the listed tasksets in full, 64 / Q per wavefront; persistent workgroups */
template <bool BUSY, int Q, bool CONT>
int launch_deep_q(gcaps_ctx *ctx, const gcaps_batch *b, int policy, int64_t *d_resp, uint8_t *d_sched, u32 kr) {
  const u32 n = b->n_tasks, N = b->n_tasksets, ts = 64u / (u32)Q;
  const size_t lds = fast::deep_lds_bytes(n, Q);
  /* Exactly as many workgroups as are resident at once (LDS and registers both limit it): a
   * workgroup's first tile is its own index, so one that had to wait for a free slot would start
   * that tile only after the others have drained the queue. */
  int per_cu = 0;
  const void *fn = (const void *)fast::rta_deep_kernel<BUSY, Q, CONT>;
  if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, fn, 64, lds) != hipSuccess || per_cu < 1) {
    (void)hipGetLastError();
    per_cu = 1;
  }
  u32 blocks = (u32)ctx->n_cu * (u32)per_cu;
  const u32 max_tiles = (N + ts - 1) / ts + fast::kListRegions;
  if (blocks > max_tiles) blocks = max_tiles;
  fast::ListSpec dl = deep_list_spec(ctx, ctx->binning != 0 && !CONT);
  if (CONT) dl = fast::ListSpec{nullptr, nullptr, 1u, N, nullptr, nullptr, nullptr}; /* every taskset */
  hipLaunchKernelGGL((fast::rta_deep_kernel<BUSY, Q, CONT>), dim3(blocks), dim3(64), lds, ctx->stream, *b, policy,
                     (long long *)d_resp, d_sched, status_of(ctx), (u32 *)ctx->pool.wide_list.ptr, dl, kr,
                     ctx->resp_stride, ctx->sched_stride, ctx->ts_offset);
  return hipGetLastError() == hipSuccess ? GCAPS_OK : GCAPS_EDEVICE;
}

/* second launch in its register form (rta_quad.hip.inc): four lanes per taskset, n <= 4 * NSMAX */
template <bool BUSY, int NSMAX, int SEGS>
int launch_quad(gcaps_ctx *ctx, const gcaps_batch *b, int policy, int64_t *d_resp, uint8_t *d_sched, u32 kr,
                const fast::ListSpec &dl) {
  const u32 n = b->n_tasks, N = b->n_tasksets;
  const size_t lds = fast::quad_lds_bytes(n);
  /* exactly as many workgroups as are resident at once: a workgroup's first tile is its own index */
  int per_cu = 0;
  const void *fn = (const void *)fast::rta_quad_kernel<BUSY, NSMAX, SEGS>;
  if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, fn, 64, lds) != hipSuccess || per_cu < 1) {
    (void)hipGetLastError();
    per_cu = 1;
  }
  u32 blocks = (u32)ctx->n_cu * (u32)per_cu;
  const u32 max_tiles = (N + 15u) / 16u + fast::kListRegions;
  if (blocks > max_tiles) blocks = max_tiles;
  hipLaunchKernelGGL((fast::rta_quad_kernel<BUSY, NSMAX, SEGS>), dim3(blocks), dim3(64), lds, ctx->stream, *b, policy,
                     (long long *)d_resp, d_sched, status_of(ctx), (u32 *)ctx->pool.wide_list.ptr, dl, kr,
                     ctx->resp_stride, ctx->sched_stride);
  return hipGetLastError() == hipSuccess ? GCAPS_OK : GCAPS_EDEVICE;
}

int launch_quad_any(gcaps_ctx *ctx, const gcaps_batch *b, int policy, int wait_mode, int64_t *d_resp,
                    uint8_t *d_sched, u32 kr, const fast::ListSpec &dl) {
  const bool busy = wait_mode == GCAPS_WAIT_BUSY;
#define GCAPS_QUAD_S(NS, SEGS)                                                  \
  (busy ? launch_quad<true, NS, SEGS>(ctx, b, policy, d_resp, d_sched, kr, dl) \
        : launch_quad<false, NS, SEGS>(ctx, b, policy, d_resp, d_sched, kr, dl))
#define GCAPS_QUAD(NS)                                                                           \
  (b->max_gseg <= 3 ? GCAPS_QUAD_S(NS, 3)                                                        \
   : b->max_gseg <= 4 ? GCAPS_QUAD_S(NS, 4)                                                      \
                    : b->max_gseg <= (u32)fast::kPrefetchSegs ? GCAPS_QUAD_S(NS, fast::kPrefetchSegs) \
                                                              : GCAPS_QUAD_S(NS, 0))
  if (b->n_tasks <= 20) return GCAPS_QUAD(5);
  if (b->n_tasks <= 24) return GCAPS_QUAD(6);
  return GCAPS_QUAD(8);
#undef GCAPS_QUAD
#undef GCAPS_QUAD_S
}

bool quad_applies(const gcaps_ctx *ctx, const gcaps_batch *b, u32 kr) {
  return !ctx->cont && ctx->deep_lanes == 4 && b->n_tasks <= fast::kQuadMaxTasks && !ctx->legacy_deep && kr <= 4u;
}

template <bool CONT>
int launch_deep_c(gcaps_ctx *ctx, const gcaps_batch *b, int policy, int wait_mode, int64_t *d_resp,
                  uint8_t *d_sched, u32 kr) {
  const bool busy = wait_mode == GCAPS_WAIT_BUSY;
  if (ctx->deep_lanes == 8)
    return busy ? launch_deep_q<true, 8, CONT>(ctx, b, policy, d_resp, d_sched, kr)
                : launch_deep_q<false, 8, CONT>(ctx, b, policy, d_resp, d_sched, kr);
  return busy ? launch_deep_q<true, 4, CONT>(ctx, b, policy, d_resp, d_sched, kr)
              : launch_deep_q<false, 4, CONT>(ctx, b, policy, d_resp, d_sched, kr);
}

int launch_deep(gcaps_ctx *ctx, const gcaps_batch *b, int policy, int wait_mode, int64_t *d_resp,
                uint8_t *d_sched, u32 kr) {
  if (quad_applies(ctx, b, kr))
    return launch_quad_any(ctx, b, policy, wait_mode, d_resp, d_sched, kr, deep_list_spec(ctx, ctx->binning != 0));
  return ctx->cont ? launch_deep_c<true>(ctx, b, policy, wait_mode, d_resp, d_sched, kr)
                   : launch_deep_c<false>(ctx, b, policy, wait_mode, d_resp, d_sched, kr);
}

/* widest tile (tasksets per wavefront) whose LDS rows fit, 0 if none */
int tile_width(const gcaps_ctx *ctx, u32 n, u32 kr) {
  for (int ts = 64; ts >= 16; ts /= 2)
    if (fast::lds_bytes(n, kr, (u32)ts, false) <= (size_t)ctx->lds_limit) return ts;
  return 0;
}


/* one chunk: every array of it stays below 4 GiB, so the kernels index with 32 bits */
int run_chunk(gcaps_ctx *ctx, const gcaps_batch *b, int policy, int wait_mode, int64_t *d_resp,
              uint8_t *d_sched, bool first_chunk) {
  if (begin_chunk(ctx, first_chunk) != GCAPS_OK) return GCAPS_EDEVICE;
  const u32 n = b->n_tasks, N = b->n_tasksets;
  const u32 kr = n > ctx->screen_tasks ? ctx->screen_tasks : n;
  const int ts_screen = n <= fast::kMaxTasks ? tile_width(ctx, n, kr) : 0;
  ctx->wide_only = ts_screen == 0 || (kr < n && fast::deep_lds_bytes(n, ctx->deep_lanes) > (size_t)ctx->lds_limit);
  if (ctx->cont) /* the full-depth launch alone */
    ctx->wide_only = n > fast::kMaxTasks || fast::deep_lds_bytes(n, ctx->deep_lanes) > (size_t)ctx->lds_limit;
  if (ctx->wide_only) return launch_wide(ctx, b, policy, wait_mode, d_resp, d_sched, nullptr, nullptr, N);
  int rc = ctx->pool.wide_list.reserve((size_t)N * sizeof(u32), !ctx->capturing);
  /* tiles of the first launch go to the list regions round-robin: a region never overflows */
  const u32 producer_tiles = (N + 15u) / 16u; /* the narrowest tile width */
  ctx->region_cap = ((producer_tiles + fast::kListRegions - 1) / fast::kListRegions) * 64u;
  if (rc == GCAPS_OK) rc = ctx->pool.deep_list.reserve((size_t)ctx->region_cap * fast::kListRegions * sizeof(u32), !ctx->capturing);
  if (rc == GCAPS_OK && ctx->binning)
    rc = ctx->pool.deep_aux.reserve((size_t)ctx->region_cap * fast::kListRegions * 2 * sizeof(u32), !ctx->capturing);
  if (rc != GCAPS_OK) return rc;

  if (ctx->cont) {
    /* continue-after-miss: nothing is settled early, the full-depth launch takes every taskset */
    rc = launch_deep(ctx, b, policy, wait_mode, d_resp, d_sched, 0u);
    if (rc != GCAPS_OK) return rc;
    const u32 *count = (const u32 *)status_of(ctx) + fast::ST_WIDE_COUNT;
    return launch_wide(ctx, b, policy, wait_mode, d_resp, d_sched, (const u32 *)ctx->pool.wide_list.ptr, count,
                       N < 65536u ? N : 65536u);
  }

  /* first launch: every taskset, the kr highest-priority tasks only */
  const u32 tiles = (N + (u32)ts_screen - 1) / (u32)ts_screen;
  rc = ts_screen == 64 ? launch_fast<64>(ctx, b, policy, wait_mode, d_resp, d_sched, kr, tiles)
     : ts_screen == 32 ? launch_fast<32>(ctx, b, policy, wait_mode, d_resp, d_sched, kr, tiles)
                       : launch_fast<16>(ctx, b, policy, wait_mode, d_resp, d_sched, kr, tiles);
  if (rc != GCAPS_OK) return rc;

  /* second launch: the tasksets still alive, in full; persistent workgroups walk the list */
  if (kr < n && ctx->binning) {
    /* the list ordered by the bucket that the first launch gave every entry */
    rc = ctx->pool.deep_sorted.reserve((size_t)N * sizeof(u32), !ctx->capturing);
    if (rc != GCAPS_OK) return rc;
    u32 *status = status_of(ctx);
    hipLaunchKernelGGL(bin::order_kernel, dim3(fast::kListRegions), dim3(256), 0, ctx->stream,
                       deep_list_spec(ctx, false), (const u32 *)(status + fast::ST_ORDER_HIST),
                       (u32 *)ctx->pool.deep_sorted.ptr, status + fast::ST_DEEP_TOTAL);
    if (hipGetLastError() != hipSuccess) return GCAPS_EDEVICE;
  }
  if (kr < n) {
    rc = launch_deep(ctx, b, policy, wait_mode, d_resp, d_sched, kr);
    if (rc != GCAPS_OK) return rc;
  }
  /* whatever the fast launches handed over is redone in 64 bit; usually nothing */
  const u32 *count = (const u32 *)status_of(ctx) + fast::ST_WIDE_COUNT;
  const u32 items = N < 65536u ? N : 65536u;
  return launch_wide(ctx, b, policy, wait_mode, d_resp, d_sched, (const u32 *)ctx->pool.wide_list.ptr, count, items);
}

/* Splits a call into chunks of tasksets small enough for the kernels' 32-bit byte offsets:
 * within a chunk every input array and each block of responses stays below 4 GiB.
 * run(sub-batch, first taskset of the chunk) is called per chunk. */
template <class F>
int for_chunks(gcaps_ctx *ctx, const gcaps_batch *b, F run) {
  const u64 n = b->n_tasks, S = b->max_gseg ? b->max_gseg : 1, N = b->n_tasksets;
  u64 chunk = (1ull << 28) / n;                 /* 8-byte responses: N*n*8 < 2^31 */
  const u64 by_seg = (1ull << 30) / (n * S);    /* 4-byte segments:  N*n*S*4 < 2^32 */
  if (by_seg < chunk) chunk = by_seg;
  if (ctx->chunk_cap && ctx->chunk_cap < chunk) chunk = ctx->chunk_cap;
  if (chunk > 64) chunk &= ~63ull;
  if (chunk < 1) chunk = 1;
  ctx->last_n_tasksets = b->n_tasksets;
  /* This call takes the status block the previous call did not use; the last kernel of its last
   * chunk prepares the other one for the call after it.  Launches that the stream is recording
   * into a HIP graph must depend on nothing that ran before the graph and leave nothing behind
   * that a later call relies on (a replay happens without this code knowing): such a call uses a
   * block of its own, always starts with the reset kernel and prepares nothing. */
  hipStreamCaptureStatus capture = hipStreamCaptureStatusNone;
  if (hipStreamIsCapturing(ctx->stream, &capture) != hipSuccess) {
    (void)hipGetLastError();
    capture = hipStreamCaptureStatusNone;
  }
  ctx->capturing = capture != hipStreamCaptureStatusNone;
  /* a call in the static scratch is as self-contained as a recorded one: a block of status words of
   * its own, reset first, nothing prepared for a later call */
  const bool isolated = ctx->capturing || ctx->static_call;
  if (isolated) {
    ctx->status_block = 2u;
  } else {
    ctx->status_parity ^= 1u;
    ctx->status_block = ctx->status_parity;
  }
  ctx->last_status = status_of(ctx);
  bool prepared = false;
  for (u64 c0 = 0; c0 < N; c0 += chunk) {
    const bool last_chunk = c0 + chunk >= N;
    ctx->next_status = (last_chunk && !isolated)
                           ? (u32 *)ctx->pool.status.ptr + (size_t)(ctx->status_parity ^ 1u) * fast::kStatusWords
                           : nullptr;
    gcaps_batch sub = *b;
    const u64 cn = N - c0 < chunk ? N - c0 : chunk;
    sub.n_tasksets = (u32)cn;
    if (sub.theta_us) sub.theta_us += c0;
    sub.eps_us += c0;
    if (sub.slice_us) sub.slice_us += c0;
    sub.cpu_us += c0 * n;
    sub.period_us += c0 * n;
    if (sub.deadline_us) sub.deadline_us += c0 * n;
    sub.prio += c0 * n;
    sub.core += c0 * n;
    sub.n_gseg += c0 * n;
    if (sub.n_cseg) sub.n_cseg += c0 * n;
    if (sub.gm_us) sub.gm_us += c0 * n * b->max_gseg;
    if (sub.ge_us) sub.ge_us += c0 * n * b->max_gseg;
    ctx->ts_offset = (u32)c0;
    const int rc = run(&sub, c0);
    ctx->next_status = nullptr;
    if (rc != GCAPS_OK) {
      if (!isolated) ctx->next_prepared = false; /* the next call resets its block itself */
      return rc;
    }
    prepared = last_chunk;
  }
  if (!isolated) ctx->next_prepared = prepared; /* a recorded call changes nothing for the others */
  return GCAPS_OK;
}

/* A call of one launch that reports through gcaps_status: a status block of its own, reset first; nothing
 * prepares the block of the call after it. */
int begin_single_call(gcaps_ctx *ctx) {
  hipStreamCaptureStatus capture = hipStreamCaptureStatusNone;
  if (hipStreamIsCapturing(ctx->stream, &capture) != hipSuccess) {
    (void)hipGetLastError();
    capture = hipStreamCaptureStatusNone;
  }
  ctx->capturing = capture != hipStreamCaptureStatusNone;
  const bool isolated = ctx->capturing || ctx->static_call;
  if (isolated) {
    ctx->status_block = 2u;
  } else {
    ctx->status_parity ^= 1u;
    ctx->status_block = ctx->status_parity;
  }
  ctx->last_status = status_of(ctx);
  ctx->next_status = nullptr;
  ctx->wide_only = true;
  ctx->last_n_tasksets = 0;
  const int rc = begin_chunk(ctx, true);
  if (!isolated) ctx->next_prepared = false;
  return rc;
}

int run_device(gcaps_ctx *ctx, const gcaps_batch *b, int policy, int wait_mode, int64_t *d_resp,
               uint8_t *d_sched) {
  const u64 n = b->n_tasks, N = b->n_tasksets;
  ctx->resp_stride = (size_t)(N * n);
  ctx->sched_stride = (size_t)N;
  return for_chunks(ctx, b, [&](const gcaps_batch *sub, u64 c0) {
    return run_chunk(ctx, sub, policy, wait_mode, d_resp + c0 * n, d_sched + c0, c0 == 0);
  });
}

/* GPU-segment priority assignment of one chunk */
int run_gprio_chunk(gcaps_ctx *ctx, const gcaps_batch *b, int wait_mode, const uint8_t *d_skip, int32_t *d_gprio,
                    int64_t *d_resp, uint8_t *d_sched, bool first_chunk) {
  if (begin_chunk(ctx, first_chunk) != GCAPS_OK) return GCAPS_EDEVICE;
  const u32 N = b->n_tasksets, n = b->n_tasks;
  u32 *status = status_of(ctx);
  /* the quad-lane kernel takes shapes up to 32 tasks; what it cannot represent in 24 bits it lists */
  ctx->wide_only = n > 32 || gprio::gprio_lds_bytes(n) > (size_t)ctx->lds_limit ||
                   gprio::tile_lds_bytes(n, 16u) > (size_t)ctx->lds_limit;
  const u32 *d_list = nullptr, *d_count = nullptr;
  u32 items = N;
  if (!ctx->wide_only && !ctx->gprio_list) {
    /* one pass: a wavefront per tile of consecutive tasksets reads them once, settles or searches them, and
     * writes their outputs */
    int rc = ctx->pool.wide_list.reserve((size_t)N * sizeof(u32), !ctx->capturing);
    if (rc != GCAPS_OK) return rc;
    u32 *wl = (u32 *)ctx->pool.wide_list.ptr;
    const bool busy = wait_mode == GCAPS_WAIT_BUSY;
    /* sixteen tasksets per wavefront: wider tiles (32, 64) fill the quads of the search better but hold fewer
     * wavefronts per compute unit, and measured slower on every workload */
    constexpr u32 tw = 16;
    const size_t lds = gprio::tile_lds_bytes(n, tw);
    const dim3 grid((N + tw - 1u) / tw), block(64);
#define GCAPS_GPRIO_TILE(BUSY, NS)                                                                       \
  hipLaunchKernelGGL((gprio::gprio_tile_kernel<BUSY, NS, 16>), grid, block, lds, ctx->stream, *b, d_skip, \
                     (int *)d_gprio, (long long *)d_resp, d_sched, status, wl, ctx->ts_offset)
    if (n <= 20) {
      if (busy) GCAPS_GPRIO_TILE(true, 5); else GCAPS_GPRIO_TILE(false, 5);
    } else {
      if (busy) GCAPS_GPRIO_TILE(true, 8); else GCAPS_GPRIO_TILE(false, 8);
    }
#undef GCAPS_GPRIO_TILE
    if (hipGetLastError() != hipSuccess) return GCAPS_EDEVICE;
    d_list = wl;
    d_count = status + fast::ST_WIDE_COUNT;
    items = N < 65536u ? N : 65536u;
  } else if (!ctx->wide_only) {
    int rc = ctx->pool.wide_list.reserve((size_t)N * sizeof(u32), !ctx->capturing);
    /* tiles of the first launch go to the list regions round-robin: a region never overflows */
    const u32 producer_tiles = (N + 63u) / 64u;
    ctx->region_cap = ((producer_tiles + fast::kListRegions - 1) / fast::kListRegions) * 64u;
    if (rc == GCAPS_OK) rc = ctx->pool.deep_list.reserve((size_t)ctx->region_cap * fast::kListRegions * sizeof(u32), !ctx->capturing);
    if (rc != GCAPS_OK) return rc;
    const fast::ListSpec dl{(u32 *)ctx->pool.deep_list.ptr, status + fast::ST_DEEP_COUNTS, fast::kListRegions,
                            ctx->region_cap, nullptr, nullptr, nullptr};
    u32 *wl = (u32 *)ctx->pool.wide_list.ptr;
    const bool busy = wait_mode == GCAPS_WAIT_BUSY;
    /* first launch: every taskset; settles what needs no search and lists the rest */
    hipLaunchKernelGGL(gprio::gprio_screen_kernel, dim3(producer_tiles), dim3(64), 0, ctx->stream, *b, d_skip,
                       (int *)d_gprio, (long long *)d_resp, d_sched, status, wl, dl, ctx->ts_offset);
    if (hipGetLastError() != hipSuccess) return GCAPS_EDEVICE;
    /* second launch: the listed searches, sixteen per wavefront, persistent workgroups */
    const size_t lds = gprio::gprio_lds_bytes(n);
    const void *fn5 = busy ? (const void *)gprio::gprio_fast_kernel<true, 5>
                           : (const void *)gprio::gprio_fast_kernel<false, 5>;
    const void *fn8 = busy ? (const void *)gprio::gprio_fast_kernel<true, 8>
                           : (const void *)gprio::gprio_fast_kernel<false, 8>;
    const void *fn = n <= 20 ? fn5 : fn8;
    int per_cu = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, fn, 64, lds) != hipSuccess || per_cu < 1) {
      (void)hipGetLastError();
      per_cu = 1;
    }
    u32 blocks = (u32)ctx->n_cu * (u32)per_cu;
    const u32 max_tiles = (N + 15u) / 16u + fast::kListRegions;
    if (blocks > max_tiles) blocks = max_tiles;
    const dim3 grid(blocks), block(64);
#define GCAPS_GPRIO_LAUNCH(BUSY, NS)                                                                          \
  hipLaunchKernelGGL((gprio::gprio_fast_kernel<BUSY, NS>), grid, block, lds, ctx->stream, *b, (int *)d_gprio, \
                     (long long *)d_resp, d_sched, status, dl)
    if (n <= 20) {
      if (busy) GCAPS_GPRIO_LAUNCH(true, 5); else GCAPS_GPRIO_LAUNCH(false, 5);
    } else {
      if (busy) GCAPS_GPRIO_LAUNCH(true, 8); else GCAPS_GPRIO_LAUNCH(false, 8);
    }
#undef GCAPS_GPRIO_LAUNCH
    if (hipGetLastError() != hipSuccess) return GCAPS_EDEVICE;
    d_list = wl;
    d_count = status + fast::ST_WIDE_COUNT;
    items = N < 65536u ? N : 65536u;
  }
  const u32 slots = wide_slots(ctx, items);
  wide::Scratch ws;
  int rc = wide_columns(ctx, n, slots, &ws);
  if (rc != GCAPS_OK) return rc;
  hipLaunchKernelGGL(gprio::gprio_wide_kernel, dim3(slots / 256), dim3(256), 0, ctx->stream, *b, wait_mode, d_skip,
                     (int *)d_gprio, (long long *)d_resp, d_sched, status, ws, d_list, d_count, ctx->ts_offset,
                     ctx->next_status, (u32)fast::kStatusWords);
  return hipGetLastError() == hipSuccess ? GCAPS_OK : GCAPS_EDEVICE;
}

int run_gprio(gcaps_ctx *ctx, const gcaps_batch *b, int wait_mode, const uint8_t *d_skip, int32_t *d_gprio,
              int64_t *d_resp, uint8_t *d_sched) {
  const u64 n = b->n_tasks;
  return for_chunks(ctx, b, [&](const gcaps_batch *sub, u64 c0) {
    return run_gprio_chunk(ctx, sub, wait_mode, d_skip ? d_skip + c0 : nullptr, d_gprio + c0 * n, d_resp + c0 * n,
                           d_sched + c0, c0 == 0);
  });
}

/* Sec. 5.4 for given GPU priorities: the quad-lane kernel over every taskset of the chunk (up to 32 tasks), then
 * the general kernel over what it listed; other shapes: the general kernel alone */
int run_gprio_given(gcaps_ctx *ctx, const gcaps_batch *b, int wait_mode, const int32_t *d_gprio, int64_t *d_resp,
                    uint8_t *d_sched) {
  const u64 n = b->n_tasks;
  return for_chunks(ctx, b, [&](const gcaps_batch *sub, u64 c0) {
    if (begin_chunk(ctx, c0 == 0) != GCAPS_OK) return (int)GCAPS_EDEVICE;
    const u32 N = sub->n_tasksets;
    const int *gp = (const int *)(d_gprio + c0 * n);
    long long *resp = (long long *)(d_resp + c0 * n);
    u32 *status = status_of(ctx);
    const size_t lds = gprio::given_lds_bytes(sub->n_tasks);
    ctx->wide_only = sub->n_tasks > 32 || lds > (size_t)ctx->lds_limit;
    const u32 *d_list = nullptr, *d_count = nullptr;
    u32 items = N;
    if (!ctx->wide_only) {
      int rc = ctx->pool.wide_list.reserve((size_t)N * sizeof(u32), !ctx->capturing);
      if (rc != GCAPS_OK) return rc;
      const bool busy = wait_mode == GCAPS_WAIT_BUSY;
      const bool small = sub->n_tasks <= 20;
      const void *fn = small ? (busy ? (const void *)gprio::gprio_given_fast_kernel<true, 5>
                                     : (const void *)gprio::gprio_given_fast_kernel<false, 5>)
                             : (busy ? (const void *)gprio::gprio_given_fast_kernel<true, 8>
                                     : (const void *)gprio::gprio_given_fast_kernel<false, 8>);
      int per_cu = 0;
      if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, fn, 64, lds) != hipSuccess || per_cu < 1) {
        (void)hipGetLastError();
        per_cu = 1;
      }
      u32 blocks = (u32)ctx->n_cu * (u32)per_cu;
      const u32 tiles = (N + 15u) / 16u;
      if (blocks > tiles) blocks = tiles;
      const dim3 grid(blocks), block(64);
      u32 *wl = (u32 *)ctx->pool.wide_list.ptr;
#define GCAPS_GIVEN_LAUNCH(BUSY, NS)                                                                            \
  hipLaunchKernelGGL((gprio::gprio_given_fast_kernel<BUSY, NS>), grid, block, lds, ctx->stream, *sub, gp, resp, \
                     d_sched + c0, status, wl, ctx->ts_offset)
      if (small) {
        if (busy) GCAPS_GIVEN_LAUNCH(true, 5); else GCAPS_GIVEN_LAUNCH(false, 5);
      } else {
        if (busy) GCAPS_GIVEN_LAUNCH(true, 8); else GCAPS_GIVEN_LAUNCH(false, 8);
      }
#undef GCAPS_GIVEN_LAUNCH
      if (hipGetLastError() != hipSuccess) return (int)GCAPS_EDEVICE;
      d_list = wl;
      d_count = status + fast::ST_WIDE_COUNT;
      items = N < 65536u ? N : 65536u;
    }
    const u32 slots = wide_slots(ctx, items);
    wide::Scratch ws;
    int rc = wide_columns(ctx, sub->n_tasks, slots, &ws);
    if (rc != GCAPS_OK) return rc;
    hipLaunchKernelGGL(gprio::gprio_given_kernel, dim3(slots / 256), dim3(256), 0, ctx->stream, *sub, wait_mode, gp, resp,
                       d_sched + c0, status, ws, d_list, d_count, ctx->ts_offset, ctx->next_status,
                       (u32)fast::kStatusWords);
    return hipGetLastError() == hipSuccess ? (int)GCAPS_OK : (int)GCAPS_EDEVICE;
  });
}

/* Schedule simulation (Sec. 6.2: observed response times) of every taskset, one lane each */
int run_simulate(gcaps_ctx *ctx, const gcaps_batch *b, const uint32_t *d_offset, const int32_t *d_gprio, int policy,
                 int wait_mode,
                 uint32_t horizon, int64_t *d_mort, uint32_t *d_jobs, uint8_t *d_flag) {
  const u64 n = b->n_tasks, N = b->n_tasksets;
  const size_t lds = sim::lds_bytes(b->n_tasks);
  if (lds > (size_t)ctx->lds_limit) return GCAPS_EINVAL;
  const u32 planes = policy == GCAPS_POLICY_BOTH ? 2u : 1u;
  return for_chunks(ctx, b, [&](const gcaps_batch *sub, u64 c0) {
    if (begin_chunk(ctx, c0 == 0) != GCAPS_OK) return (int)GCAPS_EDEVICE;
    ctx->wide_only = true;
    /* one launch per policy plane, as many single-wavefront workgroups as are resident at once; their lanes take
     * further tasksets as they finish.  The last launch prepares the status words of the next call. */
    const bool busy = wait_mode == GCAPS_WAIT_BUSY;
    for (u32 plane = 0; plane < planes; ++plane) {
      const bool gc = (policy == GCAPS_POLICY_BOTH ? (int)plane + 1 : policy) == GCAPS_POLICY_GCAPS;
      auto fn = gc ? (busy ? sim::simulate_kernel<true, true> : sim::simulate_kernel<true, false>)
                   : (busy ? sim::simulate_kernel<false, true> : sim::simulate_kernel<false, false>);
      int per_cu = 0;
      if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, (const void *)fn, 64, lds) != hipSuccess || per_cu < 1) {
        (void)hipGetLastError();
        per_cu = 1;
      }
      u32 blocks = (u32)ctx->n_cu * (u32)per_cu;
      const u32 tiles = (sub->n_tasksets + 63u) / 64u;
      if (blocks > tiles) blocks = tiles;
      if (ctx->sim_blocks_cap && blocks > ctx->sim_blocks_cap) blocks = ctx->sim_blocks_cap;
      hipLaunchKernelGGL(fn, dim3(blocks), dim3(64), lds, ctx->stream, *sub, d_offset ? d_offset + c0 * n : nullptr,
                         d_gprio ? (const int *)(d_gprio + c0 * n) : nullptr, plane, horizon,
                         (long long *)(d_mort + c0 * n), d_jobs + c0 * n, d_flag + c0, (size_t)(N * n), (size_t)N,
                         status_of(ctx), ctx->ts_offset, plane + 1 == planes ? ctx->next_status : nullptr,
                         (u32)fast::kStatusWords);
      if (hipGetLastError() != hipSuccess) return (int)GCAPS_EDEVICE;
    }
    return (int)GCAPS_OK;
  });
}

int check_simulate(const gcaps_batch *b, int policy, int wait_mode, uint32_t horizon, const void *mort,
                   const void *jobs, const void *flag) {
  if (!b || !mort || !jobs || !flag) return GCAPS_EINVAL;
  if (b->n_tasksets == 0 || b->n_tasks == 0 || b->n_tasks > sim::kMaxTasks || b->max_gseg > 255) return GCAPS_EINVAL;
  if (!b->theta_us || !b->eps_us || !b->slice_us || !b->cpu_us || !b->period_us || !b->prio || !b->core || !b->n_gseg)
    return GCAPS_EINVAL;
  if (b->max_gseg > 0 && (!b->gm_us || !b->ge_us)) return GCAPS_EINVAL;
  if (policy < GCAPS_POLICY_GCAPS || policy > GCAPS_POLICY_BOTH) return GCAPS_EINVAL;
  if (wait_mode != GCAPS_WAIT_BUSY && wait_mode != GCAPS_WAIT_SUSPEND) return GCAPS_EINVAL;
  if (horizon == 0 || horizon > 0x80000000u) return GCAPS_EINVAL;
  return GCAPS_OK;
}

int check_gprio_batch(const gcaps_batch *b, int wait_mode, const void *gprio, const void *resp, const void *sched) {
  if (!b || !gprio || !resp || !sched) return GCAPS_EINVAL;
  if (b->n_tasksets == 0 || b->n_tasks == 0 || b->n_tasks > 255 || b->max_gseg > 255) return GCAPS_EINVAL;
  if (!b->eps_us || !b->cpu_us || !b->period_us || !b->deadline_us || !b->prio || !b->core || !b->n_gseg)
    return GCAPS_EINVAL;
  if (b->max_gseg > 0 && (!b->gm_us || !b->ge_us)) return GCAPS_EINVAL;
  if (wait_mode != GCAPS_WAIT_BUSY && wait_mode != GCAPS_WAIT_SUSPEND) return GCAPS_EINVAL;
  return GCAPS_OK;
}

/* Device copy of a host batch in the context's staging buffer (one allocation, every array
 * aligned to 256 bytes), queued on the context's stream.  skip (may be null): one more
 * per-taskset byte array, its device copy in *d_skip. */
int upload_batch(gcaps_ctx *ctx, const gcaps_batch *batch, gcaps_batch *dev, const uint8_t *skip,
                 const uint8_t **d_skip) {
  const size_t N = batch->n_tasksets, n = batch->n_tasks, S = batch->max_gseg;
  auto up = [](size_t x) { return (x + 255) / 256 * 256; };
  const size_t sz_ts = up(N * 4), sz_task4 = up(N * n * 4), sz_task1 = up(N * n), sz_seg = up(N * n * S * 4);
  const size_t in_bytes = 3 * sz_ts + 4 * sz_task4 + 2 * sz_task1 + 2 * sz_seg + up(N);
  int rc = ctx->staging_in.reserve(in_bytes);
  if (rc != GCAPS_OK) return rc;
  char *cur = (char *)ctx->staging_in.ptr;
  bool ok = true;
  auto put = [&](const void *src, size_t bytes, size_t reserved) -> const void * {
    void *dst = cur;
    cur += reserved;
    if (!src) return nullptr;
    if (bytes && hipMemcpyAsync(dst, src, bytes, hipMemcpyHostToDevice, ctx->stream) != hipSuccess) ok = false;
    return dst;
  };
  gcaps_batch d = *batch;
  d.theta_us = (const u32 *)put(batch->theta_us, N * 4, sz_ts);
  d.eps_us = (const u32 *)put(batch->eps_us, N * 4, sz_ts);
  d.slice_us = (const u32 *)put(batch->slice_us, N * 4, sz_ts);
  d.cpu_us = (const u32 *)put(batch->cpu_us, N * n * 4, sz_task4);
  d.period_us = (const u32 *)put(batch->period_us, N * n * 4, sz_task4);
  d.deadline_us = (const u32 *)put(batch->deadline_us, N * n * 4, sz_task4);
  d.prio = (const int32_t *)put(batch->prio, N * n * 4, sz_task4);
  d.core = (const uint8_t *)put(batch->core, N * n, sz_task1);
  d.n_gseg = (const uint8_t *)put(batch->n_gseg, N * n, sz_task1);
  d.n_cseg = nullptr;
  d.gm_us = S ? (const u32 *)put(batch->gm_us, N * n * S * 4, sz_seg) : nullptr;
  d.ge_us = S ? (const u32 *)put(batch->ge_us, N * n * S * 4, sz_seg) : nullptr;
  const uint8_t *ds = (const uint8_t *)put(skip, N, up(N));
  if (d_skip) *d_skip = ds;
  if (!ok) {
    (void)hipGetLastError();
    return GCAPS_EDEVICE;
  }
  *dev = d;
  return GCAPS_OK;
}

}  // namespace

extern "C" int gcaps_create(gcaps_ctx **out, int device_id, void *hip_stream) {
  if (!out) return GCAPS_EINVAL;
  *out = nullptr;
  int count = 0;
  if (hipGetDeviceCount(&count) != hipSuccess || count <= 0) {
    (void)hipGetLastError();
    return GCAPS_EDEVICE;
  }
  if (device_id < 0 || device_id >= count) return GCAPS_EINVAL;
  gcaps_ctx *ctx = new (std::nothrow) gcaps_ctx;
  if (!ctx) return GCAPS_ENOMEM;
  ctx->device = device_id;
  ctx->stream = (hipStream_t)hip_stream;
  if (const char *e = getenv("GCAPS_CHUNK_TASKSETS")) {
    const long v = strtol(e, nullptr, 10);
    if (v >= 1) ctx->chunk_cap = (u64)v;
  }
  if (const char *e = getenv("GCAPS_SIM_BLOCKS")) {
    const long v = strtol(e, nullptr, 10);
    if (v >= 1 && v <= 65535) ctx->sim_blocks_cap = (u32)v;
  }
  if (const char *e = getenv("GCAPS_SCREEN_TASKS")) {
    const long v = strtol(e, nullptr, 10);
    if (v >= 1 && v <= 255) ctx->screen_tasks = (u32)v;
  }
  if (const char *e = getenv("GCAPS_DEEP_KERNEL")) ctx->legacy_deep = e[0] == 'l';
  if (const char *e = getenv("GCAPS_GPRIO_KERNEL")) ctx->gprio_list = e[0] == 'l';
  if (const char *e = getenv("GCAPS_GEN_KERNEL")) ctx->gen_by_taskset = e[0] == 't';
  if (const char *e = getenv("GCAPS_DEEP_LANES")) {
    const long v = strtol(e, nullptr, 10);
    if (v == 4 || v == 8) ctx->deep_lanes = (u32)v;
  }
  DeviceGuard guard(device_id);
  int rc = guard.ok ? GCAPS_OK : GCAPS_EDEVICE;
  hipDeviceProp_t prop;
  if (rc == GCAPS_OK && hipGetDeviceProperties(&prop, device_id) != hipSuccess) rc = GCAPS_EDEVICE;
  if (rc == GCAPS_OK) {
    ctx->n_cu = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256;
    rc = ctx->pool.status.reserve(3 * fast::kStatusWords * sizeof(u32));
    ctx->last_status = (u32 *)ctx->pool.status.ptr;
  }
  if (rc == GCAPS_OK) {
    /* the static scratch of this device, cut into the buffers of a pool */
    static_assert(kStaticStatusBytes >= 3 * fast::kStatusWords * sizeof(u32), "status blocks");
    char *base = (char *)scratch_on_device(device_id);
    if (!base) rc = GCAPS_EDEVICE;
    auto slice = [&](DeviceBuffer &buf, size_t bytes) {
      buf.ptr = base;
      buf.bytes = bytes;
      buf.fixed = true;
      base += bytes;
    };
    if (rc == GCAPS_OK) {
      Pool &sp = ctx->static_pool;
      slice(sp.status, kStaticStatusBytes);
      slice(sp.wide_list, kStaticListBytes);
      slice(sp.deep_sorted, kStaticListBytes);
      slice(sp.deep_list, kStaticDeepBytes);
      slice(sp.deep_aux, 2 * kStaticDeepBytes);
      slice(sp.wide_scratch, kStaticColumnBytes);
    }
  }
  if (rc == GCAPS_OK) {
    /* the fast kernel's tiles live in dynamic LDS: raise the per-workgroup limit to what the CU has */
    size_t want = prop.sharedMemPerBlock;
    if (prop.maxSharedMemoryPerMultiProcessor > want) want = prop.maxSharedMemoryPerMultiProcessor;
    if (want > 160u * 1024u) want = 160u * 1024u;
    const void *kernels[] = {
        (const void *)fast::rta_fast_kernel<64, 0>,  (const void *)fast::rta_fast_kernel<64, 4>,
        (const void *)fast::rta_fast_kernel<64, 8>,  (const void *)fast::rta_fast_kernel<64, 16>,
        (const void *)fast::rta_fast_kernel<64, 24>, (const void *)fast::rta_fast_kernel<64, 32>,
        (const void *)fast::rta_fast_kernel<32, 0>,  (const void *)fast::rta_fast_kernel<16, 0>,
        (const void *)fast::rta_screen_kernel<true>, (const void *)fast::rta_screen_kernel<false>,
        (const void *)fast::rta_deep_kernel<true, 4, false>, (const void *)fast::rta_deep_kernel<false, 4, false>,
        (const void *)fast::rta_deep_kernel<true, 8, false>, (const void *)fast::rta_deep_kernel<false, 8, false>,
        (const void *)fast::rta_deep_kernel<true, 4, true>, (const void *)fast::rta_deep_kernel<false, 4, true>,
        (const void *)fast::rta_deep_kernel<true, 8, true>, (const void *)fast::rta_deep_kernel<false, 8, true>,
#define GCAPS_QUAD_KERNELS(NS)                                                                                        \
  (const void *)fast::rta_quad_kernel<true, NS, 3>, (const void *)fast::rta_quad_kernel<false, NS, 3>,                \
      (const void *)fast::rta_quad_kernel<true, NS, 4>, (const void *)fast::rta_quad_kernel<false, NS, 4>,            \
      (const void *)fast::rta_quad_kernel<true, NS, fast::kPrefetchSegs>,                                             \
      (const void *)fast::rta_quad_kernel<false, NS, fast::kPrefetchSegs>,                                            \
      (const void *)fast::rta_quad_kernel<true, NS, 0>, (const void *)fast::rta_quad_kernel<false, NS, 0>
        GCAPS_QUAD_KERNELS(5), GCAPS_QUAD_KERNELS(6), GCAPS_QUAD_KERNELS(8)};
#undef GCAPS_QUAD_KERNELS
    bool raised = want > 65536;
    for (size_t k = 0; k < sizeof(kernels) / sizeof(kernels[0]) && raised; ++k)
      raised = hipFuncSetAttribute(kernels[k], hipFuncAttributeMaxDynamicSharedMemorySize, (int)want) == hipSuccess;
    (void)hipGetLastError();
    ctx->lds_limit = raised ? (int)want : 65536;
    ctx->lds_total = want > 65536 ? want : 65536;
  }
  if (rc == GCAPS_OK && hipHostMalloc((void **)&ctx->host_status, 8 * sizeof(u32), hipHostMallocDefault) != hipSuccess)
    rc = GCAPS_ENOMEM;
  if (rc != GCAPS_OK) {
    (void)hipGetLastError();
    ctx->pool.release();
    delete ctx;
    return rc;
  }
  *out = ctx;
  return GCAPS_OK;
}

extern "C" void gcaps_destroy(gcaps_ctx *ctx) {
  if (!ctx) return;
  DeviceGuard guard(ctx->device);
  (void)hipStreamSynchronize(ctx->stream);
  ctx->pool.release();
  ctx->staging_in.release();
  ctx->staging_out.release();
  if (ctx->host_status) (void)hipHostFree(ctx->host_status);
  delete ctx;
}

extern "C" int gcaps_set_binning(gcaps_ctx *ctx, int enable) {
  if (!ctx || (enable != 0 && enable != 1)) return GCAPS_EINVAL;
  ctx->binning = enable;
  return GCAPS_OK;
}

extern "C" int gcaps_set_continue_after_miss(gcaps_ctx *ctx, int enable) {
  if (!ctx || (enable != 0 && enable != 1)) return GCAPS_EINVAL;
  ctx->cont = enable;
  return GCAPS_OK;
}

extern "C" int gcaps_rta_batch_device(gcaps_ctx *ctx, const gcaps_batch *batch, int policy, int wait_mode,
                                      int64_t *d_out_resp, uint8_t *d_out_sched) {
  if (!ctx) return GCAPS_EINVAL;
  int rc = check_batch(batch, policy, wait_mode, d_out_resp, d_out_sched);
  if (rc != GCAPS_OK) return rc;
  DeviceGuard guard(ctx->device);
  if (!guard.ok) return GCAPS_EDEVICE;
  return run_device(ctx, batch, policy, wait_mode, d_out_resp, d_out_sched);
}

extern "C" int gcaps_rta_batch_device_static(gcaps_ctx *ctx, const gcaps_batch *batch, int policy, int wait_mode,
                                             int64_t *d_out_resp, uint8_t *d_out_sched) {
  if (!ctx) return GCAPS_EINVAL;
  int rc = check_batch(batch, policy, wait_mode, d_out_resp, d_out_sched);
  if (rc != GCAPS_OK) return rc;
  if (batch->n_tasksets > kStaticMaxTasksets || batch->n_tasks > kStaticMaxTasks) return GCAPS_ESIZE;
  DeviceGuard guard(ctx->device);
  if (!guard.ok) return GCAPS_EDEVICE;
  /* the launches of gcaps_rta_batch_device with the fixed slices of the static array in place of the
   * context's own buffers: every reserve() is then a size check */
  std::swap(ctx->pool, ctx->static_pool);
  ctx->static_call = true;
  rc = run_device(ctx, batch, policy, wait_mode, d_out_resp, d_out_sched);
  ctx->static_call = false;
  std::swap(ctx->pool, ctx->static_pool);
  return rc;
}

extern "C" int gcaps_status(gcaps_ctx *ctx, uint32_t *first_bad_taskset) {
  if (!ctx) return GCAPS_EINVAL;
  DeviceGuard guard(ctx->device);
  if (!guard.ok) return GCAPS_EDEVICE;
  if (hipMemcpyAsync(ctx->host_status, ctx->last_status, sizeof(u32), hipMemcpyDeviceToHost, ctx->stream) !=
          hipSuccess ||
      hipStreamSynchronize(ctx->stream) != hipSuccess) {
    (void)hipGetLastError();
    return GCAPS_EDEVICE;
  }
  if (*ctx->host_status != 0xffffffffu) {
    if (first_bad_taskset) *first_bad_taskset = *ctx->host_status;
    return GCAPS_ETASK;
  }
  return GCAPS_OK;
}

extern "C" int gcaps_last_wide_count(gcaps_ctx *ctx, uint32_t *count) {
  if (!ctx || !count) return GCAPS_EINVAL;
  DeviceGuard guard(ctx->device);
  if (!guard.ok) return GCAPS_EDEVICE;
  if (hipMemcpyAsync(ctx->host_status, ctx->last_status, 4 * sizeof(u32), hipMemcpyDeviceToHost, ctx->stream) !=
          hipSuccess ||
      hipStreamSynchronize(ctx->stream) != hipSuccess) {
    (void)hipGetLastError();
    return GCAPS_EDEVICE;
  }
  *count = ctx->wide_only ? ctx->last_n_tasksets : ctx->host_status[1] + ctx->host_status[3];
  return GCAPS_OK;
}

extern "C" int gcaps_rta_batch(gcaps_ctx *ctx, const gcaps_batch *batch, int policy, int wait_mode,
                               int64_t *out_resp, uint8_t *out_sched, uint32_t *first_bad_taskset) {
  if (!ctx) return GCAPS_EINVAL;
  int rc = check_batch(batch, policy, wait_mode, out_resp, out_sched);
  if (rc != GCAPS_OK) return rc;
  DeviceGuard guard(ctx->device);
  if (!guard.ok) return GCAPS_EDEVICE;

  const size_t N = batch->n_tasksets, n = batch->n_tasks;
  const size_t P = (size_t)npol(policy);
  auto up = [](size_t x) { return (x + 255) / 256 * 256; };
  const size_t resp_bytes = up(P * N * n * 8), sched_bytes = up(P * N);
  gcaps_batch d;
  rc = upload_batch(ctx, batch, &d, nullptr, nullptr);
  if (rc == GCAPS_OK) rc = ctx->staging_out.reserve(resp_bytes + sched_bytes);
  if (rc != GCAPS_OK) return rc;
  int64_t *d_resp = (int64_t *)ctx->staging_out.ptr;
  uint8_t *d_sched = (uint8_t *)ctx->staging_out.ptr + resp_bytes;
  rc = run_device(ctx, &d, policy, wait_mode, d_resp, d_sched);
  if (rc != GCAPS_OK) return rc;
  rc = gcaps_status(ctx, first_bad_taskset);
  if (rc != GCAPS_OK) return rc;
  if (hipMemcpyAsync(out_resp, d_resp, P * N * n * 8, hipMemcpyDeviceToHost, ctx->stream) != hipSuccess ||
      hipMemcpyAsync(out_sched, d_sched, P * N, hipMemcpyDeviceToHost, ctx->stream) != hipSuccess ||
      hipStreamSynchronize(ctx->stream) != hipSuccess) {
    (void)hipGetLastError();
    return GCAPS_EDEVICE;
  }
  return GCAPS_OK;
}

extern "C" int gcaps_gprio_assign_batch_device(gcaps_ctx *ctx, const gcaps_batch *batch, int wait_mode,
                                               const uint8_t *d_skip, int32_t *d_out_gprio, int64_t *d_out_resp,
                                               uint8_t *d_out_sched) {
  if (!ctx) return GCAPS_EINVAL;
  int rc = check_gprio_batch(batch, wait_mode, d_out_gprio, d_out_resp, d_out_sched);
  if (rc != GCAPS_OK) return rc;
  DeviceGuard guard(ctx->device);
  if (!guard.ok) return GCAPS_EDEVICE;
  return run_gprio(ctx, batch, wait_mode, d_skip, d_out_gprio, d_out_resp, d_out_sched);
}

extern "C" int gcaps_gprio_assign_batch(gcaps_ctx *ctx, const gcaps_batch *batch, int wait_mode,
                                        const uint8_t *skip, int32_t *out_gprio, int64_t *out_resp,
                                        uint8_t *out_sched, uint32_t *first_bad_taskset) {
  if (!ctx) return GCAPS_EINVAL;
  int rc = check_gprio_batch(batch, wait_mode, out_gprio, out_resp, out_sched);
  if (rc != GCAPS_OK) return rc;
  DeviceGuard guard(ctx->device);
  if (!guard.ok) return GCAPS_EDEVICE;
  const size_t N = batch->n_tasksets, n = batch->n_tasks;
  auto up = [](size_t x) { return (x + 255) / 256 * 256; };
  const size_t resp_bytes = up(N * n * 8), gprio_bytes = up(N * n * 4), sched_bytes = up(N);
  gcaps_batch d;
  const uint8_t *d_skip = nullptr;
  rc = upload_batch(ctx, batch, &d, skip, &d_skip);
  if (rc == GCAPS_OK) rc = ctx->staging_out.reserve(resp_bytes + gprio_bytes + sched_bytes);
  if (rc != GCAPS_OK) return rc;
  int64_t *d_resp = (int64_t *)ctx->staging_out.ptr;
  int32_t *d_gprio = (int32_t *)((char *)ctx->staging_out.ptr + resp_bytes);
  uint8_t *d_sched = (uint8_t *)ctx->staging_out.ptr + resp_bytes + gprio_bytes;
  rc = run_gprio(ctx, &d, wait_mode, d_skip, d_gprio, d_resp, d_sched);
  if (rc != GCAPS_OK) return rc;
  rc = gcaps_status(ctx, first_bad_taskset);
  if (rc != GCAPS_OK) return rc;
  if (hipMemcpyAsync(out_resp, d_resp, N * n * 8, hipMemcpyDeviceToHost, ctx->stream) != hipSuccess ||
      hipMemcpyAsync(out_gprio, d_gprio, N * n * 4, hipMemcpyDeviceToHost, ctx->stream) != hipSuccess ||
      hipMemcpyAsync(out_sched, d_sched, N, hipMemcpyDeviceToHost, ctx->stream) != hipSuccess ||
      hipStreamSynchronize(ctx->stream) != hipSuccess) {
    (void)hipGetLastError();
    return GCAPS_EDEVICE;
  }
  return GCAPS_OK;
}

extern "C" int gcaps_gprio_rta_batch_device(gcaps_ctx *ctx, const gcaps_batch *batch, int wait_mode,
                                            const int32_t *d_gprio, int64_t *d_out_resp, uint8_t *d_out_sched) {
  if (!ctx) return GCAPS_EINVAL;
  int rc = check_gprio_batch(batch, wait_mode, d_gprio, d_out_resp, d_out_sched);
  if (rc != GCAPS_OK) return rc;
  DeviceGuard guard(ctx->device);
  if (!guard.ok) return GCAPS_EDEVICE;
  return run_gprio_given(ctx, batch, wait_mode, d_gprio, d_out_resp, d_out_sched);
}

extern "C" int gcaps_gprio_rta_batch(gcaps_ctx *ctx, const gcaps_batch *batch, int wait_mode, const int32_t *gprio,
                                     int64_t *out_resp, uint8_t *out_sched, uint32_t *first_bad_taskset) {
  if (!ctx) return GCAPS_EINVAL;
  int rc = check_gprio_batch(batch, wait_mode, gprio, out_resp, out_sched);
  if (rc != GCAPS_OK) return rc;
  DeviceGuard guard(ctx->device);
  if (!guard.ok) return GCAPS_EDEVICE;
  const size_t N = batch->n_tasksets, n = batch->n_tasks;
  auto up = [](size_t x) { return (x + 255) / 256 * 256; };
  const size_t resp_bytes = up(N * n * 8), gprio_bytes = up(N * n * 4), sched_bytes = up(N);
  gcaps_batch d;
  rc = upload_batch(ctx, batch, &d, nullptr, nullptr);
  if (rc == GCAPS_OK) rc = ctx->staging_out.reserve(resp_bytes + gprio_bytes + sched_bytes);
  if (rc != GCAPS_OK) return rc;
  int64_t *d_resp = (int64_t *)ctx->staging_out.ptr;
  int32_t *d_gprio = (int32_t *)((char *)ctx->staging_out.ptr + resp_bytes);
  uint8_t *d_sched = (uint8_t *)ctx->staging_out.ptr + resp_bytes + gprio_bytes;
  if (hipMemcpyAsync(d_gprio, gprio, N * n * 4, hipMemcpyHostToDevice, ctx->stream) != hipSuccess) {
    (void)hipGetLastError();
    return GCAPS_EDEVICE;
  }
  rc = run_gprio_given(ctx, &d, wait_mode, d_gprio, d_resp, d_sched);
  if (rc != GCAPS_OK) return rc;
  rc = gcaps_status(ctx, first_bad_taskset);
  if (rc != GCAPS_OK) return rc;
  if (hipMemcpyAsync(out_resp, d_resp, N * n * 8, hipMemcpyDeviceToHost, ctx->stream) != hipSuccess ||
      hipMemcpyAsync(out_sched, d_sched, N, hipMemcpyDeviceToHost, ctx->stream) != hipSuccess ||
      hipStreamSynchronize(ctx->stream) != hipSuccess) {
    (void)hipGetLastError();
    return GCAPS_EDEVICE;
  }
  return GCAPS_OK;
}

extern "C" int gcaps_simulate_batch_device(gcaps_ctx *ctx, const gcaps_batch *batch, const uint32_t *d_offset,
                                           const int32_t *d_gprio, int policy, int wait_mode, uint32_t horizon, int64_t *d_out_mort,
                                           uint32_t *d_out_jobs, uint8_t *d_out_flag) {
  if (!ctx) return GCAPS_EINVAL;
  int rc = check_simulate(batch, policy, wait_mode, horizon, d_out_mort, d_out_jobs, d_out_flag);
  if (rc != GCAPS_OK) return rc;
  DeviceGuard guard(ctx->device);
  if (!guard.ok) return GCAPS_EDEVICE;
  return run_simulate(ctx, batch, d_offset, d_gprio, policy, wait_mode, horizon, d_out_mort, d_out_jobs, d_out_flag);
}

extern "C" int gcaps_simulate_batch(gcaps_ctx *ctx, const gcaps_batch *batch, const uint32_t *offset,
                                    const int32_t *gprio, int policy,
                                    int wait_mode, uint32_t horizon, int64_t *out_mort, uint32_t *out_jobs,
                                    uint8_t *out_flag, uint32_t *first_bad_taskset) {
  if (!ctx) return GCAPS_EINVAL;
  int rc = check_simulate(batch, policy, wait_mode, horizon, out_mort, out_jobs, out_flag);
  if (rc != GCAPS_OK) return rc;
  DeviceGuard guard(ctx->device);
  if (!guard.ok) return GCAPS_EDEVICE;
  const size_t N = batch->n_tasksets, n = batch->n_tasks, P = policy == GCAPS_POLICY_BOTH ? 2 : 1;
  auto up = [](size_t x) { return (x + 255) / 256 * 256; };
  const size_t mort_bytes = up(P * N * n * 8), jobs_bytes = up(P * N * n * 4), flag_bytes = up(P * N),
               off_bytes = up(N * n * 4);
  gcaps_batch d;
  rc = upload_batch(ctx, batch, &d, nullptr, nullptr);
  if (rc == GCAPS_OK) rc = ctx->staging_out.reserve(mort_bytes + jobs_bytes + flag_bytes + 2 * off_bytes);
  if (rc != GCAPS_OK) return rc;
  char *base = (char *)ctx->staging_out.ptr;
  int64_t *d_mort = (int64_t *)base;
  uint32_t *d_jobs = (uint32_t *)(base + mort_bytes);
  uint8_t *d_flag = (uint8_t *)(base + mort_bytes + jobs_bytes);
  uint32_t *d_off = offset ? (uint32_t *)(base + mort_bytes + jobs_bytes + flag_bytes) : nullptr;
  if (offset && hipMemcpyAsync(d_off, offset, N * n * 4, hipMemcpyHostToDevice, ctx->stream) != hipSuccess) {
    (void)hipGetLastError();
    return GCAPS_EDEVICE;
  }
  int32_t *d_gprio = gprio ? (int32_t *)(base + mort_bytes + jobs_bytes + flag_bytes + off_bytes) : nullptr;
  if (gprio && hipMemcpyAsync(d_gprio, gprio, N * n * 4, hipMemcpyHostToDevice, ctx->stream) != hipSuccess) {
    (void)hipGetLastError();
    return GCAPS_EDEVICE;
  }
  rc = run_simulate(ctx, &d, d_off, d_gprio, policy, wait_mode, horizon, d_mort, d_jobs, d_flag);
  if (rc != GCAPS_OK) return rc;
  rc = gcaps_status(ctx, first_bad_taskset);
  if (rc != GCAPS_OK) return rc;
  if (hipMemcpyAsync(out_mort, d_mort, P * N * n * 8, hipMemcpyDeviceToHost, ctx->stream) != hipSuccess ||
      hipMemcpyAsync(out_jobs, d_jobs, P * N * n * 4, hipMemcpyDeviceToHost, ctx->stream) != hipSuccess ||
      hipMemcpyAsync(out_flag, d_flag, P * N, hipMemcpyDeviceToHost, ctx->stream) != hipSuccess ||
      hipStreamSynchronize(ctx->stream) != hipSuccess) {
    (void)hipGetLastError();
    return GCAPS_EDEVICE;
  }
  return GCAPS_OK;
}

extern "C" int gcaps_taskgen_device(gcaps_ctx *ctx, const gcaps_taskgen_spec *sp, const gcaps_batch *b) {
  if (!ctx || !sp || !b) return GCAPS_EINVAL;
  if (b->n_tasksets == 0 || b->n_tasks == 0 || b->n_tasks > 255 || b->max_gseg > 255) return GCAPS_EINVAL;
  if (!b->theta_us || !b->eps_us || !b->slice_us || !b->cpu_us || !b->period_us || !b->deadline_us || !b->prio ||
      !b->core || !b->n_gseg || (b->max_gseg > 0 && (!b->gm_us || !b->ge_us)))
    return GCAPS_EINVAL;
  if (sp->n_cores == 0 || sp->n_cores > 255 || sp->tasks_per_core == 0 ||
      (uint64_t)sp->n_cores * sp->tasks_per_core != b->n_tasks || sp->eta_lo > sp->eta_hi ||
      sp->eta_hi > b->max_gseg || sp->period_lo == 0 || sp->period_lo > sp->period_hi ||
      sp->overhead_lo > sp->overhead_hi || !(sp->util_lo <= sp->util_hi) || !(sp->share_lo <= sp->share_hi) ||
      (!sp->slice_fixed && sp->slice_us == 0))
    return GCAPS_EINVAL;
  DeviceGuard guard(ctx->device);
  if (!guard.ok) return GCAPS_EDEVICE;
  /* one lane per task where three words per task of 16 tasksets fit LDS and element indices fit 32 bits */
  if (!ctx->gen_by_taskset && gen::element_lds_bytes(b->n_tasks) <= (size_t)ctx->lds_limit &&
      (uint64_t)b->n_tasksets * b->n_tasks * (b->max_gseg ? b->max_gseg : 1u) < (1ull << 32)) {
    hipLaunchKernelGGL(gen::generate_element_kernel, dim3((b->n_tasksets + 15u) / 16u), dim3(64),
                       gen::element_lds_bytes(b->n_tasks), ctx->stream, *b, *sp);
    return hipGetLastError() == hipSuccess ? GCAPS_OK : GCAPS_EDEVICE;
  }
  /* one lane per taskset: stores gathered through LDS where a taskset's per-task values fit; else the plain kernel */
  const u32 S = b->max_gseg;
  u32 tb = S ? 16u / S : 1u;
  if (tb < 1u) tb = 1u;
  if (tb > b->n_tasks) tb = b->n_tasks;
  const size_t staged = gen::staged_lds_bytes(b->n_tasks, S, tb);
  const dim3 grid((b->n_tasksets + 63u) / 64u), block(64);
  if (staged <= (size_t)ctx->lds_limit)
    hipLaunchKernelGGL(gen::generate_staged_kernel, grid, block, staged, ctx->stream, *b, *sp, tb);
  else
    hipLaunchKernelGGL(gen::generate_kernel, grid, block, (size_t)b->n_tasks * 64 * sizeof(u32), ctx->stream, *b, *sp,
                       (u32 *)nullptr, 0u);
  return hipGetLastError() == hipSuccess ? GCAPS_OK : GCAPS_EDEVICE;
}

namespace {
int check_table3(const gcaps_table3_spec *sp) {
  if (!sp) return GCAPS_EINVAL;
  if (sp->n_cpus == 0 || sp->n_cpus > 8 || sp->per_cpu_lo == 0 || sp->per_cpu_lo > sp->per_cpu_hi ||
      (uint64_t)sp->n_cpus * sp->per_cpu_hi > 255 || sp->eta_lo == 0 || sp->eta_lo > sp->eta_hi || sp->eta_hi > 255 ||
      sp->period_lo == 0 || sp->period_lo > sp->period_hi || !(sp->util_lo > 0.0) || !(sp->util_lo <= sp->util_hi) ||
      !(sp->gpu_ratio_lo >= 0.0) || !(sp->gpu_ratio_lo <= sp->gpu_ratio_hi) || !(sp->gpu_ratio_hi <= 1.0) ||
      !(sp->gc_lo >= 0.0) || !(sp->gc_lo <= sp->gc_hi) || !(sp->gm_lo >= 0.0) || !(sp->gm_lo <= sp->gm_hi) ||
      !(sp->gm_hi <= 1.0) || sp->slice_us == 0)
    return GCAPS_EINVAL;
  return GCAPS_OK;
}
}  // namespace

extern "C" int gcaps_table3_count_device(gcaps_ctx *ctx, const gcaps_table3_spec *sp, uint32_t n_tasksets,
                                         uint32_t *d_n_tasks) {
  if (!ctx || !d_n_tasks || n_tasksets == 0) return GCAPS_EINVAL;
  int rc = check_table3(sp);
  if (rc != GCAPS_OK) return rc;
  DeviceGuard guard(ctx->device);
  if (!guard.ok) return GCAPS_EDEVICE;
  rc = begin_single_call(ctx); /* gcaps_status then reports on this call (nothing to report: it waits) */
  if (rc != GCAPS_OK) return rc;
  hipLaunchKernelGGL(gen::table3_count_kernel, dim3((n_tasksets + 63u) / 64u), dim3(64), 0, ctx->stream, *sp, n_tasksets,
                     d_n_tasks);
  return hipGetLastError() == hipSuccess ? GCAPS_OK : GCAPS_EDEVICE;
}

extern "C" int gcaps_table3_generate_device(gcaps_ctx *ctx, const gcaps_table3_spec *sp, const uint32_t *d_index,
                                            const gcaps_batch *b) {
  if (!ctx || !b) return GCAPS_EINVAL;
  int rc = check_table3(sp);
  if (rc != GCAPS_OK) return rc;
  if (b->n_tasksets == 0 || b->n_tasks < sp->n_cpus * sp->per_cpu_lo || b->n_tasks > sp->n_cpus * sp->per_cpu_hi ||
      b->max_gseg < sp->eta_hi || b->max_gseg > 255)
    return GCAPS_EINVAL;
  if (!b->theta_us || !b->eps_us || !b->slice_us || !b->cpu_us || !b->period_us || !b->deadline_us || !b->prio ||
      !b->core || !b->n_gseg || !b->gm_us || !b->ge_us)
    return GCAPS_EINVAL;
  const size_t lds = gen::table3_lds_bytes(b->n_tasks);
  if (lds > 65536) return GCAPS_EINVAL; /* 64 tasks */
  DeviceGuard guard(ctx->device);
  if (!guard.ok) return GCAPS_EDEVICE;
  /* a generator call stands alone: it reports through the status block of a call of its own */
  rc = begin_single_call(ctx);
  if (rc != GCAPS_OK) return rc;
  hipLaunchKernelGGL(gen::table3_generate_kernel, dim3((b->n_tasksets + 63u) / 64u), dim3(64), lds, ctx->stream, *b, *sp,
                     d_index, status_of(ctx) + fast::ST_FIRST_BAD);
  return hipGetLastError() == hipSuccess ? GCAPS_OK : GCAPS_EDEVICE;
}

extern "C" int gcaps_last_sim_steps(gcaps_ctx *ctx, uint64_t *steps) {
  if (!ctx || !steps) return GCAPS_EINVAL;
  DeviceGuard guard(ctx->device);
  if (!guard.ok) return GCAPS_EDEVICE;
  if (hipMemcpyAsync(ctx->host_status, ctx->last_status, 8 * sizeof(u32), hipMemcpyDeviceToHost, ctx->stream) !=
          hipSuccess ||
      hipStreamSynchronize(ctx->stream) != hipSuccess) {
    (void)hipGetLastError();
    return GCAPS_EDEVICE;
  }
  *steps = (uint64_t)ctx->host_status[sim::kStatusSteps] | (uint64_t)ctx->host_status[sim::kStatusSteps + 1] << 32;
  return GCAPS_OK;
}

extern "C" int gcaps_valu_probe(gcaps_ctx *ctx, gcaps_valu_rates *out) {
  if (!ctx || !out) return GCAPS_EINVAL;
  DeviceGuard guard(ctx->device);
  if (!guard.ok) return GCAPS_EDEVICE;
  hipDeviceProp_t prop;
  if (hipGetDeviceProperties(&prop, ctx->device) != hipSuccess) return GCAPS_EDEVICE;
  out->cu_count = prop.multiProcessorCount;
  out->clock_khz = prop.clockRate;
  out->wavefront_size = prop.warpSize;
  out->simd_per_cu = 4; /* CDNA: four SIMDs of 16 lanes per compute unit */
  out->spec_lane_ops_per_s = (double)out->cu_count * out->simd_per_cu * 16.0 * (double)out->clock_khz * 1e3;
  const u32 blocks = (u32)ctx->n_cu * 8u; /* 256 threads each: eight wavefronts per SIMD */
  DeviceBuffer sink;
  int rc = sink.reserve((size_t)blocks * sizeof(u32));
  if (rc != GCAPS_OK) return rc;
  hipEvent_t e0 = nullptr, e1 = nullptr;
  bool ok = hipEventCreate(&e0) == hipSuccess && hipEventCreate(&e1) == hipSuccess;
  for (int kind = 0; kind < GCAPS_PROBE_KINDS && ok; ++kind) {
    double best_ms = 0.0;
    for (int rep = 0; rep < 4 && ok; ++rep) { /* the first repetition warms up; the fastest of the rest counts */
      ok = hipEventRecord(e0, ctx->stream) == hipSuccess &&
           probe::launch_kind(kind, ctx->stream, blocks, (u32 *)sink.ptr) == hipSuccess &&
           hipEventRecord(e1, ctx->stream) == hipSuccess && hipEventSynchronize(e1) == hipSuccess;
      float ms = 0.0f;
      ok = ok && hipEventElapsedTime(&ms, e0, e1) == hipSuccess;
      if (ok && rep > 0 && (best_ms == 0.0 || ms < best_ms)) best_ms = ms;
    }
    out->lane_ops_per_s[kind] = best_ms > 0.0 ? probe::lane_ops(kind, blocks) / (best_ms * 1e-3) : 0.0;
  }
  if (e0) (void)hipEventDestroy(e0);
  if (e1) (void)hipEventDestroy(e1);
  sink.release();
  if (!ok) {
    (void)hipGetLastError();
    return GCAPS_EDEVICE;
  }
  return GCAPS_OK;
}

extern "C" int gcaps_hbm_probe(gcaps_ctx *ctx, size_t bytes, gcaps_hbm_rates *out) {
  if (!ctx || !out || bytes < (1u << 20) || bytes % 16 != 0) return GCAPS_EINVAL;
  DeviceGuard guard(ctx->device);
  if (!guard.ok) return GCAPS_EDEVICE;
  DeviceBuffer src, dst, sink;
  int rc = src.reserve(bytes);
  if (rc == GCAPS_OK) rc = dst.reserve(bytes);
  if (rc == GCAPS_OK) rc = sink.reserve(256);
  if (rc != GCAPS_OK) {
    src.release();
    dst.release();
    sink.release();
    return rc;
  }
  out->bytes = bytes;
  /* one workgroup per 256 * kUnroll accesses (the kernels stride by the grid where that exceeds 2^20 workgroups) */
  const size_t per_block = (size_t)256 * hbm::kUnroll * 16;
  const u32 blocks = (u32)std::min<size_t>((bytes + per_block - 1) / per_block, (size_t)1 << 20);
  hipEvent_t e0 = nullptr, e1 = nullptr;
  bool ok = hipEventCreate(&e0) == hipSuccess && hipEventCreate(&e1) == hipSuccess;
  /* the source holds defined values before anything reads it */
  ok = ok && hbm::launch_kind(GCAPS_HBM_WRITE, ctx->stream, blocks, nullptr, src.ptr, bytes, (u32 *)sink.ptr) == hipSuccess;
  for (int kind = 0; kind < GCAPS_HBM_KINDS && ok; ++kind) {
    double best_ms = 0.0;
    for (int rep = 0; rep < 4 && ok; ++rep) { /* the first repetition warms up; the fastest of the rest counts */
      ok = hipEventRecord(e0, ctx->stream) == hipSuccess &&
           hbm::launch_kind(kind, ctx->stream, blocks, src.ptr, dst.ptr, bytes, (u32 *)sink.ptr) == hipSuccess &&
           hipEventRecord(e1, ctx->stream) == hipSuccess && hipEventSynchronize(e1) == hipSuccess;
      float ms = 0.0f;
      ok = ok && hipEventElapsedTime(&ms, e0, e1) == hipSuccess;
      if (ok && rep > 0 && (best_ms == 0.0 || ms < best_ms)) best_ms = ms;
    }
    out->bytes_per_s[kind] = best_ms > 0.0 ? hbm::bytes_moved(kind, bytes) / (best_ms * 1e-3) : 0.0;
  }
  if (e0) (void)hipEventDestroy(e0);
  if (e1) (void)hipEventDestroy(e1);
  if (hipStreamSynchronize(ctx->stream) != hipSuccess) ok = false;
  src.release();
  dst.release();
  sink.release();
  if (!ok) {
    (void)hipGetLastError();
    return GCAPS_EDEVICE;
  }
  return GCAPS_OK;
}

extern "C" const char *gcaps_strerror(int code) {
  switch (code) {
    case GCAPS_OK: return "success";
    case GCAPS_EINVAL: return "invalid argument (null pointer, size out of range or unknown selector)";
    case GCAPS_ETASK:
      return "a taskset violates the task model (T = 0, D = 0, D > T, L = 0, eta^g > S, or GPU priorities that "
             "disagree with the CPU priorities on a core)";
    case GCAPS_ENOMEM: return "host or device allocation failed";
    case GCAPS_EDEVICE: return "a HIP runtime call failed";
    case GCAPS_ESIZE:
      return "the call needs more device scratch than it may take (a recorded call larger than every direct call "
             "before it, or a batch beyond the limits of gcaps_rta_batch_device_static)";
    default: return "unknown gcaps error code";
  }
}
