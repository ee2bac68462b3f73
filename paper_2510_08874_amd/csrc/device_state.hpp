// Host-side device resources of the library (included by exec.hip): error bookkeeping, the
// slab and scratch pools, the work-table uploader and the per-plan device state.
#pragma once

#include <hip/hip_runtime.h>

#include <cstring>
#include <mutex>
#include <new>
#include <vector>

#include "dmm.h"

namespace dmm {

// ------------------------------------------------------------------ host state

thread_local int g_last_hip_error = 0;

#define DMM_HIP(call)                            \
  do {                                           \
    hipError_t e_ = (call);                      \
    if (e_ != hipSuccess) {                      \
      g_last_hip_error = (int)e_;                \
      return DMM_EHIP;                           \
    }                                            \
  } while (0)

// One device buffer plus two pinned staging slots and their events.  Slabs are
// recycled through a process-wide pool (in the spirit of the memory pool of
// Section 4.2: allocate once, sub-allocate from the CPU side), so creating and
// destroying plans in a loop does not hit hipMalloc / hipHostMalloc each time.
struct Slab {
  int device = -1;       // the device its buffer and events belong to
  char *dev = nullptr;
  char *pinned[2] = {nullptr, nullptr};
  hipEvent_t ev[2] = {nullptr, nullptr};
  size_t cap = 0;
  // Host copy of what the device buffer holds (empty: unknown).  It stays with the slab through
  // the pool, so a new plan whose tables equal those of a destroyed one (plan + execute in a
  // loop over the same buffers) finds them already on the device and uploads nothing.
  std::vector<char> *mirror = nullptr;
};

class SlabPool {
 public:
  int acquire(size_t bytes, Slab *out) {
    int device = 0;
    DMM_HIP(hipGetDevice(&device));
    {
      std::lock_guard<std::mutex> g(mu_);
      int best = -1;
      for (size_t i = 0; i < free_.size(); ++i)
        if (free_[i].device == device && free_[i].cap >= bytes &&
            (best < 0 || free_[i].cap < free_[(size_t)best].cap))
          best = (int)i;
      if (best >= 0) {
        *out = free_[(size_t)best];
        free_.erase(free_.begin() + best);
        return DMM_OK;
      }
    }
    size_t want = 64 * 1024;
    while (want < bytes) want *= 2;
    Slab s;
    hipError_t e = hipMalloc((void **)&s.dev, want);
    for (int i = 0; i < 2 && e == hipSuccess; ++i) {
      e = hipHostMalloc((void **)&s.pinned[i], want, hipHostMallocDefault);
      if (e == hipSuccess) e = hipEventCreateWithFlags(&s.ev[i], hipEventDisableTiming);
    }
    if (e != hipSuccess) {
      destroy(&s);
      g_last_hip_error = (int)e;
      return e == hipErrorOutOfMemory ? DMM_ENOMEM : DMM_EHIP;
    }
    s.cap = want;
    s.device = device;
    s.mirror = new (std::nothrow) std::vector<char>;
    if (!s.mirror) {
      destroy(&s);
      return DMM_ENOMEM;
    }
    *out = s;
    return DMM_OK;
  }
  // The caller guarantees that no stream work still uses the slab.
  void release(Slab *s) {
    if (!s->dev) return;
    std::lock_guard<std::mutex> g(mu_);
    if (free_.size() < 16) free_.push_back(*s);
    else destroy(s);
    *s = Slab();
  }

 private:
  static void destroy(Slab *s) {
    delete s->mirror;
    if (s->dev) (void)hipFree(s->dev);
    for (int i = 0; i < 2; ++i) {
      if (s->pinned[i]) (void)hipHostFree(s->pinned[i]);
      if (s->ev[i]) (void)hipEventDestroy(s->ev[i]);
    }
    *s = Slab();
  }
  std::mutex mu_;
  std::vector<Slab> free_;
};

SlabPool &pool() {
  static SlabPool *p = new SlabPool;   // never destroyed: outlives the HIP runtime teardown order
  return *p;
}

// One stream per device for work-table uploads (default priority, created on first use and
// kept for the life of the process): a table copy then overlaps whatever the caller's stream
// is still running, instead of queueing behind it.
int copy_stream(hipStream_t *out) {
  static std::mutex mu;
  static hipStream_t streams[64] = {};
  int dev = 0;
  DMM_HIP(hipGetDevice(&dev));
  if (dev < 0 || dev >= 64) return DMM_EINVAL;
  std::lock_guard<std::mutex> g(mu);
  if (!streams[dev]) DMM_HIP(hipStreamCreateWithFlags(&streams[dev], hipStreamNonBlocking));
  *out = streams[dev];
  return DMM_OK;
}

// upload() copies host bytes to the slab's device buffer on the copy stream and makes the
// caller's stream wait for that copy; it skips the copy when those bytes are already resident.
// `busy_until`, if given, is an event after which earlier readers of the device buffer (kernels
// of a previous call on this plan) are done: the copy waits for it.
struct Uploader {
  Slab slab;
  bool ev_used[2] = {false, false};
  int cur = 0;

  char *dev() const { return slab.dev; }
  int upload(const void *src, size_t bytes, hipStream_t stream, hipEvent_t busy_until = nullptr) {
    if (bytes == 0) return DMM_OK;
    if (bytes > slab.cap) {
      // growing: the old slab may still be read by enqueued work of this plan, on this stream or,
      // from an earlier call, on another one (busy_until is behind all of it)
      if (slab.dev) {
        if (busy_until) DMM_HIP(hipEventSynchronize(busy_until));
        DMM_HIP(hipStreamSynchronize(stream));
        pool().release(&slab);
      }
      int rc = pool().acquire(bytes, &slab);
      if (rc) return rc;
      ev_used[0] = ev_used[1] = false;
    }
    std::vector<char> &resident = *slab.mirror;
    if (resident.size() == bytes && std::memcmp(resident.data(), src, bytes) == 0) {
      // already resident; the caller's stream (possibly another one than last time) still has to
      // be ordered behind the copy that put it there, if this uploader made that copy (a copy made
      // for an earlier owner of the slab finished before the slab went back to the pool)
      if (ev_used[cur]) DMM_HIP(hipStreamWaitEvent(stream, slab.ev[cur], 0));
      return DMM_OK;
    }
    resident.clear();                      // unknown contents until the copy below has been enqueued
    cur ^= 1;
    if (ev_used[cur]) DMM_HIP(hipEventSynchronize(slab.ev[cur]));  // slot last used two uploads ago
    std::memcpy(slab.pinned[cur], src, bytes);
    hipStream_t cs = nullptr;
    int rc = copy_stream(&cs);
    if (rc) return rc;
    if (busy_until) DMM_HIP(hipStreamWaitEvent(cs, busy_until, 0));
    DMM_HIP(hipMemcpyAsync(slab.dev, slab.pinned[cur], bytes, hipMemcpyHostToDevice, cs));
    DMM_HIP(hipEventRecord(slab.ev[cur], cs));
    DMM_HIP(hipStreamWaitEvent(stream, slab.ev[cur], 0));
    ev_used[cur] = true;
    resident.assign((const char *)src, (const char *)src + bytes);
    return DMM_OK;
  }
  // Orders `stream` behind the copy that put the resident bytes in place (for a caller that knows
  // by other means that they are the bytes it wants).
  int order_behind_copy(hipStream_t stream) {
    if (slab.dev && ev_used[cur]) DMM_HIP(hipStreamWaitEvent(stream, slab.ev[cur], 0));
    return DMM_OK;
  }
  // The caller guarantees that no stream work still uses the slab: in particular its last copy has
  // completed, so the mirror describes the buffer.
  void release() {
    // (a call that failed between the upload and its launches may have left the copy in flight)
    if (slab.dev && ev_used[cur]) (void)hipEventSynchronize(slab.ev[cur]);
    pool().release(&slab);
  }
};

// Device-only buffers for the partial sums of K-split items, recycled like the slabs.
class ScratchPool {
 public:
  int acquire(size_t bytes, char **out, size_t *cap) {
    int device = 0;
    DMM_HIP(hipGetDevice(&device));
    {
      std::lock_guard<std::mutex> g(mu_);
      int best = -1;
      for (size_t i = 0; i < free_.size(); ++i)
        if (free_[i].device == device && free_[i].cap >= bytes &&
            (best < 0 || free_[i].cap < free_[(size_t)best].cap))
          best = (int)i;
      if (best >= 0) {
        *out = free_[(size_t)best].p;
        *cap = free_[(size_t)best].cap;
        free_.erase(free_.begin() + best);
        return DMM_OK;
      }
    }
    size_t want = (size_t)4 << 20;
    while (want < bytes) want *= 2;
    char *p = nullptr;
    hipError_t e = hipMalloc((void **)&p, want);
    if (e != hipSuccess) {
      g_last_hip_error = (int)e;
      return e == hipErrorOutOfMemory ? DMM_ENOMEM : DMM_EHIP;
    }
    *out = p;
    *cap = want;
    return DMM_OK;
  }
  // The caller guarantees that no stream work still uses the buffer (and is on its device).
  void release(char **p, size_t *cap) {
    if (!*p) return;
    int device = 0;
    (void)hipGetDevice(&device);
    std::lock_guard<std::mutex> g(mu_);
    if (free_.size() < 8) free_.push_back({*p, *cap, device});
    else (void)hipFree(*p);
    *p = nullptr;
    *cap = 0;
  }

 private:
  struct Entry {
    char *p;
    size_t cap;
    int device;
  };
  std::mutex mu_;
  std::vector<Entry> free_;
};

ScratchPool &scratch_pool() {
  static ScratchPool *p = new ScratchPool;   // never destroyed, like the slab pool
  return *p;
}

// Where the replica sum's (or the broadcast's) tables sit in a device buffer.
struct RedLaunch {
  char *dev_base = nullptr;   // device address of the buffer the offsets below refer to
  size_t n_items = 0;
  size_t o_items = 0, o_tiles = 0, o_parts = 0, o_lds = 0;
  int nparts = 0;
  bool vec_ok = true;
};

// Where the merged macro-tiles' tables sit in the plan's device table.
struct MergedLaunch {
  size_t n_items = 0, o_a = 0, o_b = 0, o_c = 0, o_k = 0, o_fix = 0, n_fix = 0, total = 0;
};

// What the launches of a dmm_execute need to know besides the device table itself.
struct ExecLayout {
  bool merged = false;
  MergedLaunch ml;                                                       // merged macro-tiles
  size_t n_items = 0, o_segs = 0, o_fix = 0, o_red = 0, n_first = 0, n_fix = 0;   // per-group macro-tiles
  bool fuse = false, one_launch = false;
  size_t n_runs = 0;
  bool uses_split = false;      // some macro-tiles store through the plan's scratch buffer
  RedLaunch red;                // the replica-sum launch behind the GEMM (n_items == 0: none)
};

struct DeviceState {
  char *split_buf = nullptr;   // partial sums of K-split items
  size_t split_cap = 0;
  Uploader gemm_table;   // [ItemDev x items][SegDev x segments]
  Uploader red_table;    // [RedItem][RedTile][part pointers][part lds]
  std::vector<char> host;  // scratch for table assembly
  hipEvent_t last_use = nullptr;      // recorded after the last launch of every call
  bool last_use_recorded = false;
  hipEvent_t t_gemm[2] = {nullptr, nullptr}, t_red[2] = {nullptr, nullptr};  // DMM_TIMING
  hipEvent_t t_mid = nullptr;         // ... between the two GEMM launches of a fused replica sum
  bool gemm_timed = false, red_timed = false, mid_timed = false;
  double launch_flops[2] = {0.0, 0.0};  // 2 m n k of the ops behind each of those two launches
  bool ran_merged = false;            // the last dmm_execute ran the merged macro-tiles
  bool ran_k_split = false;           // ... and cut macro-tiles along K
  int ran_fused = 0;                  // ... and fused the replica sum into the GEMM: in 1 launch, in 2; 0 = not
  // The inputs of the last successful dmm_execute (element type, flags, device, the six pointer
  // and leading-dimension arrays) and the layout of the device table it left in gemm_table: a call
  // with the same inputs launches from that table as it stands.
  std::vector<char> exec_key, key_scratch;
  ExecLayout exec_layout;
  bool exec_cached = false;
  bool table_reused = false;          // the last dmm_execute did
};

void destroy_device_state(DeviceState *d) {
  if (!d) return;
  // wait for this plan's own work only, then hand the buffers back to the pool
  if (d->last_use_recorded) (void)hipEventSynchronize(d->last_use);
  d->gemm_table.release();
  d->red_table.release();
  scratch_pool().release(&d->split_buf, &d->split_cap);
  if (d->last_use) (void)hipEventDestroy(d->last_use);
  for (int i = 0; i < 2; ++i) {
    if (d->t_gemm[i]) (void)hipEventDestroy(d->t_gemm[i]);
    if (d->t_red[i]) (void)hipEventDestroy(d->t_red[i]);
  }
  if (d->t_mid) (void)hipEventDestroy(d->t_mid);
  delete d;
}

}  // namespace dmm
