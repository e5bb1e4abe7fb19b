// Pinned host staging for the small per-call metadata uploads (attention tile lists, positions,
// scatter rows): a ring of slots, each with an event that marks the end of its last copy, so that
// a call neither allocates nor waits for the GPU unless the host is a whole ring ahead of it.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>

namespace mllm {

struct PinnedRing {
  static constexpr int SLOTS = 4;
  struct Slot {
    void* p = nullptr;
    size_t bytes = 0;
    hipEvent_t done = nullptr;
    bool pending = false;
  };
  Slot slot[SLOTS];
  int next = 0;

  // Makes every slot at least `bytes` large.  Allocates (and, for a slot whose copy is still in
  // flight, waits): meant for set-up calls, not for the launch path.
  hipError_t reserve(size_t bytes) {
    for (Slot& s : slot) {
      hipError_t e = grow(s, bytes);
      if (e != hipSuccess) return e;
    }
    return hipSuccess;
  }

  // The next slot of the ring, ready to be filled by the host.  Waits only if that slot's previous
  // copy (SLOTS calls ago) has not finished; allocates only if the slot is smaller than `bytes`.
  hipError_t acquire(size_t bytes, Slot** out) {
    Slot& s = slot[next];
    next = (next + 1) % SLOTS;
    hipError_t e = settle(s);
    if (e != hipSuccess) return e;
    if (s.bytes < bytes && (e = grow(s, bytes)) != hipSuccess) return e;
    *out = &s;
    return hipSuccess;
  }

  // Call after the asynchronous copy out of the slot has been enqueued on `stream`.
  hipError_t commit(Slot* s, hipStream_t stream) {
    hipError_t e = hipEventRecord(s->done, stream);
    if (e == hipSuccess) s->pending = true;
    return e;
  }

  void destroy() {
    for (Slot& s : slot) {
      (void)settle(s);
      if (s.done) (void)hipEventDestroy(s.done);
      if (s.p) (void)hipHostFree(s.p);
      s = Slot();
    }
  }

 private:
  static hipError_t settle(Slot& s) {
    if (!s.pending) return hipSuccess;
    s.pending = false;
    return hipEventSynchronize(s.done);
  }
  static hipError_t grow(Slot& s, size_t bytes) {
    hipError_t e;
    if (!s.done && (e = hipEventCreateWithFlags(&s.done, hipEventDisableTiming)) != hipSuccess) return e;
    if (s.bytes >= bytes) return hipSuccess;
    if ((e = settle(s)) != hipSuccess) return e;
    if (s.p) (void)hipHostFree(s.p);
    s.p = nullptr;
    s.bytes = 0;
    const size_t want = bytes + bytes / 2 + 4096;    // headroom: microbatches of one run differ a little
    if ((e = hipHostMalloc(&s.p, want, hipHostMallocDefault)) != hipSuccess) return e;
    s.bytes = want;
    return hipSuccess;
  }
};

}  // namespace mllm
