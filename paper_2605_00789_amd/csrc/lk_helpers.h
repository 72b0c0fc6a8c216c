// Helper streams of the library (host side).  Some calls run independent halves side by side: they fork from the
// caller's stream onto helper streams and rejoin it before they return.  The helpers are host-side handles, kept per
// device in small pools, created on first need outside stream capture at default priority and never destroyed.
//
// Why pools: while a caller's stream is being captured into a graph, a helper stream that forked from it belongs to
// that capture until the caller ends it -- long after the call has returned.  Another caller (eager, or capturing
// a graph of its own) must not touch that helper meanwhile, or the capture is invalidated.  So a call takes a set
// whose streams are idle, or already part of the caller's own capture; if every set is held by other captures and
// no new one can be made (pool full, or the caller itself is capturing), the call gets none and enqueues everything
// on the caller's stream in order.
#pragma once
#include <hip/hip_runtime.h>
#include <mutex>

namespace lk {

constexpr int HELPER_SETS_PER_DEVICE = 4;
constexpr int HELPER_MAX_DEVICES = 64;

template <int N_STREAMS, int N_EVENTS>
struct HelperSet {
  hipStream_t stream[N_STREAMS] = {};
  hipEvent_t event[N_EVENTS] = {};
  bool ready = false;
  std::mutex in_use;   // one caller at a time enqueues its fork ... join sequence on a set
};

// Returns a usable set for a call on `main` with `guard` holding its in_use mutex, or nullptr (then: no helpers).
template <int N_STREAMS, int N_EVENTS>
HelperSet<N_STREAMS, N_EVENTS> *acquire_helpers(hipStream_t main, std::unique_lock<std::mutex> &guard) {
  using Set = HelperSet<N_STREAMS, N_EVENTS>;
  static Set pool[HELPER_MAX_DEVICES][HELPER_SETS_PER_DEVICE];
  static std::mutex mu[HELPER_MAX_DEVICES];
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= HELPER_MAX_DEVICES) return nullptr;
  hipStreamCaptureStatus cs = hipStreamCaptureStatusNone;
  unsigned long long cid = 0;
  if (hipStreamGetCaptureInfo(main, &cs, &cid) != hipSuccess) { (void)hipGetLastError(); return nullptr; }
  const bool capturing = cs != hipStreamCaptureStatusNone;
  std::lock_guard<std::mutex> lock(mu[dev]);
  for (int k = 0; k < HELPER_SETS_PER_DEVICE; ++k) {
    Set &h = pool[dev][k];
    if (!h.ready) {
      if (capturing) continue;   // never create objects while the caller is capturing
      bool ok = true;
      int ns = 0, ne = 0;
      for (; ok && ns < N_STREAMS; ++ns) ok = hipStreamCreateWithFlags(&h.stream[ns], hipStreamNonBlocking) == hipSuccess;
      for (; ok && ne < N_EVENTS; ++ne) ok = hipEventCreateWithFlags(&h.event[ne], hipEventDisableTiming) == hipSuccess;
      if (!ok) {   // give back what was made; the slot stays empty and is tried again by a later call
        (void)hipGetLastError();
        for (int i = 0; i < N_STREAMS; ++i) if (h.stream[i]) { (void)hipStreamDestroy(h.stream[i]); h.stream[i] = nullptr; }
        for (int i = 0; i < N_EVENTS; ++i) if (h.event[i]) { (void)hipEventDestroy(h.event[i]); h.event[i] = nullptr; }
        (void)hipGetLastError();
        return nullptr;
      }
      h.ready = true;
    }
    // idle, or already part of this caller's capture?
    std::unique_lock<std::mutex> g(h.in_use, std::try_to_lock);
    if (!g.owns_lock()) {
      // another host thread is enqueueing on it right now: wait for it only if it is the last resort
      if (k + 1 < HELPER_SETS_PER_DEVICE) continue;
      g.lock();
    }
    bool usable = true;
    for (int i = 0; usable && i < N_STREAMS; ++i) {
      hipStreamCaptureStatus hs = hipStreamCaptureStatusNone;
      unsigned long long hid = 0;
      if (hipStreamGetCaptureInfo(h.stream[i], &hs, &hid) != hipSuccess) { (void)hipGetLastError(); usable = false; break; }
      if (hs != hipStreamCaptureStatusNone && !(capturing && hid == cid)) usable = false;
    }
    if (!usable) continue;
    guard = std::move(g);
    return &h;
  }
  return nullptr;
}

}  // namespace lk
