// Pool of host staging buffers for descriptor uploads, written against a small backend interface so that the slot
// state machine can be exercised on the CPU with several threads (the library plugs in pinned memory and hipEvents).
//
// A slot is FREE, RESERVED (handed to one caller, who is filling it; its event has not been recorded for this use and
// must not be queried) or IN_FLIGHT (the copy that reads it has been enqueued and its event recorded; the slot becomes
// free again once that event has completed). Only FREE slots, and IN_FLIGHT slots whose event has completed, are handed
// out, so two threads never fill the same buffer.
#pragma once
#include <cstddef>
#include <mutex>
#include <vector>

template <class Backend>
class zp_staging_pool {
 public:
  enum State { FREE = 0, RESERVED = 1, IN_FLIGHT = 2 };
  struct Slot {
    void *host = nullptr;
    size_t cap = 0;
    typename Backend::event_t ev{};
    State state = FREE;
  };

  // Reserves a slot of at least `bytes` for the caller (allocating one if none is free). Returns 0 or the backend's error.
  int acquire(size_t bytes, int *slot_out, void **host_out) {
    std::lock_guard<std::mutex> lk(mu_);
    for (size_t i = 0; i < slots_.size(); i++) {
      Slot &s = slots_[i];
      if (s.cap < bytes || s.state == RESERVED) continue;
      if (s.state == IN_FLIGHT && !Backend::event_done(s.ev)) continue;
      s.state = RESERVED;
      *slot_out = (int)i;
      *host_out = s.host;
      return 0;
    }
    Slot s;
    s.cap = bytes < min_bytes_ ? min_bytes_ : ((bytes + 255) & ~(size_t)255);
    int rc = Backend::alloc(&s.host, s.cap);
    if (rc) return rc;
    rc = Backend::event_create(&s.ev);
    if (rc) {
      Backend::release(s.host);
      return rc;
    }
    s.state = RESERVED;
    slots_.push_back(s);
    *slot_out = (int)slots_.size() - 1;
    *host_out = s.host;
    return 0;
  }
  // The caller has enqueued the copy out of the slot: records the slot's event behind it on `stream`; the slot stays
  // busy until the event completes. On a backend error the slot is freed (nothing reads it).
  int submitted(int slot, typename Backend::stream_t stream) {
    std::lock_guard<std::mutex> lk(mu_);
    Slot &s = slots_[slot];
    const int rc = Backend::event_record(s.ev, stream);
    s.state = rc ? FREE : IN_FLIGHT;
    return rc;
  }
  // The caller gives a reserved slot back without having enqueued anything that reads it.
  void abandon(int slot) {
    std::lock_guard<std::mutex> lk(mu_);
    slots_[slot].state = FREE;
  }
  size_t size() {
    std::lock_guard<std::mutex> lk(mu_);
    return slots_.size();
  }

 private:
  std::mutex mu_;
  std::vector<Slot> slots_;
  size_t min_bytes_ = 1 << 16;
};
