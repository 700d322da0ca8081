// Device memory, pinned host memory and events between calls.  A handle is often short-lived
// (analyse, plan, free, again with the next trace), and hipMalloc / hipFree / hipHostMalloc /
// hipEventDestroy cost 0.05 to 0.3 ms of host time each: what a call releases is kept here, up
// to a limit, and handed to the next request of a fitting size.  g10_trim() returns everything
// kept to the driver.  A block is only released by its owner after the work that used it has
// been waited for, so a kept block is idle and can serve any stream.
#include "g10_internal.h"

#include <mutex>
#include <new>
#include <vector>

void mem_trim();

namespace {

struct Block {
  void* p;
  size_t bytes;
  int dev;                                        // (-1: pinned host memory)
};

struct State {
  std::mutex mu;
  std::vector<Block> live, kept;                  // handed out; released and kept (oldest first)
  size_t kept_bytes = 0;
  std::vector<hipEvent_t> events[G10_MEM_MAX_DEVICES];
};

// (never destroyed: at process exit the HIP runtime may already be gone)
State& state() {
  static State* s = new State();
  return *s;
}

const size_t KEEP_MAX_BYTES = (size_t)4 << 30;    // of kept blocks together
const size_t KEEP_MAX_BLOCKS = 96;
const size_t KEEP_MAX_EVENTS = 256;               // per device

void give_back(const Block& b) {
  if (b.dev < 0) (void)hipHostFree(b.p);
  else (void)hipFree(b.p);
}

// a kept block serves a request it is not much larger than
bool fits(size_t have, size_t want) { return have >= want && have - want <= want / 8 + ((size_t)1 << 20); }

int alloc(void** out, size_t bytes, int dev) {
  State& st = state();
  if (!bytes) bytes = 256;
  {
    std::lock_guard<std::mutex> g(st.mu);
    size_t best = st.kept.size();
    for (size_t i = 0; i < st.kept.size(); ++i)
      if (st.kept[i].dev == dev && fits(st.kept[i].bytes, bytes) && (best == st.kept.size() || st.kept[i].bytes < st.kept[best].bytes))
        best = i;
    if (best != st.kept.size()) {
      const Block b = st.kept[best];
      st.kept.erase(st.kept.begin() + (long)best);
      st.kept_bytes -= b.bytes;
      st.live.push_back(b);
      *out = b.p;
      return G10_OK;
    }
  }
  void* q = nullptr;
  for (int attempt = 0; attempt < 2; ++attempt) {
    const hipError_t e = dev < 0 ? hipHostMalloc(&q, bytes, hipHostMallocDefault) : hipMalloc(&q, bytes);
    if (e == hipSuccess) break;
    (void)hipGetLastError();
    q = nullptr;
    if (attempt == 0) mem_trim();                 // what is kept may be what is missing
  }
  if (!q) return G10_ENOMEM;
  std::lock_guard<std::mutex> g(st.mu);
  st.live.push_back(Block{q, bytes, dev});
  *out = q;
  return G10_OK;
}

void release(void* p) {
  if (!p) return;
  State& st = state();
  std::vector<Block> out;                         // given back to the driver outside the lock
  {
    std::lock_guard<std::mutex> g(st.mu);
    size_t i = 0;
    while (i < st.live.size() && st.live[i].p != p) ++i;
    if (i == st.live.size()) return;              // (not one of ours: nothing is known about it)
    const Block b = st.live[i];
    st.live[i] = st.live.back();
    st.live.pop_back();
    if (b.bytes > KEEP_MAX_BYTES / 2) out.push_back(b);
    else {
      st.kept.push_back(b);
      st.kept_bytes += b.bytes;
      while (st.kept_bytes > KEEP_MAX_BYTES || st.kept.size() > KEEP_MAX_BLOCKS) {
        out.push_back(st.kept.front());
        st.kept_bytes -= st.kept.front().bytes;
        st.kept.erase(st.kept.begin());
      }
    }
  }
  for (const Block& b : out) give_back(b);
}

}  // namespace

int mem_dev_alloc(void** out, size_t bytes) {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) { (void)hipGetLastError(); return G10_EDEVICE; }
  return alloc(out, bytes, dev);
}
void mem_dev_free(void* p) { release(p); }

int mem_host_alloc(void** out, size_t bytes) { return alloc(out, bytes, -1); }
void mem_host_free(void* p) { release(p); }

int mem_event_get(hipEvent_t* out) {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) { (void)hipGetLastError(); return G10_EDEVICE; }
  if (dev >= 0 && dev < G10_MEM_MAX_DEVICES) {
    State& st = state();
    std::lock_guard<std::mutex> g(st.mu);
    if (!st.events[dev].empty()) {
      *out = st.events[dev].back();
      st.events[dev].pop_back();
      return G10_OK;
    }
  }
  G10_HIP(hipEventCreate(out));
  return G10_OK;
}

void mem_event_put(hipEvent_t e, int dev) {
  if (!e) return;
  if (dev >= 0 && dev < G10_MEM_MAX_DEVICES) {
    State& st = state();
    std::lock_guard<std::mutex> g(st.mu);
    if (st.events[dev].size() < KEEP_MAX_EVENTS) { st.events[dev].push_back(e); return; }
  }
  (void)hipEventDestroy(e);
}

void mem_trim() {
  State& st = state();
  std::vector<Block> out;
  std::vector<hipEvent_t> ev;
  {
    std::lock_guard<std::mutex> g(st.mu);
    out.swap(st.kept);
    st.kept_bytes = 0;
    for (auto& v : st.events) { ev.insert(ev.end(), v.begin(), v.end()); v.clear(); }
  }
  for (const Block& b : out) give_back(b);
  for (hipEvent_t e : ev) (void)hipEventDestroy(e);
}

extern "C" void g10_trim(void) { mem_trim(); }
