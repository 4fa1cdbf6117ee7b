// CPU stand-in for the part of the HIP runtime that the library's host code calls (see fake_hip.h).
#include "fake_hip.h"

#include <algorithm>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <deque>
#include <map>

struct ihipEvent_t {
  uint64_t recorded = 0;   // records queued so far
  uint64_t completed = 0;  // highest record that has run
};

namespace {
struct Op {
  enum Kind { COPY, KERNEL, RECORD, WAIT } kind;
  hipEvent_t ev = nullptr;
  uint64_t gen = 0;
  void* dst = nullptr;
  const void* src = nullptr;
  size_t n = 0;
  std::function<void()> fn;
};
}  // namespace

struct ihipStream_t {
  std::deque<Op> q;
};

namespace {
ihipStream_t g_null_stream;
std::vector<ihipStream_t*> g_streams{&g_null_stream};
std::vector<ihipEvent_t*> g_dead_events;  // kept: queued operations may still name them
std::map<void*, size_t> g_host, g_dev;
bool g_ignore_waits = false;
int g_copy_fault_in = 0;  // > 0: that many hipMemcpyAsync calls from now, one fails

ihipStream_t* S(hipStream_t st) { return st ? st : &g_null_stream; }

bool runnable(const Op& op) {
  return op.kind != Op::WAIT || g_ignore_waits || op.ev->completed >= op.gen;
}

void run(Op& op) {
  switch (op.kind) {
    case Op::COPY: std::memcpy(op.dst, op.src, op.n); break;
    case Op::KERNEL: op.fn(); break;
    case Op::RECORD: op.ev->completed = std::max(op.ev->completed, op.gen); break;
    case Op::WAIT: break;
  }
}

uint64_t next(uint64_t& s) {  // xorshift64*
  s ^= s >> 12; s ^= s << 25; s ^= s >> 27;
  return s * 0x2545F4914F6CDD1DULL;
}
}  // namespace

namespace fakehip {
void enqueue_kernel(hipStream_t st, std::function<void()> fn) {
  Op op;
  op.kind = Op::KERNEL;
  op.fn = std::move(fn);
  S(st)->q.push_back(std::move(op));
}

bool step(hipStream_t st) {
  ihipStream_t* s = S(st);
  if (s->q.empty() || !runnable(s->q.front())) return false;
  Op op = std::move(s->q.front());
  s->q.pop_front();
  run(op);
  return true;
}

int pump_random(uint64_t& rng, int max_ops, const std::vector<hipStream_t>& prefer) {
  int done = 0;
  while (done < max_ops) {
    std::vector<ihipStream_t*> can, can_pref;
    for (ihipStream_t* s : g_streams)
      if (!s->q.empty() && runnable(s->q.front())) {
        can.push_back(s);
        if (std::find(prefer.begin(), prefer.end(), s) != prefer.end()) can_pref.push_back(s);
      }
    if (can.empty()) break;
    auto& from = (!can_pref.empty() && next(rng) % 4 != 0) ? can_pref : can;
    step(from[next(rng) % from.size()]);
    ++done;
  }
  return done;
}

void drain() {
  for (;;) {
    bool progress = false, left = false;
    for (ihipStream_t* s : g_streams) {
      while (step(s)) progress = true;
      left |= !s->q.empty();
    }
    if (!left) {  // nothing queued names a destroyed event any more
      for (ihipEvent_t* e : g_dead_events) delete e;
      g_dead_events.clear();
      return;
    }
    if (!progress) {
      std::printf("fake HIP: queues left that can never run (a wait on a record that is not queued)\n");
      std::abort();
    }
  }
}

void set_ignore_waits(bool on) { g_ignore_waits = on; }
void fail_copy_in(int calls) { g_copy_fault_in = calls; }

size_t pending_ops() {
  size_t n = 0;
  for (ihipStream_t* s : g_streams) n += s->q.size();
  return n;
}
}  // namespace fakehip

extern "C" {

hipError_t hipDeviceSynchronize(void) { fakehip::drain(); return hipSuccess; }
hipError_t hipGetLastError(void) { return hipSuccess; }

hipError_t hipStreamCreateWithFlags(hipStream_t* stream, unsigned int) {
  *stream = new ihipStream_t;
  g_streams.push_back(*stream);
  return hipSuccess;
}

// Everything queued on the stream so far has run when this returns (other streams advance as far as
// that needs).
hipError_t hipStreamSynchronize(hipStream_t stream) {
  ihipStream_t* s = S(stream);
  while (!s->q.empty()) {
    if (fakehip::step(s)) continue;
    bool progress = false;  // blocked on a wait: let another stream advance by one operation
    for (ihipStream_t* o : g_streams)
      if (o != s && fakehip::step(o)) { progress = true; break; }
    if (!progress) {
      std::printf("fake HIP: hipStreamSynchronize on a stream that can never drain\n");
      std::abort();
    }
  }
  return hipSuccess;
}

hipError_t hipStreamDestroy(hipStream_t stream) {
  if (!stream) return hipErrorInvalidHandle;
  fakehip::drain();
  g_streams.erase(std::find(g_streams.begin(), g_streams.end(), stream));
  delete stream;
  return hipSuccess;
}

hipError_t hipStreamWaitEvent(hipStream_t stream, hipEvent_t event, unsigned int) {
  if (!event) return hipErrorInvalidHandle;
  if (event->recorded == 0) return hipSuccess;  // never recorded: nothing to wait for
  Op op;
  op.kind = Op::WAIT;
  op.ev = event;
  op.gen = event->recorded;
  S(stream)->q.push_back(std::move(op));
  return hipSuccess;
}

hipError_t hipEventCreateWithFlags(hipEvent_t* event, unsigned) { *event = new ihipEvent_t; return hipSuccess; }
hipError_t hipEventCreate(hipEvent_t* event) { *event = new ihipEvent_t; return hipSuccess; }

hipError_t hipEventRecord(hipEvent_t event, hipStream_t stream) {
  if (!event) return hipErrorInvalidHandle;
  Op op;
  op.kind = Op::RECORD;
  op.ev = event;
  op.gen = ++event->recorded;
  S(stream)->q.push_back(std::move(op));
  return hipSuccess;
}

hipError_t hipEventDestroy(hipEvent_t event) {
  if (!event) return hipErrorInvalidHandle;
  g_dead_events.push_back(event);
  return hipSuccess;
}

hipError_t hipEventSynchronize(hipEvent_t event) {
  if (!event) return hipErrorInvalidHandle;
  fakehip::drain();
  return hipSuccess;
}

hipError_t hipEventElapsedTime(float* ms, hipEvent_t start, hipEvent_t stop) {
  if (!start || !stop) return hipErrorInvalidHandle;
  if (start->completed < start->recorded || stop->completed < stop->recorded) return hipErrorNotReady;
  *ms = 0.001f;
  return hipSuccess;
}

hipError_t hipEventQuery(hipEvent_t event) {
  if (!event) return hipErrorInvalidHandle;
  return event->completed >= event->recorded ? hipSuccess : hipErrorNotReady;
}

hipError_t hipPointerGetAttributes(hipPointerAttribute_t* at, const void* ptr) {
  std::memset(at, 0, sizeof(*at));
  for (auto* m : {&g_host, &g_dev}) {
    auto it = m->upper_bound(const_cast<void*>(ptr));
    if (it == m->begin()) continue;
    --it;
    if ((const char*)ptr < (const char*)it->first + it->second) {
      at->type = m == &g_host ? hipMemoryTypeHost : hipMemoryTypeDevice;
      return hipSuccess;
    }
  }
  return hipErrorInvalidValue;
}

hipError_t hipMalloc(void** ptr, size_t size) {
  *ptr = std::malloc(size ? size : 1);
  if (!*ptr) return hipErrorOutOfMemory;
  std::memset(*ptr, 0xCD, size);  // nothing may rely on fresh device memory
  g_dev[*ptr] = size;
  return hipSuccess;
}

hipError_t hipHostMalloc(void** ptr, size_t size, unsigned int) {
  *ptr = std::malloc(size ? size : 1);
  if (!*ptr) return hipErrorOutOfMemory;
  std::memset(*ptr, 0xEE, size);
  g_host[*ptr] = size;
  return hipSuccess;
}

hipError_t hipStreamIsCapturing(hipStream_t, hipStreamCaptureStatus* status) {
  *status = hipStreamCaptureStatusNone;
  return hipSuccess;
}

hipError_t hipMemsetAsync(void* dst, int value, size_t n, hipStream_t stream) {
  Op op;
  op.kind = Op::KERNEL;
  op.fn = [=] { std::memset(dst, value, n); };
  S(stream)->q.push_back(std::move(op));
  return hipSuccess;
}

hipError_t hipHostGetDevicePointer(void** dev, void* host, unsigned int) {
  *dev = host;  // "device" memory is host memory here
  return hipSuccess;
}

hipError_t hipFree(void* ptr) {
  if (!ptr) return hipSuccess;
  fakehip::drain();  // frees synchronise with the device
  if (!g_dev.erase(ptr)) return hipErrorInvalidValue;
  std::free(ptr);
  return hipSuccess;
}

hipError_t hipHostFree(void* ptr) {
  if (!ptr) return hipSuccess;
  fakehip::drain();
  if (!g_host.erase(ptr)) return hipErrorInvalidValue;
  std::free(ptr);
  return hipSuccess;
}

hipError_t hipMemcpy(void* dst, const void* src, size_t n, hipMemcpyKind) {
  fakehip::drain();
  std::memcpy(dst, src, n);
  return hipSuccess;
}

hipError_t hipMemcpyAsync(void* dst, const void* src, size_t n, hipMemcpyKind, hipStream_t stream) {
  if (g_copy_fault_in > 0 && --g_copy_fault_in == 0) return hipErrorUnknown;  // injected fault: nothing is queued
  Op op;
  op.kind = Op::COPY;
  op.dst = dst;
  op.src = src;
  op.n = n;
  S(stream)->q.push_back(std::move(op));
  return hipSuccess;
}

}  // extern "C"
