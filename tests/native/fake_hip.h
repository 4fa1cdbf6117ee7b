// A stand-in for the HIP runtime that runs on the CPU, for tests of the library's host-side ordering.
// "Device" memory is host memory.  Streams are queues of operations (copy, kernel, event record,
// wait on an event) that execute only when the test pumps them, in any order the stream and event
// semantics allow: an operation runs after everything queued before it on its stream, a wait runs
// once the record it refers to (the latest one queued when the wait was queued) has run, a wait on
// an event that was never recorded is a no-op, a query of such an event reports success.
#pragma once
#include <hip/hip_runtime_api.h>

#include <cstddef>
#include <cstdint>
#include <functional>
#include <vector>

namespace fakehip {
// Queues a "kernel": fn runs when the stream reaches it.
void enqueue_kernel(hipStream_t st, std::function<void()> fn);
// Runs the operation at the head of st if it can run; false if the queue is empty or blocked.
bool step(hipStream_t st);
// Runs up to max_ops operations, each from a randomly chosen stream that can make progress
// (streams listed in `prefer` are chosen with probability 3/4 when they can); returns how many ran.
int pump_random(uint64_t& rng_state, int max_ops, const std::vector<hipStream_t>& prefer);
// Runs everything; aborts with a message if queues are left that can never run.
void drain();
// All waits become no-ops (to show that a check notices missing ordering).
void set_ignore_waits(bool on);
// The `calls`-th hipMemcpyAsync from now fails (hipErrorUnknown) without queueing anything; 0 = none.
void fail_copy_in(int calls);
size_t pending_ops();
}  // namespace fakehip
