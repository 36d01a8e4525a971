// Optional device-side time stamps (build option VTE_TRACE_STAMPS, off in the product library).
// A kernel marks points of its timeline with VTE_STAMP(i): lane 0 of every wave of the first
// 1024 workgroups stores the device's constant 100 MHz clock (10 ns steps) for point i.  The
// host reads the table of the most recent launch with vte_trace_stamps_read() and sees, wave by
// wave, when the launch arguments were in, when the first operands arrived, when the stream was
// through and what the tail cost -- the breakdown a kernel trace of whole launches cannot give.
// Reading the clock waits for the wave's outstanding LDS and scalar operations (not for its
// vector loads), which costs a traced launch a few hundred ns: the trace is for where the time
// goes, the untraced library for how much it is.
#pragma once
#ifdef VTE_TRACE_STAMPS
constexpr int kTraceWorkgroups = 1024, kTraceWaves = 8, kTracePoints = 8;
static __device__ unsigned long long vte_trace_stamps[kTraceWorkgroups * kTraceWaves * kTracePoints];
#define VTE_STAMP(i)                                                                                   \
  do {                                                                                                 \
    __builtin_amdgcn_sched_barrier(0);                                                                 \
    const unsigned long long t_ = wall_clock64();                                                      \
    if ((threadIdx.x & 63) == 0 && blockIdx.x < kTraceWorkgroups && blockIdx.y == 0 && blockIdx.z == 0) \
      vte_trace_stamps[(blockIdx.x * kTraceWaves + (threadIdx.x >> 6)) * kTracePoints + (i)] = t_;     \
    __builtin_amdgcn_sched_barrier(0);                                                                 \
  } while (0)
#else
#define VTE_STAMP(i) do { } while (0)
#endif
