// Host-side support of the cluster kernels (see cluster.hpp).
#include <mutex>
#include <stdlib.h>
#include "cluster.hpp"

namespace bpc {

__global__ void slots_reset_kernel(double *slots, uint32_t n, uint32_t *status, uint32_t *tickets) {
  uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) slots[i] = -1.0;
  if (i == 0) status[0] = 0;  // no wait has given up
  if (tickets && i < (uint32_t)kTicketClasses) tickets[i * (kTicketStride / 4)] = 0;  // next ticket of every class
}

int cluster_capacity(const void *kernel, int threads, size_t dyn_lds) {
  int dev = 0, cus = 0, per_cu = 0;
  if (hipGetDevice(&dev) != hipSuccess) return 0;
  if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return 0;
  if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, kernel, threads, dyn_lds) != hipSuccess) return 0;
  return cus * per_cu;
}

int lds_limit_raised(const void *kernel, size_t bytes) {
  if (hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes) == hipSuccess) return 1;
  (void)hipGetLastError();
  return 0;
}

namespace {
std::mutex g_mu;
hipEvent_t g_event[kMaxDevices];
hipStream_t g_last_stream[kMaxDevices];
bool g_have[kMaxDevices];
}  // namespace

// While `stream` is being captured into a graph nothing is chained: the graph orders its own
// nodes, and an event recorded during capture is not one a later eager launch could wait for.
// Keeping replays of such a graph apart from cluster kernels launched elsewhere at the same
// time is then up to the caller.
static bool is_capturing(hipStream_t stream) {
  hipStreamCaptureStatus st = hipStreamCaptureStatusNone;
  if (hipStreamIsCapturing(stream, &st) != hipSuccess) return false;
  return st != hipStreamCaptureStatusNone;
}

// The event is recorded only when it is needed: when a launch comes on another stream than the
// one before, on that earlier stream (it then covers the earlier kernel and whatever that
// stream was given since, which is more than needed and never less).  Recording one after
// every launch cost each call some microseconds of idle device time.
hipError_t cluster_launch_begin(hipStream_t stream) {
  if (is_capturing(stream)) return hipSuccess;
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(g_mu);
  if (!g_have[dev] || g_last_stream[dev] == stream) return hipSuccess;
  if (is_capturing(g_last_stream[dev])) return hipSuccess;   // (nothing can be recorded on it now)
  if (!g_event[dev]) {
    e = hipEventCreateWithFlags(&g_event[dev], hipEventDisableTiming);
    if (e != hipSuccess) return e;
  }
  e = hipEventRecord(g_event[dev], g_last_stream[dev]);
  if (e != hipSuccess) {
    // the earlier stream is gone: wait for everything on the device instead
    (void)hipGetLastError();
    return hipDeviceSynchronize();
  }
  return hipStreamWaitEvent(stream, g_event[dev], 0);
}

hipError_t cluster_prepare_device() {
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(g_mu);
  if (g_event[dev]) return hipSuccess;
  return hipEventCreateWithFlags(&g_event[dev], hipEventDisableTiming);
}

hipError_t cluster_launch_end(hipStream_t stream) {
  if (is_capturing(stream)) return hipSuccess;
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(g_mu);
  g_last_stream[dev] = stream;
  g_have[dev] = true;
  return hipSuccess;
}

}  // namespace bpc
