// Host-side bookkeeping for the libraries whose work-queue kernels keep their counters in a
// static device array: which block of that array a stream's launches use.
//
// Launches on one stream run one after the other, so one block per stream is never shared by
// two running kernels; a block, once given to a stream, stays with it (streams are few and
// long-lived; the 33rd on a device gets none, and its calls run the kernels that need no
// counters).  Two kinds of stream get none either: the per-thread default stream, whose one
// handle stands for a different stream in every host thread, and a stream that is being
// captured into a graph, because a graph can be replayed on any stream, next to anything.
#pragma once

#include <hip/hip_runtime.h>

#include <mutex>

namespace rms {
namespace host {

constexpr int kStreamSlots = 32;    // blocks handed to streams, per device
constexpr int kSlotDevices = 64;    // devices a process is expected to see at most

class StreamSlots {
 public:
  // The block (0 .. kStreamSlots - 1) of `stream` on the current device; -1 if this call has
  // to do without counters.
  int block_of(hipStream_t stream) {
    if (stream == hipStreamPerThread) return -1;
    hipStreamCaptureStatus capture = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(stream, &capture) != hipSuccess) {
      (void)hipGetLastError();
      return -1;
    }
    if (capture != hipStreamCaptureStatusNone) return -1;
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kSlotDevices) return -1;
    std::lock_guard<std::mutex> lock(mu_);
    Table& tb = tables_[dev];
    for (int k = 0; k < tb.used; ++k)
      if (tb.owner[k] == stream) return k;
    if (tb.used == kStreamSlots) return -1;
    tb.owner[tb.used] = stream;
    return tb.used++;
  }

 private:
  struct Table {
    hipStream_t owner[kStreamSlots];
    int used;
  };
  std::mutex mu_;
  Table tables_[kSlotDevices] = {};
};

}  // namespace host
}  // namespace rms
