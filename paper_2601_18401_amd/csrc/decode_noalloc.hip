// Decode span-attention for callers that cannot allocate (code under HIP graph capture, tight
// serving loops, harnesses that forbid hipMalloc): the partial records of the split-KV kernels,
// which sl_span_attention_decode takes from a caller workspace, live in a device array of the
// library instead.  The kernels are the ones of decode_attention.hip; they receive the array's
// address as their workspace argument.
//
// Every GPU holds its own copy of the array at its own address.  `scratch` below is, in host
// code, only a stand-in for the symbol: the device address is looked up once per device with
// hipGetSymbolAddress, with that device current, and only the looked-up pointer is ever handed to
// a kernel.
#include <mutex>

#include "kernels.h"

namespace sl {

namespace {

constexpr size_t kScratchBytes = (size_t)8 << 20;  // 3.5x what a 1M- or 10M-token step with 16 + 1 slots needs
constexpr int kMaxDevices = 64;

static __device__ __align__(256) unsigned char scratch[kScratchBytes];

std::mutex g_mu;
void* g_scratch_of_device[kMaxDevices];  // zero-initialised; filled on the first call on a device

}  // namespace

size_t decode_attention_static_scratch_bytes() { return kScratchBytes; }

sl_status decode_attention_static(const Problem& pb, const void* Q, const void* K, const void* V,
                                  const int32_t* idx, void* O, float* LSE, hipStream_t st) {
  if (decode_attention_ws_bytes(pb) > kScratchBytes) return SL_ERR_UNSUPPORTED;  // nothing enqueued
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return SL_ERR_LAUNCH;
  void* ptr = nullptr;
  {
    std::lock_guard<std::mutex> lock(g_mu);
    if (!g_scratch_of_device[dev]) {
      void* found = nullptr;
      if (hipGetSymbolAddress(&found, HIP_SYMBOL(scratch)) != hipSuccess || !found) return SL_ERR_LAUNCH;
      g_scratch_of_device[dev] = found;
    }
    ptr = g_scratch_of_device[dev];
  }
  // Every partial record a call's reduction reads is written by that call's K/V kernel first (an
  // empty slot or chunk writes an empty record), so the array needs no clearing between calls.
  return decode_attention(pb, Q, K, V, idx, O, LSE, ptr, st);
}

}  // namespace sl
