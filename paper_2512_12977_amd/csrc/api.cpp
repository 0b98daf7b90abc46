// Error reporting, version, RoPE frequency table.
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <mutex>

#include "vlc_internal.h"

namespace vlc {

static thread_local char g_err[512] = "";

int fail(int code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return code;
}

int ensure_dynamic_lds(const void* kernel, int bytes) {
  // a fixed table, so that no call on the launch path touches the heap: the library has a few dozen kernel
  // instantiations with dynamic LDS, times the devices of one node
  struct Entry { int dev; const void* kernel; };
  constexpr int kMax = 1024;
  static std::mutex mu;
  static Entry done[kMax];
  static int n_done = 0;
  int dev = 0;
  VLC_CHECK_HIP(hipGetDevice(&dev));
  std::lock_guard<std::mutex> lock(mu);
  for (int i = 0; i < n_done; ++i)
    if (done[i].dev == dev && done[i].kernel == kernel) return VLC_OK;
  VLC_CHECK_HIP(hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes));
  if (n_done < kMax) done[n_done++] = Entry{dev, kernel};   // a full table only costs the repeated call
  return VLC_OK;
}

RopeFreq make_rope_freq(double base, int D, int mrope_h, int mrope_w) {
  RopeFreq f;
  for (int i = 0; i < 64; ++i) {
    f.inv_freq[i] = 0.0;
    f.axis[i] = 0;
  }
  for (int i = 0; i < D / 2 && i < 64; ++i) {
    f.inv_freq[i] = std::pow(base, -2.0 * (double)i / (double)D);
    // interleaved 3-axis layout: height on i = 1, 4, 7, ... < 3*mrope_h, width on i = 2, 5, 8, ... < 3*mrope_w
    if (i % 3 == 1 && i < 3 * mrope_h) f.axis[i] = 1;
    if (i % 3 == 2 && i < 3 * mrope_w) f.axis[i] = 2;
  }
  return f;
}

}  // namespace vlc

extern "C" const char* vlc_last_error(void) { return vlc::g_err; }
extern "C" int vlc_version(void) { return 100; }
