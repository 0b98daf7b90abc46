// Error reporting, version, RoPE frequency table.
#include <cmath>
#include <cstdarg>
#include <cstdio>

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
