// Error reporting and version of the C ABI.
#include <string.h>

#include "photon_host.h"

namespace photon {

char* error_buffer() {
  static thread_local char buf[512] = {0};
  return buf;
}

void clear_error() { error_buffer()[0] = 0; }

int32_t fail(int32_t code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(error_buffer(), 512, fmt, ap);
  va_end(ap);
  return code;
}

}  // namespace photon

extern "C" int32_t photon_version(void) { return 100; }

extern "C" const char* photon_last_error(void) { return photon::error_buffer(); }
