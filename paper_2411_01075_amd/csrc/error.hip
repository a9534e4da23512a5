#include "common.h"
#include <cstring>

namespace cephalo {

char* error_buffer() {
  static thread_local char buf[512] = {0};
  return buf;
}

int fail(int code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(error_buffer(), 512, fmt, ap);
  va_end(ap);
  return code;
}

}  // namespace cephalo

extern "C" const char* cephalo_last_error(void) { return cephalo::error_buffer(); }
