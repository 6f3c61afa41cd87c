// Library-wide state of the C ABI: error reporting and version.
#include "pit_common.hpp"

namespace pit {
int& last_hip_error() {
  static thread_local int code = 0;
  return code;
}
}  // namespace pit

extern "C" int pit_last_hip_error(void) { return pit::last_hip_error(); }
extern "C" int pit_version(void) { return 100; }
