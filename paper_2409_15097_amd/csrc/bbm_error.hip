// Error reporting and version of libbbm.
#include "bbm_internal.h"

namespace bbm {
static thread_local char g_err[512] = "";

int fail(int code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return code;
}
void clear_error() { g_err[0] = '\0'; }
}  // namespace bbm

extern "C" __attribute__((visibility("default"))) const char* bbm_last_error(void) { return bbm::g_err; }
extern "C" __attribute__((visibility("default"))) int bbm_version(void) { return 300; }  // 0.3.0: packed words of all-zero slabs are no longer written; DENSE_BASELINE needs the class bytes; bbm_probe_mfma_bf16 added
