#include "common.h"
#include <cstring>

namespace sm {
static thread_local char g_err[512] = "";
static thread_local int g_compute = 0, g_copy = 0;

void set_error(const char* fmt, ...) {
  va_list ap; va_start(ap, fmt); vsnprintf(g_err, sizeof(g_err), fmt, ap); va_end(ap);
}
int fail(int code, const char* fmt, ...) {
  va_list ap; va_start(ap, fmt); vsnprintf(g_err, sizeof(g_err), fmt, ap); va_end(ap);
  return code;
}
void count_reset() { g_compute = 0; g_copy = 0; }
void count_compute(int n) { g_compute += n; }
void count_copy(int n) { g_copy += n; }
const char* last_error() { return g_err; }
int counts(int* a, int* b) { if (a) *a = g_compute; if (b) *b = g_copy; return SM_OK; }
}  // namespace sm

extern "C" const char* sm_last_error(void) { return sm::last_error(); }
extern "C" int sm_abi_version(void) { return 1; }
extern "C" int sm_last_launch_counts(int* n_compute, int* n_copy) { return sm::counts(n_compute, n_copy); }
