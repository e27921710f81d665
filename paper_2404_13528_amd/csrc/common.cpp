#include "common.h"
#include <cstring>
#include <map>
#include <mutex>
#include <vector>
#include <hip/hip_runtime_api.h>

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

namespace {
struct Rec { std::string label; hipEvent_t a, b; };
std::mutex t_mu;
bool t_on = false;
std::vector<Rec> t_recs;
}
Timed::Timed(const char* label, void* stream) : stream_(stream), slot_(-1) {
  if (!t_on) return;
  std::lock_guard<std::mutex> lock(t_mu);
  Rec r; r.label = label;
  if (hipEventCreate(&r.a) != hipSuccess || hipEventCreate(&r.b) != hipSuccess) return;
  (void)hipEventRecord(r.a, (hipStream_t)stream);
  t_recs.push_back(r);
  slot_ = (int)t_recs.size() - 1;
}
Timed::~Timed() {
  if (slot_ < 0) return;
  std::lock_guard<std::mutex> lock(t_mu);
  (void)hipEventRecord(t_recs[slot_].b, (hipStream_t)stream_);
}
int timing_enable(int on) {
  std::lock_guard<std::mutex> lock(t_mu);
  for (auto& r : t_recs) { (void)hipEventDestroy(r.a); (void)hipEventDestroy(r.b); }
  t_recs.clear();
  t_on = on != 0;
  return SM_OK;
}
int timing_report(char* buf, int n) {
  std::lock_guard<std::mutex> lock(t_mu);
  std::map<std::string, std::pair<int, double>> agg;
  std::vector<std::string> order;
  for (auto& r : t_recs) {
    if (hipEventSynchronize(r.b) != hipSuccess) return fail(SM_ERR_DEVICE, "sm_timing_report: event synchronisation failed");
    float ms = 0.f;
    if (hipEventElapsedTime(&ms, r.a, r.b) != hipSuccess) return fail(SM_ERR_DEVICE, "sm_timing_report: elapsed time failed");
    if (!agg.count(r.label)) order.push_back(r.label);
    agg[r.label].first += 1; agg[r.label].second += ms;
  }
  std::string out;
  for (auto& l : order) {
    char line[256];
    snprintf(line, sizeof(line), "%s\t%d\t%.6f\n", l.c_str(), agg[l].first, agg[l].second);
    out += line;
  }
  if ((int)out.size() + 1 > n) return fail(SM_ERR_INVALID_ARG, "sm_timing_report: buffer of %d bytes, %zu needed", n, out.size() + 1);
  std::memcpy(buf, out.c_str(), out.size() + 1);
  return SM_OK;
}
int timing_sequence(char* buf, int n) {
  std::lock_guard<std::mutex> lock(t_mu);
  std::string out;
  for (auto& r : t_recs) { out += r.label; out += '\n'; }
  if ((int)out.size() + 1 > n) return fail(SM_ERR_INVALID_ARG, "sm_timing_sequence: buffer of %d bytes, %zu needed", n, out.size() + 1);
  std::memcpy(buf, out.c_str(), out.size() + 1);
  return SM_OK;
}
}  // namespace sm

extern "C" const char* sm_last_error(void) { return sm::last_error(); }
extern "C" int sm_abi_version(void) { return 1; }
extern "C" int sm_last_launch_counts(int* n_compute, int* n_copy) { return sm::counts(n_compute, n_copy); }
extern "C" int sm_timing_enable(int on) { return sm::timing_enable(on); }
extern "C" int sm_timing_sequence(char* buf, int n) { if (!buf || n < 1) return sm::fail(SM_ERR_INVALID_ARG, "sm_timing_sequence: bad buffer"); return sm::timing_sequence(buf, n); }
extern "C" int sm_timing_report(char* buf, int n) { if (!buf || n < 1) return sm::fail(SM_ERR_INVALID_ARG, "sm_timing_report: bad buffer"); return sm::timing_report(buf, n); }
