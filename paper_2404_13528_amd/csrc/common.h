// Host-side helpers shared by the C-ABI translation units.
#pragma once
#include <cstdarg>
#include <cstdio>
#include <string>
#include "../../include/smartmem.h"

namespace sm {
void set_error(const char* fmt, ...);
int fail(int code, const char* fmt, ...);
inline size_t dtype_size(int dtype) { return dtype == SM_F32 ? 4 : 2; }
inline bool dtype_ok(int dtype) { return dtype == SM_F32 || dtype == SM_BF16; }
inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }
// launch bookkeeping for sm_last_launch_counts
void count_reset();
void count_compute(int n = 1);
void count_copy(int n = 1);
const char* last_error();
int counts(int* a, int* b);
// Optional per-kernel timing: when enabled, every launch made through Timed is bracketed by two
// events on its stream; sm_timing_report sums them per label.
int timing_enable(int on);
int timing_report(char* buf, int n);
int timing_sequence(char* buf, int n);      // the labels of the recorded launches in launch order, one per line
struct Timed {
  Timed(const char* label, void* stream);
  ~Timed();
  void* stream_; int slot_;
};
}  // namespace sm
