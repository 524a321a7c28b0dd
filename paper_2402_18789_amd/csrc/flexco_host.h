// Error reporting and small helpers shared by every source of the library.  No device headers: the host-only
// sources (index maps, scheduler, graph pruning) include this file alone, so they also build with a plain C++
// compiler, e.g. under the host sanitizers.
#pragma once
#include <stdint.h>
#include <stddef.h>

#include "flexco.h"

namespace flexco {

int32_t fail(int32_t code, const char* fmt, ...);
void clear_error();

#define FLEXCO_CHECK(cond, code, ...) \
  do { if (!(cond)) return ::flexco::fail((code), __VA_ARGS__); } while (0)
#define FLEXCO_TRY(expr) \
  do { int32_t rc_ = (expr); if (rc_ != FLEXCO_OK) return rc_; } while (0)

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline size_t esize(int dtype) { return dtype == FLEXCO_BF16 ? 2 : 4; }
inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

}  // namespace flexco
