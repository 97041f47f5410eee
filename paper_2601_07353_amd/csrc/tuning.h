// Tuning builds only (-DTALON_TUNING): time stamps of the single-launch expansion kernel and
// environment overrides of the launch heuristics.  The default build does not include this
// file: its heuristics are the constants of tuned_int()'s callers and it writes no time stamps.
#pragma once

#include <hip/hip_runtime.h>
#include <stdlib.h>

namespace talon {

#ifdef TALON_TUNING_MARKS   // defined by the one source file that owns the time stamps
// g_tl[d][i]: 100 MHz wall-clock stamps of layer d.  i = 0/1: workgroup 0 enters / leaves the
// layer; 2/3: the workgroup that selects for a sequence starts / has published the selection.
// Row 31: the end of the loop (0) and the end of the masks (1).
__device__ unsigned long long g_tl[32][4];

#define TL_MARK(d, i) do { if (threadIdx.x == 0 && blockIdx.x == 0 && (d) < 32) g_tl[d][i] = wall_clock64(); } while (0)
#define TL_ANY(d, i) do { if (threadIdx.x == 0 && (d) < 32) g_tl[d][i] = wall_clock64(); } while (0)
#endif

inline int tuned_int(const char* name, int dflt) {
  const char* e = getenv(name);
  if (!e) return dflt;
  const int v = atoi(e);
  return v > 0 ? v : dflt;
}

}  // namespace talon

#ifdef TALON_TUNING_MARKS
extern "C" int talon_tuning_read_timeline(unsigned long long* host) {
  return static_cast<int>(hipMemcpyFromSymbol(host, HIP_SYMBOL(talon::g_tl), sizeof(unsigned long long) * 32 * 4));
}
#endif
