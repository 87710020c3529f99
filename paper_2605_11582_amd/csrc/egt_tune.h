// Developer tuning knobs of the launchers (tiles per wave, waves per workgroup, a path
// switched off for A/B timing).  They exist only in a build with -DEGT_TUNE, which reads
// them from the environment at every launch; the ordinary build compiles them out, so the
// library reads no environment and keeps no state.  Every launcher clamps what it gets to
// the range its kernels were instantiated for: a bad value changes the launch shape, never
// the result, and never turns a valid call into an error.
//
//   EGT_M1_TUNE=tpi,wpp      2:4 M = 1            EGT_M1N1_TUNE=tpi,wpp    1:4 M = 1
//   EGT_M1T_TUNE=tpi,wpp     several-token form   EGT_DENSE_TUNE=tpi,wpp   dense INT4
//   EGT_SM_TUNE=waves,blocks_per_cu   small M     EGT_READ_TUNE=unroll,blocks_per_cu  streaming read
//   EGT_STACK_TUNE=waves,tpi_mode  EGT_STREAM_TUNE=force,blocks_per_cu  EGT_STREAM_WAVES=waves  EGT_STREAM_ITEM=kilobytes
//   EGT_SM_KS=slices,row_blocks    (multi-matrix launches; K split at small M)
//   EGT_NO_M1T, EGT_M1_NOLIN, EGT_M1N1_NOLIN, EGT_M1_NOONE, EGT_M1_NOEVEN, EGT_SM_NOXS   (set = that path is not used)
//   EGT_SM_XS   (set = the small-M form with X held in LDS wherever it applies, not only where it is the faster one)
#ifndef EGT_TUNE_H
#define EGT_TUNE_H

#ifdef EGT_TUNE
#include <cstdio>
#include <cstdlib>
#endif

namespace egt {

inline void tune_pair(const char *name, int &a, int &b) {
#ifdef EGT_TUNE
  if (const char *e = getenv(name)) {
    int ta = a, tb = b;
    if (sscanf(e, "%d,%d", &ta, &tb) >= 1) { a = ta; b = tb; }
  }
#else
  (void)name; (void)a; (void)b;
#endif
}

inline bool tune_flag(const char *name) {
#ifdef EGT_TUNE
  return getenv(name) != nullptr;
#else
  (void)name;
  return false;
#endif
}

}  // namespace egt
#endif
