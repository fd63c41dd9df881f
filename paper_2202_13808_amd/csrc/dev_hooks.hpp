// Development-only instrumentation of the DropIT gfx950 library, in one place.
// The shipped library is built WITHOUT -DDROPIT_DEV: every hook below is then an empty statement or
// a constant, no environment variable is read and no kernel carries a time stamp.  A development
// build (-DDROPIT_DEV) gets
//   DROPIT_DEV_STAMP(p, i, cond)  p[i] = the 100 MHz wall clock, in the threads where cond holds
//   dev_env(name, dflt)           an integer override from the environment (tuning sweeps)
#pragma once

#ifdef DROPIT_DEV
#include <cstdlib>
#define DROPIT_DEV_STAMP(p, i, cond) do { if (cond) (p)[i] = wall_clock64(); } while (0)
namespace dropit {
inline long dev_env(const char *name, long dflt)
{
    const char *e = std::getenv(name);
    return e ? std::atol(e) : dflt;
}
}  // namespace dropit
#else
#define DROPIT_DEV_STAMP(p, i, cond) do { } while (0)
namespace dropit {
constexpr long dev_env(const char *, long dflt) { return dflt; }
}  // namespace dropit
#endif
