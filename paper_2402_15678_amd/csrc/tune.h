// Experiment switches.  A normal build has none: tune_int() returns its default and the compiler folds it
// away.  A build with -DMN_TUNING reads the named environment variable once per call site instead, which
// is how the launch parameters (waves per workgroup, k-splits, attention workgroups, ...) were swept.
#pragma once

#ifdef MN_TUNING
#include <cstdlib>
#endif

namespace mn {

#ifdef MN_TUNING
#define MN_TUNE(NAME, DEFAULT)                       \
  ([]() -> int {                                     \
    static const int v_ = [] {                       \
      const char* e_ = std::getenv(NAME);            \
      return e_ ? std::atoi(e_) : (DEFAULT);         \
    }();                                             \
    return v_;                                       \
  }())
#else
#define MN_TUNE(NAME, DEFAULT) (DEFAULT)
#endif

}  // namespace mn
