// Tuning overrides of the dispatcher (tests, tuning runs, profiles): which kernel
// variant, how many k ranges, whether to pack, which convolution route.  The
// environment is read once, at the first call; afterwards the values change only
// through mipgemm_set_tuning, which replaces the set as a whole: a reader never sees
// a half-written one.
#pragma once

namespace mip {

struct Tuning {
  char variant[32] = "";  // MIPGEMM_VARIANT: "" = the dispatcher decides
  int splitk = 0;         // MIPGEMM_SPLITK: 0 = the dispatcher decides
  int pack = 0;           // MIPGEMM_PACK: 0 by size, 1 "always", -1 "never"
  int conv = 0;           // MIPGEMM_CONV: 0 by shape, 1 "im2col", 2 "rows"
  int stagger = -1;       // MIPGEMM_STAGGER: 10 ns ticks between the tile rows of an XCD's patch in the
                          // kernel for large problems; -1 = the built-in value
};

// The current set: immutable, valid for the life of the process.
const Tuning &tuning();

// name: one of the MIPGEMM_* variable names; value: as in the environment, null or "" to clear.
// Returns false for an unknown name or a value that does not parse.
bool set_tuning(const char *name, const char *value);

}  // namespace mip
