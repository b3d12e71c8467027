// The dispatcher's tuning overrides: read from the environment once, replaced as a
// whole by mipgemm_set_tuning.  Host only.
#include "tuning.h"

#include <atomic>
#include <cstdlib>
#include <cstring>
#include <mutex>

#include "../../include/mipgemm.h"

namespace mip {

namespace {

std::atomic<const Tuning *> g_current{nullptr};
std::mutex g_writer;  // serialises writers; readers only load the pointer

bool apply(Tuning *t, const char *name, const char *value) {
  const char *v = value ? value : "";
  if (!std::strcmp(name, "MIPGEMM_VARIANT")) {
    if (std::strlen(v) >= sizeof(t->variant)) return false;
    std::strcpy(t->variant, v);
    return true;
  }
  if (!std::strcmp(name, "MIPGEMM_SPLITK")) {
    const int n = std::atoi(v);
    if (*v && n < 0) return false;
    t->splitk = n > 0 ? n : 0;
    return true;
  }
  if (!std::strcmp(name, "MIPGEMM_PACK")) {
    if (!*v) t->pack = 0;
    else if (!std::strcmp(v, "always")) t->pack = 1;
    else if (!std::strcmp(v, "never")) t->pack = -1;
    else return false;
    return true;
  }
  if (!std::strcmp(name, "MIPGEMM_STAGGER")) {
    const int n = std::atoi(v);
    if (*v && (n < 0 || n > 100000)) return false;
    t->stagger = *v ? n : -1;
    return true;
  }
  if (!std::strcmp(name, "MIPGEMM_CONV")) {
    if (!*v) t->conv = 0;
    else if (!std::strcmp(v, "im2col")) t->conv = 1;
    else if (!std::strcmp(v, "rows")) t->conv = 2;
    else return false;
    return true;
  }
  return false;
}

const Tuning *from_environment() {
  Tuning *t = new Tuning();
  for (const char *name : {"MIPGEMM_VARIANT", "MIPGEMM_SPLITK", "MIPGEMM_PACK", "MIPGEMM_CONV", "MIPGEMM_STAGGER"})
    if (const char *v = std::getenv(name)) (void)apply(t, name, v);  // an unparsable value is ignored
  return t;
}

}  // namespace

const Tuning &tuning() {
  const Tuning *t = g_current.load(std::memory_order_acquire);
  if (t) return *t;
  std::lock_guard<std::mutex> lock(g_writer);
  t = g_current.load(std::memory_order_acquire);
  if (!t) {
    t = from_environment();
    g_current.store(t, std::memory_order_release);
  }
  return *t;
}

bool set_tuning(const char *name, const char *value) {
  if (!name) return false;
  const Tuning &old = tuning();
  std::lock_guard<std::mutex> lock(g_writer);
  // Sets are few (tests, tuning scripts) and a call in flight may still read the old one:
  // superseded sets are kept for the life of the process rather than freed.
  Tuning *t = new Tuning(*g_current.load(std::memory_order_acquire));
  (void)old;
  if (!apply(t, name, value)) {
    delete t;
    return false;
  }
  g_current.store(t, std::memory_order_release);
  return true;
}

}  // namespace mip

extern "C" int mipgemm_set_tuning(const char *name, const char *value) {
  return mip::set_tuning(name, value) ? 0 : -1;
}
