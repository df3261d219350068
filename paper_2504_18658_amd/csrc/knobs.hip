// Host-only: the diagnostic switches, read from the environment when the library is loaded.
#include "knobs.h"

#include <cstdlib>

#include "../../include/pccl_local.h"

namespace pccl {

namespace {

Knobs read_env() {
  Knobs k;
  const char* v;
  k.two_level_kernel = 0;
  if ((v = std::getenv("PCCL_FORCE_TWO_LEVEL_KERNEL"))) k.two_level_kernel = v[0] == 's' ? 1 : v[0] == 'l' ? 2 : 0;
  k.two_level_waves = 0;
  if ((v = std::getenv("PCCL_TWO_LEVEL_WAVES"))) {
    const int w = std::atoi(v);
    if (w == 4 || w == 8 || w == 16) k.two_level_waves = w;
  }
  k.flat_kernel = 0;
  if ((v = std::getenv("PCCL_FORCE_FLAT_KERNEL"))) k.flat_kernel = v[0] == 's' ? 1 : v[0] == 't' ? 2 : v[0] == 'f' ? 3 : 0;
  k.flat_waves = 0;
  if ((v = std::getenv("PCCL_FLAT_WAVES"))) {
    const int w = std::atoi(v);
    if (w == 4 || w == 8 || w == 16) k.flat_waves = w;
  }
  k.flat_local = 1;
  if ((v = std::getenv("PCCL_FLAT_LOCAL"))) k.flat_local = v[0] != '0';
  k.permute_order = 0;
  if ((v = std::getenv("PCCL_PERMUTE_ORDER"))) k.permute_order = v[0] == 's' ? 2 : 1;
  k.permute_skew = -1;
  if ((v = std::getenv("PCCL_PERMUTE_SKEW"))) {
    const long long t = std::atoll(v);
    if (t >= 0 && t <= 0xFFFFFFFFll) k.permute_skew = t;
  }
  k.share_launches = 0;
  if ((v = std::getenv("PCCL_SHARE_LAUNCHES"))) k.share_launches = v[0] == '2' ? 2 : v[0] == '1' ? 1 : 0;
  k.two_level_npt = 0;
  if ((v = std::getenv("PCCL_TWO_LEVEL_NPT"))) {
    const int w = std::atoi(v);
    if (w == 4 || w == 8) k.two_level_npt = w;
  }
  k.two_level_pipe = 1;
  if ((v = std::getenv("PCCL_TWO_LEVEL_PIPE"))) k.two_level_pipe = v[0] != '0';
  k.grid_x_limit = 0;
  if ((v = std::getenv("PCCL_GRID_X_LIMIT"))) {
    const long long t = std::atoll(v);
    if (t > 0) k.grid_x_limit = (size_t)t;
  }
  k.check_pointers = 0;
  if ((v = std::getenv("PCCL_CHECK_POINTERS")) && v[0] != '\0' && v[0] != '0') k.check_pointers = v[0] == '2' ? 2 : 1;
  k.step_launches = 0;
  if ((v = std::getenv("PCCL_STEP_LAUNCHES"))) k.step_launches = v[0] == '1';
  return k;
}

Knobs g_knobs = read_env();  // runs when the library is loaded

}  // namespace

const Knobs& knobs() { return g_knobs; }

}  // namespace pccl

extern "C" void pccl_diag_reload_env(void) { pccl::g_knobs = pccl::read_env(); }

// Identity of the sources this library was built from (the build script hashes them and passes
// the hash in); the binding compares it with the sources on disk before it loads the library.
#ifndef PCCL_BUILD_ID
#define PCCL_BUILD_ID "unknown"
#endif
extern "C" const char* pccl_build_id(void) {
  static const char id[] = "pccl-build-id:" PCCL_BUILD_ID;
  return id + sizeof("pccl-build-id:") - 1;
}
