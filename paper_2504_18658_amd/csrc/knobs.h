// Diagnostic switches of the library (kernel choice, block shapes, launch limits, checked
// mode).  They exist for tests and for A/B runs under a profiler; nothing in normal use sets
// them.  The PCCL_* environment variables are read ONCE, when the library is loaded, into the
// structure below; a launch only reads the structure.  pccl_diag_reload_env() reads them again
// (tests change a variable, reload, call, restore, reload).
#pragma once
#include <cstddef>

namespace pccl {

struct Knobs {
  int two_level_kernel;    // PCCL_FORCE_TWO_LEVEL_KERNEL: 0 chooser, 1 "stream", 2 "lds"
  int two_level_waves;     // PCCL_TWO_LEVEL_WAVES: 0 chooser, else 4 / 8 / 16 wavefronts per block
  int flat_kernel;         // PCCL_FORCE_FLAT_KERNEL: 0 chooser, 1 "stream", 2 "two-level", 3 "flat"
  int flat_waves;          // PCCL_FLAT_WAVES: 0 chooser, else 4 / 8 / 16
  int flat_local;          // PCCL_FLAT_LOCAL: 1 (default) XCD-major slices and cached loads, 0 neither
  int permute_order;       // PCCL_PERMUTE_ORDER: 0 chooser, 1 "dst", 2 "src"
  long long permute_skew;  // PCCL_PERMUTE_SKEW: -1 chooser, else tiles
  int share_launches;      // PCCL_SHARE_LAUNCHES: 0 one launch for both phases of a share where that is faster, 1: wherever that form exists, 2: one per phase
  int two_level_npt;       // PCCL_TWO_LEVEL_NPT: 0 default; 4: four nodes per wavefront and tile where the default is eight
  int two_level_pipe;      // PCCL_TWO_LEVEL_PIPE: 1 (default) loads kept in flight across tile boundaries where the shape allows, 0 the plain loop
  size_t grid_x_limit;     // PCCL_GRID_X_LIMIT: 0 = the hardware's, else work-items in x
  int check_pointers;      // PCCL_CHECK_POINTERS: 0 off, 1 ranges, 2 also device-resident tables
  int step_launches;         // PCCL_STEP_LAUNCHES: 0 one launch for a whole replay, 1 one launch per step
};

const Knobs& knobs();

}  // namespace pccl
