// Encoder instantiations whose rotation switch and scaling coefficient are read from the
// configuration at run time (App. "Ablation Study": rotation off, scaling off, scaling by the
// maximum or the mean magnitude).  -ffp-contract=off, as for every user of the encoder header.
#include "oscar_append_kernel.h"

int oscar_launch_append_switched(const AppendParams& P, dim3 grid, hipStream_t st) {
  return launch_append<XF_SWITCHED>(P, grid, st);
}
