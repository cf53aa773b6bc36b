// Tile path placeholder: routes to the gather kernels until the MFMA tile kernels land.
#include "sga_internal.h"

namespace sga {

sga_status launch_tile_explicit(const AttnArgs& a) { return launch_gather_explicit(a, true, nullptr); }
sga_status launch_tile_implicit(const AttnArgs& a) { return launch_gather_implicit(a); }

}  // namespace sga
