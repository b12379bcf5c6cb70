// Instantiation of the LDS-tile kernels of the tree phase (tier, list and retry kernels)
// for one value type and operator, all compile-time group widths; a file of its
// own so that the instantiations compile in parallel.
#include "ftred_fused.h"
#include "ftred_kernels.h"
#include "ftred_shape.h"
#include "ftred_wave.h"
#include "ftred_wave_general.h"
#include "ftred_wave_unit.h"

namespace ftred {
FTRED_DEFINE_LAUNCHERS(u32_sum, uint32_t, 0)
FTRED_DEFINE_SHAPE_LAUNCHER(u32_sum, uint32_t, 0)
}  // namespace ftred
