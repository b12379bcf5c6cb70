// Instantiation of the register kernel of the deepest tier for one value per process (eight lanes per subtree)
// for one value type and operator, all compile-time group widths; a file of its
// own so that the instantiations compile in parallel.
#include "ftred_fused.h"
#include "ftred_kernels.h"
#include "ftred_wave.h"
#include "ftred_wave_general.h"
#include "ftred_wave_unit.h"

namespace ftred {
FTRED_DEFINE_UNIT_LAUNCHER(i64_bor, unsigned long long, 1)
}  // namespace ftred
