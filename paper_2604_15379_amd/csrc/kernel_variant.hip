// One flavour of the persistent kernel (both cache layouts) per translation unit: compiled
// with -DFLEET_VARIANT=<0..6>, so that the build compiles the flavours in parallel.
// fleet.hip declares these instantiations extern and takes their addresses.
#include <hip/hip_runtime.h>

#include "../../include/fleet.h"
#include "graph.hpp"
#include "kernels.hip.inc"

#ifndef FLEET_VARIANT
#error "compile with -DFLEET_VARIANT=<0..6>"
#endif

template __global__ void fleet_persistent_kernel<FLEET_VARIANT, false>(dev::Params);
template __global__ void fleet_persistent_kernel<FLEET_VARIANT, true>(dev::Params);
