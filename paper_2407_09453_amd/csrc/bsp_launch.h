// Internal launch entry points, one per kernel family.  Each returns a bsp_status.
#ifndef BSP_LAUNCH_H
#define BSP_LAUNCH_H

#include <hip/hip_runtime.h>

#include "bsp.h"
#include "bsp_device.h"

int bsp_launch_general(const ConvParams& p, int dtype, int bo, int bi, hipStream_t st);

#endif
