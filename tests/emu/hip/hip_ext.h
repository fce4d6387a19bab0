// Host emulation of the HIP pieces libdgs uses: everything is in hip_runtime.h.
#pragma once
#include "hip_runtime.h"
