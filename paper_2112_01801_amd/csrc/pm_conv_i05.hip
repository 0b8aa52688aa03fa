// conv_rows instances: fp32, B_ONE, X_GATHER_CAT
#include "pm_conv_kernel.h"
PM_CONV_INSTANCE(0, B_ONE, X_GATHER_CAT)
