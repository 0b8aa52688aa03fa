// conv_rows instances: fp32, B_DIRS, X_DIRECT
#include "pm_conv_kernel.h"
PM_CONV_INSTANCE(0, B_DIRS, X_DIRECT)
