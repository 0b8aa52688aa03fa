// conv_rows instances: bf16, B_DIRS, X_DIRECT
#include "pm_conv_kernel.h"
PM_CONV_INSTANCE(1, B_DIRS, X_DIRECT)
