// conv_rows instances: bf16, B_ONE, X_GATHER_CAT
#include "pm_conv_kernel.h"
PM_CONV_INSTANCE(1, B_ONE, X_GATHER_CAT)
