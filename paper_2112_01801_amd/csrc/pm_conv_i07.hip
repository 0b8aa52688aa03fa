// conv_rows instances: bf16, B_NORMAL, X_GATHER_SUM
#include "pm_conv_kernel.h"
PM_CONV_INSTANCE(1, B_NORMAL, X_GATHER_SUM)
