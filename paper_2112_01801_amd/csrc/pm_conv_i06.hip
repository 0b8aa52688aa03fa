// conv_rows instances: bf16, B_NORMAL, X_DIRECT
#include "pm_conv_kernel.h"
PM_CONV_INSTANCE(1, B_NORMAL, X_DIRECT)
