#define DLC_S 128
#include "dlc_fused_impl.h"
