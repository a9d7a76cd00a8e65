#define DLC_S 64
#include "dlc_fused_impl.h"
