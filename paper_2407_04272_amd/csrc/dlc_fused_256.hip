#define DLC_S 256
#include "dlc_fused_impl.h"
