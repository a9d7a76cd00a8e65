#define DLC_S 256
#include "dlc_carry_impl.h"
