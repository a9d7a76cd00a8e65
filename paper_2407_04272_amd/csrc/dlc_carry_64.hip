#define DLC_S 64
#include "dlc_carry_impl.h"
