#define DLC_S 128
#include "dlc_carry_impl.h"
