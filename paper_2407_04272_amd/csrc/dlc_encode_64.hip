#define DLC_S 64
#include "dlc_encode_impl.h"
