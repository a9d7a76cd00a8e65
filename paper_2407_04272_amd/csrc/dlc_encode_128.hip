#define DLC_S 128
#include "dlc_encode_impl.h"
