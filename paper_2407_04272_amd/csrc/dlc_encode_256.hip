#define DLC_S 256
#include "dlc_encode_impl.h"
