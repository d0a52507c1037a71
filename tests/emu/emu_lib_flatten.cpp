// Host build of the library (lock-step emulation): the convolution <-> fully-connected layout conversion.
#define TT_HOST_EMULATION 1
#include "flatten.hip"
