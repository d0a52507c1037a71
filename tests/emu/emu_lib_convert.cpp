// Host build of the library (lock-step emulation): the retile / gate / reduce kernels and their launch code.
#define TT_HOST_EMULATION 1
#include "convert.hip"
