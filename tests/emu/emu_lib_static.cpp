// Host build of the library (lock-step emulation): the execute call whose scratch is part of the library.
#define TT_HOST_EMULATION 1
#include "static_scratch.hip"
