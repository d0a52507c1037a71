// What `#include <hip/hip_runtime.h>` finds in the host emulation build of the library's sources.
#pragma once
#include "../emu_device.h"
