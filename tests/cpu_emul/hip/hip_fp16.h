// Half precision for the host-thread build: everything lives in hip_runtime.h.
#pragma once
#include <hip/hip_runtime.h>
