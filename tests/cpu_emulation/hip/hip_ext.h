// stand-in: the extended launch is declared in hip_runtime.h of this directory
#pragma once
#include "hip_runtime.h"
