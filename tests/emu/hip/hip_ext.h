// the extension header of the model: everything lives in hip_runtime.h
#pragma once
#include "hip_runtime.h"
