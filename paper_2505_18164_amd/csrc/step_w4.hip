// The persistent decode step for workgroups of 4 wavefronts (two workgroups per compute unit: launches that carry several messages).
#define MDI_STEP_WAVES 4
#include "step_impl.h"
