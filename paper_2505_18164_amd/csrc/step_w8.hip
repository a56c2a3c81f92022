// The persistent decode step for workgroups of 8 wavefronts (one workgroup per compute unit: launches that carry one message).
#define MDI_STEP_WAVES 8
#include "step_impl.h"
