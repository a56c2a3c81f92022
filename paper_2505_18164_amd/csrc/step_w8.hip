// The persistent decode step for workgroups of 8 wavefronts (one workgroup per compute unit): launches that carry one
// message (k_step), launches that take several messages through one pass over the weights (k_step_batch), and the
// output layers (k_logits for one sample, k_logits_batch for several).
#define MDI_STEP_WAVES 8
#include "step_impl.h"
#include "step_batch.h"
#include "head_batch.h"
