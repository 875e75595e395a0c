// placeholder until the decoder kernels land
#include "internal.h"
rv_status rv_dec_plan(rv_stage*) { return RV_E_INVAL; }
void rv_dec_free(rv_stage*) {}
rv_status rv_dec_forward(rv_stage*, rv_slot&, const void*, void*) { return RV_E_INVAL; }
rv_status rv_dec_backward(rv_stage*, rv_slot&, const void*, void*) { return RV_E_INVAL; }
