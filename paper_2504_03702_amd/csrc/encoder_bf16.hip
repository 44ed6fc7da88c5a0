// placeholder until the MFMA kernels land
#include "internal.h"
void run_encoder_bf16(const ps_model*, int32_t, const Workspace&, hipStream_t) {}
