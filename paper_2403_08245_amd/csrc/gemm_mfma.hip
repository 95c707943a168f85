#include "common.h"
bool s2s_mfma_supported(const S2SArgs &) { return false; }
bool dw_mfma_supported(const DWArgs &) { return false; }
int launch_s2s_mfma(hipStream_t, const S2SArgs &, int) { return SMOE_ERR_UNSUPPORTED; }
int launch_dw_mfma(hipStream_t, const DWArgs &, int) { return SMOE_ERR_UNSUPPORTED; }
