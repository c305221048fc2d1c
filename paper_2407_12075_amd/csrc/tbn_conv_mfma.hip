#include "tbn_common.h"
namespace tbn {
bool conv_mfma_supported(const ConvArgs &) { return false; }
tbn_status launch_conv_mfma(const ConvArgs &) { set_error("not built"); return TBN_ERR_UNSUPPORTED; }
}
