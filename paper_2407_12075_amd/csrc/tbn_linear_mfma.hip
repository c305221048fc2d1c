#include "tbn_common.h"
namespace tbn {
bool linear_mfma_supported(const LinearArgs &) { return false; }
tbn_status launch_linear_mfma(const LinearArgs &) { set_error("not built"); return TBN_ERR_UNSUPPORTED; }
}
