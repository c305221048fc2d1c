#include "tbn_common.h"
namespace tbn {
bool linear_rows_supported(const LinearArgs &) { return false; }
tbn_status launch_linear_rows(const LinearArgs &) { set_error("not built"); return TBN_ERR_UNSUPPORTED; }
}
