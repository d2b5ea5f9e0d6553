#include "lot_internal.h"
namespace lot {
int run_fused(const Args&, bool) { return LOT_ERR_PATH; }
}
