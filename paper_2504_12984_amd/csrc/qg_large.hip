// placeholder until the tiled kernel lands
#include "qg_common.h"
#ifndef QG_WT
#error "compile with -DQG_WT=<weight type index>"
#endif
namespace qg {
#define QG_CAT2(a, b) a##b
#define QG_CAT(a, b) QG_CAT2(a, b)
int QG_CAT(large_launch_wt, QG_WT)(const GemmParams&, int, int, hipStream_t) { return QG_EUNSUPPORTED; }
}
