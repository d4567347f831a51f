#define UNIT_DT 5
#define UNIT_EPI_RQ EPI_RAW
#define UNIT_TILES_DEF "tiles_fp8.def"
#define UNIT_LAUNCH_NAME launch_igemm_fp8
#include "igemm_launch.inc"
