#define UNIT_DT 2
#define UNIT_EPI_RQ EPI_RAW
#define UNIT_LAUNCH_NAME launch_igemm_bf16
#include "igemm_launch.inc"
