#define UNIT_DT 0
#define UNIT_EPI_RQ EPI_REQUANT
#define UNIT_LAUNCH_NAME launch_igemm_i8
#include "igemm_launch.inc"
