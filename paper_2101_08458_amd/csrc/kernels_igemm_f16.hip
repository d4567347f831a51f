#define UNIT_DT 1
#define UNIT_LAUNCH_NAME launch_igemm_f16
#include "igemm_launch.inc"
