#define UNIT_DT 0
#define UNIT_LAUNCH_NAME launch_igemm_i8
#include "igemm_launch.inc"
