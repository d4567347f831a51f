#define UNIT_UNSIGNED_BYTES 1
#define UNIT_LAUNCH_NAME launch_igemm_u8
#include "igemm_launch.inc"
