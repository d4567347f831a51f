#define UNIT_DT 1
#define UNIT_EPI_RQ EPI_RAW   /* fp16 has no requantise epilogue */
#define UNIT_LAUNCH_NAME launch_igemm_f16
#include "igemm_launch.inc"
