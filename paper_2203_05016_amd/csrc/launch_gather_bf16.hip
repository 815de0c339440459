// Gather-kernel launchers for bfloat16 operands.
#define SHFLBW_LAUNCH_BF true
#define SHFLBW_LAUNCH_NAME run_gather_bf16
#define SHFLBW_LAUNCH_OUT16 __bf16
#include "launch_gather.inc"
