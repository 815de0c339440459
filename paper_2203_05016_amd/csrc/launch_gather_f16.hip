// Gather-kernel launchers for binary16 operands.
#define SHFLBW_LAUNCH_BF false
#define SHFLBW_LAUNCH_NAME run_gather_f16
#define SHFLBW_LAUNCH_OUT16 _Float16
#include "launch_gather.inc"
