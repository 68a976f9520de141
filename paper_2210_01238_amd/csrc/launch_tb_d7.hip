#define JK_TB_DEPTH 7
#define JK_TB_MINW_F64 3
#define JK_TB_MINW_F32 2
#include "launch_tb.inc.h"
