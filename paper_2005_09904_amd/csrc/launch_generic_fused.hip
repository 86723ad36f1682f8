// Generic query kernel, tables built from X in LDS (the fused multiply).
#define BIQ_GENERIC_FUSED true
#define BIQ_GENERIC_NAME launch_query_generic_fused
#include "launch_generic.inc"
