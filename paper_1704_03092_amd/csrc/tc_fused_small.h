// The fused kernel in its small geometry (128 x 64 tiles, 256 threads, two workgroups per compute unit): namespace
// tc::fused_small.  See tc_fused_body.h.
#pragma once
#define TC_GEO_SMALL 1
#include "tc_fused_body.h"
#undef TC_GEO_SMALL
