// The fused kernel in its standard geometry (128 x 128 tiles, 512 threads): namespace tc::fused.  See tc_fused_body.h.
#pragma once
#define TC_GEO_SMALL 0
#include "tc_fused_body.h"
#undef TC_GEO_SMALL
