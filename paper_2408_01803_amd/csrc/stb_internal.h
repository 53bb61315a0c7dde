// Declarations shared by the host and device translation units of libstb (not part of the public ABI).
#ifndef STB_INTERNAL_H
#define STB_INTERNAL_H
#include "stb.h"

#ifdef __cplusplus
extern "C" {
#endif
// STB_OK iff the size fields agree with the closed form for L->cfg and every required plane pointer is
// set and 16-byte aligned.
int stb_layout_check(const stb_layout_t* L);
#ifdef __cplusplus
}
#endif
#endif
