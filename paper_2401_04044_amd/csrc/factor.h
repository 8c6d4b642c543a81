// Internal: rank-r factors of the remainder matrices on the device (randomised range finder).
#pragma once
#include "common.h"
#include "layout.h"

namespace ffsplit {

size_t factorize_ws_bytes(const ffsplit_desc_t& d);
// rest: the remainder neurons ascending (device).  factors: host array of the six device
// pointers P1, Q1, Pg, Qg, P2, Q2 in desc.dtype.  ws: factorize_ws_bytes(d) bytes after the
// caller's own prefix.
int launch_factorize(const ffsplit_desc_t& d, const void* W1, const void* Wg, const void* W2, const int32_t* rest,
                     uint32_t seed, void* const* factors, char* ws, hipStream_t st);

}  // namespace ffsplit
