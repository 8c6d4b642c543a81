// Internal: the 8-bit heavy / 3-bit remainder split (Sec. 5.2, the setting for the LLMs).
#pragma once
#include "common.h"
#include "layout.h"

namespace ffsplit {

// rest: remainder neurons ascending; idx: heavy neurons in the caller's order
int launch_w3h8_pack(const ffsplit_desc_t& d, const Layout& L, const void* W1, const void* Wg, const void* W2,
                     const int32_t* rest, const int32_t* idx, char* split, hipStream_t st);
// what: 0..2 remainder W1 / Wg / W2, 3..5 heavy likewise
int launch_w3h8_export(const ffsplit_desc_t& d, const Layout& L, const char* split, int what, int8_t* q_out,
                       uint16_t* s_out, hipStream_t st);
// bf16 image of the split in the DENSE layout LD (tiled): every weight bf16(float(s) * q)
int launch_w3h8_expand(const ffsplit_desc_t& d, const Layout& L, const Layout& LD, const char* split, char* image,
                       hipStream_t st);

// forward for at most 32 tokens (one pass): the packed codes are streamed once per product
// (weight-streaming kernels of skinny.hip), scratch laid out by make_fwd_ws
int w3h8_forward_small(const ffsplit_desc_t& d, const Layout& L, const FwdWs& w, const char* split, const void* X,
                       int M, void* Y, void* Y_heavy, void* Y_rem, const Epilogue& ep, char* ws, hipStream_t st);

}  // namespace ffsplit
