// Internal: group-wise int4 remainder (Sec. 5.2's round-to-nearest quantiser):
// packing at build time and the weight-streaming decode kernels.
#pragma once
#include "common.h"
#include "layout.h"
#include "prep.h"

namespace ffsplit {

int launch_rest_order(const int32_t* idx, int k, int d_ff, int32_t* rest, int32_t* flags, hipStream_t st);
int launch_int4_pack(const ffsplit_desc_t& d, const Layout& L, const void* W1, const void* Wg, const void* W2,
                     const int32_t* rest, const int32_t* idx, char* split, hipStream_t st);
int launch_int4_export(const ffsplit_desc_t& d, const Layout& L, const char* split, int what, int8_t* q_out,
                       uint16_t* s_out, hipStream_t st);
// bf16 image of an int4 split in the DENSE layout LD (tiled): heavy blocks copied, remainder
// codes times their fp16 group scales, rounded to bf16; padding zero.
int launch_int4_expand(const ffsplit_desc_t& d, const Layout& L, const Layout& LD, const char* split, char* image,
                       hipStream_t st);
int int4_forward(const ffsplit_desc_t& d, const Layout& L, const FwdWs& w, const char* split, const void* X, int M,
                 void* Y, void* Y_heavy, void* Y_rem, const Epilogue& ep, char* ws, hipStream_t st);

}  // namespace ffsplit
