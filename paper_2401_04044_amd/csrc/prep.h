// Internal: launchers of the packing / reduction kernels (prep.hip) and of the
// heavy-hitter selection (select.hip).
#pragma once
#include "common.h"

namespace ffsplit {

// dst[f(n)][coff + c] = src[cmap(c)][nmap(n)] for n < n_count, c < c_count, where
// f(n) = row_off + n                         (glu_mode 0)
//      = row_off + (n/32)*64 + n%32 (+32)    (glu_mode 1 gate / 2 up: interleaved 32-row blocks)
// nmap / cmap NULL = identity; *_off is added to the map index.
struct PermArgs {
  const void* src;
  int64_t lds;
  void* dst;
  int64_t ldd;
  int n_count, c_count;
  const int32_t* nmap;
  int nmap_off;
  const int32_t* cmap;
  int cmap_off;
  int coff;
  int64_t row_off;
  int glu_mode;
  int dst_tiled;   // dst in the 32x16-block tiled layout of gemm_bf16.hip, ldd = padded K
};

int launch_fill_zero(void* p, size_t bytes, hipStream_t st);
int launch_permute_transpose(const PermArgs& a, int esize, hipStream_t st);
int launch_reduce_partials(const float* p2, const float* p1, int tiles, int n_out, int d_ff, float* acc,
                           hipStream_t st);
int launch_finalize_scores(const void* W2, int bf16, int d_model, int d_ff, const float* acc, float t_total,
                           int kind, float* scores, hipStream_t st);

// per-token RMS normalisation of an fp32 stream into bf16 or fp32 (the pre-norm of a layer stack)
int launch_token_rmsnorm(const float* x, int64_t T, int d, float eps, int bf16, void* out, hipStream_t st);
// a layer's neuron biases in the packed split's neuron order, fp32, zero on the padding
int launch_pack_neuron_bias(const void* b1, int bf16, const int32_t* idx, const int32_t* rest, int k, int kp, int m,
                            int mp, float* out, hipStream_t st);

// select.hip
size_t select_workspace_bytes(int d_ff);
int launch_select(const float* scores, int d_ff, int k, int32_t* idx, int32_t* perm, int32_t* nan_flag,
                  void* ws, hipStream_t st);
// the same on the library's own static device scratch (d_ff <= select_static_max_dff())
int select_static_max_dff();
int launch_select_static(const float* scores, int d_ff, int k, int32_t* idx, int32_t* perm, int32_t* nan_flag,
                         hipStream_t st);

}  // namespace ffsplit
