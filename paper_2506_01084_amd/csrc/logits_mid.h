// The base part of extended_logits on the weight-streaming kernel (up to 192 hidden rows; logits_mid.hip): one
// part per tile of 256 weight rows, z2z_logits_mid_tiles(w_rows) of them; `a` carries H, rows, d, the part arrays,
// n_parts and part0.
#pragma once

#include "logits_common.h"

int z2z_logits_mid_prepare(z2z_ctx* c);
bool z2z_logits_mid_ok(const z2z_ctx* c, int rows);
int z2z_logits_mid_tiles(int w_rows);
int z2z_launch_logits_mid(z2z_ctx* c, z2z_logits::LogitsArgs a, const void* W, int w_rows, int col0, hipStream_t s);

// a dense layer on R <= 128 rows: ksplit fp32 partial tiles [ksplit][R][N] into `partial` (see logits_mid.hip)
int z2z_launch_linear_mid(z2z_ctx* c, const void* A, const void* W, int R, const int32_t* rows_dev, int N, int K,
                          float* partial, size_t partial_floats, int* ksplit_out, hipStream_t s);
int z2z_linear_mid_ksplit(int N, int K);
