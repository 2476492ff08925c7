// Arguments of the register-tiled partition DP kernel (L <= 128).
#pragma once

#include "pp_common.h"

#define DPT_THREADS 256

struct dp_tile_args {
    int L, D, S, K;
    long long N;
    long long chunk;               // consecutive candidates walked by one wave
    unsigned long long fit_limit;  // keys are usable iff hdr->vmax < fit_limit
    int validate;                  // orderings came from the caller: check them
    const pp_ws_header *hdr;
    const int *p32;   // P[min(l, L)] for l = 0..8*NT
    const int *xkt;   // [link][b][j] keys ((XF+XB) << K) | k for k = 8j+b, infinite if k == 0 or k >= L
    const int *ord;   // [N][S] explicit orderings
    long long *C_out;
    int *bounds_out;
    int32_t *status;
};

// grid workgroups of wpb waves; wave w walks candidates [w*chunk, (w+1)*chunk)
int pp_launch_dp_tile(const dp_tile_args &a, int nt, int grid, int wpb, hipStream_t st);
