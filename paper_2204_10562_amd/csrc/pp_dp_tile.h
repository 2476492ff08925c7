// Arguments of the register-tiled partition DP kernel (L <= 128).
#pragma once

#include "pp_common.h"
#include "pp_dp_generic.h"

#define DPT_ARENA_ROWS 64  // backtrack rows a wave keeps before it must write plans out
#define DPT_PENDING 64     // candidates whose plans are written out together (one per lane)

struct dp_tile_args {
    int L, D, S, K;
    long long N;
    long long chunk;  // consecutive candidates walked by one wave
    int validate;     // orderings came from the caller: check them
    int prio_left[3]; // priority k+1 while more than prio_left[k] candidates of the chunk are left
    const int *xkt;   // [link][b][j] keys ((XF+XB) << K) | k for k = 8j+b, infinite if k == 0 or k >= L
    const int *xct;   // [link][a][h][r] the same keys for the cells l = 8(hH+r)+a+1, H = ceil(nt/2)
    dp_args g;        // tables, outputs and the generic fallback's arguments
};

// LDS bytes one wave needs: S key rows, the backtrack arena, the pending candidates' row slots
// and (used by the stage-count search only) the key of cell L of each of their rows.
__host__ __device__ static inline size_t pp_dp_tile_lds_per_wave(int S, int nt) {
    size_t rows = (size_t)S * (8 * nt + 4) * 4;
    size_t arena = (size_t)DPT_ARENA_ROWS * (8 * nt + 4);
    size_t slots = (size_t)DPT_PENDING * S;
    size_t tops = (size_t)DPT_PENDING * S * 4;
    return (rows + arena + slots + tops + 15) & ~(size_t)15;
}

// grid workgroups of wpb waves; wave w walks candidates [w*chunk, (w+1)*chunk)
int pp_launch_dp_tile(const dp_tile_args &a, int nt, int grid, int wpb, hipStream_t st);
