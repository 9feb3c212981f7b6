/*
 * signmuon_debug.h -- host-side check hooks of libsignmuon (no GPU work, no context).
 *
 * They expose two pieces of host logic of the Newton-Schulz path (Alg. PolarNS) so that
 * tests can check them without a device: how a grouped GEMM launch deals its output
 * tiles to the eight XCDs, the order in which a matrix's tiles are listed, and the coefficients of the two-steps-at-a-time form of the
 * cubic iteration.  Not part of the optimizer path.
 */
#ifndef SIGNMUON_DEBUG_H
#define SIGNMUON_DEBUG_H

#ifdef __cplusplus
extern "C" {
#endif

/* Tile bookkeeping of one grouped GEMM launch over n_prob problems (HOST arrays of
 * length n_prob: M, N, K, batch, and mate = index of a second problem dealt together
 * with this one, or 0; mate may be NULL).  sym != 0: symmetric outputs (upper triangle of
 * tiles only).  ts: tile size, 128 or 256.  Fills xcd_begin[9] (XCD x owns tiles
 * [xcd_begin[x], xcd_begin[x+1]) of the launch's tile list) and tile_begin[n_prob].
 * Returns the total number of tiles, or -1 on bad arguments. */
int signmuon_debug_tile_ranges(int n_prob, const int* M, const int* N, const int* K, const int* batch,
                               const int* mate, int sym, int ts, int* xcd_begin, int* tile_begin);

/* Entry t of the tile list of one matrix whose output is a tiles_m x tiles_n grid of ts-wide
 * tiles (ts = 128 or 256), as the GEMM kernels decode it; sym != 0: square grid, only tiles
 * with tile_m <= tile_n are listed, t < tiles_m (tiles_m + 1) / 2.  The list runs through bands of
 * 4 (ts = 256) or 8 (ts = 128) tile rows, column by column inside a band, so that the tiles an
 * XCD works on at one time share operand panels.  Writes *tile_m, *tile_n (HOST pointers);
 * returns 0, or -1 on bad arguments (t out of range included). */
int signmuon_debug_tile_of(int t, int tiles_m, int tiles_n, int sym, int ts, int* tile_m, int* tile_n);

/* out5 = {h, u, b^4, g, a^2} with (a + b x)(a + b x (a + b x)^2) = b^4 E (E + u) + g x + a^2,
 * E = x (x + h): two steps of Y <- Y (a I + b Y^T Y) on an eigenvalue x of the Gram matrix. */
void signmuon_debug_pair_coefficients(float a, float b, float* out5);

#ifdef __cplusplus
}
#endif
#endif /* SIGNMUON_DEBUG_H */
