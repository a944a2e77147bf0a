/*
 * mttkrp_ablation.h -- the paper's own three matrix-free schedules as plain
 * HIP kernels, for side-by-side measurements against the streaming kernel of
 * mttkrp.h, and the paper's tile-volume heuristic.
 *
 * All three compute the same result as mttkrp_dense_* (Sec. II-B, Eq. (elem),
 * lambda = 1), with the same layouts, index base, ownership and error rules
 * (see mttkrp.h).  They keep what defines each schedule in Sec. III:
 *
 *   MTTKRP_SCHEDULE_ELEM  Sec. III-B, Alg. "MTTKRP-ELEM": one team thread per
 *       tensor entry, linear index -> multi-index by integer division, the
 *       whole Hadamard product recomputed per entry (d-1 multiplications per
 *       column), one atomic update of M per entry and column.
 *   MTTKRP_SCHEDULE_SUB   Sec. III-C: one team thread per mode-k subtensor,
 *       serial walk over its N/I_k entries with precomputed offsets (no
 *       division in the loop), conflict-free plain store of the row of M.
 *   MTTKRP_SCHEDULE_TILE  Sec. III-D, Alg. "MTTKRP-TILE": one team thread per
 *       tile of a subtensor, serial accumulation over the tile, one atomic
 *       update per tile and column; X is re-read for every chunk of columns.
 *       Tiles are regular cubes of `tile_width` entries along each of the d-1
 *       modes other than k, clipped at the tensor's edges.
 *
 * A "team thread" is a group of b_y lanes that share one tensor entry and
 * split the R columns among themselves (the paper's vector range p_y); a
 * workgroup holds 128 / b_y of them (Sec. IV-A: b_x = 128 / b_y).
 *
 * Because of the atomic updates, the ELEM and TILE results depend on the order
 * in which the hardware serialises them: equal to the definition up to
 * rounding, but not bit-identical from run to run.
 */
#ifndef MTTKRP_ABLATION_H
#define MTTKRP_ABLATION_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    MTTKRP_SCHEDULE_ELEM = 1,
    MTTKRP_SCHEDULE_SUB = 2,
    MTTKRP_SCHEDULE_TILE = 3
} mttkrp_schedule;

/*
 * M = X_(k) (Khatri-Rao of all A_m, m != k) by one of the paper's schedules.
 *   schedule    one of mttkrp_schedule
 *   tile_width  TILE only: entries per tile along every mode other than k,
 *               >= 1 (widths beyond an extent are clipped to it); ignored by
 *               ELEM and SUB
 *   other arguments, layouts, ownership: as mttkrp_dense_f64 / _f32.  M is
 *   overwritten (the library clears it first where the schedule accumulates
 *   with atomics).  No workspace is used.
 * Returns an mttkrp_status; MTTKRP_ERR_INVALID_ARG also for an unknown
 * schedule or tile_width < 1 with TILE; MTTKRP_ERR_UNSUPPORTED when a subtensor
 * would hold 2^40 tiles or more.
 */
int mttkrp_ablation_f64(int schedule, int ndim, const int64_t* dims, const double* X,
                        const double* const* factors, int R, int k, int64_t tile_width,
                        double* M, void* stream);
int mttkrp_ablation_f32(int schedule, int ndim, const int64_t* dims, const float* X,
                        const float* const* factors, int R, int k, int64_t tile_width,
                        float* M, void* stream);

/*
 * Tile-volume heuristic, Sec. IV-C, Eq. (heuristic): the largest regular tile
 * (integer width w along each of the d-1 modes, volume N_T = w^(d-1)) such
 * that c/2 tiles' worth of factor entries fit a quarter of the middle cache
 * level, capped by the smallest extent:
 *
 *     w = min( floor( ((s_LM / 4) / (s_f * c / 2))^(1/(d-1)) ),  min_n I_n ),   w >= 1
 *
 *   ndim, dims   the tensor (host array)
 *   cache_bytes  s_LM: bytes of the middle cache level per cache unit
 *                (L1 per SM / CU on a GPU, L2 per core on a CPU)
 *   value_bytes  s_f: bytes per value (8 or 4)
 *   tiles_per_unit  c: most tiles resident per cache unit at once (>= 1)
 *   width, volume   host outputs: w and w^(d-1)
 * Pure host arithmetic in integers; touches no device.  With the paper's
 * H100 figures (256 KiB, 8, 64) it gives 216 for a 4-way and 256 for a 5-way
 * tensor, the values the paper reports.
 */
int mttkrp_tile_volume(int ndim, const int64_t* dims, int64_t cache_bytes, int value_bytes,
                       int64_t tiles_per_unit, int64_t* width, int64_t* volume);

#ifdef __cplusplus
}
#endif
#endif /* MTTKRP_ABLATION_H */
