/*
 * finemoe_measure.h - measurement and test switches of libfinemoe.  NOT part of the contract of
 * finemoe.h: they exist so that a benchmark can time one kernel of an entry point and so that tests
 * can force a code path; values and meaning may change with any version.  They travel in
 * fine_shape.flags next to FINE_FLAG_LOCALITY (which is the only flag a caller of the library
 * needs); a flags word with none of them set runs every entry point as finemoe.h describes it.
 */
#ifndef FINEMOE_MEASURE_H
#define FINEMOE_MEASURE_H

enum {
    FINE_FLAG_SIMPLE_FFN = 2,    /* tests: plain tiled FMA kernels instead of MFMA in fine_grouped_ffn */
    FINE_FLAG_ONLY_GEMM1 = 4,    /* timing: fine_grouped_ffn runs only X[Wg|Wu] + SwiGLU (H into ws)    */
    FINE_FLAG_ONLY_GEMM2 = 8,    /* timing: fine_grouped_ffn runs only H Wd (H as left in ws)           */
    FINE_FLAG_TILE_SHIFT = 8,    /* bits 8-9, tests: row tile of the MFMA kernels, 0 = chosen from the  */
    FINE_FLAG_TILE_MASK = 0x300, /*   shape, 1 = 64 rows, 2 = 128 rows, 3 = 256 rows                    */
    /* bits 12-14, timing: fine_backward runs one stage only; the stages of a pass must then be called
     * in the order 1 .. 5 on one workspace: 1 = gradient of combine (and the recomputation of the
     * pre-activations when act_save is NULL), 2 = dH with the SwiGLU gradient, 3 = dXp,
     * 4 = weight gradients, 5 = gradient of permute */
    FINE_MEASURE_BWD_STAGE_SHIFT = 12,
    FINE_MEASURE_BWD_STAGE_MASK = 0x7000
};

#endif /* FINEMOE_MEASURE_H */
