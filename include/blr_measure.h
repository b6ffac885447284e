/*
 * blr_measure.h - flag bits of the forward calls of blr.h that exist for tests and measurements only.
 * An application never needs them; bench.py uses the stage flags to time the kernels of a multi-kernel
 * call one by one, the tests use BLR_FORCE_GENERIC to cross-check the two GPU code paths.
 */
#ifndef BLR_MEASURE_H
#define BLR_MEASURE_H

/* every forward: run the portable scalar-ALU kernels even where an MFMA kernel exists */
#define BLR_FORCE_GENERIC           0x100u
/* Monarch, low-rank and BLAST forwards: enqueue only the kernels up to and including the one that
 * writes the workspace intermediate (FIRST), or only the kernel that consumes it (LAST; the workspace
 * must hold the intermediate of an earlier call with identical arguments). Mutually exclusive;
 * BLR_ERR_UNSUPPORTED, with nothing enqueued, where the call is a single kernel. Where BLAST walks the
 * tokens in several chunks the workspace holds one chunk only, so LAST is then good for timing, not
 * for values. */
#define BLR_ONLY_FIRST_STAGE        0x200u
#define BLR_ONLY_LAST_STAGE         0x400u

#endif /* BLR_MEASURE_H */
