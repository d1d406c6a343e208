/*
 * rapid_tuning.h -- benchmark and tuning hooks of librapid_hip.so.  NOT part of the product ABI in
 * rapid.h: nothing here is needed to compute anything, the results of every call in rapid.h are the
 * same whatever is set here (up to the fp32 rounding noted at keys 17 and 20), and two of the calls below
 * wait for the device, which no call in rapid.h ever does.  bench.py and the tests of the kernels'
 * launch geometries use them.
 */
#ifndef RAPID_TUNING_H
#define RAPID_TUNING_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Process-wide switches (host state; each is one atomic word, read once per call: a call that races
 * with a change sees the old or the new value).
 * key 1: per-stage event timing on (1) / off (0, default); see rapid_profile_read.
 * key 2: waves per workgroup of the contraction kernels: 0 (default) = each kernel's own choice (8,
 *        i.e. 2 x 4 waves of 128 x 64, for the logits kernels and dW; 4, i.e. 2 x 2 waves of 128 x 128,
 *        for dHidden), or 4 / 8 / 16 for all of them.  Same 256 x 256 tile and same results either way.
 * keys 10, 11, 12: tile-order blocking (tiles along the first tile dimension that share one tile of
 *        the second before the order moves on) of the logits kernels, the dHidden kernel (0 = all)
 *        and the dW kernel; defaults 4, 0, 2 were measured best on MI355X.  Results are identical.
 * key 13: token-row tiles (of 256 rows) per launch of the two logits kernels (forward and dz),
 *        default 64: they sweep all of W over one such block of rows at a time so that the block's
 *        hidden rows stay in the memory-side cache.  Results are identical.
 * key 14: 1 (default) / 0: the dHidden kernel reads W from a tile-blocked copy (one contiguous
 *        32 KiB block per 256-row tile and 64-column step) / from the row-major copy.  Results
 *        are identical.
 * key 15: with logits_cache = 1, token-row tiles (of 256 rows) per launch of the dHidden kernel,
 *        default 256 (0 = all rows of the chunk in one launch; multiples of 128 fill whole rounds of
 *        workgroups).  Results depend on it only through which tiles key 17 cuts.
 * key 16: K steps (of 64 vocabulary entries; a power of two; default 0 = off) between meetings
 *        of the dHidden kernel's workgroups: they count themselves in on a workspace word and wait,
 *        for a bounded time, for the others, so that all XCDs sweep W together and share it through
 *        the memory-side cache.  A timing hint only: results are identical, and a meeting that runs
 *        out of time switches the pacing off for the rest of the launch.
 * key 17: 1 (default) / 0: the dHidden kernel cuts the contraction of the tiles of a partly filled last round of
 *        workgroups into equal segments and deals the (tile, segment) units out in short rounds (the pieces of a
 *        tile are summed in a fixed order by a small second kernel), instead of leaving workgroups idle for a
 *        whole tile.  The sums are taken in another order: results differ by fp32 rounding of the accumulators.
 * key 18: cache rows (a multiple of 256, default 90112) of the size rapid_workspace_bytes recommends for
 *        RAPID_OP_IW_PG_FWD_BWD_CACHED.  A call uses whatever its workspace affords; this only moves the
 *        recommendation.
 * key 19: 1 (default) / 0: generations without gradient (a group whose rewards are all 0, a zero coefficient
 *        override) are ordered behind the others and left out of the backward's contractions; 0 keeps them in,
 *        for measuring what that saves.  Same results up to the order of the sums.
 * key 20: row tiles (of 256 rows) per dW launch of the cached backward; 0 (default) = all rows of the chunk in one
 *        launch.  dW sums over its launches in a fixed order, so results depend on the key only through fp32
 *        rounding.
 * key 21: 0 (default), or a variant of the forward logits kernel that takes K steps of 32 with W from a K-blocked
 *        copy (which adds Vpad x dpad x 2 bytes to every workspace size while the key is set: set it before
 *        asking for sizes): 1 = two 4-wave workgroups per CU on 256 x 128 tiles, three LDS stages; 2 = one 8-wave
 *        workgroup per CU on 256 x 256 tiles, four stages, requests three steps ahead; 3 = the same with 4 waves
 *        of 128 x 128.  Identical results; measured slower or equal, kept for those measurements.
 * key 22: 0 (default) / 1: the dW kernel with K steps of 32 rows through four LDS stages, requests three steps
 *        ahead.  Identical results; measured 2 % slower, kept for that measurement. */
int rapid_set_tuning(int key, int value);

/* Per-stage timing for benchmarks.  rapid_set_tuning(1, 1) makes every later call bracket each of
 * its stages with HIP events on the caller's stream (host objects, no device memory);
 * rapid_profile_read waits for those events, writes the milliseconds and the number of timed spans
 * per stage into two HOST arrays of n_stages >= RAPID_N_STAGES entries, and clears the record.
 * Stage order: 0 compaction/gather, 1 operand packing (with rms_weight: the final norm), 2 forward
 * logits+log-sum-exp kernel, 3 sampled-token logits and log-sum-exp merge, 4 estimator reductions
 * (ratios, advantages, loss, row coefficients), 5 zeroing of masked gradient rows (with rms_weight
 * also the norm's backward), 6 dz kernel (with logits_cache: the row-factor pass), 7 unused,
 * 8 dHidden kernel, 9 dW kernel, 10 fp32 path, 11 dW conversion. */
#define RAPID_N_STAGES 12
int rapid_profile_read(double* ms_by_stage, int64_t* spans_by_stage, int n_stages);

/* Diagnostic for benchmarks: the rate the bf16 matrix pipe sustains on its own (32 x 32 x 16 MFMAs
 * out of registers on every SIMD of the device, no LDS or memory traffic), the ceiling the roofline
 * of the contraction kernels (Sec. 3.1's LM head; the backward of Eq. (3)) can be read against at
 * the clock the chip holds under load.  random_operands = 0 uses small-integer operands (the
 * published peak is reached), 1 uses random bf16 values in [-1, 1] (the power management lowers the
 * clock).  Runs `iters` (1 .. 10^7) MFMAs per accumulator on `stream`, WAITS for them, and writes
 * TFLOP/s and the elapsed milliseconds to HOST pointers (either may be NULL).  Allocates nothing.
 * Errors: RAPID_ERR_SHAPE (iters out of range), RAPID_ERR_ARCH, RAPID_ERR_HIP. */
int rapid_mfma_probe(int random_operands, int iters, double* tflops_out, double* ms_out, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* RAPID_TUNING_H */
