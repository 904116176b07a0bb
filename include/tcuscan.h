/*
 * tcuscan -- prefix sums on MI355X (gfx950) computed as products against all-ones
 * triangular matrices on the MFMA units.
 *
 * The operation is the one the paper states in Section 1 (notation paragraph) and
 * Section 2: given a vector x of size n, return its prefix sums
 *
 *     inclusive:  y[i] = x[0] + ... + x[i]            (the paper's default meaning of "scan")
 *     exclusive:  y[0] = 0,  y[i] = x[0] + ... + x[i-1]   (the inclusive result shifted by one)
 *
 * Algorithm 1 (MatMulScan) computes it as local scans L_s * T of s-element columns
 * (procedure BatchMatMul), a base-s up-sweep over block totals and a down-sweep that
 * broadcast-adds the carries (matrix B_s).  This library runs level 0 on the MFMA
 * units, the higher levels inside a workgroup on the vector unit (as Section 2.3
 * suggests for the B_s step), and replaces the remaining levels -- and Section 2.2's
 * "scan the segment totals, broadcast-add them" steps for n that is not a power of
 * s -- by a single-pass carry chain between workgroups.  The result is the same
 * prefix sum; zero-padding of the last tile is BatchMatMul's zero-pad.
 *
 * Plain C ABI.  Every pointer named d_* is a DEVICE pointer owned by the caller; the
 * library allocates nothing and frees nothing.  Calls are asynchronous: they enqueue
 * on `stream` (a hipStream_t passed as void*) and return; outputs are valid once the
 * stream reaches that point.  No call prints, throws or exits, and none blocks except
 * tcuscan_workspace_fault, which waits for the stream and copies one word to the host
 * (so it cannot be used while the stream is being captured).
 *
 * Inputs must be finite.  The local scans are products with 0/1 matrices, and 0 x Inf
 * and 0 x NaN are NaN: one non-finite input turns every output computed by the same
 * matrix instruction into NaN -- including outputs in front of it, up to 128 elements
 * away for 16-bit inputs -- where a sequential sum would only spoil what follows.
 */
#ifndef TCUSCAN_H
#define TCUSCAN_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    TCUSCAN_OK              = 0,
    TCUSCAN_ERR_INVALID_ARG = 1, /* null pointer with work to do, misaligned pointer, in/out overlap rule broken */
    TCUSCAN_ERR_UNSUPPORTED = 2, /* unknown dtype, size beyond the 32-bit tile index range                        */
    TCUSCAN_ERR_WORKSPACE   = 3, /* workspace missing or smaller than tcuscan_workspace_bytes()                   */
    TCUSCAN_ERR_HIP         = 4  /* the HIP runtime refused the launch                                            */
} tcuscan_status_t;

/* input element type -> output (= accumulator) element type */
typedef enum {
    TCUSCAN_I32_I32  = 0, /* int32 in, int32 out; sums are exact modulo 2^32 (four signed-byte planes on the i8 MFMA) */
    TCUSCAN_F16_F32  = 1, /* IEEE half in, fp32 accumulate and out (f16 MFMA)                                        */
    TCUSCAN_I8_I32   = 2, /* int8 in, int32 out (i8 MFMA); exact modulo 2^32                                         */
    TCUSCAN_F32_F32  = 3, /* fp32 in, fp32 out (f32 MFMA)                                                            */
    TCUSCAN_BF16_F32 = 4  /* bfloat16 in, fp32 accumulate and out (bf16 MFMA)                                        */
} tcuscan_dtype_t;

typedef void *tcuscan_stream_t; /* a hipStream_t; NULL is the default stream */

/*
 * Bytes of device workspace a call on `rows` rows of `cols` elements needs (0 when
 * every row fits one workgroup tile).  The workspace holds the carry chain between
 * workgroups (Algorithm 1's up-sweep rounds t >= 3 and Section 2.2 steps 2-3): one
 * 8-byte status word per tile, kept in a 64-byte slot of its own, plus a 256-byte header.
 *
 * The count is taken for a row together with the fewer-than-16 bytes in front of it down
 * to a 16-byte boundary, which is how rows that do not start at such a boundary are
 * tiled; for row lengths within 16 bytes of a multiple of the tile this is one word per
 * row more than the rows alone would need.  (Workspaces sized without that word are
 * still accepted; such rows then take the other tile size, a few per cent slower.)
 *
 * The caller zero-fills it ONCE after allocation (hipMemset, or tcuscan_workspace_init)
 * and may then reuse it for any number of calls whose requirement is not larger: every
 * call tags its status words with a fresh per-process call number, so older words read
 * as "not published".  The tags repeat after 2^30 - 2 calls; the library keeps track of
 * which workspaces it has seen since the last repeat and clears the status words of the
 * others itself (a fill kernel in front of the call), so the caller never has to.  A
 * call recorded by stream capture is replayed with the tag it was recorded with and
 * therefore clears its status words first (one extra fill kernel in the graph).  Two
 * calls that are in flight at the same time must not share a workspace.
 */
size_t tcuscan_workspace_bytes(size_t rows, size_t cols, tcuscan_dtype_t dt);

/* Enqueue a fill kernel that zeroes the workspace (usable under stream capture). */
tcuscan_status_t tcuscan_workspace_init(void *d_ws, size_t ws_bytes, tcuscan_stream_t stream);

/*
 * y <- inclusive prefix sums of x (Algorithm 1's input/output contract: same length,
 * may be in place).
 *   d_in   n elements of the input type, dense.  Aligned to the element size.
 *   d_out  n elements of the output type, dense.  Aligned to 4 bytes.  May equal d_in
 *          when input and output elements have the same size (I32_I32, F32_F32);
 *          any other overlap is undefined.
 *   n      element count; n == 0 returns TCUSCAN_OK and enqueues nothing.
 *   d_ws, ws_bytes   workspace, see tcuscan_workspace_bytes(1, n, dt); may be NULL/0
 *          when that is 0.
 * 16-byte aligned d_in and d_out take the 128-bit load/store path.  Other alignments are
 * accepted: an input that does not start at a 16-byte boundary (and, in the row-wise calls,
 * rows whose length in bytes is not a multiple of 16) is tiled from the boundary below, the
 * elements in front read as zero and never written; an output whose alignment differs from
 * the input's is written element by element.
 * Floating-point results are any valid fp32 summation order (MFMA accumulation order
 * and the carry chain's grouping are not fixed), so they may differ in the last bits
 * from run to run; integer results are unique.
 */
tcuscan_status_t tcuscan_inclusive(const void *d_in, void *d_out, size_t n, tcuscan_dtype_t dt,
                                   void *d_ws, size_t ws_bytes, tcuscan_stream_t stream);

/* y <- exclusive prefix sums of x: y[0] = 0, y[i] = inclusive[i-1].  The local scans
 * use the strictly lower triangular all-ones matrix (L_s with a zero diagonal).
 * Arguments as tcuscan_inclusive. */
tcuscan_status_t tcuscan_exclusive(const void *d_in, void *d_out, size_t n, tcuscan_dtype_t dt,
                                   void *d_ws, size_t ws_bytes, tcuscan_stream_t stream);

/*
 * Row-wise scans of a dense rows x cols matrix (row stride = cols), each row
 * independent along the last dimension (Section 2.2 step 1: Algorithm 1 on each
 * contiguous segment in parallel).  `exclusive` != 0 selects the exclusive scan.
 * Workspace: tcuscan_workspace_bytes(rows, cols, dt).  rows == 0 or cols == 0 is OK
 * and enqueues nothing.
 */
tcuscan_status_t tcuscan_batched(const void *d_in, void *d_out, size_t rows, size_t cols,
                                 tcuscan_dtype_t dt, int exclusive,
                                 void *d_ws, size_t ws_bytes, tcuscan_stream_t stream);

/*
 * The general form: row-wise scans with option flags.
 *   TCUSCAN_EXCLUSIVE  exclusive instead of inclusive
 *   TCUSCAN_REVERSE    every row is scanned from its end: y[i] = x[i] + ... + x[cols-1] (inclusive) or
 *                      x[i+1] + ... + x[cols-1] (exclusive) -- the suffix sums, i.e. the scan of the reversed
 *                      row, reversed.  In Algorithm 1's terms the local products use the upper triangular
 *                      all-ones matrix (the transpose of L_s) and the carries travel from the last block to
 *                      the first.
 * Unknown flag bits return TCUSCAN_ERR_INVALID_ARG.  Everything else as tcuscan_batched.
 */
#define TCUSCAN_EXCLUSIVE 1u
#define TCUSCAN_REVERSE   2u
tcuscan_status_t tcuscan_scan(const void *d_in, void *d_out, size_t rows, size_t cols, tcuscan_dtype_t dt, unsigned flags,
                              void *d_ws, size_t ws_bytes, tcuscan_stream_t stream);

/*
 * Segmented scans: `rows` rows of different lengths stored back to back (the CSR layout); row r is the elements
 * d_offsets[r] .. d_offsets[r+1]-1 of d_in / d_out, and each row is scanned on its own (Section 2.2 step 1 with
 * segments of arbitrary lengths; empty rows are allowed).  Flags as for tcuscan_scan.
 *   d_offsets  rows + 1 signed 64-bit element offsets on the DEVICE, non-decreasing, within [0, total]; 8-byte aligned
 *   total      number of elements d_in and d_out hold (an upper bound for d_offsets[rows]); sizes the launch
 *   d_ws       tcuscan_segmented_workspace_bytes(rows, total, dt) bytes, zero-filled once like every workspace here
 * Four steps are enqueued: tiles per row, their exclusive scan (this library's int32 scan), one descriptor per
 * tile (its row's extent and its place in the row), the scan itself; with fewer than 4096 rows the first three are one
 * launch.  The tile size follows the average row length total / rows.  Short rows (average below 2048 / 4096 / 8192 elements for 32- / 16- / 8-bit inputs) take another
 * form, three launches: the row starts become one bit per element, and the range the rows cover is scanned like one
 * row whose sums restart at every set bit (tcuscan_set_segmented_form(0) switches that form off).
 * Rows may start at any element: a row is tiled from the 16-byte boundary at or below its start, the few elements in
 * front of it are read as zero and not written.  Offsets that decrease or leave [0, total] are not followed: the
 * workspace's fault word is set to 2 (see tcuscan_workspace_fault) and the results of the call are unspecified (such
 * rows are skipped or clipped, rows may overlap); no access outside the n = total elements is made.
 * A segmented call keeps row maps in its workspace besides status words, at places that depend on its shape, so it
 * clears its status words in front of every run, and the library clears them again before another kind of call uses the
 * same workspace.  It cannot see a segmented call being REPLAYED from a graph: give such a graph a workspace that no
 * call outside the graph uses.
 */
size_t tcuscan_segmented_workspace_bytes(size_t rows, size_t total, tcuscan_dtype_t dt);
tcuscan_status_t tcuscan_segmented(const void *d_in, void *d_out, const long long *d_offsets, size_t rows, size_t total,
                                   tcuscan_dtype_t dt, unsigned flags, void *d_ws, size_t ws_bytes, tcuscan_stream_t stream);

/* Elements the small workgroup tile covers (rows no longer than this need no workspace), and the
 * large and huge tiles that long inputs use (more elements wait in registers per compute unit while
 * the carry chain's latency is paid, and fewer status words are published and polled per byte).  All
 * are multiples of s^2 = 256: a tile is a whole number of BatchMatMul chunks. */
size_t tcuscan_tile_elems(tcuscan_dtype_t dt);
size_t tcuscan_large_tile_elems(tcuscan_dtype_t dt);
size_t tcuscan_huge_tile_elems(tcuscan_dtype_t dt);

/*
 * Tile-size policy, process-wide: 0 = choose by shape (default: small tiles for short rows, large
 * ones from 2^13 .. 2^18 elements per row on depending on the input width, huge ones beyond
 * 2^22 .. 2^23, and only when the call then still has 512 / 256 tiles to fill the chip), 1 = always the
 * small tile, 2 / 3 = the large / huge tile for every row longer than a small tile.  A measurement and
 * test knob; results do not depend on it beyond floating-point summation order.
 */
tcuscan_status_t tcuscan_set_tile_policy(int policy);

/*
 * How tiles are handed to workgroups, process-wide.  0 (default): a workgroup scans the tile with its own index in the
 * grid; a tile waits only for tiles with smaller indices, so the carry chain makes progress as long as the hardware
 * starts workgroups in index order (never a workgroup while one with a smaller index is still waiting for a place),
 * which is how the dispatcher of this device family behaves and what every run of this library has shown.  1: a
 * workgroup draws its tile from a counter in the workspace when it starts running, so every tile it can wait for
 * belongs to a workgroup that is running or done whatever the dispatch order is; one atomic on one address per tile
 * makes long chains several times slower.  For callers who cannot rely on dispatch order (another dispatcher, a
 * simulator, a partitioned device).  Results are the same up to floating-point summation order.
 */
tcuscan_status_t tcuscan_set_chain_policy(int policy);

/* 1 (default): short rows of a segmented scan are scanned as one range with row-start bits; 0: every
 * row gets tiles of its own, as for all other segmented calls.  Process-wide; a measurement and test knob, results do
 * not depend on it beyond floating-point summation order. */
tcuscan_status_t tcuscan_set_segmented_form(int flat);

/*
 * Copy the workspace's sticky fault word to *h_fault (host pointer) after draining
 * `stream`.  1 means a carry-chain wait ran into its spin bound in some earlier
 * call (results of that call are invalid); this never happens in correct operation and
 * exists so that a protocol failure ends in an error instead of a hung GPU.  2 means a
 * segmented scan was given offsets that decrease or leave [0, total].
 */
tcuscan_status_t tcuscan_workspace_fault(const void *d_ws, tcuscan_stream_t stream, unsigned *h_fault);

/*
 * tcuscan_scan for callers that cannot allocate and have no workspace to pass: code running under stream capture,
 * tight serving loops, harnesses that forbid hipMalloc.  Same arguments and results as tcuscan_scan, without d_ws /
 * ws_bytes: the carry chain's status words live in a fixed array of TCUSCAN_STATIC_SCRATCH_BYTES inside the library's
 * device code (one copy per GPU, held until the process ends).  The call allocates and frees nothing.  Shapes whose
 * tcuscan_workspace_bytes() exceed the array (more than 65,536 small tiles: e.g. one row of more than 2^29 elements)
 * return TCUSCAN_ERR_WORKSPACE.  All calls on one GPU share the array: calls that overlap in time on the same GPU
 * (two streams, two threads) race and give wrong results; calls in stream order are fine, whatever their shapes.  The
 * array's address is looked up on the first call on each GPU (hipGetSymbolAddress, with that GPU current); make that
 * first call outside stream capture.  Its fault word is read with tcuscan_workspace_fault(TCUSCAN_STATIC_SCRATCH, ..).
 */
#define TCUSCAN_STATIC_SCRATCH_BYTES 4194560 /* 256-byte header + 65,536 status slots of 64 bytes */
#define TCUSCAN_STATIC_SCRATCH ((const void *)(size_t)1)
tcuscan_status_t tcuscan_scan_static(const void *d_in, void *d_out, size_t rows, size_t cols, tcuscan_dtype_t dt, unsigned flags,
                                     tcuscan_stream_t stream);

/*
 * Which way tcuscan_scan takes for this input pointer, shape and workspace size (a host-side query, nothing is
 * enqueued; d_in is only looked at for its alignment).  Rows that start at 16-byte boundaries take ROWS or TILES; other
 * rows are tiled from the boundary below (Section 2.2's segments, with BatchMatMul's zero-pad in front), unless the
 * workspace has status words for neither tile size that takes -- then ELEMENTWISE, the plain tiles read element by
 * element, several times slower.  A workspace of tcuscan_workspace_bytes() never gets ELEMENTWISE.  Returns -1 for an
 * unknown dtype or an empty shape.
 */
#define TCUSCAN_PATH_ROWS                0 /* one row per wavefront, no carry chain */
#define TCUSCAN_PATH_TILES               1 /* workgroup tiles and the carry chain */
#define TCUSCAN_PATH_TILES_FROM_BOUNDARY 2 /* the same for rows that do not start at 16-byte boundaries */
#define TCUSCAN_PATH_ELEMENTWISE         3
int tcuscan_path_for(const void *d_in, size_t rows, size_t cols, tcuscan_dtype_t dt, size_t ws_bytes);

/*
 * Measurement only: a streaming kernel with a scan's memory traffic and none of its work, the yardstick the benchmark
 * prices the scans against (a scan reads every input once and writes every output once; Section 2.3's cost model
 * counts the matrix products, the device counts the bytes).  Writes out_bytes (a multiple of 64) to d_out and reads
 * in_bytes_per_out_word (0: nothing, 1, 2 or 4) bytes from d_in for every 4 bytes written -- the mix of 8-, 16- and
 * 32-bit inputs with 32-bit outputs.  Both pointers 16-byte aligned.  variant: bits 0-2 = log2 of the 16-byte loads
 * (write-only: stores) each lane has in flight (1, 2, 4, 8, 16, 32), bit 8 = non-temporal loads, bit 9 = every wavefront reads
 * a run of consecutive KiB (a scan tile's shape) instead of interleaving with its workgroup's other wavefronts, bit 10 =
 * a grid of 2048 workgroups that walk over the data instead of one workgroup per chunk, bits 11-12 = a pause between
 * the arrival of a chunk's loads and its stores (0: none, 1: 512 cycles, 2: 2048 cycles; with 1 or 2 loads per lane
 * and an input only) -- a scan computes between its loads and its stores, and a kernel that stores the moment its
 * loads land is not the fastest streaming kernel; a caller takes the best of them.
 * 128-bit loads, non-temporal 128-bit stores, 1 KiB per wavefront and instruction, no dependencies.  The output is a
 * function of the input that nobody needs.
 */
tcuscan_status_t tcuscan_measure_stream(const void *d_in, void *d_out, size_t out_bytes, int in_bytes_per_out_word,
                                        unsigned variant, tcuscan_stream_t stream);

/*
 * Test hooks, process-wide; not for production use.
 *   tcuscan_test_advance_calls   adds `calls` to the process's call counter, as if that many calls had drawn status-word
 *                                tags (tcuscan_test_tag_period() of them bring the same tag round again).
 *   tcuscan_test_chain_fault     spin_limit: polls of one status word before a carry-chain wait gives up and raises
 *                                fault word 1 (0: back to the default, 2^24); mute_tile: the workgroup tile with this
 *                                index does not publish its status word (negative: none; plain scans only).  With a
 *                                muted tile and a small limit every later tile of the row gives up, all kernels end
 *                                normally, the results are wrong and the fault word says so.
 */
tcuscan_status_t tcuscan_test_advance_calls(unsigned long long calls);
unsigned long long tcuscan_test_tag_period(void);
tcuscan_status_t tcuscan_test_chain_fault(unsigned spin_limit, long long mute_tile);

/*
 * Algorithm 1 (MatMulScan) executed literally with s = 16: one kernel launch per round, k = log_s n
 * up-sweep rounds (gather x[s^t - 1 :: s^t], BatchMatMul with L_s, scatter) followed by k - 1
 * down-sweep rounds (gather x[s^t - 1 :: s^(t-1)], BatchMatMul with B_s, scatter); both constant
 * matrices run on the MFMA unit.  Inclusive scan only, and only n = 16^k (k >= 1), the lengths
 * Algorithm 1 is defined for; other n return TCUSCAN_ERR_UNSUPPORTED.  This is the unfused
 * reference schedule for measurements and schedule checks, not the fast path.
 *   d_in, d_out   as tcuscan_inclusive (d_out holds accumulator-typed values after round 0)
 *   rounds        number of rounds to execute, in Algorithm 1's order; negative = all 2k - 1.
 *                 With fewer rounds d_out holds the paper's intermediate state (Figure 1).
 *   d_matmuls     optional device counter (8-byte aligned, caller-zeroed): incremented by the number
 *                 of s x s products issued (Lemma 1).  Pass NULL when timing: counting costs atomics.
 * No workspace.  Asynchronous on `stream`.
 */
tcuscan_status_t tcuscan_matmulscan_levels(const void *d_in, void *d_out, size_t n, tcuscan_dtype_t dt,
                                           int rounds, unsigned long long *d_matmuls, tcuscan_stream_t stream);

/*
 * The same executor for the other radices the matrix unit has a native shape for: s = 4 (sixteen 4 x 4
 * blocks per MFMA instruction), s = 16 (as above) and s = 32 (32 x 32 MFMA); n = s^k.  Algorithm 1 is
 * stated for any s >= 2; Lemma 1 gives its depth 2 log_s n - 1 and its product count, and the paper's
 * comparison table (Section 3) is the fan-in against depth trade-off this call lets one measure.
 * Other s return TCUSCAN_ERR_UNSUPPORTED.  Arguments as tcuscan_matmulscan_levels.
 */
tcuscan_status_t tcuscan_matmulscan_levels_radix(const void *d_in, void *d_out, size_t n, tcuscan_dtype_t dt, int s,
                                                 int rounds, unsigned long long *d_matmuls, tcuscan_stream_t stream);

/*
 * Applications the paper's introduction gives as its motivation, built on the exclusive scan of a 0/1
 * int8 mask (the I8_I32 MFMA path).  The caller provides every scratch buffer; workspace as for
 * tcuscan_exclusive(.., n, TCUSCAN_I8_I32, ..).  n < 2^32.  Asynchronous on `stream`.
 *
 * Stream compaction: d_out receives, in order, the 32-bit d_values[i] whose d_mask[i] (int8) is non-zero
 * (mask entries must be 0 or 1).
 *   d_positions  n int32: on return the exclusive scan of the mask (the destination indices), or NULL: then the
 *                positions are not materialised and the scatter is fused into the scan (one pass over mask and
 *                values, one kernel)
 *   d_count      optional device word: number of kept elements
 */
tcuscan_status_t tcuscan_compact_u32(const void *d_values, const void *d_mask, void *d_out, size_t n,
                                     void *d_positions, unsigned *d_count,
                                     void *d_ws, size_t ws_bytes, tcuscan_stream_t stream);

/*
 * Radix sort by Blelloch's reduction to prefix sums: `bits` stable split passes, least significant bit
 * first; pass b scans the mask "bit b is 0" and sends the zeros to the front and the ones behind them,
 * both in their old order.  Sorts the n unsigned 32-bit d_keys in place by their low `bits` bits (32 for a
 * full sort); d_vals, if not NULL, are n 32-bit payloads permuted along with the keys (so the sort is
 * observably stable).
 *   d_keys_tmp, d_vals_tmp   scratch, n words each (d_vals_tmp only with d_vals); keys buffers 16-byte aligned
 *   d_flags                  scratch, n bytes, 16-byte aligned
 *   d_positions              scratch, n int32
 * This answers "can the matrix unit sort?".  By default a pass is one fused kernel (flags built from the keys, scanned
 * on the MFMA unit, keys scattered; d_flags is not used and d_positions only holds 96 counters) and splits on two bits
 * at once -- four buckets, the flags of two digits sharing a byte of the scanned operand -- so a full sort is 16
 * passes; an odd `bits` ends with one pass on a single bit.  tcuscan_set_sort_fusion(2) keeps the fused kernel to one
 * bit per pass, tcuscan_set_sort_fusion(0) selects the three-kernel form of the reduction (mask kernel,
 * tcuscan_exclusive, scatter kernel per bit), which is also what n < 96 takes.
 */
tcuscan_status_t tcuscan_split_radix_sort_u32(void *d_keys, void *d_vals, size_t n, int bits,
                                              void *d_keys_tmp, void *d_vals_tmp, void *d_flags, void *d_positions,
                                              void *d_ws, size_t ws_bytes, tcuscan_stream_t stream);

/* 1 (default): fused split passes on two bits; 2: fused passes on one bit; 0: mask kernel + tcuscan_exclusive + scatter
 * kernel per bit; anything else TCUSCAN_ERR_INVALID_ARG.  Process-wide; a measurement and test knob, the sorted result
 * is the same. */
tcuscan_status_t tcuscan_set_sort_fusion(int fused);

/* Static, human-readable name of a status code. */
const char *tcuscan_status_string(tcuscan_status_t st);

#ifdef __cplusplus
}
#endif
#endif /* TCUSCAN_H */
