/*
 * lookupffn.h -- C ABI of the MI355X (gfx950) LookupFFN inference forward pass.
 *
 * The operation (paper notation, h tables called `k` here):
 *
 *   Hash    (Sec. 3.1, hyperplane hash; Sec. 3.2, eq. "hadamard"):
 *           z = x R,  R = D_1 H D_2 H ... D_R H,  D_r = +-1 diagonals, H = Walsh-Hadamard
 *           transform in Sylvester order scaled by d_pad^(-1/2); x is zero-padded at the
 *           tail to d_pad = next power of two >= d.  When k*tau > d_pad, P =
 *           ceil(k*tau/d_pad) independent projections (own diagonals each) are
 *           concatenated.  Table j owns coordinates [j*tau, (j+1)*tau) of that
 *           concatenation (Sec. 3.2, "The problem") and
 *           code_j = sum_b [ z[j*tau+b] >= 0 ] << b     (decimal(sign(z_j)), 0-based).
 *   Gather  (Sec. 3.1, eq. "lookup" with the top-1 choice of eq. "optimal_index"):
 *           y = sum_{j<k} tables[j][code_j][:]          (plain sum, no 1/k)
 *
 *   Weighted variant (Sec. 4, "Overview"; the form the paper's experiments use; the
 *           linearly scaled eq. "partial_softmax" with the single row g(z_j)):
 *           w_j = <z_j,S_g> exp(<z_j,S_g>) / prod_b (exp(z_jb) + exp(-z_jb)),  S_g = sign(z_j)
 *           y   = sum_{j<k} w_j * tables[j][code_j][:]
 *
 * Conventions for every entry point
 *   - Every data pointer is a DEVICE pointer owned by the caller and valid on the
 *     current HIP device; the library never frees or retains them.
 *   - Arrays are dense and row-major:
 *       x      [n_tokens][d]                 fp32, bf16 or IEEE half (16-bit patterns)
 *       signs  [P][n_rounds][d_pad]          int8, a negative entry means "flip"
 *       codes  [n_tokens][k]                 uint16
 *       weights[n_tokens][k]                 fp32 (weighted variant only)
 *       tables [k][2^tau][d_out]             fp32, bf16 or IEEE half, or the prepared copy (lookupffn_prepare_tables)
 *       y      [n_tokens][d_out]             fp32
 *   - `hip_stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Work is enqueued on it and the call returns without synchronising.
 *   - Scratch memory.  Entry points with a (workspace, workspace_bytes) pair keep their intermediates
 *     (codes, weights, the staged gather's re-packed copies) there.  With a caller workspace (device
 *     memory, 256-byte aligned, at least the matching lookupffn_workspace_bytes*() bytes) the call only
 *     launches kernels on `hip_stream`: it allocates nothing, frees nothing, never synchronises, and --
 *     once lookupffn_init() has run on the device -- makes no other runtime call, so it may be captured in a
 *     HIP graph.  Calls that share a workspace must be ordered on one stream.  workspace == NULL is a
 *     convenience for simple callers: the library then uses a per-device buffer of its own, which it grows
 *     with hipMalloc when a call needs more (old buffers are kept until lookupffn_release_workspace(), so
 *     enqueued work stays valid; a growing call cannot be captured, and all NULL-workspace calls on a
 *     device must be ordered on one stream because they share that buffer).  The size queries take any
 *     arguments: a count that no buffer can have (beyond 2^63 bytes) comes back as INT64_MAX rounded down
 *     to a multiple of 256, which every workspace is smaller than.
 *   - Return value: 0 on success, a negative lffn_status otherwise.  Arguments are
 *     validated before the first HIP call, so error paths need no GPU.
 *     n_tokens == 0 is a successful no-op.  Nothing is printed, nothing aborts.
 *   - Arithmetic: the hash runs in fp32 (round to nearest, no fused multiply-add,
 *     butterflies in ascending stride order), bf16 and half inputs are widened exactly; the
 *     gather accumulates in fp32 in table order j = 0..k-1.  The weights are evaluated in
 *     fp32 as |z_j|_1 / prod_b (1 + exp(-2|z_jb|)) (the same quotient with exp(|z_j|_1) divided
 *     out, so nothing overflows) with the hardware exp2 and reciprocal; the weighted gather
 *     is one fused multiply-add per element and table.
 */
#ifndef LOOKUPFFN_H
#define LOOKUPFFN_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum { LFFN_F32 = 0, LFFN_BF16 = 1, LFFN_F16 = 2 /* IEEE binary16 */ } lffn_dtype;
/* OR-ed into a `table_dtype` argument: `tables` is the buffer lookupffn_prepare_tables() wrote (from
 * tables of the dtype in the low bits).  OR-ed into a `block` argument of the BH entry points: `bmats`
 * is the buffer lookupffn_prepare_bh() wrote. */
#define LFFN_PREPARED 0x100
/* OR-ed into a `table_dtype` argument of a gather / forward entry point: y is stored as bf16 / IEEE half
 * instead of fp32 (the fp32 sums rounded once, to nearest even, when they are stored; y then 8-byte aligned).
 * At most one of the two.  lookupffn_forward_stack rounds only the last layer's output: the values handed from
 * layer to layer stay fp32. */
#define LFFN_Y_BF16 0x200
#define LFFN_Y_F16 0x400

typedef enum {
    LFFN_OK = 0,
    LFFN_E_NULL = -1,         /* a required pointer is NULL */
    LFFN_E_SIZE = -2,         /* n_tokens < 0, d/k/d_out/n_rounds < 1, or a size product overflows */
    LFFN_E_TAU = -3,          /* tau outside [1, 16] */
    LFFN_E_DTYPE = -4,        /* dtype is none of LFFN_F32, LFFN_BF16, LFFN_F16 */
    LFFN_E_ALIGN = -5,        /* tables or y not 16-byte aligned, x/codes not element aligned,
                                 or d_out not a multiple of 4 (fp32 tables) / 8 (16-bit tables) */
    LFFN_E_UNSUPPORTED = -6,  /* a shape the kernels are not built for: d_pad above 4096; the BH
                                 entry points state their own limits */
    LFFN_E_WORKSPACE = -7,    /* caller workspace (or a prepare call's output buffer) smaller than the matching
                                 *_bytes() query says */
    LFFN_E_HIP = -8           /* a HIP call failed; see lookupffn_last_hip_error() */
} lffn_status;

/*
 * Once per device (with that device current), before the first capture of any entry point into a HIP
 * graph: registers the dynamic-LDS need of every kernel that uses more than 64 KB with the runtime and
 * caches the device's compute-unit count, so that later calls with a caller workspace consist of kernel
 * launches only.  Optional otherwise (each kernel does it on first use).  For callers under graph capture.
 */
int lookupffn_init(void);

/*
 * Hash step alone (Sec. 3.1 "Two main operations", (a)): writes codes[n_tokens][k].
 */
int lookupffn_hash(const void *x, const int8_t *signs, uint16_t *codes,
                   int64_t n_tokens, int d, int k, int tau,
                   int n_rounds, int x_dtype, void *hip_stream);

/*
 * Gather step alone (Sec. 3.1 "Two main operations", (b), unweighted; eq. "lookup"):
 * y[t] = sum_j tables[j][codes[t][j] mod 2^tau].  Codes are reduced modulo 2^tau, so no
 * value of `codes` can make the kernel read outside `tables`.  Scratch:
 * lookupffn_workspace_bytes_gather(n_tokens, k) bytes (the LDS-staged kernel reads the codes re-packed).
 */
int lookupffn_gather(const uint16_t *codes, const void *tables, void *y,
                     int64_t n_tokens, int k, int tau, int d_out,
                     int table_dtype, void *workspace, int64_t workspace_bytes, void *hip_stream);
int64_t lookupffn_workspace_bytes_gather(int64_t n_tokens, int k);

/*
 * Whole forward pass: Hash then Gather on the same stream (Sec. 3.1, eq. "lookup").
 * Scratch: lookupffn_workspace_bytes(n_tokens, k) bytes (0 if n_tokens == 0).
 * Batches of up to 512 tokens ("small_tokens" below) whose shape lookupffn_forward_stack takes run as that
 * call's single launch with n_layers = 1 (no scratch touched); y has the same bits either way.
 */
int lookupffn_forward(const void *x, const int8_t *signs, const void *tables, void *y,
                      int64_t n_tokens, int d, int k, int tau, int d_out,
                      int n_rounds, int x_dtype, int table_dtype,
                      void *workspace, int64_t workspace_bytes, void *hip_stream);
int64_t lookupffn_workspace_bytes(int64_t n_tokens, int k);

/*
 * Several chained layers of the forward pass in ONE kernel launch, for batches of a few tokens where the
 * launches and the empty chip, not the arithmetic, set the time (Sec. 3.1; each layer is eq. "hadamard",
 * the sign codes, eq. "lookup"): layer 0 reads x, layer l + 1 reads layer l's output as its input (so
 * d_out == d when n_layers > 1; no residual and no normalisation in between), y receives the last layer's
 * output.  `signs` and `tables` are HOST arrays of n_layers DEVICE pointers (read during the call, not kept):
 * signs[l] as in lookupffn_hash, tables[l] as in lookupffn_gather, all layers with the same k, tau, dtypes
 * and layout (LFFN_PREPARED in table_dtype: every tables[l] is a prepared copy).  One workgroup per token;
 * the per-element sums are the same sequential fp32 sums as lookupffn_forward makes, so the result equals
 * a loop of n_layers lookupffn_forward calls bit for bit.  No scratch memory, no allocation, no
 * synchronisation: the call can be captured in a HIP graph.
 * Shapes: 512 < d <= 1024, n_rounds <= 4, n_layers <= 32, one layer's tables below 2 GiB, signs 16-byte
 * aligned, x rows 16-byte aligned when d % 4 == 0; anything else returns LFFN_E_UNSUPPORTED and the caller
 * loops over lookupffn_forward instead.  n_layers > 1 with d_out != d returns LFFN_E_SIZE.
 */
int lookupffn_forward_stack(const void *x, const int8_t *const *signs, const void *const *tables, void *y,
                            int64_t n_tokens, int d, int k, int tau, int d_out,
                            int n_rounds, int n_layers, int x_dtype, int table_dtype, void *hip_stream);

/*
 * lookupffn_forward for callers that cannot allocate device memory or pass a workspace: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same kernels and
 * bit-identical y, but the intermediates live in a device array that is part of the library's code object
 * (lookupffn_static_scratch_bytes() = 16 MiB per GPU, held from load until the process ends), so the call
 * allocates nothing and frees nothing.  Batches whose intermediates (lookupffn_workspace_bytes(n_tokens, k))
 * exceed that size return LFFN_E_WORKSPACE (k = 96: batches up to about 39000 tokens fit).  All calls on one GPU
 * share the one array: calls that overlap in time on a GPU (two streams, two threads) race on it; order
 * them on one stream.  Nothing in the array needs clearing between calls (every word a call reads, it
 * wrote first).  The array's address is looked up on the first call on a device, or by lookupffn_init().
 */
int lookupffn_forward_static(const void *x, const int8_t *signs, const void *tables, void *y,
                             int64_t n_tokens, int d, int k, int tau, int d_out,
                             int n_rounds, int x_dtype, int table_dtype, void *hip_stream);
int64_t lookupffn_static_scratch_bytes(void);

/*
 * One-time preparation of the learned tables T_1 .. T_k of eq. "lookup" (Sec. 3.1): they are constants of
 * the model, so the layout the gather kernels stream best is written once, outside the forward pass.
 * lookupffn_prepare_tables copies tables[k][2^tau][d_out] (fp32, bf16 or half) into `prepared` as fp32 (16-bit rows
 * widened exactly), slice-major: the 128-byte (tau <= 8) or 64-byte (tau >= 9) column slice of all rows of
 * all tables is one contiguous run, ragged last slice zero-filled.  `prepared`: device memory, 256-byte
 * aligned, lookupffn_prepared_tables_bytes() bytes (0 for arguments the call would reject), owned by the
 * caller.  Every gather / forward entry point takes it in place of `tables` with
 * table_dtype = LFFN_PREPARED | <dtype of the source tables>; results are bit-identical to those with
 * the row-major tables.  16-bit tables take the LDS-staged gather only in this form (it reads fp32 rows).
 */
int64_t lookupffn_prepared_tables_bytes(int k, int tau, int d_out, int table_dtype);
int lookupffn_prepare_tables(const void *tables, int k, int tau, int d_out, int table_dtype,
                             void *prepared, int64_t prepared_bytes, void *hip_stream);

/*
 * Weighted variant (Sec. 4, "Overview").  lookupffn_hash_weighted writes codes[n_tokens][k]
 * and weights[n_tokens][k] (4-byte aligned; LFFN_E_UNSUPPORTED when d_pad = 4096, where the
 * kernel's working set no longer fits).  lookupffn_gather_weighted computes
 * y[t] = sum_j weights[t][j] * tables[j][codes[t][j] mod 2^tau].  lookupffn_forward_weighted
 * chains the two like lookupffn_forward.
 */
int lookupffn_hash_weighted(const void *x, const int8_t *signs, uint16_t *codes, float *weights,
                            int64_t n_tokens, int d, int k, int tau,
                            int n_rounds, int x_dtype, void *hip_stream);
int lookupffn_gather_weighted(const uint16_t *codes, const float *weights, const void *tables, void *y,
                              int64_t n_tokens, int k, int tau, int d_out,
                              int table_dtype, void *workspace, int64_t workspace_bytes, void *hip_stream);
int64_t lookupffn_workspace_bytes_gather_weighted(int64_t n_tokens, int k);
int lookupffn_forward_weighted(const void *x, const int8_t *signs, const void *tables, void *y,
                               int64_t n_tokens, int d, int k, int tau, int d_out,
                               int n_rounds, int x_dtype, int table_dtype,
                               void *workspace, int64_t workspace_bytes, void *hip_stream);
int64_t lookupffn_workspace_bytes_weighted(int64_t n_tokens, int k);

/*
 * Multi-probe lookup (Sec. 3.1, eq. "partial_softmax" with the neighbourhood "rows within one sign
 * flip of sign(z_j)"): per table the selected row and its tau one-bit neighbours, each weighted by its
 * soft-max share exp(<z_j,S_i>) / prod_b (exp(z_jb) + exp(-z_jb)):
 *   y = sum_j sum_{probe=0..tau} shares[t][j][probe] * tables[j][code_j ^ flip(probe)][:],
 *   flip(0) = 0, flip(probe) = 1 << (probe-1).
 * lookupffn_hash_probes writes codes[n_tokens][k] and shares[n_tokens][k][1+tau] (fp32, 4-byte
 * aligned); lookupffn_gather_probes does the sum ((1 + tau) row reads per token and table);
 * lookupffn_forward_probes chains them.  Same hash, conventions and limits as the weighted variant.
 */
int lookupffn_hash_probes(const void *x, const int8_t *signs, uint16_t *codes, float *shares,
                          int64_t n_tokens, int d, int k, int tau,
                          int n_rounds, int x_dtype, void *hip_stream);
int lookupffn_gather_probes(const uint16_t *codes, const float *shares, const void *tables, void *y,
                            int64_t n_tokens, int k, int tau, int d_out,
                            int table_dtype, void *workspace, int64_t workspace_bytes, void *hip_stream);
int64_t lookupffn_workspace_bytes_gather_probes(int64_t n_tokens, int k, int tau);
int lookupffn_forward_probes(const void *x, const int8_t *signs, const void *tables, void *y,
                             int64_t n_tokens, int d, int k, int tau, int d_out,
                             int n_rounds, int x_dtype, int table_dtype,
                             void *workspace, int64_t workspace_bytes, void *hip_stream);
int64_t lookupffn_workspace_bytes_probes(int64_t n_tokens, int k, int tau);

/*
 * BH{m} hash (Sec. 3.2, eq. "block_acdc"): z = x R with R = prod_{i=1..n_factors} B_i H per
 * projection, B_i block-diagonal with `block` x `block` blocks (16, 32 or 64), H as above; codes as
 * above.  (v B)_j = sum_c v_c B[c][j] over j's block is accumulated in fp32 as a chain of fused
 * multiply-adds, c ascending, from +0 (on the matrix cores).
 *   bmats [P][n_factors][d_pad/block][block][block] fp32, element [p][i][blk][c][j] = B_i[blk*block+c][blk*block+j]
 * Supported: 64 <= d_pad <= 1024 (LFFN_E_UNSUPPORTED otherwise, and for other block sizes).
 * The kernels read the factors in matrix-core operand order.  The B_i are learned constants: write that
 * order once with lookupffn_prepare_bh (`prepared`: device memory, 256-byte aligned,
 * lookupffn_prepared_bh_bytes() bytes) and pass it as `bmats` with block = LFFN_PREPARED | block.  Given
 * the row-major factors instead, every call re-orders them into its workspace first.
 * lookupffn_forward_bh = this hash + the plain gather.  Scratch: lookupffn_workspace_bytes_bh() bytes
 * (`block` as it will be passed to the call, flag included).
 */
int64_t lookupffn_prepared_bh_bytes(int d, int k, int tau, int block, int n_factors);
int lookupffn_prepare_bh(const float *bmats, int d, int k, int tau, int block, int n_factors,
                         void *prepared, int64_t prepared_bytes, void *hip_stream);
int lookupffn_hash_bh(const void *x, const float *bmats, uint16_t *codes,
                      int64_t n_tokens, int d, int k, int tau, int block, int n_factors, int x_dtype,
                      void *workspace, int64_t workspace_bytes, void *hip_stream);
int lookupffn_forward_bh(const void *x, const float *bmats, const void *tables, void *y,
                         int64_t n_tokens, int d, int k, int tau, int d_out, int block, int n_factors,
                         int x_dtype, int table_dtype,
                         void *workspace, int64_t workspace_bytes, void *hip_stream);
int64_t lookupffn_workspace_bytes_bh(int64_t n_tokens, int d, int k, int tau, int block, int n_factors);

/*
 * BH{m} hash with the weighted gather (the configuration of the paper's experiments: Sec. 3.2 hash,
 * Sec. 4 forward pass): lookupffn_hash_bh_weighted writes codes[n_tokens][k] and weights[n_tokens][k]
 * (fp32, 4-byte aligned) with w_j as in lookupffn_hash_weighted, computed from the z of the BH hash;
 * lookupffn_forward_bh_weighted = that + lookupffn_gather_weighted, with
 * lookupffn_workspace_bytes_bh_weighted() bytes of scratch.
 * Supported: the shapes of lookupffn_hash_bh, every tau (with tau = 4, 8 or 16 a table lies inside one
 * 16-coordinate tile of z and is reduced in registers; with any other tau -- the paper's RoBERTa-base row is
 * tau = 9 -- the kernel forms the weights from z through a window in LDS).
 */
int lookupffn_hash_bh_weighted(const void *x, const float *bmats, uint16_t *codes, float *weights,
                               int64_t n_tokens, int d, int k, int tau, int block, int n_factors, int x_dtype,
                               void *workspace, int64_t workspace_bytes, void *hip_stream);
int lookupffn_forward_bh_weighted(const void *x, const float *bmats, const void *tables, void *y,
                                  int64_t n_tokens, int d, int k, int tau, int d_out, int block, int n_factors,
                                  int x_dtype, int table_dtype,
                                  void *workspace, int64_t workspace_bytes, void *hip_stream);
int64_t lookupffn_workspace_bytes_bh_weighted(int64_t n_tokens, int d, int k, int tau, int block, int n_factors);

/* Frees the library-owned buffers of workspace == NULL calls (all devices; synchronises each device
 * first).  Safe to call when none exist. */
int lookupffn_release_workspace(void);

/*
 * Kernel timing for benchmarks.  `mask` selects which launches are bracketed by a pair of
 * HIP events recorded on the launch stream: bit 0 = hash kernel, bit 1 = gather kernel
 * (0 = off, 3 = both; each bracketed launch costs a few microseconds of queue time).
 * lookupffn_timing_read synchronises on the recorded events and returns, for
 * `which` (0 = hash kernel, 1 = gather kernel), the summed elapsed milliseconds and the
 * number of launches since the last reset; lookupffn_timing_read_each copies the first `capacity`
 * launches' own durations (milliseconds, launch order) to the host array `ms_out` and returns the launch
 * count.  Off by default.
 */
int lookupffn_timing_enable(int mask);
int lookupffn_timing_reset(void);
int lookupffn_timing_read(int which, double *total_ms, int64_t *launches);
int lookupffn_timing_read_each(int which, double *ms_out, int64_t capacity, int64_t *launches);

/*
 * Launch-shape knobs of the gather kernel, for tuning sweeps (0 = library default):
 *   "lanes_per_token"  1,2,4,...,64   lanes (16 bytes each) that share one token's row slice
 *   "xcd_order"        1 / -1         force the XCD-sliced block order on / off
 *   "gather_path"      1 / 2 / 4      1: always the direct kernel; 2: the LDS-staged kernel whenever the shape
 *                                     allows it (tau 7 .. 10, fp32 or prepared rows), whatever the batch size; 4: the lagged ring
 *                                     kernel where it exists (prepared tables, tau 7 or 8, plain sum), else as 2
 *   "ring_threads"     512 / 1024     workgroup size of the ring kernel
 *   "slice_lanes"      4 / 8          staged kernel: 64-byte column slices (4 lanes per token) where
 *                                     they exist (fp32 tables, tau 8 .. 10) / 128-byte ones (tau 7 .. 9);
 *                                     default: 128 bytes up to tau = 8, 64 bytes from tau = 9 on
 *   "small_tokens"     -1 / 1..2^20   lookupffn_forward: batches up to this many tokens take the single-launch
 *                                     kernel of lookupffn_forward_stack when the shape is that kernel's and no
 *                                     hash or gather path is forced (default 512; -1: never)
 *   "token_slots"      1 .. 32        staged kernels: at most this many tokens per lane group and chunk
 *   "hash_path"        1 / 2 / 3      1: always the generic hash kernel; 2: never the token-per-lane-row kernel
 *                                     (four tokens per wavefront at d_pad = 1024, eight at 512); 3: that kernel
 *                                     for every batch size.  Default for n_rounds <= 4: the lane-row kernel when
 *                                     d_pad is 1024 or 512, d is a multiple of 16, the batch has at least 2048
 *                                     tokens (4096 with weights; at d_pad = 512: 6144 and 12288), codes alone or
 *                                     codes and gather weights are asked for (not the multi-probe shares) and
 *                                     its constants fit 64 KB of LDS; else, at d_pad = 1024, the two-layout
 *                                     one-token-per-wavefront kernel; else the generic one
 *   "hash_blocks"      1..65536       grid cap of the lane-row and two-layout hash kernels
 * Returns LFFN_E_SIZE for an unknown key or a value outside the documented set.  Process-wide; a call
 * reads the knobs once when it starts.
 */
int lookupffn_set_option(const char *key, int value);

const char *lookupffn_strerror(int status);
/* Text of the last HIP error seen by this thread's most recent failing call ("" if none). */
const char *lookupffn_last_hip_error(void);
/* Which gather kernel the calling thread's most recent gather launch used: "gather_kernel" (direct, rows
 * fetched through L2), "gather_lds_kernel" (table slices staged in LDS, double-buffered) or
 * "forward_stack_kernel" (hash and gather of a few tokens in one launch), "gather_ring_kernel" (on request: prepared tables of up to 256 rows, plain sum; slices staged in an LDS ring,
 * token groups lagged so that their reads never meet in a bank); "" before the first launch. */
const char *lookupffn_last_gather_kernel(void);
/* The same for the sign-diagonal hash: "hash_row_kernel" (d_pad = 1024 or 512, a token per row of 16 or 8
 * lanes), "hash1024_kernel" (d_pad = 1024, one token per wavefront), "hash_kernel" (any width) or
 * "forward_stack_kernel"; "" before the first launch (the BH hash has one kernel and is not reported). */
const char *lookupffn_last_hash_kernel(void);
/* major*10000 + minor*100 + patch */
int lookupffn_version(void);

#ifdef __cplusplus
}
#endif
#endif /* LOOKUPFFN_H */
