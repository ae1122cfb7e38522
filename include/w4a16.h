/*
 * w4a16.h - C ABI of the fused W4A16 skinny GEMM for AMD MI355X (gfx950).
 *
 * Operation (paper "Accelerating a Triton Fused Kernel for W4A16 Quantized Inference with
 * SplitK work decomposition", Section 2 first paragraph and Algorithm 1):
 *
 *     C[m, n] = A[m, k] . W[k, n],   W[kk, j] = (q[kk, j] - z[kk / g, j]) * s[kk / g, j]
 *
 * with q and z stored as 4-bit fields, eight per int32 word.  Dequantisation, the product and
 * the reduction of the split-k partial sums happen inside one kernel launch.
 *
 * Buffers (all DEVICE pointers, row-major, contiguous, 16-byte aligned, owned by the caller;
 * the library neither frees nor keeps them after the call's work has run):
 *     A        fp16   [m, k]             activations
 *     qweight  int32  [k / 8, n]         field i (bits 4i..4i+3) of word (r, j) is q[8r + i][j]
 *     scales   fp16   [k / g, n]
 *     qzeros   int32  [k / g, n / 8]     field i of word (gi, c) is z[gi][8c + i]
 *     C        fp16   [m, n]             overwritten (never accumulated into)
 * `stream` is a hipStream_t passed as void* (NULL = the null stream).  Calls enqueue work on
 * that stream and return without synchronising; results are valid once the stream is.
 *
 * Limits: m >= 1.  The paper's regime is m <= 16.  More rows are served too: the SplitK entry
 * points of every field width with group_size 128 or 256 (and, for w4a16_gemm_ex, tile_cols 0 or
 * 256, waves 0 or 4, reduce AUTO, ATOMIC_PK_F16 or ATOMIC_PK_F16_PHASE) take up to 64 rows per
 * launch as row tiles that share one pass over the weights; everything else, the data-parallel
 * kernel included, runs one launch per 16 rows, each streaming the weights again.  n a multiple of 8;
 * g (group_size) one of 32, 64, 128, 256; k a multiple of g; k * n < 2^32.  A split_k requested from w4a16_gemm must cut k into equal
 * shares of whole groups (k / split_k a multiple of g), as Algorithm 1 has it.  The library's own
 * choice (split_k == 0) and w4a16_gemm_ex are not bound by that: they deal out k in compute
 * groups (min(g, 128) consecutive k) to the k parts in order, the first ones getting one group
 * more when the count does not divide, so that any k (llama's 11008 = 86 groups) gets a
 * balanced launch.
 *
 * Return value: W4A16_OK or a negative W4A16_ERR_* code.  Argument checks run before any HIP
 * call, so they behave the same on a machine without a GPU.  Nothing is printed, nothing
 * aborts.
 *
 * Split-k scratch: depending on the reduction flavour (W4A16_REDUCE_*) the split-k entry points
 * keep partial sums, arrival counters or per-tile flags in scratch memory that every call leaves
 * as it found it (sums back at zero, counters one call further).  By default that memory is the
 * library's, one set of buffers per device (at most 16 * n 64-bit words, split_k * m * n floats
 * for the workspace flavour, and, for the in-kernel zeroing, 16 KiB * (1 + split_k) per distinct
 * split_k used), allocated by the first call that needs it (hipMalloc + a synchronous clear; use
 * w4a16_reserve_scratch to do that ahead of time) and never moved or freed before
 * w4a16_release_scratch: a buffer that is outgrown stays alive, so a HIP graph captured earlier
 * keeps working.  A call that would have to allocate while its stream is being captured returns
 * W4A16_ERR_STATE instead.  Split-k calls that overlap in time on one device share the library's
 * buffers and must not be issued on different streams; a caller with several streams gives each
 * its own memory with w4a16_set_workspace, and calls on different streams are then independent.
 *
 * Failure of the in-kernel zeroing (W4A16_REDUCE_ATOMIC_PK_F16_PHASE): its waits are bounded, so
 * a kernel always ends.  A wait that runs out (only possible when the per-tile words were
 * corrupted: overlapping calls on shared scratch, an aborted kernel) is counted, adds NaN to the
 * tile's first output pair, and raises a sticky per-device word in pinned host memory that every
 * later split-k call on the library's or a bound scratch checks first, without synchronising:
 * such calls return W4A16_ERR_STATE until w4a16_release_scratch.
 */
#ifndef W4A16_H
#define W4A16_H

#ifdef __cplusplus
extern "C" {
#endif

#define W4A16_OK 0
#define W4A16_ERR_NULL (-1)        /* a required pointer is NULL */
#define W4A16_ERR_SHAPE (-2)       /* m < 1, n % 8, bad group_size, k % group_size */
#define W4A16_ERR_SPLIT (-3)       /* split_k < 0; w4a16_gemm: k % split_k, (k / split_k) % group_size; _ex: more
                                      k parts than compute groups, uneven parts where they must be equal */
#define W4A16_ERR_UNSUPPORTED (-4) /* group_size not in {32,64,128,256}, misaligned pointer, bad tuning value,
                                      split_k above 65535 (the grid's second dimension) */
#define W4A16_ERR_HIP (-5)         /* a HIP runtime call failed (allocation, launch) */
#define W4A16_ERR_STATE (-6)       /* an earlier wait of the in-kernel zeroing ran out on this device (see above), or
                                      scratch would have to be allocated during a stream capture */
#define W4A16_ERR_LIMIT (-7)       /* beyond a fixed capacity: w4a16_gemm_static's static array, a bound workspace's
                                      n_max, the table of bound workspaces */

/* How split-k partial sums reach C (Section 2.1 of the paper discusses the atomic form). */
#define W4A16_REDUCE_AUTO 0
#define W4A16_REDUCE_ATOMIC_F32 1   /* fp32 atomic adds into scratch; last block of a tile rounds to fp16 */
#define W4A16_REDUCE_ATOMIC_PK_F16 2 /* packed-fp16 atomic adds straight into C (C zeroed by a fill kernel); every
                                       add rounds to fp16, so the error grows like sqrt(split_k) * 2e-4: the
                                       library's own choice of split_k stays at 32 or below with this flavour and
                                       the next but one, a requested split_k is taken as given */
#define W4A16_REDUCE_WORKSPACE 3    /* plain fp32 partial tiles in scratch; last block sums them in fixed order */
#define W4A16_REDUCE_ATOMIC_FIXED 4 /* 64-bit fixed-point atomic adds that also count arrivals: one round trip,
                                       order-independent (bit-reproducible) sum; split_k <= 64; partial sums
                                       are clamped to +-131071 (an fp16 infinity in C either way) and a NaN
                                       partial sum makes the element NaN */
#define W4A16_REDUCE_ATOMIC_PK_F16_PHASE 5 /* packed-fp16 atomic adds straight into C with no launch before the
                                       GEMM kernel: the first k slice's workgroup zeroes its tile of C inside
                                       the kernel and the others wait for that through a per-tile flag;
                                       split_k 2..64; n <= 65536 */

/*
 * SplitK kernel (Algorithm 1): the grid is (column tiles) x split_k; every workgroup owns one
 * output tile and a contiguous 1/split_k share of k, and adds its partial tile to the result.
 * split_k == 1 stores directly.  split_k == 0 lets the library choose.
 */
int w4a16_gemm(const void* A, const void* qweight, const void* scales, const void* qzeros, void* C,
               int m, int n, int k, int group_size, int split_k, void* stream);

/*
 * w4a16_gemm for callers that cannot allocate device memory (code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc): same operation, same kernels and launch plan,
 * but the split-k state lives in a static device array of the library (2.7 MiB per GPU, held
 * until the process ends) instead of allocated buffers.  The call allocates nothing and frees
 * nothing.  Limits: m <= 16, n <= 16384, and a split_k (given or chosen) of at most 32 when
 * m > 4; beyond them W4A16_ERR_LIMIT.  All calls on one GPU share the array, which every call
 * leaves as it found it; calls that overlap in time on one GPU (different streams) race on it
 * and must not be issued.  A wait of the in-kernel zeroing that runs out is counted
 * (w4a16_phase_timeouts) and poisons its tile with NaN, but raises no sticky error here.
 */
int w4a16_gemm_static(const void* A, const void* qweight, const void* scales, const void* qzeros, void* C,
                      int m, int n, int k, int group_size, int split_k, void* stream);

/*
 * Data-parallel tiled kernel (Section 3, first paragraph: one workgroup alone computes a whole
 * output tile over all of k and stores it; no atomics, no scratch).  Deterministic.
 */
int w4a16_gemm_dp(const void* A, const void* qweight, const void* scales, const void* qzeros, void* C,
                  int m, int n, int k, int group_size, void* stream);

/*
 * StreamK decomposition (the paper's Conclusion names it as the successor of SplitK to explore):
 * `workgroups` persistent workgroups (0 = library default, one per compute unit) share the
 * iterations (256-column tile x 128 consecutive k) evenly, whatever the shape; each adds the
 * pieces of the tiles it touched to C with packed-fp16 atomic adds (C zeroed by a fill kernel
 * on the same stream) and stores the tiles it computed alone.  group_size 128 or 256
 * (W4A16_ERR_UNSUPPORTED otherwise); no scratch; more than 16 rows run one launch per 16.
 */
int w4a16_gemm_streamk(const void* A, const void* qweight, const void* scales, const void* qzeros, void* C,
                       int m, int n, int k, int group_size, int workgroups, void* stream);
/* The same decomposition for the other field widths (bits = 8, 3, 2 with the layouts described below; 4 is
 * w4a16_gemm_streamk itself; W4A16_ERR_UNSUPPORTED for any other width). */
int w4a16_gemm_streamk_bits(int bits, const void* A, const void* qweight, const void* scales, const void* qzeros,
                            void* C, int m, int n, int k, int group_size, int workgroups, void* stream);

/*
 * 8-bit fields (Section 2 of the paper remarks that the method carries over to other n-bit
 * quantisation schemes).  Same operation and rules as w4a16_gemm / w4a16_gemm_dp with four
 * fields per word:
 *     qweight  int32  [k / 4, n]         field i (bits 8i..8i+7) of word (r, j) is q[4r + i][j], 0..255
 *     qzeros   int32  [k / g, n / 4]     field i of word (gi, c) is z[gi][4c + i]
 * The launch is the library's (per-wave kernel, two strips per wave or streaming kernel for SplitK;
 * 16- to 64-column tiles for the data-parallel kernel; w4a16_plan_bits reports it); more than 16
 * rows as described above (row tiles of the streaming kernel for SplitK).  w8a16_algorithmic_bytes: qweight + scales + qzeros + A + C for
 * this layout.
 */
int w8a16_gemm(const void* A, const void* qweight, const void* scales, const void* qzeros, void* C,
               int m, int n, int k, int group_size, int split_k, void* stream);
int w8a16_gemm_dp(const void* A, const void* qweight, const void* scales, const void* qzeros, void* C,
                  int m, int n, int k, int group_size, void* stream);
long long w8a16_algorithmic_bytes(int m, int n, int k, int group_size);

/*
 * 2-bit fields, sixteen per word, in the same way:
 *     qweight  int32  [k / 16, n]        field i (bits 2i, 2i+1) of word (r, j) is q[16r + i][j], 0..3
 *     qzeros   int32  [k / g, n / 16]    field i of word (gi, c) is z[gi][16c + i]
 * n must be a multiple of 16 (W4A16_ERR_SHAPE otherwise).
 */
int w2a16_gemm(const void* A, const void* qweight, const void* scales, const void* qzeros, void* C,
               int m, int n, int k, int group_size, int split_k, void* stream);
int w2a16_gemm_dp(const void* A, const void* qweight, const void* scales, const void* qzeros, void* C,
                  int m, int n, int k, int group_size, void* stream);
long long w2a16_algorithmic_bytes(int m, int n, int k, int group_size);

/*
 * 3-bit fields (Section 2's remark again; a width that does not divide 32).  32 consecutive
 * values form a stream of 96 bits, value u at stream bits [3u, 3u + 2], low bit first; stream bit
 * b is bit (b % 32) of word (b / 32) of three consecutive words (the layout of GPTQ's 3-bit
 * checkpoints), so values 10 and 21 of a stream lie across two words:
 *     qweight  int32  [3 k / 32, n]      word rows 3t, 3t+1, 3t+2 of column j: q[32t .. 32t+31][j], 0..7
 *     qzeros   int32  [k / g, 3 n / 32]  words 3t, 3t+1, 3t+2 of row gi: z[gi][32t .. 32t+31]
 * n must be a multiple of 32 (W4A16_ERR_SHAPE otherwise).  Otherwise as w8a16_gemm.
 */
int w3a16_gemm(const void* A, const void* qweight, const void* scales, const void* qzeros, void* C,
               int m, int n, int k, int group_size, int split_k, void* stream);
int w3a16_gemm_dp(const void* A, const void* qweight, const void* scales, const void* qzeros, void* C,
                  int m, int n, int k, int group_size, void* stream);
long long w3a16_algorithmic_bytes(int m, int n, int k, int group_size);

/*
 * Activation ordering (GPTQ's act-order; outside the paper, whose groups are contiguous runs of
 * k): the group of row kk is g_idx[kk] instead of kk / g, W[kk, j] = (q[kk, j] - z[g_idx[kk], j])
 * * s[g_idx[kk], j], where g_idx (device, int32 [k]) gives every group exactly g rows.
 *
 * w4a16_actorder_prepare, once per weight matrix: perm (device, int32 [k]) <- the rows sorted
 * by group, ascending row order inside a group; qweight_sorted (device, int32 [k / 8, n], not
 * qweight itself) <- the rows of qweight in that order; *status (device, int32) <- 0, or 1 when
 * some group does not have exactly g rows (then perm and qweight_sorted are unusable; no access
 * leaves the buffers whatever g_idx holds).  Asynchronous on `stream` like everything else; it
 * clears *status with a small kernel, so it can be captured in a HIP graph.
 *
 * w4a16_gemm_actorder, per call: A_work (device, fp16 [m, k], 16-byte aligned, caller's scratch,
 * not A) <- A[:, perm], then the SplitK GEMM of A_work with qweight_sorted, scales and qzeros as
 * w4a16_gemm does it (same rules for split_k).  The gather is one more small kernel per call; a
 * caller whose previous operation can write A[:, perm] itself passes that to w4a16_gemm together
 * with qweight_sorted and needs no gather.
 */
int w4a16_actorder_prepare(const void* qweight, const void* g_idx, void* qweight_sorted, void* perm, void* status,
                           int n, int k, int group_size, void* stream);
int w4a16_gemm_actorder(const void* A, const void* qweight_sorted, const void* scales, const void* qzeros,
                        const void* perm, void* A_work, void* C, int m, int n, int k, int group_size, int split_k,
                        void* stream);

/*
 * Same operations with the tuning knobs exposed (0 = library default for each):
 *   tile_cols  output columns per workgroup: 16, 32 or 64 (every wave owns the whole tile and the
 *              waves divide the workgroup's k range), 128 (SplitK only, group_size 128 or 256:
 *              as 64, but every wave multiplies its activations with two adjacent 64-column
 *              strips; split_k * waves must equal k / 128, waves <= 4, split_k 2..64,
 *              reduce W4A16_REDUCE_AUTO or W4A16_REDUCE_ATOMIC_PK_F16_PHASE), or 256 (SplitK only, group_size 128 or
 *              256: four waves own a 64-column strip each and share their activations
 *              through LDS; waves = 4 or 8, i.e. one or two such sets dividing the k range;
 *              reduce W4A16_REDUCE_ATOMIC_PK_F16 or W4A16_REDUCE_ATOMIC_PK_F16_PHASE)
 *   waves      wavefronts per workgroup, 1..16
 *   reduce     one of W4A16_REDUCE_* (ignored when split_k == 1)
 * split_k here is any value >= 1 (0 = library default) with split_k * (k parts of a workgroup:
 * waves, or waves / 4 for 256-column tiles) <= k / min(group_size, 128); the parts' shares may
 * differ by one compute group, except with 256-column tiles and 8 waves, whose two k parts meet
 * at a barrier per group and must be equal (W4A16_ERR_SPLIT otherwise).
 */
int w4a16_gemm_ex(const void* A, const void* qweight, const void* scales, const void* qzeros, void* C,
                  int m, int n, int k, int group_size, int split_k,
                  int tile_cols, int waves, int reduce, void* stream);
int w4a16_gemm_dp_ex(const void* A, const void* qweight, const void* scales, const void* qzeros, void* C,
                     int m, int n, int k, int group_size, int tile_cols, int waves, void* stream);

/*
 * The launch the library would use: fills split_k, tile_cols, waves, reduce (any may be NULL)
 * for a SplitK call (dp == 0) or a data-parallel call (dp != 0).  Host only; no HIP call.
 * `split_k` in: the requested value (0 = choose).
 */
int w4a16_plan(int m, int n, int k, int group_size, int dp, int* split_k, int* tile_cols, int* waves, int* reduce);
/* The same for w8a16_gemm, w3a16_gemm, w2a16_gemm and their _dp forms (bits = 8, 3, 2; 4 = w4a16_plan):
 * the values are outputs only, except `split_k` in.  W4A16_ERR_UNSUPPORTED for any other width. */
int w4a16_plan_bits(int bits, int m, int n, int k, int group_size, int dp, int* split_k, int* tile_cols,
                    int* waves, int* reduce);

/* Argument check alone (host only, no HIP call): what w4a16_gemm would return before launching
 * (equal shares required of a requested split_k). */
int w4a16_check(int m, int n, int k, int group_size, int split_k);

/*
 * Test probes that run the same device unpack / dequantise routines as the GEMM kernels.
 *   w4a16_unpack:  q_u8 [k, n] and z_u8 [k / g, n] (device, uint8) <- the 4-bit fields
 *   w4a16_dequant: W fp16 [k, n] (device) <- fp16_rne((q - z) * s)
 */
int w4a16_unpack(const void* qweight, const void* qzeros, void* q_u8, void* z_u8,
                 int n, int k, int group_size, void* stream);
int w4a16_dequant(const void* qweight, const void* scales, const void* qzeros, void* W,
                  int n, int k, int group_size, void* stream);

/*
 * Measurement probe: a plain coalesced read of `bytes` (a multiple of 16) from a 16-byte aligned
 * device buffer, result discarded.  Timed like a GEMM call on the same buffers it gives the
 * ceiling that any kernel which has to read them can reach on this machine.  `shape` 0..4
 * picks one of five launch shapes (loads in flight per lane x workgroups x threads: 8 x one
 * pass x 256, 8 x 2048 x 256, 4 x 2048 x 512, 2 x 8192 x 256, 1 x 16384 x 256), 5..9 the same
 * five with the non-temporal hint on the loads; which is fastest depends on the size, so a
 * bench takes the best of them.  Any other shape: W4A16_ERR_UNSUPPORTED.
 */
int w4a16_read_probe(const void* buffer, long long bytes, int shape, void* stream);

/* Bytes every call has to move at least once: qweight + scales + qzeros + A + C. */
long long w4a16_algorithmic_bytes(int m, int n, int k, int group_size);

/* Static text for a return code. */
const char* w4a16_strerror(int code);

/* After a W4A16_ERR_HIP on this host thread: which HIP call failed and HIP's text for it. */
const char* w4a16_last_hip_error(void);

/*
 * W4A16_REDUCE_ATOMIC_PK_F16_PHASE only: how many wavefronts on the current device have so far
 * given up waiting for a tile's zeroing (library scratch, bound workspaces and the static array
 * together).  0 unless the per-tile words were corrupted, e.g. by two overlapping calls or an
 * aborted kernel; releasing the scratch resets them.  Synchronises the device.  Negative: a
 * W4A16_ERR_* code.
 */
long long w4a16_phase_timeouts(void);

/*
 * Test hook for the failure path above: the number of polls after which a wait gives up
 * (0 = the library's default, 131072).  A kernel ends normally whatever the value.
 */
int w4a16_set_phase_spin_limit(int polls);

/*
 * A caller-owned workspace for the split-k state of the calls issued on `stream` (current device):
 * `workspace` is device memory, 256-byte aligned, of at least w4a16_workspace_bytes(n_max) bytes
 * (about 34 MiB + 192 bytes per column; 0 for a bad n_max: a multiple of 8 up to 65536), which
 * the caller keeps alive and untouched while bound.  The call clears it on `stream` (a kernel, so
 * it may be captured) and binds it: from then on calls on that stream with n <= n_max use it and
 * are independent of calls on other streams; n > n_max returns W4A16_ERR_LIMIT.  Only the partial
 * tiles of W4A16_REDUCE_WORKSPACE, which have no bound, stay in the library's own buffer.
 * workspace == NULL unbinds the stream.  Up to 64 bindings per process.
 */
long long w4a16_workspace_bytes(int n_max);
int w4a16_set_workspace(void* workspace, long long bytes, int n_max, void* stream);

/*
 * Allocate, now, everything the library's own scratch can need for calls with up to n_max columns
 * (about 36 MiB at n_max = 16384), so that no later call allocates, e.g. before capturing graphs.
 */
int w4a16_reserve_scratch(int n_max);

/*
 * Release the library's scratch of the current device, retired buffers included (synchronises the
 * device), forget its bound workspaces, clear the static array and the sticky error.  Graphs
 * captured before this call must not be replayed after it.
 */
int w4a16_release_scratch(void);

#ifdef __cplusplus
}
#endif
#endif /* W4A16_H */
