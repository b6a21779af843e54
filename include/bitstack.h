/*
 * bitstack.h -- C ABI of the MI355X (gfx950) BitStack linear-layer library.
 *
 * A weight matrix W_t (out x in, PyTorch-linear orientation, y = W_t x) is held
 * as a stack of n residual blocks (BitStack, arxiv 2410.23918, Section 2.1):
 * block i is a +-1 sign matrix S_i (1 bit per weight, packed), and two rank-k
 * fp16 magnitude factors U_i (out x k) and V_i (in x k); a positive scale
 * vector s (one entry per input channel) comes from activation-aware scaling.
 * With the first n_loaded blocks resident the layer computes
 *
 *     y = ( sum_{i < n_loaded} S_i (.) (U_i V_i^T) ) diag(1/s) x        (Eq. 4, Eq. 8)
 *
 * without writing the reconstructed weight to device memory (the optional
 * materialising path further down restores it into a scratch buffer the caller
 * lends for the duration of a call).
 * (Paper orientation: X (p x m), W (m x n), Y = X W; here out = n_paper,
 *  in = m_paper, U = B', V = A', S = W_sign^T.)
 *
 * Conventions for every function
 *   - returns 0 (BITSTACK_OK) or a negative BITSTACK_E* code; never throws,
 *     never aborts; bitstack_strerror() names the code.
 *   - pointers marked "host" are ordinary host memory, "device" are HIP device
 *     pointers on the current device.  The library never allocates or frees
 *     device memory: all of it is owned by the caller (e.g. a torch tensor),
 *     which must keep it alive while a handle points into it.
 *   - fp16 values cross the ABI as raw IEEE binary16 bit patterns (uint16_t).
 *   - supported shapes: k == 16, in % 256 == 0, out % 32 == 0.
 *
 * Canonical sign packing (the bit-exact interchange format; the paper only says
 * the sign matrix is packed into an integer type, Section 2.1.2 / Fig. 3):
 * uint32 words, row-major [block][out][in/32]; bit b of word w of a row is
 * column 32*w + b; bit value 1 <=> S = +1; sign(0) = sign(-0) = +1.
 * The layout inside the device buffer is private to the library and round-trips
 * to the canonical form through bitstack_unpack_blocks().
 */
#ifndef BITSTACK_H
#define BITSTACK_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* hipStream_t is an opaque pointer; declared as void* so that this header does
 * not need the HIP headers.  NULL is the default stream. */
typedef void* bitstack_stream_t;

typedef struct bitstack_weight bitstack_weight_t; /* host handle of one packed stack */

enum {
    BITSTACK_OK        = 0,
    BITSTACK_E_NULL    = -1, /* a required pointer is NULL                        */
    BITSTACK_E_SHAPE   = -2, /* k != 16, in % 256, out % 32, or non-positive dims */
    BITSTACK_E_RANGE   = -3, /* n_loaded outside [0, n], batch outside [1, max]   */
    BITSTACK_E_ALIGN   = -4, /* device pointer not 16-byte (x, y) / 256-byte (buf) aligned */
    BITSTACK_E_SCALE   = -5, /* an entry of s is not finite or not > 0            */
    BITSTACK_E_BUFSIZE = -6, /* buffer smaller than bitstack_packed_bytes()       */
    BITSTACK_E_HIP     = -7, /* a HIP runtime call failed: bitstack_last_hip_error() */
    BITSTACK_E_ARG     = -8  /* unknown dtype / kernel selector, invalid block order */
};

/* output element types for bitstack_linear_batched */
enum { BITSTACK_Y_F16 = 0, BITSTACK_Y_F32 = 1 };

/* kernel selectors (bitstack_linear_select); AUTO is what bitstack_linear uses */
enum {
    BITSTACK_KERNEL_AUTO      = 0,
    BITSTACK_KERNEL_REFERENCE = 1, /* plain vector-ALU kernel, any batch <= max_batch            */
    BITSTACK_KERNEL_DECODE    = 2, /* matrix-core sign-stream kernel, up to 4 tokens per launch  */
    BITSTACK_KERNEL_PANEL     = 3, /* batch kernels: weight rebuilt on chip (Eq. 8) and multiplied
                                      with the activations on the matrix cores, any batch        */
    BITSTACK_KERNEL_MATERIALISE = 4 /* restore the weight to a dense scratch, then a dense product:
                                       the scratch lent to bitstack_linear_batched_ws, else the
                                       activation scratch inside an image packed with
                                       max_batch > 64 (BITSTACK_E_BUFSIZE if that holds fewer
                                       than 1024 rows of the dense weight)                       */
};

/* Bytes of one residual block: (out*in + 16*k*(out+in)) / 8, Eq. (9) of the
 * appendix on minimal transmission units.  This is the "block-stream" byte count
 * of the throughput metric.  Returns 0 for unsupported shapes. */
size_t bitstack_block_bytes(int out, int in, int k);

/* Device bytes bitstack_pack_blocks needs for a stack of n blocks: 1/s, the n
 * blocks (each contiguous and self-contained, exactly bitstack_block_bytes long),
 * per-channel maxima of V (in*2 bytes per block), an accumulation workspace
 * (n * in/1024 rows of out floats) and, for max_batch > 64, a scratch area of
 * max_batch (rounded up to 32) * in fp16 values in which a large batch of
 * activations is rearranged once per call.  0 for unsupported shapes. */
size_t bitstack_packed_bytes(int out, int in, int k, int n, int max_batch);

/* Host only.  Canonical packing of the sign matrix of a float residual:
 * bit = 1 where residual >= 0 (Section 2.1.2: W = W_sign (.) |W|, W_sign in {+-1}).
 * residual: host [out][in] float32; sign_words: host [out][in/32] uint32 (written). */
int bitstack_pack_signs_from_f32(int out, int in, const float* residual, uint32_t* sign_words);

/* Host only.  Builds the private device image of a whole stack in host memory
 * (what bitstack_pack_blocks copies to the device).  Lets the layout be tested
 * without a GPU.
 *   sign_words host [n][out][in/32] canonical; U host [n][out][k]; V host [n][in][k];
 *   s host [in], every entry finite and > 0; image host, image_bytes >=
 *   bitstack_packed_bytes(out,in,k,n,max_batch). */
int bitstack_pack_image_host(int out, int in, int k, int n, int max_batch,
                             const uint32_t* sign_words, const uint16_t* U, const uint16_t* V,
                             const float* s, void* image, size_t image_bytes);

/* Host only.  Inverse of bitstack_pack_image_host for one block: image ->
 * canonical sign words, U, V (any output pointer may be NULL to skip it). */
int bitstack_unpack_image_host(int out, int in, int k, int n, int max_batch,
                               const void* image, int block,
                               uint32_t* sign_words, uint16_t* U, uint16_t* V);

/* Packs a stack into caller-owned device memory and returns a handle
 * (Section 2: residual blocks are the units that are loaded into memory; a
 * weight is a stack of them, loaded in order).
 *   device_buf: device, 256-byte aligned, device_buf_bytes >= bitstack_packed_bytes().
 *   stream: copies are enqueued here and the stream is synchronised before return.
 *   handle: receives a library-owned host object; free it with bitstack_release().
 * The workspace part of the buffer is zeroed.  Two bitstack_linear calls that
 * use the same handle must not overlap in time (they share that workspace). */
int bitstack_pack_blocks(int out, int in, int k, int n, int max_batch,
                         const uint32_t* sign_words, const uint16_t* U, const uint16_t* V,
                         const float* s,
                         void* device_buf, size_t device_buf_bytes,
                         bitstack_stream_t stream, bitstack_weight_t** handle);

/* Device layout -> canonical form for one block (for bit-exactness tests).
 * Outputs are host arrays (NULL to skip).  Synchronises the stream. */
int bitstack_unpack_blocks(const bitstack_weight_t* w, int block,
                           uint32_t* sign_words, uint16_t* U, uint16_t* V,
                           bitstack_stream_t stream);

/* ---- Dynamic loading (Section 2.2: the model is a set of stacks of residual blocks that are
 * loaded into and offloaded from memory one block at a time, in stack order, as the available
 * memory changes; the appendix on minimal transmission units: a block is the unit that moves). */

/* Host bytes of one block in device form plus its derived per-channel maxima, as
 * bitstack_stage_block_host writes and bitstack_push_block reads them. */
size_t bitstack_block_staging_bytes(int out, int in, int k);

/* Host only.  Re-tiles one block (canonical sign words [out][in/32], U [out][k], V [in][k]) into
 * its device form in `staging` (host memory of the caller, ideally pinned, at least
 * bitstack_block_staging_bytes long). */
int bitstack_stage_block_host(int out, int in, int k, const uint32_t* sign_words, const uint16_t* U,
                              const uint16_t* V, void* staging, size_t staging_bytes);

/* A stack with room for n_slots blocks and none loaded: stores 1/s and clears the workspace
 * in caller-owned device memory of bitstack_packed_bytes(out,in,k,n_slots,max_batch) bytes.
 * Synchronises the stream before returning. */
int bitstack_create_stack(int out, int in, int k, int n_slots, int max_batch, const float* s,
                          void* device_buf, size_t device_buf_bytes, bitstack_stream_t stream,
                          bitstack_weight_t** handle);

/* Loads the next block of the stack (index = bitstack_resident_blocks) from a staged host copy:
 * two asynchronous host-to-device copies of exactly bitstack_block_bytes + in*2 bytes enqueued on
 * `stream`; calls enqueued on that stream afterwards may use the block.  `staging` must stay
 * unchanged until the copies have run.  BITSTACK_E_RANGE when every slot is taken. */
int bitstack_push_block(bitstack_weight_t* w, const void* staging, bitstack_stream_t stream);

/* The same from canonical arrays that already are in device memory (what bitstack_decompose
 * writes: one block's sign words [out][in/32], U [out][k] 16-byte aligned, V [in][k]): a
 * re-tiling kernel writes the block and its row maxima into the next free slot, no host copy.
 * The slot ends up byte for byte as bitstack_stage_block_host + bitstack_push_block leave it.
 * Asynchronous; the arrays must stay valid until the stream has passed the call. */
int bitstack_push_block_device(bitstack_weight_t* w, const uint32_t* sign_words, const uint16_t* U,
                               const uint16_t* V, bitstack_stream_t stream);

/* Offloads the last loaded block: no device work, its slot is free for the next push.  Calls
 * already enqueued that use the block must have finished before the slot is overwritten.
 * BITSTACK_E_RANGE when no block is loaded. */
int bitstack_pop_block(bitstack_weight_t* w);

/* Number of loaded blocks, and their bytes by Eq. (9): resident * bitstack_block_bytes. */
int bitstack_resident_blocks(const bitstack_weight_t* w);
size_t bitstack_resident_bytes(const bitstack_weight_t* w);

/* ---- Block manager: many stacks under one byte budget (Section 2.2: residual blocks are loaded
 * or offloaded as the available memory changes; Section 2.3: all blocks of all stacks sit in one
 * universal stack, level by level -- no stack takes its block i+1 before every stack has its
 * block i -- and inside a level in order of importance; Eq. 9 is the size of a block).
 * Host logic over bitstack_push_block / bitstack_pop_block; the importance scores that fix the
 * order inside a level come from the caller (the paper measures them on calibration data). */
typedef struct bitstack_manager bitstack_manager_t;

/* Host only.  Is `order` (entry e = index of the stack whose next block is loaded e-th) a valid
 * universal stack for stacks with slots[s] blocks each?  BITSTACK_E_ARG when some stack would
 * take block i+1 while another still lacks its block i, BITSTACK_E_RANGE for a stack index out
 * of range or more entries for a stack than it has blocks.  A prefix of a full order is valid. */
int bitstack_order_check(int n_stacks, const int* slots, const int* order, int count);

/* Host only.  How far down the universal stack a byte budget reaches: the largest `position`
 * such that the blocks of entries [0, position) fit, sum of block_bytes[order[e]] <= budget
 * (loading stops at the first block that does not fit: the order is an order of importance,
 * nothing is skipped).  *bytes (optional) receives that sum. */
int bitstack_budget_position(int n_stacks, const size_t* block_bytes, const int* order, int count,
                             size_t budget, int* position, size_t* bytes);

/* A manager over n_stacks stacks made by bitstack_create_stack, all empty; it keeps the
 * pointers (the stacks must outlive it and are not released by it). */
int bitstack_manager_create(int n_stacks, bitstack_weight_t* const* stacks, bitstack_manager_t** handle);
void bitstack_manager_release(bitstack_manager_t* m);

/* Where block `block` of stack `stack` waits in host memory (a buffer written by
 * bitstack_stage_block_host, caller-owned, unchanged while the manager lives; pinned memory
 * makes the copies asynchronous). */
int bitstack_manager_set_block(bitstack_manager_t* m, int stack, int block, const void* staging);

/* The universal stack (checked with bitstack_order_check against the stacks' slot counts).
 * Only while nothing is loaded (BITSTACK_E_ARG otherwise). */
int bitstack_manager_set_order(bitstack_manager_t* m, const int* order, int count);

/* Moves to the position bitstack_budget_position gives for budget_bytes: offloads from the top
 * of the universal stack (no device work) and/or loads the next entries (host-to-device copies
 * enqueued on `stream`; forward calls enqueued on that stream afterwards see the new blocks,
 * and calls enqueued on it earlier have read a popped slot before a later push overwrites it).
 * Bytes are counted by Eq. 9 exactly: afterwards bitstack_manager_resident_bytes <= budget and
 * the next entry, if any, does not fit.  *loaded / *offloaded (optional) count the blocks moved.
 * BITSTACK_E_NULL when a block on the way up has not been given with set_block: nothing moves. */
int bitstack_manager_set_budget(bitstack_manager_t* m, size_t budget_bytes, bitstack_stream_t stream,
                                int* loaded, int* offloaded);

/* Entries of the universal stack that are loaded; their bytes by Eq. 9; loaded blocks of one stack
 * (the n_loaded to pass to the forward calls). */
int bitstack_manager_position(const bitstack_manager_t* m);
size_t bitstack_manager_resident_bytes(const bitstack_manager_t* m);
int bitstack_manager_n_loaded(const bitstack_manager_t* m, int stack);

/* The forward pass for one token (batch-1 decode):
 *   y = ( sum_{i < n_loaded} S_i (.) (U_i V_i^T) ) diag(1/s) x           (Eq. 4 + Eq. 8)
 *   x: device fp16 [in], 16-byte aligned.   y: device fp16 [out], 16-byte aligned.
 *   n_loaded in [0, resident blocks]: the prefix of the stack to use; 0 gives y = 0.
 * Asynchronous: work is enqueued on stream and the call returns.
 * Accuracy: sums are exact integers or fp32 and y is rounded once; the one lossy step is the panel
 *   diag(x/s) V_i, held as 16-bit fixed point against its largest entry per block and range of up
 *   to 8192 columns, with groups of 32 columns that are at least 4x quieter kept 4x or 8x finer.
 *   Measured against an fp64 evaluation, max |y - y_ref| / max |y_ref| is 3e-4 ... 5e-4 for
 *   Gaussian activations and stays below 1e-3 with 1 to 32 channels 30x to 1000x above the
 *   rest and for heavy-tailed (Student-t, 3 degrees of freedom) activations; the bound this path
 *   is held to is 2e-3.  x/s is formed in fp32 and must stay finite in it; a zero x gives y = 0. */
int bitstack_linear(const void* x, const bitstack_weight_t* blocks, int n_loaded,
                    void* y, bitstack_stream_t stream);

/* A sequence of batch-1 forward passes enqueued back to back on one stream from
 * native code (one token through many linears, e.g. the 224 linears of a decoder,
 * each with its own n_loaded as the sorted stack leaves them, Section 2.2).
 * Same results as calling bitstack_linear(jobs[i].x, jobs[i].blocks, jobs[i].n_loaded,
 * jobs[i].y, stream) for i = 0..count-1, the whole list `repeat` times.
 * Up to four consecutive jobs that read the same x (the q/k/v or the gate/up projections
 * of a decoder layer) are independent of each other and are merged into one kernel
 * launch, provided they use different stacks, their outputs overlap neither each other
 * nor x, and the stacks' input widths agree; such jobs then run concurrently, not in
 * list order.  Stops at the first failing job or launch and returns its error. */
typedef struct bitstack_job {
    const void* x;                   /* device fp16 [in]  */
    const bitstack_weight_t* blocks; /* packed stack      */
    int n_loaded;
    void* y;                         /* device fp16 [out] */
} bitstack_job_t;
int bitstack_linear_many(const bitstack_job_t* jobs, int count, int repeat, bitstack_stream_t stream);

/* A token plan: the job list of bitstack_linear_many prepared once -- which consecutive jobs
 * share a launch, the work split of every launch, the kernels' argument blocks -- and then
 * launched once per token with no host work besides the launches themselves (a decoder sends
 * the same 224 linears through the library for every token; only the contents of the x and y
 * buffers change, Section 2.2's n_loaded per matrix stays until the memory budget moves).
 *   create: checks every job as bitstack_linear would (null pointers, n_loaded against the
 *           loaded blocks, alignment), enqueues nothing.  The plan keeps the pointers of the
 *           jobs (x, y, stacks), not the job array itself.
 *   launch: enqueues the plan's launches on `stream`.  Same bits in every y as
 *           bitstack_linear_many(jobs, count, 1, stream) gives for the same buffers.
 *           BITSTACK_E_RANGE if a stack now holds fewer blocks than its job uses: make a new
 *           plan after the budget has moved.
 *   steps:  number of kernel launches per bitstack_plan_launch.
 * A plan may be launched any number of times, also into a HIP graph capture (it allocates
 * nothing and records kernels only); it is not tied to a stream. */
typedef struct bitstack_plan bitstack_plan_t;
int bitstack_plan_create(const bitstack_job_t* jobs, int count, bitstack_plan_t** handle);
int bitstack_plan_launch(const bitstack_plan_t* plan, bitstack_stream_t stream);
int bitstack_plan_steps(const bitstack_plan_t* plan);
void bitstack_plan_release(bitstack_plan_t* plan);

/* Same for a batch of tokens.  x: device fp16 [batch][in] row-major;
 * y: device [batch][out] row-major of y_dtype (BITSTACK_Y_F16 / BITSTACK_Y_F32);
 * 1 <= batch <= max_batch given at pack time.  The library picks the kernel from the shape,
 * the batch and the number of loaded blocks; for prefill-sized batches that can be the
 * materialising path below in row slabs through the image's own activation scratch
 * (max_batch x in x 2 bytes, there in every image packed with max_batch > 64), when that
 * holds at least 1024 rows of the dense weight. */
int bitstack_linear_batched(const void* x, int batch, const bitstack_weight_t* blocks,
                            int n_loaded, void* y, int y_dtype, bitstack_stream_t stream);

/* As bitstack_linear_batched with an explicit kernel choice (tests, benchmarks). */
int bitstack_linear_select(const void* x, int batch, const bitstack_weight_t* blocks,
                           int n_loaded, void* y, int y_dtype, int kernel,
                           bitstack_stream_t stream);

/* The materialising path (appendix "Inference with BitStack models", throughput of the
 * restoration levels: its level 2 restores the weight, then multiplies).  For prefill-sized
 * batches it is faster than the kernels that rebuild weight tiles on chip, at the price of
 * out x in x 2 bytes of scratch; one scratch buffer can serve every stack of a model.
 *
 * bitstack_restore_weight writes
 *     w_dense[o][j] = ( sum_{i < n_loaded} S_i[o][j] * (U_i V_i^T)[o][j] ) / s[j]     (Eq. 8, Eq. 4)
 * as fp16, row-major [out][in], summed in fp32 over the blocks and rounded once.
 *   w_dense: device, caller-owned, 256-byte aligned, w_dense_bytes >= bitstack_dense_bytes(out, in)
 *   (BITSTACK_E_BUFSIZE otherwise).  n_loaded in [0, min(resident blocks,
 *   bitstack_restore_max_blocks())], 0 gives a zero matrix; BITSTACK_E_RANGE otherwise, also when the
 *   loaded blocks take 4 GiB or more (the kernel reaches them through 32-bit offsets).
 * bitstack_linear_dense computes y = x w_dense^T for x device fp16 [batch][in], y device
 *   [batch][out] of y_dtype; `blocks` supplies the shape; 1 <= batch <= max_batch given at pack
 *   time (BITSTACK_E_RANGE otherwise); x and w_dense below 4 GiB each.
 *   w_dense must hold what bitstack_restore_weight wrote for a stack of the same shape.
 * bitstack_linear_materialised is the two in sequence on one stream; all arguments are checked
 *   before anything is enqueued.  Its scratch may be smaller than the whole matrix: with room for
 *   R rows (R a multiple of 256, at least 1024; BITSTACK_E_BUFSIZE below that) the weight is
 *   restored and multiplied in slabs of R rows, one after the other through the same scratch --
 *   same results, a few launches more, and a scratch that stays inside the last-level cache
 *   when it is a few tens of MB.
 * All three are asynchronous and allocate nothing. */
size_t bitstack_dense_bytes(int out, int in);
int bitstack_restore_max_blocks(void);

/* bitstack_linear_batched with an optional scratch buffer (device, caller-owned, 256-byte
 * aligned, may be NULL): when it holds at least 1024 rows of the dense weight (1024 x in x 2
 * bytes; the whole matrix, bitstack_dense_bytes(out, in), avoids slabs) and the materialising
 * path is estimated to be faster for this batch and stack height, that path is taken and
 * overwrites the buffer; otherwise the buffer is left alone.  A buffer smaller than the image's
 * own activation scratch is left alone too (the image's is used where the path is taken).
 * Same results contract and errors as bitstack_linear_batched.
 * bitstack_choose_kernel (host only, no device work) returns the BITSTACK_KERNEL_* value that
 * call would pick for a stack of this shape (BITSTACK_KERNEL_AUTO for n_loaded = 0, where y is
 * only cleared), or a negative error code for an unsupported shape / out-of-range arguments. */
int bitstack_linear_batched_ws(const void* x, int batch, const bitstack_weight_t* blocks,
                               int n_loaded, void* y, int y_dtype, void* workspace,
                               size_t workspace_bytes, bitstack_stream_t stream);
int bitstack_choose_kernel(int out, int in, int n_slots, int max_batch, int batch, int n_loaded,
                           size_t workspace_bytes);
int bitstack_restore_weight(const bitstack_weight_t* blocks, int n_loaded, void* w_dense,
                            size_t w_dense_bytes, bitstack_stream_t stream);
int bitstack_linear_dense(const void* x, int batch, const bitstack_weight_t* blocks,
                          const void* w_dense, void* y, int y_dtype, bitstack_stream_t stream);
int bitstack_linear_materialised(const void* x, int batch, const bitstack_weight_t* blocks,
                                 int n_loaded, void* w_dense, size_t w_dense_bytes, void* y,
                                 int y_dtype, bitstack_stream_t stream);

/* The decomposition itself on the device (Section 2.1: activation-aware scaling, Eq. 3-4, and
 * the iterative absolute value decomposition, Eq. 5-7):
 *     R_0 = W diag(s);   per block i:  S_i = sign(R_i) (sign(0) = +1),
 *     U_i V_i^T = the top-k singular triplets of |R_i| with sqrt(sigma) on either side (Eq. 2),
 *     rounded to fp16;   R_{i+1} = R_i - S_i (.) (U_i V_i^T)  with the factors as stored.
 * The singular triplets come from a block power (subspace) iteration with k + 16 columns and
 * `iterations` rounds (0 = 16; one round applies |R| |R|^T once; the residual norm after a block
 * exceeds the exact truncation's by ~3e-4 / 7e-5 / 2e-5 / 8e-6 relative with 8 / 12 / 16 / 20 rounds) followed by a Rayleigh-Ritz step.  The rounds multiply
 * bf16 copies of |R| on the matrix cores with fp32 sums; the Rayleigh-Ritz step, which fixes the
 * factors, works on the fp32 residual (small Gram, Cholesky and eigenvalue problems in fp64).
 *   W: device fp32 [out][in] row-major, 16-byte aligned (not modified).
 *   s: HOST fp32 [in], every entry finite and > 0 (BITSTACK_E_SCALE otherwise); copied to the
 *   device by a copy enqueued on stream: keep it valid and unchanged until the stream has passed it.
 *   sign_words: device uint32 [n][out][in/32], canonical layout (bit b of word w = column 32w+b,
 *   1 = +1);  U: device fp16 bits [n][out][k];  V: device fp16 bits [n][in][k] -- the inputs of
 *   bitstack_pack_blocks once copied to the host.
 *   workspace: device, caller-owned, 256-byte aligned, at least
 *   bitstack_decompose_workspace_bytes(out, in, k) bytes (BITSTACK_E_BUFSIZE otherwise); it holds
 *   the fp32 residual (out x in x 4 bytes), two bf16 copies of its absolute values (2 x out x
 *   in x 2 bytes) and the iteration's tall matrices.
 * Asynchronous, allocates nothing.  The factors of a block are unique only
 * up to the sign of each column pair and rotations inside clusters of equal singular values;
 * U_i V_i^T and the residual norms are what can be compared between implementations. */
size_t bitstack_decompose_workspace_bytes(int out, int in, int k);
int bitstack_decompose(const float* W, const float* s, int out, int in, int k, int n, int iterations,
                       uint32_t* sign_words, uint16_t* U, uint16_t* V, void* workspace,
                       size_t workspace_bytes, bitstack_stream_t stream);

/* For callers that cannot allocate or lend device memory (code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc): bitstack_linear
 * for one token with the split-accumulation workspace (partial rows, arrival
 * counters) in a static device array of the library instead of the stack's own
 * buffer.  Calls no allocating routine.  bitstack_static_workspace_bytes() is the
 * size of that array (4 MiB of partial rows + 64 KiB of counters); every GPU the
 * library runs on holds its own copy until the process ends.
 *   x, y, blocks, n_loaded, stream: as bitstack_linear (fp16 in, fp16 out).
 * BITSTACK_E_BUFSIZE when the stack's partial rows cannot fit the array in any
 * work split (out * 4 bytes * ceil(in / 8192) > 4 MiB): nothing is enqueued.
 * All calls on one GPU share the array: two calls that overlap in time on one
 * GPU (different streams, different threads) race, whatever their stacks; calls
 * on one stream are ordered and safe.  Same results as bitstack_linear up to the
 * order of the fp32 partial sums (the work split may differ). */
size_t bitstack_static_workspace_bytes(void);
int bitstack_linear_static(const void* x, const bitstack_weight_t* blocks, int n_loaded, void* y,
                           bitstack_stream_t stream);

/* Shape queries on a handle. */
int bitstack_weight_shape(const bitstack_weight_t* w, int* out, int* in, int* k, int* n,
                          int* max_batch);

/* Frees the host handle only; the device buffer stays the caller's. */
void bitstack_release(bitstack_weight_t* w);

const char* bitstack_strerror(int code);

/* hipError_t value of the most recent failing HIP call on this thread (0 if none). */
int bitstack_last_hip_error(void);

#ifdef __cplusplus
}
#endif
#endif /* BITSTACK_H */
