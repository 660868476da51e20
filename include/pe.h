/*
 * pe.h — C ABI of the Parallel Evoformer block for AMD MI355X (gfx950).
 *
 * The block is the one proposed in "Efficient AlphaFold2 Training using
 * Parallel Evoformer and Branch Parallelism" (Section "Parallel Evoformer",
 * Figure 1(c)): the MSA branch (row-wise gated self-attention with pair bias,
 * column-wise gated self-attention, transition) and the pair branch (triangle
 * multiplicative update outgoing/incoming, triangle self-attention around
 * starting/ending node, transition) are independent inside a block, and the
 * outer product mean of the MSA branch's output is added to the pair branch's
 * output at the end of the block.  The sub-operations are the ones named in
 * Section "Evoformer"; their definitions follow AlphaFold2, to which the paper
 * defers.  Section "Branch Parallelism" places the two branches on two
 * devices; this library runs them on two HIP streams of one device and
 * replaces the broadcast / all-reduce of that section by event waits and one
 * add (gradient of the input pair representation = pair-branch term +
 * row-attention-bias term).
 *
 * Conventions
 *  - All tensor pointers are DEVICE pointers unless stated otherwise.
 *    msa[s][r][c_m] and pair[r][r][c_z] are row-major, channel fastest, of the
 *    storage type dims->dtype (fp32 or bf16).  Masks and parameters are fp32.
 *  - The caller owns every buffer and both streams.  The library allocates no
 *    device memory in the compute calls; scratch comes from `workspace`.
 *  - Calls only ENQUEUE work.  At entry stream_pair is made to wait for the
 *    work already queued on stream_msa (inputs have to be ready with respect
 *    to stream_msa); at return both streams are joined, so outputs may be
 *    consumed on either stream.  stream_msa == stream_pair is allowed and
 *    serialises the branches.
 *  - Results are deterministic: no atomics, every reduction in a fixed order.
 *    A call that has the device to itself (stream_msa == stream_pair, one
 *    branch selected with PE_OPT_BRANCHES, or PE_VARIANT_AF2, whose data flow
 *    is serial) takes a parameter-gradient kernel
 *    that sums the contraction index in another fixed order than the
 *    two-stream call does: outputs and input cotangents are bit-identical
 *    between the two modes, bf16-path parameter gradients agree to fp32
 *    rounding.
 *  - Return value 0 = PE_OK, negative = error (see pe_strerror).  Arguments
 *    are validated before anything is launched.
 */
#ifndef PE_H
#define PE_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

enum { PE_F32 = 0, PE_BF16 = 1 };

/* Block orderings of Figure 1.  The sub-operations and parameters are the same; only the place of
 * the outer product mean differs.
 *   PE_VARIANT_PARALLEL (c): both stacks read the block's inputs, the outer product mean of the
 *     MSA stack's output is added to the pair stack's output (the two stacks overlap on two streams).
 *   PE_VARIANT_AF2 (a): the outer product mean of the MSA stack's output is added to the pair
 *     representation before the pair stack (serial; row attention is biased by the block's input).
 *   PE_VARIANT_MULTIMER (b): the outer product mean of the block's input MSA representation is
 *     added to the pair representation first; row attention's bias and the pair stack read that
 *     sum (the stacks overlap after the outer product mean).                                     */
enum { PE_VARIANT_PARALLEL = 0, PE_VARIANT_AF2 = 1, PE_VARIANT_MULTIMER = 2 };

enum {
  PE_OK = 0,
  PE_ERR_NULL = -1,      /* a required pointer is NULL                               */
  PE_ERR_DIMS = -2,      /* unsupported dims (see pe_check_dims)                     */
  PE_ERR_WORKSPACE = -3, /* workspace smaller than pe_workspace_bytes / stack bytes  */
  PE_ERR_ALIAS = -4,     /* a buffer the call writes (outputs, ctx of the forward, d_params, workspace)
                            overlaps another buffer of the call                       */
  PE_ERR_HIP = -5,       /* a HIP call failed; text in pe_last_error                 */
  PE_ERR_ARG = -6        /* bad option / count / capacity                            */
};

/* Shape of one block.  Requirements checked by pe_check_dims (pe_dims_error names the one that
 * failed):
 *   s, r >= 1 with s*r < 2^31 and r*r < 2^31; n_trans >= 1;
 *   c_m, c_z, h_msa*d_msa, h_pair*d_pair, c_tri, c_opm: multiples of 8 in [8, 1024], and
 *     c_z <= 256, c_tri <= 192, n_trans*c_m <= 4096, n_trans*c_z <= 4096;
 *   h_msa, h_pair in [1, 8]; d_msa, d_pair in {8, 16, 24, 32};
 *   col_global in {0, 1}; with col_global = 1 additionally d_msa <= 8;
 *   dtype PE_F32 or PE_BF16; variant one of PE_VARIANT_*; ln_eps, opm_eps > 0.                    */
typedef struct pe_dims {
  int s, r, c_m, c_z;    /* msa[s,r,c_m], pair[r,r,c_z]                              */
  int h_msa, d_msa;      /* MSA attention heads x head dim                           */
  int h_pair, d_pair;    /* triangle attention heads x head dim                      */
  int c_tri, c_opm;      /* triangle-multiplication hidden, outer-product hidden     */
  int n_trans;           /* transition expansion factor                              */
  int col_global;        /* 0 column attention, 1 global column attention (extra MSA)*/
  int dtype;             /* PE_F32 | PE_BF16: storage of activations and cotangents  */
  float ln_eps;          /* LayerNorm epsilon (1e-5)                                 */
  float opm_eps;         /* outer-product-mean normaliser epsilon (1e-3)             */
  int variant;           /* where the outer product mean sits (Figure 1): PE_VARIANT_* */
} pe_dims;

typedef struct pe_handle pe_handle;

/* One entry of the flat fp32 parameter buffer (the paper's fusion of all
 * parameter tensors into one tensor).  Weight matrices are row-major
 * [in, out] = shape[0] x shape[1]; vectors have ndim 1.
 * kind: 0 weight, 1 LayerNorm gain, 2 LayerNorm offset, 3 bias.             */
typedef struct pe_param_entry {
  char name[32];
  long long offset;      /* in fp32 elements from the start of the block's parameters */
  int ndim;
  int shape[2];
  int fan_in;            /* rows of a weight matrix, 0 for vectors                   */
  int kind;
} pe_param_entry;

/* One saved activation inside ctx (introspection for tests and debugging).
 * dtype: PE_F32 or PE_BF16 storage of that entry.                            */
typedef struct pe_ctx_entry {
  char name[32];
  long long offset_bytes;
  long long count;       /* elements */
  int dtype;
} pe_ctx_entry;

/* Handle: owns a few hipEvents used to fork/join the streams and, once
 * PE_OPT_SIDE_STREAMS has been set, two side streams (default priority).
 * Host state only.  Not thread safe: one handle per host thread; calls on one
 * handle must not overlap.  The compute calls may be captured into a HIP
 * graph by the caller (they allocate nothing, never synchronise the host and
 * record no memset nodes); keep PE_OPT_KERNEL_TIMING and PE_OPT_SYNC_DEBUG off
 * while capturing.                                                            */
int pe_create(pe_handle** h);
int pe_destroy(pe_handle* h);

/* Options.  PE_OPT_BRANCHES: bit 0 = run the MSA branch (+ outer product
 * mean), bit 1 = run the pair branch; default 3.  With a branch disabled its
 * outputs are left untouched (used to time each branch alone; only
 * PE_VARIANT_PARALLEL has independent branches, the other variants return
 * PE_ERR_ARG unless both bits are set).
 * PE_OPT_SYNC_DEBUG: 1 = hipStreamSynchronize + error check after each
 * sub-operation (slow; for fault isolation).
 * PE_OPT_KERNEL_TIMING: 1 = bracket every kernel launch with a pair of HIP
 * events on the stream it is launched on; read the result with
 * pe_timing_collect (measurement only: events add launch overhead).
 * PE_OPT_SIDE_STREAMS (default 0): 1 = the backward pass runs parameter-
 * gradient kernels (dW GEMMs, bias sums, partial reductions) on one library-
 * owned side stream per branch, forked from / joined to the caller's streams
 * with events; results are bit-identical.  Measured slower on MI355X (each
 * cross-stream event wait costs more than the overlap wins), hence off.
 * PE_OPT_STACK_KEEP_CTX (default 0): 1 = pe_stack_fwd_bwd keeps every block's
 * saved activations (pe_stack_workspace_bytes_keep bytes of workspace: about
 * 1.3 GiB per main block at s=128, r=256, which 288 GB of HBM hold for the whole
 * trunk) and recomputes nothing; results are bit-identical to the default,
 * which saves block inputs only and recomputes each block's forward.
 * PE_OPT_STACK_OVERLAP (default 0): 1 = with PE_OPT_STACK_KEEP_CTX and two distinct streams,
 * pe_stack_fwd_bwd enqueues the part of the NEXT block's forward that needs the new MSA
 * representation only (weight preparation of the MSA branch, LayerNorm and q / k / v / gate
 * projection of the row attention) on stream_msa before the current block's outer product
 * mean waits for the pair branch (Section "Branch Parallelism": the MSA representation is final
 * before the outer product mean; the next row attention needs the new pair representation for
 * its bias only).  Results are bit-identical.  Measured without gain on one MI355X (the chip
 * is already full beside the pair branch's tail), hence off.                                 */
enum { PE_OPT_BRANCHES = 1, PE_OPT_SYNC_DEBUG = 2, PE_OPT_KERNEL_TIMING = 3, PE_OPT_SIDE_STREAMS = 4,
       PE_OPT_STACK_KEEP_CTX = 5, PE_OPT_STACK_OVERLAP = 6 };
int pe_set_option(pe_handle* h, int option, int value);

/* Per-kernel timing since the last collect, aggregated by launch label.
 * flops / bytes are the ALGORITHMIC work of those launches (2*M*N*K per
 * contraction; minimal reads + writes for the memory-bound kernels).
 * pe_timing_collect synchronises the device and returns the number of
 * entries; with out == NULL it only reports that number, otherwise it fills
 * out (cap >= number) and clears the records.                                */
typedef struct pe_timing_entry {
  char name[32];         /* launch label, e.g. "attn qkvg"                           */
  char kernel[64];       /* kernel (template) name the label ran                     */
  int launches;
  double total_ms;
  double flops;
  double bytes;
} pe_timing_entry;
int pe_timing_collect(pe_handle* h, pe_timing_entry* out, int cap);

/* Host-side shape queries (no GPU needed). */
int pe_check_dims(const pe_dims* d);                                   /* PE_OK or PE_ERR_DIMS */
const char* pe_dims_error(const pe_dims* d);   /* which requirement pe_check_dims found violated ("" if none); static text */
long long pe_param_count(const pe_dims* d);                            /* fp32 elements / block */
int pe_param_table(const pe_dims* d, pe_param_entry* out, int cap);    /* returns #entries      */
int pe_ctx_table(const pe_dims* d, pe_ctx_entry* out, int cap);        /* returns #entries      */
size_t pe_ctx_bytes(const pe_dims* d);                                 /* saved activations + prepared weights */
/* Scratch needed by pe_block_fwd / pe_block_bwd: the two branches' work
 * arenas plus, for the backward pass, the fp32 partial sums of every
 * parameter gradient of the block (they are reduced into d_params at the end
 * of the call).  with_ctx != 0 adds room for an internal ctx (needed when
 * ctx == NULL is passed to pe_block_bwd).                                   */
size_t pe_workspace_bytes(const pe_dims* d, int with_ctx);
/* Scratch needed by pe_stack_fwd_bwd (saved block inputs + one block's needs). */
size_t pe_stack_workspace_bytes(int n_extra, const pe_dims* extra, int n_main, const pe_dims* main_);
/* The same with PE_OPT_STACK_KEEP_CTX set (every block's ctx kept, no recompute). */
size_t pe_stack_workspace_bytes_keep(int n_extra, const pe_dims* extra, int n_main, const pe_dims* main_);

/* Forward of one Parallel Evoformer block (Figure 1(c)).
 *   msa_in [s,r,c_m], pair_in [r,r,c_z]: inputs (dtype per dims), read only.
 *   msa_mask [s,r], pair_mask [r,r]: fp32 0/1.  A masked key gets attention
 *     weight exactly 0, a softmax row without valid key gives 0; triangle and
 *     outer-product projections are multiplied by the mask.
 *   params: fp32 flat buffer, pe_param_count elements, layout pe_param_table.
 *   msa_out, pair_out: outputs, must not alias any input.
 *   ctx: NULL, or pe_ctx_bytes bytes (256-byte aligned) that receive the
 *     activations saved for pe_block_bwd and the storage-type (transposed and
 *     plain) copies of the weights the kernels read.  pe_block_bwd with this
 *     ctx uses those copies: params must be unchanged between the two calls.
 *   workspace: 256-byte aligned, >= pe_workspace_bytes(dims, ctx == NULL)
 *     bytes (without a caller ctx the intermediates live in the workspace).
 *   stream_msa, stream_pair: hipStream_t (NULL = default stream).            */
int pe_block_fwd(pe_handle* h, const pe_dims* dims,
                 const void* msa_in, const void* pair_in,
                 const float* msa_mask, const float* pair_mask,
                 const float* params,
                 void* msa_out, void* pair_out,
                 void* ctx,
                 void* workspace, size_t workspace_bytes,
                 void* stream_msa, void* stream_pair);

/* For callers that cannot allocate device memory (code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc): pe_block_fwd without ctx and without a workspace
 * argument.  The scratch that pe_block_fwd carves from `workspace` (work arenas, internal saved
 * activations, prepared weights) comes from one array that the library holds in device memory on
 * every device it is loaded on, pe_static_scratch_bytes() = 32 MiB, from load until the process
 * ends; its address on the handle's device is looked up once in pe_create.  The call allocates
 * nothing (no hipMalloc / hipFree, no allocating library routine) and only enqueues.
 *   Arguments as pe_block_fwd; the caller still passes inputs and outputs.
 *   Returns PE_ERR_WORKSPACE (sizes in pe_last_error) when pe_workspace_bytes(dims, 1) exceeds
 *   pe_static_scratch_bytes(): e.g. s=24, r=48 at the tiny channel widths fits, s=128, r=256 does
 *   not.  PE_ERR_ARG when the current device is not the one the handle was created on.
 *   Every call on a device shares that device's array, which keeps the last call's contents
 *   (nothing in it has to start at zero: every kernel writes what it later reads).  Calls that
 *   overlap on one device — two handles, two host threads, or a second call enqueued on other
 *   streams before the first has finished — race on it; order them (same streams, or an event). */
size_t pe_static_scratch_bytes(void);
int pe_block_fwd_static(pe_handle* h, const pe_dims* dims,
                        const void* msa_in, const void* pair_in,
                        const float* msa_mask, const float* pair_mask,
                        const float* params,
                        void* msa_out, void* pair_out,
                        void* stream_msa, void* stream_pair);

/* Backward of one block (data flow of Section "Branch Parallelism": the
 * cotangent of the pair output feeds the pair branch AND the outer product
 * mean; d_pair_in = pair-branch term + row-attention-bias term).
 *   d_msa_out, d_pair_out: cotangents of the outputs (dtype per dims).
 *   d_msa_in, d_pair_in: overwritten with the input cotangents.
 *   d_params: fp32 flat, same layout as params, ACCUMULATED (+=).
 *   ctx: what pe_block_fwd wrote for the same inputs, or NULL: then the
 *     forward is recomputed internally and workspace must hold
 *     pe_workspace_bytes(dims, 1).                                           */
int pe_block_bwd(pe_handle* h, const pe_dims* dims,
                 const void* msa_in, const void* pair_in,
                 const float* msa_mask, const float* pair_mask,
                 const float* params,
                 const void* d_msa_out, const void* d_pair_out,
                 void* d_msa_in, void* d_pair_in,
                 float* d_params,
                 const void* ctx,
                 void* workspace, size_t workspace_bytes,
                 void* stream_msa, void* stream_pair);

/* Forward and backward of a trunk: n_extra extra-MSA blocks (dims `extra`,
 * operating on extra_msa and pair) followed by n_main main blocks (dims
 * `main_`, operating on msa and pair); Figure 2 caption: the extra MSA stack is
 * made of Evoformer blocks, 52 = 4 + 48.  Only the pair representation flows
 * from the extra blocks into the main blocks; the extra-MSA representation is
 * dropped (its output cotangent is zero).  Block inputs are saved in the
 * forward pass and each block's forward is recomputed in the backward pass
 * (with PE_OPT_STACK_KEEP_CTX every block's activations are kept instead).
 *   params / d_params: the blocks' flat buffers back to back, extra first.
 *   msa_out, pair_out: final representations.  d_msa_out, d_pair_out: their
 *   cotangents.  d_extra_msa_in, d_msa_in, d_pair_in: overwritten.
 *   n_extra == 0 allows extra*, n_main == 0 allows msa* pointers to be NULL.
 *   extra and main_ must agree in r, c_z and dtype.                          */
int pe_stack_fwd_bwd(pe_handle* h,
                     int n_extra, const pe_dims* extra, int n_main, const pe_dims* main_,
                     const void* extra_msa_in, const void* msa_in, const void* pair_in,
                     const float* extra_msa_mask, const float* msa_mask, const float* pair_mask,
                     const float* params,
                     const void* d_msa_out, const void* d_pair_out,
                     void* msa_out, void* pair_out,
                     void* d_extra_msa_in, void* d_msa_in, void* d_pair_in, float* d_params,
                     void* workspace, size_t workspace_bytes,
                     void* stream_msa, void* stream_pair);

const char* pe_strerror(int code);
const char* pe_last_error(pe_handle* h);   /* text of the last PE_ERR_HIP on this handle */

#ifdef __cplusplus
}
#endif
#endif /* PE_H */
