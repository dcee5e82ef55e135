/* C ABI: a block with different input and output channel counts, composed from one kernel template.
 *
 * Canvas searches a single template [C, H, W] => [C, H, W] and applies it to a general convolution
 * [C_in, H, W] => [C_out, H, W], where one of the two channel counts is a multiple of the other (Section 4 of the
 * paper, "Main focus: convolutions").  The figure that draws the composition is not part of the paper's text; this
 * library composes as follows (with a convolution as the template the block is then exactly the convolution
 * C_in => C_out whose weight matrix is cut into square blocks), with C = min(C_in, C_out) and m = max / min:
 *
 *   C_out = m * C_in  (expand)  m instances of the template, each with weights of its own, all read x; instance j
 *                               writes channels [j * C, (j + 1) * C) of y.  dx is the sum of the instances' dx.
 *   C_in  = m * C_out (reduce)  instance j reads channels [j * C, (j + 1) * C) of x; y is the sum of the instances'
 *                               outputs.  dx of instance j is channels [j * C, (j + 1) * C) of dx.
 *
 * The instances run one after the other through the plan of canvas_dag.h compiled for [N, C, H, W]; channel slices
 * are regrouped into dense tensors and back by one launch of the library's own kernels per direction, the instances'
 * results are added in fp32 in instance order and rounded to the element type once.  (The normalisation that the paper's code generator inserts, Section 7, is a layer
 * of the surrounding network and not part of a block.)
 *
 * Pointers: device pointers unless stated, owned by the caller, 16-byte aligned, contiguous NCHW.  All functions
 * return a canvas_status (0 = OK); canvas_last_error() has the message.  Calls on one handle must not overlap.
 */
#ifndef CANVAS_BLOCK_H
#define CANVAS_BLOCK_H

#include "canvas_dag.h"

#ifdef __cplusplus
extern "C" {
#endif

typedef struct canvas_block canvas_block;

typedef struct canvas_block_info {
    int32_t instances;         /* m */
    int32_t expand;            /* 1: C_out = m * C_in, 0: C_in = m * C_out */
    int64_t template_channels; /* C */
    int32_t n_weights;         /* weight tensors of ONE instance (their shapes: canvas_dag_info of the template plan) */
    int32_t reserved0;
    uint64_t workspace_bytes;  /* device bytes forward/backward need: m plan workspaces + 2 m dense tensors [N, C, H, W] */
    canvas_dag_info plan;      /* the template's plan at [N, C, H, W] */
} canvas_block_info;

/* Host only.  blob: the template as micro-DAG text (host pointer, not retained); it must map [C, H, W] to [C, H, W]
 * (no taps left on the output).  in_shape: N, C_in, H, W.  c_out: output channels.  Errors: those of
 * canvas_dag_compile; SHAPE_MISMATCH when neither channel count is a multiple of the other or the template does not
 * keep its shape; UNSUPPORTED for inference plans (a block is a training step). */
int canvas_block_compile(const void* blob, size_t blob_len, const int64_t in_shape[4], int64_t c_out, canvas_dtype dt,
                         const canvas_options* opt, canvas_block** out);

int canvas_block_query(const canvas_block* block, canvas_block_info* info);

/* x [N, C_in, H, W] read; weights: host array of instances * n_weights device pointers, instance-major (all weights of
 * instance 0 first); y [N, C_out, H, W] written; workspace: workspace_bytes bytes, carries what backward needs
 * (reduce blocks: also the dense slices of x), so it must stay untouched until the matching backward call. */
int canvas_block_forward(canvas_block* block, const void* x, const void* const* weights, void* y, void* workspace,
                         size_t workspace_bytes, void* stream);

/* After canvas_block_forward with the same x, weights and workspace.  dy [N, C_out, H, W] read; dx [N, C_in, H, W]
 * written; dweights: host array like weights, fp32 tensors of the weights' shapes, written. */
int canvas_block_backward(canvas_block* block, const void* x, const void* const* weights, const void* dy, void* dx,
                          void* const* dweights, void* workspace, size_t workspace_bytes, void* stream);

void canvas_block_destroy(canvas_block* block);

#ifdef __cplusplus
}
#endif
#endif
