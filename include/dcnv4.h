/*
 * dcnv4.h -- C ABI of the MI355X (gfx950) DCNv4 spatial-aggregation library.
 *
 * The operator (paper Sec. 3.1, Eq. 1-2, with the softmax over the taps removed as
 * "Enhancing dynamic property" prescribes; thread/channel organisation after
 * Sec. 3.2 "Eliminating redundant workload / memory instructions"):
 *
 *   y[n,oh,ow,g*Cg+c] = sum_{k} m[n,oh,ow,g,k] * bilinear(x[n,:,:,g*Cg+c], hy_k, wx_k)
 *   hy_k = oh*stride_h - pad_h + i*dil_h + offset_scale * offset[n,oh,ow,g,k,1]
 *   wx_k = ow*stride_w - pad_w + j*dil_w + offset_scale * offset[n,oh,ow,g,k,0]
 *   k = j*kernel_h + i   (j: window column, slow; i: window row, fast)
 *
 * Whole-number coordinates are pixel centres; the four neighbours are floor and
 * floor+1; a neighbour outside the image reads zero.  m is used as given
 * (unbounded, not normalised).
 *
 * Memory: every tensor pointer is a DEVICE pointer owned by the caller, dense and
 * contiguous, 16-byte aligned, all of one element type `dtype`:
 *   x, grad_x            [N, H,  W,  G*Cg]     channel-last
 *   offset, grad_offset  [N, Ho, Wo, G, 9, 2]
 *   mask, grad_mask      [N, Ho, Wo, G, 9]
 *   y, grad_y            [N, Ho, Wo, G*Cg]
 *   offset_mask, grad_offset_mask  [N, Ho, Wo, G, 32]   (the *_merged entry points: per (pixel, group)
 *                        the 18 offsets, then the 9 mask values, then 5 unused entries)
 * with (Ho, Wo) as returned by dcnv4_output_hw().  The library allocates nothing and
 * keeps nothing between calls except the test switches below; it enqueues its kernels
 * on `stream` (a hipStream_t, NULL = the default stream) and returns without
 * synchronising.  Outputs must not alias inputs.  (The module entry points further down
 * need memory for the tensors between their layers: dcnv4_module_forward takes it from the
 * caller, dcnv4_module_forward_static from a 32 MiB device array that is part of the library.)
 *
 * Supported: square windows of 3x3 (every entry point and kernel), 1x1 and 5x5 (dcnv4_forward in
 * F32 and F16, dcnv4_backward in F32, through the direct kernels; 5x5 forward needs Cg >= 16; K = 1 or
 * 25 replaces 9 in the layouts above); stride, dilation >= 1; pad >= 0; Cg in {8, 16, 32, 64};
 * dtype F32 or F16.  F16 is fp16 storage with fp32 positions and accumulation and one
 * round-to-nearest at the store; where the forward runs out of its ring of input rows
 * in LDS (fp16, Cg 16, maps of several hundred pixels) the four products m * corner
 * weight of a tap are rounded to fp16 before they multiply the (fp16) inputs; products
 * and sums stay fp32.  The fp16 backward exists for Cg 8, 16 and 32.  Byte
 * offsets inside one image are 32-bit: one image of x and of y, and the farthest
 * clamped sampling position (about twice the image extent), must stay below 2 GiB;
 * larger images are refused with DCNV4_ERR_UNSUPPORTED.
 *
 * Errors: every call validates its arguments on the host first and returns a
 * nonzero DCNV4_ERR_* without launching or writing anything; nothing throws or
 * aborts.  DCNV4_ERR_LAUNCH reports a HIP launch failure.
 */
#ifndef DCNV4_H
#define DCNV4_H

#ifdef __cplusplus
extern "C" {
#endif

enum { DCNV4_F32 = 0, DCNV4_F16 = 1 };

enum {
    DCNV4_OK = 0,
    DCNV4_ERR_NULL = 1,        /* a required pointer is NULL */
    DCNV4_ERR_SHAPE = 2,       /* a size is non-positive, the window does not fit, or a workspace is too small */
    DCNV4_ERR_UNSUPPORTED = 3, /* kernel size, Cg, dtype or tensor size outside the supported set */
    DCNV4_ERR_ALIGN = 4,       /* a tensor pointer is not 16-byte aligned */
    DCNV4_ERR_LAUNCH = 5,      /* the HIP runtime refused the launch */
    DCNV4_ERR_TOO_LARGE = 6    /* dcnv4_module_forward_static: the call needs more than the built-in workspace */
};

/* Output extent of the sliding window: Ho = (H + 2*pad_h - dil_h*(kernel_h-1) - 1)/stride_h + 1,
 * likewise Wo (Sec. 3.1: the operator slides like a regular convolution).
 * Host pointers H_out/W_out; returns DCNV4_ERR_SHAPE if the window does not fit. */
int dcnv4_output_hw(int H, int W, int kernel_h, int kernel_w, int stride_h, int stride_w,
                    int pad_h, int pad_w, int dil_h, int dil_w, int *H_out, int *W_out);

/* Forward aggregation, Eq. 1-2 (gather the 4 neighbours of each of the 9 taps for a run of
 * channels, interpolate, modulate by m, reduce over the taps).  Overwrites y. */
int dcnv4_forward(const void *x, const void *offset, const void *mask, void *y,
                  int N, int H, int W, int G, int Cg,
                  int kernel_h, int kernel_w, int stride_h, int stride_w,
                  int pad_h, int pad_w, int dil_h, int dil_w,
                  float offset_scale, int dtype, void *stream);

/* The same with offsets and mask values in ONE buffer [N,Ho,Wo,G,32].  Sec. 3.2 "Micro design" merges
 * the two linear layers that produce offsets and mask values into one; this is the tensor such a
 * layer hands over when its 27 outputs per group are padded to 32 (this library's choice: records
 * of 64 bytes in fp16, 128 in fp32, never straddling more than two cache lines).  Entries 0..17 of
 * a (pixel, group) are its offsets (tap-major, width then height), 18..26 its mask values, 27..31
 * are ignored.  Runs through the LDS-staged kernels only; a shape none of them takes is refused
 * with DCNV4_ERR_UNSUPPORTED. */
int dcnv4_forward_merged(const void *x, const void *offset_mask, void *y,
                         int N, int H, int W, int G, int Cg,
                         int kernel_h, int kernel_w, int stride_h, int stride_w,
                         int pad_h, int pad_w, int dil_h, int dil_w,
                         float offset_scale, int dtype, void *stream);

/* Backward of Eq. 1 by the chain rule (the paper gives no backward):
 *   grad_mask_k  = sum_c gy[c] * S_k[c]
 *   grad_offset  = offset_scale * m_k * sum_c gy[c] * dS_k[c]/d(wx, hy)   (right-hand derivative
 *                  at whole-number coordinates)
 *   grad_x      += m_k * corner weight * gy[c]   at the in-image neighbours
 * Overwrites all three outputs; grad_x is zero-filled on `stream` first.  grad_offset/grad_mask are
 * fp32 sums, rounded once in F16.  In the LDS-staged path grad_x is summed per tile in 32-bit fixed
 * point with 22 fractional bits (every term m * weight * gy[c] rounded to a multiple of 2^-22, the
 * sum itself exact and independent of the order); terms of magnitude 64 or more, and whatever would
 * take a tile's sum for one pixel beyond 512, are added straight to memory in fp32 instead.  The
 * tile sums (a pixel is touched by the few tiles that reach it) go to memory through fp32 atomics,
 * packed fp16 atomics in F16.  With Cg 32 or 64 (fp32) the group's channels are processed in slices
 * and grad_offset/grad_mask are summed with fp32 atomics, so their last bits can differ between
 * runs, like grad_x's. */
int dcnv4_backward(const void *x, const void *offset, const void *mask, const void *grad_y,
                   void *grad_x, void *grad_offset, void *grad_mask,
                   int N, int H, int W, int G, int Cg,
                   int kernel_h, int kernel_w, int stride_h, int stride_w,
                   int pad_h, int pad_w, int dil_h, int dil_w,
                   float offset_scale, int dtype, void *stream);

/* dcnv4_backward for the merged buffer: grad_offset_mask has the layout of
 * offset_mask (gradients of the 18 offsets, of the 9 mask values, 5 zeros); it is zero-filled on
 * `stream` first, like grad_x.  Same restrictions as dcnv4_forward_merged. */
int dcnv4_backward_merged(const void *x, const void *offset_mask, const void *grad_y,
                          void *grad_x, void *grad_offset_mask,
                          int N, int H, int W, int G, int Cg,
                          int kernel_h, int kernel_w, int stride_h, int stride_w,
                          int pad_h, int pad_w, int dil_h, int dil_w,
                          float offset_scale, int dtype, void *stream);

/* The DCNv3 form of Eq. 1 (Sec. 3.1: there the K modulation scalars of a sampling location are
 * softmax-normalised; DCNv4 removes exactly this): `mask_logits` [N,Ho,Wo,G,9] holds logits, and
 * m = softmax over the 9 taps is formed inside the kernels, in registers, before the aggregation
 * (expf of the shifted logits in fp32).  Everything else as in dcnv4_forward.  Runs through the
 * LDS-staged kernels only (ring of rows or input rectangle); a shape they do not take is refused with
 * DCNV4_ERR_UNSUPPORTED. */
int dcnv4_forward_softmax(const void *x, const void *offset, const void *mask_logits, void *y,
                          int N, int H, int W, int G, int Cg,
                          int kernel_h, int kernel_w, int stride_h, int stride_w,
                          int pad_h, int pad_w, int dil_h, int dil_w,
                          float offset_scale, int dtype, void *stream);

/* Backward of dcnv4_forward_softmax: grad_x and grad_offset as in dcnv4_backward with the normalised
 * m; grad_mask_logits[k] = m_k * (g_k - sum_j m_j * g_j), g being the gradient w.r.t. m. */
int dcnv4_backward_softmax(const void *x, const void *offset, const void *mask_logits, const void *grad_y,
                           void *grad_x, void *grad_offset, void *grad_mask_logits,
                           int N, int H, int W, int G, int Cg,
                           int kernel_h, int kernel_w, int stride_h, int stride_w,
                           int pad_h, int pad_w, int dil_h, int dil_w,
                           float offset_scale, int dtype, void *stream);

/* A linear layer over the channel axis -- the 1x1 point-wise convolution that Sec. 3.1 puts before and
 * after the operator, and the layer of Sec. 3.2 "Micro design" that predicts offsets and modulation
 * scalars:  y[p][o] = sum_k x[p][k] * w[o][k] + b[o].
 * Device pointers, dense row-major: x [P][K], w [Nout][K], b [Nout] or NULL (no bias), y [P][Nout];
 * x, w and y 16-byte aligned.  On the matrix cores with fp32 accumulation; y is rounded once in F16.
 * Needs K * element size a multiple of 32 bytes, Nout a multiple of 32, and every tensor below 2 GiB
 * (else DCNV4_ERR_UNSUPPORTED).  Allocates nothing; enqueues on `stream`. */
int dcnv4_linear(const void *x, const void *w, const void *b, void *y,
                 long long P, int K, int Nout, int dtype, void *stream);

/* The 3x3 depthwise convolution of the separable structure that computes offsets and scalars in the
 * module (Sec. 3.2 "Micro design"), zero padding, stride 1, channel-last:
 *     y[n,h,w,c] = b[c] + sum_{i,j in 0..2} w[i][j][c] * x[n, h+i-1, w+j-1, c]      (x = 0 outside the map)
 * Device pointers, 16-byte aligned: x, y [N,H,W,C]; w [3][3][C] (i: height tap, j: width tap); b [C] or
 * NULL.  fp32 accumulation, one rounding at the store.  Needs C * element size a multiple of 16 bytes and
 * the tensor below 2 GiB (else DCNV4_ERR_UNSUPPORTED). */
int dcnv4_depthwise3x3(const void *x, const void *w, const void *b, void *y,
                       int N, int H, int W, int C, int dtype, void *stream);

/* Forward of the DCNv4 module (Sec. 3.2 "Micro design"; the two variants of the module-level
 * benchmark of the appendix):
 *     value = x W_in^T + b_in          (w_in == w_out == NULL: the "lightweight" variant, value = x)
 *     x'    = depthwise3x3(x; w_dw, b_dw)   (w_dw == NULL: x' = x -- the paper notes the convolution can go
 *                                      where latency matters)
 *     om    = x' W_om^T + b_om         ONE layer for offsets and scalars, in the merged layout above:
 *                                      w_om [G*32][C], b_om [G*32]; row g*32 + e produces entry e of
 *                                      group g (0..17 offsets, 18..26 scalars, 27..31 ignored)
 *     y_op  = dcnv4_forward_merged(value, om)
 *     y     = y_op W_out^T + b_out     (left out in the lightweight variant: y = y_op)
 * x, y [N,H,W,C], C = G*Cg; w_in, w_out [C][C]; w_dw [3][3][C]; biases may be NULL.  The window must be
 * 3x3 and keep the map's size (stride 1, pad = dilation), C * element size a multiple of 32 bytes.
 * `workspace`: device memory of at least dcnv4_module_workspace_bytes() bytes, 16-byte aligned, owned by
 * the caller; it holds om, value, y_op and x' during the call and may be reused afterwards.  Without the
 * depthwise convolution the value projection and the merged layer run as one kernel that reads x once.
 * Tensors between the layers are stored in `dtype`.  On an error y is untouched (the workspace may
 * have been written). */
int dcnv4_module_forward(const void *x, const void *w_in, const void *b_in,
                         const void *w_dw, const void *b_dw,
                         const void *w_om, const void *b_om,
                         const void *w_out, const void *b_out,
                         void *workspace, long long workspace_bytes, void *y,
                         int N, int H, int W, int G, int Cg,
                         int kernel_h, int kernel_w, int stride_h, int stride_w,
                         int pad_h, int pad_w, int dil_h, int dil_w,
                         float offset_scale, int dtype, void *stream);

/* Bytes of workspace dcnv4_module_forward needs (lightweight != 0: without the two projections;
 * depthwise != 0: with the depthwise convolution); -1 for a bad argument.  Host-only helper. */
long long dcnv4_module_workspace_bytes(int N, int H, int W, int G, int Cg, int dtype, int lightweight,
                                       int depthwise);

/* dcnv4_module_forward for callers that cannot allocate device memory or hand over a workspace -- code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc: the same kernels, with
 * the workspace in a buffer built into the library (a static device array of
 * dcnv4_module_static_workspace_limit() = 32 MiB bytes; every GPU the library runs on holds its own copy
 * until the process ends).  No allocation of any kind happens in the call.  A call that needs more than the
 * limit (dcnv4_module_workspace_bytes() tells) returns DCNV4_ERR_TOO_LARGE and does nothing; at 32 MiB
 * that is e.g. one 200x320x128 fp16 map, or 16 maps of 56x56x128, with both projections.
 * All calls on one GPU share that GPU's buffer: calls that overlap in time on one GPU (different streams,
 * different host threads) race on it; on one stream they are ordered and safe.  Nothing in the buffer
 * has to start at zero (every tensor in it is written in full before it is read).  The first call on a
 * device looks the buffer's address up (hipGetSymbolAddress): make one call before capturing a graph. */
int dcnv4_module_forward_static(const void *x, const void *w_in, const void *b_in,
                                const void *w_dw, const void *b_dw,
                                const void *w_om, const void *b_om,
                                const void *w_out, const void *b_out, void *y,
                                int N, int H, int W, int G, int Cg,
                                int kernel_h, int kernel_w, int stride_h, int stride_w,
                                int pad_h, int pad_w, int dil_h, int dil_w,
                                float offset_scale, int dtype, void *stream);

/* Size in bytes of the built-in workspace of dcnv4_module_forward_static.  Host-only helper. */
long long dcnv4_module_static_workspace_limit(void);

/* Bytes the ideal memory-access model of Sec. 3.2 ("2HWC + 27HWG", every value touched
 * once) assigns to one forward call: x + offset + mask + y.  Host-only helper. */
long long dcnv4_forward_algorithmic_bytes(int N, int H, int W, int G, int Cg,
                                          int H_out, int W_out, int dtype);

/* Same model for one backward call: reads x, offset, mask, grad_y; writes grad_x,
 * grad_offset, grad_mask (the zero-fill of grad_x is not counted). */
long long dcnv4_backward_algorithmic_bytes(int N, int H, int W, int G, int Cg,
                                           int H_out, int W_out, int dtype);

/* The two models with the merged buffer: 32 instead of 27 values per (pixel, group). */
long long dcnv4_forward_merged_algorithmic_bytes(int N, int H, int W, int G, int Cg,
                                                 int H_out, int W_out, int dtype);
long long dcnv4_backward_merged_algorithmic_bytes(int N, int H, int W, int G, int Cg,
                                                  int H_out, int W_out, int dtype);

/* TEST AND BENCHMARK SWITCHES, not an application interface: they force a kernel or a tile shape so
 * that every path can be checked on every shape (process-wide, not thread-safe).  An application
 * never calls this; the library's own choice is the value 0 of every switch.
 *   "reset"       (any value) puts every switch back to 0
 *   "fwd_path"    1 = direct global gather, 2 = input rectangle staged in LDS, 3 = ring of input rows
 *                 in LDS (fp16, Cg 16); 0 = ring on maps of 512 pixels or more, else rectangle where a
 *                 useful tile fits, else direct
 *   "bwd_path"    1 = one kernel with global atomics for grad_x (fp32), 2 = two LDS-staged kernels
 *                 (gathers for grad_offset/grad_mask; fixed-point accumulation of grad_x in LDS),
 *                 0 = staged where a useful tile fits, else the first
 *   "fwd_single"  LDS rectangle buffers of the staged gather kernels: 1 = always two (the next tile
 *                 streams in during the current one), 2 = always one (bigger rectangle, refilled
 *                 between tiles), 0 = whichever the tile chooser estimates to be cheaper
 *   "wg_per_cu"   persistent workgroups per compute unit of the rectangle kernels (1..32, as far as
 *                 LDS allows)
 *   "module_rows" 1 = dcnv4_module_forward keeps the tensors between its layers channel-last (default: the
 *                 full module keeps them plane-major, one (image, group) after the other)
 *   "gom_coop"    1 = the fp32 grad_offset/grad_mask pass moves its values through per-wave LDS slices
 *                 even for whole groups (default: each lane reads and writes its own pixel's values)
 *   "gx_threads"  workgroup size of the staged grad_x kernel (256, 512 or 768)
 *   "halo"        displacement in pixels (rows, for the ring) that the staged window allows for;
 *                 samples beyond it are still exact, they take the path through global memory
 *   "lds_kb"      LDS budget per workgroup of the staged kernels (8..160)
 *   "fwd_threads" workgroup size of the staged forward (64, 128, 256, 512, 640 or 768 for the
 *                 rectangle kernel; 256 = four waves instead of eight for the ring)
 *   "fwd_cpt"     channels per thread in the direct forward kernel (8 or 16)
 *   "bwd_cpt"     channels per thread in the direct backward kernel (1, 2, 4, 8 or 16)
 *   "xcd_remap"   1 = hand consecutive tiles to one XCD (default), 0 = plain block order
 * Returns DCNV4_ERR_UNSUPPORTED for an unknown key or value. */
int dcnv4_set_option(const char *key, int value);

/* Name of the kernel that the most recent dcnv4_forward (backward = 0) or dcnv4_backward
 * (backward = 1) call launched, as it appears in a profiler's kernel trace.  Static storage;
 * NULL before the first such call. */
const char *dcnv4_last_kernel_name(int backward);

const char *dcnv4_status_string(int status);

#ifdef __cplusplus
}
#endif
#endif /* DCNV4_H */
