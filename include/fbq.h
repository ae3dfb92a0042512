/*
 * fbq.h - C ABI of the MI355X (gfx950) library for FBQuant's inference hot path: the
 * sub-branched weight-only-quantized linear layer
 *
 *     y = x . Wq^T + (x . A) . B          Wq = s * (q - z), q = packed INT3/INT4 codes
 *
 * i.e. y = x . W_F^T with the paper's feedback-reconstructed weight
 * W_F = Q(W - Sigma) + Sigma, Sigma = B.A (Sec. 4.1 definition of W_F; Sec. 4.2 low-rank
 * parametrisation; Sec. 4.3 kernel fusion: de-quantization, main projection and up-projection
 * in one kernel sharing one output tensor, the down-projection x.A a separate small kernel).
 *
 * Conventions
 *   N = output features, K = input features, M = tokens, r = rank of the sub-branch,
 *   g = group size along K (one fp16 scale and one fp16 zero per row n and group), G = K/g,
 *   b = bits per code (3 or 4), qmax = 2^b - 1.
 *   The paper writes Sigma = B.A with A [r, d_in] and B [d_out, r]; this library takes the
 *   transposes A [K, r] and B [r, N] so that y = x.A.B:  Sigma[n,k] = sum_j A[k,j] * B[j,n].
 *   All matrices are dense row-major.  fp16 is IEEE binary16, passed as uint16_t on the host.
 *
 * Device layout (what fbq_pack writes and the kernels read)
 *   qweight  uint32 words, rows contiguous, K*b/32 words per row.
 *            b = 4: word k/8 holds code k%8 = i at bits [4i, 4i+4).
 *            b = 3: the 32 codes k/32 = u live in words 3u..3u+2.  For j = k%32 < 30: word j/10,
 *                   field i = j%10; fields 0..4 at bits [3i, 3i+3), fields 5..9 at bits
 *                   [16+3(i-5), 16+3(i-5)+3).  Code 30 is spread over bit 15 of the three words
 *                   (bit c of the code in word c), code 31 over bit 31.  No code straddles a
 *                   16-bit half, so a mask yields two codes at once as an fp16 pair.
 *   scales   [N, G] fp16      zeros  [N, G] fp16 (real-valued zero point, not an integer)
 *   At       [r, K] fp16 (A transposed: K contiguous)   Bt  [N, r] fp16 (B transposed: one output's r taps contiguous)
 *
 * Ownership and errors
 *   The library owns no memory and keeps no state.  Pointers marked "host" are read or
 *   written by the CPU during the call; pointers marked "device" must be device memory valid on
 *   the current HIP device, 16-byte aligned, owned by the caller, and are accessed asynchronously
 *   on `stream` (a hipStream_t passed as void*; NULL is the default stream).  Device entry points
 *   validate everything on the host first and return an error WITHOUT launching; they never
 *   allocate and never synchronise.  Outputs are fully overwritten, never accumulated into.
 */
#ifndef FBQ_H
#define FBQ_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    FBQ_OK = 0,
    FBQ_ERR_NULL = 1,        /* a required pointer is NULL */
    FBQ_ERR_SHAPE = 2,       /* N, K, M < 1; r < 0; K % group; K % 32; r % 8; a code above qmax */
    FBQ_ERR_UNSUPPORTED = 3, /* bits not in {3, 4}; group != 128; r > 256; K > 32768; packed codes, or B, of 1 GiB or more */
    FBQ_ERR_ALIGN = 4,       /* a device pointer is not 16-byte aligned */
    FBQ_ERR_WORKSPACE = 5,   /* workspace smaller than fbq_workspace_bytes() */
    FBQ_ERR_HIP = 6          /* the HIP runtime refused a launch (hipGetLastError) */
} fbq_status;

/* One quantized layer.  r == 0 is the branch-free layer (A and Bt may then be NULL). */
typedef struct {
    int32_t N;      /* output features */
    int32_t K;      /* input features, multiple of group */
    int32_t r;      /* rank of the sub-branch, multiple of 8, 0..256 */
    int32_t bits;   /* 3 or 4 */
    int32_t group;  /* 128 */
} fbq_desc;

typedef void *fbq_stream;   /* hipStream_t */

const char *fbq_status_string(fbq_status s);

/* Validates a descriptor (FBQ_OK, FBQ_ERR_NULL, FBQ_ERR_SHAPE or FBQ_ERR_UNSUPPORTED). */
fbq_status fbq_check_desc(const fbq_desc *d);

/* Bytes of the packed code buffer, N * K * bits / 8.  0 for an invalid descriptor. */
size_t fbq_packed_bytes(const fbq_desc *d);

/* Bytes of device scratch fbq_linear needs for M tokens.  M <= 2: the down-projection t = x.A on its
 * way from the blocks that compute it to the blocks that use it, as tagged 8-byte words, one per token,
 * column of A and K slice (0 when r == 0).  3 <= M <= 64: the same hand-over for 16 token rows, per
 * K slice and summed, once for every 16 tokens or part of them (0 when r == 0) - unless the layer is so large that
 * 17..64 tokens take the path of M > 64.  M > 64: room for those hand-over words (left alone by this path, so
 * that one workspace can serve calls of every token count), then the activations
 * re-ordered for the matrix cores (M rounded up to 128 rows of K fp16), t as two fp16 halves and its
 * partial sums, and, where the launch splits K over blocks, fp32 partial outputs (up to 8 x M x N);
 * not 0 even when r == 0.  0 for an invalid descriptor or M < 1.
 * The size is NOT monotonic in M (fewer tokens can mean more K slices or a K split with partial outputs): a workspace
 * meant for several token counts takes the largest of their sizes. */
size_t fbq_workspace_bytes(const fbq_desc *d, int M);

/*
 * fbq_pack - host side, off the hot path.  Converts canonical tensors into the device layout
 * above (the caller then copies the outputs to the GPU).  INT3/INT4 storage of the main-path
 * weights with floating-point inputs and outputs is the paper's setting (Sec. 1); the bit
 * layout is this library's own.
 *   codes      host [N, K] uint8, each in 0..qmax        qweight_out host, fbq_packed_bytes()
 *   scales     host [N, G] fp16                           scales_out  host [N, G] fp16
 *   zeros      host [N, G] fp16                           zeros_out   host [N, G] fp16
 *   A          host [K, r] fp16 (NULL if r == 0)          At_out      host [r, K] fp16
 *   B          host [r, N] fp16 (NULL if r == 0)          Bt_out      host [N, r] fp16
 * Returns FBQ_ERR_SHAPE if a code exceeds qmax (outputs are then unspecified).
 */
fbq_status fbq_pack(const fbq_desc *d, const uint8_t *codes, const uint16_t *scales, const uint16_t *zeros,
                    const uint16_t *A, const uint16_t *B, uint32_t *qweight_out, uint16_t *scales_out,
                    uint16_t *zeros_out, uint16_t *At_out, uint16_t *Bt_out);

/*
 * fbq_linear - the hot path (Sec. 4.3).  y[m,n] = sum_k x[m,k] * s[n,k/g] * (q[n,k] - z[n,k/g])
 *                                               + sum_j (sum_k x[m,k] * At[j,k]) * Bt[n,j]
 * in fp32 accumulation, rounded once to fp16.  M <= 2 runs the decode GEMV in ONE launch per token
 * count (packed words streamed once per token, unpacked in registers; the down-projection runs in
 * the same launch, one column of A per block as a small job in front of the block's first tile).  3 <= M <= 16 streams the packed words once for all
 * tokens against a 16-token matrix-core tile, also in ONE launch whose first blocks do the
 * down-projection; 17 <= M <= 64 is the same launch with the sets of 16 tokens side by side (the packed words are read
 * once per 16 tokens, which for most layers is still cheaper there than unpacking them into fp16 tiles; one or two
 * tokens left over go through the GEMV; a layer so large that reading it two to four times costs more takes the path
 * of M > 64 instead).  M > 64 runs the fp16 MFMA GEMM after a pass that
 * re-orders x and a separate down-projection; a layer with too few output tiles to fill the GPU has
 * its K range split over up to 8 blocks per tile, summed in fp32 by a last small launch.
 *   x         device [M, K] fp16             qweight, scales, zeros, At, Bt: device, layout above
 *   y         device [M, N] fp16, overwritten
 *   workspace device, >= fbq_workspace_bytes(d, M) bytes (may be NULL when that is 0).  Zero-fill it
 *             once after allocating it; after that it needs no care between calls, on any stream
 *             and under graph replay: every launch marks what it writes with its own identity.
 *             Calls that may run concurrently must not share a workspace.
 * Errors: FBQ_ERR_NULL, _SHAPE, _UNSUPPORTED, _ALIGN, _WORKSPACE before any launch; FBQ_ERR_HIP.
 * Up to 16 tokens the blocks that use t wait a bounded number of polls (32768, about 10 ms) for the
 * blocks of the same launch that compute it, then compute their share themselves (same results, slower;
 * every kernel still ends): see fbq_test_set_spin_limit.
 */
fbq_status fbq_linear(const fbq_desc *d, int M, const void *x, const void *qweight, const void *scales,
                      const void *zeros, const void *At, const void *Bt, void *y, void *workspace,
                      size_t workspace_bytes, fbq_stream stream);

/*
 * fbq_linear_static - fbq_linear for callers that cannot allocate device memory (code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc) and therefore cannot supply a
 * workspace: the same kernels, with the hand-over scratch taken from a device array inside the
 * library (544 KiB per GPU the library runs on, held until the process ends).  The call itself
 * allocates nothing and frees nothing.
 *   Arguments as for fbq_linear, without workspace and workspace_bytes.  M <= 16 only: larger token
 *   counts need scratch that grows with M, N and K and are refused with FBQ_ERR_UNSUPPORTED;
 *   FBQ_ERR_WORKSPACE if the layer's scratch would not fit the array (it always fits for r <= 256).
 *   All calls on one GPU share that GPU's array, on whatever stream: calls that may overlap in time on
 *   one GPU race on it and must be ordered by the caller.  Nothing needs clearing between calls (the
 *   array starts zeroed and every launch marks what it writes with its own identity).
 *   The first call on a device looks the array's address up (once per device); make that call outside
 *   a graph capture.
 * Errors: those of fbq_linear, before any launch; FBQ_ERR_HIP if the array cannot be found.
 */
fbq_status fbq_linear_static(const fbq_desc *d, int M, const void *x, const void *qweight, const void *scales,
                             const void *zeros, const void *At, const void *Bt, void *y, fbq_stream stream);

/*
 * fbq_test_set_spin_limit - test hook, not for production use.  Sets, for the whole process and every
 * later launch, how many polls a block waits for the down-projection's hand-over words before it
 * computes them itself: clamped to at most the default 32768; a negative value sends every block down
 * that fall-back path at once, which is how the tests check a path no healthy run takes.  Returns the
 * value that was in force.  Launches already enqueued keep the value they were launched with.
 */
int fbq_test_set_spin_limit(int polls);

/* One layer of a grouped call: the arguments fbq_linear takes, per layer. */
typedef struct {
    fbq_desc desc;
    const void *x;          /* device [M, K] fp16 (layers may share it: q/k/v, gate/up) */
    const void *qweight;    /* device, layout above */
    const void *scales;
    const void *zeros;
    const void *At;         /* NULL if desc.r == 0 */
    const void *Bt;         /* NULL if desc.r == 0 */
    void *y;                /* device [M, N] fp16, overwritten */
    void *workspace;        /* as for fbq_linear; one per layer, never shared or overlapping */
    size_t workspace_bytes;
} fbq_layer_call;

/*
 * fbq_linear_group - the hot path for several independent layers at once (Sec. 4.3 lists launch
 * overhead as part of the sub-branch's cost; on this GPU a launch costs about as much as streaming
 * a 4096x4096 INT4 layer, so layers that do not depend on each other - q/k/v, gate/up - should share
 * one).  Every layer gets exactly the result fbq_linear gives it.  For M <= 2, layers with the same
 * bits, the same K-derived kernel variant and a sub-branch (or all without one) are served by ONE
 * launch, up to 8 layers per launch, in the order they appear.  For 3 <= M <= 16, layers with the
 * same bits and K that read the SAME x (the same pointer) and all have a sub-branch (or all have
 * none) share one launch, up to 4 layers.  Anything else, and every layer when M > 16, is launched
 * on its own.
 *   calls host array of n layers (read during the call only); M tokens, the same for all layers
 * Errors: those of fbq_linear for any layer, and FBQ_ERR_WORKSPACE if the workspaces of two layers
 * overlap, reported before ANY launch.
 */
fbq_status fbq_linear_group(const fbq_layer_call *calls, int n, int M, fbq_stream stream);

/*
 * fbq_reconstruct - validation.  W_hat[n,k] = s*(q - z) + sum_j At[j,k]*Bt[n,j], the paper's
 * W_F = Q(W - Sigma) + Sigma (Sec. 4.1), as fp32.   W_hat device [N, K] fp32, overwritten.
 */
fbq_status fbq_reconstruct(const fbq_desc *d, const void *qweight, const void *scales, const void *zeros,
                           const void *At, const void *Bt, float *W_hat, fbq_stream stream);

/* fbq_unpack_codes - validation.  codes_out device [N, K] uint8 = the integer codes q. */
fbq_status fbq_unpack_codes(const fbq_desc *d, const void *qweight, uint8_t *codes_out, fbq_stream stream);

/*
 * fbq_quantize_feedback - the step before the path: the feedback quantizer Q(W - Sigma) of
 * Sec. 4.1 / Alg. 1 (forward line), group-wise asymmetric round-to-nearest, computed on the GPU
 * in fp64 and written straight into the device layout.  Per row and group: mn, mx of
 * R = W - Sigma; s = fp16((mx - mn)/qmax) (1 if the group is constant, never below the smallest
 * normal fp16); z = fp16(-mn/s); s is stepped to the next fp16 until both ends of the range lie
 * within half a step of [0, qmax]; q = clamp(round_half_even(R/s + z), 0, qmax).
 *   W device [N, K] fp16; At device [r, K]; Bt device [N, r] (both NULL if r == 0)
 *   qweight_out device fbq_packed_bytes(); scales_out, zeros_out device [N, G] fp16
 */
fbq_status fbq_quantize_feedback(const fbq_desc *d, const void *W, const void *At, const void *Bt,
                                 void *qweight_out, void *scales_out, void *zeros_out, fbq_stream stream);

/*
 * fbq_linear_unfused - comparator, not the product path: the conventional arrangement of a quantized
 * layer with a low-rank sub-branch that Sec. 3.2 describes and Sec. 4.3 replaces (Fig. 4, left).  Same
 * arguments and result as fbq_linear for M <= 16, computed as three launches: the quantized main path
 * y = x . Wq^T (this library's kernel without the sub-branch), t = x . A rounded to fp16 as a
 * stand-alone kernel's output is, and y += t . B, which reads y back and writes it again.  The time it
 * takes beyond the branch-free layer, against what fbq_linear takes beyond it, is the share of the
 * sub-branch's cost that the fusion removes (the paper reports 60 % for its kernels, Sec. 4.3).
 *   workspace: fbq_workspace_bytes(d, M) bytes as for fbq_linear (its first M r fp16 hold t); one of its own, not
 *   one that fbq_linear calls also use (those expect to find nothing but their own hand-over words there).
 * Errors: as fbq_linear; FBQ_ERR_UNSUPPORTED for M > 16.  Differs from fbq_linear by the fp16
 * rounding of t (about 2^-11 relative on the sub-branch's share of y).
 */
fbq_status fbq_linear_unfused(const fbq_desc *d, int M, const void *x, const void *qweight, const void *scales,
                              const void *zeros, const void *At, const void *Bt, void *y, void *workspace,
                              size_t workspace_bytes, fbq_stream stream);

/*
 * fbq_measure_read_stream - measurement aid, not part of the method.  One launch that reads every
 * 16-byte piece of buf[0, bytes) once and writes nothing.  Timed like the decode kernels (back to back
 * on a stream, over buffers no cache holds) it gives what the memory system delivers to a launch of
 * that size on this GPU: the ceiling the decode path's GB/s is quoted against beside the nominal HBM
 * peak (Sec. 1 names weight loading as the bottleneck the quantized layer is up against).
 *   buf device, 16-byte aligned, bytes >= 16 (a tail of less than 16 bytes is not read).
 * Errors: FBQ_ERR_NULL, FBQ_ERR_SHAPE (bytes < 16), FBQ_ERR_ALIGN before the launch; FBQ_ERR_HIP.
 */
fbq_status fbq_measure_read_stream(const void *buf, size_t bytes, fbq_stream stream);

/*
 * Layer-wise reconstruction (Alg. 1, Sec. 4.2): gradient descent on the sub-branch of one layer so
 * that the quantized layer reproduces the fp16 layer's outputs on calibration activations X [T,K].
 * Loss and gradient depend on X only through H = X^T X (Sec. 4.2: L = tr(Delta_F H Delta_F^T) with
 * Delta_F = W - Q(W - Sigma) - Sigma; dL/dSigma = -2 Delta_F H once the feedback is detached), so H
 * is formed once per layer and every iteration works from it.
 *
 * fbq_train_workspace_bytes - device scratch for fbq_gram (T tokens) and fbq_train_step: x
 *   transposed, or fp16 copies of the branch, Delta_F in both orientations, the r-row products
 *   and the partial sums of contractions whose K range is split over blocks (about 4 N K bytes).
 *   0 for an invalid descriptor, r < 1 or T < 1.
 *
 * fbq_gram - H16_out [K,K] fp16 = fp16(h_scale * X^T X), accumulated in fp32 on the matrix cores.
 *   X device [T,K] fp16.  h_scale > 0 keeps H inside fp16's range: h_scale * max_k sum_t x[t,k]^2
 *   must stay below 65504 (1/T suits unit-variance activations).  d->N, d->r, d->bits are not used
 *   beyond validation.
 *
 * fbq_train_step - one iteration of the loop body of Alg. 1.
 *   in:     W device [N,K] fp16; H16, h_scale from fbq_gram
 *   in/out: At32 device [r,K] fp32, Bt32 device [N,r] fp32: the master copies of the branch
 *           (Alg. 1 initialises A ~ N(0, sigma^2), B = 0), updated in place:
 *           master <- master - lr * gradient (plain gradient descent)
 *   out, all describing the branch BEFORE the update, i.e. a consistent layer for fbq_linear:
 *           At16_out [r,K], Bt16_out [N,r] = fp16 of the masters (what the forward pass uses);
 *           qweight_out, scales_out, zeros_out = Q(W - Sigma16) exactly as fbq_quantize_feedback
 *           would write them; grad_At [r,K], grad_Bt [N,r] fp32 = dL/dAt, dL/dBt with W and
 *           Q(W - Sigma16) held constant; loss: one fp32 = || W X^T - W_F X^T ||_F^2 (the square:
 *           the trace form and the printed gradient are those of the squared norm), or NULL:
 *           the gradients need only products with r rows (H is symmetric, so Delta_F H At^T =
 *           Delta_F (At H)^T), the loss alone needs Delta_F H (2 N K^2 flop) and is skipped then.
 *   lr = 0 evaluates without moving the masters.  Delta_F, H and their products enter the matrix
 *   cores as fp16 with fp32 accumulation: gradients and loss carry a relative error of a few 1e-4.
 *   Nothing is allocated; everything is enqueued on `stream`.  Needs r >= 1.
 * Errors: FBQ_ERR_NULL, _SHAPE, _UNSUPPORTED, _ALIGN, _WORKSPACE before any launch; FBQ_ERR_HIP.
 */
size_t fbq_train_workspace_bytes(const fbq_desc *d, int T);
fbq_status fbq_gram(const fbq_desc *d, int T, const void *X, float h_scale, void *H16_out, void *workspace,
                    size_t workspace_bytes, fbq_stream stream);
fbq_status fbq_train_step(const fbq_desc *d, const void *W, const void *H16, float h_scale, float *At32, float *Bt32,
                          float lr, void *qweight_out, void *scales_out, void *zeros_out, void *At16_out,
                          void *Bt16_out, float *grad_At, float *grad_Bt, float *loss, void *workspace,
                          size_t workspace_bytes, fbq_stream stream);

#ifdef __cplusplus
}
#endif
#endif /* FBQ_H */
