/*
 * peqa.h -- C-ABI of the MI355X (gfx950) PEQA quantized-linear library.
 *
 * PEQA (arXiv 2305.14152, Sec. 3.2) replaces a fully-connected weight
 * W0 in R^{N x K} by  What = (s0 + ds) . (Q - z0)  with frozen b-bit integer
 * codes Q (b = 3 or 4), zero-points z0 and scales s0 per output channel
 * (optionally per group of g input features, Sec. 4.2 and Table 5), and trains only ds.
 *
 * Conventions for every call
 *   - Every tensor argument is a DEVICE pointer owned by the caller, contiguous,
 *     row-major, 16-byte aligned (PEQA_ERR_ALIGN otherwise); outputs must not
 *     alias inputs.  Descriptor structs (peqa_layout, peqa_adamw) are HOST pointers.
 *   - `stream` is a hipStream_t passed opaquely (NULL = the default stream).
 *     Calls only enqueue work; they never synchronise and never allocate or free device
 *     memory.  All work of a call is ordered after what the stream held before the call and
 *     before what is enqueued after it; the library creates no streams and (outside peqa_trace_begin) no events,
 *     so every call may be recorded by stream capture.
 *   - Arguments are validated on the host before the device is touched, so the
 *     error paths work on a machine without a GPU.  Return value: peqa_status.
 *   - bf16 tensors are passed as uint16_t bit patterns.
 *   - G = number of groups per channel = K / group_size, or 1 when group_size = 0.
 *     Scale-shaped arrays (s0, ds, d_ds, m, v, z0) are [N, G] row-major.
 *
 * Shape limits: N % 128 == 0, K % 128 == 0 (every LLaMA-family linear satisfies
 * this).  group_size is 0 or a multiple of 64 that divides K.
 *
 * Options.  The library reads nothing from the process environment.  Three switches exist for tests and
 * comparisons, set explicitly with peqa_set_option (process-wide, not thread-safe; none is needed):
 * PEQA_OPT_GEMM_WAVES = 4 | 8 forces one of the two forms of the tiled contraction kernel (0, the default:
 * a launch with more than one 128 x 256 tile per compute unit runs four-wave workgroups, two per
 * compute unit, any other launch eight-wave ones); PEQA_OPT_BWD_PAIR = 0 makes a per-channel backward
 * that is asked for both gradients run its two contractions as launches of their own, 1 as one launch of
 * four-wave workgroups (-1, the default: one launch unless PEQA_OPT_GEMM_WAVES is 8);
 * PEQA_OPT_GROUPED_DDS = 1 selects the older of two routes to the scale gradient of group-wise
 * layers (0, the default: the contraction over tokens).  Results agree within rounding.
 *
 * Stacking.  The packed array is stored by rows of 128-channel tiles and the scale-shaped
 * arrays by channel, so layers with equal K, bits and group_size that read the same input
 * (the query, key and value projections; gate and up) can be laid one after the other in
 * memory -- each quantized by its own peqa_quantize call into its slice of packed, s0, z0 --
 * and then run as ONE layer with N = the sum of theirs: Y and dY are [T, sum N] with every
 * member a column range, d_ds is the members' gradients one after the other, and dX is the
 * gradient of the shared input (the sum of the members' dX) from a single contraction.
 * Results per member are those of running it alone -- bit for bit when both runs take the same
 * form of the contraction kernel (see Options; the forms add the same products in a different
 * order), else to the last bf16 bit; only dX, a sum, is new.
 */
#ifndef PEQA_H
#define PEQA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    PEQA_OK = 0,
    PEQA_ERR_NULL = 1,      /* a required pointer is NULL                       */
    PEQA_ERR_SHAPE = 2,     /* N, K or T out of the supported range             */
    PEQA_ERR_BITS = 3,      /* bits is not 3 or 4                               */
    PEQA_ERR_GROUP = 4,     /* group_size invalid for this K                    */
    PEQA_ERR_ALIGN = 5,     /* a device pointer is not 16-byte aligned          */
    PEQA_ERR_WORKSPACE = 6, /* workspace missing or smaller than required       */
    PEQA_ERR_DEVICE = 7,    /* the HIP runtime reported a launch error          */
    PEQA_ERR_PARAM = 8      /* an optimizer or other scalar parameter is invalid */
} peqa_status;

typedef struct {
    int32_t n_out;      /* N: output channels = rows of W0 (the paper's n)             */
    int32_t k_in;       /* K: input features = columns of W0 (the paper's m)           */
    int32_t bits;       /* b: 3 or 4                                                    */
    int32_t group_size; /* 0 = one (s, z) per channel; else g with g % 64 == 0, K % g == 0   */
} peqa_layout;

typedef enum {
    PEQA_OP_FWD = 0,      /* peqa_linear_fwd        */
    PEQA_OP_BWD = 1,      /* peqa_linear_bwd        */
    PEQA_OP_FWD_KEEP = 2, /* peqa_linear_fwd_keep   */
    PEQA_OP_BWD_KEPT = 3, /* peqa_linear_bwd_kept   */
    PEQA_OP_FWD_Z = 4,    /* peqa_linear_fwd_z      */
    PEQA_OP_BWD_Z = 5     /* peqa_linear_bwd_z      */
} peqa_op;

/* Host-only helpers (no device access). */
peqa_status peqa_check_layout(const peqa_layout *L);
size_t peqa_packed_words(const peqa_layout *L);   /* N*K*bits/32 uint32 words; 0 if invalid */
size_t peqa_num_scales(const peqa_layout *L);     /* N*G; 0 if invalid                      */
/* Bytes of scratch the given call needs for T tokens (0 if invalid). */
size_t peqa_workspace_bytes(const peqa_layout *L, int32_t T, int32_t op);
const char *peqa_status_string(int32_t status);

/* Test and comparison switches (see Options above).  peqa_set_option returns PEQA_ERR_PARAM for an unknown
 * option or a value outside those listed; peqa_get_option returns the current value (INT32_MIN if unknown). */
typedef enum {
    PEQA_OPT_GEMM_WAVES = 0,   /* 0 (default), 4, 8 */
    PEQA_OPT_BWD_PAIR = 1,     /* -1 (default), 0, 1 */
    PEQA_OPT_GROUPED_DDS = 2   /* 0 (default), 1 */
} peqa_option;
peqa_status peqa_set_option(int32_t option, int32_t value);
int32_t peqa_get_option(int32_t option);

/*
 * Word and bit (0..31) that hold bit `t` of the code of channel i, feature k in the
 * packed array.  The paper fixes only the density (exactly b bits per weight,
 * Table 4); the placement is this library's and is part of its contract:
 * 8x8 blocks of (channel, feature) of 2b words each, stored tile by tile so that every
 * kernel streams contiguous memory: a tile is 128 channels x 32 features (16 x 4 blocks,
 * 256 b bytes), tile (i/128, k/32) has number (i/128) * (K/32) + k/32, and block
 * (i/8, k/8) is block ((i/8)%16) * 4 + (k/8)%4 of its tile, i.e. it starts at word
 * (64 * tile + block) * 2b; inside a block r = i%8, c = k%8 and
 *   b = 4: word r, bits [4p, 4p+4) with p = c/2 + 4*(c%2);
 *   b = 3: u = 4*(r/2) + c/2; u < 15: word 2*(u/5) + r%2, bits [16*(c%2) + 3*(u%5), +3);
 *          u = 15: code bit t is bit 15 + 16*(c%2) of word 2t + r%2.
 * Host-only.  Returns PEQA_ERR_SHAPE for indices out of range.
 */
peqa_status peqa_bit_location(const peqa_layout *L, int32_t i, int32_t k, int32_t t,
                              size_t *word, int32_t *bit);

/*
 * Eq. 1, round-to-nearest with a min-max range, then dense packing.
 * Per channel i and group g:  xmin = min(min w, 0), xmax = max(max w, 0),
 * s0 = (xmax - xmin) / (2^b - 1), z0 = rint(-xmin / s0),
 * Q = clamp(rint(w / s0) + z0, 0, 2^b - 1); rint rounds half to even; every step is one
 * IEEE fp32 operation.  A group whose s0 evaluates to 0 gets s0 = 1, z0 = 0.
 *   W0      [N, K] fp32, in
 *   packed  peqa_packed_words() uint32, out
 *   s0      [N, G] fp32, out;   z0  [N, G] uint8, out
 */
peqa_status peqa_quantize(const peqa_layout *L, const float *W0, uint32_t *packed,
                          float *s0, uint8_t *z0, void *stream);

/*
 * Error-minimising initialisation.  Sec. 3.2 wants s0, z0 chosen so that the Frobenius norm of W0 - What0 is
 * smallest, and gives no procedure (the experiments use the plain range of Eq. 1); this is the usual grid
 * over clipped ranges.
 * For j = 0 .. n_ratios-1 with r_j = 1 - j * (1 - min_ratio) / (n_ratios - 1)  (r_0 = 1: Eq. 1 itself),
 * every (channel, group) is quantized with the range [r_j xmin, r_j xmax] exactly as in peqa_quantize,
 * and the candidate with the smallest sum_k (w - s (Q - z))^2 is kept (the first of equal ones).
 * Residuals are formed in fp32 and their squares summed in fp64.  n_ratios = 1 equals peqa_quantize.
 *   1 <= n_ratios <= 1024, 0 < min_ratio <= 1 (PEQA_ERR_PARAM otherwise);
 *   supported where a row block fits on chip: K <= 12288 and 384 G + 9 K <= 153600 (PEQA_ERR_SHAPE).
 *   Arguments as peqa_quantize.
 */
peqa_status peqa_quantize_search(const peqa_layout *L, const float *W0, int32_t n_ratios,
                                 float min_ratio, uint32_t *packed, float *s0, uint8_t *z0,
                                 void *stream);

/*
 * Eq. 2 forward:  Y[t,i] = sum_k X[t,k] * (s0+ds)[i,g(k)] * (Q[i,k] - z0[i,g(k)]).
 *   ds may be NULL (= 0).  X [T, K] bf16 in, Y [T, N] bf16 out, T >= 1.
 *   bf16 operands, fp32 accumulation.  T <= 16 takes the bandwidth-bound
 *   matrix-vector path of Sec. 3.1 ("Inference Latency").
 *   Per-channel layers and the T <= 16 path contract over the exact integer codes and
 *   apply scale and zero-point in fp32 afterwards; group-wise layers with T > 16 (and
 *   their dX) form every weight (s0+ds)(Q - z0) in fp32 and round it once to bf16 before
 *   the contraction.
 *   workspace: peqa_workspace_bytes(L, T, PEQA_OP_FWD) bytes, contents undefined on return.
 */
peqa_status peqa_linear_fwd(const peqa_layout *L, const uint32_t *packed, const float *s0,
                            const float *ds, const uint8_t *z0, const uint16_t *X, int32_t T,
                            uint16_t *Y, void *workspace, size_t workspace_bytes, void *stream);

/*
 * peqa_linear_fwd for callers that cannot allocate device memory and have no workspace to pass: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same kernels and the same
 * result bit for bit as peqa_linear_fwd; the scratch a forward needs (row sums of X, the group table, or the
 * partial sums of the T <= 16 path) lives in an array of PEQA_STATIC_SCRATCH_BYTES that is part of the library's
 * device image (every GPU the library runs on holds its own copy until the process ends).  The call allocates
 * nothing and frees nothing.  A forward that needs more scratch than that (peqa_workspace_bytes(L, T,
 * PEQA_OP_FWD) > PEQA_STATIC_SCRATCH_BYTES) is refused with PEQA_ERR_WORKSPACE before anything is enqueued.
 * All calls on one GPU share that GPU's array: calls that overlap in time on one GPU (two streams, two
 * threads) race on it; calls on one stream are ordered and safe.  Nothing in the array needs to start at zero.
 * The array's device address is looked up once per device, at the first call on that device (not a stream
 * operation: make that first call outside a capture).
 */
#define PEQA_STATIC_SCRATCH_BYTES (16u << 20)
peqa_status peqa_linear_fwd_static(const peqa_layout *L, const uint32_t *packed, const float *s0,
                                   const float *ds, const uint8_t *z0, const uint16_t *X, int32_t T,
                                   uint16_t *Y, void *stream);

/*
 * The same forward for 1..PEQA_MAX_FUSED layers that read the same X (the query / key / value
 * projections of an attention block; the gate and up projections of its MLP): equal to calling
 * peqa_linear_fwd once per item, every item writing its own Y.  All items must share k_in, bits
 * and group_size (PEQA_ERR_PARAM otherwise).  With T <= 16 (Sec. 3.1, "Inference Latency": bound by
 * the weight bytes streamed) the layers run side by side in one launch, which matters because
 * a single LLaMA-size layer at such T is too short to fill the machine; larger T runs them one
 * after the other.  `items` is a HOST array; workspace: peqa_workspace_bytes_fused() bytes.
 */
#define PEQA_MAX_FUSED 4
typedef struct {
    peqa_layout layout;
    const uint32_t *packed;
    const float *s0;
    const float *ds;     /* may be NULL */
    const uint8_t *z0;
    uint16_t *Y;         /* [T, layout.n_out] bf16 out */
} peqa_fwd_item;

size_t peqa_workspace_bytes_fused(int32_t n, const peqa_fwd_item *items, int32_t T);
peqa_status peqa_linear_fwd_fused(int32_t n, const peqa_fwd_item *items, const uint16_t *X, int32_t T,
                                  void *workspace, size_t workspace_bytes, void *stream);

/*
 * The linears of a decoder block behind one call (Sec. 3.1 motivates PEQA by the cost of the fully-connected
 * layers of a block: the query / key / value / output projections and the gate / up / down projections of
 * LLaMA; Eq. 2 is applied to each).  An item is one layer with its own input: peqa_block_fwd equals
 * peqa_linear_fwd per item, peqa_block_bwd equals peqa_linear_bwd per item, up to the order of floating-point
 * additions.  Items are independent of each other: no item's input may be another item's output of the same
 * call.  Layers that read one input are best passed stacked as one item (see Stacking); items may also
 * simply share an X pointer.  All items share T and the bit width (PEQA_ERR_PARAM otherwise); shapes and
 * group sizes may differ.
 *   T <= 16 (the deployment path of Sec. 3.1): every layer of the call runs in ONE launch, whose workgroups
 *     get equal shares of the packed bytes, plus one short launch that adds up the feature slices of the
 *     layers that were sliced.
 *   T > 16, per-channel layers: forward = the row sums of all distinct inputs in one launch, then all
 *     items' contractions in one launch of four-wave tiles, longest contraction first.  Backward = all scale-gradient
 *     contractions in one launch whose grid also carries the scaling of dY for every item, then all dX
 *     contractions in one launch whose grid also carries the fixed-order sums of the scale-gradient partials.
 *     Group-wise layers: forward = the scale tables of all items in one launch, then all contractions in one
 *     launch.  Backward = the tables, then all dX contractions in one launch whose grid also writes the
 *     transposed copies of X (once per distinct X) and dY, then the token contractions of all scale
 *     gradients in one launch and the sums of their chunks in another.  (Always the token-contraction
 *     route: PEQA_OPT_GROUPED_DDS is not consulted.)
 *   row_sums (optional, [T, 2] fp32 per distinct X, caller-owned): when not NULL, peqa_block_fwd stores the row
 *     sums of the item's X there (see peqa_row_sums) and peqa_block_bwd reads them instead of taking them again;
 *     items that share X may share the array.  Ignored by T <= 16 and by group-wise layers.
 *   `items` is a HOST array of 1..PEQA_MAX_BLOCK entries; workspace: peqa_block_workspace_bytes(n, items, T, op)
 *   with op = PEQA_OP_FWD or PEQA_OP_BWD, contents undefined on return.  dX and d_ds may be NULL per item (skipped).
 */
#define PEQA_MAX_BLOCK 8
typedef struct {
    peqa_layout layout;
    const uint32_t *packed;
    const float *s0;
    const float *ds;       /* may be NULL */
    const uint8_t *z0;
    const uint16_t *X;     /* [T, layout.k_in] bf16, in (both calls; may be NULL in the backward when d_ds is) */
    uint16_t *Y;           /* [T, layout.n_out] bf16, out of peqa_block_fwd (unused by the backward)           */
    const uint16_t *dY;    /* [T, layout.n_out] bf16, in of peqa_block_bwd (unused by the forward)             */
    uint16_t *dX;          /* [T, layout.k_in] bf16, out of peqa_block_bwd, or NULL                            */
    float *d_ds;           /* [N, G] fp32, out of peqa_block_bwd (overwritten), or NULL                        */
    float *row_sums;       /* optional, see above                                                              */
} peqa_block_item;

size_t peqa_block_workspace_bytes(int32_t n, const peqa_block_item *items, int32_t T, int32_t op);
peqa_status peqa_block_fwd(int32_t n, const peqa_block_item *items, int32_t T, void *workspace,
                           size_t workspace_bytes, void *stream);
peqa_status peqa_block_bwd(int32_t n, const peqa_block_item *items, int32_t T, void *workspace,
                           size_t workspace_bytes, void *stream);

/*
 * Backward of Eq. 2 by the chain rule (only the scales are trained, Sec. 3.2):
 *   dX[t,k]   = sum_i dY[t,i] * (s0+ds)[i,g(k)] * (Q[i,k] - z0[i,g(k)])
 *   d_ds[i,g] = sum_t dY[t,i] * sum_{k in g} X[t,k] * (Q[i,k] - z0[i,g])
 *   dX [T, K] bf16 out, or NULL to skip; d_ds [N, G] fp32 out (overwritten, not
 *   accumulated), or NULL to skip.  X may be NULL when d_ds is NULL.
 *   The result is deterministic (fixed reduction order, no atomics): the same call gives the
 *   same bits.  A call that skips one gradient may run the other's contraction in another form of
 *   the kernel than a call that asks for both (see Options): the same products added in
 *   another order, so the two agree to the last bf16 bit of dX / 1e-5 of |d_ds|, not bit for bit.
 *   Group-wise layers take d_ds by the other order of the two sums,
 *   d_ds[i,g] = sum_{k in g} (sum_t dY[t,i] X[t,k]) (Q[i,k] - z0[i,g]); their backward workspace
 *   therefore also holds transposed copies of X and dY (2 (K + N) T' bytes, T' = T rounded up to 64).
 */
peqa_status peqa_linear_bwd(const peqa_layout *L, const uint32_t *packed, const float *s0,
                            const float *ds, const uint8_t *z0, const uint16_t *X,
                            const uint16_t *dY, int32_t T, uint16_t *dX, float *d_ds,
                            void *workspace, size_t workspace_bytes, void *stream);

/*
 * Row sums shared between calls.  The per-channel contractions for T > 16 take the code offset and the
 * zero-point out of the contraction through the sums of every row of X over the two halves of K,
 *   row_sums[t] = ( sum_{k < ks} X[t,k],  sum_{k >= ks} X[t,k] ),   ks = (K / 2) rounded down to 64,
 * which peqa_linear_fwd(_fused) and peqa_linear_bwd otherwise take themselves at every call (a launch of
 * several microseconds each).  A training step can take them once per activation with peqa_row_sums
 * ([T, 2] fp32: 8 T bytes to keep until the backward) and hand them to the forward of the layers that read
 * that X and, later, to their backward.  row_sums = NULL makes these calls equal to the plain ones; calls
 * that do not use such sums (T <= 16, group-wise layers) ignore the argument.
 */
peqa_status peqa_row_sums(const uint16_t *X, int32_t T, int32_t K, float *row_sums, void *stream);
peqa_status peqa_linear_fwd_fused_rs(int32_t n, const peqa_fwd_item *items, const uint16_t *X,
                                     const float *row_sums, int32_t T, void *workspace,
                                     size_t workspace_bytes, void *stream);
peqa_status peqa_linear_bwd_rs(const peqa_layout *L, const uint32_t *packed, const float *s0,
                               const float *ds, const uint8_t *z0, const uint16_t *X,
                               const float *row_sums, const uint16_t *dY, int32_t T, uint16_t *dX,
                               float *d_ds, void *workspace, size_t workspace_bytes, void *stream);

/*
 * Optional trade of activation memory for arithmetic, per-channel layers only (PEQA_ERR_GROUP for
 * group-wise ones).  In the scale gradient of Eq. 2,  d_ds[i] = sum_t dY[t,i] * P[t,i]  with
 *   P[t,i] = sum_k X[t,k] * (Q[i,k] - z0[i]),
 * and Y[t,i] = (s0+ds)[i] * P[t,i]: the forward already forms P.  peqa_linear_fwd_keep writes it
 * (fp32, [T, N], caller-owned: 4 T N bytes per layer, against the memory motive of Sec. 3.1) next to
 * the same Y as peqa_linear_fwd; peqa_linear_bwd_kept then takes d_ds from dY and P with one pass
 * over both instead of the contraction over X, so that forward + backward cost 4 T N K flops, not
 * 6 T N K.  dX, NULL arguments and determinism as in peqa_linear_bwd; P may be NULL when d_ds is.
 *   any T >= 1 (the forward always runs the tiled contraction);
 *   workspace: peqa_workspace_bytes(L, T, PEQA_OP_FWD_KEEP / PEQA_OP_BWD_KEPT).
 */
peqa_status peqa_linear_fwd_keep(const peqa_layout *L, const uint32_t *packed, const float *s0,
                                 const float *ds, const uint8_t *z0, const uint16_t *X, int32_t T,
                                 uint16_t *Y, float *P, void *workspace, size_t workspace_bytes,
                                 void *stream);
peqa_status peqa_linear_bwd_kept(const peqa_layout *L, const uint32_t *packed, const float *s0,
                                 const float *ds, const uint8_t *z0, const float *P,
                                 const uint16_t *dY, int32_t T, uint16_t *dX, float *d_ds,
                                 void *workspace, size_t workspace_bytes, void *stream);

/*
 * Trainable zero-points (Appendix K, "Choice of Updating Quantization Scales or Zero-Points": zero-points
 * only, or zero-points and scales together).  The zero-point becomes the real number z = z0 + dz with
 * dz [N, G] fp32 (NULL = 0); the codes stay frozen and Eq. 2 reads What = (s0+ds) (Q - z).
 *   peqa_linear_fwd_z:  Y as peqa_linear_fwd with z in place of z0 (every T, per-channel and group-wise).
 *   peqa_linear_bwd_z:  dX and d_ds as peqa_linear_bwd with z in place of z0, and
 *     d_dz[i,g] = -(s0+ds)[i,g] * sum_t dY[t,i] * sum_{k in g} X[t,k]      [N, G] fp32 out, or NULL to skip
 *   (z enters What only through -s z).  X may be NULL when d_ds and d_dz both are.
 *   dz is updated with peqa_scale_update(n, dz, d_dz, m, v, s0, opt): with opt->weight_decay = 0 the
 *   s0 argument is read but has no effect (pass the scales).
 *   workspace: peqa_workspace_bytes(L, T, PEQA_OP_FWD_Z / PEQA_OP_BWD_Z).
 */
peqa_status peqa_linear_fwd_z(const peqa_layout *L, const uint32_t *packed, const float *s0,
                              const float *ds, const uint8_t *z0, const float *dz, const uint16_t *X,
                              int32_t T, uint16_t *Y, void *workspace, size_t workspace_bytes,
                              void *stream);
peqa_status peqa_linear_bwd_z(const peqa_layout *L, const uint32_t *packed, const float *s0,
                              const float *ds, const uint8_t *z0, const float *dz, const uint16_t *X,
                              const uint16_t *dY, int32_t T, uint16_t *dX, float *d_ds, float *d_dz,
                              void *workspace, size_t workspace_bytes, void *stream);

/*
 * One AdamW step on ds (Appendix A names AdamW with a linearly decaying learning rate;
 * the schedule is the caller's, who passes the current lr).  step is 1-based.
 *   m <- b1 m + (1-b1) g;  v <- b2 v + (1-b2) g^2
 *   ds <- ds - lr * ( (m / (1-b1^step)) / (sqrt(v / (1-b2^step)) + eps) + wd * (s0 + ds) )
 * ds, m, v [n] fp32 in/out (m, v zero-initialised by the caller); d_ds, s0 [n] fp32 in.
 */
typedef struct {
    float lr, beta1, beta2, eps, weight_decay;
    int32_t step;
} peqa_adamw;

peqa_status peqa_scale_update(size_t n_scales, float *ds, const float *d_ds, float *m, float *v,
                              const float *s0, const peqa_adamw *opt, void *stream);

/*
 * The same step on the scales of 1..PEQA_MAX_UPDATE layers in one launch (a decoder block's seven
 * updates are each a few microseconds of work behind a launch): equal to calling peqa_scale_update
 * once per item with the same `opt`.  `items` is a HOST array.
 */
#define PEQA_MAX_UPDATE 16
typedef struct {
    size_t n_scales;
    float *ds;           /* in/out */
    const float *d_ds;
    float *m, *v;        /* in/out */
    const float *s0;
} peqa_update_item;

peqa_status peqa_scale_update_multi(int32_t n, const peqa_update_item *items, const peqa_adamw *opt,
                                    void *stream);

/* Compute units and peak engine clock (kHz) of the current device, as the HIP runtime reports them
 * (for benchmark reports: the denominators of roofline fractions). */
peqa_status peqa_device_info(int32_t *compute_units, int32_t *clock_khz);

/*
 * Per-kernel timing for benchmarks.  peqa_trace_begin() makes every kernel the library
 * launches afterwards be bracketed by HIP events on its stream (it creates the events:
 * call it outside any region that must not allocate).  peqa_trace_end() synchronises those
 * events, stops tracing and fills, for up to `max_kernels` distinct kernels, a name
 * (static string), the number of launches and the summed duration in milliseconds;
 * it returns the number of distinct kernels seen.  Not thread-safe.
 */
peqa_status peqa_trace_begin(int32_t max_launches);
/* Restricts tracing to the kernels whose reported name starts with `prefix` (NULL or "": all kernels, the
 * default).  Bracketing only the kernel of interest leaves the other launches of a timed region back to back,
 * as they are without tracing.  Names are at most 31 characters (PEQA_ERR_PARAM otherwise). */
peqa_status peqa_trace_select(const char *prefix);
int32_t peqa_trace_end(int32_t max_kernels, const char **names, int32_t *launches, float *total_ms);

#ifdef __cplusplus
}
#endif
#endif /* PEQA_H */
