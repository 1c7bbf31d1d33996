/*
 * symb.h -- C ABI of the MI355X (gfx950) base-executor layer with per-client adapters.
 *
 * One call runs ONE frozen linear layer over the flattened, padding-free token batch
 * of many clients and applies each client's own adapter to that client's token
 * segment.  Method: Symbiosis (arXiv 2507.03220):
 *   - Sec. 3.2 "Base Executor": requests of many clients for one layer are batched,
 *     the layer is executed once, the result is split per client.
 *   - Sec. 3.7: token position is irrelevant for nn.Linear, so all clients' tokens
 *     are concatenated along one token axis with no padding.
 *   - Sec. 3.6: the layer is frozen; backward multiplies the output gradient by the
 *     parameters, saves nothing from forward, and may run on a different batch.
 *   - Sec. 3.8 eqs. (1)-(3): optional bias; a bias-free pass exists.
 *   - Sec. 1 and Sec. 3.2 "Client": every client chooses its own PEFT method and
 *     parameters (LoRA rank and alpha, IA3).  The paper keeps the adapter at the
 *     client; here client and executor share one GPU (its "local" placement, Sec. 3.3)
 *     and the adapter term is fused into the same call.  kind NONE for every segment
 *     gives exactly the paper's executor.
 *
 * Notation.  S segments; segment i owns rows off[i] .. off[i+1]-1 of every [T][*]
 * tensor, T = off[S].  For a row t of segment i:
 *     Y0[t][j] = sum_k X[t][k] W[j][k] (+ bias[j])
 *     NONE : Y = Y0
 *     LORA : H[t][p] = sum_k X[t][k] A_i[p][k];   Y[t][j] = Y0[t][j] + s_i sum_p H[t][p] B_i[j][p]
 *     IA3  : Y[t][j] = l_i[j] Y0[t][j]
 *   backward (on the backward batch's own segments):
 *     NONE : dX[t][k] = sum_j dY[t][j] W[j][k]
 *     LORA : dH[t][p] = s_i sum_j dY[t][j] B_i[j][p];  dX[t][k] = sum_j dY[t][j] W[j][k] + sum_p dH[t][p] A_i[p][k]
 *            dA_i[p][k] = sum_{t in i} dH[t][p] X[t][k];   dB_i[j][p] = s_i sum_{t in i} dY[t][j] H[t][p]
 *     IA3  : dX[t][k] = sum_j dY[t][j] l_i[j] W[j][k];     dl_i[j] = sum_{t in i} dY[t][j] Y0[t][j]
 *
 * Types and layouts.  All matrices are dense row-major with no row stride argument.
 * Activations, weights, bias and adapter tensors are bf16; accumulation is fp32;
 * base and adapter terms are summed in fp32 and rounded once (nearest-even) to bf16
 * at the store (H and dH travel between kernels as a bf16 value plus a bf16 rounding
 * residual, i.e. with about 16 significand bits).  Adapter gradients
 * are fp32 in the layout of the tensor they belong to.  Device pointers must be
 * 16-byte aligned; d_in and d_out must be multiples of 8.
 *
 * Ownership.  The caller owns every device buffer and the workspace.  Host arrays
 * (offsets, descriptors) are copied during the call and may be freed on return.
 * The library allocates device memory only inside symb_create.
 *
 * Ordering.  All GPU work is enqueued on the given stream (a hipStream_t passed as
 * void*; NULL = the default stream); calls return without synchronising.  Calls on
 * different streams may be in flight together as long as their output buffers and
 * workspaces are distinct.  Calls on one handle from several host threads must be
 * serialised by the caller.
 *
 * Errors.  Every entry point returns a symb_status; nothing throws or aborts.  All
 * argument checks happen before the first launch: a failing call enqueues nothing,
 * leaves outputs untouched and the handle usable.  The library is stateless across
 * calls (Sec. 3.6): no call depends on an earlier one.
 */
#ifndef SYMB_H
#define SYMB_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    SYMB_OK = 0,
    SYMB_ERR_INVALID_ARG = 1,         /* null pointer, bad dimension, bad flag, misaligned pointer */
    SYMB_ERR_BAD_SEGMENTS = 2,        /* off[0] != 0 or offsets decrease */
    SYMB_ERR_UNSUPPORTED = 3,         /* valid request this build cannot run (e.g. rank > SYMB_MAX_RANK) */
    SYMB_ERR_WORKSPACE_TOO_SMALL = 4,
    SYMB_ERR_DEVICE = 5               /* a HIP call failed; see symb_last_error */
} symb_status;

typedef enum {
    SYMB_ADAPTER_NONE = 0,
    SYMB_ADAPTER_LORA = 1,
    SYMB_ADAPTER_IA3 = 2,             /* output scaling, l[d_out] */
    SYMB_ADAPTER_IA3_IN = 3           /* input scaling, l[d_in]: y = (l * x) W^T */
} symb_adapter_kind;

enum { SYMB_MAX_RANK = 128 };

typedef enum { SYMB_OP_FWD = 0, SYMB_OP_BWD_INPUT = 1, SYMB_OP_ADAPTER_GRAD = 2,
               /* the per-segment forms called with output buffers that overlap input buffers (see below) */
               SYMB_OP_FWD_INPLACE = 3, SYMB_OP_BWD_INPUT_INPLACE = 4 } symb_op;

/* flags of symb_base_linear_bwd_input */
enum { SYMB_BWD_FULL = 0,             /* dX includes each segment's adapter branch */
       SYMB_BWD_BASE_ONLY = 1,        /* dX = dY W only: what the paper's executor returns (Sec. 3.6) */
       /* (with SYMB_BWD_FULL) dH = s dY B is taken from `ws` instead of being computed: `ws` must be the very
        * workspace a preceding symb_adapter_grad call used for this same batch and dY (a call that wanted dA
        * of every LoRA segment, so that it computed dH for all of them), untouched since.  A gradient call
        * followed by the input gradient this way reads dY twice instead of three times: for ranks up to 16
        * the gradient call forms dB and dH in one pass.  The caller carries the workspace over; the
        * library stays stateless. */
       SYMB_BWD_REUSE_DH = 2 };
/* flags of symb_adapter_grad */
enum { SYMB_GRAD_OVERWRITE = 0, SYMB_GRAD_ACCUMULATE = 1,
       /* dH is taken from `ws` instead of being recomputed: `ws` must be the very workspace a
        * preceding symb_base_linear_bwd_input(SYMB_BWD_FULL) call used for this same batch and dY,
        * untouched since (the caller, not the library, carries it over: the library stays stateless) */
       SYMB_GRAD_REUSE_DH = 2,
       /* Hs = s (X A^T) is taken from `ws` instead of being recomputed: `ws` must be the very
        * workspace a preceding symb_base_linear_fwd call used for this same batch and X, and any
        * call in between must have been on this same batch too (their regions do not overlap Hs) */
       SYMB_GRAD_REUSE_HS = 4 };

/* One segment's adapter (Sec. 3.2 "Client": method and parameters are per client). */
typedef struct {
    int32_t kind;      /* symb_adapter_kind */
    int32_t rank;      /* LoRA: r >= 1 (any integer up to SYMB_MAX_RANK); otherwise ignored */
    float scale;       /* LoRA: s = alpha / r, passed explicitly; otherwise ignored */
    const void* A;     /* DEVICE. LoRA: bf16 [rank][d_in].  IA3: bf16 l[d_out].  IA3_IN: bf16 l[d_in] */
    const void* B;     /* DEVICE. LoRA: bf16 [d_out][rank].  otherwise NULL */
    void* dA;          /* DEVICE fp32, layout of A (IA3: dl[d_out], IA3_IN: dl[d_in]); NULL = no gradient wanted */
    void* dB;          /* DEVICE fp32, layout of B; NULL = no gradient wanted */
} symb_adapter;

/* Storage of the frozen weight.  The base layers the paper serves are nn.Linear or Conv1D
 * (Sec. 3.7, 3.8): the same linear map, the weight stored output-major or input-major. */
typedef enum { SYMB_WEIGHT_LINEAR = 0,   /* W [d_out][d_in]: y = x W^T + b  (nn.Linear) */
               SYMB_WEIGHT_CONV1D = 1    /* W [d_in][d_out]: y = x W + b    (Conv1D of GPT-2-style models) */
             } symb_weight_layout;

/* A flattened batch (Sec. 3.7): segment offsets plus one adapter per segment. */
typedef struct {
    int32_t d_in, d_out, num_segments;
    const int32_t* seg_offsets;    /* HOST, num_segments+1 entries, off[0]=0, non-decreasing; T = off[S] */
    const symb_adapter* adapters;  /* HOST, num_segments entries */
    int32_t weight_layout;         /* symb_weight_layout of the W passed with this batch; adapters keep their layouts */
} symb_batch;

typedef struct symb_context* symb_handle;

/* Creates a context on HIP device `device`: descriptor staging (pinned host ring +
 * device ring, 32 slots of 2 MiB each).  The only call that allocates.  A later call
 * whose offsets, adapters and buffers give the same descriptor bytes as an earlier call
 * on the same stream reads the copy already on the device instead of sending it again.
 * A call's descriptors (about 170 bytes per segment plus 16 per row tile and row chunk) must fit
 * one slot: batches beyond roughly 12 000 segments are refused with SYMB_ERR_UNSUPPORTED before
 * anything is launched.  SYMB_ERR_DEVICE if HIP fails. */
symb_status symb_create(symb_handle* out, int device);
symb_status symb_destroy(symb_handle h);

/* Host-only checks shared by every entry point (no GPU needed): dimensions, offsets
 * (Sec. 3.7), per-segment descriptors.  Empty segments, S = 1, T = 0 are legal. */
symb_status symb_validate_batch(const symb_batch* b);

/* seg(t) = i <=> off[i] <= t < off[i+1], written to host_out[0..T-1] (Sec. 3.2: the
 * split of the flattened batch back into clients).  Host-only. */
symb_status symb_debug_row_segment_map(const symb_batch* b, int32_t* host_out);

/* Host-only planner: for row tiles of `tile_m` rows, tile u covers rows
 * [u*tile_m, min(T,(u+1)*tile_m)) and meets the non-empty segments seg_lo[u]..seg_hi[u]
 * (inclusive).  Writes ceil(T/tile_m) entries to each array; *num_tiles gets the count. */
symb_status symb_plan_row_tiles(const symb_batch* b, int32_t tile_m, int32_t* seg_lo,
                                int32_t* seg_hi, int32_t* num_tiles);

/* Bytes of caller-owned device workspace an operation needs for this batch (may be 0).
 * Host-only.  For some forward and input-gradient calls the figure ends with a region for
 * fp32 partial tiles: such a call computes output tiles in several workgroups, one per
 * range of the inner dimension -- every tile of a batch of a few hundred rows (which alone
 * would leave most of the chip idle), or the tiles of a last round of workgroups that
 * would be partly empty (up to 160 MiB).  Before it, for a batch of at most 16 rows, come
 * the regions of the weight-streaming kernels such calls take (a flat copy of the rows and,
 * where the weight is read N-contiguous, up to 8 MiB of fp32 partial sums per K range).  These
 * trailing regions are optional: a workspace that covers everything before them (in
 * particular none at all for a batch without adapters) makes the call take the tiled kernel
 * without the split, only slower; anything smaller fails with SYMB_ERR_WORKSPACE_TOO_SMALL.
 * The figure depends on the batch and the operation alone (not on the handle or its options).  Every call is deterministic (the same arguments give the
 * same bits, whatever order the workgroups finish in); a split call sums the inner dimension
 * in a different order than an unsplit one, so the two can differ in the last rounding.  For
 * SYMB_OP_ADAPTER_GRAD the figure includes room for the partial sums of LoRA gradients of
 * segments longer than 1536 tokens (summed in runs of 1024 tokens, the runs added in order: a
 * segment's gradient does not depend on what else is in the batch) and, for ranks up to 16 on
 * layers at least 16384 wide, for the partial sums of dH of the pass that forms dB and dH together. */
symb_status symb_workspace_bytes(const symb_batch* b, int32_t op, size_t* out);

/*
 * Forward (Sec. 3.2, 3.7; eqs. of Sec. 3.8 for the bias):  Y = adapter_i(X W^T + bias).
 *   X [T][d_in] bf16 DEVICE, W [d_out][d_in] bf16 DEVICE (nn.Linear layout),
 *   bias [d_out] bf16 DEVICE or NULL, Y [T][d_out] bf16 DEVICE (written),
 *   Ybase [T][d_out] bf16 DEVICE or NULL: if given, receives Y0 (the pre-adapter
 *   output the paper's executor would have returned; needed later for IA3 dl).  Rows of
 *   IA3_IN segments hold (l * x) W^T + bias there: their input is scaled before the layer.
 *   ws: DEVICE workspace of at least symb_workspace_bytes(.., SYMB_OP_FWD, ..) bytes.
 */
symb_status symb_base_linear_fwd(symb_handle h, const symb_batch* b, const void* X, const void* W,
                                 const void* bias, void* Y, void* Ybase, void* ws, size_t ws_bytes,
                                 void* stream);

/*
 * Activation privacy (Sec. 3.8, eqs. (1)-(3)).  A client hides its activations by adding noise n
 * before the layer and removing the noise effect n_eff afterwards; because the layer (and a LoRA
 * or IA3 adapter on it) is linear, the result is the one the plain call would have given.
 *   (1) n_eff = layer(n) without bias: symb_base_linear_fwd on a batch whose segments hold the
 *       noise rows, with bias == NULL (the bias-nullifying flow), the clients' own adapters.
 *   (2) y_noisy = layer(x + n) + b, (3) y = y_noisy - n_eff: symb_noise_add, then
 *       symb_base_linear_fwd_denoise, which subtracts n_eff in the epilogue, in fp32, before the
 *       single rounding to bf16.
 * A segment's noise tensor: rows == 1 broadcasts one row over the segment, rows == n_i gives
 * every token its own row; ptr NULL = nothing for this segment.  Rows are dense bf16 DEVICE
 * memory, 16-byte aligned, of width d_in (noise) or d_out (noise effect).
 */
typedef struct {
    const void* ptr;
    int32_t rows;
    int32_t reserved;
} symb_noise;

/* Xn[t][k] = bf16(X[t][k] + n_seg(t)[.][k]) over the flattened batch (width b->d_in); the sum is
 * formed in fp32 and rounded once.  noise: HOST array of b->num_segments entries. */
symb_status symb_noise_add(symb_handle h, const symb_batch* b, const void* X, const symb_noise* noise,
                           void* Xn, void* stream);

/* symb_base_linear_fwd with  Y = (adapter-applied output, bias included) - n_eff  per segment.
 * noise_effect: HOST array of b->num_segments entries (rows of width d_out).  No Ybase output. */
symb_status symb_base_linear_fwd_denoise(symb_handle h, const symb_batch* b, const void* Xn, const void* W,
                                         const void* bias, const symb_noise* noise_effect, void* Y,
                                         void* ws, size_t ws_bytes, void* stream);

/*
 * Input gradient (Sec. 3.6):  dX = dY W (+ adapter branch unless SYMB_BWD_BASE_ONLY).
 *   dY [T'][d_out] bf16 DEVICE, W as above, dX [T'][d_in] bf16 DEVICE (written).
 *   The batch is the backward batch's own (any subset / regrouping of clients).
 */
symb_status symb_base_linear_bwd_input(symb_handle h, const symb_batch* b, const void* dY,
                                       const void* W, void* dX, uint32_t flags, void* ws,
                                       size_t ws_bytes, void* stream);
/* The same, with an optional second output dXbase [T'][d_in] bf16 DEVICE: the input gradient
 * before the input-side adapter terms (LoRA branch, IA3 input scale), i.e. what the paper's
 * executor hands back (Sec. 3.6).  A client with an IA3_IN adapter keeps it for dl (below). */
symb_status symb_base_linear_bwd_input_ex(symb_handle h, const symb_batch* b, const void* dY,
                                          const void* W, void* dX, void* dXbase, uint32_t flags,
                                          void* ws, size_t ws_bytes, void* stream);

/*
 * Per-client buffers (Sec. 3.5: the executor and a local client share pre-allocated buffers).  The
 * same forward / input gradient with the rows of segment i read from X_seg[i] (dY_seg[i]) and
 * written to Y_seg[i] (dX_seg[i]) instead of one flattened tensor each: no concatenation before
 * the call, no split after it.  The arrays are HOST arrays of num_segments DEVICE pointers (dense
 * bf16 rows, 16-byte aligned; an empty segment's entry is ignored).  The input buffers of one call
 * must lie within one 4 GiB window (SYMB_ERR_UNSUPPORTED otherwise): carve them from one arena.
 * With an IA3_IN segment in the batch the forward multiplies a flat, scaled copy of all rows (in the
 * workspace, as the flat call does) and the window rule does not apply.  No Ybase / dXbase output in
 * this form: a client that needs the pre-adapter output for an IA3 gradient keeps its own output of
 * an all-NONE call, one that needs the input gradient before the input scale for an IA3_IN gradient
 * keeps the rows a SYMB_BWD_BASE_ONLY call wrote for it, which is the paper's flow (Sec. 3.6).
 *
 * One buffer per client for both directions (Sec. 3.5: each client pre-allocates a single tensor of
 * batch x sequence x max(d_in, d_out) elements and every layer's input and output travel through
 * it): an output buffer may overlap any input buffer of the call, in particular
 * Y_seg[i] == X_seg[i] (dX_seg[i] == dY_seg[i]), rows dense at their own widths.  The library
 * detects the overlap; such a call computes into a flat copy in the workspace and then scatters
 * the rows, in stream order, so every input row is read before any output row lands.  It needs the
 * larger workspace that SYMB_OP_FWD_INPLACE / SYMB_OP_BWD_INPUT_INPLACE report (the plain figure
 * plus T x width x 2 bytes; SYMB_ERR_WORKSPACE_TOO_SMALL otherwise) and costs one extra pass over
 * the output.  Output buffers must not overlap each other.  After an in-place input gradient dY is
 * gone: run symb_adapter_grad_seg first.
 */
symb_status symb_base_linear_fwd_seg(symb_handle h, const symb_batch* b, const void* const* X_seg,
                                     const void* W, const void* bias, void* const* Y_seg, void* ws,
                                     size_t ws_bytes, void* stream);
symb_status symb_base_linear_bwd_input_seg(symb_handle h, const symb_batch* b, const void* const* dY_seg,
                                           const void* W, void* const* dX_seg, uint32_t flags, void* ws,
                                           size_t ws_bytes, void* stream);
/* Adapter gradients from per-client buffers.  Ybase_seg[i] is what client i kept for its dl: the
 * pre-adapter output rows [n_i][d_out] of an IA3 segment, the rows [n_i][d_in] of the input gradient
 * before the input scale (dY W) of an IA3_IN segment; ignored for other segments; the array may be
 * NULL if no such segment wants dl.  No window restriction here; the SYMB_GRAD_REUSE_* flags work as
 * in the flat call. */
symb_status symb_adapter_grad_seg(symb_handle h, const symb_batch* b, const void* const* X_seg,
                                  const void* const* dY_seg, const void* const* Ybase_seg, uint32_t flags,
                                  void* ws, size_t ws_bytes, void* stream);

/*
 * Adapter gradients per segment (the client-side autograd of Sec. 3.2, fused here):
 * for every segment whose descriptor has dA / dB non-NULL, writes (OVERWRITE) or adds
 * to (ACCUMULATE; flags may be OR-ed with SYMB_GRAD_REUSE_DH / SYMB_GRAD_REUSE_HS) dA_i, dB_i (LoRA) or dl_i (IA3, through dA).  An empty segment
 * writes zeros (OVERWRITE) or leaves the buffers alone (ACCUMULATE).
 *   X [T'][d_in], dY [T'][d_out] bf16 DEVICE; Ybase [T'][d_out] bf16 DEVICE, required
 *   iff some IA3 segment wants dl (else may be NULL -> SYMB_ERR_INVALID_ARG if needed).
 */
symb_status symb_adapter_grad(symb_handle h, const symb_batch* b, const void* X, const void* dY,
                              const void* Ybase, uint32_t flags, void* ws, size_t ws_bytes,
                              void* stream);
/* The same, with dXbase [T'][d_in] bf16 DEVICE (from symb_base_linear_bwd_input_ex), required iff
 * some IA3_IN segment wants dl:  dl_i[k] = sum_t X[t][k] * dXbase[t][k]. */
symb_status symb_adapter_grad_ex(symb_handle h, const symb_batch* b, const void* X, const void* dY,
                                 const void* Ybase, const void* dXbase, uint32_t flags, void* ws,
                                 size_t ws_bytes, void* stream);

/*
 * Measurement hook (not part of the method): while enabled, every launch of the base
 * GEMM kernel is bracketed by a pair of HIP events on the caller's stream, so a bench
 * can read that kernel's own duration inside its timed region.  `variant` names the
 * instantiation symb_gemm16_kernel<NBLK, NN, PLAIN>: bit 0 = NN (the weight is read
 * N-contiguous: input gradient of an nn.Linear weight), bit 1 = the 128x128 tile (NBLK 4, else
 * 256x256, NBLK 8), bit 2 = the full epilogue (PLAIN false); 0..7.
 * read synchronises on the recorded events and returns the totals since the last
 * enable call (which clears them).  At most 4096 launches are recorded after an
 * enable; later ones are not timed.  `flops_total` is the algorithmic work of those launches
 * (2*M*N*K plus the fused LoRA term 2*n_i*r_i*N per segment).
 */
symb_status symb_debug_gemm_timing_enable(symb_handle h, int32_t on);
symb_status symb_debug_gemm_timing_read(symb_handle h, int32_t variant, double* ms_total,
                                        int64_t* launches, double* flops_total);

/*
 * For callers that cannot allocate device memory (code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc): symb_base_linear_fwd with its workspace inside the
 * library, in a file-scope device array of SYMB_STATIC_SCRATCH_BYTES that every GPU the library
 * runs on holds until the process ends.  Same arguments otherwise, same kernels, same results as
 * symb_base_linear_fwd given a workspace of that size.  The call allocates nothing and frees
 * nothing.  A batch whose mandatory workspace (symb_workspace_bytes minus the optional region of
 * K-split partial tiles) exceeds the array fails with SYMB_ERR_WORKSPACE_TOO_SMALL before anything
 * is enqueued.  All calls on one GPU share that GPU's array: calls that overlap in time on one GPU
 * (different streams, different handles) race; keep them on one stream.  Nothing in the array has
 * to start at zero (every region is written before it is read within the call).
 */
enum { SYMB_STATIC_SCRATCH_BYTES = 32 << 20 };
symb_status symb_base_linear_fwd_static(symb_handle h, const symb_batch* b, const void* X, const void* W,
                                        const void* bias, void* Y, void* Ybase, void* stream);

/*
 * Measurement switches (not part of the method), per handle, all on by default; value 0 turns one
 * off.  symb_workspace_bytes does not depend on them.
 *   SYMB_OPT_DESCRIPTOR_REUSE    a call whose descriptor bytes are already on the device reads them in
 *                                place (off: every call sends them, as a job whose batch layout
 *                                changes from call to call does)
 *   SYMB_OPT_K_SPLIT             output tiles computed by several workgroups, one per K range
 *   SYMB_OPT_SMALL_BATCH_KERNELS the weight-streaming kernels for calls of at most 16 rows
 *   SYMB_OPT_SKINNY_DEEP         the deep-prefetch build of the LoRA shrink for launches of few workgroups
 */
typedef enum { SYMB_OPT_DESCRIPTOR_REUSE = 0, SYMB_OPT_K_SPLIT = 1, SYMB_OPT_SMALL_BATCH_KERNELS = 2,
               SYMB_OPT_SKINNY_DEEP = 3 } symb_debug_option;
symb_status symb_debug_set_option(symb_handle h, int32_t option, int32_t value);

/* The K-split keeps all workgroups of one output tile on one XCD (behind one L2), which relies on
 * the dispatcher sending workgroup number g to XCD g mod 8.  symb_create measures that (a probe
 * launch records the hardware XCD id of 2048 workgroups); *holds is 1 if every workgroup of a residue
 * class mod 8 ran on the same XCD, and only then is the K-split ever used on this handle.
 * xcc_of_residue (8 entries, may be NULL) receives the XCD id seen for residues 0..7. */
symb_status symb_debug_xcd_rule(symb_handle h, int32_t* holds, int32_t* xcc_of_residue);

/* Test aid: how many calls on this handle so far sent their descriptors to the device
 * (`sent`) and how many found them already there (`in_place`); see symb_create. */
symb_status symb_debug_descriptor_stats(symb_handle h, int64_t* sent, int64_t* in_place);

const char* symb_status_string(symb_status s);
/* Text of the last error on this handle (h == NULL: of handle-free calls on this thread). */
const char* symb_last_error(symb_handle h);

#ifdef __cplusplus
}
#endif
#endif /* SYMB_H */
