/*
 * compactfusion.h -- C ABI of the MI355X (gfx950) residual codec.
 *
 * The codec is the per-layer, per-step hot path of CompactFusion
 * (arxiv 2507.17511).  For every activation tensor X_t in R^{N x C} of a
 * diffusion step it
 *   a1  forms the residual against the stored reconstruction,
 *         r = x_t - recon_{t-1}                               (Sec. 3.1; App. H, residual recursion)
 *   a2  applies error feedback (see cf_ef_mode)               (Sec. 3.2; App. D "Residual Base and Error Feedback")
 *   a3  reduces the scales of z                               (App. D "Quantization": v_j = mean_i |z_ij|)
 *   a4  selects low-bit codes, a5 packs them                  (App. D: +-1; {-2,-0.5,+0.5,+2})
 *   a6  decodes them, D = level(code) * scale                 (App. D: Q(X) = q(X) (.) scale)
 *   a7  updates the sender's error buffer, e_t = z - D        (Sec. 3.2)
 *   a8  updates the reconstruction, recon_t = recon_{t-1} + D (App. H: a~_t = a~_{t-1} + C(Delta a*_t))
 * and a warm-up call seeds the state with an uncompressed step, recon_0 = x_0,
 * e_0 = 0 (App. D "Warmup Implementation"; App. H.2).
 *
 * Memory and streams.  Every tensor pointer is a DEVICE pointer owned by the
 * caller; the pointer *arrays* are HOST arrays of `count` device pointers.  The
 * library allocates and frees no device memory: its scratch lives in the
 * caller's workspace (cf_workspace_bytes), which it may overwrite on every
 * call.  `stream` is a hipStream_t passed as void* (NULL = the null stream).
 * All calls enqueue work on it and return without synchronising; buffers must
 * stay valid until the stream has passed that work.  A context is not
 * thread-safe: use it from one host thread at a time, on one stream at a time.
 *
 * Layouts (all dense, row-major, C contiguous; base pointers 16-byte aligned):
 *   x, recon : [N, C] of `dtype`
 *   err      : [N, C] of `err_dtype`
 *   codes    : [N, C*bits/8] bytes; byte k of a row holds channels
 *              (8/bits)*k ... (8/bits)*k + 8/bits - 1, channel (8/bits)*k + m in
 *              bits [bits*m, bits*m + bits)  (least significant first)
 *   scales   : fp32 [C] (CF_SCALE_CHANNEL), fp32 [N, C/group] (CF_SCALE_GROUP),
 *              fp32 v[C] followed by u[N] (CF_SCALE_RANK1); none (CF_SPARSE_NM: the
 *              entry is ignored and may be null)
 *   codes with CF_LOWRANK: U [N, 32] then V [C, 32], both in `dtype`
 *   codes with CF_SPARSE_NM: [N, C/8] mask bytes (bit m of byte k = channel 8k+m
 *              kept), then, from the next multiple of 16 bytes on (the bytes in
 *              between are never written), the kept values in
 *              `dtype`, token-major, `bits` per block of `group` channels in channel order
 * x must not alias recon or err; codes and scales must alias nothing.
 *
 * Codes.  1-bit: bit = 1 for z < 0.  2-bit: bit1 = sign, bit0 = magnitude
 * (0 -> 0.5, 1 -> 2), magnitude bit set iff |z| > 1.25*scale.  4-bit (this
 * library's extension; the paper defines no 4-bit activation code): q =
 * round-half-even(z / scale) clamped to [-7, 7] as a two's-complement nibble,
 * scale = max|z| / 7 over the column or the group.  All value arithmetic is
 * IEEE fp32, one rounding per operation; channel sums use a balanced binary
 * tree over the token index (padded with zeros to a power of two), so results
 * do not depend on the launch shape.  NaN or Inf inputs give undefined values
 * (never a fault).
 *
 * x, recon, err, codes and scales of one tensor must not overlap one another
 * (checked on byte ranges; buffers of different tensors are the caller's business).
 *
 * Errors.  Every entry point returns a cf_status; nothing is thrown.  Arguments,
 * shapes, state and workspace are validated before anything is enqueued: on
 * every status but CF_ERR_DEVICE no work was enqueued and no state changed.
 * CF_ERR_DEVICE means a HIP call failed part of the way through a call's launch
 * sequence: kernels enqueued before it still run, so the tensors of that call
 * hold undefined values and must be warmed up again.
 *
 * Streams and graphs.  The device pointers of a call reach the kernels through a
 * table in the workspace that a small kernel of the same call fills; the library
 * skips that upload when the pointers are the ones it uploaded last on the same
 * stream.  A call on another stream than the last one, or on a stream that is
 * being captured into a HIP graph, uploads the whole table again, and after a
 * captured call the next call does too: a captured call is self-contained and may
 * be replayed at any time, as long as no other use of the context is in flight.
 */
#ifndef COMPACTFUSION_H
#define COMPACTFUSION_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct cf_ctx cf_ctx; /* opaque; host memory owned by the library */

typedef enum {
    CF_OK = 0,
    CF_ERR_INVALID_ARG = 1, /* null pointer, bad range, misaligned tensor pointer */
    CF_ERR_SHAPE = 2,       /* N < 1, C < 8, C % 8 != 0, C % group != 0, group != 128 */
    CF_ERR_UNSUPPORTED = 3, /* (bits, scale) pair, dtype or option outside the supported set */
    CF_ERR_STATE = 4,       /* codec step on a tensor that was never warmed up */
    CF_ERR_WORKSPACE = 5,   /* workspace null, too small or not 256-byte aligned */
    CF_ERR_DEVICE = 6       /* a HIP call failed; see cf_last_hip_error */
} cf_status;

typedef enum { CF_F32 = 0, CF_BF16 = 1 } cf_dtype;

/* What a scale spans.  CHANNEL: all N tokens of one channel (the paper's v_j
 * with u = 1).  GROUP: `group` consecutive channels of one token (4-bit only).
 * RANK1: the paper's u v^T (App. D "Quantization"), s_ij = u_i * v_j with v_j as
 * for CHANNEL and u_i = rowmean_i|z| / mean|z| (0 when z is all zero); 1-/2-bit
 * only, C <= 131072 (CF_ERR_SHAPE beyond), two-kernel path only (the
 * single-pass flag is ignored for a context that holds such a tensor).
 *
 * CF_SPARSE_NM is not a scale but the other compressor of the paper's kernel set
 * (Sec. 3.4, N:M block sparsifier): of every `group` = M in {8, 16} consecutive
 * channels (C a multiple of M) of a
 * token the `bits` = N in {1, 2, 4} of largest magnitude are kept and travel in
 * `dtype` (bf16 values rounded to nearest even), the rest are dropped into the
 * error.  Magnitudes are ordered by the bit pattern of |z| (NaN above infinity),
 * equal ones by channel, lowest first.  No scales, no reduction over tokens.
 *
 * CF_LOWRANK is the low-rank compressor (Alg. 3; App. D "Low-Rank Compression"): the
 * residual A [N, C] travels as rank-32 factors U = A Q [N, 32] and V = Q [C, 32] in
 * `dtype`, found by `bits` = T in {1, 2, 4} steps of subspace iteration
 *   Q <- orth(Q0);  T x { Z <- A^T (A Q); Q <- orth(Z) };  U <- A Q
 * (orth = Gram-Schmidt over the columns; a column left with less than 1e-4 of its
 * length is dropped to zero; U is not normalised, so U V^T is the projection of A
 * onto span(Q)).  D = U V^T is formed from the travelled (rounded) factors in fp32
 * on the matrix cores.  `group` = 32 (the rank); C a multiple of 32, at most 3072;
 * CF_EF_RECON only.  The `scales` entry of such a tensor is an INPUT of the sender:
 * the start matrix Q0 [C, 32] fp32 that the caller draws; the receiver ignores it
 * (it must still be a valid pointer).  Results agree with an fp64 evaluation to
 * fp32 rounding, not bit for bit. */
typedef enum { CF_SCALE_CHANNEL = 0, CF_SCALE_GROUP = 1, CF_SCALE_RANK1 = 2, CF_SPARSE_NM = 3, CF_LOWRANK = 4 } cf_scale_kind;

/* How the error buffer enters (a2) and is updated (a7).
 *   CF_EF_RECON   z = x_t - recon_{t-1}; e_t = z - D.  The residual against the
 *                 reconstruction already carries last step's error, so e is
 *                 written every step and never read; recon_t + e_t = x_t.
 *   CF_EF_LITERAL z = (x_t - recon_{t-1}) + e_{t-1}; e_t = z - D.
 *   CF_EF_OFF     z = (x_t - recon_{t-1}) - e_{t-1} (the true residual
 *                 x_t - x_{t-1}: the paper's no-feedback ablation);
 *                 e_t = e_{t-1} + (z - D).
 *   CF_EF_NAIVE   z = x_t: the activation itself is compressed (Sec. 3.1, the
 *                 baseline residual compression is compared with); recon_t = D,
 *                 e_t = z - D = x_t - recon_t; neither recon nor e is read. */
typedef enum { CF_EF_RECON = 0, CF_EF_LITERAL = 1, CF_EF_OFF = 2, CF_EF_NAIVE = 3 } cf_ef_mode;

typedef struct {
    int64_t n_tokens;   /* N >= 1 */
    int64_t n_channels; /* C >= 8, multiple of 8 (and of group for CF_SCALE_GROUP) */
    int32_t dtype;      /* cf_dtype of x and recon */
    int32_t bits;       /* 1, 2 or 4 (CF_SPARSE_NM: values kept per block; CF_LOWRANK: subspace iterations) */
    int32_t scale;      /* cf_scale_kind; supported (bits, scale): (1|2|4, CHANNEL), (4, GROUP), (1|2, RANK1),
                           (1|2|4, SPARSE_NM), (1|2|4, LOWRANK) */
    int32_t group;      /* 128 when scale == CF_SCALE_GROUP, 8 or 16 when CF_SPARSE_NM, 32 when CF_LOWRANK, ignored otherwise */
} cf_tensor_desc;

typedef struct {
    int32_t ef;        /* cf_ef_mode */
    int32_t err_dtype; /* cf_dtype of every error buffer; CF_F32 by default */
    uint32_t flags;    /* CF_FLAG_* */
    /* The two fields below are for TESTING ONLY (leave them 0): they force launch shapes the library
       otherwise picks by itself, so that tests can show that no result depends on them. */
    int32_t tile_rows;   /* rows per workgroup tile of the two-kernel path's scale reduction: 8, 16, 32 or 64 */
    int32_t encode_rows; /* rows per workgroup of the receiver's kernel (cf_decompress): 1..64 */
} cf_options;

/* A channel scale needs every token of a channel before any code of that
 * channel.  The single-pass kernel keeps the operands of a 256-row x 128-channel
 * item in registers across that reduction, so that x, recon (and err, where it is
 * an operand) are read once; the workgroups of one 128-channel stripe of a tensor
 * publish their partial sums to each other through the workspace.  It covers every
 * CF_SCALE_CHANNEL tensor of a context without CF_SCALE_RANK1 tensors, in every
 * error-feedback mode.  Otherwise one kernel reduces and a second one, which
 * reads the operands again, writes the codes.  Results are bit-identical either
 * way.  By default a call takes the single pass where it applies, every
 * channel-scale tensor of the context has at least 256 tokens and at most 48
 * items per stripe (12288 tokens of bf16 in the default feedback mode) and the
 * call covers at least 64 items: it is about 30 % faster on MI355X at the sizes
 * of the paper's models, slower on tiny batches, and slower than two kernels
 * where 64 and more workgroups have to agree on a scale (16384 tokens and up).
 * CF_FLAG_SINGLE_PASS takes it whenever it applies, CF_FLAG_TWO_KERNEL never.
 *
 * Waiting in the single pass.  A workgroup normally finds the partial sums of its
 * stripe within microseconds, because the workgroups of a stripe are launched
 * next to each other.  It does not depend on that: a workgroup that has waited
 * for a partial sum for some milliseconds gives its item up (it has written
 * nothing but its own partial sum by then), and a second launch of the same
 * kernel, which is part of every call and normally finds nothing to do, does the
 * given-up items once all partial sums are there.  So the call finishes, with the
 * same bits, whatever else runs on the device and in whatever order workgroups
 * are started; it needs no co-residency and no cooperative launch.
 * cf_given_up_items tells how many items of the last call went that way.
 * CF_FLAG_FIXED_GRID launches as many workgroups as fit the device at once and
 * lets them loop over the items, for callers who want the codec to hold a fixed
 * number of workgroup slots next to other kernels (about 15 % slower when it has
 * the device to itself). */
#define CF_FLAG_SINGLE_PASS 0x1u
#define CF_FLAG_TWO_KERNEL 0x2u
#define CF_FLAG_FIXED_GRID 0x8u
/* TESTING ONLY: workgroups of the single pass do not wait at all: an item whose stripe's partial
 * sums are not all there at the first look is given up and done by the second launch.  Slow;
 * results unchanged. */
#define CF_FLAG_TEST_NO_WAIT 0x100u
/* CF_LOWRANK tensors of the context send their factors as 4-bit integers (Sec. 3.4 and App. D name INT4
 * factors without a format; this one is the library's): every factor row of 32 entries has one fp32 scale
 * s = absmax / 7 and travels as nibbles q = clamp(round-half-even(f / s), -7, 7), two's complement, entry k
 * in byte k / 2 with even k in the low nibble; D is formed from q * s.  The codes buffer then holds
 * U nibbles [N, 16 bytes], V nibbles [C, 16 bytes], U scales [N] fp32, V scales [C] fp32: (N + C) * 20 bytes. */
#define CF_FLAG_LOWRANK_INT4 0x4u

/* Byte sizes of one tensor's buffers.  Any output pointer may be NULL.
 * CF_ERR_SHAPE / CF_ERR_UNSUPPORTED as for cf_init. */
cf_status cf_sizes(const cf_tensor_desc *desc, const cf_options *opts, size_t *codes_bytes,
                   size_t *scales_bytes, size_t *recon_bytes, size_t *err_bytes);

/* Bytes of workspace cf_init needs for these tensors (0 if they are invalid). */
size_t cf_workspace_bytes(const cf_tensor_desc *descs, int32_t n_tensors, const cf_options *opts);

/* Create a context for `n_tensors` layer tensors (App. H.2: state is kept per
 * layer tensor).  Validates every descriptor, lays the workspace out and
 * uploads the descriptor table to it on `stream`.  `opts` may be NULL
 * (CF_EF_RECON, fp32 error).  The workspace must be device memory, 256-byte
 * aligned, at least cf_workspace_bytes() long, and outlive the context.
 * Uses the device that is current at the call. */
cf_status cf_init(cf_ctx **out, const cf_tensor_desc *descs, int32_t n_tensors, const cf_options *opts,
                  void *workspace, size_t workspace_bytes, void *stream);

/* a0, warm-up of tensors [first, first+count): recon <- x0, err <- 0; the step
 * counts as sent uncompressed (App. D "Warmup Implementation", option 1). */
cf_status cf_warmup(cf_ctx *ctx, int32_t first, int32_t count, const void *const *x0,
                    void *const *recon, void *const *err, void *stream);

/* Declare tensors warm (or not) without touching memory: resuming from state
 * buffers the caller restored, or a receiver whose base arrived elsewhere. */
cf_status cf_set_warm(cf_ctx *ctx, int32_t first, int32_t count, int32_t warm);

/* Sender half (a1-a7): reads x and recon, reads/writes err, writes codes and
 * scales.  recon is not modified. */
cf_status cf_compress(cf_ctx *ctx, int32_t first, int32_t count, const void *const *x,
                      const void *const *recon, void *const *err, void *const *codes,
                      void *const *scales, void *stream);

/* Receiver half (a6, a8): reads codes and scales, updates recon in place. */
cf_status cf_decompress(cf_ctx *ctx, int32_t first, int32_t count, const void *const *codes,
                        const void *const *scales, void *const *recon, void *stream);

/* One whole codec step (a1-a8) for tensors [first, first+count) in one batched
 * launch: bit-identical, in every output, to cf_compress followed by
 * cf_decompress on the same buffers. */
cf_status cf_step_fused(cf_ctx *ctx, int32_t first, int32_t count, const void *const *x,
                        void *const *recon, void *const *err, void *const *codes,
                        void *const *scales, void *stream);

/* For callers that cannot allocate device memory (code that runs under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc): one whole codec
 * step, as cf_step_fused over all `n_tensors` tensors, with NO context and NO
 * workspace argument.  Its scratch is a device array inside the library
 * (CF_STATIC_SCRATCH_BYTES per GPU, held until the process ends); the call
 * allocates nothing, on the device or through any library.  The tensors must need
 * no more workspace than that (compare cf_workspace_bytes): otherwise
 * CF_ERR_WORKSPACE, nothing enqueued.  There is no warm-up call for it: the caller
 * vouches that recon and err hold valid state (recon = x_0, err = 0 after the
 * uncompressed step).  Outputs are bit-identical to cf_step_fused on the same
 * buffers.  All calls on one GPU share that GPU's array: calls that overlap in
 * time on one GPU race, whatever their streams; calls in stream order are fine,
 * with any mix of shapes (the tables are laid out again when the tensors or the
 * options change).  Uses the device that is current at the call; not thread-safe.
 * The bounded waits of the single-pass kernel apply as for cf_step_fused, but
 * there is no context to ask about them: pass CF_FLAG_TWO_KERNEL for a launch
 * sequence without any wait between workgroups. */
#define CF_STATIC_SCRATCH_BYTES ((size_t)16 << 20)
cf_status cf_step_fused_static(const cf_tensor_desc *descs, int32_t n_tensors, const cf_options *opts,
                               const void *const *x, void *const *recon, void *const *err,
                               void *const *codes, void *const *scales, void *stream);

/* Frees the host-side context (never device memory).  NULL is allowed. */
void cf_destroy(cf_ctx *ctx);

const char *cf_status_string(cf_status s);

/* The hipError_t value of the last failed HIP call in this context (0 if none). */
int32_t cf_last_hip_error(const cf_ctx *ctx);

/* Synchronises `stream`; CF_ERR_DEVICE with cf_last_hip_error() != 0 if that fails (a kernel
 * enqueued before it faulted), CF_ERR_DEVICE with cf_last_hip_error() == 0 if the library's own
 * consistency check on the device tripped (the second launch of a single pass found a partial sum
 * missing, which the design rules out); the context is then unusable. */
cf_status cf_check_device(cf_ctx *ctx, void *stream);

/* Synchronises `stream` and reports in *count how many items of the LAST single pass were given
 * up by their first workgroup and done by the second launch (see "Waiting in the single pass";
 * 0 in ordinary operation). */
cf_status cf_given_up_items(cf_ctx *ctx, void *stream, uint32_t *count);

/* Instrumentation for benchmarks (no part of the method).  With `events` set
 * (a host array of 2*n_pairs hipEvent_t created by the caller), the NEXT
 * cf_compress / cf_decompress / cf_step_fused call records events[2k] before
 * and events[2k+1] after its k-th kernel launch on the call's stream, for as
 * many launches as there are pairs, then switches itself off again.  The
 * launches of a call are, in order: pointer-table uploads (only when a pointer
 * changed), then the codec kernels named by cf_profile_kernel_name.  NULL/0
 * switches it off. */
cf_status cf_profile_next_call(cf_ctx *ctx, void *const *events, int32_t n_pairs);

/* After a profiled call: how many launches it made, and the name of the k-th
 * (a static string; NULL if k is out of range). */
int32_t cf_profile_launch_count(const cf_ctx *ctx);
const char *cf_profile_kernel_name(const cf_ctx *ctx, int32_t k);

#ifdef __cplusplus
}
#endif
#endif
