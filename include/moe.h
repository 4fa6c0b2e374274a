/*
 * moe.h - C ABI of the MI355X (gfx950) MoE-layer forward library.
 *
 * One Mixture-of-Experts layer, forward only, as defined in the paper's Sec. 2.1:
 *   Eq. 1   s = softmax(W_r x)
 *   Eq. 2   T = top-k(s) = {(e_i, w_i)}
 *   Eq. 3   y = sum_i w_i * FFN_{e_i}(x)
 *   Eq. 4   FFN_e(x) = (SiLU(x W_gate_e) (.) x W_up_e) W_down_e
 * executed as the five stages of Sec. 3.1: route, permute into expert-contiguous
 * order (Sec. 3.5), fused gate+up grouped GEMM (Sec. 3.2-3.3), down grouped GEMM,
 * weighted un-permute / combine (Sec. 3.5, Eq. 3).
 *
 * Conventions common to every entry point
 *   - Every data pointer is a DEVICE pointer owned by the caller.  The library never
 *     allocates, frees or keeps a pointer beyond the work it enqueues.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls only
 *     enqueue kernels; they never synchronise.  The caller keeps all buffers alive until
 *     the stream has drained.  No host<->device copy happens anywhere.
 *   - bf16 tensors are uint16 bit patterns, row-major, base pointer 16-byte aligned.
 *   - Stored weight matrices are [out, in] with the reduction dimension contiguous
 *     (Sec. 3.2's "E*N x K" flattened layout): W_r [E,d], W_gate,W_up [E,F,d], W_down [E,d,F].
 *     Eq. 4's "x W" is therefore x times the transpose of the stored matrix.
 *   - Notation: T tokens, d model dim, F expert FFN dim, E experts, k experts per token,
 *     R = T*k expanded rows, n_e rows routed to expert e.
 *   - Limits: 1 <= k <= E <= 256, d % 64 == 0, F % 64 == 0, T >= 0, T*k <= 2^30, and the
 *     activation buffers (x, x_perm, h: T*k*max(d,F) elements of 2 bytes) below 4 GiB: the GEMM
 *     kernels address their rows with 32-bit byte offsets.  Beyond: MOE_ERR_UNSUPPORTED.
 *     T == 0 returns MOE_OK and enqueues nothing.
 *   - Stream capture: the calls record kernel launches only and may be captured into a HIP
 *     graph; replays equal the eager result.  The first use of a GEMM kernel in a process sets
 *     a function attribute (its LDS size), which HIP does not allow during capture: run the
 *     call once eagerly with the same configuration before capturing it.
 *   - All argument checks run on the host before anything is enqueued: a call that returns
 *     an error has had no effect on device memory.  Errors are return codes only.
 */
#ifndef MOE_H_
#define MOE_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    MOE_OK = 0,
    MOE_ERR_NULL = -1,        /* a required pointer is NULL */
    MOE_ERR_SHAPE = -2,       /* T<0, k<1, k>E, E<1, d<1, F<1, unknown gating */
    MOE_ERR_ALIGN = -3,       /* a tensor base pointer is not 16-byte aligned */
    MOE_ERR_WORKSPACE = -4,   /* workspace smaller than the matching *_workspace_size() */
    MOE_ERR_UNSUPPORTED = -5, /* E > 256, d % 64 != 0, F % 64 != 0, T*k > 2^30, or T*k*max(d,F)*2 bytes >= 4 GiB */
    MOE_ERR_HIP = -6          /* a kernel launch reported a HIP error */
} moe_status;

typedef enum {
    MOE_GATE_SOFTMAX = 0,        /* w_i = softmax(z)[e_i]                      (Eq. 1-2) */
    MOE_GATE_SOFTMAX_RENORM = 1, /* w_i = softmax(z)[e_i] / sum_j softmax(z)[e_j]        */
    MOE_GATE_SIGMOID_NORM = 2    /* w_i = sigmoid(z_{e_i}) / sum_j sigmoid(z_{e_j})  (Sec. 3.4) */
} moe_gating;

/* moe_config.flags */
/* moe_forward folds the weighted combine (Eq. 3) into the down projection instead of launching
 * it as a fifth kernel (the paper's limitation 1): the workgroup that writes the last of a token's
 * k expert rows sums them, in slot order, from the bf16 rows in memory, so y is bit-identical to
 * moe_combine's whichever workgroup arrives last.  One launch fewer per layer; the GEMM
 * workgroups pay for it with latency-bound reads at their end, which costs more than the launch
 * it saves once T*k exceeds a few hundred rows (measured), so it is off unless asked for.
 * Needs packed weights and more than a handful of rows (the kernels that serve row-major weights
 * and the K-split kernel have no such epilogue): otherwise the flag is ignored. */
#define MOE_FLAG_FUSE_COMBINE 1

typedef struct {
    int32_t T, d, F, E, k;
    int32_t gating;       /* moe_gating */
    int32_t tile_m;       /* rows per block-schedule tile (Alg. 1's M); 0 = chosen from T*k/E */
    int32_t flags;        /* bit set of MOE_FLAG_*; unknown bits are refused (MOE_ERR_SHAPE) */
} moe_config;

/* Byte offsets of moe_forward's intermediates inside its workspace (all 256-byte aligned). */
typedef struct {
    size_t topk_idx;  /* int32 [T,k] */
    size_t topk_w;    /* float [T,k] */
    size_t counts;    /* int32 [E]   */
    size_t offsets;   /* int32 [E+1] */
    size_t row_of;    /* int32 [R]   */
    size_t src_of;    /* int32 [R]   */
    size_t x_perm;    /* zero-length: moe_forward reads x rows through src_of and writes no permuted copy */
    size_t h;         /* bf16  [R,F] */
    size_t y_perm;    /* bf16  [R,d] */
    size_t scratch;   /* internal: partial logit tiles, chunk histograms, block schedule */
    size_t total;     /* bytes needed */
} moe_workspace_layout;

const char* moe_status_string(moe_status s);

/* Tile height (Alg. 1's M) the library uses for this config: cfg->tile_m if non-zero
 * (must be 32, 64, 96, 128, 160, 192 or 256), else 256 (the GEMM kernels adapt to the rows each
 * block really holds), 128 for many experts of a few rows each at up to 128 tokens (kernels built
 * for two workgroups per CU), or 32 when there are so few rows in all that the down projection
 * is run by the K-split kernel.
 * Returns 0 for an invalid config. */
int32_t moe_tile_m(const moe_config* cfg);

/* Workspace sizes in bytes (0 for an invalid config).  Host only, no GPU needed. */
size_t moe_route_workspace_size(const moe_config* cfg);
size_t moe_permute_workspace_size(const moe_config* cfg);
size_t moe_ffn_workspace_size(const moe_config* cfg);
size_t moe_forward_workspace_size(const moe_config* cfg);
/* The workspace moe_forward needs: the same value as moe_forward_workspace_size(). */
size_t moe_workspace_size(const moe_config* cfg);
/* Fills *out with the layout moe_forward uses; returns MOE_OK or the config error. */
moe_status moe_forward_workspace_layout(const moe_config* cfg, moe_workspace_layout* out);
/* Name of the GEMM kernel instance the library launches for this config (stage 0: fused
 * gate+up, 1: down; packed != 0: with moe_pack_weights' layout), e.g. for matching profiler
 * output.  Returns a static string, NULL for an invalid config or stage. */
const char* moe_ffn_kernel_name(const moe_config* cfg, int32_t stage, int32_t packed);
/* Upper bound on Alg. 1's block count for tile height M: floor(R/M) + min(E, R); 0 for an
 * invalid config or M outside [1, 2^30]. */
int32_t moe_max_blocks(const moe_config* cfg, int32_t M);

/* Stage 1, router (Eq. 1-2, Sec. 3.4).
 *   x [T,d] bf16, W_r [E,d] bf16, bias [E] fp32 or NULL (added to the logits)
 *   -> topk_idx [T,k] int32, topk_w [T,k] fp32.
 * Logits z = W_r x + bias are accumulated in fp64 (exact products of the bf16 operands).  The
 * k experts are chosen by k rounds of arg-max over z with the winner masked; a tie goes to the
 * lower expert index; outputs are in selection order (descending score).  Weights follow
 * cfg->gating.  workspace: moe_route_workspace_size(cfg) bytes (partial logit tiles). */
moe_status moe_route(const moe_config* cfg, const void* x, const void* W_r, const float* bias,
                     int32_t* topk_idx, float* topk_w, void* workspace, size_t ws_bytes, void* stream);

/* Stage 2, permutation into expert-contiguous order (Sec. 2.2, Sec. 3.5).
 *   topk_idx [T,k] (any valid assignment: values in [0,E), as Sec. 4.7 injects them)
 *   -> counts [E] (n_e), offsets [E+1] (exclusive prefix sum, offsets[E] = R),
 *      row_of [R] (row of flat slot j = t*k+i after a STABLE sort by expert id),
 *      src_of [R] (inverse: slot stored at row r), x_perm [R,d] = x[src_of[r]/k, :].
 * x and x_perm may both be NULL to compute the index arrays only.
 * An index outside [0,E) cannot be reported (that would need a device->host sync); it is
 * clamped into [0,E-1], so every row index the kernels produce stays inside the buffers. */
moe_status moe_permute(const moe_config* cfg, const void* x, const int32_t* topk_idx,
                       int32_t* counts, int32_t* offsets, int32_t* row_of, int32_t* src_of,
                       void* x_perm, void* workspace, size_t ws_bytes, void* stream);

/* moe_permute for callers that cannot allocate device memory and have no workspace to hand in
 * (code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc): the same
 * kernels and the same results as moe_permute, with the chunk histograms (the only scratch the
 * stage needs: ceil(R/1024) * E int32) in a file-scope device array of the library instead of a
 * workspace argument.  The array holds MOE_PERMUTE_STATIC_MAX_INTS int32 (256 KiB) on every GPU
 * the library is used on, for the life of the process.  A configuration with
 * ceil(T*k/1024) * E above that returns MOE_ERR_UNSUPPORTED.  The call allocates nothing and frees
 * nothing.  Nothing in the array has to start at zero (every entry that is read has been written
 * earlier in the same call), so it is never cleared; its contents after a call are unspecified.
 * All calls on one GPU share the one array: two calls whose kernels overlap on the same GPU
 * (different streams, or different host threads on different streams) race and give wrong
 * results; calls on one stream are ordered and safe. */
#define MOE_PERMUTE_STATIC_MAX_INTS 65536
moe_status moe_permute_static(const moe_config* cfg, const void* x, const int32_t* topk_idx,
                              int32_t* counts, int32_t* offsets, int32_t* row_of, int32_t* src_of,
                              void* x_perm, void* stream);

/* Alg. 1 on the device: blocks [max_blocks,2] int32 = (expert, b*M) in emission order,
 * *num_blocks (device int32) = sum_e ceil(n_e/M).  Entries past *num_blocks are untouched.
 * `blocks` must hold moe_max_blocks(cfg, M) pairs.  1 <= M <= 2^30, else MOE_ERR_SHAPE. */
moe_status moe_block_schedule(const moe_config* cfg, const int32_t* offsets, int32_t M,
                              int32_t* blocks, int32_t* num_blocks, void* stream);

/* One-time weight packing (the weights of an inference layer are static).  THE PACKED COPY IS
 * THE SERVING LAYOUT: the GEMM kernels are built around it, and a caller that serves traffic
 * should pack once at load time and pass W_packed from then on.  The row-major tensors of
 * Sec. 3.2 are accepted by every entry point as the interchange layout (same integers, floats
 * within the stated tolerance) and run through a slower kernel (about 1.4x at the Mixtral shape).
 * Sec. 3.2 stores each projection as a flattened E*N x K matrix; the GEMM kernels read it
 * through per-lane 16-byte loads whose lanes touch 32 different rows.  moe_pack_weights
 * re-orders the same bf16 values into the order those loads consume them, so that every load
 * instruction reads 1 KiB contiguous and a wavefront streams one contiguous region:
 *   unit = 16 bytes; order [expert][row block of 32][k step of 64][matrix][slot 0..3][lane 0..63];
 *   unit (rb, kt, m, s, lane) = W_m[expert][32 rb + lane%32][64 kt + 16 s + 8 (lane/32) .. +8];
 *   gate and up are interleaved (m = 0, 1) in the first 4*E*F*d bytes, the down projection
 *   (m = 0 only) follows.
 * `packed` must hold moe_packed_weights_size(cfg) bytes (= 6*E*d*F, the size of the three
 * weight tensors), 256-byte aligned.  A packed buffer depends on d, F and E only, not on T, k. */
size_t moe_packed_weights_size(const moe_config* cfg);
moe_status moe_pack_weights(const moe_config* cfg, const void* W_gate, const void* W_up, const void* W_down,
                            void* packed, void* stream);

/* Stages 3+4, expert FFN as two block-scheduled grouped GEMMs (Sec. 3.2, 3.3, Eq. 4).
 *   x_perm [R,d] bf16 expert-contiguous, offsets [E+1]
 *   W_gate, W_up [E,F,d] bf16, W_down [E,d,F] bf16
 *   W_packed: NULL, or moe_pack_weights' output for these weights; when it is given the kernels
 *             read only the packed copy and W_gate, W_up, W_down may be NULL
 *   -> h [R,F] bf16 = SiLU(x W_gate^T) (.) (x W_up^T)  (fp32 accumulate, SiLU and product in
 *      fp32 registers, one rounding to bf16), y_perm [R,d] bf16 = h W_down^T (fp32 accumulate).
 * The block schedule is built on the device from `offsets`; no host synchronisation. */
moe_status moe_grouped_ffn(const moe_config* cfg, const void* x_perm, const int32_t* offsets,
                           const void* W_gate, const void* W_up, const void* W_down, const void* W_packed,
                           void* h, void* y_perm, void* workspace, size_t ws_bytes, void* stream);

/* Stage 5, un-permute + weighted combine (Eq. 3, Sec. 3.5).
 *   y[t,:] = sum_{i<k} topk_w[t,i] * y_perm[row_of[t*k+i], :], fp32 accumulation in slot
 *   order, one rounding to bf16.  No atomics: results are bit-reproducible. */
moe_status moe_combine(const moe_config* cfg, const void* y_perm, const int32_t* row_of,
                       const float* topk_w, void* y, void* stream);

/* The whole layer: stages 1-5 enqueued back to back on `stream`, intermediates in
 * `workspace` at moe_forward_workspace_layout()'s offsets.  y [T,d] bf16.  W_packed as above.
 * The permutation stage builds the index arrays only: the gate+up GEMM fetches expert-contiguous
 * row r straight from x[src_of[r] / k] while it loads its token tile, so the permuted copy of x
 * (Sec. 3.1 step 2; the paper lists removing it as future work) is never written.  Results are
 * identical to moe_permute + moe_grouped_ffn on the materialised copy. */
moe_status moe_forward(const moe_config* cfg, const void* x, const void* W_r, const float* bias,
                       const void* W_gate, const void* W_up, const void* W_down, const void* W_packed,
                       void* y, void* workspace, size_t ws_bytes, void* stream);

/* moe_forward with timing hooks: `events` is an array of n_events hipEvent_t handles (as void*,
 * entries may be NULL, the array itself may be NULL when n_events == 0) recorded on `stream`
 *   [0] before the router, [1] after it, [2] after the permutation (index arrays; the row gather runs inside gate+up),
 *   [3] after the fused gate+up GEMM, [4] after the down GEMM, [5] after the combine.
 * Entries beyond index 5 are ignored.  Everything else is exactly moe_forward (Sec. 3.1's
 * five stages; the per-stage breakdown mirrors the paper's Table 6). */
#define MOE_NUM_STAGE_EVENTS 6
moe_status moe_forward_staged(const moe_config* cfg, const void* x, const void* W_r, const float* bias,
                              const void* W_gate, const void* W_up, const void* W_down, const void* W_packed,
                              void* y, void* workspace, size_t ws_bytes, void* stream,
                              void* const* events, int32_t n_events);

#ifdef __cplusplus
}
#endif
#endif /* MOE_H_ */
