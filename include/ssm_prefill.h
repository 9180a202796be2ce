/*
 * ssm_prefill.h -- C ABI of the MI355X (gfx950) SSM-layer prefill library.
 *
 * One call scans a packed batch of variable-length requests through one
 * Mamba2-style SSM layer.  Each request may start from a cached recurrent
 * state (a prefix-cache hit) and may ask for the full fp32 state after any
 * of its tokens (the checkpoints that become cache entries).
 *
 * Per head h, channel p, state index n and sequence-local token t = 1..len:
 *
 *     a_t      = exp(dt[t,h] * A[h])
 *     S_t[p,n] = a_t * S_{t-1}[p,n] + dt[t,h] * x[t,h,p] * B[t,g(h),n]
 *     y[t,h,p] = sum_n C[t,g(h),n] * S_t[p,n] + D[h] * x[t,h,p]
 *
 * with g(h) = h / (nheads / ngroups) and S_0 the request's initial state.
 * (Paper Section 2.1 and Section 3: the state is a constant-size summary that
 * every token overwrites in place.  Section 2.2: on a cache hit the prefix
 * state is fetched before prefill.  Section 4.1, "Obtaining states during
 * prefill": states are materialised during a chunked prefill, optionally at
 * the exact token; a two-pass prefill resumes from the prefix state.)
 *
 * All tensors are row-major with the last index fastest.  "device" pointers
 * are HIP device pointers on the current device; "host" pointers are ordinary
 * process memory.  Every entry point returns SSM_OK (0) or a negative
 * ssm_status_t; on error nothing has been enqueued and ssm_last_error()
 * returns a message for the calling thread.  Nothing here throws or aborts.
 */
#ifndef SSM_PREFILL_H
#define SSM_PREFILL_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    SSM_OK = 0,
    SSM_ERR_INVALID_ARG = -1,       /* NULL where a pointer is required, bad sizes      */
    SSM_ERR_BAD_CU_SEQLENS = -2,    /* cu_seqlens[0] != 0 or decreasing                 */
    SSM_ERR_BAD_CHECKPOINT = -3,    /* position outside 1..len, duplicate or unsorted   */
    SSM_ERR_UNSUPPORTED_SHAPE = -4, /* shape outside what the kernels handle            */
    SSM_ERR_WORKSPACE_TOO_SMALL = -5,
    SSM_ERR_MISALIGNED = -6,        /* a device pointer is not 16-byte aligned          */
    SSM_ERR_HIP = -7                /* a HIP runtime call failed                        */
} ssm_status_t;

typedef enum { SSM_DT_F32 = 0, SSM_DT_BF16 = 1 } ssm_dtype_t; /* type of x, dt, B, C, y */

/* Storage type of cached states: the initial states a call reads and the checkpoints it writes.  The paper's cache
 * holds FP16 states (Section 5.1; Appendix A.1 counts 2 bytes per state element); fp32 keeps every bit of the
 * running state.  The running state inside a call is fp32 whatever the storage type; a reduced-precision
 * checkpoint is that fp32 state rounded once, to nearest even. */
typedef enum { SSM_ST_F32 = 0, SSM_ST_F16 = 1, SSM_ST_BF16 = 2 } ssm_state_dtype_t;

typedef struct {
    int32_t nheads;    /* H */
    int32_t headdim;   /* P */
    int32_t d_state;   /* N */
    int32_t ngroups;   /* G, divides H; heads of a group are contiguous */
    int32_t chunk;     /* Q: tokens per chunk of the chunked scan (Section 4.1); a tuning
                          knob that changes rounding order only, never which state is
                          returned.  16 <= Q <= 256, multiple of 16. */
    int32_t io_dtype;  /* ssm_dtype_t */
    int32_t state_dtype; /* ssm_state_dtype_t */
} ssm_shape_t;

typedef struct ssm_plan ssm_plan_t; /* opaque; owned by the library */

/* Which kernel family a plan selected (ssm_plan_info). */
enum { SSM_PATH_VALU_F32 = 0, SSM_PATH_MFMA_BF16 = 1 };

typedef struct {
    int32_t batch;
    int32_t n_ckpt;        /* total checkpoints = number of fp32 [H,P,N] slots in state_out */
    int64_t total_tokens;  /* T = cu_seqlens[batch] */
    int32_t n_tiles;       /* token tiles the kernels walk (sequence-local, split at checkpoints) */
    int32_t tile_tokens;   /* upper bound of a tile's length */
    int32_t path;          /* SSM_PATH_* */
    int32_t n_workgroups;  /* grid size of the scan kernel */
    int32_t n_stretches;   /* stretches the scan walks: one per sequence, more when long sequences are cut
                              (ssm_plan_stretch) */
} ssm_plan_info_t;

/*
 * Build the host-side plan for one packed batch: validate the request mix and
 * cut every sequence into tiles.  Tiles never cross a sequence boundary and
 * always end at each requested checkpoint position, so a checkpoint is the
 * scan's running state at a tile end (exact position, Section 4.1).  Host
 * only: touches no GPU.  A plan can be reused for every SSM layer of the
 * batch (24 layers in the paper's 7B hybrid, Section 5.1).
 *
 *   cu_seqlens_host [batch+1]  host; [0] == 0, non-decreasing; len 0 allowed
 *   cu_ckpt_host    [batch+1]  host; CSR offsets into ckpt_pos_host; may be
 *                              NULL when no checkpoint is requested at all
 *   ckpt_pos_host              host; per sequence strictly ascending token
 *                              COUNTS p, 1 <= p <= len: slot k receives the
 *                              state after exactly p tokens of its sequence
 *   out                        receives the plan; free with ssm_plan_destroy
 */
int ssm_plan_create(const ssm_shape_t *shape, int32_t batch,
                    const int32_t *cu_seqlens_host,
                    const int32_t *cu_ckpt_host,
                    const int32_t *ckpt_pos_host,
                    ssm_plan_t **out);

/* Copy the plan's summary into *info: what the planner of Section 4.1's chunked prefill decided for this batch
 * (how many tiles, which kernel family, how many checkpoint slots).  SSM_ERR_INVALID_ARG if either pointer is NULL. */
int ssm_plan_info(const ssm_plan_t *plan, ssm_plan_info_t *info);

/* Read tile i (0 <= i < n_tiles) of the plan: first packed token, length,
 * owning sequence, and the checkpoint slot filled at its end (-1: none).
 * This is the chunking of Section 4.1 made visible: a caller can check that
 * every requested position is a tile end.  Any output pointer may be NULL;
 * SSM_ERR_INVALID_ARG if the plan is NULL or i is out of range. */
int ssm_plan_tile(const ssm_plan_t *plan, int32_t i, int32_t *tok0, int32_t *len,
                  int32_t *seq, int32_t *ckpt_slot);

/* Launch order of the matrix-core scan, for inspection: how the planner spreads the chunked prefill of Section 4.1
 * over the GPU when the batch mixes long and short requests (the request mix of Section 5.1's traces).  Work items
 * are (rank of a non-empty sequence by decreasing tile count, head, channel slice), numbered by rank, then head, then
 * slice; the launch has n_blocks workgroups, dealt round-robin to the GPU's 8 dies, and ssm_plan_launch_item tells
 * which item a workgroup takes.
 *   by_length  [batch]  host, out, may be NULL; by_length[r] = index of the sequence of rank r (ties: lower index first)
 *   slices              out, may be NULL; channel slices per head (items per sequence = nheads * slices)
 *   n_items             out, may be NULL; non-empty sequences * nheads * slices
 *   n_blocks            out, may be NULL; workgroups of the launch (a multiple of 8, >= n_items)
 * SSM_ERR_INVALID_ARG if plan is NULL. */
int ssm_plan_launch_order(const ssm_plan_t *plan, int32_t *by_length, int32_t *slices, int32_t *n_items,
                          int64_t *n_blocks);

/* The work item (see ssm_plan_launch_order) of workgroup `block`, 0 <= block < n_blocks, or -1 if that workgroup has
 * none and leaves at once.  Every item belongs to exactly one workgroup.  SSM_ERR_INVALID_ARG if a pointer is NULL or
 * block is out of range. */
int ssm_plan_launch_item(const ssm_plan_t *plan, int64_t block, int32_t *item);

/* Stretch i (0 <= i < n_stretches) of the plan: the tiles [tile_begin, tile_end) that one workgroup per (head,
 * channel slice) scans in order.  Normally a stretch is a whole sequence.  When a batch has too few sequences to
 * occupy the GPU, a long sequence is cut into several stretches that are scanned at the same time, the later ones
 * from a zero state (starts_from_zero = 1); the state their predecessor ends with is then carried over, and what it
 * adds to their outputs and checkpoints (the recurrence of Section 2.1's state update is linear in the state) is added
 * by a second kernel of the same call.  Results are those of the plain scan up to rounding.  Any output pointer may
 * be NULL; SSM_ERR_INVALID_ARG if the plan is NULL or i is out of range. */
int ssm_plan_stretch(const ssm_plan_t *plan, int32_t i, int32_t *tile_begin, int32_t *tile_end,
                     int32_t *starts_from_zero);

/* Bytes of device workspace ssm_prefill needs for this plan (may be 0): the
 * per-(tile, group) operands that the heads of a group share in the chunked
 * scan of Section 4.1.  The caller allocates it, 256-byte aligned, owns it,
 * and may reuse it between calls that do not overlap; its contents mean
 * nothing between calls. */
int ssm_plan_workspace_bytes(const ssm_plan_t *plan, size_t *bytes);

/*
 * Enqueue the scan of one SSM layer on `hip_stream` (a hipStream_t, NULL =
 * the default stream): the chunked prefill of Section 4.1 with cached-state
 * resume (Section 2.2) and exact-position checkpoints.
 *
 * Synchronisation: the first call with a plan on a GPU makes three small
 * device allocations owned by the plan and waits once for the upload of the
 * plan's tables on `hip_stream`; every later call with that plan only
 * enqueues and never synchronises.  The plan itself is not modified (the
 * device tables are a cache behind it).  Calls that share a plan must be
 * ordered against each other (one stream, or events): they share the plan's
 * buffer of state pointers.
 *
 *   x      [T,H,P]  io_dtype  device  read only
 *   dt     [T,H]    io_dtype  device  read only; final step sizes, positive
 *                                     (no softplus, bias or clamp is applied)
 *   A      [H]      fp32      device  read only; negative decay rates
 *   B, C   [T,G,N]  io_dtype  device  read only
 *   D      [H]      fp32      device  read only; skip weight per head
 *   init_state_ptrs [batch]   HOST array of DEVICE pointers to [H,P,N] in the
 *                             plan's state_dtype; the array or any entry may
 *                             be NULL (zero state).  The states are read only:
 *                             they are live cache entries.  The array has been
 *                             copied when the call returns.
 *   y_out  [T,H,P]  io_dtype  device  written
 *   state_out [n_ckpt,H,P,N]  state_dtype, device, written; slot order =
 *                             sequence major, then ascending position (CSR
 *                             order); a slot may be passed back as an initial
 *                             state of a later call unchanged.  May be NULL if
 *                             n_ckpt is 0.
 *   workspace       device, >= ssm_plan_workspace_bytes, 256-byte aligned;
 *                   may be NULL if that is 0
 *
 * Device pointers must be 16-byte aligned.  T == 0 succeeds and enqueues
 * nothing.  Errors: SSM_ERR_INVALID_ARG (a required pointer is NULL),
 * SSM_ERR_MISALIGNED, SSM_ERR_WORKSPACE_TOO_SMALL, SSM_ERR_HIP.
 */
int ssm_prefill(const ssm_plan_t *plan,
                const void *x, const void *dt, const float *A,
                const void *B, const void *C, const float *D,
                const void *const *init_state_ptrs,
                void *y_out, void *state_out,
                void *workspace, size_t workspace_bytes,
                void *hip_stream);

/*
 * ssm_prefill for callers that cannot allocate device memory: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments, same results and same errors as ssm_prefill, but the plan's tile
 * and sequence tables and the initial-state pointers are written (by small
 * kernels on `hip_stream`) into a fixed device array that is part of the
 * library image instead of buffers allocated on a plan's first use.  The call
 * makes no hipMalloc, hipFree, memory copy or other allocating call, never
 * synchronises, and touches nothing of the plan.
 *
 * Limits: at most 16384 tiles (ssm_plan_info n_tiles) and 1024 sequences per
 * call, otherwise SSM_ERR_UNSUPPORTED_SHAPE and nothing is enqueued.  The
 * array (312 KiB per GPU the library runs on, held until the process ends) is
 * shared by every call on that GPU: calls that overlap on one GPU, on
 * different streams, race.  Calls on one stream are ordered by the stream.
 * Every call rewrites all it reads of the array, so nothing carries over from
 * one call to the next.
 */
int ssm_prefill_noalloc(const ssm_plan_t *plan,
                        const void *x, const void *dt, const float *A,
                        const void *B, const void *C, const float *D,
                        const void *const *init_state_ptrs,
                        void *y_out, void *state_out,
                        void *workspace, size_t workspace_bytes,
                        void *hip_stream);

/*
 * Roll cached states forward (Section 4.1, "Obtaining states during
 * prefill": a kernel that rolls a checkpointed state forward by a few tokens
 * to reach an exact position); with one token per sequence it is the decode
 * step.  Every sequence of the plan brings its own [H,P,N] state in the
 * plan's state_dtype, which is advanced IN PLACE by the sequence's tokens with
 * the token recurrence in fp32 and rounded once on the way back.
 *
 *   state_ptrs [batch]  HOST array of DEVICE pointers; a NULL entry leaves
 *                       that sequence alone (its y rows are not written)
 *   y_out      [T,H,P]  io_dtype, device, or NULL if y is not wanted
 *
 * Checkpoints of the plan are ignored.  d_state must be a power of two in
 * 4..256, else SSM_ERR_UNSUPPORTED_SHAPE.  Enqueues on hip_stream; first use
 * of a plan as for ssm_prefill.
 */
int ssm_state_advance(const ssm_plan_t *plan,
                      const void *x, const void *dt, const float *A,
                      const void *B, const void *C, const float *D,
                      void *const *state_ptrs, void *y_out, void *hip_stream);

/*
 * Causal depthwise convolution in front of the scan, with cached-state resume
 * and state checkpoints (the conv_1d state of Appendix A.1: in_channels x
 * conv_kernel values per layer).  For channel c, kernel width K =
 * kernel_width (1..4) and the sequence-local token t:
 *
 *     out[t,c] = act(bias[c] + sum_{j<K} weight[c,j] * z[t-K+1+j, c])
 *
 * where z continues the input to the left by the cached prefix's last inputs
 * (zeros without one); weight[c,K-1] multiplies the current token; activation
 * 0 is the identity, 1 is SiLU.
 *
 *   in, out    [T,channels]   io_dtype of the plan, device; two buffers that do
 *                             not overlap
 *   weight     [channels,K]   fp32, device;  bias [channels] fp32 or NULL
 *   init_state_ptrs           NULL, or HOST array [batch] of DEVICE pointers
 *                             (NULL entry: zeros) to [channels,K] in io_dtype:
 *                             the last K inputs of the cached prefix, oldest
 *                             first
 *   state_out  [n_ckpt,channels,K] io_dtype: one state per checkpoint of the
 *                             plan, in the plan's slot order; a slot can be
 *                             passed back as an initial state unchanged
 *
 * Only the plan's sequences, checkpoints and io_dtype are used, not its head
 * shape.  channels must make a row a multiple of 16 bytes.
 */
int ssm_conv1d_prefill(const ssm_plan_t *plan, int32_t channels, int32_t kernel_width,
                       const void *in, const float *weight, const float *bias,
                       const void *const *init_state_ptrs, void *out, void *state_out,
                       int32_t activation, void *hip_stream);

/*
 * Measurement aid (no passage of the paper: it serves the per-kernel timing of
 * the benchmark).  ssm_prefill on a matrix-core plan launches the operand
 * preparation, the scan and, when long sequences were cut into stretches
 * (ssm_plan_stretch), the kernels that add the carried states' contribution.
 * With non-NULL events (hipEvent_t created by the caller with timing enabled),
 * every later ssm_prefill / ssm_prefill_noalloc call of the calling thread
 * records the first event on its stream after the preparation kernel and the
 * second after the scan kernel, so that the caller can time each kernel alone;
 * NULL switches an event off again.  Nothing else changes.
 */
void ssm_profile_mark(void *after_first_kernel, void *after_second_kernel);

/* Release the plan and the device tables it made on first use (Section 4.1's
 * plan lives exactly as long as the batch it describes).  NULL is accepted. */
void ssm_plan_destroy(ssm_plan_t *plan);

/* Message of the last error on the calling thread ("" if none).  Every entry
 * point above sets it when it returns a negative ssm_status_t.  The pointer
 * stays valid until the next failing call on this thread. */
const char *ssm_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* SSM_PREFILL_H */
