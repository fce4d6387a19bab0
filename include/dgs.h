/*
 * libdgs -- the data-parallel hot path of DGS (dual-way gradient sparsification
 * with sparsification-aware momentum, arXiv 1910.10929) on one AMD MI355X.
 *
 * C ABI.  No allocation of device memory happens inside the library: the caller
 * owns every device buffer, including the workspace.  Unless marked "host", a
 * pointer argument is a DEVICE pointer.  Every call enqueues its work on the
 * context's HIP stream and returns without waiting for the GPU (exceptions are
 * stated per call).  Return value: 0 on success, a negative DGS_E* code
 * otherwise; nothing is thrown across the boundary.
 *
 * Concurrency.  A context serialises its calls through its stream and keeps per-call
 * scratch in its workspace: call it from one host thread at a time, and do not run two
 * calls of one context at once on the GPU (they would race on the workspace).  Different
 * contexts, each with its own workspace and stream, are independent -- e.g. a worker
 * context and a server context whose steps overlap.
 *
 * Notation: J tensors packed back to back in one flat fp32 buffer of n elements,
 * tensor j occupying [offsets[j], offsets[j+1]); n_j its size;
 * k_j = ceil(density * n_j) evaluated in IEEE double; K = sum_j k_j;
 * key(x) = bits(x) & 0x7FFFFFFF, the magnitude of an fp32 as a 31-bit integer.
 *
 * Selection rule used by the worker step and the pull ("thr <- R% of |x|" in
 * Algorithms 1-3, with density = 1 - R/100): per tensor, exactly the k_j entries
 * with the largest key; equal keys are resolved towards the lower index.  The
 * result is therefore unique, and identical on every code path of the library.
 */
#ifndef DGS_H
#define DGS_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct dgs_ctx dgs_ctx; /* opaque; host-side plan + views into the workspace */

enum {
    DGS_OK = 0,
    DGS_EINVAL = -1,    /* bad argument (NULL, misaligned, out of range) */
    DGS_ENOMEM = -2,    /* workspace too small / host allocation failed */
    DGS_ENOTSUP = -3,   /* valid request the library does not implement */
    DGS_ECAPACITY = -4, /* output capacity exceeded */
    DGS_EHIP = -5       /* a HIP runtime call failed */
};

/* Options for dgs_set_option(). */
enum {
    DGS_OPT_FORCE_EXACT = 1, /* How a call finds its candidate thresholds.  0 (default): from the previous
                                call on the same state (one pass over the data); a call without a usable
                                prediction -- the first one, a new density -- estimates them from a
                                histogram of a sixteenth of the data and goes on in one pass.  1: every
                                call takes two passes (full histogram, then collection).  2: every call
                                estimates from the sample.  The results are the same in all three: a
                                threshold that lets too few candidates through is repaired inside the
                                call */
    DGS_OPT_PROFILE = 2,     /* 1: attach start/stop HIP events to the kernels of each call */
    DGS_OPT_VALIDATE = 3,    /* 1: dgs_server_push checks idx on the device (synchronises) */
    DGS_OPT_MARGIN_PCT = 4,  /* candidate over-provisioning in percent of k_j (default 50) */
    DGS_OPT_STREAM_QUADS = 5,/* 4096-element groups per workgroup of the streaming kernel */
    DGS_OPT_SEGMENTED = 6,   /* which tensors continue through the multi-kernel chain behind the
                                selection: 0 automatic (candidate lists too long for one workgroup,
                                dense requests), 1 every tensor of at least 65536 elements, 2 never */
    DGS_OPT_REPAIR_ROUND = 7,/* 1 (default): the selection launch carries the workgroups that collect
                                again, with a fresh threshold, the tensors whose predicted threshold
                                failed (they wait inside the launch and return at once when their
                                tensor is fine); 0: such tensors are selected from the state buffer
                                by one workgroup (slow on large tensors) */
    DGS_OPT_WIRE_VALUE_BITS = 9, /* 32 (default): the wire form carries fp32 values and is lossless; 16: every
                                value travels as a bfloat16 (the upper half of the fp32, rounded to nearest,
                                halfway cases to even, NaN kept) -- what dgs_decode returns then differs
                                from what was encoded by up to 2^-9 relative.  Applies to dgs_wire_bytes,
                                dgs_encode and dgs_decode.  Not part of the paper's method (its Section 6
                                leaves quantisation to future work): the caller decides what to do with
                                the rounding error */
    DGS_OPT_SPIN_LIMIT = 8   /* polls after which a waiting workgroup of the selection gives up
                                (default 2^20, far beyond any wait that ends); it is then counted
                                in dgs_stats.internal_errors.  A tensor whose prediction failed in
                                that launch is then left unselected: after a call that raised
                                internal_errors the outputs and the context are not to be used */
};

/* Kernel classes reported by dgs_profile_read(). */
enum {
    DGS_PROF_WORKER_STREAM = 0, /* accumulate + candidate pass over grad/state */
    DGS_PROF_WORKER_SELECT = 1,
    DGS_PROF_PULL_STREAM = 2,   /* candidate pass over one difference row */
    DGS_PROF_PULL_SELECT = 3,
    DGS_PROF_PUSH = 4,
    DGS_PROF_EXACT_EXTRA = 5,   /* second (collecting) pass of the non-predicted path */
    DGS_PROF_WORKER_SEGMENTED = 6, /* chain kernels behind the selection, first begin to last end */
    DGS_PROF_PULL_SEGMENTED = 7,
    DGS_PROF_ENCODE = 8,        /* dgs_encode */
    DGS_PROF_DECODE = 9,        /* dgs_decode */
    DGS_PROF_KINDS = 10
};

typedef struct dgs_stats {
    uint64_t calls_worker, calls_pull, calls_push;
    uint64_t exact_calls;      /* calls that ran the two-pass (non-predicted) path */
    uint64_t fallback_tensors; /* tensors selected from the buffers by one workgroup after everything else failed */
    uint64_t fallback_elems;   /* elements re-read by those */
    uint64_t candidates;       /* candidates collected by streaming passes */
    uint64_t internal_errors;  /* must stay 0 */
    uint64_t segmented_tensors; /* tensors resolved through the chain kernels */
    uint64_t repaired_tensors;  /* tensors whose prediction failed and that were resolved inside the call with
                                   a fresh threshold: lists trimmed in place, or collected a second time */
} dgs_stats;

/*
 * Bytes of device workspace needed for this layout and W server-side workers
 * (W may be 0 for a worker-only context).  Pure host computation.
 * offsets: host, J+1 entries, elements, offsets[0] == 0, strictly increasing
 * (every tensor has at least one element), offsets[J] = n < 2^32.
 * Returns 0 on invalid arguments.
 */
size_t dgs_workspace_bytes(const uint64_t *offsets, uint32_t J, uint32_t W);

/*
 * Build a context.  `workspace` is device memory of at least
 * dgs_workspace_bytes() bytes, 256-byte aligned, owned by the caller and left
 * untouched by the caller until dgs_destroy().  `hip_stream` is a hipStream_t
 * (NULL = the default stream).  Uploads the launch plan and clears the
 * workspace's counters on that stream, then waits for that to finish.
 */
/*
 * What a context remembers between calls.  Besides the layout it keeps, per tensor, the
 * threshold hints that make the one-pass path possible: one set for worker steps and one per
 * server worker slot (W sets).  A hint describes the buffer it was learned from, so a context
 * serves ONE worker state (momentum or residual buffer) and, per slot, one difference or sent
 * row: stepping two different states through the same context alternately stays exact -- a
 * failed prediction is always collected again -- but pays that second collection on most
 * calls.  Give every state its own context (the workspace is about 4.4 bytes per element).
 * Calls on one context must not overlap; contexts are independent.
 *
 * Launch plans (k_j, output offsets, wire layout) are cached per density, 8 densities per
 * context, least recently used evicted.  While the context's stream is being captured into a
 * HIP graph a density that is not yet cached returns DGS_ENOTSUP (planning copies tables to
 * the device, which a capture must not contain): call once with that density before the
 * capture.  Plans used during a capture are never evicted.
 */
int dgs_create(dgs_ctx **out, const uint64_t *offsets /*host*/, uint32_t J, uint32_t W,
               void *workspace, size_t workspace_bytes, void *hip_stream);

/* Waits for the stream, then releases host resources.  Frees no device memory. */
int dgs_destroy(dgs_ctx *ctx);

/* K = sum_j ceil(density * n_j).  Pure host. density must be in (0, 1]. */
int dgs_nnz(const dgs_ctx *ctx, double density, uint64_t *K_out /*host*/);

/*
 * One worker iteration after the backward pass: Algorithm 3 (accumulate with
 * momentum, per-tensor threshold, mask, send, rescale the unsent part; Eq. 11-12),
 * or Algorithm 1 (residual accumulation) -- everything between "Backward" and
 * "Send encode(g)".
 *
 *   grad      n floats, read only: the stochastic gradient.
 *   momentum  n floats, in/out, or NULL.
 *   residual  n floats, in/out, or NULL.  Exactly one of the two must be given.
 *   lr        learning rate eta.
 *   m         momentum coefficient in [0, 1); must be 0 when `residual` is used.
 *   density   fraction kept per tensor, in (0, 1].
 *   idx_out   K x u32: flat indices of the sent entries, ascending; tensor j's
 *             k_j entries start at sum_{i<j} k_i.
 *   val_out   K x f32: the sent values.
 *   nnz_out   host, optional: receives K immediately (it is static).
 *
 * Arithmetic, per element i:  a_i = fmaf(lr, grad_i, state_i)   (one rounding,
 * denormals kept);  sent entries: val = a_i, state_i = m * a_i;  unsent entries:
 * state_i = a_i.
 *
 * State convention.  With `momentum`, the buffer holds s = m * u where u is the
 * paper's velocity: Algorithm 3 keeps u = a for sent entries and rescales unsent
 * ones to u = a / m, and its next accumulate multiplies by m again (the
 * cancellation Eq. 13 relies on); storing s removes the division, keeps
 * "sent + kept == accumulated" exact, and makes m = 0 legal.  Read the paper's
 * velocity as u = s / m.  With `residual` (m = 0) the buffer is Algorithm 1's v:
 * sent entries become 0, unsent ones keep the accumulated value.
 * Both buffers given (separate momentum and residual, as in momentum-corrected
 * schemes) is not part of this method: DGS_ENOTSUP.
 *
 * Buffers must be 4-byte aligned; 16-byte alignment gives the fast path.
 *
 * Graph capture.  Once a call at `density` has been made eagerly on this context (the
 * launch plan of a density is uploaded on its first use, and the first call of a stream
 * takes the two-pass path), dgs_worker_step, dgs_server_push / dgs_server_push_model
 * (without DGS_OPT_VALIDATE) and dgs_server_pull / dgs_server_pull_sent enqueue kernels only
 * -- no memset or copy nodes, no host wait -- and may be captured into a HIP graph on the
 * context's stream.  The choice between the predicted and the two-pass path is taken on
 * the host when the call is made, i.e. at capture time; everything a failed prediction
 * needs afterwards runs on the device, so replays stay exact.
 */
int dgs_worker_step(dgs_ctx *ctx, const float *grad, float *momentum, float *residual,
                    float lr, float m, double density,
                    uint32_t *idx_out, float *val_out, uint64_t *nnz_out /*host*/);

/*
 * dgs_worker_step for callers that cannot allocate device memory or copy to it: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments,
 * arithmetic and results as dgs_worker_step, without a context: the layout is given with the
 * call (offsets: host, J + 1 entries, as for dgs_create), the work is enqueued on `hip_stream`
 * (NULL = the default stream), and the workspace is an array of DGS_STATIC_SCRATCH_BYTES bytes
 * that the library holds in device memory on every GPU it runs on, until the process ends.
 * The call makes no hipMalloc / hipFree / hipHostMalloc, creates no events, issues no copies
 * and does not wait: the layout tables travel as kernel arguments.
 * Limits: J <= DGS_STATIC_MAX_TENSORS, and dgs_workspace_bytes(offsets, J, 0) <=
 * DGS_STATIC_SCRATCH_BYTES (about 1e7 parameters); beyond them DGS_ECAPACITY is returned and
 * nothing is enqueued.  Nothing is remembered between calls (each starts from a cleared
 * workspace and takes the two-pass path), so it is slower than a context.
 * All calls on one GPU share that GPU's array: two calls whose work overlaps on the GPU (two
 * streams, two threads) race; order them.
 */
#define DGS_STATIC_SCRATCH_BYTES (48u << 20)
#define DGS_STATIC_MAX_TENSORS 256
int dgs_worker_step_static(const uint64_t *offsets /*host*/, uint32_t J, const float *grad,
                           float *momentum, float *residual, float lr, float m, double density,
                           uint32_t *idx_out, float *val_out, uint64_t *nnz_out /*host*/,
                           void *hip_stream);

/*
 * Give the server side its per-worker difference buffers: W rows of n floats,
 * row-major, row w = D_w = M - v_w in the notation of Eq. 1-6 (the part of the
 * accumulated update M that worker w has not been sent yet).  The caller
 * allocates and zero-initialises it (M_0 = 0, v_w = 0) and keeps it alive.
 */
int dgs_server_attach(dgs_ctx *ctx, float *diff);

/*
 * The server receives one decoded update g from `worker_id` (Algorithm 2,
 * "M <- M - decode(g)"; Eq. 1):  model[idx] -= val, and D_w[idx] -= val for every
 * worker w (Eq. 3: the difference owed to every worker, the sender included,
 * moves with M).  g already carries the learning rate.
 *   model  n floats in/out (theta_0 + M), or NULL to keep only the differences.
 *   idx    nnz x u32, strictly ascending (hence unique: the scatter needs no atomics);
 *   val    nnz x f32.
 * With DGS_OPT_VALIDATE the order/range precondition is checked on the device
 * (this synchronises) and DGS_EINVAL is returned on violation, before anything is
 * modified.
 */
int dgs_server_push(dgs_ctx *ctx, float *model, uint32_t worker_id,
                    const uint32_t *idx, const float *val, uint64_t nnz);

/*
 * The server answers `worker_id` with secondary compression (Algorithm 2, the
 * per-tensor threshold loop on G; Eq. 6): G = the k_j largest-magnitude entries
 * per tensor of D_k; afterwards those entries of D_k are +0 (v_k += G), the rest
 * stays accumulated on the server.  Outputs as in dgs_worker_step.  If a tensor
 * of D_k has fewer than k_j nonzeros, zero-valued entries at its lowest indices
 * complete the message (exactly K pairs are always produced).
 */
int dgs_server_pull(dgs_ctx *ctx, uint32_t worker_id, double density,
                    uint32_t *idx_out, float *val_out, uint64_t *nnz_out /*host*/);

/*
 * The server state as Algorithm 2 prints it (Eq. 3-6), an alternative to the
 * difference rows above: one global model (theta_0 + M) and, per worker, what that
 * worker has been sent so far, sent_k = theta_0 + v_k.  A push then touches the model
 * only (nnz read-modify-writes, independent of W); a pull streams two buffers
 * (8 bytes per parameter instead of 4).  Worth it for many workers or dense pushes.
 *
 *   dgs_server_attach_sent   W rows of n floats, row-major, caller-allocated, each row
 *                            initialised by the caller to the initial model theta_0.
 *   dgs_server_push_model    model[idx] -= val  ("M <- M - decode(g)", Eq. 1); idx strictly
 *                            ascending; DGS_OPT_VALIDATE as for dgs_server_push.
 *   dgs_server_pull_sent     G = per tensor the k_j largest-magnitude entries of
 *                            model - sent_k (one fp32 subtraction per element; the
 *                            printed "G <- M - v_k" followed by the threshold loop), then
 *                            sent_k[idx] += val ("v_k <- v_k + G", the sign Eq. 4 and
 *                            Eq. 6 require; one fp32 addition).  Outputs as in
 *                            dgs_server_pull.  In exact arithmetic this is the same message
 *                            as dgs_server_pull's; in fp32 the two forms round differently.
 * A context uses one of the two forms for a given worker id: they share that worker's
 * threshold hints.
 */
int dgs_server_attach_sent(dgs_ctx *ctx, float *sent);
int dgs_server_push_model(dgs_ctx *ctx, float *model, const uint32_t *idx, const float *val,
                          uint64_t nnz);
int dgs_server_pull_sent(dgs_ctx *ctx, const float *model, uint32_t worker_id, double density,
                         uint32_t *idx_out, float *val_out, uint64_t *nnz_out /*host*/);

/*
 * The server answers `worker_id` without secondary compression (Algorithm 2 with
 * the switch off; Eq. 3-4): G = every entry of D_k with a nonzero magnitude,
 * ascending; afterwards D_k == 0.  nnz is data dependent: the call waits for
 * the stream and writes the count to nnz_out (host).  If the count exceeds
 * `capacity`, nothing is modified, nnz_out still receives the count and
 * DGS_ECAPACITY is returned.
 */
int dgs_server_pull_all(dgs_ctx *ctx, uint32_t worker_id, uint32_t *idx_out, float *val_out,
                        uint64_t capacity, uint64_t *nnz_out /*host*/);
/* The same on the printed state (after dgs_server_attach_sent): G = every nonzero of
 * model - sent_k (Eq. 3), then sent_k += G on those (Eq. 6). */
int dgs_server_pull_all_sent(dgs_ctx *ctx, const float *model, uint32_t worker_id, uint32_t *idx_out,
                             float *val_out, uint64_t capacity, uint64_t *nnz_out /*host*/);

/*
 * Worker applies a decoded message (Algorithm 1/3, "theta <- SGD(theta,
 * decode(G))"; Eq. 5 with sign = +1):  dst[idx] = fmaf(sign, val, dst[idx]).
 * dst: n floats.  idx must be unique; an index outside [0, n) is skipped.  With
 * DGS_OPT_VALIDATE the message is checked on the device as for dgs_server_push (strictly
 * ascending, in range; this synchronises) and DGS_EINVAL is returned before dst is touched.
 */
int dgs_apply_sparse(dgs_ctx *ctx, float *dst, const uint32_t *idx, const float *val,
                     uint64_t nnz, float sign);

/*
 * Wire form of a message: the encode() / decode() of Algorithms 1-3, which the paper
 * describes only as packing the nonzero entries into coordinate format.  The (idx, val)
 * pairs of the calls above are that format in memory; these two calls turn a message into
 * the bytes to put on a network and back, without loss.  The layout is this library's own:
 *   bytes [0, 4K)  the K = dgs_nnz(density) values, fp32 little-endian, in message order;
 *   then, tensor after tensor, the k_j local indices idx - off_j of tensor j, b_j bits each
 *   (b_j = number of bits of n_j - 1, at least 1), entry e in bits [e b_j, (e + 1) b_j) of
 *   the tensor's block, least significant bit first, bit i of a block in bit i mod 8 of its
 *   byte i / 8, each block padded with zero bits to a multiple of 4 bytes.
 * With DGS_OPT_WIRE_VALUE_BITS = 16 the value area is instead K bfloat16 values of 2 bytes,
 * little-endian, padded with zero bytes to a multiple of 4 (lossy: see the option); the index
 * blocks are the same.
 * Both ends derive k_j, b_j and every offset from the layout and the density: no header.
 * A message is what dgs_worker_step, dgs_server_pull or dgs_server_pull_sent returned for
 * `density`: exactly k_j ascending entries per tensor (not dgs_server_pull_all's).
 *   dgs_wire_bytes  size of the wire form in bytes (host result; a multiple of 4).
 *   dgs_encode      idx, val: device, K entries; wire: device, 4-byte aligned,
 *                   dgs_wire_bytes(density) bytes, written completely.
 *   dgs_decode      the reverse; idx_out, val_out: device, K entries.
 * Asynchronous on the context's stream.  With DGS_OPT_VALIDATE both calls check on the device
 * that every entry lies inside its tensor (this synchronises) and return DGS_EINVAL if not;
 * without it such an index is cut to b_j bits (encode) or passed on as decoded (decode;
 * dgs_server_push, dgs_server_push_model and dgs_apply_sparse skip indices outside [0, n)).
 */
int dgs_wire_bytes(dgs_ctx *ctx, double density, uint64_t *bytes_out /*host*/);
int dgs_encode(dgs_ctx *ctx, double density, const uint32_t *idx, const float *val, void *wire);
int dgs_decode(dgs_ctx *ctx, double density, const void *wire, uint32_t *idx_out, float *val_out);

int dgs_set_option(dgs_ctx *ctx, int option, int64_t value);

/* Waits for the stream, then copies the counters to `out` (host). */
int dgs_get_stats(dgs_ctx *ctx, dgs_stats *out /*host*/);

/*
 * With DGS_OPT_PROFILE on: waits for the stream, then reports, for kernel class
 * `kind`, how many launches were timed since the last read and their summed
 * duration in milliseconds (HIP events attached to each kernel dispatch on the
 * context's stream: begin to end of the kernel); resets that class.  At most
 * 4096 launches per class are kept between reads.
 */
int dgs_profile_read(dgs_ctx *ctx, int kind, uint64_t *launches /*host*/, double *total_ms /*host*/);

const char *dgs_strerror(int code);

#ifdef __cplusplus
}
#endif
#endif /* DGS_H */
