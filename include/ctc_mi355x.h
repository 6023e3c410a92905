/*
 * ctc_mi355x.h -- batched CTC cost and gradient on one MI355X (gfx950).
 *
 * The library computes, for B independent utterances at once, the Connectionist
 * Temporal Classification cost of Section 3.3, Eq. (ctc),
 *
 *     cost_b = -ln  sum_{pi in Align(x_b, y_b)}  prod_{t < T_b}  softmax(x[t,b,:])[pi_t]
 *
 * and its derivative with respect to the pre-softmax activations x, by the
 * forward (alpha) / backward (beta) passes over the blank-interleaved label and
 * the per-character reduction described in the appendix "GPU Implementation of
 * CTC Loss Function".  The output softmax of Section 3.1 is fused into the path.
 * On the same lattice it also finds the most probable alignment of Section 5.1
 * (ctc_best_path).
 *
 * Plain C ABI: pointers and sizes only.  Each pointer argument is marked (host)
 * or (device).  The library allocates no device memory: every buffer, including
 * the scratch workspace, belongs to the caller (Section 4.3 motivates keeping
 * allocation off the training step).  All device work is enqueued on the given
 * stream and the calls return without waiting for it (never: see below); host
 * arrays are consumed before the call returns.
 *
 * State the library keeps, process-wide, behind one mutex (calls from several
 * threads are serialised while they prepare and enqueue, a few microseconds):
 *   - Per device, pinned host memory for the per-call metadata image that the
 *     first kernel of a host-metadata call reads: 8 slots of 256 KiB, allocated
 *     in one piece by the first call on that device and kept until the process
 *     ends.  A slot is free again once the call's second kernel has run.  No
 *     later call allocates, with two exceptions that each happen once: a batch
 *     whose image (72 bytes per utterance + 4 per label symbol) exceeds a slot
 *     gets a pool of larger slots, and a caller with more calls in flight than
 *     there are slots (it enqueues that far ahead of the GPU) gets a pool of
 *     twice as many.  The host never waits for a slot.  Pools stop growing at
 *     256 MiB per device; a call that then finds every slot in flight returns
 *     CTC_STATUS_NOT_READY immediately, with nothing enqueued.
 *     ctc_loss_and_grad_device uses none of this.
 *   - The poll budget of ctc_debug_set_poll_budget, and the calling thread's
 *     last HIP error code.
 */
#ifndef CTC_MI355X_H
#define CTC_MI355X_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    CTC_STATUS_SUCCESS = 0,
    CTC_STATUS_INVALID_VALUE = 1,       /* null pointer, size or id out of range, overlapping buffers */
    CTC_STATUS_WORKSPACE_TOO_SMALL = 2, /* workspace_bytes below what ctc_workspace_size reports */
    CTC_STATUS_HIP_ERROR = 3,           /* a HIP runtime call failed; see ctc_last_hip_error */
    CTC_STATUS_UNSUPPORTED = 4,         /* a size beyond what the kernels index: a label longer than
                                           CTC_MAX_LABEL_LENGTH, more than 65535 utterances, ... */
    CTC_STATUS_NOT_READY = 5            /* host-metadata calls only: so many earlier calls are still in
                                           flight that their metadata images fill the pinned memory the
                                           library may hold (256 MiB per device); nothing was enqueued:
                                           synchronise the stream, or call again later */
} ctc_status_t;

/* The HIP stream type, declared as hip_runtime_api.h declares it so that this header needs no
 * HIP include (repeating an identical typedef is allowed in C11 and C++). */
typedef struct ihipStream_t *hipStream_t;

/* Element type of activations AND gradients.  Arithmetic is always fp32/fp64 inside. */
typedef enum {
    CTC_DTYPE_F32 = 0,
    CTC_DTYPE_BF16 = 1
} ctc_dtype_t;

/* Longest label string one utterance may carry (lattice of 2*L+1 states). */
#define CTC_MAX_LABEL_LENGTH 1023

/* Kernel launches of one call, in order; index into ctc_profile_kernels' output. */
enum {
    CTC_KERNEL_SOFTMAX = 0,    /* row-wise log-softmax statistics + emission gather (for alphabets
                                  wider than 2048 also the dense part of the gradient) */
    CTC_KERNEL_LATTICE = 1,    /* alpha and beta recursions, one launch */
    CTC_KERNEL_GRADIENT = 2,   /* softmax minus normalised occupancy, zero fill of padding */
    /* A short copy launch (the per-call metadata, from pinned host memory into the workspace)
       precedes these three and is not timed separately; the grouping of each label's positions
       by symbol and the costs of degenerate utterances are prepared by extra workgroups of the
       softmax launch. */
    CTC_NUM_KERNELS = 3,       /* timed launches of any one call */
    CTC_KERNEL_BACKTRACE = 3   /* name index only: third launch of ctc_best_path (in place of the gradient) */
};

/*
 * Bytes of device workspace that ctc_loss_and_grad needs for this batch shape.
 * (Workspace sizing for the memory-allocation concern of Section 4.3.)
 *
 *   T, B, A          time steps of the tensor, utterances, alphabet size incl. blank; all >= 1;
 *                    more than 65535 utterances per call are refused (UNSUPPORTED)
 *   label_lengths    (host) [B], each in 0..CTC_MAX_LABEL_LENGTH
 *   input_lengths    (host) [B], each in 0..T
 *   bytes_out        (host) receives the size; the workspace must be 256-byte aligned
 *
 * Pure host computation: touches no GPU.  Returns INVALID_VALUE / UNSUPPORTED as above.
 */
ctc_status_t ctc_workspace_size(int T, int B, int A,
                                const int32_t *label_lengths,
                                const int32_t *input_lengths,
                                ctc_dtype_t dtype,
                                size_t *bytes_out);

/*
 * CTC cost and gradient for a minibatch (Section 3.3 Eq. (ctc); Section 3.1 softmax;
 * appendix on the GPU CTC implementation for the alpha/beta/reduction structure).
 *
 *   activations   (device) [T, B, A], A fastest, pre-softmax logits of type `dtype`.
 *                 Rows t >= input_lengths[b] are never read.
 *   flat_labels   (host) the B label strings back to back, sum(label_lengths) ids,
 *                 each in [0, A) and different from `blank`
 *   label_lengths (host) [B]
 *   input_lengths (host) [B]
 *   blank         id of the blank symbol, in [0, A)
 *   costs         (device) [B] float: -ln p_b in nats, per utterance, not averaged;
 *                 +inf when no alignment exists (fewer frames than symbols plus
 *                 adjacent repeats); 0 for an empty label with zero frames
 *   grads         (device) [T, B, A] of type `dtype`: d cost_b / d activations.
 *                 Rows t >= input_lengths[b], and all rows of an utterance with
 *                 infinite cost, are written as zeros.  Must not overlap activations.
 *                 NULL: costs only (the raw CTC cost that Section 5.1 uses as a filter
 *                 feature); the backward recursion and the gradient pass are then left out.
 *   workspace     (device) 256-byte aligned scratch of at least ctc_workspace_size bytes;
 *                 contents on entry are irrelevant, contents on exit are unspecified
 *   stream        the stream all work is enqueued on; NULL is the default stream
 *
 * Errors are reported by status only; nothing is printed or thrown.  On an error
 * found during validation nothing has been enqueued.  Results are bitwise
 * repeatable from run to run on one device.  Concurrent calls need distinct
 * workspaces.
 */
ctc_status_t ctc_loss_and_grad(const void *activations,
                               const int32_t *flat_labels,
                               const int32_t *label_lengths,
                               const int32_t *input_lengths,
                               int T, int B, int A, int blank,
                               ctc_dtype_t dtype,
                               float *costs,
                               void *grads,
                               void *workspace, size_t workspace_bytes,
                               hipStream_t stream);

/*
 * Same computation as ctc_loss_and_grad, but brackets each kernel with HIP events
 * on `stream`, waits for the stream, and reports the device time of each kernel of
 * this call in milliseconds (each interval less what two events recorded back to back
 * read, i.e. the cost of the bracketing itself).  For measurement (the per-kernel timings that the
 * paper's Table "gpucpuctc" aggregates per epoch), not for the training loop.
 *
 *   kernel_ms     (host) [CTC_NUM_KERNELS]; with grads == NULL there is no third launch and
 *                 the third entry is (close to) zero
 */
ctc_status_t ctc_profile_kernels(const void *activations,
                                 const int32_t *flat_labels,
                                 const int32_t *label_lengths,
                                 const int32_t *input_lengths,
                                 int T, int B, int A, int blank,
                                 ctc_dtype_t dtype,
                                 float *costs,
                                 void *grads,
                                 void *workspace, size_t workspace_bytes,
                                 hipStream_t stream,
                                 float *kernel_ms);

/*
 * The same computation for callers that keep lengths and labels on the device and cannot
 * take a detour through the host: code recorded into a HIP graph and replayed with new
 * contents in the same buffers, or a training step whose batch metadata never leaves the GPU
 * (keeping host work and transfers off the step: the theme of Section 4.3).  The call only
 * enqueues kernels on `stream`: it reads no host memory, copies nothing, waits for nothing and
 * touches no memory of the library's own, so it may be captured; every replay reads the
 * device arrays afresh.
 *
 * Since the host sees no lengths, the caller states bounds instead and everything is laid out
 * for the largest utterance they allow:
 *
 *   labels            (device) [B, max_label_length] int32, one padded row per utterance;
 *                     every entry is read, but only the first label_lengths[b] of row b are
 *                     looked at: the padding may hold anything
 *   label_lengths     (device) [B]
 *   input_lengths     (device) [B]
 *   max_label_length  0..CTC_MAX_LABEL_LENGTH; B is limited to 4096
 *   status_out        (device) [1] int32: what the host-side validation reports for the other
 *                     entry points, found on the device.  CTC_STATUS_SUCCESS, or
 *                     CTC_STATUS_INVALID_VALUE if some length is out of range (label_lengths[b]
 *                     not in 0..max_label_length, input_lengths[b] not in 0..T) or some label is
 *                     outside [0, A) or equal to blank; the utterances concerned get a NaN cost
 *                     and a zero gradient, the others are computed as usual.
 *   workspace         at least ctc_workspace_size_device bytes (larger than the exact-size
 *                     query of the host-metadata calls: T x B x (max_label_length + 1) lattice pairs)
 *   grads             may be NULL (costs only), as for ctc_loss_and_grad
 *   everything else as for ctc_loss_and_grad.  Results are the same numbers up to rounding:
 *                     bitwise those of ctc_loss_and_grad where both calls plan an utterance's chains
 *                     alike, which they do unless the bounds (B x max_label_length) make this call
 *                     plan its launch for total work, or use the one-barrier-per-step kernel, where
 *                     the actual labels would not.
 *
 * The return value covers what the host can check (pointers, T, B, A, blank, dtype, bounds,
 * workspace size, launch errors).
 */
ctc_status_t ctc_workspace_size_device(int T, int B, int A, int max_label_length,
                                       ctc_dtype_t dtype, size_t *bytes_out);

ctc_status_t ctc_loss_and_grad_device(const void *activations,
                                      const int32_t *labels,
                                      const int32_t *label_lengths,
                                      const int32_t *input_lengths,
                                      int max_label_length,
                                      int T, int B, int A, int blank,
                                      ctc_dtype_t dtype,
                                      float *costs,
                                      void *grads,
                                      int32_t *status_out,
                                      void *workspace, size_t workspace_bytes,
                                      hipStream_t stream);

/* ctc_loss_and_grad_device with per-launch device times, as ctc_profile_kernels (it waits for the
 * stream, so it cannot be captured): kernel_ms (host) [CTC_NUM_KERNELS] = softmax, lattice, gradient;
 * where a planning launch precedes the softmax launch (alphabets wider than 64 symbols, more than
 * 512 utterances) it is not timed separately. */
ctc_status_t ctc_profile_kernels_device(const void *activations,
                                        const int32_t *labels,
                                        const int32_t *label_lengths,
                                        const int32_t *input_lengths,
                                        int max_label_length,
                                        int T, int B, int A, int blank,
                                        ctc_dtype_t dtype,
                                        float *costs,
                                        void *grads,
                                        int32_t *status_out,
                                        void *workspace, size_t workspace_bytes,
                                        hipStream_t stream,
                                        float *kernel_ms);

/*
 * ctc_loss_and_grad_device without a workspace argument, for callers that cannot allocate device
 * memory or have it allocated for them: code recorded into a HIP graph, tight serving loops,
 * harnesses that forbid hipMalloc.  The workspace is an array of CTC_STATIC_WORKSPACE_BYTES that is
 * part of the library's device code: every GPU the library runs on holds its own copy from the
 * moment the library is loaded until the process ends.  The call allocates nothing (no hipMalloc,
 * no hipHostMalloc, no pinned staging); on its first use on a device it looks up the array's
 * address there, nothing more.
 *
 *   arguments, results and status_out as for ctc_loss_and_grad_device;
 *   a batch shape whose ctc_workspace_size_device exceeds CTC_STATIC_WORKSPACE_BYTES is refused
 *   with CTC_STATUS_WORKSPACE_TOO_SMALL before anything is enqueued (64 MiB hold, for instance,
 *   16 utterances of 750 frames and up to 250 label symbols over a 29-symbol alphabet).
 *
 * All calls on one GPU share that GPU's array, whatever their streams: calls that overlap in time
 * on one GPU race and give wrong results; calls on one stream, or otherwise ordered, are fine.  The
 * array keeps the previous call's contents; nothing in it needs clearing between calls (every word
 * a call reads it has written before).
 */
#define CTC_STATIC_WORKSPACE_BYTES (64u << 20)

ctc_status_t ctc_loss_and_grad_device_static(const void *activations,
                                             const int32_t *labels,
                                             const int32_t *label_lengths,
                                             const int32_t *input_lengths,
                                             int max_label_length,
                                             int T, int B, int A, int blank,
                                             ctc_dtype_t dtype,
                                             float *costs,
                                             void *grads,
                                             int32_t *status_out,
                                             hipStream_t stream);

/*
 * Most probable alignment of each utterance (Section 5.1, "Dataset Construction": the
 * alignment step of the segmentation pipeline),
 *
 *     l*_b = argmax_{pi in Align(x_b, y_b)}  prod_{t < T_b}  softmax(x[t,b,:])[pi_t],
 *
 * found on the same blank-interleaved lattice with the maximum in place of the sum and a
 * backtrace over the recorded predecessor choices.
 *
 *   activations, flat_labels, label_lengths, input_lengths, T, B, A, blank, dtype,
 *   workspace, workspace_bytes, stream: as for ctc_loss_and_grad (same workspace size)
 *   scores        (device) [B] float: -ln of the probability of l*_b, in nats; +inf when
 *                 no alignment exists; 0 for an empty label with zero frames
 *   alignment     (device) [B, T] int32, T fastest (utterance-major, unlike the activations):
 *                 for t < input_lengths[b] the lattice state of frame t, an index s into the
 *                 blank-interleaved label (s even: blank; s odd: label symbol (s-1)/2 of the
 *                 utterance), from which the frame's symbol and its position in the
 *                 transcript both follow; -1 for t >= input_lengths[b] and for every frame
 *                 of an utterance without an alignment.  Must not overlap the workspace.
 *
 * When several alignments are equally probable one of them is returned, the same one on
 * every run.  Status and error behaviour as for ctc_loss_and_grad.
 */
ctc_status_t ctc_best_path(const void *activations,
                           const int32_t *flat_labels,
                           const int32_t *label_lengths,
                           const int32_t *input_lengths,
                           int T, int B, int A, int blank,
                           ctc_dtype_t dtype,
                           float *scores,
                           int32_t *alignment,
                           void *workspace, size_t workspace_bytes,
                           hipStream_t stream);

/* ctc_best_path with per-launch device times, as ctc_profile_kernels:
 * kernel_ms (host) [CTC_NUM_KERNELS] = softmax, lattice (max recursion), backtrace. */
ctc_status_t ctc_profile_best_path(const void *activations,
                                   const int32_t *flat_labels,
                                   const int32_t *label_lengths,
                                   const int32_t *input_lengths,
                                   int T, int B, int A, int blank,
                                   ctc_dtype_t dtype,
                                   float *scores,
                                   int32_t *alignment,
                                   void *workspace, size_t workspace_bytes,
                                   hipStream_t stream,
                                   float *kernel_ms);

/* Prefix of the name under which launch `index` (0..CTC_KERNEL_BACKTRACE) appears in a profiler
 * trace (the full name depends on the variant chosen for the batch shape); NULL otherwise. */
const char *ctc_kernel_name(int index);

/* Static, human-readable name of a status code. */
const char *ctc_status_string(ctc_status_t status);

/* Raw hipError_t value of the most recent HIP failure seen by the calling thread (0 if none). */
int ctc_last_hip_error(void);

/*
 * Diagnostics.  The wavefronts that share a long label's recursion wait for each other by
 * polling a counter in LDS, at most `polls` times per wavefront and call (default 2^22, which
 * only a stuck neighbour exhausts); a wavefront that runs out carries on with what it has and
 * the utterance's cost is reported as NaN.  Setting the budget to 0 makes every such wait give
 * up at once, which lets a test see that error path with every kernel still running to its
 * end.  Negative values restore the default.  Applies to calls made afterwards, process-wide.
 */
void ctc_debug_set_poll_budget(int polls);

/*
 * Diagnostics.  Where a call's recursions leave compute units idle (fewer chains than three
 * quarters of the compute units, alphabets of at most 64 symbols), the gradient rows of the
 * utterances whose chains end early are written inside the recursions' launch, as soon as both
 * chains of an utterance have ended, and the gradient launch that follows only writes the rest.
 * `percent`: 0 switches that off for calls made afterwards, process-wide (for measurements of the
 * two forms side by side); 1..100 sets the share of the launch's expected duration within which an
 * utterance's chains must end for its rows to be written that way; negative restores the default.
 * Results are bitwise the same whatever the setting.
 */
void ctc_debug_set_overlap(int percent);

/*
 * Diagnostics, for one measurement: the order of the paper's own GPU design (CTC appendix: the forward
 * pass, then the backward pass) against this library's, which runs the two recursions side by side.
 * Nonzero `on`: host-metadata gradient calls made afterwards, process-wide, run the forward chains in
 * one launch and the backward chains in a second one after it (and no gradient rows inside those
 * launches); 0 restores the default.  Results are bitwise the same.
 */
void ctc_debug_set_sequential_chains(int on);

/*
 * Diagnostics, host only (no GPU is touched).  The recursions read their emissions several steps
 * ahead and without bounds checks, up to three chunks past either end of an utterance's block;
 * margins around the emission regions of the workspace are there to take those reads.  This
 * function replays, on the host, every emission read that the chains of the given batch would
 * make -- the very schedule and address arithmetic the kernels are built from -- against the
 * workspace layout, and returns the number of reads outside their region (0 is the only acceptable
 * answer), or -1 for arguments that ctc_workspace_size refuses.
 *
 *   max_label_length  negative: the layout of ctc_loss_and_grad (exact sizes); otherwise the layout
 *                     of ctc_loss_and_grad_device for that bound
 *   margin_floats     (host, may be NULL) receives the smallest distance, in floats, between a read
 *                     and an end of its region
 */
long ctc_debug_replay_emission_fetches(int T, int B, int A,
                                       const int32_t *label_lengths,
                                       const int32_t *input_lengths,
                                       int max_label_length,
                                       long *margin_floats);

/* Diagnostics: how many times the library has allocated pinned host memory so far in this
 * process (all devices).  1 after the first host-metadata call on one device, and still 1 after
 * any number of further calls that keep within 8 in flight and 256 KiB of metadata. */
long ctc_debug_staging_allocations(void);

#ifdef __cplusplus
}
#endif

#endif /* CTC_MI355X_H */
