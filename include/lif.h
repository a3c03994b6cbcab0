/*
 * lif.h - C ABI of the MI355X (gfx950) sparse-FFN hot path of "LLM in a flash"
 * (arXiv 2312.11514): per-token FFN inference over predicted-active neurons held
 * in an HBM neuron cache that is fed from pinned host memory (standing in for flash).
 *
 * One handle (lif_layer) = one FFN layer.  Per token (or per batch of tokens) the
 * caller issues, on one HIP stream and without any host synchronisation,
 *
 *     lif_predict -> lif_update_window -> lif_load_bundles -> lif_sparse_ffn
 *
 * All counts (added / removed neurons, rows in use) stay on the device, so the four
 * calls chain without a host round trip and can be captured into a HIP graph.
 *
 * Conventions
 *   - Plain C; every call returns a status (LIF_OK = 0).  No call blocks or
 *     synchronises except lif_get_state, lif_get_counters and lif_profile_collect.
 *   - "device" pointers are HBM addresses valid on the GPU that is current when
 *     lif_create is called; "host" pointers are CPU addresses.  Streams are passed
 *     as void* holding a hipStream_t (NULL = the default stream).
 *   - The library allocates no device memory: every array, including the scratch
 *     workspace, is owned by the caller and must outlive the handle.
 *   - Element type E is fp32 (LIF_F32) or IEEE fp16 (LIF_F16).  G = 2 vectors per
 *     bundle (up row | down column), G = 3 for gated layers (gate row | up row | down column).
 *   - Shape limits: d_model, rank multiples of 8 (fp16) or 4 (fp32); d_ffn a multiple
 *     of 8 and at most 65536; rank at most 2048; max_batch at most 8; window_k at most 256.
 *   - A device-detected error (capacity overflow) sets a sticky flag: until lif_reset
 *     every hot call becomes a no-op on the device; lif_get_state reports the flag.
 *   - Calls on one handle must not overlap (one stream at a time).
 */
#ifndef LIF_H
#define LIF_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct lif_layer lif_layer;

enum lif_status {
    LIF_OK = 0,
    LIF_INVALID_ARG = 1,   /* null pointer, unsupported shape, batch > max_batch */
    LIF_BAD_STATE = 2,     /* calls out of order (see lif_update_window / lif_load_bundles) */
    LIF_CAPACITY = 3,      /* reported by lif_get_state: active set exceeded capacity_rows */
    LIF_HIP_ERROR = 4      /* a HIP runtime call failed; see lif_last_error_string */
};

enum lif_dtype { LIF_F32 = 0, LIF_F16 = 1 };

/* How lif_sparse_ffn reads the cache (Section 3.3, inference over the cached rows). */
enum lif_ffn_mode {
    LIF_FFN_SKIP_DEAD = 0, /* do not read the down column of rows whose activation is zero */
    LIF_FFN_FULL_BUNDLE = 1 /* read every cached bundle completely */
};

/* What decides which neurons are predicted active (step 1). */
enum lif_predictor {
    LIF_PRED_LOWRANK = 0,  /* low-rank predictor (x A) B + c > theta (Section 3.1, Fig. 3b)               */
    LIF_PRED_GATE = 1      /* the resident gate projection itself (Appendix, Llama 2, "Alternative         */
                           /* approaches"): mask_i = gate_i . x + b_i > theta, exact; bundles = up | down; */
                           /* y_t = sum_s relu(gate . x_t + b)_s * (up_s . x_t) * down_s; glu = 0; batches */
                           /* and passes of several tokens as with the low-rank predictor                  */
};

typedef struct lif_config {
    int32_t d_model;        /* d: length of the up row and of the down column              */
    int32_t d_ffn;          /* F: number of intermediate neurons of the layer              */
    int32_t rank;           /* r: rank of the low-rank predictor (Section 3.1, Fig. 3b)    */
    int32_t window_k;       /* k: sliding window in steps, current step included (Fig. 4b) */
    int32_t capacity_rows;  /* rows preallocated in the cache ("Req_i", Section 3.3)       */
    int32_t max_batch;      /* largest batch of tokens per step (1..8)                     */
    int32_t glu;            /* 0: bundle = up|down, 1: bundle = gate|up|down               */
    int32_t dtype;          /* enum lif_dtype: type of x, y, A, B and the bundles          */
    int32_t ffn_mode;       /* enum lif_ffn_mode                                           */
    int32_t shrink_window;  /* 1: dynamic window (Appendix, Persimmon / Phi-2): when the active  */
                            /* set would exceed capacity_rows the oldest masks leave the window  */
                            /* until it fits; 0: such a step is a LIF_CAPACITY error             */
    int32_t predictor;      /* enum lif_predictor                                          */
    float threshold;        /* theta: neuron i is predicted active iff logit_i > theta     */
} lif_config;

typedef struct lif_buffers {
    /* predictor (device, read-only): logits = (x A) B + c                               */
    const void* A;          /* LIF_PRED_LOWRANK: the first predictor matrix stored with the */
                            /* contraction dimension contiguous, [rank x d_model] row-major, E */
                            /* (row j = column j of the paper's d_model x rank matrix);     */
                            /* LIF_PRED_GATE: the gate projection [d_ffn x d_model]         */
                            /* row-major, E (row i = gate weights of neuron i)              */
    const void* B;          /* [rank x d_ffn] row-major, E; unused (may be NULL) with       */
                            /* LIF_PRED_GATE                                                */
    const float* c;         /* [d_ffn] per-neuron offset, fp32; may be NULL (= 0)         */
    /* bias of the ReLU'd projection per original neuron (device, read-only)             */
    const float* b;         /* [d_ffn] fp32                                               */
    /* bundle store: PINNED HOST memory (hipHostMalloc or equivalent), read-only         */
    const void* host_bundles; /* [d_ffn x G*d_model] E, row i = (gate_i |) up_i | down_i   */
    /* neuron cache (device, read-write; Section 3.3 "matrix", "pointers", "bias")       */
    void* matrix;           /* [capacity_rows x G*d_model] E                              */
    int32_t* pointers;      /* [capacity_rows] slot -> original neuron id                 */
    float* bias;            /* [capacity_rows] fp32                                       */
    /* scratch (device, read-write), at least lif_workspace_bytes(cfg) bytes, 256-aligned; it
     * also holds the window state ("last_k_active": the last window_k step masks) and the
     * device-resident counts                                                             */
    void* workspace;
    size_t workspace_bytes;
    /* optional second part of the bundle store (PINNED HOST memory, read-only), normally NULL.  If set, the store is
     * NOT bundled (the layout that Section 3.2's bundling replaces, kept for measuring what bundling buys):
     * host_bundles then holds only the activation vectors, [d_ffn x (G-1)*d_model] E (row i = (gate_i |) up_i), and
     * host_down the down columns, [d_ffn x d_model] E; every new neuron costs two reads.  The cache rows, and so
     * every result, are the same as with the bundled store. */
    const void* host_down;
} lif_buffers;

typedef struct lif_state {
    int32_t num_used;       /* rows of the cache in use                                   */
    int32_t step;           /* number of completed lif_update_window calls since reset    */
    int32_t error;          /* LIF_OK or LIF_CAPACITY (sticky until lif_reset)            */
    int32_t last_added;     /* |added| of the last lif_update_window                      */
    int32_t last_removed;   /* |removed| of the last lif_update_window                    */
    int32_t last_moved;     /* rows moved by the last deletion                            */
    int32_t window_len;     /* step masks in the window after the last update (<= window_k) */
} lif_state;

typedef struct lif_counters {
    uint64_t steps;         /* lif_update_window calls that committed                     */
    uint64_t added;         /* sum of |added|                                             */
    uint64_t removed;       /* sum of |removed|                                           */
    uint64_t rows_moved;    /* rows rewritten inside the cache by deletions               */
    uint64_t h2d_bytes;     /* bytes read from the host bundle store                      */
    uint64_t ffn_calls;     /* lif_sparse_ffn calls                                       */
    uint64_t ffn_rows;      /* sum over those calls of the rows in use                    */
    uint64_t ffn_active;    /* sum over those calls of the rows with a non-zero activation */
} lif_counters;

/* Kernels timed by the profiling hooks, in the order of lif_profile_collect's arrays. */
enum lif_kernel_id {
    LIF_K_PREDICT_XA = 0,   /* t = x A                                                    */
    LIF_K_PREDICT_MASK = 1, /* logits = t B + c, threshold, pack                          */
    LIF_K_WINDOW = 2,       /* window diff, added / removed ids, deletion plan            */
    LIF_K_LOAD = 3,         /* row moves + host-to-device bundle append                   */
    LIF_K_FFN_UP = 4,       /* activations of all cached rows                             */
    LIF_K_FFN_DOWN = 5,     /* y = sum of activation x down column                        */
    LIF_K_COUNT = 6
};

/* Bytes of scratch lif_create needs for this configuration (0 if cfg is invalid). */
size_t lif_workspace_bytes(const lif_config* cfg);

/*
 * Build a layer handle over caller-owned arrays (Section 3.3: everything is
 * preallocated once).  Validates shapes and alignment, records the device alias of
 * the pinned bundle store, and enqueues nothing: call lif_reset before the first step.
 * Errors: LIF_INVALID_ARG (null/unsupported), LIF_HIP_ERROR (bundle store is not
 * device-accessible pinned memory).
 */
int lif_create(const lif_config* cfg, const lif_buffers* buf, lif_layer** out);

/* Frees the host-side handle only (never the caller's arrays). NULL is accepted. */
int lif_destroy(lif_layer* layer);

/*
 * Empty the cache (Section 3.3: num_used starts at zero): num_used = 0, every
 * window empty, step = 0, error flag and counters cleared.  Enqueued on `stream`; does
 * not touch the matrix contents.
 */
int lif_reset(lif_layer* layer, void* stream);

/*
 * Step 1, low-rank predictor (Section 3.1 "Anticipating ReLU Sparsity", Fig. 3b;
 * active = positive output, Section 3.1 "The Sliding Window Technique").
 *   x_dev          [batch x d_model] E, device, read-only
 *   masks_dev      [batch x d_ffn/8] bytes, device, written: bit (i mod 8) of byte i/8
 *                  of row t is 1 iff ((x_t A) B)_i + c_i > threshold
 *   step_mask_dev  [d_ffn/8] bytes, device, 8-byte aligned, written: OR of the batch's masks;
 *                  may equal masks_dev when batch == 1
 * Sums are accumulated in fp64 so the decision does not depend on summation order
 * beyond ~1e-15 relative.  NaN logits compare false (inactive).
 */
int lif_predict(lif_layer* layer, const void* x_dev, int32_t batch,
                uint8_t* masks_dev, uint8_t* step_mask_dev, void* stream);

/*
 * Step 2, sliding window (Section 3.1 "The Sliding Window Technique", Fig. 4b).
 * With S_t = union of the last window_k step masks (this one included):
 *   added_dev    [d_ffn] int32, device, written: S_t \ S_{t-1}, ascending neuron id
 *   removed_dev  [d_ffn] int32, device, written: S_{t-1} \ S_t, ascending neuron id
 *   n_added_dev, n_removed_dev  [1] int32, device, written: the two counts
 * Records the mask in the window state and advances the step counter.  If |S_t| would exceed
 * capacity_rows: with shrink_window = 0 nothing is changed, both counts are written as 0 and
 * the sticky error flag is set to LIF_CAPACITY; with shrink_window = 1 the oldest masks are
 * dropped from the window for good, one by one, until the union fits (S_t = union of the
 * newest window_len masks, window_len maximal), and only a step mask that does not fit on
 * its own is a LIF_CAPACITY error.
 * Must alternate with lif_load_bundles (LIF_BAD_STATE otherwise): the cache has to
 * hold S_{t-1} when the window moves.
 */
int lif_update_window(lif_layer* layer, const uint8_t* step_mask_dev,
                      int32_t* added_dev, int32_t* n_added_dev,
                      int32_t* removed_dev, int32_t* n_removed_dev, void* stream);

/*
 * Step 2 for a verification pass of speculative decoding (Section 4.3 "Speculative Decoding";
 * Appendix, related work on speculative decoding: the window then moves by several tokens at once).
 *   masks_dev  [n_tokens x d_ffn/8] bytes, device, 8-byte aligned: the per-token masks of the
 *              pass (as written by lif_predict with batch = n_tokens); d_ffn % 64 == 0
 *   keep       0..n_tokens: the first `keep` tokens (those expected to be accepted; the paper's
 *              choice is about alpha * (lambda + 1) for acceptance ratio alpha) enter the window,
 *              one entry per token, exactly as if pushed one after the other; the masks of the
 *              remaining tokens are needed for this pass only and leave with the next update.
 * The cache must hold, for this pass, the union of the last window_k kept token masks and of
 * the transient masks: added / removed are the difference to what it holds now.  If that exceeds
 * capacity_rows: with shrink_window = 0 a LIF_CAPACITY error; with shrink_window = 1 the oldest window
 * masks leave for good, one by one, until the masks of the pass and the remaining window fit (only a
 * pass whose own masks do not fit is a LIF_CAPACITY error).  Alternates with
 * lif_load_bundles like lif_update_window; follow with lif_sparse_ffn(batch = n_tokens).
 */
int lif_update_window_tokens(lif_layer* layer, const uint8_t* masks_dev, int32_t n_tokens, int32_t keep,
                             int32_t* added_dev, int32_t* n_added_dev, int32_t* removed_dev,
                             int32_t* n_removed_dev, void* stream);

/*
 * Step 3, cache update (Section 3.3 items 1 and 2, Fig. 6; bundles per Section 3.2).
 * Deletion: with c = *n_removed_dev and n' = num_used - c, the rows whose neuron left
 * the window are overwritten by the last rows: the j-th lowest dead slot below n'
 * receives the j-th highest live slot at or above n' (matrix row, pointer and bias
 * move together; at most c rows move).  Insertion: the bundle of the j-th added
 * neuron a_j is read from host_bundles[a_j] and written to row n' + j, with
 * pointers[n'+j] = a_j and bias[n'+j] = b[a_j]; num_used = n' + *n_added_dev.
 * The arguments must be the arrays written by the preceding lif_update_window.
 * Adds |added| x bundle bytes to the h2d_bytes counter.  LIF_BAD_STATE if no
 * lif_update_window is pending.
 */
int lif_load_bundles(lif_layer* layer, const int32_t* added_dev, const int32_t* n_added_dev,
                     const int32_t* removed_dev, const int32_t* n_removed_dev, void* stream);

/*
 * Step 4, FFN over the cached rows (Section 3.3 item 3):
 *   y_t = sum_{s < num_used} relu(up_s . x_t + bias_s) * down_s
 *   gated:  y_t = sum_s relu(gate_s . x_t + bias_s) * (up_s . x_t) * down_s
 * over every row in use (the whole window union).  Products of E-typed values,
 * fp32 accumulation, y rounded once to E.
 *   x_dev  [batch x d_model] E, device, read-only
 *   y_dev  [batch x d_model] E, device, overwritten (zeros when the cache is empty)
 * The summation order is fixed (slot order within fixed strides), so results are
 * reproducible run to run bit for bit.
 */
int lif_sparse_ffn(lif_layer* layer, const void* x_dev, int32_t batch, void* y_dev, void* stream);

/*
 * lif_sparse_ffn for callers that cannot allocate and want no scratch of their own in the call: code under HIP
 * graph capture, tight serving loops, harnesses that forbid allocation.  Same arguments, same arithmetic
 * and bit-identical results; the activations and the partial outputs of the call (the scratch that
 * lif_sparse_ffn keeps in the layer's workspace) live in a static device array inside the library instead, of
 * lif_static_scratch_bytes() = 5 MiB, which every GPU the library runs on holds until the process ends.  The call
 * allocates nothing and frees nothing.
 *   limit   256-byte-rounded 4 * batch * capacity_rows  +  4 * 32 * batch * d_model  <=  lif_static_scratch_bytes()
 *           (batch 8 at d_model 4096 fits up to 32768 rows, a single token at any shape); beyond it LIF_INVALID_ARG,
 *           nothing is launched
 *   errors  as lif_sparse_ffn; LIF_HIP_ERROR if the array's address could not be obtained on the layer's device
 * All layers on one GPU share the array: calls that overlap on one GPU (different streams, different layers)
 * race on it; calls on one stream are safe.  Nothing in the array has to be cleared between calls (every value a
 * call reads was written by that call), and its contents after a call are unspecified.
 */
int lif_sparse_ffn_static(lif_layer* layer, const void* x_dev, int32_t batch, void* y_dev, void* stream);

/* Size in bytes of the static scratch array behind lif_sparse_ffn_static. */
size_t lif_static_scratch_bytes(void);

/*
 * One whole step in one call: lif_predict, lif_update_window, lif_load_bundles and
 * lif_sparse_ffn on the same x, with the same arguments, results and error behaviour as the
 * four calls in sequence.  The cache update and the activation stage of the FFN share one
 * launch: the host-link gather keeps few compute units busy, the others compute the
 * activations of the resident rows meanwhile (Section 3.3 items 2 and 3 overlapped).  For
 * batch == 1 the loaders compute the activations of the rows they write, with the same
 * summation order; for fp16 batches a short second pass covers those rows.  y, masks, ids,
 * counts and the cache are bit-identical to the four-call sequence.
 */
int lif_step(lif_layer* layer, const void* x_dev, int32_t batch, void* y_dev, uint8_t* masks_dev,
             uint8_t* step_mask_dev, int32_t* added_dev, int32_t* n_added_dev, int32_t* removed_dev,
             int32_t* n_removed_dev, void* stream);

/*
 * One speculative verification pass in one call (Section 4.3): lif_predict on the n_tokens
 * consecutive tokens of x, lif_update_window_tokens with keep_tokens, lif_load_bundles and
 * lif_sparse_ffn, with the same arguments, results and error behaviour as those four calls in
 * sequence, and the same shared launches as lif_step.
 */
int lif_step_tokens(lif_layer* layer, const void* x_dev, int32_t n_tokens, int32_t keep_tokens, void* y_dev,
                    uint8_t* masks_dev, uint8_t* step_mask_dev, int32_t* added_dev, int32_t* n_added_dev,
                    int32_t* removed_dev, int32_t* n_removed_dev, void* stream);

/*
 * Performance hint: the number of rows the cache
 * typically holds (for example the mean num_used of an earlier run).  lif_sparse_ffn then
 * launches that many waves and lets each request its first row before the device-side row
 * count has arrived.  0 removes the hint.  Results never depend on it.
 */
int lif_set_expected_rows(lif_layer* layer, int32_t rows);

/*
 * Performance knob of lif_step's bundle gather (Section 3.3 item 2): the number of loader wave pairs (one bundle in
 * flight per pair), 1..64; 0 restores the default, which is chosen from the bundle size (256 KiB of reads
 * outstanding, within 5..32 pairs).  Results never depend on it.
 */
int lif_set_loader_pairs(lif_layer* layer, int32_t pairs);

/* Synchronises `stream`, then copies the device-side state / counters to the host. */
int lif_get_state(lif_layer* layer, lif_state* out, void* stream);
int lif_get_counters(lif_layer* layer, lif_counters* out, void* stream);

/*
 * Per-kernel timing with HIP events recorded on the caller's stream around every
 * kernel of the hot calls.  lif_profile_begin(layer, max_launches) creates the events
 * (host objects only) and switches timing on; lif_profile_collect synchronises the
 * stream, adds up elapsed milliseconds and launch counts per enum lif_kernel_id into
 * ms[LIF_K_COUNT] / launches[LIF_K_COUNT], destroys the events and switches timing off.
 * Launches beyond max_launches are not timed.
 */
int lif_profile_begin(lif_layer* layer, int32_t max_launches);
int lif_profile_collect(lif_layer* layer, double* ms, int64_t* launches, void* stream);

/*
 * Bandwidth reference of the box, for the roofline figures of a benchmark (not part of the method): one launch of a
 * plain streaming-read kernel over [src_dev, src_dev + bytes) (16-byte loads, every byte read once, nothing
 * written unless the folded words hit one magic value: sink_dev, 4 bytes of device memory, is then written).
 * bytes = 0 launches an empty kernel (the launch floor).  src_dev 16-byte aligned, bytes a multiple of 16.
 */
int lif_profile_read(const void* src_dev, size_t bytes, void* sink_dev, void* stream);

/*
 * Cost reference of the box for a benchmark (not part of the method): what it costs to hand the results of all
 * workgroups of a kernel to one workgroup of the same launch instead of to a second launch.  One launch of 256
 * workgroups that read 16 KiB each and produce 8 bytes (the shape of the mask kernel of lif_predict).
 *   mode 0  no hand-off (the plain kernel)
 *   mode 1  every workgroup passes a device-scope fence and takes a ticket, the last to arrive reads the 2 KiB back;
 *           no workgroup waits
 *   mode 2  no fences: results go out as 64-bit words carrying `stamp`, by relaxed device-scope atomic stores, and
 *           workgroup 0 polls them with relaxed device-scope atomic loads; the wait is bounded (it gives up after
 *           20000 polls per word and counts that in the 32-bit word at scratch + 256 * 16384 + 4100)
 *   scratch_dev  device memory, 256-byte aligned, lif_profile_handoff_bytes() bytes, zeroed once before the first call;
 *                calls on one scratch must not overlap
 *   stamp        mode 2: a value no earlier launch on this scratch has used (and not 0)
 */
int lif_profile_handoff(void* scratch_dev, int32_t mode, uint32_t stamp, void* stream);
size_t lif_profile_handoff_bytes(void);

/* Message of the last LIF_HIP_ERROR / LIF_INVALID_ARG on the calling thread. */
const char* lif_last_error_string(void);

/* Library version, for the loader check. */
int lif_version(void);

#ifdef __cplusplus
}
#endif
#endif /* LIF_H */
