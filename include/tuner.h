/*
 * tuner.h — C ABI of the MI355X full-space sweep of an ANN performance model.
 *
 * Problem wrapped (paper: Falch & Elster, "Machine Learning Based Auto-tuning
 * for Enhanced OpenCL Performance Portability", Section 5): given the value
 * lists of P tuning parameters (Section 5.1, Table 2), a trained bagged ensemble
 * of small sigmoid networks (Section 5.2) and M, predict the (log) execution
 * time of EVERY configuration of the Cartesian product (Section 5.3, first
 * paragraph) and return the M configurations with the lowest predictions
 * (Section 5.3, third paragraph).  Configurations that are statically known to
 * be invalid (Section 5.2, last paragraph) are masked.
 *
 * Conventions
 *  - Every function returns a status code (TUNER_OK = 0, negative = error),
 *    never throws or aborts; output parameters are untouched on error.
 *    tuner_last_error() gives a thread-local message for the last failure.
 *  - "host" pointers are ordinary CPU memory, read during the call only.
 *    "DEVICE" pointers are GPU memory owned by the caller (for instance a
 *    PyTorch tensor's data_ptr()) on the device that is current at call time.
 *  - The library allocates no device memory: outputs and the workspace are
 *    caller-allocated (tuner_predict_topk_static brings a fixed device array of
 *    its own instead of a workspace).  Work is enqueued on the given HIP stream (a
 *    hipStream_t passed as void*, NULL = default stream) and the functions
 *    return without synchronising; results are ready once the stream is.
 *  - Index order of the Cartesian product: parameter 0 is the most significant
 *    digit, the last parameter varies fastest.  Indices are < 2^32 on the
 *    device; spaces of up to exactly 2^32 configurations are accepted.
 */
#ifndef TUNER_H_
#define TUNER_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct tuner_space tuner_space; /* opaque host object */

enum {
  TUNER_OK = 0,
  TUNER_EINVAL = -1,     /* null pointer, bad size, bad enum, range outside the space */
  TUNER_ETOOLARGE = -2,  /* space > 2^32, too many parameters/values/rules, layer too wide, k too large */
  TUNER_ENOMEM = -3,     /* host allocation failed */
  TUNER_EWORKSPACE = -4, /* workspace missing or smaller than tuner_workspace_bytes() */
  TUNER_EHIP = -5        /* a HIP runtime call failed (message has the HIP error string) */
};

enum { TUNER_SCALE_LINEAR = 0, TUNER_SCALE_LOG2 = 1 };
enum { TUNER_FP32 = 0, TUNER_BF16_MFMA = 1 };
/*
 * How a TUNER_FP32 network is evaluated (all meet the fp32 tolerance of 1e-5):
 *   AUTO     the library's choice (currently MFMA)
 *   MFMA     fp32 matrix instructions, fp32 accumulate
 *   VALU     plain vector-ALU FMAs, one configuration per lane, weights broadcast from LDS
 *   SPLIT16  every operand split into two f16 planes (22 significand bits), three f16
 *            matrix products per fp32 product, fp32 accumulate; weights must satisfy
 *            |w| * 1.4427 < 65504 (f16 range)
 * TUNER_BF16_MFMA precision accepts AUTO or MFMA only.
 */
enum { TUNER_ALGO_AUTO = 0, TUNER_ALGO_MFMA = 1, TUNER_ALGO_VALU = 2, TUNER_ALGO_SPLIT16 = 3 };

/* Limits of this build. */
#define TUNER_MAX_PARAMS 31       /* P */
#define TUNER_MAX_VALUES 254      /* sum of the list lengths */
#define TUNER_MAX_CONSTRAINTS 8
#define TUNER_MAX_CONSTRAINT_ENTRIES 64 /* (rule, parameter) pairs with a non-zero term */
#define TUNER_MAX_TERM_WORDS 192  /* total length of the non-zero term tables */
#define TUNER_MAX_WIDTH 128       /* hidden-layer width */
#define TUNER_MAX_K 16384

/*
 * The ensemble (Section 5.2: k networks, prediction = mean of their outputs;
 * Section 4.2: a neuron is a weighted sum followed by an activation).  Hidden
 * layers use the logistic sigmoid 1/(1+exp(-t)), the single output is linear
 * (it is the predicted log execution time).  Plain data, caller-owned.
 */
typedef struct {
  int32_t n_members;        /* E >= 1 (the paper uses 11) */
  int32_t n_layers;         /* dense layers including the output layer: 2 or 3 */
  const int32_t* widths;    /* host, [n_layers+1] = {P, H1, (H2,) 1} */
  const float* weights_dev; /* DEVICE, fp32, per member and per layer:
                               W[out][in] row-major, then b[out];
                               i.e. W1,b1,(W2,b2,)w_o,b_o ; members back to back */
  int32_t precision;        /* TUNER_FP32, or TUNER_BF16_MFMA: features, weights and hidden
                               activations rounded to bf16 (nearest even) before each matrix
                               product, fp32 accumulate; biases, sigmoid, output layer and mean
                               in fp32 (tolerance 1e-2) */
  int32_t algo;             /* TUNER_ALGO_* */
} tuner_model;

/*
 * Builds the space object (host only; copies every array, so the caller may
 * free its arrays on return).
 *   n_params          P, 1..TUNER_MAX_PARAMS
 *   radices[P]        length of each parameter's value list (>= 1)
 *   values[sum r]     host, the lists concatenated (Table 2 style)
 *   scales[P]         TUNER_SCALE_LINEAR: feature = value; TUNER_SCALE_LOG2:
 *                     feature = log2(value) (values must be > 0); either way
 *                     min-max normalised to [0,1] over the list, computed in
 *                     double and rounded once to fp32 (a constant list -> 0)
 *   n_constraints     C, 0..TUNER_MAX_CONSTRAINTS
 *   constraint_terms  host, [C][sum r] integer terms T_c, same order as values
 *   constraint_bounds host, [C]; configuration with digits d is valid iff for
 *                     every c: sum_p T_c[offset_p + d_p] <= bound_c
 * Errors: EINVAL (null, radix < 1, bad scale, log2 of a value <= 0, non-finite
 * value, sum of |terms| not representable in int32), ETOOLARGE (limits above,
 * or more than 2^32 configurations), ENOMEM.
 */
int tuner_space_create(int32_t n_params, const int32_t* radices, const double* values,
                       const int32_t* scales, int32_t n_constraints,
                       const int32_t* constraint_terms, const int64_t* constraint_bounds,
                       tuner_space** out);
void tuner_space_destroy(tuner_space* space);

/* Number of configurations N = product of the radices (Section 5.1). */
int tuner_space_size(const tuner_space* space, uint64_t* n_configs);

/*
 * Host helpers for one configuration.  decode: index -> digits[P], and (if
 * non-null) values[P] (the parameter values), features[P] (fp32 network
 * inputs) and *valid (0/1).  encode: digits[P] -> index.  EINVAL if the index
 * or a digit is out of range.
 */
int tuner_space_decode(const tuner_space* space, uint64_t index, int32_t* digits,
                       double* values, float* features, int32_t* valid);
int tuner_space_encode(const tuner_space* space, const int32_t* digits, uint64_t* index);

/*
 * Host check of the device decoder's arithmetic: evaluates, on the CPU, the
 * very routine the kernels use (multiply-shift division constants, validity
 * sums in 32 bits).  Used by the CPU tests; same outputs as tuner_space_decode
 * minus the values.
 */
int tuner_space_decode_device_arith(const tuner_space* space, uint64_t index, int32_t* digits,
                                    float* features, int32_t* valid);

/*
 * Bytes of DEVICE workspace needed by tuner_predict_topk / tuner_predict_all
 * for this model and k (k may be 0 for predict_all).  Returns 0 on invalid
 * arguments (see tuner_last_error).  Does not depend on the index range.
 */
size_t tuner_workspace_bytes(const tuner_space* space, const tuner_model* model, int32_t k);

/*
 * How a range sweep of this model over this space evaluates layer 1 (host only).
 * Consecutive configurations share all but their last few parameter values (the space
 * is a Cartesian product, Section 5.1): the parameters whose stride is a multiple of 32
 * have one value per tile of 32 configurations, and the fp32 matrix network computes
 * their share of the layer-1 pre-activations once per tile instead of once per
 * configuration.  *n_hoisted receives the number of such parameters this library
 * treats that way (0: none; always 0 for the other network evaluations and for
 * tuner_predict_indices).
 */
int tuner_hoisted_parameters(const tuner_space* space, const tuner_model* model, int32_t* n_hoisted);

/*
 * Companion of tuner_hoisted_parameters (host only).  When the remaining parameters
 * (stride < 32) span exactly 32 configurations, configuration c of every tile has the
 * same values for them (Section 5.1: Cartesian product, last parameter fastest), and
 * their share of the layer-1 pre-activations is a [units][32] table per member, built
 * when the weights are packed, instead of matrix work per configuration.  The library
 * does this when the larger packed members still fit the 160 KB of LDS either all at
 * once or as two stage buffers.  *n_tabulated receives the number of parameters served
 * from the table (0: none).
 */
int tuner_tabulated_parameters(const tuner_space* space, const tuner_model* model, int32_t* n_tabulated);

/*
 * What a sweep of this range would launch (host only; nothing is enqueued).  The
 * library cuts the range into tiles of consecutive configurations (Section 5.1:
 * the space is a Cartesian product, so consecutive indices share their leading
 * parameter values), tiles into chunks (waves x tiles_per_wave x tile
 * configurations, one chunk per workgroup at a time) and chunks into units of a
 * work queue; short ranges get smaller chunks so that every compute unit has work.
 * Uses the current device's compute-unit count and LDS size, or MI355X's when the
 * process has no GPU.  k = 0 asks about tuner_predict_all, k >= 1 about
 * tuner_predict_topk.  Errors as for those calls, minus the workspace.
 */
typedef struct {
  int32_t network;                /* 0 fp32 matrix, 1 bf16 matrix, 2 two-plane f16 matrix, 3 vector ALU */
  int32_t layer1;                 /* 0 plain; 1 tile-constant parameters once per tile; 2 also the rest from a table */
  int32_t waves;                  /* waves per workgroup */
  int32_t tile;                   /* configurations per tile */
  int32_t variant_tiles_per_wave; /* tiles per wave and chunk the kernel is built for */
  int32_t tiles_per_wave;         /* ... and the number this range uses */
  int32_t workgroups;
  uint32_t n_chunks;
  int32_t chunks_per_unit;
  uint32_t n_units;
  int32_t dynamic_queue;          /* units beyond a workgroup's first come from an atomic counter */
  int32_t live_chunk_list;        /* a classification pass lists the chunks with a valid configuration */
  int32_t members_per_stage;      /* networks held in LDS at a time */
  int32_t n_stages;
  int32_t double_buffer;          /* the next stage loads while the current one is evaluated */
  int32_t pool_in_lds;            /* the workgroup's candidate pool lives in LDS */
  int32_t lds_bytes;              /* dynamic LDS of the sweep kernel */
  int32_t merge_launches;         /* kernels after the sweep (top-k, merge = 0; the running result
                                     of a merging call is one more list and can add a launch) */
  size_t workspace_bytes;         /* workspace the call itself needs (<= tuner_workspace_bytes) */
} tuner_sweep_plan_info;
int tuner_sweep_plan(const tuner_space* space, const tuner_model* model, uint64_t index_begin,
                     uint64_t index_count, int32_t k, tuner_sweep_plan_info* out);

/*
 * Sweep of indices [index_begin, index_begin + index_count) and selection of
 * the k valid configurations with the smallest predictions, ordered by
 * (prediction, then index), ascending (Section 5.3).
 *   merge_with_existing  0: the outputs are overwritten.  1: the outputs hold
 *                        the running result of earlier calls (values, indices
 *                        and *n_found as this function wrote them, same k) and
 *                        are replaced by the top-k of the union; used to stream
 *                        a large space chunk by chunk, in any chunk order.  The
 *                        ranges of the merged calls must not overlap (a
 *                        configuration swept twice would be listed twice).
 *   topk_values_dev      DEVICE, k floats
 *   topk_indices_dev     DEVICE, k uint32
 *   n_found_dev          DEVICE, one int32 = min(k, number of valid
 *                        configurations seen so far); entries past it are
 *                        (+INF, 0xFFFFFFFF)
 *   workspace_dev        DEVICE, >= tuner_workspace_bytes(), 256-byte aligned;
 *                        contents need not be preserved between calls
 * index_count may be 0 (the result is then the existing one, or empty).
 * Calls that share a workspace must be ordered on one stream.
 * Errors: EINVAL (null, k < 1, range outside the space, model/space mismatch,
 * unsupported precision), ETOOLARGE (k > TUNER_MAX_K, width > TUNER_MAX_WIDTH),
 * EWORKSPACE, EHIP.
 */
int tuner_predict_topk(const tuner_space* space, const tuner_model* model,
                       uint64_t index_begin, uint64_t index_count, int32_t k,
                       int32_t merge_with_existing, float* topk_values_dev,
                       uint32_t* topk_indices_dev, int32_t* n_found_dev, void* workspace_dev,
                       size_t workspace_bytes, void* hip_stream);

/*
 * Sweeps of one model over one space, call after call (the chunks of a streamed
 * space, the repeated sweeps of a tuning session): what every call would derive
 * again from the same inputs is made once.  tuner_prepare writes the sweep's
 * header, the space's decoder tables (Section 5.1) and the ensemble's weights in
 * the operand order of the kernels (Section 5.2) into the workspace;
 * tuner_predict_topk_prepared and tuner_predict_all_prepared are
 * tuner_predict_topk and tuner_predict_all without that step (one kernel fewer
 * per call; the same results, bit for bit).
 *   - The workspace must be the one tuner_prepare wrote, for the same space and
 *     model (same widths, precision, algo and weights), of at least
 *     tuner_workspace_bytes(space, model, k) bytes for the largest k used.
 *   - Between prepared calls its contents must be left alone; calls are ordered
 *     on one stream.  tuner_predict_topk, tuner_predict_all and
 *     tuner_predict_indices on the same workspace write their own preparation
 *     over it: prepare again after them, after a failed call, and whenever the
 *     weights change.
 *   - model->weights_dev is not read by the prepared calls.
 * Errors as for the calls they replace.
 */
int tuner_prepare(const tuner_space* space, const tuner_model* model, void* workspace_dev,
                  size_t workspace_bytes, void* hip_stream);
int tuner_predict_topk_prepared(const tuner_space* space, const tuner_model* model,
                                uint64_t index_begin, uint64_t index_count, int32_t k,
                                int32_t merge_with_existing, float* topk_values_dev,
                                uint32_t* topk_indices_dev, int32_t* n_found_dev,
                                void* workspace_dev, size_t workspace_bytes, void* hip_stream);
int tuner_predict_all_prepared(const tuner_space* space, const tuner_model* model,
                               uint64_t index_begin, uint64_t index_count, float* predictions_dev,
                               uint8_t* valid_mask_dev, void* workspace_dev, size_t workspace_bytes,
                               void* hip_stream);

/*
 * tuner_predict_topk for callers that cannot allocate device memory or bring a
 * workspace: code under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc.  Same arguments, results and errors as tuner_predict_topk
 * minus the workspace: its place is taken by a device array of
 * TUNER_STATIC_SCRATCH_BYTES that lives in the library (each GPU the library is
 * used on holds one copy until the process ends).  The call allocates nothing,
 * on the host side of the GPU or on the device.
 *   - A space, model and k whose tuner_workspace_bytes() exceeds
 *     TUNER_STATIC_SCRATCH_BYTES is refused with TUNER_ETOOLARGE (the message
 *     gives both sizes); the five benchmark configurations fit.
 *   - Every call on a GPU uses that GPU's one array: calls that may run at the
 *     same time on one GPU (different streams, different threads) race.  Calls
 *     ordered on one stream are safe; nothing needs to be cleared between them.
 *   - It is not timed by tuner_profile_enable (timing creates HIP events).
 */
#define TUNER_STATIC_SCRATCH_BYTES (64u << 20)
int tuner_predict_topk_static(const tuner_space* space, const tuner_model* model,
                              uint64_t index_begin, uint64_t index_count, int32_t k,
                              int32_t merge_with_existing, float* topk_values_dev,
                              uint32_t* topk_indices_dev, int32_t* n_found_dev, void* hip_stream);

/*
 * Sweep of the range writing every prediction (Section 5.3, first paragraph).
 *   predictions_dev  DEVICE, index_count floats; +INF where invalid
 *   valid_mask_dev   DEVICE, optional (NULL to skip), index_count bytes 0/1
 */
int tuner_predict_all(const tuner_space* space, const tuner_model* model, uint64_t index_begin,
                      uint64_t index_count, float* predictions_dev, uint8_t* valid_mask_dev,
                      void* workspace_dev, size_t workspace_bytes, void* hip_stream);

/*
 * Decoder output for a range, for checking steps one by one: digits
 * (DEVICE, [index_count][P] int32, optional), features (DEVICE,
 * [index_count][P] fp32, optional) and validity (DEVICE, index_count bytes,
 * optional), produced by the same device routine the sweep uses.
 */
int tuner_decode_range(const tuner_space* space, uint64_t index_begin, uint64_t index_count,
                       int32_t* digits_dev, float* features_dev, uint8_t* valid_mask_dev,
                       void* hip_stream);

/*
 * Ensemble evaluation at an arbitrary list of configurations (the held-out
 * configurations of Section 6, first paragraph; the training samples of
 * Section 5.2): the same network evaluation as tuner_predict_all, with
 * configuration indices read from a list instead of a range.  A range sweep
 * may compute layer 1 in a different order (see tuner_hoisted_parameters and
 * tuner_tabulated_parameters), so for the same configuration the two agree
 * within the fp32 tolerance (a few 1e-7 relative), not bit for bit; each of
 * them is repeatable bit for bit.
 *   indices_dev      DEVICE, n uint32 configuration indices (each < N; an index
 *                    outside the space is not detected)
 *   predictions_dev  DEVICE, n floats; +INF where the configuration is invalid
 *   valid_mask_dev   DEVICE, optional, n bytes 0/1
 * Workspace as for tuner_predict_all (tuner_workspace_bytes with k = 0).
 */
int tuner_predict_indices(const tuner_space* space, const tuner_model* model, uint64_t n,
                          const uint32_t* indices_dev, float* predictions_dev,
                          uint8_t* valid_mask_dev, void* workspace_dev, size_t workspace_bytes,
                          void* hip_stream);

/*
 * Random choice of training configurations (Section 5.2: the benchmarks are
 * run "on several randomly chosen parameter configurations"; invalid ones are
 * ignored).  Draw c = 0, 1, 2, ... is the configuration index
 *     floor(z_c * N / 2^64),  z_c = splitmix64 output function of seed + (c + 1) * 0x9E3779B97F4A7C15
 * and the sample is the first n_samples DISTINCT, statically VALID indices in
 * draw order among draws 0 .. max_draws - 1 (sampling without replacement).
 *   indices_dev   DEVICE out, n_samples uint32 (entries past *n_found_dev are 0xFFFFFFFF)
 *   n_found_dev   DEVICE out, one int32 = number of indices written (< n_samples
 *                 only if max_draws draws did not yield enough)
 *   workspace     DEVICE, >= tuner_sample_workspace_bytes(max_draws), 256-byte aligned
 * Errors: EINVAL (null, n_samples < 1, max_draws < n_samples), ETOOLARGE
 * (max_draws > 2^24), EWORKSPACE, EHIP.
 */
size_t tuner_sample_workspace_bytes(uint64_t max_draws);
int tuner_sample_valid(const tuner_space* space, uint64_t seed, uint32_t n_samples,
                       uint64_t max_draws, uint32_t* indices_dev, int32_t* n_found_dev,
                       void* workspace_dev, size_t workspace_bytes, void* hip_stream);

/*
 * Training of the bagged ensemble (Section 5.2): E networks P -> hidden -> 1
 * (sigmoid hidden units, linear output); the training data is split into E
 * parts and network e is trained on all the data except part e; the target is
 * the natural logarithm of the measured execution time and the loss of network
 * e is the mean squared error over its training samples,
 *     L_e = 1/n_e * sum_s (y_e(x_s) - ln t_s)^2.
 * The paper names no training algorithm; this library uses full-batch gradient
 * descent with momentum from caller-supplied initial weights:
 *     v <- momentum * v - learning_rate * dL_e/dw,   w <- w + v,   v_0 = 0,
 * for a fixed number of epochs, in fp32.  A sample is ignored (Section 5.2,
 * last paragraph) when its configuration is statically invalid or its time is
 * not a finite number > 0 (a failed run).
 *   sample_indices_dev   DEVICE, n_samples uint32 configuration indices
 *   sample_times_dev     DEVICE, n_samples floats, measured execution times
 *   sample_parts_dev     DEVICE, n_samples int32; network e skips samples with part == e
 *   initial_weights_dev  DEVICE, E x (hidden * P + hidden + hidden + 1) floats, layout of
 *                        tuner_model.weights_dev (W1[hidden][P], b1, w_o, b_o per network)
 *   weights_out_dev      DEVICE out, same size (may alias initial_weights_dev)
 *   loss_history_dev     DEVICE out, optional, [E][epochs + 1] floats: L_e before each
 *                        update, and last the loss of the final weights
 * A network with no usable training sample keeps its initial weights (loss 0).
 * All workgroups of the launch (n_members x workgroups_per_network, at most 256)
 * must be able to run at the same time; on a GPU busy with other work a run may
 * give up (see barrier_poll_limit), which shows as NaN weights.
 * Limits: 1 <= hidden <= 64, n_samples <= 2^24, epochs >= 0.
 * Workspace: >= tuner_train_workspace_bytes(space, n_samples), 256-byte aligned.
 */
typedef struct {
  int32_t epochs;
  float learning_rate;
  float momentum;
  int32_t workgroups_per_network; /* 0: the library's choice; 1..16: each network's samples are
                                     split over this many workgroups, which add their partial
                                     gradient sums once per epoch (the result depends on it only
                                     through the order of fp32 additions) */
  int32_t barrier_poll_limit;     /* 0: default (2^22).  The workgroups of a network meet at a
                                     barrier once per epoch; one that has polled this many times
                                     without seeing the others gives up, the whole run stops, and
                                     every network that did not finish returns NaN weights and
                                     NaN losses (never a partial result) */
} tuner_train_options;

size_t tuner_train_workspace_bytes(const tuner_space* space, uint64_t n_samples);
int tuner_train_ensemble(const tuner_space* space, int32_t n_members, int32_t hidden,
                         uint64_t n_samples, const uint32_t* sample_indices_dev,
                         const float* sample_times_dev, const int32_t* sample_parts_dev,
                         const float* initial_weights_dev, const tuner_train_options* options,
                         float* weights_out_dev, float* loss_history_dev, void* workspace_dev,
                         size_t workspace_bytes, void* hip_stream);

/*
 * Model accuracy as the paper reports it (Section 6, first paragraph): the mean
 * relative error |exp(prediction) - t| / t over configurations that were not
 * used for training, invalid configurations and failed runs (time not a finite
 * number > 0) left out.  Predictions are log-times (natural logarithm).
 *   predictions_dev  DEVICE, n floats (as written by tuner_predict_indices)
 *   times_dev        DEVICE, n floats, measured times
 *   mean_error_dev   DEVICE out, one float (0 if no configuration counts)
 *   n_used_dev       DEVICE out, one int32
 */
int tuner_mean_relative_error(uint64_t n, const float* predictions_dev, const float* times_dev,
                              float* mean_error_dev, int32_t* n_used_dev, void* hip_stream);

/*
 * Second stage of the tuner (Section 5.3, third paragraph): among the M
 * candidates whose execution times were measured, the one with the lowest
 * time; ties go to the earlier entry; failed runs (time not a finite number
 * > 0) are skipped.
 *   best_pos_dev   DEVICE out, one int32: position in the list, -1 if every
 *                  candidate failed (the tuner then returns nothing)
 *   best_time_dev  DEVICE out, one float (+INF if none)
 */
int tuner_best_of(uint64_t m, const float* times_dev, int32_t* best_pos_dev, float* best_time_dev,
                  void* hip_stream);

/*
 * Timing of the dominant kernels (the fused sweep of Section 5.3; the training
 * kernel of Section 5.2) for roofline reports.  While enabled, every predict
 * call brackets its sweep kernel, and every tuner_train_ensemble call its
 * training kernel, with a pair of HIP events on the caller's stream.
 * tuner_profile_read / tuner_profile_read_train wait for the recorded events of
 * their kind, return the summed kernel time in milliseconds and the number of
 * launches, and forget them.  tuner_profile_enable(0) drops whatever was recorded
 * and not read.  Process-wide, not thread-safe; off by default.
 */
int tuner_profile_enable(int32_t on);
int64_t tuner_profile_pending(void);   /* recorded launches not yet read (of both kinds) */
int tuner_profile_read(double* sweep_ms_total, int64_t* n_sweep_launches);
int tuner_profile_read_train(double* train_ms_total, int64_t* n_train_launches);

/* Message for the last error on this thread; valid until the next call. */
const char* tuner_last_error(void);

/* Library version string. */
const char* tuner_version(void);

#ifdef __cplusplus
}
#endif
#endif /* TUNER_H_ */
