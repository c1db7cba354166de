/*
 * dbsn.h — C ABI of libdbsn: on-line (batch size 1) back-propagation through big plain
 * multi-layer perceptrons and on-the-fly elastic + affine deformation of 28x28 images,
 * hand-written for AMD MI355X (gfx950).
 *
 * Method: Ciresan, Meier, Gambardella, Schmidhuber, "Deep Big Simple Neural Nets Excel on
 * Handwritten Digit Recognition" (sections and appendix parts are cited per call below).
 *
 * Conventions
 *  - Every function returns int32_t: DBSN_OK (0) or a negative DBSN_E_* code; nothing throws or
 *    aborts.  dbsn_last_error() gives a thread-local message for the last failing call.
 *    On an argument error no device work is issued.
 *  - Pointers named *_dev are DEVICE pointers, *_host are HOST pointers.  All device memory is
 *    allocated and owned by the caller; the library allocates no device memory and never frees
 *    caller memory.  Device pointers must be 16-byte aligned unless stated otherwise.
 *  - `hip_stream` is a hipStream_t passed as void* (NULL = the default stream).  A network keeps
 *    the stream it was initialised with; all its calls are asynchronous on that stream except
 *    the dbsn_mlp_get_* / dbsn_mlp_status calls, which synchronise it.
 *  - A network handle must not be used from two host threads at once.
 *  - Arithmetic is IEEE binary32 throughout (the paper's nets are single precision).
 */
#ifndef DBSN_H
#define DBSN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define DBSN_OK          0
#define DBSN_E_ARG      -1   /* null pointer, negative count, label or layer out of range, ...      */
#define DBSN_E_SHAPE    -2   /* unsupported shape, misaligned pointer, arena too small               */
#define DBSN_E_HIP      -3   /* a HIP runtime call failed                                            */
#define DBSN_E_TIMEOUT  -4   /* a wait inside the persistent kernel gave up (reported by _status)   */

#define DBSN_MAX_LAYERS  16     /* weight layers (n_sizes - 1)                                        */
#define DBSN_MAX_WIDTH   4096   /* neurons in any layer, inputs included                              */
#define DBSN_MAX_CLASSES 64     /* neurons in the output layer                                        */
#define DBSN_MAX_KTAPS   63     /* taps of the 1-D Gaussian                                           */
#define DBSN_STATIC_SCRATCH_BYTES (64u << 20)   /* device memory dbsn_classify_static stages through  */
#define DBSN_IMG_SIDE    28
#define DBSN_IMG_PIXELS  784

typedef struct dbsn_mlp dbsn_mlp;   /* opaque host handle */

/* Deformation parameters (section "Deforming images to get more training instances"):
 * sigma, alpha: Gaussian width (pixels) and scale of the elastic displacement field;
 * beta_deg: an angle is drawn uniformly from [-beta, +beta] degrees per image; it is a rotation,
 * or, when shear != 0, a horizontal shear whose tangent is the ratio of horizontal displacement
 * to image height;
 * gamma_pct: x and y scale factors drawn independently from [1-gamma/100, 1+gamma/100];
 * ktaps: odd number of taps of the 1-D Gaussian (the appendix uses a 21 x 21 kernel). */
typedef struct {
    float   sigma;
    float   alpha;
    float   beta_deg;
    float   gamma_pct;
    int32_t ktaps;
    int32_t shear;
    int32_t kernel;   /* DBSN_DEFORM_KERNEL_*: which of two kernels with bit-identical results runs */
} dbsn_deform_params;

/* AUTO: the kernel specialised for the paper's 21 taps when ktaps == 21, the general one otherwise.
 * GENERAL: the general kernel whatever ktaps is (for comparing the two). */
#define DBSN_DEFORM_KERNEL_AUTO    0
#define DBSN_DEFORM_KERNEL_GENERAL 1

/* Execution mode of dbsn_bp_steps / dbsn_bp_step.  0: one kernel launch per layer phase;
 * 1 (default): one persistent kernel per call, whose workgroups hand partial sums to each other
 * through tagged words in device memory.  Both compute the same step; they add partial sums in
 * different (each fixed) orders, so results agree to rounding, and each mode is bit-reproducible
 * from run to run.  Shapes the persistent kernel does not hold (no hidden layer; an output layer of
 * more than 16384 weights, counting its classes rounded up to a multiple of 4, or of more than 2048
 * inputs; a layer whose 256 tiles would exceed 224 rows each) run in mode 0 whatever is selected,
 * and so does every shape on a device with fewer than 256 compute units, which cannot hold the
 * persistent kernel's 256 workgroups at once. */
#define DBSN_MODE_LAUNCHES   0
#define DBSN_MODE_PERSISTENT 1

/* Bytes of device memory a network of the given layer sizes needs (weights, biases, activations,
 * deltas, partial sums, flags).  sizes[0] = inputs, sizes[n_sizes-1] = classes.  Returns 0 for an
 * unsupported shape (n_sizes < 2 or > DBSN_MAX_LAYERS+1, a size < 1 or > DBSN_MAX_WIDTH, more than
 * DBSN_MAX_CLASSES outputs).  Host-only; touches no device. */
size_t dbsn_mlp_arena_bytes(const int32_t* sizes_host, int32_t n_sizes);

/* Create a network in the caller's arena (arena_dev: device, 256-byte aligned, at least
 * dbsn_mlp_arena_bytes() long, owned by the caller and kept alive until dbsn_mlp_free) and fill
 * it (section "Architectures"): every weight and bias uniform in [-0.05, 0.05), drawn from the
 * library's counter generator so that the result depends on `seed` alone.  The bias is the weight
 * of a constant-1 input, as in the appendix's kernels.  *out receives the handle.  The first call
 * on a device also runs a short probe kernel and waits for it (is the chip eight dies of 32 compute
 * units, see dbsn_mlp_set_variant); later calls only enqueue work on hip_stream. */
int32_t dbsn_mlp_init(dbsn_mlp** out, const int32_t* sizes_host, int32_t n_sizes, uint64_t seed,
                      void* arena_dev, size_t arena_bytes, void* hip_stream);

/* Frees the host handle only (after synchronising its stream). */
int32_t dbsn_mlp_free(dbsn_mlp* mlp);

/* Copy layer `layer` (1 .. L) from / to dense host arrays: W_host[n_l][n_{l-1}] row-major,
 * b_host[n_l].  Either pointer may be NULL to skip that part.  Both synchronise the stream. */
int32_t dbsn_mlp_set_weights(dbsn_mlp* mlp, int32_t layer, const float* W_host, const float* b_host);
int32_t dbsn_mlp_get_weights(dbsn_mlp* mlp, int32_t layer, float* W_host, float* b_host);

/* State left by the last dbsn_bp_step / dbsn_forward, for inspection: x_host[n_l] = outputs of
 * layer `layer` (1 .. L-1: scaled-tanh activations; L: softmax probabilities); d_host[n_l] =
 * deltas of layer `layer` (1 .. L) of the last bp step (dbsn_forward leaves them alone).
 * Synchronise the stream. */
int32_t dbsn_mlp_get_activations(dbsn_mlp* mlp, int32_t layer, float* x_host);
int32_t dbsn_mlp_get_deltas(dbsn_mlp* mlp, int32_t layer, float* d_host);

/* Select DBSN_MODE_*.  */
int32_t dbsn_mlp_set_mode(dbsn_mlp* mlp, int32_t mode);

/* How the persistent kernel is launched.  Its 256 workgroups wait for each other, so all of them
 * must get onto the chip while none can finish: a COOPERATIVE launch (default) has the driver see to
 * that against everything else on the device, at about 18 us per call; a PLAIN launch leaves it to
 * the situation: kernels that end by themselves only delay it, and the library keeps the training
 * kernels of this process apart (a call on another stream than the last one first waits for that
 * one's kernel), so what remains is another PROCESS training with this library on the same device
 * at the same time: two such kernels can hold each other's compute units until their waits give up
 * (reported by dbsn_mlp_status as DBSN_E_TIMEOUT, weights undefined).  Choose PLAIN when the device
 * is this process's own and calls are short (dbsn_bp_step: 54 instead of 72 us on the 12 M-weight
 * net, 15 instead of 33 us on 784-300-10); results are the same bit for bit.  No device work. */
#define DBSN_LAUNCH_COOPERATIVE 0
#define DBSN_LAUNCH_PLAIN       1
int32_t dbsn_mlp_set_launch(dbsn_mlp* mlp, int32_t kind);

/* Polls a workgroup of the persistent kernel may spend waiting for one set of partial sums before
 * it gives up (default 2^22, seconds of waiting).  Exists so that the time-out path can be
 * exercised from the host. */
int32_t dbsn_mlp_set_spin_limit(dbsn_mlp* mlp, uint32_t polls);

/* The pauses of the persistent kernel (see dbsn_mlp_autotune), in units of 64 shader clocks, 0 .. 48:
 * fwd_host[l-1] for the forward phase of layer l = 1 .. L (L: the output phase), bwd_host[l-1] for
 * the backward phase of layer l; either pointer may be NULL to leave / skip that direction.  Speed
 * only: results never depend on them.  Defaults: 17 forward, 0 backward. */
int32_t dbsn_mlp_set_pauses(dbsn_mlp* mlp, const int32_t* fwd_host, const int32_t* bwd_host);
int32_t dbsn_mlp_get_pauses(dbsn_mlp* mlp, int32_t* fwd_host, int32_t* bwd_host);

/* Variant of the persistent kernel, for measurements and tests (the default, chosen at
 * dbsn_mlp_init, is the fastest the network and the device allow).  stationary = 1: the weights of
 * the hidden layers stay in registers for the whole call when they all fit (58 MB; else as 0); 0:
 * every phase loads its tile from memory and the backward phase stores it back.  fixed_layout = 1:
 * networks that fit one of the compiled register layouts use it; 0: registers packed at run time.
 * banded = 1: where two hidden layers follow each other, the neurons between them are split into
 * eight bands, one per die of the chip, so that the partial sums those two layers exchange never
 * leave a die (used when the device is eight dies of 32 compute units, which dbsn_mlp_init probes,
 * and the banded tiles fit the registers; the workgroups of a launch number themselves by the die
 * they find themselves on, so nothing is assumed about where the hardware puts them); 0: every
 * layer cut the same way, all hand-overs across the chip.  stationary and fixed_layout do not change the order of any sum: those variants agree
 * to rounding (they are separately compiled kernels); banded changes how partial sums are grouped,
 * like DBSN_MODE_LAUNCHES does.  Synchronises the stream.
 * dbsn_mlp_get_variant reports what is in force: stationary (0/1), the register layout (0: packed
 * at run time) and the number of banded pairs of layers (0: the plain cut); pointers may be NULL. */
int32_t dbsn_mlp_set_variant(dbsn_mlp* mlp, int32_t stationary, int32_t fixed_layout, int32_t banded);
int32_t dbsn_mlp_get_variant(dbsn_mlp* mlp, int32_t* stationary, int32_t* layout, int32_t* banded_pairs);

/* Optional tuning of the persistent kernel for this network on this device.  Between the phases
 * of a step a workgroup pauses before it first looks for the partial sums of the phase before (a
 * look that comes too early costs a round trip through memory, one that comes late costs the
 * delay); the best pauses depend on the layer sizes and on the machine.  This call finds them by
 * timing launches of min(n, 512) steps over the given samples with eta = 0, which leave every
 * weight as it was, bit for bit (w - 0 * delta * x = w), and keeps them for all later calls.
 * Results never depend on the pauses, only speed does.  samples_dev: [n][sizes[0]] float,
 * labels_dev: [n] int32, device memory, n >= 64.  Takes a second or two and synchronises the
 * network's stream; a no-op in DBSN_MODE_LAUNCHES.  Not part of the paper's method: for callers
 * that want the last few per cent. */
int32_t dbsn_mlp_autotune(dbsn_mlp* mlp, const float* samples_dev, const int32_t* labels_dev, int64_t n);

/* Synchronise the network's stream and report deferred errors: DBSN_E_TIMEOUT if a wait inside a
 * persistent kernel gave up (the weights are then undefined), DBSN_E_HIP for a failed launch. */
int32_t dbsn_mlp_status(dbsn_mlp* mlp);

/* Deform n images (section "Deforming images ...", appendix "Deformations"): for image k, all
 * random numbers are a function of (seed, first_index + k) only, so splitting a set into chunks
 * does not change the result.  Per image: rotation angle and two scale factors; two displacement
 * fields uniform in [-1,1) per pixel, each smoothed with the separable ktaps-tap Gaussian of
 * width sigma (taps sum to 1, field taken as zero outside the image) and multiplied by alpha;
 * output pixel (r,c) is the bilinear sample of the source at the rotated (or sheared) and scaled
 * position of (r,c) about the image centre plus the displacement at (r,c), pixels outside the source counting
 * as 0; the result is mapped to intensity/127.5 - 1 (section "Data").
 * src_dev: [n][784] uint8 (any alignment); dst_dev: [n][784] float.  n == 0 is a no-op. */
int32_t dbsn_deform_batch(const dbsn_deform_params* params_host, const uint8_t* src_dev, int64_t n,
                          uint64_t seed, uint64_t first_index, float* dst_dev, void* hip_stream);

/* The same with one bound of the angle per image, beta_deg_dev: [n] float (degrees, finite), which
 * replaces params->beta_deg: the paper rotates or shears digits 1 and 7 by at most 7.5 degrees
 * and the others by at most 15 (section "Deforming images ..."), so the bound follows the label. */
int32_t dbsn_deform_batch_beta(const dbsn_deform_params* params_host, const uint8_t* src_dev,
                               const float* beta_deg_dev, int64_t n, uint64_t seed, uint64_t first_index,
                               float* dst_dev, void* hip_stream);

/* The same with the bound of the angle following the class label of each image (section
 * "Deforming images ..."): look-alike classes are rotated or sheared less than the others; the
 * paper uses 7.5 degrees for the digits 1 and 7 and 15 degrees otherwise.  labels_dev: [n] int32
 * (device); an image whose class c (0 .. 63) has bit c set in similar_mask takes
 * beta_similar_deg, every other image (any other label included) params->beta_deg.
 * The paper's rule: similar_mask = (1 << 1) | (1 << 7), beta_similar_deg = 7.5, beta_deg = 15. */
int32_t dbsn_deform_batch_labels(const dbsn_deform_params* params_host, const uint8_t* src_dev,
                                 const int32_t* labels_dev, uint64_t similar_mask, float beta_similar_deg,
                                 int64_t n, uint64_t seed, uint64_t first_index, float* dst_dev,
                                 void* hip_stream);

/* n on-line back-propagation steps, strictly in order (sections "Architectures", "Training
 * algorithm"; appendix "Forward propagation", "Backward propagation", "Weight updating"): for
 * each sample, forward through scaled-tanh hidden layers y = 1.7159 tanh(0.6666 a) and a softmax
 * output, output delta p - onehot(label), deltas back-propagated through the weights as they were
 * before the step, then every weight w_ji -= eta * delta_j * x_i (no momentum, batch size 1).
 * samples_dev: [n][sizes[0]] float; labels_dev: [n] int32 in 0 .. classes-1 (device memory; an
 * out-of-range label is clamped into range by the kernel); loss_dev: [n] float receiving
 * -log p_label per step, or NULL.  n == 0 is a no-op. */
int32_t dbsn_bp_steps(dbsn_mlp* mlp, const float* samples_dev, const int32_t* labels_dev, int64_t n,
                      float eta, float* loss_dev);

/* One step on one sample with a host-side label: dbsn_bp_steps with n = 1.  (A call of the
 * persistent kernel brings the weights into registers at its start and writes them back at its
 * end, tens of microseconds on the big nets: train through dbsn_bp_steps with as many samples per
 * call as are at hand, one by one only where a sample depends on the step before.) */
int32_t dbsn_bp_step(dbsn_mlp* mlp, const float* sample_dev, int32_t label, float eta);

/* Forward propagation of one sample; probs_dev: [classes] float softmax outputs. */
int32_t dbsn_forward(dbsn_mlp* mlp, const float* sample_dev, float* probs_dev);

/* Forward-only classification of n samples: labels_out_dev[s] = index of the largest output
 * (lowest index on ties), as used for validation and test passes (sections "Data", "Results").
 * samples_dev: [n][sizes[0]] float, labels_out_dev: [n] int32, both device memory, 4-byte aligned.
 * The samples go through the layers 16384 at a time as dense products on the fp32 matrix units:
 * products and sums in binary32 like dbsn_forward, in another order, so the two agree wherever the
 * two largest outputs differ by more than rounding.  Fastest when sizes[0] is a multiple of 4 and
 * samples_dev is 16-byte aligned (other shapes take a slower kernel, same results).  Asynchronous
 * on the network's stream; n == 0 is a no-op. */
int32_t dbsn_classify(dbsn_mlp* mlp, const float* samples_dev, int64_t n, int32_t* labels_out_dev);

/* dbsn_classify for callers that cannot allocate device memory or must not see a memset: code
 * that records the stream into a HIP graph, tight serving loops, harnesses that forbid hipMalloc.
 * Same kernels and same labels as dbsn_classify, but the activations of the pass are staged in a
 * static device array of DBSN_STATIC_SCRATCH_BYTES inside the library (one copy per GPU, held
 * until the process ends) instead of the arena's buffers, all n samples in ONE pass: the call makes
 * no hipMalloc / hipFree / memset and no allocating library call.  Limit: 2 * n * 4 * w bytes must
 * fit the array, w = the widest layer after the input rounded up to a multiple of 4 (3355 samples
 * for a 2500-wide net, 8388 for a 1000-wide one); a larger n is rejected with DBSN_E_SHAPE and a
 * message that names the largest n allowed, and no work is issued.  Every call on a GPU shares that
 * GPU's array (each call clears what it uses with a kernel first): calls that overlap on one GPU,
 * from different streams or host threads, race; calls on one stream are ordered and safe.
 * Asynchronous on the network's stream. */
int32_t dbsn_classify_static(dbsn_mlp* mlp, const float* samples_dev, int64_t n, int32_t* labels_out_dev);

/* Error count of a validation or test pass (section "Results"): *count_dev (int64, device, 8-byte
 * aligned) = number of s < n with predicted_dev[s] != labels_dev[s] (both [n] int32, device).
 * n == 0 writes 0.  Asynchronous on hip_stream. */
int32_t dbsn_count_errors(const int32_t* predicted_dev, const int32_t* labels_dev, int64_t n,
                          int64_t* count_dev, void* hip_stream);

/* Mean of the per-step losses of an epoch: *mean_dev (float, device) = the sum of loss_dev[0 .. n)
 * taken in binary64 in a fixed order, divided by n, rounded to binary32.  n >= 1. */
int32_t dbsn_mean_loss(const float* loss_dev, int64_t n, float* mean_dev, void* hip_stream);

/* Measurement aid, not part of the method: the memory traffic of a streamed training step without
 * its arithmetic.  `sweeps` times over buf_dev[0 .. n_floats): one kernel that reads every float,
 * one that reads it and writes it back (adding 0.0f), i.e. 12 bytes per float and sweep, the mix
 * of forward read, backward read and update write.  Timed by the caller (events on hip_stream), it
 * gives the bandwidth this mix can reach over a footprint of 4 * n_floats bytes.  buf_dev: device,
 * 16-byte aligned, n_floats a multiple of 4; sink_dev: [4 * workgroups] floats of device memory the
 * read kernel leaves its sums in; workgroups of 256 threads each, 1 .. 65536. */
int32_t dbsn_probe_stream(float* buf_dev, int64_t n_floats, int32_t workgroups, int32_t sweeps,
                          float* sink_dev, void* hip_stream);

/* Measurement aid, not part of the method: the bare hand-over of the persistent training kernel.
 * 256 workgroups; in each of `rounds` rounds every workgroup publishes 64 tagged words and polls 8
 * words of 8 others until they carry the round's number.  within_die = 0: partners all over the
 * chip, device-scope stores; 1: partners on the same die, taking workgroup g to run on die g % 8
 * (true of a launch on an otherwise idle chip, which is how this probe is meant to be run; the
 * training kernel does not rely on it), workgroup-scope stores that stop in the die's L2.  Timed by the caller, time / rounds is the cost
 * of one hand-over.  buf_dev: 2 * 256 * 64 uint64 of device memory (the call clears it);
 * *gave_up_dev (int32, device) receives the number of workgroups whose polls gave up (0 when the
 * assumption about the dies holds).  One cooperative launch on hip_stream. */
int32_t dbsn_probe_handover(int32_t within_die, int32_t rounds, uint64_t* buf_dev, int32_t* gave_up_dev,
                            void* hip_stream);

/* Message for the last error on this host thread ("" if none). */
const char* dbsn_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* DBSN_H */
