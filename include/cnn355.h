/*
 * cnn355 -- on-line (per-image) back-propagation training of the CNN variant of
 * Ciresan, Meier, Masci, Gambardella, Schmidhuber, "High-Performance Neural Networks for
 * Visual Object Classification" (IDSIA TR 01-11, 2011), as hand-written HIP kernels for
 * gfx950 (MI355X).
 *
 * C ABI.  Pointers named d_* are DEVICE pointers (memory of the current HIP device, owned
 * by the caller); pointers named host_* are HOST pointers.  The library allocates no
 * device memory: everything it needs on the device lives in the workspace the caller
 * hands to cnn_create and must keep alive until cnn_destroy.  All arithmetic is fp32
 * (the paper's GPU precision, Sec. 4); indices are integers.
 *
 * Errors: every int-returning call gives 0 on success or one of the negative codes below;
 * nothing throws or aborts across this boundary.  Device work is asynchronous on the
 * stream given at creation unless a call says it synchronises; a device-side failure shows
 * up at the next synchronising call.  cnn_last_error gives a readable message.
 *
 * Calls on one handle must not overlap in time (one handle = one network = one stream).
 */
#ifndef CNN355_H
#define CNN355_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct cnn cnn_t; /* opaque; owns host metadata only */

enum {
  CNN_OK = 0,
  CNN_E_SYNTAX = -1,    /* architecture string does not follow the grammar              */
  CNN_E_SHAPE = -2,     /* a map size is not positive, a pooling rectangle does not tile
                           its map, or a size exceeds what the kernels support           */
  CNN_E_ARG = -3,       /* null pointer, label out of range, size mismatch, bad index    */
  CNN_E_WORKSPACE = -4, /* workspace too small or misaligned                             */
  CNN_E_HIP = -5,       /* a HIP call or a kernel reported failure                       */
  CNN_E_STATE = -6      /* call not valid in the handle's current state                  */
};

/* layer kinds reported by cnn_layer_info */
enum { CNN_LAYER_INPUT = 0, CNN_LAYER_CONV = 1, CNN_LAYER_POOL = 2, CNN_LAYER_FC = 3 };

/* execution modes for cnn_set_mode */
enum {
  CNN_MODE_STAGES = 0,    /* one kernel launch per stage of the step                      */
  CNN_MODE_PERSISTENT = 1,/* one cooperative launch per call; stages separated by grid
                             barriers, images of cnn_*_many looped on the device          */
  CNN_MODE_RESIDENT = 2   /* one cooperative launch per call; every workgroup owns whole
                             maps and keeps their weights in LDS for the whole call; what
                             workgroups exchange per image travels as tagged words, with no
                             grid barrier.  Needs one to six convolutional and one to four
                             fully connected layers and a network whose per-workgroup share
                             fits the LDS (cnn_mode_supported tells).  Weights in the
                             workspace are read at the start of a call and written back at
                             its end.                                                       */
};

/* output units for cnn_set_output_units */
enum {
  CNN_OUTPUT_SOFTMAX_XENT = 0, /* soft-max outputs, cross-entropy error E = -log p[label];
                                  delta_k = p_k - [k == label] (default)                    */
  CNN_OUTPUT_TANH_SQERR = 1    /* the scaled hyperbolic tangent of Sec. 4 on the output
                                  neurons too, E = 1/2 sum_k (y_k - t_k)^2 with targets
                                  t = +1 for the image's class and -1 otherwise;
                                  delta_k = (y_k - t_k) f'(y_k)                             */
};

/*
 * Architecture string (all structural parameters of Sec. 2.2-2.4 are run-time data):
 *     <C>x<H>x<W> { -<M>C<K>[S<s>] | -MP<K> | -<N>N }+
 *   <C>x<H>x<W>   network input: C maps of H rows x W columns
 *   <M>C<K>[S<s>] convolutional layer (Sec. 2.2): M maps, KxK kernel, skipping factor s in
 *                 both directions (default 0; consecutive kernel positions are s+1 pixels
 *                 apart), scaled-tanh units, fully connected map table unless
 *                 cnn_set_connection_table replaces it.  Output size by Eq. 1, rounded down
 *                 where the fraction is not integral (the kernel stays inside the map).
 *   MP<K>         max-pooling over non-overlapping KxK rectangles (Sec. 2.3); must follow a
 *                 convolutional layer and K must divide the map size.
 *   K and s may each be written <y>x<x>, rows then columns (Sec. 2.2 and 2.3 give kernel sizes,
 *   skipping factors and pooling rectangles an x and a y value): "8C4x2S1x0", "MP2x5".  Eq. 1
 *   then holds axis by axis.  Layers whose x and y values differ run on the vector kernels
 *   of the stage and persistent modes and in cnn_forward_batch; the resident mode refuses
 *   them (CNN_E_STATE).
 *   <N>N          fully connected layer of N neurons (Sec. 2.4).  The last token must be
 *                 one: the output layer, one unit per class.  Hidden fully connected layers
 *                 use the scaled tanh y = 1.7159 tanh(0.6666 a) (Sec. 4); the output layer
 *                 is a soft-max trained with the cross-entropy error by default (the paper
 *                 names no error function); cnn_set_output_units switches to scaled-tanh
 *                 output neurons trained on the squared error.
 *   Example: "1x29x29-20C4-MP2-40C5-MP3-150N-10N".
 *
 * Layer numbering used by the calls below: layer 0 is the network input (after the fixed
 * front-end, if one is set); layers 1..n-1 are the tokens in order.
 */

/* Host-only: parse `arch` and report its layers.  info receives, per layer, 6 int32:
 * {kind, maps, rows, cols, K, S}; at most max_layers layers are written; *n_layers gets
 * the full count.  No device is touched. */
int cnn_arch_info(const char* arch, int32_t* n_layers, int32_t* info, int32_t max_layers);
/* The same with 8 int32 per layer: {kind, maps, rows, cols, Ky, Sy, Kx, Sx} (cnn_arch_info reports the y values). */
int cnn_arch_info_xy(const char* arch, int32_t* n_layers, int32_t* info, int32_t max_layers);

/* Host-only: bytes of device workspace cnn_create needs for `arch` (an upper bound that
 * also covers any connection table and front-end set later).  Fails with CNN_E_SHAPE when a
 * layer is larger than the kernels support. */
int cnn_workspace_bytes(const char* arch, size_t* bytes);

/* Host-only: the stages one training step of `arch` is issued as (one text line per stage:
 * kind, layer, work items, tiling), written NUL-terminated into buf (truncated to n). */
int cnn_plan_text(const char* arch, char* buf, size_t n);

/* The same for an existing network, with its connection tables and front-end as they are now. */
int cnn_get_plan_text(const cnn_t* net, char* buf, size_t n);

/* Build a network.  d_workspace: device memory of at least cnn_workspace_bytes bytes,
 * 256-byte aligned, owned by the caller, used exclusively by this handle.  hip_stream: a
 * hipStream_t (NULL = the default stream) on which all device work of the handle is
 * issued.  Weights start at zero; fill them with cnn_set_weights.  Synchronises. */
int cnn_create(const char* arch, void* d_workspace, size_t bytes, void* hip_stream, cnn_t** out);
void cnn_destroy(cnn_t* net);

/* Replace the map connection table of the conv_index-th convolutional layer (0-based)
 * (Sec. 2.2 "connection table", Sec. 3.1).  host_table is [M_out][M_in] bytes, non-zero =
 * connected; every output map needs at least one input.  Changes cnn_num_weights and
 * zeroes all weights: set tables before weights.  Synchronises. */
int cnn_set_connection_table(cnn_t* net, int conv_index, const uint8_t* host_table);

/* Put a fixed, never-trained image-processing layer in front of the network (Sec. 2.1):
 * n_filters (= C of the architecture string) KxK filters; filter f is correlated (valid
 * region, no bias, no non-linearity) with channel host_src_channel[f] of the raw image.
 * A raw image then has n_src_channels maps of (H+K-1) x (W+K-1).  K <= 32.  No delta is
 * propagated into it.  Synchronises. */
int cnn_set_fixed_frontend(cnn_t* net, int n_filters, int K, int n_src_channels,
                           const float* host_filters, const int32_t* host_src_channel);

size_t cnn_num_weights(const cnn_t* net); /* trainable parameters, after tables are set   */
size_t cnn_image_size(const cnn_t* net);  /* floats in one raw image                      */
int cnn_num_layers(const cnn_t* net);
int cnn_num_classes(const cnn_t* net);
/* {kind, maps, rows, cols, K, S} of one layer */
int cnn_layer_info(const cnn_t* net, int layer, int32_t* info6);
/* {kind, maps, rows, cols, Ky, Sy, Kx, Sx} of one layer */
int cnn_layer_info_xy(const cnn_t* net, int layer, int32_t* info8);

/*
 * Canonical weight order for get/set, n = cnn_num_weights: layer by layer in network
 * order.  Convolutional layer: bias[M], then one KxK block per connection -- output map
 * ascending, connected input map ascending within it -- each block row-major [ky][kx],
 * applied without flipping (the receptive field of output x is inputs x(S+1)..x(S+1)+K-1,
 * Sec. 3.3).  Fully connected layer: bias[N], then W[N][n_in] row-major, n_in index =
 * (map*rows + y)*cols + x of the layer below.  One bias per map / neuron (Sec. 3.2).
 * Both calls synchronise the stream.
 */
int cnn_get_weights(cnn_t* net, float* host_dst, size_t n);
int cnn_set_weights(cnn_t* net, const float* host_src, size_t n);

/* Forward propagation of many images at once (Sec. 3.2; validation and test passes change no
 * weight, Sec. 4, so their images are independent).  Every layer becomes one matrix product over
 * the whole batch on the matrix cores, fp32 in and out; results agree with cnn_forward_many to
 * rounding (other summation order), whatever the mode of the handle.
 *   cnn_forward_batch_scratch_bytes: device memory the call needs for `batch` images in flight
 *     (re-packed weights, the layer outputs of one batch); the caller allocates it.
 *   cnn_forward_batch: d_images [n][cnn_image_size], d_probs [n][cnn_num_classes] (probabilities, or
 *     the outputs with CNN_OUTPUT_TANH_SQERR), both device memory; d_scratch: device memory,
 *     256-byte aligned, at least scratch_bytes, owned by the caller, free for other use once the
 *     stream has passed the call.  The n images are run `batch` at a time.  The weights are read as
 *     they stand when the call reaches them on the stream.  Asynchronous.
 * Errors: CNN_E_ARG (NULL, batch 0, misaligned scratch), CNN_E_WORKSPACE (scratch too small),
 * CNN_E_SHAPE (a single input map of some layer, times the images one workgroup touches, exceeds
 * 148 KB of LDS: maps beyond about 135 x 135), CNN_E_HIP. */
int cnn_forward_batch_scratch_bytes(cnn_t* net, size_t batch, size_t* bytes);
int cnn_forward_batch(cnn_t* net, const float* d_images, size_t n, float* d_probs, void* d_scratch,
                      size_t scratch_bytes, size_t batch);

/* For callers that cannot allocate device memory (code under HIP graph capture, tight serving loops,
 * harnesses that forbid it): cnn_forward_batch with its scratch memory taken from an array inside the
 * library's device image (CNN_FORWARD_BATCH_STATIC_SCRATCH_BYTES bytes, which every GPU the library runs on
 * holds until the process ends) instead of from the caller.  Same arguments otherwise, same kernels, same
 * bits.  The call allocates and frees nothing on the device, it launches kernels on the handle's stream only.
 * Call it with the device current on which the network was created (CNN_E_STATE otherwise).  A batch whose
 * scratch need (cnn_forward_batch_scratch_bytes) exceeds the array is refused with CNN_E_WORKSPACE and a
 * message that names both sizes.  Every call on a GPU, from any handle, uses that GPU's one array, which keeps
 * the previous call's contents (every part that is read is written first in each call): calls that overlap in
 * time on one GPU race and must be serialised by the caller.  Asynchronous. */
#define CNN_FORWARD_BATCH_STATIC_SCRATCH_BYTES (64u << 20)
int cnn_forward_batch_static(cnn_t* net, const float* d_images, size_t n, float* d_probs, size_t batch);

/* Forward propagation of one image (Sec. 3.2).  d_image: cnn_image_size floats, maps then
 * rows then columns.  d_probs: cnn_num_classes floats (may be NULL).  Asynchronous. */
int cnn_forward(cnn_t* net, const float* d_image, float* d_probs);

/* One step of on-line gradient descent (Sec. 1, Sec. 4): forward propagation (Sec. 3.2),
 * deltas pulled back through every layer with the weights still at their old values
 * (Sec. 3.3), weight gradients and w <- w - lr * dE/dw for every weight (Sec. 3.4).
 * Asynchronous; the next call on the handle sees the updated weights. */
int cnn_train_step(cnn_t* net, const float* d_image, int32_t label, float lr);

/* n train steps on consecutive images, in order, exactly as n calls of cnn_train_step.
 * d_images: n * cnn_image_size floats; d_labels: n int32, each in [0, classes) -- a label
 * outside the range makes the device skip that image's update and the next synchronising
 * call return CNN_E_ARG.  Asynchronous. */
int cnn_train_many(cnn_t* net, const float* d_images, const int32_t* d_labels, size_t n, float lr);

/* n forward propagations; d_probs: n * cnn_num_classes floats.  Asynchronous. */
int cnn_forward_many(cnn_t* net, const float* d_images, size_t n, float* d_probs);

/* Choose how a step is issued (CNN_MODE_*).  CNN_MODE_STAGES and CNN_MODE_PERSISTENT give
 * identical bits, except for networks with wide layers while the matrix cores are on
 * (cnn_set_matrix_cores): there only CNN_MODE_STAGES pulls the deltas on the matrix cores, and
 * the two agree to rounding.  CNN_MODE_RESIDENT sums in another order and agrees with them to
 * rounding.  Switching to or from CNN_MODE_STAGES re-plans the stage list (synchronises).
 * CNN_E_STATE when the mode cannot run this network (the mode is then unchanged).  Setting a
 * connection table or a front-end re-plans the network: if resident mode can no longer run it
 * the handle drops to CNN_MODE_PERSISTENT (cnn_get_mode tells). */
int cnn_set_mode(cnn_t* net, int mode);
int cnn_get_mode(const cnn_t* net);
/* 1 when `mode` can run this network on this device, else 0 (cnn_last_error says why). */
int cnn_mode_supported(cnn_t* net, int mode);

/* Resident mode: size and placement of the team.  n_ranks workgroups share the maps (0 =
 * automatic: one per map of the widest convolutional layer, at most one per compute unit);
 * xcd_stride 8 launches 8 x n_ranks workgroups of which every eighth works, which puts the
 * whole team on one XCD (at most 32 ranks); 1 spreads the team over all XCDs; 0 = automatic.
 * Results do not depend on the placement, and for a given n_ranks they are reproducible bit
 * for bit.  Synchronises. */
int cnn_set_team(cnn_t* net, int n_ranks, int xcd_stride);

/* What the last layer computes and which error the net is trained on (Sec. 4 gives every neuron
 * the scaled hyperbolic tangent and names no error function: both readings are offered).  With
 * CNN_OUTPUT_TANH_SQERR the d_probs arguments receive the outputs y_k instead of probabilities
 * and cnn_get_loss the squared error.  Every mode honours it; weights, tables and the weight
 * count are unchanged.  kind outside the enum: CNN_E_ARG.  Synchronises. */
int cnn_set_output_units(cnn_t* net, int kind);
int cnn_get_output_units(const cnn_t* net);

/* Stage and persistent modes: whether wide convolutional layers (full table, at least 64 output
 * maps and 256 inputs x taps per output) run their forward pass -- and, in the stage mode, the
 * delta pull through them (at least 32 input maps, skipping factor 0) -- as implicit GEMMs on the
 * matrix cores (fp32 MFMA) -- on by default -- or through the vector kernels like every other layer.
 * Results agree to rounding.  Weights and tables are kept.  Synchronises. */
int cnn_set_matrix_cores(cnn_t* net, int on);

/* CNN_MODE_STAGES launches every stage of every image by itself (10 - 14 launches per image for the wide nets of
 * Sec. 4.2 and 4.3, about 2.5 us each whatever the kernel does).  With images_per_graph > 0 cnn_train_many and
 * cnn_forward_many replay instead a graph that holds the launches of that many consecutive images: as many whole
 * graphs as the call has images for when it has at least twice that many, the rest stage by stage as before.
 * Same kernels, same order, same results bit for bit.  Off (0) by default: an empty kernel costs 1.5 us as a node
 * of a graph against 2.5 us launched, but with the stage kernels of the benchmark nets a replay takes as long as
 * the launches (measured on 1024 images: the widest net 132.6 against 132.0 us per image, the benchmark net 43.3
 * against 44.5).  At most 1024 images per graph.  The graph is built at the first call that uses it and again after
 * anything that changes the stage list (mode, tables, output variant, matrix cores).  CNN_E_ARG for a value
 * outside the range. */
int cnn_set_launch_graph(cnn_t* net, int images_per_graph);

/* Persistent mode: number of workgroups of the cooperative launch (0 = automatic: the
 * largest stage's work items, capped at the number of compute units).  Values above what
 * can be co-resident are clamped. */
int cnn_set_grid(cnn_t* net, int n_workgroups);

/* Persistent mode: grid barrier between stages.  0 = one arrival counter with a device-scope
 * release and acquire in every workgroup; 1 (default) = two levels, one arrival counter per
 * XCD and one across XCDs, so that only one workgroup per XCD writes that XCD's L2 back.
 * Results are identical. */
int cnn_set_barrier(cnn_t* net, int kind);

/* Persistent mode: how many times a workgroup polls a grid barrier before it gives up,
 * raises the abort flag and leaves the kernel (the next synchronising call then returns
 * CNN_E_HIP).  Every wave therefore terminates even if a barrier can never complete. */
int cnn_set_spin_limit(cnn_t* net, unsigned int polls);

/* Wait for the stream; returns the first device-side error since the last call. */
int cnn_synchronize(cnn_t* net);

/* ---- parity taps: synchronous, host destinations, state of the last step/forward ---- */

/* Output of a layer: conv = after the scaled tanh, pool = pooled values, fully connected
 * = after the scaled tanh, output layer = probabilities.  maps*rows*cols floats. */
int cnn_get_activation(cnn_t* net, int layer, float* host_dst);
/* dE/d(pre-activation) of a convolutional or fully connected layer after a train step or
 * cnn_debug_gradients, dense, maps*rows*cols floats (for a pooled convolutional layer:
 * zero except at the arg-max of each rectangle). */
int cnn_get_delta(cnn_t* net, int layer, float* host_dst);
/* Winner index dy*K+dx (first maximum in row-major order) of every rectangle of a
 * max-pooling layer, maps*rows*cols bytes. */
int cnn_get_argmax(cnn_t* net, int pool_layer, uint8_t* host_dst);
/* Cross-entropy error of the last train step / debug-gradient call. */
int cnn_get_loss(cnn_t* net, float* host_loss);
/* Persistent mode only: device timestamps of the last image of the last call, as seen by
 * workgroup 0.  host_us receives, per stage, 2 floats: microseconds spent on the stage's work
 * items and microseconds spent in the grid barrier after it (0 for stages skipped by a
 * forward-only call); *n_stages gets the stage count.  Synchronises. */
int cnn_get_stage_times(cnn_t* net, float* host_us, int max_stages, int* n_stages);

/* Measurement aids for the bound that caps a chain of dependent stages (one image at a time, every layer
 * waits for the one before): what one crossing between compute units costs, and what one kernel launch costs,
 * on this device, now.
 *   cnn_measure_crossing: n_ranks workgroups (2 .. one per compute unit) each store words_per_rank tagged words
 *     and fetch those of all ranks -- the exchange of the resident mode between two layers -- `rounds` times in
 *     one cooperative launch; *host_us = microseconds per round (device clock of rank 0).  Uses the network's
 *     exchange buffers (CNN_E_WORKSPACE if they are too small for the request).  Synchronises.
 *   cnn_measure_launch: `rounds` launches of an empty kernel back to back on the handle's stream, timed with
 *     events; *host_us = microseconds per launch: the floor under every stage of CNN_MODE_STAGES.  Synchronises. */
int cnn_measure_crossing(cnn_t* net, int n_ranks, int words_per_rank, int rounds, float* host_us);
int cnn_measure_launch(cnn_t* net, int rounds, float* host_us);

/* ---- a resident kernel compiled for the handle's own network ---------------------------------
 * The resident mode (spec: the whole on-line step of Sec. 3.2 - 3.4 without per-stage launches) runs a
 * benchmark network in a kernel compiled for it, every size, offset and trip count a literal, and any other
 * network in a kernel that reads its plan at run time, at about 1.5 x the time per image.  These calls give
 * any network the first kind of kernel:
 *   cnn_resident_spec_source: writes into host_buf (n bytes, NUL-terminated, truncated if too small) the text of
 *     a C++ header that describes this handle's network as it stands now (layer shapes, connection-table
 *     statistics, output variant, team) to the library's own kernel source, and returns the length of the whole
 *     text (call with n = 0 to size the buffer).  CNN_E_STATE when resident mode cannot run the network.
 *     Compiling csrc/cnn355_flow.hip for gfx950, device code only, with -DCNN355_SPECIAL_HEADER="<path of that
 *     header>" gives a code object (paper_1102_0183_amd/specialize.py does both steps and keeps the result).
 *   cnn_load_resident_code: loads such a code object (host_path: a file) into the handle.  The plan compiled into
 *     it must equal the handle's own plan word for word, else CNN_E_STATE and nothing changes; a file that is no
 *     such code object gives CNN_E_ARG.  From then on resident-mode calls run that kernel; whenever the plan changes
 *     (another table, output variant or team) the handle falls back to the compiled-in kernels by itself and
 *     returns to the loaded one when the plan is that one again.  Results are bit for bit those of the compiled-in
 *     kernels (same source, same order of operations).  Synchronises.  The code object stays loaded until
 *     cnn_destroy or the next cnn_load_resident_code.
 *   cnn_resident_code_active: 1 while resident-mode calls would run the loaded kernel, else 0. */
int cnn_resident_spec_source(const cnn_t* net, char* host_buf, size_t n);
int cnn_load_resident_code(cnn_t* net, const char* host_path);
int cnn_resident_code_active(const cnn_t* net);

/* Parity tap of the batched forward pass (Sec. 3.2 for many images): runs cnn_forward_batch's kernels on n images
 * as one batch (d_scratch as for cnn_forward_batch with batch = n) up to and including trainable layer
 * `trainable_layer` (0 = the first convolutional or fully connected layer of the architecture string, counting
 * those two kinds only) and copies that layer's outputs to host_out: [image][map][Hp][Wp] pooled activations of
 * a convolutional layer (its own activations when no pooling follows), [image][unit] activations of a hidden fully
 * connected layer, [image][class] the sums of the output layer before the output units.  *host_floats_per_image
 * receives the floats per image (host_out must hold n times that: at most the largest layer output).
 * Synchronises.  CNN_E_ARG for a layer index beyond the last. */
int cnn_debug_forward_batch_layer(cnn_t* net, const float* d_images, size_t n, int trainable_layer, float* host_out,
                                  size_t* host_floats_per_image, void* d_scratch, size_t scratch_bytes);

/* Forward + backward for (d_image, label) with the update replaced by a store of dE/dw:
 * host_grad receives cnn_num_weights floats in canonical order; weights are unchanged. */
int cnn_debug_gradients(cnn_t* net, const float* d_image, int32_t label, float* host_grad);

/* ---- on-line deformation of training images --------------------------------------------------
 * Sec. 4.1: every presentation of a training image is deformed anew by a combination of affine maps
 * (translation, rotation, scaling, horizontal shearing) and an elastic deformation (Simard et al. 2003);
 * Sec. 4.2 and 4.3: random translations of at most 5 % of the image side.  The paper gives no formulas;
 * what this call computes, with every range a parameter:
 *   presentation t = first_index + k of the stream (output image k; all C maps share one deformation)
 *   draws: mix64(key + G (j + 1)), key = mix64(seed + G (t + 1)), mix64 = SplitMix64's output function,
 *          G = 0x9E3779B97F4A7C15; a 32-bit half b of a draw gives sym(b) = 2 (b >> 8) / 2^24 - 1
 *   draw 0: tx = sym(hi) max_translation W, ty = sym(lo) max_translation H          (pixels)
 *   draw 1: theta = sym(hi) max_rotation (degrees), shear = sym(lo) max_shear
 *   draw 2: sx = 1 + sym(hi) max_scaling, sy = 1 + sym(lo) max_scaling
 *   draw 3 + y W + x: the two random fields rx[y][x] = sym(hi), ry[y][x] = sym(lo)
 *   Dx = alpha (g (x) g) * rx, Dy likewise: g[i] = exp(-i^2 / (2 sigma^2)), |i| <= ceil(3 sigma), normalised to
 *          sum 1; the fields are zero outside the image; sigma == 0 or alpha == 0: no elastic part
 *   A = Rot(theta) [[1, shear], [0, 1]] diag(sx, sy) about the centre ((W-1)/2, (H-1)/2)
 *   output pixel (y, x) is the source map sampled at (cx + A (x - cx, y - cy) + (tx, ty) + (Dx, Dy)[y][x]) by
 *   bilinear interpolation; a neighbour outside the map counts as `fill`.
 * The result depends on (seed, t) only, not on how presentations are grouped into calls.
 *
 * d_src: device, n_src images [C][H][W] (fp32, contiguous); d_dst: device, n images, must not overlap d_src.
 * d_src_index (device, n int32, or NULL): source image of every output; NULL means output k is image k
 * (then n <= n_src); an entry outside [0, n_src) gives an image of `fill`.  d_displacement (device,
 * [n][2][H][W], or NULL): receives, per output pixel, its source position minus its own (x, then y).
 * hip_stream: a hipStream_t (NULL: the default stream).  Asynchronous; nothing is allocated; the caller owns
 * every buffer.  Limits: H x (W rounded up to odd) <= 9312 (so 96 x 96 fits), C <= 1024, sigma <= 16, max_scaling < 1, ranges >= 0 and finite.
 * Errors: CNN_E_ARG, CNN_E_SHAPE, CNN_E_HIP; the message is cnn_last_error(NULL)'s. */
typedef struct cnn_deform_params {
  float max_translation; /* fraction of the image side                                   */
  float max_rotation;    /* degrees                                                      */
  float max_scaling;     /* fraction: factors in [1 - m, 1 + m), x and y independently   */
  float max_shear;       /* horizontal shear coefficient: x += shear * y                 */
  float sigma;           /* std of the smoothing Gaussian, pixels                        */
  float alpha;           /* amplitude of the elastic part, pixels                        */
  float fill;            /* value outside the source image                               */
} cnn_deform_params;
int cnn_deform_images(void* hip_stream, const float* d_src, size_t n_src, float* d_dst, size_t n, int C, int H, int W,
                      const cnn_deform_params* p, uint64_t seed, uint64_t first_index,
                      const int32_t* d_src_index, float* d_displacement);

/* Message for the last error on this handle (or, with net == NULL, of the last failed
 * cnn_create / cnn_workspace_bytes / cnn_arch_info / cnn_deform_images on this thread).  Never NULL. */
const char* cnn_last_error(const cnn_t* net);

#ifdef __cplusplus
}
#endif
#endif /* CNN355_H */
