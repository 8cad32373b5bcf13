// Descriptors shared by the host planner and the gfx950 kernels.  Plain data only.
#pragma once
#include <stddef.h>
#include <stdint.h>

// Pointers into device memory.  The kernel translation unit defines CNN_GLOBAL as the global
// address space for its device pass, so that loads and stores through these fields compile to
// global (not flat) memory instructions; everywhere else it is empty and the layout is the same.
#ifndef CNN_GLOBAL
#define CNN_GLOBAL
#endif

namespace cnn355 {

constexpr int WG = 1024;  // threads per workgroup: 16 wavefronts of 64, one workgroup per CU

// LDS carve-up, in floats.  One static block per workgroup (gfx950 has 160 KB per CU); every
// stage cuts it its own way.
constexpr int LDS_IN = 20480;   // staged input maps / rebuilt delta maps (80 KB)
constexpr int LDS_AUX = 6144;   // filters / deltas (24 KB)
constexpr int LDS_AUX2 = 6144;  // winner coordinates (24 KB)
constexpr int MAX_TILE_PIX = 2 * WG;     // conv outputs per workgroup tile (up to 2 per thread)
constexpr int LDS_RED = WG + MAX_TILE_PIX;  // cross-split partial sums + one output tile (12 KB)
constexpr int LDS_FLOATS = LDS_IN + LDS_AUX + LDS_AUX2 + LDS_RED;  // 35840 floats = 140 KB

constexpr int MAX_POOLED_PIX = LDS_AUX; // pooled positions of one map that fit the staging area
constexpr int MAX_FC_OUT = LDS_AUX;     // neurons of one fully connected layer (delta staged in LDS)
constexpr int MAX_LAYERS = 32;
constexpr int MAX_STAGES = 96;
constexpr int MAX_FRONTEND_K = 32;

enum LayerKind : int { L_CONV = 1, L_FC = 3 };

// One trainable layer as the kernels see it.  A max-pooling layer is folded into the
// convolutional layer it follows (Kp = 1 when there is none).
struct LayerDev {
  int kind;
  // convolution geometry: Mi maps of Hi x Wi in, Mo maps of Ho x Wo out, K x Kx kernel,
  // skipping factors S, Sx (strides S+1, Sx+1), pooled by Kp x Kpx to Hp x Wp
  int Mi, Hi, Wi, Mo, Ho, Wo, K, S, Kp, Hp, Wp;
  // Sec. 2.2 and 2.3 give kernel, skipping factor and pooling rectangle an x and a y value each: K, S, Kp are
  // the y (row) values, Kx, Sx, Kpx the x (column) values; rect = some pair differs (such a layer runs on the
  // vector stage kernels only)
  int Kx, Sx, Kpx, rect;
  int n_in, n_out;     // fully connected: W is [n_out][n_in]
  int is_output;       // output layer
  int out_units;       // output layer: 0 soft-max + cross-entropy, 1 scaled tanh + squared error (targets +-1)
  int in_is_image;     // input is the image handed to the call (no stored activation below)
  int max_conn;        // longest row of the connection table
  int full_table;      // every output map reads every input map (slot of (j, i) is j * Mi + i)
  const CNN_GLOBAL float* in;     // input activations (NULL when in_is_image)
  CNN_GLOBAL float* act;          // conv: after tanh, full resolution; fc: after tanh / probabilities
  CNN_GLOBAL float* out;          // what the layer above reads (conv: pooled values; fc: == act)
  CNN_GLOBAL uint8_t* arg;        // conv: winner index dy*Kp+dx per pooled position
  CNN_GLOBAL int* argyx;          // conv: (y << 16) | x of the winner in conv-output coordinates
  CNN_GLOBAL float* delta;        // dE/d(pre-activation): conv at the winners [Mo][Hp][Wp]; fc [n_out]
  CNN_GLOBAL float* dact;         // derivative of the activation function where a delta can arrive: conv at the
                                  // winners [Mo][Hp][Wp]; hidden fc [n_out] (written by the forward pass)
  CNN_GLOBAL float* bias;
  CNN_GLOBAL float* w;            // conv: one K*K block per connection, CSR order; fc: [n_out][n_in]
  long long w_canon;   // offset of w in the canonical weight vector (for gradient taps)
  long long b_canon;
  const CNN_GLOBAL int* csr_ptr;  // [Mo+1] forward table (C^n of Sec. 3.1): row j -> slots
  const CNN_GLOBAL int* csr_idx;  // [n_conn] input map of every slot
  const CNN_GLOBAL int* csc_ptr;  // [Mi+1] backward table (C_BP of Sec. 3.1): input map i -> entries
  const CNN_GLOBAL int* csc_j;    // [n_conn] output map of every entry
  const CNN_GLOBAL int* csc_slot; // [n_conn] weight slot of every entry (WIDX_BP of Sec. 3.1)
  CNN_GLOBAL float* mm_part;      // [slices][Mo][Ho*Wo] partial sums of the matrix-core forward pass (shared scratch)
};

enum StageKind : int {
  ST_FRONTEND = 1,   // fixed image-processing filters
  ST_CONV_FWD = 2,   // convolution + bias + tanh + max-pool + arg-max
  ST_FC_FWD = 3,     // hidden fully connected layer + tanh
  ST_HEAD = 4,       // output layer, soft-max, error, output delta, and its own backward+update
  ST_FC_BWD = 5,     // hidden fully connected layer: pull deltas + update its weights
  ST_CONV_BWD = 6,   // pull deltas through a convolutional layer
  ST_CONV_WGRAD = 7, // convolutional weight gradients + update
  ST_CONV_FWD_MFMA = 8, // wide convolutional layer as an implicit GEMM on the matrix cores: partial sums
  ST_CONV_EPI = 9,      // ... then: sum of the partial sums + bias + tanh + max-pool + arg-max
  ST_CONV_BWD_MFMA = 10, // delta pull through a wide layer as FP's mirror image on the matrix cores: partial sums
  ST_CONV_BWD_EPI = 11,  // ... then: sum of the partial sums, times the activation derivative of the layer below
  ST_CONV_WGRAD_MFMA = 12, // weight gradients of a wide layer as a matrix product over the output pixels, and the adjustment
};
constexpr int MFMA_MAX_SLICES = 64;  // partial-sum slices (splits of the contraction) per layer

struct Stage {
  int kind;
  int layer;          // index into ProgramDev::layers
  int n_items;        // independent work items (one workgroup each)
  int barrier_after;  // persistent mode: all workgroups must finish this stage before the next starts
  int train_only;     // skipped by forward-only calls
  // tiling parameters (meaning depends on kind)
  int tile_rows;      // CONV_FWD: conv rows per tile (multiple of Kp)
  int n_tiles;        // CONV_FWD / CONV_BWD: tiles per map; CONV_WGRAD: connection chunks per output map
  int chunk;          // maps staged per pass (CONV_FWD: input maps, CONV_BWD: output maps, CONV_WGRAD: input maps)
  int tw_log2;        // log2 of the lane group width used when staging one map; CONV_BWD: log2 of the pixel tile
  int pix_per_thread; // CONV_FWD: 1 or 2
  int rows_per_wg;    // FC_FWD: neurons per work item (power of two, 1..16); CONV_FWD_MFMA / CONV_EPI: partial-sum slices
  int cm_log2;        // FC_BWD / HEAD: log2 of columns per tile
};

struct FrontendDev {
  int n_filters, K, n_src, Hr, Wr, H, W;  // raw image n_src x Hr x Wr -> n_filters x H x W
  int pad;
  const CNN_GLOBAL float* filters;  // [n_filters][K][K]
  const CNN_GLOBAL int* src;        // [n_filters]
  CNN_GLOBAL float* out;            // [n_filters][H][W]
};

struct ProgramDev {
  int n_layers;
  int n_stages;
  int n_classes;
  int has_frontend;
  FrontendDev fe;
  LayerDev layers[MAX_LAYERS];
  Stage stages[MAX_STAGES];
};

// Device-side status block.
struct StatusDev {
  unsigned int barrier_count;  // monotone arrival counter of the grid barrier
  unsigned int abort_flag;     // set when a barrier wait gave up; every workgroup then leaves
  unsigned int bad_label;      // set when a label outside [0, classes) was met
  float loss;                  // cross-entropy error of the last trained image
  // two-level barrier: one line per XCD (index x * 32), plus the cross-XCD counter
  unsigned int top_count;
  unsigned int pad_[27];
  unsigned int xcd_members[16 * 32];  // workgroups of this launch that run on XCD x
  unsigned int xcd_count[16 * 32];    // monotone arrivals on XCD x
  unsigned int xcd_go[16 * 32];       // last barrier number released on XCD x
  // persistent mode, last image of the last call, seen from workgroup 0 (100 MHz ticks):
  // stamps[0] = image start; stamps[1 + 2 s] = stage s items done; stamps[2 + 2 s] = its barrier passed
  unsigned long long stamps[2 * MAX_STAGES + 2];
};

// Per-call arguments.
// What a replayed graph of stage launches cannot carry in its nodes: the arguments of the call it is launched for.
// They lie in device memory; a node knows its image's place inside the graph (RunArgs::t_local), the first node of
// the graph moves t0 on by the images of one graph.
struct CallArgs {
  const CNN_GLOBAL float* images;
  const CNN_GLOBAL int* labels;
  CNN_GLOBAL float* probs_out;
  long long image_stride;
  long long t0;          // image of the call the graph being replayed starts at
  float lr;
  int train;
};

struct RunArgs {
  const CNN_GLOBAL CallArgs* call;  // set in the nodes of a graph: images, labels, outputs, rate and image number
  int t_local;                      //   come from there (image call->t0 + t_local), not from the fields below
  const CNN_GLOBAL float* images;   // first image
  const CNN_GLOBAL int* labels;     // device labels, or NULL to use label_imm
  CNN_GLOBAL float* probs_out;      // optional [n_images][n_classes]
  CNN_GLOBAL float* grad_out;       // when set: store dE/dw here (canonical order) instead of updating
  long long n_images;
  long long image_stride; // floats
  int label_imm;
  int train;             // 0: forward only
  float lr;
  unsigned int spin_limit; // grid-barrier polls before giving up
  int barrier_kind;        // 0: one counter, full fences in every workgroup; 1: two-level (per XCD)
  unsigned int epoch_base; // resident mode: image t of this call carries tag epoch_base + t + 1
};

// ---- resident mode -----------------------------------------------------------------------
// Every workgroup ("rank") of a team owns whole maps: output maps j = rank, rank + G, ... of every
// convolutional layer.  For those it keeps in LDS, for the whole call, the filters it needs going
// forward (row j of the connection table) and, for the maps it owns in the layer below, a second
// copy of the filters that read them (column i), so that neither the forward pass nor the delta
// pull nor the weight adjustment touches another rank's weights.  What ranks exchange per image
// -- pooled outputs, partial sums of the first fully connected layer, deltas -- travels through
// global memory as 64-bit words {value, tag}, written and polled with device-scope atomics; the
// tag names the image, so a reader needs no barrier: it polls the word until the tag matches.
typedef unsigned long long tagged_t;

constexpr int FLOW_MAX_CONV = 6;
constexpr int FLOW_MAX_FC = 4;
// the arena a rank carves up, in floats (154 KB of the 160 KB of a gfx950 CU; the rest holds a copy
// of the descriptors)
constexpr int FLOW_LDS_FLOATS_MAX = 39424;
constexpr long long FLOW_SHARE_MIN_MACS = 1ll << 18;  // multiply-adds of one map's delta pull from which ranks share it
constexpr int FLOW_STRIP_MAX = 7;  // output pixels one lane accumulates in registers

// What the resident kernel needs besides the plan (cnn355_flowspec.h): where things lie in global memory.
struct FlowConvPtrs {
  CNN_GLOBAL float* w;            // one K*K block per connection, CSR order (canonical)
  CNN_GLOBAL float* bias;
  CNN_GLOBAL float* act;          // parity taps: full-resolution outputs,
  CNN_GLOBAL float* out;          //   pooled values,
  CNN_GLOBAL uint8_t* arg;        //   winner index dy*Kp+dx,
  CNN_GLOBAL int* argyx;          //   winner coordinates,
  CNN_GLOBAL float* delta;        //   deltas at the winners
  const CNN_GLOBAL int* csr_ptr;
  const CNN_GLOBAL int* csr_idx;
  const CNN_GLOBAL int* csc_ptr;
  const CNN_GLOBAL int* csc_j;
  const CNN_GLOBAL int* csc_slot;
  CNN_GLOBAL tagged_t* x_out;    // [2][Mo*Hp*Wp] pooled outputs, when a convolutional layer follows
  CNN_GLOBAL tagged_t* x_delta;  // [2][Mo*Hp*Wp] deltas at the winners (layers above the first)
  CNN_GLOBAL tagged_t* x_yx;     // [2][Mo*Hp*Wp] their coordinates
  CNN_GLOBAL tagged_t* x_part;   // [2][Mi][shares - 1][Hi*Wi] pulled sums of the shares beyond the first, for the map's owner
  CNN_GLOBAL tagged_t* x_w;      // [2][connections * K*K] streamed plans: the filters as their pull-copy holders have just
                                 //   adjusted them, in table order, for the holders of the forward copies
  long long w_canon, b_canon;    // offsets in the canonical weight vector (gradient tap)
};
struct FlowFcPtrs {
  CNN_GLOBAL float* w;
  CNN_GLOBAL float* bias;
  CNN_GLOBAL float* act;
  CNN_GLOBAL float* delta;
  long long w_canon, b_canon;
  // a layer held by columns (FcSpec::by_cols): the ranks' partial sums [2][ranks][n_out] going forward, the deltas
  // of the layer's inputs [2][n_in] going back (tagged words)
  CNN_GLOBAL tagged_t* x_part;
  CNN_GLOBAL tagged_t* x_dprev;
};
struct FlowPtrs {
  FlowConvPtrs conv[FLOW_MAX_CONV];
  FlowFcPtrs fc[FLOW_MAX_FC];
  CNN_GLOBAL tagged_t* xp;  // [2][n_col_ranks][n_out of the first FC layer] partial sums
  CNN_GLOBAL tagged_t* xsum;  // [2][n_out of the first FC layer] their sums plus bias, from the ranks that own them
};

// ---- batched forward pass ----------------------------------------------------------------
// One layer over a whole batch as a matrix product on the matrix cores (cnn355_batch.hip).
struct BatchGemm {
  const CNN_GLOBAL float* in;    // [batch] images of [Mi][Hi][Wi], in_stride floats apart
  const CNN_GLOBAL float* wt;    // [Mi*K*Kx][MoPad]: k = (input map, ky, kx) by output map, zero where unconnected
  const CNN_GLOBAL float* bias;  // [Mo]
  CNN_GLOBAL float* out;         // [batch][Mo][P], out_stride floats per image (P: see below)
  long long in_stride, out_stride;
  long long N;                   // columns: batch * P
  int Mi, Hi, Wi, K, stride, Mo, MoPad, Wo, P;  // Wo, P: width and size of the column grid of one image
  int Kx, stride_x, Kpx;         // x (column) values of kernel, stride and pooling window; K, stride, Kp are the y values
  int Kp;                        // Kp * Kpx > 1: a column is a pooled pixel, its Kp x Kpx window is maximised inside the product
  int IC;                        // input maps staged per chunk
  int n_img_max;                 // images the 128 columns of a workgroup can touch
  int MT;                        // map tiles per workgroup: 1, 2 or 4 of 32 maps, or 2 .. 6 of 16
  int TR;                        // maps per tile: 32 (v_mfma_f32_32x32x2_f32) or 16 (v_mfma_f32_16x16x4_f32)
  int KS, chunks_per_slice;      // the k range is cut into KS slices of so many chunks, one per blockIdx.z,
  long long slice_stride;        //   each writing its own plane of `out`, slice_stride floats apart
  int prefetch;                  // the next chunk is fetched into registers during the arithmetic
  int fuse;                      // 0: raw sums (pooling follows); 1: bias + scaled tanh; 2: bias only (output layer)
};
struct BatchPool {
  const CNN_GLOBAL float* sums;  // [batch][Mo][Ho][Wo] raw sums
  const CNN_GLOBAL float* bias;
  CNN_GLOBAL float* out;         // [batch][Mo][Hp][Wp]
  long long total;               // batch * Mo * Hp * Wp
  long long slice_stride;        // floats between the planes of partial sums
  int Mo, Ho, Wo, Kp, Kpx, Hp, Wp, n_slices;  // pooling window Kp rows x Kpx columns
  int act;                       // 1: scaled tanh, 0: none
};
struct BatchPack {
  const CNN_GLOBAL float* w;     // conv: [n_conn][K*Kx] in table order; fc: [n_out][n_in]
  CNN_GLOBAL float* wt;          // [Kdim][MoPad]
  const CNN_GLOBAL int* csr_ptr;
  const CNN_GLOBAL int* csr_idx;
  long long total;               // weights of the layer (biases apart)
  int is_fc, full_table, Mi, Mo, K, Kx, n_in, MoPad;
};

// ---- on-line deformation of training images ---------------------------------------------------
constexpr int DEFORM_MAX_R = 48;          // taps reach 48 pixels either way (sigma up to 16)
constexpr int DEFORM_MAX_PIXELS = 9312;   // rows x (columns rounded up to odd) of one map: four float planes of it fit in LDS

struct DeformJob {
  const CNN_GLOBAL float* src;      // [..][C][H][W]
  CNN_GLOBAL float* dst;            // [n][C][H][W]
  CNN_GLOBAL float* disp;           // [n][2][H][W] (x, then y displacement of every pixel's source), or null
  const CNN_GLOBAL int* src_index;  // [n] source image of every output, or null: output k comes from image k
  long long n, n_src;
  int C, H, W;
  int R;                            // taps on either side of the Gaussian's centre; -1: no elastic part
  double max_tx, max_ty;            // pixels
  double max_rot;                   // radians
  double max_shear, max_scale;      // (the affine part of a source position is worked out in double: in float
                                    // its rounding error grows with the displacement and with the map size)
  float alpha, fill;
  unsigned long long seed, first_index;
  float taps[2 * DEFORM_MAX_R + 1]; // normalised to sum 1
};

}  // namespace cnn355
