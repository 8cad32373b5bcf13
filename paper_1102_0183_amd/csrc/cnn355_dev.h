// Descriptors shared by the host planner and the gfx950 kernels.  Plain data only.
#pragma once
#include <stddef.h>
#include <stdint.h>

namespace cnn355 {

constexpr int WG = 256;  // threads per workgroup: 4 wavefronts of 64

// LDS carve-up, in floats.  One static block per workgroup; every stage cuts it its own way.
constexpr int LDS_IN = 8192;    // staged input maps (32 KB)
constexpr int LDS_AUX = 3072;   // filters / deltas
constexpr int LDS_AUX2 = 3072;  // arg-max coordinates
constexpr int LDS_RED = 1280;   // cross-split partial sums (256) + one output tile (1024)
constexpr int LDS_FLOATS = LDS_IN + LDS_AUX + LDS_AUX2 + LDS_RED;  // 15616 floats = 61 KB

constexpr int MAX_TILE_PIX = 1024;   // conv outputs per workgroup tile (4 per thread)
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
  // convolution geometry: Mi maps of Hi x Wi in, Mo maps of Ho x Wo out, K x K kernel,
  // skipping factor S (stride S+1), pooled by Kp to Hp x Wp
  int Mi, Hi, Wi, Mo, Ho, Wo, K, S, Kp, Hp, Wp;
  int n_in, n_out;     // fully connected: W is [n_out][n_in]
  int is_output;       // soft-max output layer
  int in_is_image;     // input is the image handed to the call (no stored activation below)
  int max_conn;        // longest row of the connection table
  int pad0;
  const float* in;     // input activations (NULL when in_is_image)
  float* act;          // conv: after tanh, full resolution; fc: after tanh / probabilities
  float* out;          // what the layer above reads (conv: pooled values; fc: == act)
  uint8_t* arg;        // conv: winner index dy*Kp+dx per pooled position
  int* argyx;          // conv: (y << 16) | x of the winner in conv-output coordinates
  float* delta;        // dE/d(pre-activation): conv at the winners [Mo][Hp][Wp]; fc [n_out]
  float* bias;
  float* w;            // conv: one K*K block per connection, CSR order; fc: [n_out][n_in]
  long long w_canon;   // offset of w in the canonical weight vector (for gradient taps)
  long long b_canon;
  const int* csr_ptr;  // [Mo+1] forward table (C^n of Sec. 3.1): row j -> slots
  const int* csr_idx;  // [n_conn] input map of every slot
  const int* csc_ptr;  // [Mi+1] backward table (C_BP of Sec. 3.1): input map i -> entries
  const int* csc_j;    // [n_conn] output map of every entry
  const int* csc_slot; // [n_conn] weight slot of every entry (WIDX_BP of Sec. 3.1)
};

enum StageKind : int {
  ST_FRONTEND = 1,   // fixed image-processing filters
  ST_CONV_FWD = 2,   // convolution + bias + tanh + max-pool + arg-max
  ST_FC_FWD = 3,     // hidden fully connected layer + tanh
  ST_HEAD = 4,       // output layer, soft-max, error, output delta, and its own backward+update
  ST_FC_BWD = 5,     // hidden fully connected layer: pull deltas + update its weights
  ST_CONV_BWD = 6,   // pull deltas through a convolutional layer
  ST_CONV_WGRAD = 7, // convolutional weight gradients + update
};

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
  int tw_log2;        // log2 of the lane group width used when staging one map
  int pix_per_thread; // CONV_FWD: 1 or 4
  int rows_per_wg;    // FC_FWD: 1, 2 or 4
  int cm_log2;        // FC_BWD / HEAD: log2 of columns per tile
};

struct FrontendDev {
  int n_filters, K, n_src, Hr, Wr, H, W;  // raw image n_src x Hr x Wr -> n_filters x H x W
  int pad;
  const float* filters;  // [n_filters][K][K]
  const int* src;        // [n_filters]
  float* out;            // [n_filters][H][W]
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
};

// Per-call arguments.
struct RunArgs {
  const float* images;   // first image
  const int* labels;     // device labels, or NULL to use label_imm
  float* probs_out;      // optional [n_images][n_classes]
  float* grad_out;       // when set: store dE/dw here (canonical order) instead of updating
  long long n_images;
  long long image_stride; // floats
  int label_imm;
  int train;             // 0: forward only
  float lr;
  unsigned int spin_limit; // grid-barrier polls before giving up
};

}  // namespace cnn355
