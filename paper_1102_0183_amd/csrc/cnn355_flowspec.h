// Resident mode: the shape of a network and the plan of a team, as plain integers, and the planner
// that derives the plan.  Everything here is constexpr, so that the same planner serves the host
// at run time (any network) and the compiler (kernels instantiated for a fixed list of networks,
// in which every size, offset and trip count is then a literal).
#pragma once
#include "cnn355_dev.h"

namespace cnn355 {

// One convolutional layer (with the max-pooling layer folded into it) and its share of a rank's LDS.
struct ConvSpec {
  int Mi, Hi, Wi, Mo, Ho, Wo, K, S, Kp, Hp, Wp;
  int max_conn;     // longest row of the connection table
  int max_back;     // longest column
  int full_table;
  int n_own;        // most output maps a rank owns: ceil(Mo / G)
  int n_own_below;  // most input maps a rank owns (maps of the layer below): ceil(Mi / G); 0 for the first layer
  int pull_shares;  // > 1 (when the layer below has at most half as many maps as there are ranks and a map's pull
                    //   is long enough, FLOW_SHARE_MIN_MACS): the delta pull
                    //   into input map i is shared by the ranks i, i + Mi, ...: share h takes the entries
                    //   [ne h / H, ne (h + 1) / H) of the map's list, holds and adjusts their filters, and hands
                    //   its sums to rank i, the map's owner.  Then n_own_below = 1
  int back_pitch;   // entries per own input map (or share of one) the pull copy has room for
  int wgrad_R_log2; // pooled positions are split 2^this ways when summing a weight gradient
  int pull_chunk;   // output maps rebuilt at full resolution per pass of the delta pull
  int fwd_strip;    // FP: a lane computes a tile of fwd_rows x fwd_strip output pixels (strip 0: one pixel per
  int fwd_rows;     //   lane, any stride)
  int pull_strip;   // same for the delta pull through this layer
  int pull_rows;
  int has_x_out;    // the pooled outputs are exchanged (a convolutional layer follows)
  int in_chunk;     // input maps held in LDS at a time: Mi, or fewer when the plan streams this layer's inputs
  int pull_slots;   // > 0 (pooled layers above the first): the delta pull through this layer visits the pooling
                    //   winners only, pull_slots connections at a time, each adding into a copy of its own of the
                    //   rank's input maps ([pull_slots][n_own_below][Hi*Wi] in the arena); 0: the pull is a
                    //   correlation over whole maps
  // LDS offsets, in floats
  int o_in;     // [Mi][Hi*Wi] inputs of the layer (the image, or every pooled map of the layer below)
  int o_wf;     // [n_own][max_conn][K*K] forward copy of the filters
  int o_bf;     // [n_own] biases
  int o_cidx;   // [n_own][max_conn] input map of every connection (int)
  int o_ncf;    // [n_own] connections of every own map (int)
  int o_wb;     // [n_own_below][back_pitch][K*K] pull copy of the filters, rotated (layers above the first)
  int o_bj;     // [n_own_below][back_pitch] output map of every entry (int)
  int o_ncb;    // [n_own_below] entries of every own input map (int)
  int o_pool;   // [n_own][Hp*Wp] pooled outputs of the own maps
  int o_yx;     // [n_own][Hp*Wp] winner coordinates (y << 16 | x) (int)
  int o_delta;  // [n_own][Hp*Wp] deltas at the winners
  int o_dact;   // [n_own][Hp*Wp] derivative of the activation function at the winners
  int o_tab_fwd;   // [3][WG] every lane's share of the FP job (int), or -1
  int o_tab_pull;  // [3][WG] every lane's share of the pull job (int), or -1
};

struct FcSpec {
  int n_in, n_out, is_output;
  int by_cols;  // second layer only: 1 when its weights are too many to keep a copy in every rank.  Then it is
                // held by columns like the first: rank r has columns r, r + G, ... (at most n_own of them),
                // the ranks exchange partial sums going forward and the deltas of their own inputs going back
  int n_own;    // by_cols: most columns a rank holds, ceil(n_in / G)
  int o_w;      // first layer: [columns of the own maps][n_out]; a layer held by columns: [n_own][n_out];
                // others: [n_out][n_in], every rank
  int o_b;      // [n_out]
  int o_act;    // [n_out]
  int o_delta;  // [n_out]
  int o_dact;   // [n_out] derivative of the activation function (hidden layers)
};

struct FlowSpec {
  int G;            // ranks
  int stride;       // rank r is workgroup r * stride of the launch (8: all ranks on one XCD)
  int n_conv, n_fc;
  int n_col_ranks;  // ranks that own maps of the last convolutional layer (and so columns of the first FC layer)
  int fc1_owned;    // 1: each sum of the first FC layer is added up by one rank (k mod G) and sent round; 0: by every rank
  int n_classes;
  int lds_floats;
  int o_act;        // [max n_own*Ho*Wo] full-resolution outputs of the own maps of the layer being computed
  int o_part;       // partial sums
  int o_scratch;    // delta maps of a chunk of output maps rebuilt at full resolution, zero border included
  int scratch_floats;
  int o_dall;       // [max Mo*Hp*Wp] deltas of every map of the layer being pulled through
  int o_yxall;      // same, winner coordinates
  int out_units;    // 0 soft-max + cross-entropy, 1 scaled tanh + squared error
  int defer;        // 1: weight adjustments nobody is waiting for are put off into the next image's waits
  int o_prev;       // [conv[1].n_own_below * Hi * Wi] the own pooled maps of the first layer, previous image
  int stream;       // 1: the inputs of every convolutional layer above the first do not stay in LDS: FP and the
                    //    adjustment of the forward copy walk them chunk by chunk (in_chunk maps at a time, fetched
                    //    from the exchange buffers into the arena the delta pull uses for its zero-bordered maps)
  int arena_shared; // 1: the pull that correlates over whole maps cannot count on its arena of zero-bordered delta
                    //    maps being zero from the last use (input chunks of a streamed plan, or the copies of
                    //    another layer's winners-only pull, lie there in between) and clears it before every use
  ConvSpec conv[FLOW_MAX_CONV];
  FcSpec fc[FLOW_MAX_FC];
};

// reasons a network cannot run in resident mode
enum FlowWhy : int {
  FLOW_OK = 0, FLOW_NO_CONV, FLOW_TOO_MANY_LAYERS, FLOW_BAD_STRIDE, FLOW_TOO_LARGE, FLOW_NO_LDS
};

constexpr int flow_min(int a, int b) { return a < b ? a : b; }
constexpr int flow_max(int a, int b) { return a > b ? a : b; }
constexpr long long flow_minl(long long a, long long b) { return a < b ? a : b; }
constexpr long long flow_maxl(long long a, long long b) { return a > b ? a : b; }

// How many ways U units share their (at most max_cnt) connections over the WG lanes: as many as fit,
// then the fewest ways that still need no more passes over the connections per lane.
constexpr int flow_split_ways(int U, int max_cnt) {
  if (U >= WG || U < 1) return 1;
  const int r_max = flow_max(1, flow_min(WG / U, max_cnt));
  const int iters = (max_cnt + r_max - 1) / r_max;
  return (max_cnt + iters - 1) / iters;
}
// floats of one zero-bordered delta map of the pull through a layer whose input maps are Hi x Wi: odd, so that
// lanes that read the same place of different maps fall on different LDS banks
constexpr long long flow_border_map(int Hi, int Wi, int K) { return ((long long)(Hi + K - 1) * (Wi + K - 1)) | 1; }
// The pull that visits winners only (pull_slots): a connection's HW winners are taken by UW lanes at a time
// (all of them when HW <= 64, else HW split into the fewest equal parts of at most 64), and a workgroup works on
// (WG / 64) * (64 / UW) such units at once when it has room for as many copies of its input maps.
// A fully connected layer behind the first is kept whole by every rank up to this many weights; a larger second
// layer (300N-100N of Sec. 4.3: 30 000) is held by columns instead, at the price of two more crossings per image.
constexpr int FLOW_FC_REPLICATE_MAX = 8192;
// Partial sums of the first fully connected layer (ranks with columns x outputs) up to which every rank reads all
// of them; beyond, reading them is what the step waits for, and one rank per output adds them up and sends the sum on.
constexpr int FLOW_FC1_DIRECT_MAX = 16384;
// Any pooling at all makes it pay (measured: 2 x 2 rectangles, a quarter of the terms: cfg4a 55.8 -> 54.0 us per
// image, cfg5 16.5 -> 16.2; 3 x 3 and 4 x 4: the benchmark net 16.3 -> 15.6, cfg3 43.3 -> 38.1).
constexpr int FLOW_WINNERS_MIN_KP = 2;
constexpr int flow_winner_parts(int HW) { return (HW + 63) / 64; }
constexpr int flow_winner_lanes(int HW) { return (HW + flow_winner_parts(HW) - 1) / flow_winner_parts(HW); }
constexpr int flow_winner_slots_max(int HW) { return (WG / 64) * (64 / flow_winner_lanes(HW)); }
// floats of partial sums a job of n_maps (or one map fewer: ranks differ by one) maps needs
constexpr long long flow_part_need(int strip, int th, int n_maps, int rows, int width, int max_cnt) {
  long long need = 0;
  for (int nm = flow_max(1, n_maps - 1); nm <= n_maps; ++nm) {
    const int U = strip ? nm * ((rows + th - 1) / th) * ((width + strip - 1) / strip) : nm * rows * width;
    need = flow_maxl(need, (long long)flow_split_ways(U, max_cnt) * nm * rows * width);
  }
  return need;
}

// Tile for a correlation job of n_maps maps of rows x width pixels with up to max_cnt connections
// each: rows (1 or 2) x strip (4, 5 or 7 pixels) per lane, the combination with the shortest
// estimated time once the connections are shared over the spare lanes (the rule the kernel
// applies).  Two things bound that time: the multiply-adds of one lane (a wavefront issues one
// vector instruction per about 5 cycles, however many wavefronts share its SIMD), and the LDS
// reads of all wavefronts together (128 bytes per cycle and compute unit: 2 cycles per wavefront
// read; with 3, to allow for bank conflicts, a sweep over all tiles showed the model passing over the fastest).  0 = one pixel per lane (any stride, any kernel size); tiles exist
// for strides 1 and 2 and kernels of 2 to 5.
// Returns strip + 16 * rows.
// The most lanes of a wavefront whose reads of one tap fall into one LDS bank (32 banks of one float): the lanes
// of a wavefront read the same tap of their tiles at once, so this many reads go through one bank one after the
// other (2 at best: 64 lanes, 32 banks).  Lane u takes tile t = u mod U and way u / U of the connections (side:
// way u mod ways, tile u / ways), tiles numbered (map, band of th rows, strip of sw pixels) as the kernel deals
// them out; a way further on reads a map further on.  pitch: floats from one input row to the next, map: from one
// map to the next.
constexpr int flow_bank_load(int n_maps, int rows, int width, int th, int sw, int stride, int pitch, long long map,
                             long long ways, int side) {
  const int NS = (width + sw - 1) / sw, NG = (rows + th - 1) / th;
  const long long U = (long long)n_maps * NG * NS;
  int cnt[32] = {};
  int worst = 0;
  for (int u = 0; u < 64; ++u) {
    const long long t = side ? u / ways : u % U, r = side ? u % ways : u / U;
    if (t >= U || r >= ways) continue;
    const int row = (int)(t / NS), sx = (int)(t - (long long)row * NS);
    const int am = row / NG, y = (row - am * NG) * th;
    const long long a = (long long)(y * pitch + sx * sw) * stride + (am + r) * map;
    const int b = (int)(a & 31);
    if (++cnt[b] > worst) worst = cnt[b];
  }
  return worst;
}

// FLOW_BANK_LOAD_MAX: how many reads of one tap may queue at one bank before the tile is chosen with the queues in
// the bill.  Up to there the bill without them picks better (measured on the benchmark net: its queues of 3 to 4
// cost less than the lanes a taller tile leaves idle); beyond, e.g. with input rows of 14, 22, 32 or 48 floats under
// strips of 4, a read takes 5 to 16 turns and the strips of 5 or 7 that spread over the banks win.
constexpr int FLOW_BANK_LOAD_MAX = 4;
constexpr int flow_tile_pick(int K, int stride, int n_maps, int rows, int width, int max_cnt, int pitch, long long map,
                             int side, bool with_banks, int* load_of_best) {
  int best = 4 + 16;
  long long best_cost = -1;
  const int widths[3] = {4, 5, 7};
  // a skipping factor of 1: one row per tile, strips of 4 or 5 (the rows a lane keeps grow with the stride)
  for (int th = 1; th <= (stride == 1 ? 2 : 1); ++th)
    for (int wi = 0; wi < (stride == 1 ? 3 : 2); ++wi) {
      const int sw = widths[wi];
      const long long U = (long long)n_maps * ((rows + th - 1) / th) * ((width + sw - 1) / sw);
      long long iters = max_cnt;
      if (U < WG) {
        const long long r_max = flow_maxl(1, flow_minl(WG / U, max_cnt));
        iters = (max_cnt + r_max - 1) / r_max;
      }
      const long long passes = (U + WG - 1) / WG;
      const long long macs = (long long)th * sw * K * K;
      const long long reads = (long long)((th - 1) * stride + K) * ((sw - 1) * stride + K) + K * K;
      const long long ways = (max_cnt + iters - 1) / iters;
      const long long waves = (flow_minl(U * ways, WG) + 63) / 64;
      const int load = flow_bank_load(n_maps, rows, width, th, sw, stride, pitch, map, ways, side);
      const long long valu = iters * macs * 5, lds = waves * iters * reads * ((with_banks && load > 2) ? load : 2);
      long long cost = passes * ((valu > lds ? valu : lds) + 200);
      // partial sums beyond 32 KB crowd out the weights and maps a rank must hold: last resort only
      if (flow_part_need(sw, th, n_maps, rows, width, max_cnt) > 8 * WG) cost += 1000000;
      if (best_cost < 0 || cost < best_cost) { best_cost = cost; best = sw + 16 * th; *load_of_best = load; }
    }
  return best;
}
constexpr int flow_tile_for(int K, int stride, int n_maps, int rows, int width, int max_cnt, int pitch, long long map,
                            int side) {
  if (stride < 1 || stride > 2 || K < 2 || K > 5) return 0;
  int load = 0;
  const int plain = flow_tile_pick(K, stride, n_maps, rows, width, max_cnt, pitch, map, side, false, &load);
  if (load <= FLOW_BANK_LOAD_MAX) return plain;
  return flow_tile_pick(K, stride, n_maps, rows, width, max_cnt, pitch, map, side, true, &load);
}

// Choose the team and lay out every rank's LDS.  On entry Z holds the shape (n_conv, n_fc,
// n_classes, out_units, and per layer Mi..Wp, max_conn, max_back, full_table / n_in, n_out, is_output); on
// success the rest of Z is filled in.  team_ranks / team_stride: 0 = automatic.
constexpr int flow_plan_as(FlowSpec& Z, int team_ranks, int team_stride, int n_cu, int stream) {
  const int n_conv = Z.n_conv, n_fc = Z.n_fc;
  Z.stream = stream;
  if (n_conv < 1) return FLOW_NO_CONV;
  if (n_conv > FLOW_MAX_CONV || n_fc > FLOW_MAX_FC || n_fc < 1) return FLOW_TOO_MANY_LAYERS;
  int max_maps = 1;
  for (int l = 0; l < n_conv; ++l) max_maps = flow_max(max_maps, Z.conv[l].Mo);
  int stride = team_stride > 0 ? team_stride : 0;
  int G = team_ranks > 0 ? team_ranks : max_maps;
  if (n_cu <= 0) n_cu = 256;
  if (stride == 0) stride = (G <= n_cu / 8) ? 8 : 1;
  if (stride != 1 && stride != 8) return FLOW_BAD_STRIDE;
  G = flow_max(1, flow_min(flow_min(G, max_maps), n_cu / stride));
  Z.G = G;
  Z.stride = stride;

  long long off = 0;
  auto take = [&off](long long n) {
    const long long o = off;
    off += (n + 3) / 4 * 4;
    return (int)flow_minl(o, 1 << 30);
  };
  long long max_act = 1, max_part = WG, max_dall = 1, max_hwd = 0;
  for (int l = 0; l < n_conv; ++l) {
    ConvSpec& C = Z.conv[l];
    const int KK = C.K * C.K, HW = C.Hp * C.Wp;
    if (C.Ho >= 32768 || C.Wo >= 65536) return FLOW_TOO_LARGE;
    if ((long long)C.Mi * C.Hi * C.Wi >= (1 << 20) || (long long)C.Mo * C.Ho * C.Wo >= (1 << 20)) return FLOW_TOO_LARGE;
    C.n_own = (C.Mo + G - 1) / G;
    C.n_own_below = l >= 1 ? (C.Mi + G - 1) / G : 0;
    C.max_back = flow_max(1, C.max_back);
    // (handing the sums over costs the owner a round trip through the L2, about what 2^17 multiply-adds of a
    // map's pull take, so two shares pay from twice that: measured, sharing gains 1.5 us on 80 entries of 5x5
    // into 13x13 maps and loses 0.8 us on 40 of them)
    // (a plan that streams its inputs does not share pulls: a share adjusts its filters from an input map of the
    // layer, which then is not at hand)
    // (a pull that visits the pooling winners only is too short to be worth the hand-over: not shared)
    const bool winners_only = l >= 1 && C.Kp >= FLOW_WINNERS_MIN_KP;
    C.pull_slots = 0;
    C.pull_shares = (l >= 1 && !stream && !winners_only && 2 * C.Mi <= G &&
                     (long long)C.max_back * KK * C.Hi * C.Wi >= FLOW_SHARE_MIN_MACS)
                        ? G / C.Mi : 1;
    C.back_pitch = (C.max_back + C.pull_shares - 1) / C.pull_shares;
    C.has_x_out = (l + 1 < n_conv) ? 1 : 0;
    C.in_chunk = C.Mi;
    C.o_in = (stream && l >= 1) ? 0 : take((long long)C.Mi * C.Hi * C.Wi);   // (streamed: the arena, set below)
    C.o_wf = take((long long)C.n_own * C.max_conn * KK);
    C.o_bf = take(C.n_own);
    C.o_cidx = take((long long)C.n_own * C.max_conn);
    C.o_ncf = take(C.n_own);
    {
      const int tile = flow_tile_for(C.K, C.S + 1, C.n_own, C.Ho, C.Wo, C.max_conn, C.Wi, (long long)C.Hi * C.Wi, 0);
      C.fwd_strip = tile & 15; C.fwd_rows = tile ? tile >> 4 : 1;
    }
    C.o_wb = 0; C.o_bj = 0; C.o_ncb = 0; C.pull_strip = 0; C.pull_rows = 1; C.pull_chunk = 1;
    if (l >= 1) {
      C.o_wb = take((long long)C.n_own_below * C.back_pitch * KK);
      C.o_bj = take((long long)C.n_own_below * C.back_pitch);
      C.o_ncb = take(C.n_own_below);
      {
        const int tile = flow_tile_for(C.K, 1, C.n_own_below, C.Hi, C.Wi, C.back_pitch, C.Wi + C.K - 1,
                                       flow_border_map(C.Hi, C.Wi, C.K), C.K & 1);
        C.pull_strip = tile & 15; C.pull_rows = tile ? tile >> 4 : 1;
      }
      max_dall = flow_maxl(max_dall, (long long)C.Mo * HW);
      if (winners_only) {   // at least one copy of the own input maps
        max_hwd = flow_maxl(max_hwd, (long long)C.n_own_below * C.Hi * C.Wi);
      } else {
        max_hwd = flow_maxl(max_hwd, flow_border_map(C.Hi, C.Wi, C.K));
        max_part = flow_maxl(max_part, flow_part_need(C.pull_strip, C.pull_rows, C.n_own_below, C.Hi, C.Wi,
                                                      flow_min(C.back_pitch, C.Mo)));
      }
    }
    C.o_pool = take((long long)C.n_own * HW);
    C.o_yx = take((long long)C.n_own * HW);
    C.o_delta = take((long long)C.n_own * HW);
    C.o_dact = take((long long)C.n_own * HW);
    max_act = flow_maxl(max_act, (long long)C.n_own * C.Ho * C.Wo);
    max_part = flow_maxl(max_part, flow_part_need(C.fwd_strip, C.fwd_rows, C.n_own, C.Ho, C.Wo, C.max_conn));
    // pooled positions split R ways when a rank has few weights to adjust (same R for both copies)
    long long n_w = (long long)C.n_own * C.max_conn * KK;
    if (l >= 1) n_w = flow_minl(n_w, (long long)C.n_own_below * C.back_pitch * KK);
    int rl2 = 0;
    while (rl2 < 6 && (n_w << (rl2 + 1)) <= WG && (2 << rl2) <= HW) ++rl2;
    C.wgrad_R_log2 = rl2;
    C.o_tab_fwd = -1;
    C.o_tab_pull = -1;
  }
  const ConvSpec& Cl = Z.conv[n_conv - 1];
  Z.n_col_ranks = flow_min(G, Cl.Mo);
  Z.fc1_owned = ((long long)Z.n_col_ranks * Z.fc[0].n_out > FLOW_FC1_DIRECT_MAX) ? 1 : 0;
  for (int f = 0; f < n_fc; ++f) {
    FcSpec& Q = Z.fc[f];
    Q.by_cols = (f == 1 && !Q.is_output && (long long)Q.n_out * Q.n_in > FLOW_FC_REPLICATE_MAX) ? 1 : 0;
    Q.n_own = Q.by_cols ? (Q.n_in + G - 1) / G : 0;
    Q.o_w = take(f == 0 ? (long long)Cl.n_own * Cl.Hp * Cl.Wp * Q.n_out
                        : Q.by_cols ? (long long)Q.n_own * Q.n_out : (long long)Q.n_out * Q.n_in);
    Q.o_b = take(Q.n_out);
    Q.o_act = take(Q.n_out);
    Q.o_delta = take(Q.n_out);
    Q.o_dact = take(Q.n_out);
  }
  max_part = flow_maxl(max_part, max_act);   // (the pooling step lays the own maps' outputs out there)
  Z.o_act = take(max_act);
  Z.o_part = take(stream ? 0 : max_part);   // (streamed plan: the partial sums go into the arena, see below)
  Z.o_dall = take(n_conv > 1 ? max_dall : 0);
  Z.o_yxall = take(n_conv > 1 ? max_dall : 0);
  Z.defer = 0;
  Z.o_prev = 0;
  // tiles read a few floats past the end of the last row of a map, and a row past its last row
  long long pad = 16;
  for (int l = 1; l < n_conv; ++l) pad = flow_maxl(pad, 16 + Z.conv[l].Wi + Z.conv[l].K);
  long long need = n_conv > 1 ? max_hwd + pad : pad;
  if (stream) {
    for (int l = 1; l < n_conv; ++l) need = flow_maxl(need, (long long)Z.conv[l].Hi * Z.conv[l].Wi + pad);
    // a job's partial sums are stored when its last chunk of maps has been read: they share the arena
    need = flow_maxl(need, max_part);
  }
  if (off + need > FLOW_LDS_FLOATS_MAX) return FLOW_NO_LDS;
  if (n_conv > 1) {
    const long long prev = (long long)Z.conv[1].n_own_below * Z.conv[1].Hi * Z.conv[1].Wi;
    if (off + prev + need <= FLOW_LDS_FLOATS_MAX) {
      Z.o_prev = take(prev);
      Z.defer = 1;
    }
  }
  // Lane tables of the correlation jobs (a rank decodes its share of a job once instead of once per
  // image), the first layers' jobs first -- but only where a table does not cost the pull a pass:
  // the zero-bordered delta maps below get what is left, and every pass over a chunk of them costs
  // more than decoding a job again.
  auto pull_passes = [&](long long floats) {   // (summed over the layers: a table must not cost any of them a pass)
    long long total = 0;
    for (int l = 1; l < n_conv; ++l) {
      const ConvSpec& C = Z.conv[l];
      if (C.Kp >= FLOW_WINNERS_MIN_KP) {   // winners only: rounds of as many connections as there are copies
        const long long copy = (long long)C.n_own_below * C.Hi * C.Wi;
        const long long units = (long long)C.n_own_below * C.back_pitch * flow_winner_parts(C.Hp * C.Wp);
        const long long sl = flow_maxl(1, flow_minl(flow_minl(flow_winner_slots_max(C.Hp * C.Wp), units), floats / copy));
        total += (units + sl - 1) / sl;
      } else {
        const long long hwd = flow_border_map(C.Hi, C.Wi, C.K);
        const long long chunk = flow_maxl(1, flow_minl(C.Mo, (floats - pad) / hwd));
        total += (C.Mo + chunk - 1) / chunk;
      }
      if (stream) {  // the chunks of input maps FP walks through the same arena
        const long long ic = flow_maxl(1, flow_minl(C.Mi, (floats - pad) / ((long long)C.Hi * C.Wi)));
        total += (C.Mi + ic - 1) / ic;
      }
    }
    return total;
  };
  for (int l = 0; l < n_conv; ++l) {
    const long long free_now = (long long)FLOW_LDS_FLOATS_MAX - off;
    if (Z.conv[l].n_own < 1024 && off + need + 3 * WG <= FLOW_LDS_FLOATS_MAX &&
        pull_passes(free_now - 3 * WG) == pull_passes(free_now))
      Z.conv[l].o_tab_fwd = take(3 * WG);
    const long long free_then = (long long)FLOW_LDS_FLOATS_MAX - off;
    if (l >= 1 && Z.conv[l].Kp < FLOW_WINNERS_MIN_KP && Z.conv[l].n_own_below < 1024 && off + need + 3 * WG <= FLOW_LDS_FLOATS_MAX &&
        pull_passes(free_then - 3 * WG) == pull_passes(free_then))
      Z.conv[l].o_tab_pull = take(3 * WG);
  }
  // the zero-bordered delta maps of the pull: the more fit, the fewer passes
  long long scratch = need;
  for (int l = 1; l < n_conv; ++l) {
    const ConvSpec& C = Z.conv[l];
    if (C.Kp >= FLOW_WINNERS_MIN_KP) {
      const long long units = (long long)C.n_own_below * C.back_pitch * flow_winner_parts(C.Hp * C.Wp);
      scratch = flow_maxl(scratch, flow_minl(flow_winner_slots_max(C.Hp * C.Wp), units) * C.n_own_below * C.Hi * C.Wi);
    } else {
      scratch = flow_maxl(scratch, (long long)C.Mo * flow_border_map(C.Hi, C.Wi, C.K) + pad);
    }
  }
  if (stream)
    for (int l = 1; l < n_conv; ++l) scratch = flow_maxl(scratch, (long long)Z.conv[l].Mi * Z.conv[l].Hi * Z.conv[l].Wi + pad);
  scratch = flow_minl(scratch, (long long)FLOW_LDS_FLOATS_MAX - off);
  Z.o_scratch = take(scratch);
  Z.scratch_floats = (int)scratch;
  Z.lds_floats = (int)off;
  Z.arena_shared = stream ? 1 : 0;
  for (int l = 1; l < n_conv; ++l)
    if (Z.conv[l].Kp >= FLOW_WINNERS_MIN_KP) Z.arena_shared = 1;
  for (int l = 1; l < n_conv; ++l) {
    ConvSpec& C = Z.conv[l];
    const long long hwd = flow_border_map(C.Hi, C.Wi, C.K);
    C.pull_chunk = (int)flow_maxl(1, flow_minl(C.Mo, (scratch - pad) / hwd));
    if (C.Kp >= FLOW_WINNERS_MIN_KP) {
      const long long units = (long long)C.n_own_below * C.back_pitch * flow_winner_parts(C.Hp * C.Wp);
      C.pull_slots = (int)flow_minl(flow_minl(flow_winner_slots_max(C.Hp * C.Wp), units),
                                    scratch / ((long long)C.n_own_below * C.Hi * C.Wi));
    }
    if (stream) {
      // the pull stores its partial sums in the arena after its one walk over the delta maps: a job with
      // more units than lanes would walk them again and meet its own sums there
      const long long U = C.pull_strip
          ? (long long)C.n_own_below * ((C.Hi + C.pull_rows - 1) / C.pull_rows) * ((C.Wi + C.pull_strip - 1) / C.pull_strip)
          : (long long)C.n_own_below * C.Hi * C.Wi;
      if (C.pull_slots == 0 && U > WG) return FLOW_NO_LDS;
      Z.o_part = Z.o_scratch;
      C.o_in = Z.o_scratch;
      C.in_chunk = (int)flow_maxl(1, flow_minl(C.Mi, (scratch - pad) / ((long long)C.Hi * C.Wi)));
    }
  }
  return FLOW_OK;
}

// The plan that keeps every layer's inputs in LDS where that fits (the fewest fetches), else the one that
// streams them.
constexpr int flow_plan(FlowSpec& Z, int team_ranks, int team_stride, int n_cu) {
  const int rc = flow_plan_as(Z, team_ranks, team_stride, n_cu, 0);
  if (rc != FLOW_NO_LDS || Z.n_conv < 2) return rc;
  return flow_plan_as(Z, team_ranks, team_stride, n_cu, 1);
}

// ---- networks the resident kernel is also compiled for, every size a literal --------------------
// A network of convolutional layers, each followed by max-pooling of Kp (1 = none), then fully
// connected layers; Eq. 1 of Sec. 2.2 gives the map sizes.  fan_in = 0: full connection table; else every
// output map reads fan_in input maps and the busiest input map is read by max_back output maps (the plan
// depends on a table through these two numbers only).
struct StaticConv { int maps, K, S, Kp, fan_in, max_back; };
constexpr FlowSpec flow_static_spec(int C0, int H0, int W0, int n_conv, const StaticConv* conv, int n_fc, const int* fc,
                                    int team_ranks, int team_stride) {
  FlowSpec Z{};
  Z.n_conv = n_conv;
  Z.n_fc = n_fc;
  int m = C0, h = H0, w = W0;
  for (int l = 0; l < n_conv; ++l) {
    ConvSpec& C = Z.conv[l];
    C.Mi = m; C.Hi = h; C.Wi = w;
    C.Mo = conv[l].maps; C.K = conv[l].K; C.S = conv[l].S; C.Kp = conv[l].Kp;
    C.Ho = (h - C.K) / (C.S + 1) + 1;
    C.Wo = (w - C.K) / (C.S + 1) + 1;
    C.Hp = C.Ho / C.Kp; C.Wp = C.Wo / C.Kp;
    C.max_conn = m; C.max_back = C.Mo; C.full_table = 1;
    if (conv[l].fan_in > 0) { C.max_conn = conv[l].fan_in; C.max_back = conv[l].max_back; C.full_table = 0; }
    m = C.Mo; h = C.Hp; w = C.Wp;
  }
  int n_in = m * h * w;
  for (int f = 0; f < n_fc; ++f) {
    Z.fc[f].n_in = n_in;
    Z.fc[f].n_out = fc[f];
    Z.fc[f].is_output = (f + 1 == n_fc) ? 1 : 0;
    n_in = fc[f];
  }
  Z.n_classes = n_in;
  flow_plan(Z, team_ranks, team_stride, 256);
  return Z;
}

// 1: 1x29x29-20C4-MP2-40C5-MP3-150N-10N (the benchmark network), automatic team
// 2: 1x29x29-40C4-MP2-80C5-MP3-300N-10N, automatic team
// 3: 4x44x44-40C5S1-MP2-80C3-MP2-100N-5N behind a fixed first layer, the second convolution reading 20 of the 40
//    maps with the busiest map read 49 times (the benchmark's seeded table), automatic team
// 4: 2x48x48-50C5-MP2-128C3-MP4-100N-5N, automatic team (a streamed plan)
// 5: 3x32x32-100C5-MP2-100C5-MP2-100C4-MP2-300N-10N, automatic team (a streamed plan)
constexpr int FLOW_N_STATIC = 5;
template <int ID>
struct StaticSpec;
template <>
struct StaticSpec<1> {
  static constexpr StaticConv conv[2] = {{20, 4, 0, 2, 0, 0}, {40, 5, 0, 3, 0, 0}};
  static constexpr int fc[2] = {150, 10};
  static constexpr FlowSpec value = flow_static_spec(1, 29, 29, 2, conv, 2, fc, 0, 0);
};
template <>
struct StaticSpec<2> {
  static constexpr StaticConv conv[2] = {{40, 4, 0, 2, 0, 0}, {80, 5, 0, 3, 0, 0}};
  static constexpr int fc[2] = {300, 10};
  static constexpr FlowSpec value = flow_static_spec(1, 29, 29, 2, conv, 2, fc, 0, 0);
};

template <>
struct StaticSpec<3> {
  static constexpr StaticConv conv[2] = {{40, 5, 1, 2, 0, 0}, {80, 3, 0, 2, 20, 49}};
  static constexpr int fc[2] = {100, 5};
  static constexpr FlowSpec value = flow_static_spec(4, 44, 44, 2, conv, 2, fc, 0, 0);
};

template <>
struct StaticSpec<4> {
  static constexpr StaticConv conv[2] = {{50, 5, 0, 2, 0, 0}, {128, 3, 0, 4, 0, 0}};
  static constexpr int fc[2] = {100, 5};
  static constexpr FlowSpec value = flow_static_spec(2, 48, 48, 2, conv, 2, fc, 0, 0);
};
template <>
struct StaticSpec<5> {
  static constexpr StaticConv conv[3] = {{100, 5, 0, 2, 0, 0}, {100, 5, 0, 2, 0, 0}, {100, 4, 0, 2, 0, 0}};
  static constexpr int fc[2] = {300, 10};
  static constexpr FlowSpec value = flow_static_spec(3, 32, 32, 3, conv, 2, fc, 0, 0);
};

// One more, defined outside this file: the network of a handle, written out by cnn_resident_spec_source() as a
// header that specialises StaticSpec<FLOW_SPECIAL_ID>.  cnn355_flow.hip compiled with -DCNN355_SPECIAL_HEADER="<that
// header>" gives a code object that holds k_resident<FLOW_SPECIAL_ID> and its plan (cnn355_special_plan) and nothing
// else; cnn_load_resident_code() loads it into a handle whose run-time plan equals that plan word for word.
constexpr int FLOW_SPECIAL_ID = 99;
#ifdef CNN355_SPECIAL_HEADER
#include CNN355_SPECIAL_HEADER
#endif

}  // namespace cnn355
