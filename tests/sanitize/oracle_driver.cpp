// Host sanitizer run of the CPU oracle (test infrastructure): the whole oracle source compiled with
// -fsanitize=address,undefined into this driver, which walks its C entry points over a set of small networks --
// skipping factors, sparse tables, rectangular kernels and pooling, a fixed front-end, both output kinds, both
// precisions, error paths.  Any report of the sanitizers ends the program with a non-zero status.
#include "../../oracle/cnn_oracle.cpp"

#include <cstdio>
#include <random>

static int fails = 0;
#define EXPECT(c) do { if (!(c)) { std::printf("FAILED line %d: %s\n", __LINE__, #c); ++fails; } } while (0)

static void run_net(const char* arch, int precision, int sparse_conv, int frontend_k, int out_units, unsigned seed) {
  oracle_t* h = nullptr;
  EXPECT(oracle_create(arch, precision, &h) == 0);
  if (!h) return;
  std::mt19937 rng(seed);
  std::uniform_real_distribution<double> U(-1.0, 1.0);
  const int n_layers = oracle_num_layers(h);
  if (sparse_conv >= 0) {
    int seen = 0;
    for (int l = 1; l < n_layers; ++l) {
      int32_t a[8], p[8];
      oracle_layer_info(h, l, a);
      oracle_layer_info(h, l - 1, p);
      if (a[0] != 1 || seen++ != sparse_conv) continue;
      std::vector<uint8_t> t((size_t)a[1] * p[1], 0);
      for (int j = 0; j < a[1]; ++j)
        for (int i = 0; i < p[1]; ++i) t[(size_t)j * p[1] + i] = ((i + j) % 2 == 0) || i == j % p[1];
      EXPECT(oracle_set_connection_table(h, sparse_conv, t.data()) == 0);
    }
  }
  int32_t in0[8];
  oracle_layer_info(h, 0, in0);
  if (frontend_k > 0) {
    std::vector<float> filt((size_t)in0[1] * frontend_k * frontend_k);
    for (float& v : filt) v = (float)U(rng) * 0.2f;
    std::vector<int32_t> src(in0[1]);
    for (int f = 0; f < in0[1]; ++f) src[f] = f % 2;
    EXPECT(oracle_set_fixed_frontend(h, in0[1], frontend_k, 2, filt.data(), src.data()) == 0);
  }
  EXPECT(oracle_set_output_units(h, out_units) == 0);
  const size_t nw = oracle_num_weights(h), sz = oracle_image_size(h);
  std::vector<double> w(nw), g(nw);
  for (double& v : w) v = 0.3 * U(rng);
  EXPECT(oracle_set_weights(h, w.data(), nw) == 0);
  EXPECT(oracle_set_weights(h, w.data(), nw + 1) != 0);
  const int n = 4;
  std::vector<float> img(sz * n);
  for (float& v : img) v = (float)U(rng);
  int32_t last[8];
  oracle_layer_info(h, n_layers - 1, last);
  const int n_cls = last[1];
  std::vector<int32_t> lab(n);
  for (int t = 0; t < n; ++t) lab[t] = (int)(rng() % n_cls);
  std::vector<double> probs((size_t)n * n_cls);
  double loss = 0;
  EXPECT(oracle_forward(h, img.data(), probs.data()) == 0);
  EXPECT(oracle_gradients(h, img.data(), lab[0], g.data(), &loss) == 0);
  EXPECT(std::isfinite(loss));
  EXPECT(oracle_gradients(h, img.data(), n_cls, g.data(), &loss) != 0);   // label out of range
  EXPECT(oracle_loss(h, img.data() + sz, lab[1], &loss) == 0);
  for (int l = 1; l < n_layers; ++l) {
    int32_t a[8];
    oracle_layer_info(h, l, a);
    std::vector<double> buf((size_t)a[1] * a[2] * a[3]);
    EXPECT(oracle_get_activation(h, l, buf.data()) == 0);
    if (a[0] == 2) {
      std::vector<uint8_t> arg(buf.size());
      EXPECT(oracle_get_argmax(h, l, arg.data()) == 0);
      int ad = 0, rj = 0;
      EXPECT(oracle_adopt_argmax_hint(h, l, arg.data(), 1e-5, &ad, &rj) == 0);
      EXPECT(ad == 0 && rj == 0);
    } else {
      EXPECT(oracle_get_delta(h, l, buf.data()) == 0);
    }
  }
  EXPECT(oracle_train_step(h, img.data(), lab[0], 0.01, &loss) == 0);
  EXPECT(oracle_forward(h, img.data() + sz, nullptr) == 0);
  EXPECT(oracle_backward_update(h, lab[1], 0.01, &loss) == 0);
  EXPECT(oracle_train_many(h, img.data(), lab.data(), n, 0.01) == 0);
  EXPECT(oracle_forward_many(h, img.data(), n, probs.data()) == 0);
  EXPECT(oracle_get_weights(h, w.data(), nw) == 0);
  double s = 0;
  for (double v : w) s += v;
  EXPECT(std::isfinite(s));
  std::printf("%-44s f%d weights %6zu checksum %+.6f\n", arch, precision, nw, s);
  oracle_destroy(h);
}

int main() {
  const char* archs[] = {
      "1x9x9-3C4-MP2-4C2-5N-3N", "2x11x11-3C3S1-4C2-MP2-4N", "3x8x8-4C3-MP3-4C2-6N-5N-4N", "1x6x6-2C3-3N",
      "2x14x11-3C4x2S1x0-MP2x5-4C1x2-5N-3N", "1x10x12-2C3x5-MP4x2-4N", "1x20x20-6C6-MP3-5C3S2-4N", "1x5x5-7N-4N",
      "1x29x29-20C4-MP2-40C5-MP3-150N-10N"};
  unsigned seed = 1;
  for (const char* a : archs)
    for (int prec : {64, 32}) {
      run_net(a, prec, -1, 0, 0, seed++);
      run_net(a, prec, 1, 0, 1, seed++);
    }
  run_net("2x12x12-3C3-MP2-4C2-5N", 64, 1, 5, 0, seed++);   // (a 2-channel 16x16 raw image behind 5x5 fixed filters)
  // error paths of the parser
  oracle_t* h = nullptr;
  for (const char* bad : {"", "1x9", "1x9x9-3C4-MP4-2N", "1x9x9-3C4", "1x9x9-3C12-2N", "axbxc-2N", "1x9x9-3C4-MP2"})
    EXPECT(oracle_create(bad, 64, &h) != 0);
  EXPECT(oracle_create("1x9x9-3C4-2N", 16, &h) != 0);
  EXPECT(oracle_conv_out_size(29, 5, 1) == 13);
  if (fails) { std::printf("%d checks failed\n", fails); return 1; }
  std::printf("oracle sanitizer run: clean\n");
  return 0;
}
