// Host sanitizer run of the library's host logic (no device is touched): architecture parser, Eq. 1 shapes,
// workspace sizing, stage planner and the resident-mode planner, through the host-only entry points of the C ABI,
// over the benchmark architectures, edge shapes, seeded random architectures and malformed strings.  Built from the
// library's sources with -fsanitize=address,undefined on the host pass; any report ends the program.
#include <cstdint>
#include <cstdio>
#include <cstring>
#include <random>
#include <string>
#include <vector>

#include "../../include/cnn355.h"
extern "C" int cnn355_resident_plan_text(const char* arch, int fan_in, int n_ranks, int xcd_stride, char* buf, size_t n);

static int fails = 0;
#define EXPECT(c) do { if (!(c)) { std::printf("FAILED line %d: %s\n", __LINE__, #c); ++fails; } } while (0)

static std::string random_arch(std::mt19937& rng) {
  auto R = [&](int lo, int hi) { return lo + (int)(rng() % (unsigned)(hi - lo + 1)); };
  int h = R(8, 48), w = (rng() % 3 == 0) ? R(8, 48) : h;
  std::string s = std::to_string(R(1, 3)) + "x" + std::to_string(h) + "x" + std::to_string(w);
  const int maps[] = {2, 5, 12, 20, 40, 64, 100, 120, 300};
  for (int c = R(1, 4); c > 0; --c) {
    const int k = R(1, std::min(7, std::min(h, w))), sk = (rng() % 3 == 0) ? R(0, 2) : 0;
    h = (h - k) / (sk + 1) + 1; w = (w - k) / (sk + 1) + 1;
    s += "-" + std::to_string(maps[rng() % 9]) + "C" + std::to_string(k) + (sk ? "S" + std::to_string(sk) : "");
    if (rng() % 10 < 7) {
      std::vector<int> d;
      for (int q = 1; q <= 4; ++q) if (h % q == 0 && w % q == 0) d.push_back(q);
      const int q = d[rng() % d.size()];
      s += "-MP" + std::to_string(q);
      h /= q; w /= q;
    }
    if (std::min(h, w) < 2) break;
  }
  for (int f = R(0, 2); f > 0; --f) s += "-" + std::to_string(R(2, 199)) + "N";
  return s + "-" + std::to_string(R(2, 11)) + "N";
}

static void walk(const std::string& arch, int fan, int ranks, int stride) {
  int32_t n = 0, info[8 * 40];
  const int rc = cnn_arch_info_xy(arch.c_str(), &n, info, 40);
  size_t bytes = 0;
  const int rw = cnn_workspace_bytes(arch.c_str(), &bytes);
  std::vector<char> buf(1 << 16);
  const int rp = cnn_plan_text(arch.c_str(), buf.data(), buf.size());
  if (rc == 0 && rw == 0) {
    EXPECT(rp == 0 && std::strlen(buf.data()) > 0 && bytes > 0);
    const int rr = cnn355_resident_plan_text(arch.c_str(), fan, ranks, stride, buf.data(), buf.size());
    EXPECT(rr == 0 && std::strlen(buf.data()) > 0);
    EXPECT(cnn_plan_text(arch.c_str(), buf.data(), 8) != 0 || std::strlen(buf.data()) < 8);   // a buffer too small is refused or cut
  } else {
    EXPECT(std::strlen(cnn_last_error(nullptr)) > 0);
  }
}

int main() {
  const char* fixed[] = {
      "1x29x29-20C4-MP2-40C5-MP3-150N-10N", "1x29x29-40C4-MP2-80C5-MP3-300N-10N", "2x48x48-50C5-MP2-128C3-MP4-100N-5N",
      "3x32x32-100C5-MP2-100C5-MP2-100C4-MP2-300N-10N", "3x32x32-300C3-MP2-300C2-MP2-300C4-MP2-300N-10N",
      "4x44x44-40C5S1-MP2-80C3-MP2-100N-5N", "2x96x96-300C6S1-MP2-500C4-MP4-500N-5N",
      "3x32x32-300C3-MP3-300C3-MP2-300C3-MP2-300N-100N-10N", "2x14x11-3C4x2S1x0-MP2x5-4C1x2-5N-3N", "1x8x600-3C3-MP2-4C2S1-5N",
      "1x28x28-6C5-MP2-100C5-MP2-8N", "1x40x40-64C5-MP2-64C1-MP2-64C3-9N", "1x5x5-7N-4N"};
  for (const char* a : fixed)
    for (int fan : {0, 3})
      for (int ranks : {0, 7, 50, 256}) walk(a, fan, ranks, ranks ? 1 : 0);
  std::mt19937 rng(1102);
  for (int t = 0; t < 600; ++t) walk(random_arch(rng), (int)(rng() % 3 ? 0 : rng() % 40), (int)(rng() % 2 ? 0 : rng() % 200), (int)(rng() % 3 ? 0 : 8));
  const char* bad[] = {"", "-", "1x9", "1x9x9", "1x9x9-", "1x9x9-3C4", "1x9x9-3C4-MP4-2N", "1x9x9-3C12-2N", "axbxc-2N", "1x9x9-3C4-MP2",
                       "1x9x9-3C4S-2N", "1x9x9-3C4x-2N", "1x9x9--2N", "0x9x9-2N", "1x9x9-0C3-2N", "1x9x9-3C0-2N", "1x9x9-3C4-0N",
                       "99999999999x9x9-2N", "1x9x9-3C4-MP2-MP2-2N", "1x200x200-3C3-4N"};
  for (const char* b : bad) {
    int32_t n = 0, info[8 * 40];
    size_t bytes = 0;
    EXPECT(cnn_arch_info_xy(b, &n, info, 40) != 0 || cnn_workspace_bytes(b, &bytes) != 0);
    walk(b, 0, 0, 0);
  }
  int32_t n = 0;
  EXPECT(cnn_arch_info(nullptr, &n, nullptr, 0) != 0);
  if (fails) { std::printf("%d checks failed\n", fails); return 1; }
  std::printf("host planner sanitizer run: clean\n");
  return 0;
}
