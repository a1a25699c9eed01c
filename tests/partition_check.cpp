// Host-side check of the 8-wave prefill kernel's work partition (compiled and run by test_prefill_partition_cpu.py).
// Replays the launches of prefill units on sets of tile ids instead of softmax states: every pass "accumulates" the
// tiles of its ranges into the image it stores (or into the block's output), the merge "combines" the images the
// merge kernel would read.  At the end every block of positions must have seen each of its tiles exactly once.
#include <cstdio>
#include <cstdlib>
#include <map>
#include <set>
#include <vector>
#include "hi_internal.h"
#include "hi_prefill_part.h"

using namespace hi;

struct Image { bool valid = false; int block = -1; std::multiset<long> tiles; };

static long fails = 0;
#define CHECK(cond, ...) do { if (!(cond)) { if (fails < 20) { printf("FAIL %s:%d: ", __FILE__, __LINE__); printf(__VA_ARGS__); printf("\n"); } ++fails; } } while (0)

// one unit: past slices of slice_rows[] rows (one launch each; the last launch also carries the chunk's own rows)
static void run_unit(int G, int C, int n_heads, int variant, const std::vector<long>& slices, long* max_tiles, long* min_tiles) {
  const int strip2 = 2 * prefill_strip(G);
  const int n_launch = slices.empty() ? 1 : (int)slices.size();
  std::vector<Image> img;
  std::map<int, std::multiset<long>> out;     // block -> tiles of the pass that wrote it directly, or of the merge
  std::set<int> written;
  PrefillLaunch pl{};
  PfShape sh{};
  for (int l = 0; l < n_launch; ++l) {
    const int last = l == n_launch - 1, first = l == 0;
    const long na = slices.empty() ? 0 : slices[l];
    pl = prefill_launch_shape(G, C, n_heads, variant, last, last);
    if (!pl.deep) return;
    CHECK(pl.carry_bytes <= prefill_carry_bound(G, C, n_heads), "carry bound G=%d C=%d nh=%d", G, C, n_heads);
    CHECK(pl.carry_bytes == (int64_t)pf_images_per_row(pl.nbk, pl.split) * prefill_grid_y(G) * n_heads * kPdLanes * kCarryFloatsPerLane * 4, "carry bytes");
    sh.nbk = pl.nbk; sh.m = strip2 / 64; sh.ta = (int)((na + 63) / 64); sh.tb_all = last ? (C + 63) / 64 : 0;
    sh.split = pl.split; sh.paired = pl.paired; sh.carried = !first;
    const int n_img = pf_images_per_row(pl.nbk, pl.split);
    if (first) img.assign(n_img, Image());
    std::vector<int> loaded(n_img, 0), stored(n_img, 0);
    std::vector<Image> next = img;
    long wmax = 0, wmin = 1L << 60;
    for (int w = 0; w < pl.nbk * pl.split; ++w) {
      long tiles_w = 0;
      for (int which = 0; which < 2; ++which) {
        const PfPass ps = pf_pass(sh, w, which, last);
        CHECK(!(ps.run && ps.init), "run and init");
        if (ps.init) {
          CHECK(ps.store >= 0 && ps.store < n_img, "init image %d of %d", ps.store, n_img);
          CHECK(!stored[ps.store]++, "image stored twice");
          next[ps.store].valid = true; next[ps.store].block = ps.bx; next[ps.store].tiles.clear();
        }
        if (!ps.run) continue;
        CHECK(ps.bx >= 0 && ps.bx < pl.nbk, "block %d", ps.bx);
        CHECK(ps.a0 >= 0 && ps.a0 <= ps.a1 && ps.a1 <= sh.ta, "past range %d %d of %d", ps.a0, ps.a1, sh.ta);
        CHECK(ps.b0 >= 0 && ps.b0 <= ps.b1 && ps.b1 <= pf_own_tiles(sh, ps.bx), "own range %d %d of %d", ps.b0, ps.b1, pf_own_tiles(sh, ps.bx));
        CHECK(ps.a1 > ps.a0 || ps.b1 > ps.b0, "empty pass runs");
        std::multiset<long> acc;
        if (ps.load >= 0) {
          CHECK(ps.load < n_img && img[ps.load].valid && img[ps.load].block == ps.bx, "load of image %d (valid %d block %d, pass block %d)", ps.load, ps.load < n_img ? (int)img[ps.load].valid : -1, ps.load < n_img ? img[ps.load].block : -1, ps.bx);
          CHECK(!loaded[ps.load]++, "image loaded twice");
          CHECK(ps.store == ps.load || ps.store < 0, "a loaded image must be stored back by its reader");
          if (ps.load < n_img) acc = img[ps.load].tiles;
        }
        for (int t = ps.a0; t < ps.a1; ++t) acc.insert(1000000L * (l + 1) + t);
        for (int t = ps.b0; t < ps.b1; ++t) acc.insert(t);
        tiles_w += (ps.a1 - ps.a0) + (ps.b1 - ps.b0);
        if (ps.store >= 0) {
          CHECK(ps.store < n_img, "store image %d of %d", ps.store, n_img);
          CHECK(!stored[ps.store]++, "image stored twice");
          if (ps.store < n_img) { next[ps.store].valid = true; next[ps.store].block = ps.bx; next[ps.store].tiles = acc; }
        } else {
          CHECK(last, "output written before the last launch");
          CHECK(!written.count(ps.bx), "block written twice");
          written.insert(ps.bx);
          out[ps.bx] = acc;
        }
      }
      if (tiles_w > wmax) wmax = tiles_w;
      if (tiles_w < wmin) wmin = tiles_w;
    }
    // an image that is loaded must not be overwritten by another workgroup in the same launch
    for (int i = 0; i < n_img; ++i) CHECK(!(loaded[i] && stored[i] > 1), "image %d", i);
    img = next;
    if (last) { *max_tiles = wmax; *min_tiles = wmin; }
  }
  // merge
  for (int b = 0; b < pl.nbk; ++b) {
    int n_e, n_x;
    pf_block_images(sh, b, n_e, n_x);
    const bool direct = n_e + n_x == 1 && pl.split == 1;
    CHECK(direct == (written.count(b) > 0), "block %d: direct %d written %d (n_e %d n_x %d)", b, (int)direct, (int)written.count(b), n_e, n_x);
    if (!direct) {
      CHECK(pl.merge, "states to merge but no merge launch");
      std::multiset<long> acc;
      for (int i = 0; i < n_e + n_x; ++i) {
        const int id = i < n_e ? pf_image_e(sh, b, i) : pf_image_x(sh, b, i - n_e);
        CHECK(id >= 0 && id < (int)img.size() && img[id].valid && img[id].block == b, "merge of block %d reads image %d", b, id);
        if (id >= 0 && id < (int)img.size()) acc.insert(img[id].tiles.begin(), img[id].tiles.end());
      }
      out[b] = acc;
    }
    // expected: every past tile of every launch, own tiles [0, o_b)
    std::multiset<long> want;
    for (int l = 0; l < n_launch; ++l) {
      const long na = slices.empty() ? 0 : slices[l];
      for (long t = 0; t < (na + 63) / 64; ++t) want.insert(1000000L * (l + 1) + t);
    }
    for (int t = 0; t < pf_own_tiles(sh, b); ++t) want.insert(t);
    CHECK(out[b] == want, "block %d of G=%d C=%d nh=%d variant=%d launches=%d: %zu tiles, %zu wanted", b, G, C, n_heads, variant, n_launch, out[b].size(), want.size());
  }
}

int main() {
  const int Gs[] = {1, 2, 4, 8};
  const int Cs[] = {1, 64, 65, 129, 700, 1536, 3000, 4096, 8192, 9000, 16384};
  const std::vector<std::vector<long>> pasts = {{}, {1}, {100}, {7003}, {512, 512, 100}, {2048, 2048, 600}, {64, 64, 64, 3}};
  long cases = 0, worst_spread = 0;
  for (int G : Gs) for (int C : Cs) for (int nh : {1, 3, 8}) for (int variant : {0, 3, 3 + 4, 3 + 8}) for (const auto& p : pasts) {
    if ((long)C * nh > 40000) continue;
    long mx = 0, mn = 0;
    run_unit(G, C, nh, variant, p, &mx, &mn);
    ++cases;
    const PrefillLaunch pl = prefill_launch_shape(G, C, nh, variant, 1, 1);
    if (pl.deep && pl.paired) {
      // balance of the paired partition: ranges of one unit differ by at most one tile, units by the odd block of an
      // odd count and the clipped last block
      if (mx - mn > worst_spread) worst_spread = mx - mn;
    }
  }
  // the plan's carry covers every launch it allows
  for (int G : Gs) for (int C : {64, 512, 4096, 8192, 16384, 32768, 65536}) for (int nh : {1, 2, 4, 8}) {
    const int64_t bound = prefill_carry_bound(G, C, nh);
    for (int len = 1; len <= C; len += (len < 300 ? 1 : 193)) for (int h = 1; h <= nh; ++h) for (int variant : {0, 1, 3, 4, 7, 8, 11}) for (int last = 0; last < 2; ++last)
      CHECK(prefill_launch_shape(G, len, h, variant, last, last).carry_bytes <= bound, "bound G=%d C=%d nh=%d len=%d h=%d", G, C, nh, len, h);
  }
  printf("%ld units replayed, %ld failures, largest spread of tiles per workgroup in a paired launch: %ld\n", cases, fails, worst_spread);
  return fails ? 1 : 0;
}
