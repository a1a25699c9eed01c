// How one launch of the 8-wave prefill kernel divides its work among workgroups (pure integer arithmetic, shared by
// the kernel, the merge kernel, the launcher and the host-side tests; no HIP call).
//
// A launch covers, for every block of query positions b (nbk blocks of `strip` positions, m = strip / 64 tiles
// each), a sequence of 64-row K/V tiles: the `ta` tiles of the past rows the launch was given, then the
// o(b) = min(tb_all, (b + 1) m) tiles of the chunk's own rows at or below the block's causal boundary (Eq. 3: row p
// sees keys 0..p).  Deep blocks have up to tb_all more tiles than shallow ones.  Two partitions:
//   * on its own (`paired` = 0): the sequence of block b is cut into `split` equal ranges, one workgroup each; with
//     split = 1 a workgroup owns its block.  All blocks are equally long when the launch has no own rows.
//   * paired (`paired` = 1, launches that include the chunk's own rows): block nbk-1-p (deep) and block p (shallow)
//     form a unit whose tiles are laid out [deep past | deep own | shallow own | shallow past] and cut into
//     2 * split equal ranges - every workgroup sweeps the same number of tiles whatever its position in the causal
//     triangle, and range k covers the same past rows in every unit, so the workgroups of a range still walk the
//     past in step.  A range may hold tiles of both blocks: the workgroup makes one pass per block.
// Each pass accumulates a softmax state (m, l, O) for one block over a set of tiles; the states of one block are
// merged at the end (any subset of keys in any order gives a valid partial state).  Images of the states:
//   E(b, j), j < split: the j-th contributor of block b - carried from launch to launch of a unit;
//   X(b, j - split):    contributors beyond `split` in a paired launch (fresh states).
#pragma once
#include <cstdint>

#if defined(__HIPCC__)
#define HI_HD __host__ __device__ __forceinline__
#else
#define HI_HD inline
#endif

namespace hi {

struct PfShape {
  int nbk;      // blocks of query positions per head
  int m;        // 64-row tiles of own rows a block adds: strip / 64
  int ta;       // past tiles of this launch
  int tb_all;   // tiles of the chunk's own rows (0: the launch has none)
  int split;    // workgroups per block
  int paired;   // balanced partition over (deep, shallow) pairs of blocks
  int carried;  // the images E hold states of earlier launches of the unit
};

struct PfPass {
  int run;      // 1: tiles to process
  int init;     // 1: nothing to process, but image `store` must receive an empty state
  int bx;       // block of positions
  int a0, a1;   // past tiles [a0, a1) of the launch
  int b0, b1;   // own tiles [b0, b1) of the chunk
  int load;     // image to start from, -1: empty state
  int store;    // image to store the state to, -1: normalise and write the output rows
};

// images per grid row (one head, one quad of query heads): E then X
HI_HD int pf_images_per_row(int nbk, int split) { return 2 * nbk * split; }
HI_HD int pf_image_e(const PfShape& s, int b, int j) { return j * s.nbk + b; }
HI_HD int pf_image_x(const PfShape& s, int b, int j) { return s.nbk * s.split + b * s.split + j; }

// boundary k of the nr equal ranges a sequence of L tiles is cut into (nr is a power of two; L * nr < 2^32)
HI_HD int pf_cut(int L, int k, int nr) { return (int)(((uint32_t)L * (uint32_t)k) >> __builtin_ctz((unsigned)nr)); }

HI_HD int pf_own_tiles(const PfShape& s, int b) {
  const int o = (b + 1) * s.m;
  return o < s.tb_all ? o : s.tb_all;
}

// the unit block b belongs to: its deep block, its shallow block (-1: on its own), the number of ranges
HI_HD void pf_unit_of_block(const PfShape& s, int b, int& deep, int& shallow, int& nr) {
  const int pairs = s.paired ? s.nbk / 2 : 0;
  if (b < pairs) { deep = s.nbk - 1 - b; shallow = b; nr = 2 * s.split; }
  else if (b >= s.nbk - pairs) { deep = b; shallow = s.nbk - 1 - b; nr = 2 * s.split; }
  else { deep = b; shallow = -1; nr = s.split; }
}

// contributors of block b (ranges of its unit that hold at least one of its tiles), and how many of them come
// before range k
HI_HD void pf_contributors(const PfShape& s, int deep, int shallow, int nr, int is_shallow, int k, int& before, int& total) {
  const int Td = s.ta + pf_own_tiles(s, deep);
  const int L = Td + (shallow >= 0 ? s.ta + pf_own_tiles(s, shallow) : 0);
  before = total = 0;
  for (int kk = 0; kk < nr; ++kk) {
    const int x0 = pf_cut(L, kk, nr), x1 = pf_cut(L, kk + 1, nr);
    const bool hit = x1 > x0 && (is_shallow ? x1 > Td : x0 < Td);
    if (hit) {
      ++total;
      if (kk < k) ++before;
    }
  }
}

// Pass `which` (0: the unit's deep block, 1: its shallow block) of workgroup w (0 .. nbk * split - 1) of a grid row.
HI_HD PfPass pf_pass(const PfShape& s, int w, int which, int last) {
  PfPass g;
  g.run = g.init = 0; g.bx = 0; g.a0 = g.a1 = g.b0 = g.b1 = 0; g.load = g.store = -1;
  int deep, shallow, nr, k;
  const int pairs = s.paired ? s.nbk / 2 : 0;
  if (w < pairs * 2 * s.split) {
    const int p = w / (2 * s.split);
    deep = s.nbk - 1 - p; shallow = p; nr = 2 * s.split; k = w - p * nr;
  } else {
    // blocks on their own: the deepest first, range z of every block before range z + 1 of any
    const int singles = s.nbk - 2 * pairs;
    const int v = w - pairs * 2 * s.split;
    deep = s.nbk - pairs - 1 - (v % singles); shallow = -1; nr = s.split; k = v / singles;
  }
  if (which == 1 && shallow < 0) return g;
  const int od = pf_own_tiles(s, deep), ob = shallow >= 0 ? pf_own_tiles(s, shallow) : 0;
  const int Td = s.ta + od;
  const int L = Td + (shallow >= 0 ? s.ta + ob : 0);
  const int x0 = pf_cut(L, k, nr), x1 = pf_cut(L, k + 1, nr);
  auto clampi = [](int x, int lo, int hi) { return x < lo ? lo : (x > hi ? hi : x); };
  if (which == 0) {
    g.bx = deep;
    g.a0 = clampi(x0, 0, s.ta); g.a1 = clampi(x1, 0, s.ta);
    g.b0 = clampi(x0 - s.ta, 0, od); g.b1 = clampi(x1 - s.ta, 0, od);
  } else {
    g.bx = shallow;
    g.b0 = clampi(x0 - Td, 0, ob); g.b1 = clampi(x1 - Td, 0, ob);
    g.a0 = clampi(x0 - Td - ob, 0, s.ta); g.a1 = clampi(x1 - Td - ob, 0, s.ta);
  }
  const bool nonempty = g.a1 > g.a0 || g.b1 > g.b0;
  int j = k, nc = nr;                 // a block on its own: range z keeps image z in every launch of the unit
  if (shallow >= 0) pf_contributors(s, deep, shallow, nr, which, k, j, nc);
  if (!nonempty) {
    if (shallow < 0 && !s.carried) { g.init = 1; g.store = pf_image_e(s, g.bx, k); }
    return g;
  }
  g.run = 1;
  if (j < s.split) {
    const int e = pf_image_e(s, g.bx, j);
    g.load = s.carried ? e : -1;
    g.store = (last && s.split == 1 && nc == 1) ? -1 : e;
  } else {
    g.store = pf_image_x(s, g.bx, j - s.split);
  }
  return g;
}

// The images the merge of block b has to combine after the unit's last launch: n_e images E(b, 0..n_e-1), then n_x
// images X(b, 0..n_x-1).  n_e + n_x == 1 with split == 1 means the block was written directly by its only pass.
HI_HD void pf_block_images(const PfShape& s, int b, int& n_e, int& n_x) {
  int deep, shallow, nr;
  pf_unit_of_block(s, b, deep, shallow, nr);
  if (shallow < 0) { n_e = s.split; n_x = 0; return; }
  int before, nc;
  pf_contributors(s, deep, shallow, nr, b == shallow ? 1 : 0, 0, before, nc);
  n_e = s.carried ? s.split : (nc < s.split ? nc : s.split);
  n_x = nc > s.split ? nc - s.split : 0;
}

}  // namespace hi
