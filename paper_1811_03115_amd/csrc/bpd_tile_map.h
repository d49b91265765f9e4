// Workgroup -> tile map of gemm_ldsx_kernel, free of any HIP dependency so that the host can check it: the kernel
// calls ldsx_tile_of() with its block indices, tests/host/host_logic_check.cpp walks whole grids through the same
// function and checks that every (group, row block, column block) is produced exactly once.
//
// Workgroups are handed to the 8 XCDs round-robin in launch order (x fastest, then y, then z) and each XCD has its own
// L2, so which tiles share an XCD decides what the L2s fetch more than once.
#pragma once

#if defined(__HIPCC__)
#define BPD_HD __host__ __device__
#else
#define BPD_HD
#endif

// what the map (and the kernel's walk over K) would otherwise divide for: the host knows the divisors
struct LdsxMap {
  int nchunks;                    // chunks of KC per K slice
  int log2g;                      // one group: column blocks per XCD are walked in runs of 2^log2g
  unsigned magic_mbg, magic_mb;   // multipliers for MB << log2g and MB
  unsigned upx;                   // several groups: units of (group, pair of column blocks) per XCD; 0: map of one group per z
  unsigned magic_mb2, magic_nbh;  // multipliers for 2 MB and NB / 2
};

// Multiplier m with n / d == div_magic(n, m) for all n with n * d < 2^32: m = ceil(2^32 / d); 0 stands for d == 1
// (whose multiplier, 2^32, does not fit)
inline unsigned magic_div(unsigned d) { return d <= 1 ? 0u : (unsigned)((0x100000000ull + d - 1) / d); }
BPD_HD inline unsigned div_magic(unsigned n, unsigned m) { return m ? (unsigned)(((unsigned long long)n * m) >> 32) : n; }

// K deep, chunks of KC, `ksplit` K slices (<= 1: none), grid of NB x MB column / row blocks, `groups` in z
inline LdsxMap ldsx_map_of(int K, int KC, int ksplit, unsigned NB, unsigned MB, unsigned groups) {
  LdsxMap m{};
  m.nchunks = K / KC / (ksplit > 1 ? ksplit : 1);
  const unsigned per = NB >> 3;
  m.log2g = (per & 3) == 0 ? 2 : ((per & 1) == 0 ? 1 : 0);
  m.magic_mbg = magic_div(MB << m.log2g);
  m.magic_mb = magic_div(MB);
  if (groups > 1 && ksplit <= 1 && NB % 2 == 0 && (groups * (NB / 2)) % 8 == 0) {
    m.upx = groups * (NB / 2) / 8;
    m.magic_mb2 = magic_div(2 * MB);
    m.magic_nbh = magic_div(NB / 2);
  }
  return m;
}

// Block (x, y, z) of an NB x MB x Z grid -> column block bx, row block by, group g (g comes in as z, or 0 for K slices).
// One group (or K slices in z): an XCD owns the column blocks (weights) congruent to its index and walks them in runs of
// G = 2^log2g, all row blocks of a run before the next run, the G column blocks fastest: the run's weights stay in L2 and
// a row block of activations is fetched once per run.  NB not a multiple of 8: column-block-major.
// Several groups, each with its own activations AND weights (the heads' output layers): with the map above an XCD would
// own column block i of every group, so each of the eight L2s would fetch every group's activations (batch 32 of
// Transformer-big: 8 x 26 MB on top of 84 MB of weights).  Instead an XCD owns whole units of (group, pair of column
// blocks) with all their row blocks, consecutive units per XCD: a group's activations then reach at most two L2s.
BPD_HD inline void ldsx_tile_of(const LdsxMap& m, unsigned NB, unsigned MB, unsigned x, unsigned y, unsigned z, int& g, int& by, int& bx) {
  const unsigned L = x + NB * y;
  if (m.upx) {
    const unsigned Lz = L + NB * MB * z, xcd = Lz & 7, j = Lz >> 3;
    const unsigned ul = div_magic(j, m.magic_mb2), within = j - ul * (2 * MB);
    const unsigned unit = xcd * m.upx + ul;
    const unsigned gg = div_magic(unit, m.magic_nbh);
    g = (int)gg;
    by = (int)(within >> 1);
    bx = (int)((unit - gg * (NB >> 1)) * 2 + (within & 1));
  } else if ((NB & 7) == 0) {
    const unsigned j = L >> 3, lg = m.log2g;
    const unsigned grp = div_magic(j, m.magic_mbg), within = j - grp * (MB << lg);
    by = (int)(within >> lg);
    bx = (int)((L & 7) + 8 * ((grp << lg) + (within & ((1u << lg) - 1))));
  } else {
    const unsigned b = div_magic(L, m.magic_mb);
    bx = (int)b; by = (int)(L - b * MB);
  }
}
