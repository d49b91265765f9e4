// Host check of the decoder stack kernel's schedule (paper_1811_03115_amd/csrc/bpd_stack_sched.h): for many shapes and
// every worker, the compute waves' walker and the helper waves' walker must emit the same sequence of workgroup
// barriers; the units a worker's compute waves consume must be exactly its tiles, each chunk once, in the order the
// helper finishes them; weights are requested inside their matrices; LDS regions fit what stack_lds_need reports.
// Built by tests/test_host_logic.py with the system compiler under -fsanitize=address,undefined.
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "../../paper_1811_03115_amd/csrc/bpd_stack_sched.h"

struct ComputeRec {
  const StackShape& s;
  int rank;
  std::vector<int> bars;
  std::vector<StackIt> consumed, loaded;
  std::vector<StackIt> slot[4];
  long bad = 0;
  ComputeRec(const StackShape& s_, int r) : s(s_), rank(r) {}
  void barrier(int kind) { bars.push_back(kind); }
  template <int S> void load(const StackIt& it) {
    // inside the matrix
    const int ntiles = stack_gemm_tiles(s, it.g), ksteps = stack_gemm_K(s, it.g) / 32;
    const long t = rank + (long)s.workers * it.jl;
    if (it.layer < 0 || it.layer >= s.n_layers || t >= ntiles || it.c < 0 || 4 * (it.c * s.KU) >= ksteps) ++bad;
    slot[S].push_back(it);
    loaded.push_back(it);
  }
  template <int S> void consume(const StackIt& it, bool last) {
    // the slot holds this very unit: it is the oldest request of the slot not yet consumed
    if (slot[S].empty()) { ++bad; return; }
    const StackIt h = slot[S].front();
    slot[S].erase(slot[S].begin());
    if (h.layer != it.layer || h.g != it.g || h.jl != it.jl || h.c != it.c) ++bad;
    if (last != (it.c == stack_chunks(s, it.g) - 1)) ++bad;
    consumed.push_back(it);
  }
};
struct HelperRec {
  const StackShape& s;
  int rank;
  std::vector<int> bars;
  std::vector<int> ops;          // layer * 8 + op of every GEMM operator finished, with its tile count
  std::vector<int> tiles;
  long bad = 0;
  int last_inst = -1;
  HelperRec(const StackShape& s_, int r) : s(s_), rank(r) {}
  void check(int inst, int producers) {
    if (inst <= last_inst) ++bad;
    last_inst = inst;
    if (inst > 0 && (producers < 1 || producers > STACK_FLAG_STRIDE)) ++bad;
  }
  // what the kernel's visitor does at these calls, as far as barriers go
  void attention(int, int, int inst, int producers) {
    check(inst, producers);
    for (int it = rank; it < s.heads * s.B; it += s.workers) bars.push_back(STACK_BAR_ATT);
  }
  void gemm(int layer, int op, int inst, int producers, int ntl) {
    check(inst, producers);
    bars.push_back(STACK_BAR_A);
    bars.push_back(STACK_BAR_B);
    ops.push_back(layer * STACK_OPS + op);
    tiles.push_back(ntl);
  }
};

static long check_shape(const StackShape& s, int attn_bytes) {
  long bad = 0;
  const int lds = stack_lds_need(s, attn_bytes);
  for (int rank = 0; rank < s.workers; ++rank) {
    ComputeRec c(s, rank);
    stack_compute_walk(s, rank, c);
    HelperRec h(s, rank);
    stack_helper_walk(s, rank, h);
    bad += c.bad + h.bad;
    if (c.bars != h.bars) {
      ++bad;
      fprintf(stderr, "barrier sequences differ: d=%d F=%d heads=%d B=%d M=%d workers=%d layers=%d rank=%d (%zu vs %zu)\n", s.d, s.F,
              s.heads, s.B, s.M, s.workers, s.n_layers, rank, c.bars.size(), h.bars.size());
    }
    // consumed units: per (layer, g) the worker's tiles in order, chunks in order; operators in the helper's order
    size_t u = 0, e = 0;
    for (int layer = 0; layer < s.n_layers; ++layer)
      for (int g = 0; g < 6; ++g) {
        const int ntl = stack_tiles_of(stack_gemm_tiles(s, g), rank, s.workers);
        if (ntl == 0) continue;
        const int op = g == 0 ? 0 : (g <= 2 ? g + 1 : g + 2);
        if (e >= h.ops.size() || h.ops[e] != layer * STACK_OPS + op || h.tiles[e] != ntl) ++bad;
        ++e;
        for (int jl = 0; jl < ntl; ++jl)
          for (int ch = 0; ch < stack_chunks(s, g); ++ch, ++u) {
            if (u >= c.consumed.size()) { ++bad; continue; }
            const StackIt& it = c.consumed[u];
            if (it.layer != layer || it.g != g || it.jl != jl || it.c != ch) ++bad;
          }
        // LDS: the operator's input block and the worker's partial sums end before the helpers' counter
        if (stack_part_offset(s.M, stack_gemm_K(s, g)) + ntl * 4096 > lds - 16) ++bad;
      }
    if (u != c.consumed.size() || e != h.ops.size()) ++bad;
    if (attn_bytes > lds - 16) ++bad;
  }
  return bad;
}

int main() {
  long bad = 0, shapes = 0;
  const int ds[] = {128, 256, 512, 768, 1024};
  const int workers[] = {32, 1, 2, 5, 16, 38, 64};
  for (int d : ds)
    for (int F : {128, 256, 640, 1024, 2048, 4096})
      for (int W : workers)
        for (int B : {1, 2, 3, 5, 16})
          for (int R : {1, 2, 5, 10, 16}) {
            if (B * R > 16) continue;
            for (int layers : {1, 2, 6}) {
              StackShape s{layers, d, F, d / 64, B, B * R, W, d / 128};
              bad += check_shape(s, 51712);
              ++shapes;
            }
          }
  printf("%ld shapes checked, %ld violations\n", shapes, bad);
  return bad ? 1 : 0;
}
