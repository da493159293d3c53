// Host-only validity check of the static plan, built with AddressSanitizer and UBSan by tests/test_plan_validity.py.
// For a network description read from stdin it builds the graph, chooses the segments and builds the schedule with
// the planner's own sources, then walks the schedule and checks what the kernels rely on:
//   * every operation reads only tensors that an earlier live operation produced and that are not yet released;
//   * no two tensors that are alive at the same time overlap in the activation arena, and all lie inside it;
//   * the reported peaks are what the walk finds.
// Input: "k plan_mode precision batch height width channels classes storage_mode n_units" then n_units lines of
// "kind cin cout ksize stride pad has_bn has_relu has_bias".  Output: "ok <arena> <peak_saved> <launches>" or an error.
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "plan.h"

using namespace oseq;

static int fail(const char* what, int op, int inst) {
  std::printf("error: %s (operation %d, tensor %d)\n", what, op, inst);
  return 1;
}

int main() {
  Plan p;
  int n_units = 0;
  optorch_seq_config_t& c = p.cfg;
  if (std::scanf("%d %d %d %d %d %d %d %d %d %d", &c.k_segments, &c.plan_mode, &c.precision, &c.batch, &c.height, &c.width,
                 &c.channels, &c.num_classes, &c.storage_mode, &n_units) != 10) return fail("bad header", -1, -1);
  for (int i = 0; i < n_units; ++i) {
    optorch_unit_t u{};
    if (std::scanf("%d %d %d %d %d %d %d %d %d", &u.kind, &u.cin, &u.cout, &u.ksize, &u.stride, &u.pad, &u.has_bn, &u.has_relu,
                   &u.has_bias) != 9) return fail("bad unit", i, -1);
    p.units.push_back(u);
  }
  if (!build_graph(p) || !choose_segments(p) || !build_schedule(p)) { std::printf("error: %s\n", p.error.c_str()); return 1; }
  const int n = (int)p.sched.size();
  std::vector<char> alive(p.insts.size(), 0);
  std::vector<int> live_list;
  uint64_t live_saved = 0, peak_saved = 0;
  int launches = 0;
  for (int i = 0; i < n; ++i) {
    const SOp& op = p.sched[i];
    if (!op.live) continue;
    launches += launches_of(op, p.fops[op.fop]);
    for (int x : op.in)
      if (x >= 0) {
        if (x >= (int)p.insts.size()) return fail("input index out of range", i, x);
        if (!alive[x]) return fail("reads a tensor that is not alive", i, x);
      }
    for (int o : op.out)
      if (o >= 0) {
        const Inst& t = p.insts[o];
        if (alive[o]) return fail("produced twice", i, o);
        if (!t.allocated || t.def_op != i) return fail("output not allocated by this operation", i, o);
        if (t.offset % kAlign != 0 || t.offset + t.bytes > p.arena_bytes) return fail("outside the arena", i, o);
        for (int other : live_list)
          if (alive[other]) {
            const Inst& q = p.insts[other];
            const uint64_t a0 = t.offset, a1 = t.offset + (t.bytes ? t.bytes : 1);
            const uint64_t b0 = q.offset, b1 = q.offset + (q.bytes ? q.bytes : 1);
            if (a0 < b1 && b0 < a1) return fail("overlaps a live tensor", i, other);
          }
        alive[o] = 1;
        live_list.push_back(o);
        if (t.held) live_saved += t.bytes;
      }
    if (live_saved > peak_saved) peak_saved = live_saved;
    for (size_t t = 0; t < p.insts.size(); ++t)
      if (alive[t] && p.insts[t].last_use == i) {
        alive[t] = 0;
        if (p.insts[t].held) live_saved -= p.insts[t].bytes;
      }
  }
  for (size_t t = 0; t < p.insts.size(); ++t)
    if (alive[t]) return fail("never released", n, (int)t);
  if (peak_saved != p.peak_saved_bytes) return fail("peak of saved bytes differs from the plan's", -1, -1);
  if (launches != p.n_launches) return fail("launch count differs from the plan's", -1, -1);
  std::printf("ok %llu %llu %d\n", (unsigned long long)p.arena_bytes, (unsigned long long)p.peak_saved_bytes, p.n_launches);
  return 0;
}
