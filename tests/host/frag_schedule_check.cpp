// Host check of paper_2601_07891_amd/csrc/frag_schedule.h: the wait counts the scorer's K loop
// uses are replayed against a model of a wavefront's in-order vector-memory queue.  The model
// issues the operations in the order the header documents (prologue, then tile by tile, group
// by group) and, at every wait, marks everything but the newest `count` operations complete;
// an operand that is used while its load is not complete is an under-wait.  It also reports the
// slack (operations that could still have been allowed) so that an over-wait shows up.
//
// usage: frag_schedule_check [--plant]   (--plant adds one to every fragment count: must fail)
#include <cstdio>
#include <cstring>
#include <map>
#include <tuple>
#include <vector>

#include "frag_schedule.h"

using namespace kvzap::frag;

struct Sim {
  int UB, NDJ, lead, nk, plant;
  int issued = 0, complete = 0;                    // operations issued; the oldest `complete` have landed
  std::map<std::tuple<int, int>, int> frag_at;     // (tile, G) -> issue index of its load
  std::map<int, int> hidden_at;                    // hidden tile -> issue index of its last load-to-LDS
  int errors = 0, max_slack = 0;

  void load_fragment(int tile, int G) { frag_at[{tile, G}] = issued++; }
  void load_hidden(int tile) { hidden_at[tile] = issued++; }
  void wait(int allowed) { if (issued - allowed > complete) complete = issued - allowed; }
  void need(int at, const char* what, int tile, int G) {
    if (at >= complete) {
      if (errors++ < 5)
        std::printf("UB=%d NDJ=%d lead=%d nk=%d: %s of tile %d (group %d) used before it arrived\n",
                    UB, NDJ, lead, nk, what, tile, G);
    }
  }

  int run() {
    const int NG = groups(UB);
    // prologue: fragments of tile 0, hidden tiles 0 and 1, (fragments of tile 1,) hidden tile 2
    for (int G = 0; G < NG; ++G) load_fragment(0, G);
    for (int d = 0; d < 2; ++d)
      for (int j = 0; j < NDJ; ++j) load_hidden(d);
    if (lead == 2)
      for (int G = 0; G < NG; ++G) load_fragment(1, G);
    for (int j = 0; j < NDJ; ++j) load_hidden(2);
    wait(prologue_wait(UB, NDJ, lead));
    for (int G = 0; G < NG; ++G) need(frag_at[{0, G}], "fragment", 0, G);
    need(hidden_at[0], "hidden tile", 0, -1);      // tile 0 reads it right away
    need(hidden_at[1], "hidden tile", 1, -1);      // and tile 0's hand-over counts on it
    for (int t = 0; t < nk; ++t) {
      const int left = nk - t, R = left < kHiddenAhead + 1 ? left : kHiddenAhead + 1;
      const bool next = R > 1, more = reloads_fragments(R, 0, lead), more_hidden = fetches_hidden(R, 0);
      for (int G = 0; G < NG; ++G) {
        if (next && G == 2 * UB) {
          wait(handover_wait(UB, NDJ, lead, R));
          need(hidden_at[t + 1], "hidden tile", t + 1, G);
        }
        if (G % 2 == 0) {                                   // one wait covers groups G and G+1
          const int count = fragment_pair_wait(UB, NDJ, lead, R, G) + plant;
          const int exact = issued - frag_at[{t, G + 1}] - 1;   // what could have been allowed
          if (exact - count > max_slack) max_slack = exact - count;
          if (count < 0) { ++errors; std::printf("negative count\n"); }
          wait(count);
        }
        need(frag_at[{t, G}], "fragment", t, G);
        if (more_hidden)
          for (int j = 0; j < NDJ; ++j)
            if (dma_group(UB, NDJ, j) == G) load_hidden(t + kHiddenAhead);
        if (more && G > 0) load_fragment(t + lead, G - 1);
      }
      if (more) load_fragment(t + lead, NG - 1);
    }
    return errors;
  }
};

int main(int argc, char** argv) {
  const int plant = (argc > 1 && !std::strcmp(argv[1], "--plant")) ? 1 : 0;
  int failed = 0, checked = 0, worst_slack = 0;
  for (int UB = 1; UB <= 5; ++UB)
    for (int NDJ = 3; NDJ <= 4; ++NDJ)
      for (int lead = 1; lead <= 2; ++lead) {
        if (!lead_is_safe(UB, NDJ, lead)) continue;           // the kernel refuses to compile these
        for (int nk = kHiddenAhead + 1; nk <= 20; ++nk) {
          Sim s{UB, NDJ, lead, nk, plant};
          failed += s.run() ? 1 : 0;
          if (s.max_slack > worst_slack) worst_slack = s.max_slack;
          ++checked;
        }
      }
  // the shapes the library instantiates must be among the safe ones
  const int built[][3] = {{1, 4, 2}, {2, 4, 2}, {3, 4, 2}, {4, 4, 2}, {5, 3, 1}, {4, 4, 1}, {1, 4, 1}};
  for (auto& b : built)
    if (!lead_is_safe(b[0], b[1], b[2])) { std::printf("built shape UB=%d NDJ=%d lead=%d is not safe\n", b[0], b[1], b[2]); ++failed; }
  std::printf("%d configurations checked, %d with an under-wait, largest over-wait %d operations\n",
              checked, failed, worst_slack);
  return failed ? 1 : 0;
}
