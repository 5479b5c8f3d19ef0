// The vector-memory schedule of score_mlp_frag_kernel's K loop and the wait counts that follow
// from it, as constant expressions (plain C++14, no device code: the kernel uses them for its
// s_waitcnt immediates and a host test simulates the queue against them).
//
// A wavefront's vector-memory operations complete in issue order.  Per K tile t, with
// NG = 4*UB MFMA groups G = (k-step, unit block), the wavefront issues, in this order:
//
//   group G:      [hand-over wait, only at G == 2*UB]
//                 [wait for A fragments G and G+1 of this tile, G even]   MFMA  MFMA
//                 [load-to-LDS j of hidden tile t+3, if G == dma_group(j)]   (tile t+3 exists)
//                 MFMA  [load A fragment G-1 of tile t+lead]  (MFMA)         (tile t+lead exists)
//   end of tile:  [load A fragment NG-1 of tile t+lead]
//
// A tile's *kind* R = min(tiles left including this one, 4) says which of those later tiles
// exist, for this tile and (R + d) for the tile d steps earlier.  The prologue issues the
// fragments of tiles 0..lead-1 and hidden tiles 0..2 and waits for all of them but (with
// lead == 2) tile 1's fragments and hidden tile 2, which it issues last, in that order.
#pragma once

namespace kvzap {
namespace frag {

constexpr int kHiddenAhead = 3;   // hidden tiles in flight

constexpr int groups(int UB) { return 4 * UB; }
// the group in which load-to-LDS j (0 .. NDJ-1) of a tile is issued: spread over k-steps 2 and 3
constexpr int dma_group(int UB, int NDJ, int j) { return 2 * UB + j * 2 * UB / NDJ; }
constexpr int dmas_between(int UB, int NDJ, int lo, int hi) {   // load-to-LDS groups in [lo, hi]
  int n = 0;
  for (int j = 0; j < NDJ; ++j) n += (dma_group(UB, NDJ, j) >= lo && dma_group(UB, NDJ, j) <= hi) ? 1 : 0;
  return n;
}
// what the tile d steps before a tile of kind R does
constexpr bool fetches_hidden(int R, int d) { return R + d > kHiddenAhead; }
constexpr bool reloads_fragments(int R, int d, int lead) { return R + d > lead; }

// Operations issued after the load of fragment G of a tile of kind R (lead tiles back) and
// before its wait: the rest of the tile that loaded it, (the tile between,) this tile so far.
// That many may stay outstanding at the wait.
constexpr int fragment_wait(int UB, int NDJ, int lead, int R, int G) {
  const int NG = groups(UB);
  int n = (NG - 1 - G) + (fetches_hidden(R, lead) ? dmas_between(UB, NDJ, G + 2, NG) : 0);
  if (lead == 2) n += (reloads_fragments(R, 1, lead) ? NG : 0) + (fetches_hidden(R, 1) ? NDJ : 0);
  n += (reloads_fragments(R, 0, lead) ? (G > 0 ? G - 1 : 0) : 0) +
       (fetches_hidden(R, 0) ? dmas_between(UB, NDJ, 0, G - 1) : 0);
  return n;
}

// One wait for two fragments: issued in front of an even group G it covers G and G+1 (groups
// come in pairs: 4*UB is even), so the odd group needs none.  Fragment G+1's load is the younger
// of the two; between this wait and where G+1's own wait would sit, group G issues its
// load-to-LDS operations (if it has any) and the re-load of fragment G-1.
constexpr int fragment_pair_wait(int UB, int NDJ, int lead, int R, int G) {
  const int in_group = (fetches_hidden(R, 0) ? dmas_between(UB, NDJ, G, G) : 0) +
                       ((reloads_fragments(R, 0, lead) && G > 0) ? 1 : 0);
  return fragment_wait(UB, NDJ, lead, R, G + 1) - in_group;
}

// The hand-over in the middle of a tile of kind R > 1: hidden tile t+1 must have landed.  Its
// last load-to-LDS (two tiles back, group dma_group(NDJ-1)) is followed by that tile's
// remaining fragment loads, the tile between and the 2*UB-1 fragment loads of this tile so far
// (the load-to-LDS operations among them are not counted: fewer allowed is the safe side).
constexpr int handover_wait(int UB, int NDJ, int lead, int R) {
  const int NG = groups(UB);
  return (reloads_fragments(R, 2, lead) ? NG - dma_group(UB, NDJ, NDJ - 1) + 1 : 0) +
         (reloads_fragments(R, 1, lead) ? NG : 0) + (reloads_fragments(R, 0, lead) ? 2 * UB - 1 : 0);
}

// What the prologue may leave outstanding.
constexpr int prologue_wait(int UB, int NDJ, int lead) { return (lead - 1) * groups(UB) + NDJ; }

// Tile 1 takes hidden tile 2 from the prologue, where nothing but (lead == 2) nothing at all
// follows it: its hand-over count then leans on tile 0's NDJ load-to-LDS operations making up
// for the fragment loads that handover_wait() assumes behind a tile's last load-to-LDS.  With
// lead == 1 the fragment waits (at most NG + NDJ outstanding) cover it in any case.
constexpr bool lead_is_safe(int UB, int NDJ, int lead) {
  return lead == 1 || NDJ >= groups(UB) - dma_group(UB, NDJ, NDJ - 1) + 1;
}

}  // namespace frag
}  // namespace kvzap
