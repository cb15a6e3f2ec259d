// Which output tile of a merge level a workgroup takes in a given round of the triangular inverse (inv_tree.hip).
//
// Level S merges pairs of neighbouring S-block diagonal blocks of the 64 x 64-tiled r x r matrix (nb tile rows): pair
// q covers tile rows a0 = 2 q S (block A) and d0 = a0 + S (block D, min(S, nb - d0) tile rows).  Both products of a
// merge have S x S output tiles (ti, tj) per pair; a tile of the first sums S - tj tile pairs, one of the second
// ti + 1.  The tiles of a level are ranked by that length, longest first, and dealt out back and forth (round 0 to
// workgroups 0, 1, ..., round 1 to ..., 1, 0), so that every workgroup sums about the same number of tile pairs.
// Plain integer arithmetic, shared by the kernel and by a host test that checks that every tile is taken exactly once.
#pragma once

#ifdef __HIPCC__
#define DION_HOST_DEVICE __host__ __device__
#else
#define DION_HOST_DEVICE
#endif

namespace dion {

// number of pairs merged at level S
DION_HOST_DEVICE inline int inv_tree_pairs(int nb, int S) { return ((nb + S - 1) / S) / 2; }
// tile rows of block D of the last pair (every other pair has S)
DION_HOST_DEVICE inline int inv_tree_last_rows(int nb, int S) {
  const int rest = nb - (2 * (inv_tree_pairs(nb, S) - 1) * S + S);
  return rest < S ? rest : S;
}
// output tiles per product of level S
DION_HOST_DEVICE inline int inv_tree_tiles(int nb, int S) {
  return ((inv_tree_pairs(nb, S) - 1) * S + inv_tree_last_rows(nb, S)) * S;
}
// rounds a workgroup goes through per product of level S
DION_HOST_DEVICE inline int inv_tree_rounds(int nb, int S, int groups) { return (inv_tree_tiles(nb, S) + groups - 1) / groups; }
// The tile workgroup `wg` of `groups` takes in `round` of product `phase` (0: T = C A^-1, 1: -D^-1 T) of level S;
// false: none (past the end of the list).  Only tiles that exist are ranked: the last pair's block D may have fewer
// than S tile rows.
DION_HOST_DEVICE inline bool inv_tree_tile(int nb, int S, int phase, int groups, int wg, int round, int& q, int& ti, int& tj) {
  const int np = inv_tree_pairs(nb, S), last = inv_tree_last_rows(nb, S);
  const int rows = (np - 1) * S + last;   // tile rows of all blocks D of the level
  const int rank = round * groups + ((round & 1) ? groups - 1 - wg : wg);
  if (rank >= rows * S) return false;
  if (phase == 0) {
    // length S - tj: by column, and within a column the rows of all pairs
    tj = rank / rows;
    const int rem = rank % rows;
    q = rem / S;
    ti = rem % S;
  } else {
    // length ti + 1: by row from the bottom; rows last .. S - 1 exist in all pairs but the last one
    const int upper = (S - last) * (np - 1) * S;
    int rem;
    if (rank < upper) {
      ti = S - 1 - rank / ((np - 1) * S);
      rem = rank % ((np - 1) * S);
    } else {
      ti = last - 1 - (rank - upper) / (np * S);
      rem = (rank - upper) % (np * S);
    }
    q = rem / S;
    tj = rem % S;
  }
  return true;
}

}  // namespace dion
