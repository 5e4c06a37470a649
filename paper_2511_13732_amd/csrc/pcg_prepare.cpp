// Host-side construction of the prepared membership layout (see pcg_prepared in pcg.h).
#include <algorithm>
#include <atomic>
#include <cstring>
#include <numeric>
#include <thread>
#include <utility>
#include <vector>

#include "../../include/pcg.h"
#include "pcg_layout.h"

namespace {

using namespace pcg;

struct Shape {
  int32_t ntiles, tile_len, chunk_groups, nchunks, blocks_per_chunk;
};

bool make_shape(int32_t V, int32_t G, int32_t chunk_groups, Shape &s) {
  if (V < 1 || G < 1) return false;
  if (chunk_groups == 0) chunk_groups = kMaxChunkGroups;
  if (chunk_groups < kChunkStep || chunk_groups > kMaxChunkGroups || chunk_groups % kChunkStep)
    return false;
  // kBanks slots after every tile are kept for padding entries (one per bank, all zero)
  s.ntiles = (V + kTileTokensMax - 1) / kTileTokensMax;
  s.tile_len = (V + s.ntiles - 1) / s.ntiles;
  s.tile_len = std::min(kTileTokensMax, (s.tile_len + 63) / 64 * 64);
  s.chunk_groups = chunk_groups;
  s.nchunks = (G + chunk_groups - 1) / chunk_groups;
  s.blocks_per_chunk = chunk_groups / kBlockGroups;
  return true;
}

// Local search on a half-wave's schedule out[n][32].  The LDS serves a half-wave's read in as
// many passes as the most loaded bank has lanes, so the cost of a time slot is that maximum
// (with the sum of squared bank loads as a tie-break: flatter slots are the ones that can lose
// a pass next).  A lane may read its own entries in any order: two of its time slots are
// exchanged whenever that lowers the summed cost; a padding entry moves to the emptiest zero
// slot of the time slot it lands in.  Repeated until a sweep finds nothing.
struct SlotLoad {
  int use[kBanks];     // lanes on each bank
  int mx, nmx, sq;     // fullest bank, how many banks are that full, sum of squares
  void recount() {
    mx = 0; nmx = 0; sq = 0;
    for (int k = 0; k < kBanks; ++k) {
      sq += use[k] * use[k];
      if (use[k] > mx) { mx = use[k]; nmx = 1; } else if (use[k] == mx) ++nmx;
    }
  }
  int cost() const { return mx * 4096 + sq; }
  // cost after one lane leaves bank `from` and one arrives on bank `to`
  int cost_moved(int from, int to) const {
    if (from == to) return cost();
    const int peak_left = (use[from] == mx && nmx == 1) ? mx - 1 : mx;
    const int peak = std::max(peak_left, use[to] + 1);
    return peak * 4096 + sq - (2 * use[from] - 1) + (2 * use[to] + 1);
  }
  int emptiest_without(int from) const {     // emptiest bank once a lane has left `from`
    int best = 0, bl = use[0] - (from == 0);
    for (int k = 1; k < kBanks; ++k) {
      const int l = use[k] - (from == k);
      if (l < bl) { bl = l; best = k; }
    }
    return best;
  }
};

void improve_schedule(std::vector<uint16_t> &out, int n, uint16_t pad_base) {
  std::vector<SlotLoad> slot(n);
  auto bank = [&](int t, int l) { return out[(size_t) t * 32 + l] % kBanks; };
  for (int t = 0; t < n; ++t) {
    std::fill(slot[t].use, slot[t].use + kBanks, 0);
    for (int l = 0; l < 32; ++l) ++slot[t].use[bank(t, l)];
    slot[t].recount();
  }
  for (int sweep = 0; sweep < 12; ++sweep) {
    bool changed = false;
    for (int t = 0; t < n; ++t) {
      for (int l = 0; l < 32; ++l) {
        SlotLoad &st = slot[t];
        if (st.mx < 2) break;                              // the slot is free of conflicts
        const int b = bank(t, l);
        if (st.use[b] < 2) continue;                       // alone on its bank
        const bool pad_t = out[(size_t) t * 32 + l] >= pad_base;
        int best = -1, best_gain = 0, best_bt = 0, best_bu = 0;
        for (int u = 0; u < n; ++u) {
          if (u == t) continue;
          const SlotLoad &su = slot[u];
          const int c = bank(u, l);
          const bool pad_u = out[(size_t) u * 32 + l] >= pad_base;
          const int bt = pad_u ? st.emptiest_without(b) : c;      // what arrives in slot t
          const int bu = pad_t ? su.emptiest_without(c) : b;      // what arrives in slot u
          const int gain = st.cost() + su.cost() - st.cost_moved(b, bt) - su.cost_moved(c, bu);
          if (gain > best_gain) { best_gain = gain; best = u; best_bt = bt; best_bu = bu; }
        }
        if (best < 0) continue;
        const int u = best, c = bank(u, l);
        SlotLoad &su = slot[u];
        const bool pad_u = out[(size_t) u * 32 + l] >= pad_base;
        uint16_t to_t = out[(size_t) u * 32 + l], to_u = out[(size_t) t * 32 + l];
        if (pad_u) to_t = (uint16_t) (pad_base + best_bt);
        if (pad_t) to_u = (uint16_t) (pad_base + best_bu);
        --st.use[b]; --su.use[c];
        out[(size_t) t * 32 + l] = to_t;
        out[(size_t) u * 32 + l] = to_u;
        ++st.use[to_t % kBanks]; ++su.use[to_u % kBanks];
        st.recount();
        su.recount();
        changed = true;
      }
    }
    if (!changed) break;
  }
}

// Greedy schedule, one time slot after the other: lanes with the most entries left choose first,
// each takes an entry whose bank is still free in this slot (preferring the bank with the most
// entries still to place); a lane that finds none waits if it has slots to spare, and otherwise
// takes the least crowded bank.
void schedule_greedy(std::vector<uint16_t> (&lists)[32], int n, uint16_t pad_base,
                     std::vector<uint16_t> &out /* [n][32] */) {
  int bank_left[kBanks] = {0};
  for (auto &l : lists)
    for (uint16_t s : l) ++bank_left[s % kBanks];
  out.assign((size_t) n * 32, 0);
  int order[32];
  for (int t = 0; t < n; ++t) {
    const int slots_left = n - t;
    int used[kBanks] = {0};
    bool placed[32] = {false};
    std::iota(order, order + 32, 0);
    std::stable_sort(order, order + 32,
                     [&](int a, int b) { return lists[a].size() > lists[b].size(); });
    for (int oi = 0; oi < 32; ++oi) {
      const int l = order[oi];
      auto &rem = lists[l];
      if (rem.empty()) continue;
      int best = -1;
      for (int e = 0; e < (int) rem.size(); ++e) {
        const int b = rem[e] % kBanks;
        if (used[b]) continue;
        if (best < 0 || bank_left[b] > bank_left[rem[best] % kBanks]) best = e;
      }
      if (best < 0) {
        if ((int) rem.size() < slots_left) continue;      // can wait for a later slot
        for (int e = 0; e < (int) rem.size(); ++e) {      // must go now: least crowded bank
          const int b = rem[e] % kBanks;
          if (best < 0 || used[b] < used[rem[best] % kBanks]) best = e;
        }
      }
      const uint16_t s = rem[best];
      rem.erase(rem.begin() + best);
      ++used[s % kBanks];
      --bank_left[s % kBanks];
      out[(size_t) t * 32 + l] = s;
      placed[l] = true;
    }
    for (int l = 0; l < 32; ++l) {
      if (placed[l]) continue;
      int b = 0;
      for (int c = 0; c < kBanks; ++c)
        if (used[c] < used[b]) b = c;
      ++used[b];
      out[(size_t) t * 32 + l] = (uint16_t) (pad_base + b);
    }
  }
}

// ---------------------------------------------------------------------------------------------
// Schedule by edge colouring.  Lanes and banks are the two sides of a bipartite multigraph, an
// entry is an edge, a time slot is a colour: a colouring in which no two edges at a node share
// a colour is a schedule without conflicts, and one with as many colours as the largest degree
// always exists (Koenig).  A bank that holds more entries than there are slots, N_b > n, must
// double up somewhere; with E = max_b (N_b - n) slots in which a bank may be read twice and
// n - E in which it may not, every bank fits, and E extra passes is the least any schedule of
// this half-wave can cost.  The entries that go into the E double slots are chosen by a flow
// (lane <= E of them, bank <= 2 E, and enough of them that what stays behind has no degree above
// n - E); both parts are then coloured by alternating paths.
// ---------------------------------------------------------------------------------------------

struct SchedEdge {
  int lane, bank;
  uint16_t slot;
  int node;        // right-hand node of the colouring the edge takes part in
  int colour;
};

// Proper colouring of the edges listed in `ids` with colours 0 .. nc-1; every node has at most
// nc of them.  atL[lane * nc + c] / atR[node * nc + c] hold the edge that has colour c there.
void colour_by_alternating_paths(std::vector<SchedEdge> &edges, const std::vector<int> &ids, int nc,
                                 int nright, std::vector<int> &atL, std::vector<int> &atR) {
  atL.assign((size_t) 32 * nc, -1);
  atR.assign((size_t) nright * nc, -1);
  std::vector<int> path;
  for (int id : ids) {
    SchedEdge &e = edges[id];
    int a = 0, b = 0;                                 // a free at the lane, b free at the node
    while (atL[(size_t) e.lane * nc + a] >= 0) ++a;
    while (atR[(size_t) e.node * nc + b] >= 0) ++b;
    if (atR[(size_t) e.node * nc + a] >= 0) {
      // a is taken at the node: flip the path of colours a, b, a, ... that starts there.  It
      // cannot reach the lane (it would arrive there through colour a, which is free at the
      // lane), so afterwards a is free at both ends.
      path.clear();
      int cur = atR[(size_t) e.node * nc + a];
      bool from_right = true;                         // the path leaves a right-hand node next
      int want = a;
      while (cur >= 0) {
        path.push_back(cur);
        want = want == a ? b : a;
        const SchedEdge &pe = edges[cur];
        cur = from_right ? atL[(size_t) pe.lane * nc + want] : atR[(size_t) pe.node * nc + want];
        from_right = !from_right;
      }
      for (int pid : path) {
        const SchedEdge &pe = edges[pid];
        atL[(size_t) pe.lane * nc + pe.colour] = -1;
        atR[(size_t) pe.node * nc + pe.colour] = -1;
      }
      for (int pid : path) {
        SchedEdge &pe = edges[pid];
        pe.colour = pe.colour == a ? b : a;
        atL[(size_t) pe.lane * nc + pe.colour] = pid;
        atR[(size_t) pe.node * nc + pe.colour] = pid;
      }
    }
    e.colour = a;
    atL[(size_t) e.lane * nc + a] = id;
    atR[(size_t) e.node * nc + a] = id;
  }
}

// Small maximum flow (augmenting paths by depth-first search; capacities are a few tens).
struct Flow {
  struct Arc { int to, cap; };
  std::vector<Arc> arcs;
  std::vector<std::vector<int>> adj;
  std::vector<char> seen;
  explicit Flow(int nodes) : adj(nodes), seen(nodes) {}
  int add(int u, int v, int cap) {
    adj[u].push_back((int) arcs.size()); arcs.push_back({v, cap});
    adj[v].push_back((int) arcs.size()); arcs.push_back({u, 0});
    return (int) arcs.size() - 2;
  }
  int push(int u, int t, int f) {
    if (u == t) return f;
    seen[u] = 1;
    for (int id : adj[u]) {
      Arc &a = arcs[id];
      if (a.cap <= 0 || seen[a.to]) continue;
      const int got = push(a.to, t, std::min(f, a.cap));
      if (got > 0) { a.cap -= got; arcs[id ^ 1].cap += got; return got; }
    }
    return 0;
  }
  int run(int s, int t) {
    int total = 0;
    while (true) {
      std::fill(seen.begin(), seen.end(), 0);
      const int got = push(s, t, 1 << 20);
      if (got == 0) return total;
      total += got;
    }
  }
};

// A schedule with E double slots; false when the entries cannot be split that way.
bool schedule_with_double_slots(const std::vector<uint16_t> (&lists)[32], int n, int E,
                                uint16_t pad_base, std::vector<uint16_t> &out /* [n][32] */) {
  std::vector<SchedEdge> edges;
  int deg_l[32] = {0}, deg_b[kBanks] = {0};
  for (int l = 0; l < 32; ++l)
    for (uint16_t s : lists[l]) {
      edges.push_back({l, s % kBanks, s, 0, -1});
      ++deg_l[l];
      ++deg_b[s % kBanks];
    }
  if (E > n) return false;
  const int single = n - E;                          // slots in which a bank is read once

  // which entries go into the double slots: a flow with lower and upper bounds
  std::vector<char> doubled(edges.size(), 0);
  if (E > 0) {
    // nodes: 0 source, 1..32 lanes, 33..64 banks, 65 sink, 66 / 67 the super source and sink that
    // carry the lower bounds
    Flow f(68);
    const int S = 0, T = 65, SS = 66, TT = 67;
    int excess[68] = {0};
    auto bounded = [&](int u, int v, int lo, int hi) {
      excess[v] += lo;
      excess[u] -= lo;
      return f.add(u, v, hi - lo);
    };
    int pair_arc[32][kBanks];
    int mult[32][kBanks] = {{0}};
    for (const SchedEdge &e : edges) ++mult[e.lane][e.bank];
    for (int l = 0; l < 32; ++l) {
      const int lo = std::max(0, deg_l[l] - single), hi = std::min(E, deg_l[l]);
      if (lo > hi) return false;
      bounded(S, 1 + l, lo, hi);
      for (int b = 0; b < kBanks; ++b)
        pair_arc[l][b] = mult[l][b] > 0 ? f.add(1 + l, 33 + b, mult[l][b]) : -1;
    }
    for (int b = 0; b < kBanks; ++b) {
      const int lo = std::max(0, deg_b[b] - single), hi = std::min(2 * E, deg_b[b]);
      if (lo > hi) return false;
      bounded(33 + b, T, lo, hi);
    }
    f.add(T, S, 1 << 20);
    int demand = 0;
    for (int v = 0; v < 66; ++v) {
      if (excess[v] > 0) { f.add(SS, v, excess[v]); demand += excess[v]; }
      if (excess[v] < 0) f.add(v, TT, -excess[v]);
    }
    if (f.run(SS, TT) != demand) return false;
    int take[32][kBanks];
    for (int l = 0; l < 32; ++l)
      for (int b = 0; b < kBanks; ++b)
        take[l][b] = pair_arc[l][b] >= 0 ? mult[l][b] - f.arcs[pair_arc[l][b]].cap : 0;
    for (size_t i = 0; i < edges.size(); ++i)
      if (take[edges[i].lane][edges[i].bank] > 0) {
        --take[edges[i].lane][edges[i].bank];
        doubled[i] = 1;
      }
  }

  // colour the two parts; in the double slots a bank is two nodes with at most E edges each
  std::vector<int> ids_single, ids_double, atL, atR;
  int seen_b[kBanks] = {0};
  for (size_t i = 0; i < edges.size(); ++i) {
    if (doubled[i]) {
      edges[i].node = edges[i].bank + (seen_b[edges[i].bank]++ < E ? 0 : kBanks);
      ids_double.push_back((int) i);
    } else {
      edges[i].node = edges[i].bank;
      ids_single.push_back((int) i);
    }
  }
  out.assign((size_t) n * 32, 0xFFFF);
  if (E > 0) {
    colour_by_alternating_paths(edges, ids_double, E, 2 * kBanks, atL, atR);
    for (int id : ids_double) out[(size_t) edges[id].colour * 32 + edges[id].lane] = edges[id].slot;
  }
  if (single > 0) {
    colour_by_alternating_paths(edges, ids_single, single, kBanks, atL, atR);
    for (int id : ids_single) out[(size_t) (E + edges[id].colour) * 32 + edges[id].lane] = edges[id].slot;
  } else if (!ids_single.empty()) {
    return false;
  }
  // padding: the emptiest bank of the slot
  for (int t = 0; t < n; ++t) {
    int use[kBanks] = {0};
    for (int l = 0; l < 32; ++l)
      if (out[(size_t) t * 32 + l] != 0xFFFF) ++use[out[(size_t) t * 32 + l] % kBanks];
    for (int l = 0; l < 32; ++l) {
      if (out[(size_t) t * 32 + l] != 0xFFFF) continue;
      int b = 0;
      for (int c = 1; c < kBanks; ++c)
        if (use[c] < use[b]) b = c;
      ++use[b];
      out[(size_t) t * 32 + l] = (uint16_t) (pad_base + b);
    }
  }
  return true;
}

// Order in which a half-wave (32 lanes, one group each) reads its lists, chosen so that the 32
// addresses of a time slot fall into different LDS banks wherever that is possible.  lists[l]
// holds lane l's tile-local slots; every lane gets exactly n entries back, its own slots plus
// padding slots pad_base + bank.  The colouring gives the schedule with the fewest extra passes
// this half-wave can have; should it not be found, the greedy schedule with the local search on
// top stands in.
void schedule_half_wave(std::vector<uint16_t> (&lists)[32], int n, uint16_t pad_base,
                        std::vector<uint16_t> &out /* [n][32] */) {
  int deg_b[kBanks] = {0}, least = 0;
  for (const auto &l : lists)
    for (uint16_t s : l) least = std::max(least, ++deg_b[s % kBanks] - n);
  // the lanes put at most one entry each into a double slot, so very uneven banks can need a
  // few more of them than the fullest bank alone asks for
  for (int E = least; E <= std::min(n, least + 4); ++E)
    if (schedule_with_double_slots(lists, n, E, pad_base, out)) return;
  schedule_greedy(lists, n, pad_base, out);
  improve_schedule(out, n, pad_base);
}

// Reorders, block by block, the chunk's groups in `order` (sorted by list length, longest
// first): each block's groups are dealt to its half-waves of 32 positions one after the other,
// every group to the half-wave whose banks it loads most evenly (least growth of the sum of
// squared bank loads over the tiles).
void balance_blocks(std::vector<int32_t> &order, int32_t g0, const Shape &sh, const int32_t *row_ptr,
                    const int32_t *members) {
  const int32_t T = sh.ntiles, ng = (int32_t) order.size();
  constexpr int kHalf = 32, kDomains = kBlockGroups / kHalf;
  std::vector<int> load((size_t) kDomains * T * kBanks), hist((size_t) T * kBanks), peak(kDomains * T);
  std::vector<int32_t> placed(kBlockGroups);
  for (int32_t b0 = 0; b0 < ng; b0 += kBlockGroups) {
    const int32_t nb = std::min(kBlockGroups, ng - b0);
    const int ndom = (nb + kHalf - 1) / kHalf;
    std::fill(load.begin(), load.end(), 0);
    std::fill(peak.begin(), peak.end(), 0);
    int fill[kDomains] = {0};
    for (int32_t i = 0; i < nb; ++i) {
      const int32_t k = order[b0 + i];
      std::fill(hist.begin(), hist.end(), 0);
      for (int32_t j = row_ptr[g0 + k]; j < row_ptr[g0 + k + 1]; ++j) {
        const int32_t h = members[j] / sh.tile_len;
        ++hist[(size_t) h * kBanks + (members[j] - h * sh.tile_len) % kBanks];
      }
      int best = -1;
      long best_cost = 0;
      for (int d = 0; d < ndom; ++d) {
        if (fill[d] >= std::min(kHalf, nb - d * kHalf)) continue;
        // growth of the sum of squared bank loads (up to a constant): flattens every bank, not
        // only the fullest; ties go to the emptier half-wave
        long dot = 0;
        for (int32_t h = 0; h < T; ++h) {
          const int *ld = &load[((size_t) d * T + h) * kBanks], *hg = &hist[(size_t) h * kBanks];
          for (int b = 0; b < kBanks; ++b) dot += (long) ld[b] * hg[b];
        }
        const long cost = dot * 64 + fill[d];
        if (best < 0 || cost < best_cost) { best = d; best_cost = cost; }
      }
      for (int32_t h = 0; h < T; ++h) {
        int *ld = &load[((size_t) best * T + h) * kBanks];
        for (int b = 0; b < kBanks; ++b) {
          ld[b] += hist[(size_t) h * kBanks + b];
          peak[best * T + h] = std::max(peak[best * T + h], ld[b]);
        }
      }
      placed[best * kHalf + fill[best]++] = k;
    }
    for (int32_t i = 0; i < nb; ++i) order[b0 + i] = placed[i];
  }
}

// Builds the layout; with blob == nullptr only sizes are computed.
// `weighted` adds the weight stream (weights may be NULL while only sizes are asked for).
int build(int32_t V, int32_t G, const int32_t *row_ptr, const int32_t *members, const float *weights,
          bool weighted, int32_t chunk_groups, uint8_t *blob, size_t blob_bytes, pcg_prepared *info) {
  Shape sh;
  if (!make_shape(V, G, chunk_groups, sh)) return PCG_ERR_BAD_SHAPE;
  if (row_ptr[0] != 0) return PCG_ERR_BAD_CSR;
  for (int32_t g = 0; g < G; ++g)
    if (row_ptr[g + 1] < row_ptr[g]) return PCG_ERR_BAD_CSR;
  for (int32_t j = 0, n = row_ptr[G]; j < n; ++j)
    if ((uint32_t) members[j] >= (uint32_t) V) return PCG_ERR_BAD_CSR;

  const int32_t T = sh.ntiles, BPC = sh.blocks_per_chunk;
  const size_t n_desc = (size_t) sh.nchunks * T * BPC;
  const size_t desc_bytes = (n_desc * 2 * sizeof(uint32_t) + 255) / 256 * 256;
  const size_t n_perm = (size_t) sh.nchunks * BPC * kBlockGroups;
  const size_t perm_bytes = (n_perm * sizeof(uint16_t) + 255) / 256 * 256;

  std::vector<uint32_t> desc(n_desc * 2, 0);
  std::vector<uint16_t> perm(n_perm, 0xFFFF);
  std::vector<int32_t> cnt;          // [group in chunk][tile]
  std::vector<int32_t> order;
  uint64_t units = 0;                // 16-byte units of data

  // pass 1: order the groups of each chunk, size the blocks
  for (int32_t c = 0; c < sh.nchunks; ++c) {
    const int32_t g0 = c * sh.chunk_groups, ng = std::min(sh.chunk_groups, G - g0);
    cnt.assign((size_t) ng * T, 0);
    for (int32_t k = 0; k < ng; ++k)
      for (int32_t j = row_ptr[g0 + k]; j < row_ptr[g0 + k + 1]; ++j)
        ++cnt[(size_t) k * T + members[j] / sh.tile_len];
    order.resize(ng);
    std::iota(order.begin(), order.end(), 0);
    // longest lists first, tile by tile; ties by group id so that the layout is unique
    std::stable_sort(order.begin(), order.end(), [&](int32_t a, int32_t b) {
      for (int32_t h = 0; h < T; ++h) {
        const int32_t ca = cnt[(size_t) a * T + h], cb = cnt[(size_t) b * T + h];
        if (ca != cb) return ca > cb;
      }
      return false;
    });
    // Position k = block * 256 + r * 64 + lane.  The 32 groups of a half-wave (positions
    // 32 i .. 32 i + 31 of a block) are read together, and what that costs grows with the load of
    // their fullest bank; inside a block the groups are therefore dealt to the half-waves so as
    // to keep those bank loads flat, in every tile.
    balance_blocks(order, g0, sh, row_ptr, members);
    for (int32_t k = 0; k < ng; ++k)
      perm[(size_t) c * BPC * kBlockGroups + k] = (uint16_t) order[k];
    for (int32_t bl = 0; bl < BPC; ++bl) {
      for (int32_t h = 0; h < T; ++h) {
        int32_t longest = 0;
        for (int32_t l = 0; l < kBlockGroups && bl * kBlockGroups + l < ng; ++l)
          longest = std::max(longest, cnt[(size_t) order[bl * kBlockGroups + l] * T + h]);
        const int32_t steps = (longest + 1) / 2;               // two slots per dword
        uint32_t *d = &desc[(((size_t) c * T + h) * BPC + bl) * 2];
        if (units > 0xFFFFFFFFull) return PCG_ERR_BAD_SHAPE;
        d[0] = (uint32_t) units;
        d[1] = (uint32_t) steps;
        units += (uint64_t) steps * 64;
      }
    }
  }
  if (units > 0xFFFFFFFFull / 4) return PCG_ERR_BAD_SHAPE;
  const size_t data_bytes = ((size_t) units * 16 + 255) / 256 * 256 + 1024;   // never empty
  const size_t weight_bytes = weighted ? 2 * data_bytes : 0;      // one float per 16-bit slot
  const size_t total = desc_bytes + perm_bytes + data_bytes + weight_bytes;
  if (info) {
    info->V = V; info->G = G;
    info->ntiles = T; info->tile_len = sh.tile_len;
    info->chunk_groups = sh.chunk_groups; info->nchunks = sh.nchunks;
    info->blocks_per_chunk = BPC; info->reserved = 0;
    info->off_desc = 0;
    info->off_perm = (int64_t) desc_bytes;
    info->off_data = (int64_t) (desc_bytes + perm_bytes);
    info->off_weights = weighted ? (int64_t) (desc_bytes + perm_bytes + data_bytes) : 0;
    info->bytes = (int64_t) total;
  }
  if (!blob) return PCG_OK;
  if (blob_bytes < total) return PCG_ERR_WORKSPACE_TOO_SMALL;

  // pass 2: emit
  std::memset(blob, 0, total);
  std::memcpy(blob, desc.data(), desc.size() * sizeof(uint32_t));
  std::memcpy(blob + desc_bytes, perm.data(), perm.size() * sizeof(uint16_t));
  uint32_t *data = reinterpret_cast<uint32_t *>(blob + desc_bytes + perm_bytes);
  float *wdata = weighted ? reinterpret_cast<float *>(blob + desc_bytes + perm_bytes + data_bytes)
                          : nullptr;
  const uint16_t pad_base = (uint16_t) sh.tile_len;   // table[tile_len .. tile_len + kBanks) is zero
  // Blocks are independent of each other and write disjoint parts of the blob: they are handed
  // out to a few threads, one block at a time (the result does not depend on who takes which).
  const int64_t nblocks = (int64_t) sh.nchunks * BPC;
  std::atomic<int64_t> next_block{0};
  auto worker = [&]() {
    std::vector<uint16_t> lists[32], sched;
    std::vector<std::pair<uint16_t, float>> share[32];   // (slot, weight) of each lane's list, by slot
    for (int64_t w = next_block.fetch_add(1); w < nblocks; w = next_block.fetch_add(1)) {
      const int32_t c = (int32_t) (w / BPC), bl = (int32_t) (w % BPC);
      const int32_t g0 = c * sh.chunk_groups;
      for (int32_t h = 0; h < T; ++h) {
        const uint32_t *d = &desc[(((size_t) c * T + h) * BPC + bl) * 2];
        const size_t off = d[0];
        const uint32_t steps = d[1];
        if (steps == 0) continue;
        for (int32_t r = 0; r < kLaneGroups; ++r) {
          for (int32_t half = 0; half < 2; ++half) {
            for (int32_t l = 0; l < 32; ++l) {
              lists[l].clear();
              share[l].clear();
              const uint16_t k = perm[((size_t) c * BPC + bl) * kBlockGroups + r * 64 + half * 32 + l];
              if (k == 0xFFFF) continue;
              for (int32_t j = row_ptr[g0 + k]; j < row_ptr[g0 + k + 1]; ++j)
                if (members[j] / sh.tile_len == h) {
                  lists[l].push_back((uint16_t) (members[j] - h * sh.tile_len));
                  if (weighted) share[l].emplace_back(lists[l].back(), weights[j]);
                }
              std::sort(share[l].begin(), share[l].end());
            }
            schedule_half_wave(lists, (int) steps * 2, pad_base, sched);
            for (uint32_t q = 0; q < steps; ++q)
              for (int32_t l = 0; l < 32; ++l) {
                const size_t unit = off + (size_t) q * 64 + half * 32 + l;
                const uint16_t s0 = sched[(size_t) (2 * q) * 32 + l];
                const uint16_t s1 = sched[(size_t) (2 * q + 1) * 32 + l];
                data[unit * 4 + r] = (uint32_t) s0 | ((uint32_t) s1 << 16);
                if (!weighted) continue;
                // a group's members are distinct, so a slot names one entry of the lane's list
                auto weight_of = [&](uint16_t s) {
                  if (s >= pad_base) return 0.f;
                  auto it = std::lower_bound(share[l].begin(), share[l].end(),
                                             std::make_pair(s, -1.f));
                  return it->second;
                };
                wdata[(unit * 4 + r) * 2] = weight_of(s0);
                wdata[(unit * 4 + r) * 2 + 1] = weight_of(s1);
              }
          }
        }
      }
    }
  };
  const unsigned hw = std::thread::hardware_concurrency();
  const int nthreads = (int) std::max<int64_t>(1, std::min<int64_t>({(int64_t) (hw ? hw : 1), 8, nblocks / 4}));
  std::vector<std::thread> pool;
  for (int i = 1; i < nthreads; ++i) pool.emplace_back(worker);
  worker();
  for (auto &t : pool) t.join();
  return PCG_OK;
}

}  // namespace

extern "C" {

size_t pcg_groups_prepare_bytes(int32_t V, int32_t G, const int32_t *row_ptr,
                                const int32_t *members, int32_t chunk_groups) {
  if (!row_ptr || (G > 0 && row_ptr[G] > 0 && !members)) return 0;
  pcg_prepared info;
  if (build(V, G, row_ptr, members, nullptr, false, chunk_groups, nullptr, 0, &info) != PCG_OK)
    return 0;
  return (size_t) info.bytes;
}

int pcg_groups_prepare_host(int32_t V, int32_t G, const int32_t *row_ptr, const int32_t *members,
                            int32_t chunk_groups, void *blob, size_t blob_bytes,
                            pcg_prepared *info) {
  if (!row_ptr || !blob || !info) return PCG_ERR_NULL_ARG;
  if (G > 0 && row_ptr[G] > 0 && !members) return PCG_ERR_NULL_ARG;
  return build(V, G, row_ptr, members, nullptr, false, chunk_groups, (uint8_t *) blob, blob_bytes,
               info);
}

size_t pcg_groups_prepare_weights_bytes(int32_t V, int32_t G, const int32_t *row_ptr,
                                        const int32_t *members, int32_t chunk_groups) {
  if (!row_ptr || (G > 0 && row_ptr[G] > 0 && !members)) return 0;
  pcg_prepared info;
  if (build(V, G, row_ptr, members, nullptr, true, chunk_groups, nullptr, 0, &info) != PCG_OK)
    return 0;
  return (size_t) info.bytes;
}

int pcg_groups_prepare_weights_host(int32_t V, int32_t G, const int32_t *row_ptr,
                                    const int32_t *members, const float *weights,
                                    int32_t chunk_groups, void *blob, size_t blob_bytes,
                                    pcg_prepared *info) {
  if (!row_ptr || !blob || !info) return PCG_ERR_NULL_ARG;
  if (G > 0 && row_ptr[G] > 0 && (!members || !weights)) return PCG_ERR_NULL_ARG;
  return build(V, G, row_ptr, members, weights, true, chunk_groups, (uint8_t *) blob, blob_bytes,
               info);
}

}  // extern "C"
