// Host-side construction of the prepared membership layout (see pcg_prepared in pcg.h).
#include <algorithm>
#include <cstring>
#include <numeric>
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

// Order in which a half-wave (32 lanes, one group each) reads its lists, chosen so that the 32
// addresses of a time slot fall into different LDS banks wherever that is possible.  lists[l]
// holds lane l's tile-local slots; every lane gets exactly n entries back, its own slots plus
// padding slots pad_base + bank.  Greedy, one time slot after the other: lanes with the most
// entries left choose first, each takes an entry whose bank is still free in this slot
// (preferring the bank with the most entries still to place); a lane that finds none waits if
// it has slots to spare, and otherwise takes the least crowded bank.
void schedule_half_wave(std::vector<uint16_t> (&lists)[32], int n, uint16_t pad_base,
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
  std::vector<uint16_t> lists[32], sched;
  std::vector<std::pair<uint16_t, float>> share[32];   // (slot, weight) of each lane's list, by slot
  for (int32_t c = 0; c < sh.nchunks; ++c) {
    const int32_t g0 = c * sh.chunk_groups;
    for (int32_t bl = 0; bl < BPC; ++bl) {
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
  }
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
