// Host-side check of pop::decode_block (csrc/pop_dev.h): for every grid shape the kernels use, the map from block
// ids to (unit, sub) is a bijection onto units x per_unit, units of whole groups of 8 sit on one XCD (ids congruent
// mod 8), left-over units on about 8 / r neighbouring XCDs, and the ORDERED form keeps `sub` growing with the id.
#include <cstdio>
#include <map>
#include <set>
#include "pop_dev.h"

int main() {
  int bad = 0;
  const int pers[] = {1, 3, 4, 8, 16, 19, 35, 37, 38, 42};
  const int offs[] = {0, 20};
  for (int units = 1; units <= 264; ++units)
    for (int per : pers)
      for (int off : offs) {
        std::set<std::pair<int, int>> seen;
        std::map<int, std::set<int>> xcds;
        std::map<int, int> last_sub;
        for (int id = 0; id < units * per; ++id) {
          int u = -1, s = -1;
          if (!pop::decode_block(id, units, per, u, s) || s < 0 || s >= per) { ++bad; continue; }
          seen.insert({u, s});
          xcds[u].insert((id + off) & 7);
          int uo = -1, so = -1;
          if (!pop::decode_block<true>(id, units, per, uo, so)) { ++bad; continue; }
          if (last_sub.count(uo) && so <= last_sub[uo]) ++bad;          // ORDERED: sub grows with the id within a unit
          last_sub[uo] = so;
        }
        if ((int)seen.size() != units * per) { ++bad; std::printf("not a bijection: units %d per_unit %d\n", units, per); }
        const int full = units & ~7, r = units - full;
        for (auto& kv : xcds) {
          const int limit = kv.first < full ? 1 : (8 + r - 1) / r + 1;
          if ((int)kv.second.size() > limit) { ++bad; std::printf("units %d per_unit %d: unit %d on %zu XCDs\n", units, per, kv.first, kv.second.size()); }
        }
      }
  {                                                                      // the headline population: 10 agents, 20 critics
    std::map<int, std::set<int>> a, c;
    int u, s;
    for (int id = 0; id < 160; ++id) { pop::decode_block(id, 10, 16, u, s); a[u].insert(id & 7); }
    for (int id = 0; id < 160; ++id) { pop::decode_block(id, 20, 8, u, s); c[u].insert(id & 7); }
    std::printf("P=10: agents 8, 9 on %zu and %zu XCDs; critics 16..19 on %zu %zu %zu %zu\n", a[8].size(), a[9].size(), c[16].size(),
                c[17].size(), c[18].size(), c[19].size());
    if (a[8].size() != 4 || a[9].size() != 4 || c[16].size() != 2 || c[19].size() != 2) ++bad;
  }
  std::printf("bad %d\n", bad);
  return bad != 0;
}
