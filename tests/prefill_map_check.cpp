// Host-side check of the workgroup id -> (unit, split, XCD) mapping of the bf16 prefill launch and of
// the dense layers' split-K launches (vs_prefill_map.h; there unit = block of output features, split =
// share of the input features), for every (units, splits, number of XCDs) the launch planners can emit:
// every (unit, split) pair is named by exactly one id of the grid, all splits of a unit carry
// ids of one residue modulo the number of XCDs, spare ids name no unit, and units that follow
// one another share a residue as long as that XCD has room.
#include <cstdio>
#include <vector>

#include "vs_prefill_map.h"

int main() {
    long checked = 0;
    for (int shift = 0; shift <= 4; ++shift) {
        for (int nsplit = 1; nsplit <= 16; ++nsplit) {
            const float inv_nsplit = 1.0f / (float)nsplit;
            for (int units = 1; units <= 1100; units += (units < 300 ? 1 : 37)) {
                const int upx = vs::prefill_units_per_xcd(units, shift);
                const unsigned ids = vs::prefill_grid_ids(units, nsplit, shift);
                if (ids != (unsigned)(upx * nsplit) << shift || upx * (1 << shift) < units) {
                    std::printf("grid too small: units %d nsplit %d shift %d\n", units, nsplit, shift);
                    return 1;
                }
                std::vector<int> seen((size_t)units * nsplit, 0), residue(units, -1);
                for (unsigned id = 0; id < ids; ++id) {
                    const vs::PrefillSlot s = vs::prefill_slot_of_id(id, units, upx, nsplit, inv_nsplit, shift);
                    if (s.xcd != (int)(id & ((1u << shift) - 1u))) { std::printf("residue\n"); return 1; }
                    if (s.unit < 0) continue;
                    if (s.unit >= units || s.split < 0 || s.split >= nsplit) { std::printf("range\n"); return 1; }
                    if (s.unit / upx != s.xcd) { std::printf("unit %d not on XCD %d\n", s.unit, s.xcd); return 1; }
                    ++seen[(size_t)s.unit * nsplit + s.split];
                    if (residue[s.unit] < 0) residue[s.unit] = s.xcd;
                    if (residue[s.unit] != s.xcd) {
                        std::printf("unit %d on two XCDs (units %d nsplit %d shift %d)\n", s.unit, units, nsplit, shift);
                        return 1;
                    }
                }
                for (size_t i = 0; i < seen.size(); ++i)
                    if (seen[i] != 1) {
                        std::printf("(unit, split) %zu named %d times (units %d nsplit %d shift %d)\n", i, seen[i], units,
                                    nsplit, shift);
                        return 1;
                    }
                ++checked;
            }
        }
    }
    // div_small against the integer division over its whole stated range of use
    for (int d = 1; d <= 64; ++d)
        for (int x = 0; x < (1 << 22); x += (x < 70000 ? 1 : 4093))
            if (vs::div_small(x, d, 1.0f / (float)d) != x / d) { std::printf("div_small(%d, %d)\n", x, d); return 1; }
    std::printf("ok %ld\n", checked);
    return 0;
}
