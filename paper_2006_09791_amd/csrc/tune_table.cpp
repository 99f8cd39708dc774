// Offline tile-table lookup: an autotuner (paper_2006_09791_amd/autotune.py) measures, per
// layer shape, which kernel family and tile configuration is fastest and writes a text
// table; a process that sets GSPC_TUNE_FILE to it gets those choices instead of the
// planners' heuristics.  The paper leaves exactly these knobs (tile sizes, unrolling) to an
// auto-tuner (Section III-C); here the search runs offline and the result is a table.
//
// Format: one layer per line, '#' starts a comment:
//   N Cin H W Cout KH KW stride pad groups dtype family index
// dtype 0 = fp32, 1 = bf16; family 'w' = 16x16x4 kernel with resident filters, 'm' = 16x16x4
// kernel, 'b' = bf16 16x16x32 kernel, 'q' = 4x4x1 kernel, 'x' = Winograd F(2x2, 3x3) kernel, 'r' = bf16 row-product kernel; index = position in that family's
// configuration list (for 'q': pixel runs per wave, 1 | 2 | 4).  Entries that a planner cannot
// realise are ignored (the heuristic choice is used).
#include <array>
#include <cstdio>
#include <cstdlib>
#include <map>
#include <mutex>

#include "gspc_internal.h"

namespace gspc {

namespace {

using Key = std::array<int, 11>;
struct Entry {
    char family;
    int index;
};
std::map<Key, Entry> g_table;
std::once_flag g_once;

void load_table() {
    const char *path = std::getenv("GSPC_TUNE_FILE");
    if (!path || !*path) return;
    FILE *f = std::fopen(path, "r");
    if (!f) {
        std::fprintf(stderr, "libgspc: cannot open GSPC_TUNE_FILE=%s, using the built-in heuristics\n", path);
        return;
    }
    char line[512];
    while (std::fgets(line, sizeof(line), f)) {
        Key k{};
        char fam = 0;
        int idx = -1;
        if (line[0] == '#') continue;
        if (std::sscanf(line, "%d %d %d %d %d %d %d %d %d %d %d %c %d", &k[0], &k[1], &k[2], &k[3], &k[4], &k[5],
                        &k[6], &k[7], &k[8], &k[9], &k[10], &fam, &idx) != 13)
            continue;
        if ((fam == 'w' || fam == 'm' || fam == 'b' || fam == 'q' || fam == 'x' || fam == 'r') && idx >= 0) g_table[k] = Entry{fam, idx};
    }
    std::fclose(f);
}

const Entry *find(const ConvParams &p) {
    std::call_once(g_once, load_table);
    if (g_table.empty()) return nullptr;
    // keyed by the caller's plane size: 1x1 layers reach the planners with re-pitched planes
    const Key k{p.N, p.Cin, p.H0, p.W0, p.Cout, p.KH, p.KW, p.stride, p.pad, p.groups, p.in_bf16 ? 1 : 0};
    auto it = g_table.find(k);
    return it == g_table.end() ? nullptr : &it->second;
}

}  // namespace

char tuned_family(const ConvParams &p) {
    const Entry *e = find(p);
    return e ? e->family : '\0';
}

int tuned_config(const ConvParams &p, char family) {
    const Entry *e = find(p);
    return e && e->family == family ? e->index : -1;
}

}  // namespace gspc
