// Test harness for the grid-row planner of the batched kernels (csrc/row_plan.hpp): reads "granule max_rows max_piece"
// and the tile counts of the items from stdin, prints one line per launch ("L <row_length>") followed by its rows
// ("R <item> <first_tile> <n_tiles>").  Built and driven by tests/test_row_plan.py.
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "../../paper_2212_05339_amd/csrc/row_plan.hpp"

struct Sink {
    std::vector<long> item, first, len;
    void add(int i, int64_t f, int64_t n) {
        item.push_back(i);
        first.push_back((long)f);
        len.push_back((long)n);
    }
    int flush(int64_t row_length) {
        std::printf("L %ld\n", (long)row_length);
        for (size_t k = 0; k < item.size(); ++k) std::printf("R %ld %ld %ld\n", item[k], first[k], len[k]);
        item.clear();
        first.clear();
        len.clear();
        return 0;
    }
};

int main() {
    long granule, max_rows, max_piece, x;
    if (std::scanf("%ld %ld %ld", &granule, &max_rows, &max_piece) != 3) return 2;
    std::vector<long> tiles;
    while (std::scanf("%ld", &x) == 1) tiles.push_back(x);
    Sink sink;
    return elixir::plan_rows((int)tiles.size(), [&](int i) -> int64_t { return tiles[i]; }, granule, (int)max_rows, max_piece, sink);
}
