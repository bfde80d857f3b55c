// Test harness for the grid-row planner of the batched kernels (csrc/row_plan.hpp): reads "granule max_rows max_piece"
// and the tile counts of the items from stdin, prints one line per launch ("L <row_length>") followed by its rows
// ("R <item> <first_tile> <n_tiles>").  With the argument "table" it drives the compact row table instead: reads rows
// "<dst address> <src address or 0> <count>" (offset units 16 and 8 bytes, 64 counts per tile) and prints every table
// handed to the launch ("T <rows> <longest> <dst_base> <src_base>", then "R <dst_off> <src_off> <count>" per row and
// "P <dst_off> <src_off> <count>" per unused entry that is not cleared).  Built and driven by tests/test_row_plan.py.
#include <cstdio>
#include <cstdlib>
#include <string>
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

struct PrintTable {
    int operator()(const elixir::CompactRows& tab, int rows, int64_t longest) const {
        std::printf("T %d %ld %llu %llu\n", rows, (long)longest, (unsigned long long)(uintptr_t)tab.dst_base, (unsigned long long)(uintptr_t)tab.src_base);
        for (int r = 0; r < rows; ++r) std::printf("R %u %u %u\n", tab.dst_off[r], tab.src_off[r], tab.count[r]);
        for (int r = rows; r < elixir::kCompactRows; ++r)
            if (tab.dst_off[r] != 0 || tab.src_off[r] != elixir::kNoSource || tab.count[r] != 0)
                std::printf("P %u %u %u\n", tab.dst_off[r], tab.src_off[r], tab.count[r]);
        return 0;
    }
};

int table_mode() {
    elixir::CompactRowBuilder<16, 8, 64, PrintTable> b{PrintTable()};
    unsigned long long d, s;
    long count;
    while (std::scanf("%llu %llu %ld", &d, &s, &count) == 3)
        if (const int rc = b.add(reinterpret_cast<char*>((uintptr_t)d), reinterpret_cast<const char*>((uintptr_t)s), count)) return rc;
    return b.flush();
}

int main(int argc, char** argv) {
    if (argc > 1 && std::string(argv[1]) == "table") return table_mode();
    long granule, max_rows, max_piece, x;
    if (std::scanf("%ld %ld %ld", &granule, &max_rows, &max_piece) != 3) return 2;
    std::vector<long> tiles;
    while (std::scanf("%ld", &x) == 1) tiles.push_back(x);
    Sink sink;
    return elixir::plan_rows((int)tiles.size(), [&](int i) -> int64_t { return tiles[i]; }, granule, (int)max_rows, max_piece, sink);
}
