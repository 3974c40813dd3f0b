// Host-side check of the launchers' XCD work split (hexi_split_units in csrc/hexi_internal.h): prints, for the
// unit-weight lists read from stdin (one list per line), the nine range starts and the grid size.
#include <cstdio>
#include <iostream>
#include <sstream>
#include <string>
#include <vector>
#include "hexi_internal.h"

int main()
{
    std::string line;
    while (std::getline(std::cin, line)) {
        std::istringstream is(line);
        std::vector<double> w;
        double x;
        while (is >> x) w.push_back(x);
        unsigned grid = 0;
        const XcdSplit s = hexi_split_units((int)w.size(), [&](int u) { return w[u]; }, &grid);
        for (int i = 0; i < 9; ++i) std::printf("%d ", s.start[i]);
        std::printf("%u\n", grid);
    }
    return 0;
}
