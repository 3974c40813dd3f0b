// Host-side check of the integer helpers the kernels and launchers really use (csrc/hexi_internal.h), compiled
// for the host alone.  Reads commands from stdin, one per line:
//   seg  n  start_0 len_0 ... start_{n-1} len_{n-1}  p_0 p_1 ...
//        prints the global position of every packed row (seg_pos_of_row), then "|", then seg_rows_le(p_i) for every p_i
//   runs nq nkv run_len  kv_of_q[0..nq-1]
//        prints shared (0/1), the number of runs, then per run "first:len:" and its heads in walking order
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
        std::string cmd;
        is >> cmd;
        if (cmd == "seg") {
            SegTable t = {};
            is >> t.n;
            int rows = 0;
            for (int s = 0; s < t.n; ++s) {
                int len;
                is >> t.start[s] >> len;
                t.row0[s] = rows;
                rows += len;
            }
            for (int s = t.n; s <= HEXI_MAX_SEGS; ++s) t.row0[s] = rows;
            t.total = rows;
            for (int r = 0; r < rows; ++r) std::printf("%d ", seg_pos_of_row(t, r));
            std::printf("|");
            int p;
            while (is >> p) std::printf(" %d", seg_rows_le(t, p));
            std::printf("\n");
        } else if (cmd == "runs") {
            int nq, nkv, run_len;
            is >> nq >> nkv >> run_len;
            signed char kv_of_q[HEXI_MAX_HEADS];
            for (int h = 0; h < nq; ++h) { int x; is >> x; kv_of_q[h] = (signed char)x; }
            HeadRuns runs;
            const bool shared = hexi_build_head_runs(kv_of_q, nq, nkv, run_len, &runs);
            std::printf("%d %d", shared ? 1 : 0, runs.n);
            for (int r = 0; r < runs.n; ++r) {
                std::printf(" %d:%d:", (int)runs.first[r], (int)runs.len[r]);
                for (int h = runs.first[r]; h >= 0; h = runs.next[h]) std::printf("%d,", h);
            }
            std::printf("\n");
        }
    }
    return 0;
}
