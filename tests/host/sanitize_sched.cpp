// The host scheduler and performance model (csrc/hexi_sched.cpp, included as is) under AddressSanitizer and
// UndefinedBehaviorSanitizer.  Reads from stdin: n, then c[n], b[n], m[n], m_static[n], alpha[n*n], bw[n*n]; then
// l_tot batch hidden head_dim n_heads dtype_bytes gamma; then m1 m2 i_max token_quantum move_tokens.  Runs
// hexi_sched_solve and hexi_sched_cost on the result and prints the schedule and its cost terms in text form, for
// comparison with the library's own answer on the same input.  Any sanitizer report aborts the run.
#include <cstdarg>
#include <cstdio>
#include <iostream>
#include <vector>
#include "hexi_sched.cpp"

int hexi_set_error(int code, const char* fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    std::vfprintf(stderr, fmt, ap);
    std::fprintf(stderr, "\n");
    va_end(ap);
    return code;
}

int main()
{
    int n;
    if (!(std::cin >> n) || n < 1) return 2;
    std::vector<double> c(n), b(n), m(n), ms(n), al((size_t)n * n), bw((size_t)n * n);
    for (auto* v : {&c, &b, &m, &ms, &al, &bw})
        for (auto& x : *v) std::cin >> x;
    hexi_model mo;
    std::cin >> mo.l_tot >> mo.batch >> mo.hidden >> mo.head_dim >> mo.n_heads >> mo.dtype_bytes >> mo.gamma_act;
    hexi_sched_opts op = {};
    std::cin >> op.m1 >> op.m2 >> op.i_max >> op.token_quantum >> op.move_tokens;
    if (!std::cin) return 2;
    const hexi_cluster cl = {n, c.data(), b.data(), m.data(), ms.data(), al.data(), bw.data()};
    std::vector<int32_t> group_of(n), n_heads(n);
    std::vector<int64_t> l_group(n), s_pre(n);
    hexi_schedule out = {0, group_of.data(), l_group.data(), s_pre.data(), n_heads.data()};
    double cost = 0.0;
    int rc = hexi_sched_solve(&cl, &mo, &op, &out, &cost);
    if (rc != HEXI_OK) { std::printf("error %d\n", rc); return 0; }
    double terms[4];
    int32_t feasible = 0;
    rc = hexi_sched_cost(&cl, &mo, &out, terms, &feasible);
    if (rc != HEXI_OK) { std::printf("error %d\n", rc); return 0; }
    std::printf("groups %d\n", out.n_groups);
    for (int d = 0; d < n; ++d) std::printf("%d %lld %d\n", group_of[d], (long long)s_pre[d], n_heads[d]);
    for (int k = 0; k < out.n_groups; ++k) std::printf("L %lld\n", (long long)l_group[k]);
    std::printf("cost %.17g terms %.17g %.17g %.17g %.17g feasible %d\n", cost, terms[0], terms[1], terms[2], terms[3], feasible);
    return 0;
}
