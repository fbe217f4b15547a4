// Driver for the sanitizer run of the library's host-side arithmetic.  Built by
// tests/test_host_sanitized.py with g++ -fsanitize=address,undefined from this file,
// csrc/nts_host.hip and csrc/nts_planner.hip (both plain C++), no GPU runtime.  Reads
// one command per line from stdin, prints one result line per command; the Python
// test compares the results with the oracle / with arithmetic of its own and
// requires a clean exit (any sanitizer report aborts with a non-zero status).
#include <inttypes.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <iostream>
#include <sstream>
#include <string>
#include <vector>

#include "nts_host.h"

// a double from the next token; strtod, because stream extraction does not read "nan"
static double next_double(std::istringstream &in)
{
    std::string tok;
    in >> tok;
    return strtod(tok.c_str(), nullptr);
}

int main()
{
    std::string line;
    while (std::getline(std::cin, line)) {
        std::istringstream in(line);
        std::string cmd;
        if (!(in >> cmd)) continue;
        if (cmd == "route") {
            int H, Ns, rs, Nd, rd, so = -1, dof = -1, w = -1;
            in >> H >> Ns >> rs >> Nd >> rd;
            const int rc = nts_host_route(H, Ns, rs, Nd, rd, &so, &dof, &w);
            printf("route %d %d %d %d\n", rc, so, dof, w);
        } else if (cmd == "route_null") {                   // one of the three result pointers missing
            int which, a = 0, b = 0, c = 0;
            in >> which;
            printf("route_null %d\n", nts_host_route(8, 2, 0, 4, 1, which == 0 ? nullptr : &a, which == 1 ? nullptr : &b,
                                                     which == 2 ? nullptr : &c));
        } else if (cmd == "geom" || cmd == "geom_nosrc" || cmd == "geom_nodst") {
            nts_desc d;
            memset(&d, 0, sizeof d);
            int64_t staging;
            unsigned flags;
            in >> d.L >> d.D >> d.elem_bytes >> d.page_size >> d.Hs >> d.Hd >> d.src_head_off >> d.dst_head_off >>
                d.w >> d.S_src >> d.S_dst >> d.src_token_stride >> d.dst_token_stride >> staging >> flags >> d.n_req;
            d.staging_bytes = staging;
            d.flags = flags;
            std::vector<int32_t> len(size_t(d.n_req > 0 ? d.n_req : 0));
            for (auto &x : len) in >> x;
            int32_t one_page = 0;
            d.ctx_len = len.data();
            d.src_pages = d.dst_pages = &one_page;          // only their being non-null matters here
            if (cmd == "geom_nosrc") d.src_pages = nullptr;
            if (cmd == "geom_nodst") d.dst_pages = nullptr;
            NtsGeometry g;
            const char *why = "";
            const int rc = nts_host_plan_geometry(&d, &g, &why);
            printf("geom %d", rc);
            if (rc == NTS_OK) {
                printf(" %" PRId64 " %" PRId64 " %" PRId64 " %" PRId64 " %" PRId64 " %" PRId64 " %" PRId64 " %" PRId64
                       " %" PRId64 " %" PRId64 " %d",
                       g.T, g.NP, g.F, g.frag_bytes, g.X, g.chunk_frags, g.chunk_bytes, g.n_chunks, g.src_stride,
                       g.dst_stride, g.vec);
                for (int32_t v : g.tok_off) printf(" %d", v);
                for (int32_t v : g.pg_off) printf(" %d", v);
                // walk the chunks: they must tile [0, F) exactly
                int64_t at = 0, bad = 0;
                for (int64_t k = 0; k < g.n_chunks; ++k) {
                    int64_t q0, n;
                    if (nts_host_chunk_range(g.F, g.chunk_frags, g.n_chunks, k, &q0, &n) != NTS_OK || q0 != at || n < 1) ++bad;
                    at = q0 + n;
                }
                int64_t q0, n;
                if (nts_host_chunk_range(g.F, g.chunk_frags, g.n_chunks, g.n_chunks, &q0, &n) == NTS_OK) ++bad;
                printf(" tiles %d", int(bad == 0 && at == g.F));
            } else {
                printf(" %s", why);
            }
            printf("\n");
        } else if (cmd == "alias") {
            int n;
            in >> n;
            std::vector<NtsByteRange> r(size_t(n > 0 ? n : 0));
            for (auto &x : r) {
                uint64_t lo, hi;
                in >> lo >> hi >> x.is_dst;
                x.lo = uintptr_t(lo);
                x.hi = uintptr_t(hi);
            }
            uint64_t stg;
            int64_t stg_bytes;
            in >> stg >> stg_bytes;
            const char *why = "";
            printf("alias %d\n", nts_host_alias_sweep(r, uintptr_t(stg), stg_bytes, &why));
        } else if (cmd == "staging") {
            int n;
            in >> n;
            std::vector<int64_t> cb(size_t(n > 0 ? n : 0));
            for (auto &x : cb) in >> x;
            printf("staging %" PRId64 "\n", nts_host_batch_staging_bytes(cb.data(), n));
        } else if (cmd == "block") {
            const double thp = next_double(in), thd = next_double(in);
            int m, P = 0, D = 0;
            in >> m;
            const int rc = nts_balanced_block(thp, thd, m, &P, &D);
            printf("block %d %d %d\n", rc, P, D);
        } else if (cmd == "ge") {
            double ge = 0;
            int tpi, tpj, P, D;
            const double thp = next_double(in);
            in >> tpi;
            const double thd = next_double(in);
            in >> tpj >> P >> D;
            const double rps = next_double(in);
            const int rc = nts_goodput_efficiency(thp, tpi, thd, tpj, P, D, rps, &ge);
            printf("ge %d %.17g\n", rc, ge);
        } else if (cmd == "plan") {
            int n_gpus, n_tiers, max_inst, max_out;
            in >> n_gpus >> n_tiers >> max_inst >> max_out;
            std::vector<nts_tier> tiers(size_t(n_tiers > 0 ? n_tiers : 0));
            for (auto &t : tiers) {
                t.rps = next_double(in);
                for (double &v : t.thp) v = next_double(in);
                for (double &v : t.thd) v = next_double(in);
            }
            std::vector<nts_alloc> out(size_t(max_out > 0 ? max_out : 0));
            int n = 0, left = 0;
            const int rc = nts_plan_cluster(n_gpus, n_tiers, tiers.data(), max_inst, out.data(), max_out, &n, &left);
            printf("plan %d %d %d", rc, n, left);
            for (int i = 0; i < n && i < max_out; ++i)
                printf(" %d %d %d %d %d %d %.17g", out[size_t(i)].tier, out[size_t(i)].tp_prefill, out[size_t(i)].tp_decode,
                       out[size_t(i)].P, out[size_t(i)].D, out[size_t(i)].gpus, out[size_t(i)].served_rps);
            printf("\n");
        } else {
            printf("unknown %s\n", cmd.c_str());
        }
    }
    return 0;
}
