// Test driver (host only, no GPU): runs the library's host-side code (strategy selector, n-gram drafter,
// static template) and the oracle's C acceptance rules under AddressSanitizer / UndefinedBehaviorSanitizer.
// Reads commands from stdin, prints results to stdout; tests/test_host_sanitizers.py builds it with
// -fsanitize=address,undefined, feeds it the host parity cases and compares the output with the Python oracles.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <string>
#include <vector>

#include "../include/tlt.h"

extern "C" {
void oracle_accept_greedy(int B, int n, int V, int stride, const int32_t* token, const int32_t* parent, const float* logits,
                          int32_t* accept_len, int32_t* path_idx, int32_t* out_tokens, int32_t* n_out);
void oracle_accept_sample_near(int B, int n, int V, int stride, float temperature, const int32_t* token, const int32_t* parent,
                               const float* logits, const float* draft_q, const uint32_t* u_accept, const uint32_t* u_final,
                               int32_t* accept_len, int32_t* path_idx, int32_t* out_tokens, int32_t* n_out, int32_t* near);
void oracle_accept_target_only_near(int B, int n, int V, int stride, float temperature, const int32_t* token,
                                    const int32_t* parent, const float* logits, const uint32_t* u_accept, const uint32_t* u_final,
                                    int32_t* accept_len, int32_t* path_idx, int32_t* out_tokens, int32_t* n_out, int32_t* near);
}

static long long rd() { long long v; if (scanf("%lld", &v) != 1) exit(3); return v; }
static double rdd() { double v; if (scanf("%lf", &v) != 1) exit(3); return v; }

int main() {
    char cmd[32];
    while (scanf("%31s", cmd) == 1) {
        std::string c = cmd;
        if (c == "tmpl") {
            int K = (int)rd(), D = (int)rd(), N = (int)rd();
            std::vector<int32_t> p(N > 0 ? N : 1), r(p.size()), d(p.size());
            int32_t n = 0;
            int rc = tlt_template_build(K, D, N, p.data(), r.data(), d.data(), &n);
            printf("%d %d", rc, rc ? 0 : n);
            for (int a = 0; a < (rc ? 0 : 3); ++a)
                for (int i = 0; i < n; ++i) printf(" %d", a == 0 ? p[i] : (a == 1 ? r[i] : d[i]));
            printf("\n");
        } else if (c == "mab") {
            int nS = (int)rd();
            std::vector<tlt_strategy> S(nS);
            for (auto& s : S) { s.draft_depth = (int)rd(); s.topk = (int)rd(); s.tokens_to_verify = (int)rd(); }
            int nT = (int)rd();
            std::vector<int32_t> T(nT);
            for (auto& t : T) t = (int)rd();
            double eps = rdd();
            int window = (int)rd(), sdthr = (int)rd(), nOps = (int)rd();
            tlt_mab* m = nullptr;
            int rc = tlt_mab_create(S.data(), nS, T.data(), nT, eps, window, sdthr, &m);
            printf("%d\n", rc);
            for (int o = 0; o < nOps; ++o) {
                char op[8];
                if (scanf("%7s", op) != 1) exit(3);
                if (op[0] == 's') {
                    int B = (int)rd();
                    uint32_t u1 = (uint32_t)rd(), u2 = (uint32_t)rd();
                    int32_t s = -7;
                    int r2 = m ? tlt_mab_select(m, B, u1, u2, &s) : -1;
                    printf("%d %d\n", r2, s);
                } else if (op[0] == 'r') {
                    int s = (int)rd();
                    double t = rdd();
                    int B = (int)rd();
                    std::vector<int32_t> lens(B);
                    for (auto& l : lens) l = (int)rd();
                    double a = 0, r = 0;
                    int r2 = m ? tlt_mab_record(m, s, t, lens.data(), B, &a, &r) : -1;
                    printf("%d %.17g %.17g\n", r2, a, r);
                } else {
                    int s = (int)rd();
                    double med = 0;
                    int32_t cnt = 0;
                    int r2 = m ? tlt_mab_median_reward(m, s, &med, &cnt) : -1;
                    printf("%d %.17g %d\n", r2, med, cnt);
                }
            }
            if (m) tlt_mab_destroy(m);
        } else if (c == "ngram") {
            int order = (int)rd(), nIns = (int)rd();
            tlt_ngram* db = nullptr;
            printf("%d\n", tlt_ngram_create(order, &db));
            for (int i = 0; i < nIns; ++i) {
                long long pid = rd();
                int len = (int)rd();
                std::vector<int32_t> t(len);
                for (auto& x : t) x = (int)rd();
                int rc = db ? tlt_ngram_insert(db, pid, t.data(), len) : -1;
                if (rc) printf("insert %d\n", rc);
            }
            int nProp = (int)rd();
            for (int i = 0; i < nProp; ++i) {
                long long pid = rd();
                int len = (int)rd();
                std::vector<int32_t> ctx(len);
                for (auto& x : ctx) x = (int)rd();
                int depth = (int)rd(), topk = (int)rd(), nn = (int)rd();
                std::vector<int32_t> tok(nn > 0 ? nn : 1), par(tok.size());
                std::vector<float> sc(tok.size());
                int rc = db ? tlt_ngram_propose(db, pid, ctx.data(), len, depth, topk, nn, tok.data(), par.data(), sc.data()) : -1;
                printf("%d", rc);
                for (int a = 0; a < (rc ? 0 : 2); ++a)
                    for (int j = 0; j < nn; ++j) printf(" %d", a == 0 ? tok[j] : par[j]);
                for (int j = 0; j < (rc ? 0 : nn); ++j) printf(" %.9g", (double)sc[j]);
                printf("\n");
            }
            if (db) tlt_ngram_destroy(db);
        } else if (c == "accept") {
            int mode = (int)rd(), B = (int)rd(), n = (int)rd(), V = (int)rd(), stride = (int)rd();
            float tau = (float)rdd();
            std::vector<int32_t> tok((size_t)B * n), par((size_t)B * n);
            std::vector<float> logits((size_t)B * n * V), q((size_t)B * n * V);
            std::vector<uint32_t> ua((size_t)B * n), uf(B);
            for (auto& x : tok) x = (int)rd();
            for (auto& x : par) x = (int)rd();
            for (auto& x : logits) x = (float)rdd();
            for (auto& x : q) x = (float)rdd();
            for (auto& x : ua) x = (uint32_t)rd();
            for (auto& x : uf) x = (uint32_t)rd();
            std::vector<int32_t> al(B), path((size_t)B * stride), out((size_t)B * stride), no(B), near(B, 0);
            if (mode == 0) oracle_accept_greedy(B, n, V, stride, tok.data(), par.data(), logits.data(), al.data(), path.data(), out.data(), no.data());
            else if (mode == 1) oracle_accept_sample_near(B, n, V, stride, tau, tok.data(), par.data(), logits.data(), q.data(), ua.data(), uf.data(), al.data(), path.data(), out.data(), no.data(), near.data());
            else oracle_accept_target_only_near(B, n, V, stride, tau, tok.data(), par.data(), logits.data(), ua.data(), uf.data(), al.data(), path.data(), out.data(), no.data(), near.data());
            for (int b = 0; b < B; ++b) {
                printf("%d %d %d", al[b], no[b], near[b]);
                for (int j = 0; j < stride; ++j) printf(" %d %d", path[(size_t)b * stride + j], out[(size_t)b * stride + j]);
                printf("\n");
            }
        } else {
            return 2;
        }
    }
    return 0;
}
