/*
 * Memory-safety exercise of the CPU oracle -- TEST INFRASTRUCTURE.
 *
 * Built together with metro_oracle.c under -fsanitize=address,undefined (tests/test_oracle_sanitize.py)
 * and run natively: every oracle entry point is called on seeded random instances whose buffers are
 * heap blocks of exactly the documented size, so a read or write one element past any of them aborts
 * the run.  Results are only checked for the invariants that need no second implementation
 * (eqs. (2)-(4) of Sec. 4.1: every pair on a replica of its expert; activated counts = popcounts;
 * the permutation lists every pair of the rank once); the numerical pins live in the Python tests.
 */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

int oracle_count(const int32_t* ids, int64_t n_pairs, int N, int32_t* cnt);
int oracle_route_metro(const int32_t* ids, int T, int k, const int32_t* slot_to_expert, int N, int G, int spr,
                       int32_t* pair_slot, int32_t* expert_slot, int32_t* rank_active, uint64_t* rank_bitmap,
                       int64_t* inspected);
int oracle_route_token_balanced(const int32_t* ids, int T, int k, const int32_t* slot_to_expert, int N, int G,
                                int spr, int32_t* pair_slot, int32_t* rank_active, uint64_t* rank_bitmap);
int oracle_bruteforce_opt(const int32_t* cnt, const int32_t* slot_to_expert, int N, int G, int spr,
                          int64_t max_assignments);
int oracle_matching_opt(const int32_t* cnt, const int32_t* slot_to_expert, int N, int G, int spr);
int oracle_permute(const int32_t* pair_slot, int T, int k, int rank, int spr, int32_t* group_offsets,
                   int32_t* perm_pair, int32_t* pair_row, int32_t* n_pairs);
int oracle_ffn(const void* x, int dtype, const int32_t* perm_pair, const int32_t* group_offsets, int k, int spr,
               int H, int I, const void* w13, const void* w2, const int32_t* rows, int n_rows, double* act_out,
               double* y_out);
int oracle_unpermute(const double* y_perm, const int32_t* pair_row, const float* topk_w, int T, int k, int H,
                     double* out);
int oracle_gate_topk(const void* x, const void* w_gate, int dtype, int T, int H, int N, int k, int32_t* ids,
                     double* w, double* logits_out, int32_t* cnt);

static uint64_t state = 0x9277;
static uint32_t rnd(void) {                      /* splitmix64 */
    uint64_t z = (state += 0x9e3779b97f4a7c15ull);
    z = (z ^ (z >> 30)) * 0xbf58476d1ce4e5b9ull;
    z = (z ^ (z >> 27)) * 0x94d049bb133111ebull;
    return (uint32_t)((z ^ (z >> 31)) >> 32);
}
static int below(int n) { return (int)(rnd() % (uint32_t)n); }
static float unit(void) { return (float)(rnd() >> 8) / 16777216.0f - 0.5f; }

#define REQUIRE(cond)                                                           \
    do {                                                                        \
        if (!(cond)) {                                                          \
            fprintf(stderr, "line %d: %s (case %d)\n", __LINE__, #cond, it);    \
            return 1;                                                           \
        }                                                                       \
    } while (0)

static void* block(size_t n, size_t elt) { return malloc(n * elt > 0 ? n * elt : 1); }

int main(void) {
    for (int it = 0; it < 300; ++it) {
        const int G = 1 + below(6), spr = 1 + below(7), S = G * spr;
        const int N = 1 + below(S), k = 1 + below(N < 4 ? N : 4), T = below(20);
        const int n = T * k;
        /* placement: every expert once, some extra replicas (never twice on a rank), some empty slots */
        int32_t* s2e = block(S, 4);
        for (int s = 0; s < S; ++s) s2e[s] = -1;
        for (int e = 0; e < N; ++e) {
            int s;
            do s = below(S); while (s2e[s] >= 0);
            s2e[s] = e;
        }
        for (int s = 0; s < S; ++s) {
            if (s2e[s] >= 0 || below(3) == 0) continue;
            const int e = below(N), g = s / spr;
            int here = 0;
            for (int q = g * spr; q < (g + 1) * spr; ++q) here |= s2e[q] == e;
            if (!here) s2e[s] = e;
        }
        /* top-k ids without repetition inside a token, a few padded pairs */
        int32_t* ids = block(n, 4);
        for (int t = 0; t < T; ++t)
            for (int j = 0; j < k; ++j) {
                int e, dup;
                do {
                    e = below(N);
                    dup = 0;
                    for (int q = 0; q < j; ++q) dup |= ids[t * k + q] == e;
                } while (dup);
                ids[t * k + j] = e;
            }
        for (int p = 0; p < n; ++p)
            if (below(10) == 0) ids[p] = -1;

        int32_t* cnt = block(N, 4);
        REQUIRE(oracle_count(ids, n, N, cnt) == 0);
        int32_t *ps_m = block(n, 4), *ps_t = block(n, 4), *es = block(N, 4), *ra_m = block(G, 4), *ra_t = block(G, 4);
        uint64_t *rb_m = block(G, 8), *rb_t = block(G, 8);
        int64_t inspected = -1;
        REQUIRE(oracle_route_metro(ids, T, k, s2e, N, G, spr, ps_m, es, ra_m, rb_m, &inspected) == 0);
        REQUIRE(oracle_route_token_balanced(ids, T, k, s2e, N, G, spr, ps_t, ra_t, rb_t) == 0);
        int lam_m = 0, lam_t = 0;
        for (int g = 0; g < G; ++g) {
            REQUIRE(ra_m[g] == __builtin_popcountll(rb_m[g]) && ra_t[g] == __builtin_popcountll(rb_t[g]));
            lam_m = ra_m[g] > lam_m ? ra_m[g] : lam_m;
            lam_t = ra_t[g] > lam_t ? ra_t[g] : lam_t;
        }
        for (int p = 0; p < n; ++p) {
            if (ids[p] < 0) {
                REQUIRE(ps_m[p] == -1 && ps_t[p] == -1);
                continue;
            }
            REQUIRE(ps_m[p] >= 0 && ps_m[p] < S && s2e[ps_m[p]] == ids[p] && ps_m[p] == es[ids[p]]);
            REQUIRE(ps_t[p] >= 0 && ps_t[p] < S && s2e[ps_t[p]] == ids[p]);
        }
        const int opt = oracle_matching_opt(cnt, s2e, N, G, spr);
        const int brute = oracle_bruteforce_opt(cnt, s2e, N, G, spr, 200000);
        REQUIRE(opt >= 0 && opt <= lam_m && opt <= lam_t);
        REQUIRE(brute == opt || brute == -4);

        /* one rank of the layer: permute, FFN (both storage types, all rows and sampled rows), combine */
        const int rank = below(G), H = 1 + below(24), I = 1 + below(12), dtype = below(2);
        int32_t *go = block(spr + 1, 4), *pp = block(n, 4), *pr = block(n, 4), np_ = -1;
        REQUIRE(oracle_permute(ps_m, T, k, rank, spr, go, pp, pr, &np_) == 0);
        REQUIRE(go[0] == 0 && go[spr] == np_ && np_ <= n);
        for (int r = 0; r < np_; ++r) REQUIRE(pp[r] >= 0 && pp[r] < n && pr[pp[r]] == r);
        const size_t eb = dtype ? 2 : 4;
        void *x = block((size_t)T * H, eb), *w13 = block((size_t)spr * 2 * I * H, eb), *w2 = block((size_t)spr * H * I, eb);
        for (size_t i = 0; i < (size_t)T * H; ++i)
            if (dtype) ((uint16_t*)x)[i] = (uint16_t)(0x3c00 + below(0x400) + (below(2) << 15));
            else ((float*)x)[i] = unit();
        for (size_t i = 0; i < (size_t)spr * 2 * I * H; ++i)
            if (dtype) ((uint16_t*)w13)[i] = (uint16_t)(0x3c00 + below(0x400) + (below(2) << 15));
            else ((float*)w13)[i] = unit();
        for (size_t i = 0; i < (size_t)spr * H * I; ++i)
            if (dtype) ((uint16_t*)w2)[i] = (uint16_t)(0x3c00 + below(0x400) + (below(2) << 15));
            else ((float*)w2)[i] = unit();
        double *y = block((size_t)np_ * H, 8), *act = block((size_t)np_ * I, 8);
        REQUIRE(oracle_ffn(x, dtype, pp, go, k, spr, H, I, w13, w2, NULL, np_, act, y) == 0);
        if (np_ > 0) {
            int32_t sample[2] = {0, np_ - 1};
            double* ys = block((size_t)2 * H, 8);
            REQUIRE(oracle_ffn(x, dtype, pp, go, k, spr, H, I, w13, w2, sample, 2, NULL, ys) == 0);
            REQUIRE(memcmp(ys, y, sizeof(double) * H) == 0);
            REQUIRE(memcmp(ys + H, y + (size_t)(np_ - 1) * H, sizeof(double) * H) == 0);
            free(ys);
        }
        float* tw = block(n, 4);
        for (int p = 0; p < n; ++p) tw[p] = unit() + 0.5f;
        double* out = block((size_t)T * H, 8);
        REQUIRE(oracle_unpermute(y, pr, tw, T, k, H, out) == 0);

        /* router gate + top-k on the same activations */
        void* wg = block((size_t)N * H, eb);
        for (size_t i = 0; i < (size_t)N * H; ++i)
            if (dtype) ((uint16_t*)wg)[i] = (uint16_t)(0x3c00 + below(0x400) + (below(2) << 15));
            else ((float*)wg)[i] = unit();
        int32_t *gid = block(n, 4), *gcnt = block(N, 4);
        double *gw = block(n, 8), *logits = block((size_t)T * N, 8);
        REQUIRE(oracle_gate_topk(x, wg, dtype, T, H, N, k, gid, gw, logits, gcnt) == 0);
        REQUIRE(oracle_gate_topk(x, wg, dtype, T, H, N, k, gid, gw, NULL, NULL) == 0);
        int total = 0;
        for (int e = 0; e < N; ++e) total += gcnt[e];
        REQUIRE(total == n);
        for (int p = 0; p < n; ++p) REQUIRE(gid[p] >= 0 && gid[p] < N);

        free(s2e); free(ids); free(cnt); free(ps_m); free(ps_t); free(es); free(ra_m); free(ra_t); free(rb_m);
        free(rb_t); free(go); free(pp); free(pr); free(x); free(w13); free(w2); free(y); free(act); free(tw);
        free(out); free(wg); free(gid); free(gcnt); free(gw); free(logits);
    }
    printf("sanitize_check: ok\n");
    return 0;
}
