/*
 * CPU oracle for the METRO hot path -- TEST INFRASTRUCTURE, NOT THE PRODUCT.
 *
 * Plain, slow, obviously-correct C written from the paper (arxiv 2512.09277).  It
 * shares no code with the HIP library and is used only by the tests, the smoke check
 * and the benchmark's CPU-baseline leg.  Floating point is carried in double.
 *
 * What is pinned and how (tests/test_oracle_*.py):
 *   - oracle_route_metro            Alg. 1 served in ascending expert id, ties to the
 *                                   lowest rank (the paper leaves both open, so the
 *                                   particular assignment is "parity unpinned" against
 *                                   the authors' nondeterministic kernel); its value
 *                                   lambda is pinned by brute force, by the matching
 *                                   solver, by closed forms and by eqs. (1)-(4).
 *   - oracle_route_token_balanced   pinned by eqs. (2)-(4), per-replica counts differing
 *                                   by at most one, and lambda >= optimum (Lemma 1).
 *   - oracle_bruteforce_opt / oracle_matching_opt   pinned against each other.
 *   - oracle_permute                pinned against a library stable sort.
 *   - oracle_ffn / oracle_unpermute pinned against library matmuls in float64 and
 *                                   hand-computable special cases.
 *   - oracle_gate_topk              router logits + top-k (the step before the routing solve,
 *                                   Sec. 4.3); pinned against a library matmul + argsort +
 *                                   softmax, one-hot closed forms, ties and brute force.  The
 *                                   paper does not define the gate itself: the reading is the
 *                                   common softmax-over-the-selected-logits router.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORACLE_OK 0
#define ORACLE_BAD_ID (-1)          /* an id outside [-1, N) */
#define ORACLE_NO_REPLICA (-2)      /* an expert with tokens has no replica */
#define ORACLE_BAD_ARG (-3)
#define ORACLE_TOO_LARGE (-4)

#ifdef _OPENMP
#include <omp.h>
int oracle_num_threads(void) { return omp_get_max_threads(); }
#else
int oracle_num_threads(void) { return 1; }
#endif

/* Sec. 4.1: T[i] = number of (token, expert) pairs of the batch that selected expert i.
 * Id -1 marks a padded pair (Sec. 5 pads batches) and is not counted. */
int oracle_count(const int32_t* ids, int64_t n_pairs, int N, int32_t* cnt) {
    for (int i = 0; i < N; ++i) cnt[i] = 0;
    for (int64_t p = 0; p < n_pairs; ++p) {
        if (ids[p] < -1 || ids[p] >= N) return ORACLE_BAD_ID;
        if (ids[p] >= 0) cnt[ids[p]]++;
    }
    return ORACLE_OK;
}

/* Placement matrix A of Sec. 4.1, carried as slotA[i*G+g] = lowest slot of expert i on
 * rank g, or -1 where A[i][g] = 0.  Slot s lives on rank s / spr.  A is binary, so a
 * second copy of an expert on the same rank collapses onto the lowest slot. */
static int build_A(const int32_t* slot_to_expert, int N, int G, int spr, int32_t* slotA) {
    for (int i = 0; i < N * G; ++i) slotA[i] = -1;
    for (int s = 0; s < G * spr; ++s) {
        int e = slot_to_expert[s];
        if (e < -1 || e >= N) return ORACLE_BAD_ID;
        if (e < 0) continue;
        int g = s / spr;
        if (slotA[e * G + g] < 0) slotA[e * G + g] = s;
    }
    return ORACLE_OK;
}

/* Fill the per-rank outputs from pair_slot: bit l of rank_bitmap[g] is set iff slot
 * g*spr+l receives at least one pair; rank_active[g] counts those slots
 * (the sum over i of y[i][g] in the expression for lambda, Sec. 4.3). */
static void fill_rank_outputs(const int32_t* pair_slot, int64_t n_pairs, int G, int spr,
                              int32_t* rank_active, uint64_t* rank_bitmap) {
    for (int g = 0; g < G; ++g) { rank_bitmap[g] = 0; rank_active[g] = 0; }
    for (int64_t p = 0; p < n_pairs; ++p) {
        int s = pair_slot[p];
        if (s < 0) continue;
        rank_bitmap[s / spr] |= (uint64_t)1 << (s % spr);
    }
    for (int g = 0; g < G; ++g)
        for (int l = 0; l < spr; ++l)
            if (rank_bitmap[g] >> l & 1) rank_active[g]++;
}

/* Alg. 1 (METRO greedy), executed serially: experts in ascending id (a legal execution,
 * since the two-phase-locked parallel loop is serialisable), each active expert taking
 * the hosting rank with the smallest activated count L[g]; equal counts go to the lowest
 * rank.  expert_slot[i] = chosen slot or -1 when T[i] = 0.  pair_slot follows x from y
 * (Sec. 4.3): all pairs of expert i go to its one activated replica.
 * *inspected = number of (expert, hosting rank) entries of A looked at (the O(|A|) claim). */
int oracle_route_metro(const int32_t* ids, int T, int k, const int32_t* slot_to_expert,
                       int N, int G, int spr, int32_t* pair_slot, int32_t* expert_slot,
                       int32_t* rank_active, uint64_t* rank_bitmap, int64_t* inspected) {
    if (T < 0 || k < 1 || N < 1 || G < 1 || spr < 1 || spr > 64) return ORACLE_BAD_ARG;
    int64_t n_pairs = (int64_t)T * k;
    int32_t* cnt = (int32_t*)malloc(sizeof(int32_t) * N);
    int32_t* slotA = (int32_t*)malloc(sizeof(int32_t) * N * G);
    int32_t* L = (int32_t*)calloc(G, sizeof(int32_t));
    int rc = oracle_count(ids, n_pairs, N, cnt);
    if (rc == ORACLE_OK) rc = build_A(slot_to_expert, N, G, spr, slotA);
    int64_t looked = 0;
    for (int i = 0; rc == ORACLE_OK && i < N; ++i) {
        expert_slot[i] = -1;
        if (cnt[i] == 0) continue;                       /* "if T[i] > 0" */
        int best = -1;
        for (int g = 0; g < G; ++g) {                    /* G_i = { g | A[i][g] = 1 } */
            if (slotA[i * G + g] < 0) continue;
            looked++;
            if (best < 0 || L[g] < L[best]) best = g;   /* smallest L[g], lowest g on ties */
        }
        if (best < 0) { rc = ORACLE_NO_REPLICA; break; }
        expert_slot[i] = slotA[i * G + best];            /* y[i][g*] = 1 */
        L[best]++;                                       /* L[g*] += 1 */
    }
    if (rc == ORACLE_OK) {
        for (int64_t p = 0; p < n_pairs; ++p) pair_slot[p] = ids[p] < 0 ? -1 : expert_slot[ids[p]];
        fill_rank_outputs(pair_slot, n_pairs, G, spr, rank_active, rank_bitmap);
        if (inspected) *inspected = looked;
    }
    free(cnt); free(slotA); free(L);
    return rc;
}

/* Token-balanced (EPLB-style) routing, Sec. 2.3 / Sec. 6.1 "Compared baselines": each
 * expert's pairs are spread evenly over its replicas.  Reading: the q-th pair of expert i
 * in flattened (token-major) order goes to replica q mod r_i, replicas in ascending slot
 * id, so per-replica counts differ by at most one. */
int oracle_route_token_balanced(const int32_t* ids, int T, int k, const int32_t* slot_to_expert,
                                int N, int G, int spr, int32_t* pair_slot,
                                int32_t* rank_active, uint64_t* rank_bitmap) {
    if (T < 0 || k < 1 || N < 1 || G < 1 || spr < 1 || spr > 64) return ORACLE_BAD_ARG;
    int64_t n_pairs = (int64_t)T * k;
    int32_t* seen = (int32_t*)calloc(N, sizeof(int32_t));
    int32_t* slotA = (int32_t*)malloc(sizeof(int32_t) * N * G);
    int rc = build_A(slot_to_expert, N, G, spr, slotA);
    for (int64_t p = 0; rc == ORACLE_OK && p < n_pairs; ++p) {
        int e = ids[p];
        if (e < -1 || e >= N) { rc = ORACLE_BAD_ID; break; }
        if (e < 0) { pair_slot[p] = -1; continue; }
        int r = 0;
        for (int g = 0; g < G; ++g) r += slotA[e * G + g] >= 0;
        if (r == 0) { rc = ORACLE_NO_REPLICA; break; }
        int want = seen[e] % r, at = 0, slot = -1;
        for (int g = 0; g < G; ++g) {                    /* ascending rank == ascending slot id */
            if (slotA[e * G + g] < 0) continue;
            if (at == want) { slot = slotA[e * G + g]; break; }
            at++;
        }
        pair_slot[p] = slot;
        seen[e]++;
    }
    if (rc == ORACLE_OK) fill_rank_outputs(pair_slot, n_pairs, G, spr, rank_active, rank_bitmap);
    free(seen); free(slotA);
    return rc;
}

/* ---- optimum of min-exp-routing (Sec. 4.1 after Lemma 1): one replica per active expert,
 * minimise the maximum number of activated experts on a rank. ---- */

static void brute_rec(const int32_t* act, int n_act, int at, const int32_t* slotA, int G,
                      int32_t* L, int* best) {
    if (at == n_act) {
        int mx = 0;
        for (int g = 0; g < G; ++g) if (L[g] > mx) mx = L[g];
        if (mx < *best) *best = mx;
        return;
    }
    int e = act[at];
    for (int g = 0; g < G; ++g) {
        if (slotA[e * G + g] < 0) continue;
        L[g]++;
        brute_rec(act, n_act, at + 1, slotA, G, L, best);
        L[g]--;
    }
}

/* Exhaustive enumeration of every assignment (no pruning).  Returns lambda*, or
 * ORACLE_TOO_LARGE when the number of assignments exceeds max_assignments. */
int oracle_bruteforce_opt(const int32_t* cnt, const int32_t* slot_to_expert, int N, int G, int spr,
                          int64_t max_assignments) {
    int32_t* slotA = (int32_t*)malloc(sizeof(int32_t) * N * G);
    int32_t* act = (int32_t*)malloc(sizeof(int32_t) * N);
    int32_t* L = (int32_t*)calloc(G, sizeof(int32_t));
    int rc = build_A(slot_to_expert, N, G, spr, slotA), n_act = 0;
    double total = 1.0;
    for (int e = 0; rc == ORACLE_OK && e < N; ++e) {
        if (cnt[e] <= 0) continue;
        int r = 0;
        for (int g = 0; g < G; ++g) r += slotA[e * G + g] >= 0;
        if (r == 0) { rc = ORACLE_NO_REPLICA; break; }
        total *= r;
        act[n_act++] = e;
    }
    if (rc == ORACLE_OK && total > (double)max_assignments) rc = ORACLE_TOO_LARGE;
    if (rc == ORACLE_OK) {
        int best = n_act + 1;
        brute_rec(act, n_act, 0, slotA, G, L, &best);
        rc = n_act == 0 ? 0 : best;
    }
    free(slotA); free(act); free(L);
    return rc;
}

/* Feasibility of a candidate lambda0 (Sec. 4.2): bipartite matching of active experts to
 * ranks where a rank may be matched at most lambda0 times; augmenting paths (Kuhn). */
static int try_augment(int e, const int32_t* slotA, int G, int cap, int32_t* load,
                       int32_t* held /*[G*cap]*/, uint8_t* visited) {
    for (int g = 0; g < G; ++g) {
        if (slotA[e * G + g] < 0 || visited[g]) continue;
        visited[g] = 1;
        if (load[g] < cap) { held[g * cap + load[g]++] = e; return 1; }
        for (int j = 0; j < cap; ++j) {
            int other = held[g * cap + j];
            if (try_augment(other, slotA, G, cap, load, held, visited)) { held[g * cap + j] = e; return 1; }
        }
    }
    return 0;
}

/* Optimal algorithm of Sec. 4.2: binary search on lambda over [1, max slots on a rank],
 * each candidate tested by the capacitated matching above.  Returns lambda*. */
int oracle_matching_opt(const int32_t* cnt, const int32_t* slot_to_expert, int N, int G, int spr) {
    int32_t* slotA = (int32_t*)malloc(sizeof(int32_t) * N * G);
    int rc = build_A(slot_to_expert, N, G, spr, slotA), n_act = 0;
    for (int e = 0; rc == ORACLE_OK && e < N; ++e) {
        if (cnt[e] <= 0) continue;
        int r = 0;
        for (int g = 0; g < G; ++g) r += slotA[e * G + g] >= 0;
        if (r == 0) rc = ORACLE_NO_REPLICA;
        n_act++;
    }
    if (rc == ORACLE_OK && n_act == 0) { free(slotA); return 0; }
    int lo = 1, hi = spr;                                /* lambda never exceeds a rank's slot count */
    while (rc == ORACLE_OK && lo < hi) {
        int mid = (lo + hi) / 2, ok = 1;
        int32_t* load = (int32_t*)calloc(G, sizeof(int32_t));
        int32_t* held = (int32_t*)malloc(sizeof(int32_t) * G * mid);
        uint8_t* visited = (uint8_t*)malloc(G);
        for (int e = 0; ok && e < N; ++e) {
            if (cnt[e] <= 0) continue;
            memset(visited, 0, G);
            ok = try_augment(e, slotA, G, mid, load, held, visited);
        }
        free(load); free(held); free(visited);
        if (ok) hi = mid; else lo = mid + 1;
    }
    free(slotA);
    return rc == ORACLE_OK ? lo : rc;
}

/* Per-replica token lists of one rank: pairs whose slot is on `rank`, ordered by local
 * slot l = slot - rank*spr, and by flattened pair index p = t*k + j within a slot.
 * group_offsets[l]..group_offsets[l+1] delimit slot l's rows; pair_row[p] = row of pair p
 * in that list, or -1 when the pair is routed elsewhere. */
int oracle_permute(const int32_t* pair_slot, int T, int k, int rank, int spr,
                   int32_t* group_offsets, int32_t* perm_pair, int32_t* pair_row, int32_t* n_pairs) {
    int64_t n = (int64_t)T * k;
    int rows = 0;
    for (int64_t p = 0; p < n; ++p) pair_row[p] = -1;
    for (int l = 0; l < spr; ++l) {
        group_offsets[l] = rows;
        for (int64_t p = 0; p < n; ++p)
            if (pair_slot[p] == rank * spr + l) { perm_pair[rows] = (int32_t)p; pair_row[p] = rows; rows++; }
    }
    group_offsets[spr] = rows;
    *n_pairs = rows;
    return ORACLE_OK;
}

/* dtype: 0 = float32, 1 = bfloat16 bit patterns (widened exactly). */
static inline double load_elem(const void* base, int dtype, int64_t idx) {
    if (dtype == 0) return (double)((const float*)base)[idx];
    uint32_t bits = (uint32_t)((const uint16_t*)base)[idx] << 16;
    float f;
    memcpy(&f, &bits, sizeof f);
    return (double)f;
}

/* SwiGLU expert FFN on the rows of one rank's token lists.  For row r of slot l, with
 * token t = perm_pair[r] / k:
 *     gate_i = sum_h x[t][h] * w13[l][i][h]          up_i = sum_h x[t][h] * w13[l][I+i][h]
 *     act_i  = gate_i / (1 + exp(-gate_i)) * up_i     (SiLU(gate) * up)
 *     y[r][c] = sum_i act_i * w2[l][c][i]
 * x[T,H]; w13[spr,2I,H]; w2[spr,H,I]; everything in double, nothing rounded in between.
 * rows == NULL computes all n_rows = group_offsets[spr] rows, else only the listed rows;
 * y_out[n_rows,H]; act_out[n_rows,I] may be NULL. */
int oracle_ffn(const void* x, int dtype, const int32_t* perm_pair, const int32_t* group_offsets,
               int k, int spr, int H, int I, const void* w13, const void* w2,
               const int32_t* rows, int n_rows, double* act_out, double* y_out) {
    int status = ORACLE_OK;
#pragma omp parallel for schedule(dynamic, 1)
    for (int q = 0; q < n_rows; ++q) {
        int r = rows ? rows[q] : q;
        int l = -1;
        for (int s = 0; s < spr; ++s)
            if (group_offsets[s] <= r && r < group_offsets[s + 1]) l = s;
        if (l < 0) { status = ORACLE_BAD_ARG; continue; }
        int64_t t = perm_pair[r] / k;
        double* act = (double*)malloc(sizeof(double) * I);
        for (int i = 0; i < I; ++i) {
            double gate = 0.0, up = 0.0;
            for (int h = 0; h < H; ++h) {
                double xv = load_elem(x, dtype, t * H + h);
                gate += xv * load_elem(w13, dtype, ((int64_t)l * 2 * I + i) * H + h);
                up += xv * load_elem(w13, dtype, ((int64_t)l * 2 * I + I + i) * H + h);
            }
            act[i] = gate / (1.0 + exp(-gate)) * up;
            if (act_out) act_out[(int64_t)q * I + i] = act[i];
        }
        for (int c = 0; c < H; ++c) {
            double acc = 0.0;
            for (int i = 0; i < I; ++i) acc += act[i] * load_elem(w2, dtype, ((int64_t)l * H + c) * I + i);
            y_out[(int64_t)q * H + c] = acc;
        }
        free(act);
    }
    return status;
}

/* Combine on one rank: out[t][c] = sum over j (ascending) of topk_w[t][j] * y[pair_row[t*k+j]][c]
 * for the pairs this rank served; tokens with no pair here get zeros. */
int oracle_unpermute(const double* y_perm, const int32_t* pair_row, const float* topk_w,
                     int T, int k, int H, double* out) {
    for (int t = 0; t < T; ++t) {
        for (int c = 0; c < H; ++c) out[(int64_t)t * H + c] = 0.0;
        for (int j = 0; j < k; ++j) {
            int r = pair_row[(int64_t)t * k + j];
            if (r < 0) continue;
            for (int c = 0; c < H; ++c)
                out[(int64_t)t * H + c] += (double)topk_w[(int64_t)t * k + j] * y_perm[(int64_t)r * H + c];
        }
    }
    return ORACLE_OK;
}

/* Router gate + top-k on the full (gathered) token set, Sec. 4.3: the step that produces the
 * global top-k ids the routing solve consumes.  The paper leaves the gate to the model; reading:
 *     logit[t][e] = sum_h x[t][h] * w_gate[e][h]
 *     ids[t][0..k) = the k experts with the largest logits, in descending logit order, equal
 *                    logits in ascending expert id
 *     w[t][j]      = exp(logit[t][ids[t][j]]) / sum_j' exp(logit[t][ids[t][j']])
 * (softmax over all experts, top-k, renormalise -- the same numbers).  Everything in double.
 * logits_out[T,N] and cnt[N] (T[i] of Sec. 4.1) may be NULL. */
int oracle_gate_topk(const void* x, const void* w_gate, int dtype, int T, int H, int N, int k,
                     int32_t* ids, double* w, double* logits_out, int32_t* cnt) {
    if (T < 0 || H < 1 || N < 1 || k < 1 || k > N) return ORACLE_BAD_ARG;
#pragma omp parallel for schedule(dynamic, 1)
    for (int t = 0; t < T; ++t) {
        double* logit = (double*)malloc(sizeof(double) * N);
        char* taken = (char*)malloc(N);
        for (int e = 0; e < N; ++e) {
            double acc = 0.0;
            for (int h = 0; h < H; ++h)
                acc += load_elem(x, dtype, (int64_t)t * H + h) * load_elem(w_gate, dtype, (int64_t)e * H + h);
            logit[e] = acc;
            taken[e] = 0;
            if (logits_out) logits_out[(int64_t)t * N + e] = acc;
        }
        for (int j = 0; j < k; ++j) {              /* selection: largest remaining, lowest id first */
            int best = -1;
            for (int e = 0; e < N; ++e)
                if (!taken[e] && (best < 0 || logit[e] > logit[best])) best = e;
            taken[best] = 1;
            ids[(int64_t)t * k + j] = best;
        }
        double top = logit[ids[(int64_t)t * k]], sum = 0.0;
        for (int j = 0; j < k; ++j) sum += exp(logit[ids[(int64_t)t * k + j]] - top);
        for (int j = 0; j < k; ++j) w[(int64_t)t * k + j] = exp(logit[ids[(int64_t)t * k + j]] - top) / sum;
        free(logit);
        free(taken);
    }
    if (cnt) {                                     /* T[i]: pairs that selected expert i */
        for (int e = 0; e < N; ++e) cnt[e] = 0;
        for (int64_t p = 0; p < (int64_t)T * k; ++p) cnt[ids[p]] += 1;
    }
    return ORACLE_OK;
}
