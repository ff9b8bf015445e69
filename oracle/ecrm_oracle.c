/*
 * ECRM sparse-update ORACLE -- test infrastructure, not product code.
 *
 * A plain, slow CPU statement of what the erasure-coded parameter-server update computes, written
 * from the paper (ECRM, arXiv 2104.01981) and from nothing else.  Only the tests, the smoke check
 * and the benchmark's CPU-baseline leg may call it; the GPU library neither links nor imports it,
 * and it shares no code with that library.
 *
 * Conventions (the paper's notation where it has one):
 *   k   data entries per parity entry, r = 1            (Sec. 3.2, "Encoder and decoder")
 *   S   number of servers, S >= k+1                      (Sec. 3.2, "Where should parities be placed?")
 *   R   number of embedding entries (rows), R % k == 0;  D floats per entry
 *   E[R][D]  entries, A[R][D] Adagrad accumulators       (Sec. 3.3.1, unnumbered Adagrad equation)
 *   PE[R/k][D], PA[R/k][D]  parity entries / parity accumulators (Sec. 3.2, Sec. 3.3.1)
 *   stripe g = rows k*g .. k*g+k-1; member j = row - k*g
 *
 * Readings taken where the paper is silent (all restated in the repository's design notes):
 *   - a key is already a dense row id; stripe g's parity lives on server g mod S and member j on
 *     server (g+1+j) mod S -- the RAID-5 rotation of Sec. 3.2 / Fig. 3, which for S = k+1 puts the
 *     k members on "the k other servers";
 *   - several updates to one entry inside a call are applied one after the other in arrival order
 *     (the system is asynchronous and per-update, Sec. 2.1, Sec. 3.3.2);
 *   - storage is fp32; inside one call the arithmetic is carried in fp64 and each table element
 *     is rounded to fp32 once, when the call ends;
 *   - epsilon sits inside the square root, and the accumulator used for update t already contains
 *     gradient t (Sec. 3.3.1: G_t = g_0^2 + ... + g_t^2).
 *
 * Pins (tests/test_oracle_pins.py): hand-computed Adagrad chains from the printed equation, the
 * eps = 0 case against torch.optim.Adagrad, the closed prefix-sum form for a run on one entry,
 * the k = 3 encode/decode example of Sec. 1 / Sec. 2.4 on dyadic values (exact), the parity
 * invariant p = sum of its k entries after every call, the load identity of Sec. 3.6 (each entry
 * update causes exactly one parity update), brute-force enumeration of the placement, and an
 * independent per-item NumPy transcription (oracle/brute.py).
 * Parity unpinned: the numeric values of lr and eps, and the id -> row hashing, which the paper
 * does not give.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* ---- placement (Sec. 3.2, rotating parity placement) --------------------------------------- */

static inline uint64_t stripe_of(uint64_t x, uint32_t k) { return x / k; }
static inline uint32_t member_of(uint64_t x, uint32_t k) { return (uint32_t)(x % k); }
static inline uint32_t parity_server_of(uint64_t g, uint32_t S) { return (uint32_t)(g % S); }
static inline uint32_t data_server_of(uint64_t g, uint32_t j, uint32_t S) { return (uint32_t)((g + 1 + j) % S); }

int ecrm_oracle_route(const uint64_t *keys, uint64_t n, uint64_t R, uint32_t k, uint32_t S,
                      uint64_t *stripe, uint32_t *member, uint32_t *data_srv, uint32_t *parity_srv)
{
    for (uint64_t i = 0; i < n; ++i) {
        uint64_t x = keys[i];
        if (x >= R) return -1;
        uint64_t g = stripe_of(x, k);
        uint32_t j = member_of(x, k);
        stripe[i] = g;
        member[i] = j;
        data_srv[i] = data_server_of(g, j, S);
        parity_srv[i] = parity_server_of(g, S);
    }
    return 0;
}

/* ---- load accounting (Sec. 3.6: every entry update is also applied to one parity; Sec. 4.3
 *      "Effect on load imbalance": count the updates that occur on each server) -------------- */

int ecrm_oracle_load(const uint64_t *keys, uint64_t n, uint64_t R, uint32_t k, uint32_t S,
                     uint64_t *load_data, uint64_t *load_parity)
{
    for (uint64_t i = 0; i < n; ++i)
        if (keys[i] >= R) return -1;
    for (uint64_t i = 0; i < n; ++i) {
        uint64_t g = stripe_of(keys[i], k);
        uint32_t j = member_of(keys[i], k);
        load_data[data_server_of(g, j, S)] += 1;
        load_parity[parity_server_of(g, S)] += 1;
    }
    return 0;
}

/* ---- sum encoder / subtraction decoder, r = 1 (Sec. 3.2 "Encoder and decoder") ------------- */

void ecrm_oracle_encode(const float *T, uint64_t R, uint32_t D, uint32_t k, float *P)
{
    for (uint64_t g = 0; g < R / k; ++g)
        for (uint32_t d = 0; d < D; ++d) {
            double p = 0.0;
            for (uint32_t j = 0; j < k; ++j) p += (double)T[(g * k + j) * D + d];
            P[g * D + d] = (float)p;
        }
}

/* e_j = p - sum_{i != j} e_i for every stripe's member `lost`; out[R/k][D] */
void ecrm_oracle_decode_member(const float *T, const float *P, uint64_t R, uint32_t D, uint32_t k,
                               uint32_t lost, float *out)
{
    for (uint64_t g = 0; g < R / k; ++g)
        for (uint32_t d = 0; d < D; ++d) {
            double e = (double)P[g * D + d];
            for (uint32_t j = 0; j < k; ++j)
                if (j != lost) e -= (double)T[(g * k + j) * D + d];
            out[g * D + d] = (float)e;
        }
}

/* ---- loss of one server (Sec. 3.4): every unit it held is rebuilt from the k other units of its
 *      stripe -- a lost entry by the subtraction decoder, a lost parity by re-encoding.  The k+1
 *      units of a stripe are on k+1 different servers, so a stripe loses at most one unit. ------- */

static void rebuild_unit(float *T, float *P, uint64_t g, uint32_t D, uint32_t k, uint32_t lost /* k = parity */)
{
    for (uint32_t d = 0; d < D; ++d) {
        if (lost == k) {
            double p = 0.0;
            for (uint32_t j = 0; j < k; ++j) p += (double)T[(g * k + j) * D + d];
            P[g * D + d] = (float)p;
        } else {
            double e = (double)P[g * D + d];
            for (uint32_t j = 0; j < k; ++j)
                if (j != lost) e -= (double)T[(g * k + j) * D + d];
            T[(g * k + lost) * D + d] = (float)e;
        }
    }
}

/* which unit of stripe g lives on `server`: -1 none, k the parity, j < k member j */
static int unit_held(uint64_t g, uint32_t k, uint32_t S, uint32_t server)
{
    if (parity_server_of(g, S) == server) return (int)k;
    for (uint32_t j = 0; j < k; ++j)
        if (data_server_of(g, j, S) == server) return (int)j;
    return -1;
}

/* stripes [g_lo, g_hi) only: the unit of work of a recovery that proceeds chunk by chunk (Sec. 3.4) */
int ecrm_oracle_recover_range(float *E, float *A, float *PE, float *PA, uint64_t R, uint32_t D, uint32_t k,
                              uint32_t S, uint32_t server, uint64_t g_lo, uint64_t g_hi)
{
    if (server >= S || g_hi > R / k) return -1;
    for (uint64_t g = g_lo; g < g_hi; ++g) {
        const int u = unit_held(g, k, S, server);
        if (u < 0) continue;
        rebuild_unit(E, PE, g, D, k, (uint32_t)u);
        rebuild_unit(A, PA, g, D, k, (uint32_t)u);
    }
    return 0;
}

int ecrm_oracle_recover_server(float *E, float *A, float *PE, float *PA, uint64_t R, uint32_t D, uint32_t k,
                               uint32_t S, uint32_t server)
{
    if (server >= S) return -1;
    for (uint64_t g = 0; g < R / k; ++g) {
        const int u = unit_held(g, k, S, server);
        if (u < 0) continue;
        rebuild_unit(E, PE, g, D, k, (uint32_t)u);
        rebuild_unit(A, PA, g, D, k, (uint32_t)u);
    }
    return 0;
}

/* marks with NaN what the server held (the test's way of losing a server) */
int ecrm_oracle_fail_server(float *E, float *A, float *PE, float *PA, uint64_t R, uint32_t D, uint32_t k,
                            uint32_t S, uint32_t server)
{
    if (server >= S) return -1;
    for (uint64_t g = 0; g < R / k; ++g) {
        const int u = unit_held(g, k, S, server);
        if (u < 0) continue;
        float *e = u == (int)k ? PE + g * D : E + (g * k + u) * D;
        float *a = u == (int)k ? PA + g * D : A + (g * k + u) * D;
        for (uint32_t d = 0; d < D; ++d) { e[d] = NAN; a[d] = NAN; }
    }
    return 0;
}

/* Degraded read (Sec. 3.4): entries of the keys while `lost` is down (lost >= S: nobody is down) */
int ecrm_oracle_degraded_read(const float *E, const float *A, const float *PE, const float *PA, uint64_t R,
                              uint32_t D, uint32_t k, uint32_t S, const uint64_t *keys, uint64_t n, uint32_t lost,
                              float *out_E, float *out_A)
{
    for (uint64_t i = 0; i < n; ++i) {
        const uint64_t x = keys[i];
        if (x >= R) return -1;
        const uint64_t g = stripe_of(x, k);
        const uint32_t j = member_of(x, k);
        const int down = lost < S && data_server_of(g, j, S) == lost;
        for (uint32_t d = 0; d < D; ++d) {
            if (!down) {
                out_E[i * D + d] = E[x * D + d];
                out_A[i * D + d] = A[x * D + d];
            } else {
                double e = (double)PE[g * D + d], a = (double)PA[g * D + d];
                for (uint32_t m = 0; m < k; ++m)
                    if (m != j) { e -= (double)E[(g * k + m) * D + d]; a -= (double)A[(g * k + m) * D + d]; }
                out_E[i * D + d] = (float)e;
                out_A[i * D + d] = (float)a;
            }
        }
    }
    return 0;
}

/* ---- the update path: Adagrad on the entry (Sec. 3.3.1), then the differences in entry and
 *      optimizer state are added to the parity entry and parity accumulator (Sec. 3.3.2) ----- */

static double *widen(const float *src, uint64_t count)
{
    double *dst = (double *)malloc(count * sizeof(double));
    if (dst) for (uint64_t i = 0; i < count; ++i) dst[i] = (double)src[i];
    return dst;
}

static void narrow(float *dst, const double *src, uint64_t count)
{
    for (uint64_t i = 0; i < count; ++i) dst[i] = (float)src[i]; /* round to nearest even */
}

/*
 * Applies the n updates (keys[i], grads[i][0..D)) in arrival order.  `threads` > 1 splits the
 * STRIPES over threads (thread t owns stripes with g % threads == t and walks all items in
 * arrival order, skipping those it does not own): stripes never interact, so every element sees
 * exactly the same sequence of operations as with one thread.
 * Returns 0, -1 on a key >= R (nothing is modified), -2 on allocation failure.
 */
int ecrm_oracle_update(float *E, float *A, float *PE, float *PA,
                       uint64_t R, uint32_t D, uint32_t k, uint32_t S, float lr_f, float eps_f,
                       const uint64_t *keys, const float *grads, uint64_t n,
                       uint64_t *load_data, uint64_t *load_parity, int threads)
{
    if (k == 0 || R % k != 0 || S < k + 1) return -3;
    for (uint64_t i = 0; i < n; ++i)
        if (keys[i] >= R) return -1;

    const double lr = (double)lr_f, eps = (double)eps_f;
    const uint64_t Gn = R / k;
    double *E64 = widen(E, R * D), *A64 = widen(A, R * D);
    double *PE64 = widen(PE, Gn * D), *PA64 = widen(PA, Gn * D);
    if (!E64 || !A64 || !PE64 || !PA64) { free(E64); free(A64); free(PE64); free(PA64); return -2; }
    if (threads < 1) threads = 1;

#pragma omp parallel num_threads(threads)
    {
#ifdef _OPENMP
        const uint64_t t = (uint64_t)omp_get_thread_num(), T = (uint64_t)omp_get_num_threads();
#else
        const uint64_t t = 0, T = 1;
#endif
        for (uint64_t i = 0; i < n; ++i) {
            const uint64_t x = keys[i];
            const uint64_t g = stripe_of(x, k);
            if (g % T != t) continue;
            double *e = E64 + x * D, *a = A64 + x * D;
            double *pe = PE64 + g * D, *pa = PA64 + g * D;
            const float *gr = grads + i * D;
            for (uint32_t d = 0; d < D; ++d) {
                const double gd = (double)gr[d];
                const double a_old = a[d], e_old = e[d];
                a[d] = a_old + gd * gd;                       /* G_t includes gradient t */
                e[d] = e_old - lr / sqrt(a[d] + eps) * gd;    /* the printed Adagrad step */
                pe[d] += e[d] - e_old;                        /* difference in entry      */
                pa[d] += a[d] - a_old;                        /* difference in state      */
            }
        }
    }

    narrow(E, E64, R * D);   narrow(A, A64, R * D);
    narrow(PE, PE64, Gn * D); narrow(PA, PA64, Gn * D);
    free(E64); free(A64); free(PE64); free(PA64);

    if (load_data && load_parity)
        ecrm_oracle_load(keys, n, R, k, S, load_data, load_parity);
    return 0;
}

/*
 * The strawman of Sec. 3.3.1 ("gradient propagation"): the gradient itself is sent to the parity
 * server, which applies Adagrad to the parity entry with the PARITY accumulator.  Kept only so a
 * test can show that the parity invariant check fails for it, as the paper argues it must.
 */
int ecrm_oracle_update_gradient_propagation(float *E, float *A, float *PE, float *PA,
                                            uint64_t R, uint32_t D, uint32_t k, float lr_f, float eps_f,
                                            const uint64_t *keys, const float *grads, uint64_t n)
{
    const double lr = (double)lr_f, eps = (double)eps_f;
    const uint64_t Gn = R / k;
    for (uint64_t i = 0; i < n; ++i)
        if (keys[i] >= R) return -1;
    double *E64 = widen(E, R * D), *A64 = widen(A, R * D);
    double *PE64 = widen(PE, Gn * D), *PA64 = widen(PA, Gn * D);
    if (!E64 || !A64 || !PE64 || !PA64) { free(E64); free(A64); free(PE64); free(PA64); return -2; }
    for (uint64_t i = 0; i < n; ++i) {
        const uint64_t x = keys[i], g = stripe_of(x, k);
        for (uint32_t d = 0; d < D; ++d) {
            const double gd = (double)grads[i * D + d];
            A64[x * D + d] += gd * gd;
            E64[x * D + d] -= lr / sqrt(A64[x * D + d] + eps) * gd;
            PA64[g * D + d] += gd * gd;
            PE64[g * D + d] -= lr / sqrt(PA64[g * D + d] + eps) * gd;
        }
    }
    narrow(E, E64, R * D);   narrow(A, A64, R * D);
    narrow(PE, PE64, Gn * D); narrow(PA, PA64, Gn * D);
    free(E64); free(A64); free(PE64); free(PA64);
    return 0;
}

/*
 * The other update rules.  optimizer 0 = Adagrad (Sec. 3.3.1); optimizer 1 = SGD with momentum, the
 * optimizer of the paper's evaluation (Sec. 4.1), for which the paper prints no formula: taken as
 *     v <- mu * v + g ;  e <- e - lr * v          (A holds v, one state float per parameter).
 * combine 0 = every update applied on its own, in arrival order (asynchronous training);
 * combine 1 = the synchronous variant of Sec. 4.4: the gradients an entry receives in the call are
 *             added up (in arrival order) and ONE update is applied per modified entry; the load
 *             counters then count one entry update and one parity update per modified entry.
 * In every case the differences in entry and state are added to the stripe's parity rows
 * (Sec. 3.3.2).  Single-threaded on purpose.  Parity unpinned by the paper: the momentum formula.
 */
static void rule_step(double *e, double *a, double g, uint32_t optimizer, double lr, double eps, double mu)
{
    if (optimizer == 0) {
        *a = *a + g * g;
        *e = *e - lr / sqrt(*a + eps) * g;
    } else {
        *a = mu * *a + g;
        *e = *e - lr * *a;
    }
}

int ecrm_oracle_update_rule(float *E, float *A, float *PE, float *PA,
                            uint64_t R, uint32_t D, uint32_t k, uint32_t S, float lr_f, float eps_f, float mu_f,
                            uint32_t optimizer, uint32_t combine,
                            const uint64_t *keys, const float *grads, uint64_t n,
                            uint64_t *load_data, uint64_t *load_parity)
{
    if (k == 0 || R % k != 0 || S < k + 1 || optimizer > 1 || combine > 1) return -3;
    for (uint64_t i = 0; i < n; ++i)
        if (keys[i] >= R) return -1;
    const double lr = (double)lr_f, eps = (double)eps_f, mu = (double)mu_f;
    const uint64_t Gn = R / k;
    double *E64 = widen(E, R * D), *A64 = widen(A, R * D);
    double *PE64 = widen(PE, Gn * D), *PA64 = widen(PA, Gn * D);
    double *sum = combine ? (double *)calloc(R * D, sizeof(double)) : NULL;
    unsigned char *hit = combine ? (unsigned char *)calloc(R, 1) : NULL;
    if (!E64 || !A64 || !PE64 || !PA64 || (combine && (!sum || !hit))) {
        free(E64); free(A64); free(PE64); free(PA64); free(sum); free(hit);
        return -2;
    }
    if (!combine) {
        for (uint64_t i = 0; i < n; ++i) {
            const uint64_t x = keys[i], g = stripe_of(x, k);
            for (uint32_t d = 0; d < D; ++d) {
                double *e = &E64[x * D + d], *a = &A64[x * D + d];
                const double e_old = *e, a_old = *a;
                rule_step(e, a, (double)grads[i * D + d], optimizer, lr, eps, mu);
                PE64[g * D + d] += *e - e_old;
                PA64[g * D + d] += *a - a_old;
            }
            if (load_data) load_data[data_server_of(g, member_of(x, k), S)] += 1;
            if (load_parity) load_parity[parity_server_of(g, S)] += 1;
        }
    } else {
        for (uint64_t i = 0; i < n; ++i) {
            const uint64_t x = keys[i];
            hit[x] = 1;
            for (uint32_t d = 0; d < D; ++d) sum[x * D + d] += (double)grads[i * D + d];
        }
        for (uint64_t x = 0; x < R; ++x) {
            if (!hit[x]) continue;
            const uint64_t g = stripe_of(x, k);
            for (uint32_t d = 0; d < D; ++d) {
                double *e = &E64[x * D + d], *a = &A64[x * D + d];
                const double e_old = *e, a_old = *a;
                rule_step(e, a, sum[x * D + d], optimizer, lr, eps, mu);
                PE64[g * D + d] += *e - e_old;
                PA64[g * D + d] += *a - a_old;
            }
            if (load_data) load_data[data_server_of(g, member_of(x, k), S)] += 1;
            if (load_parity) load_parity[parity_server_of(g, S)] += 1;
        }
    }
    narrow(E, E64, R * D);   narrow(A, A64, R * D);
    narrow(PE, PE64, Gn * D); narrow(PA, PA64, Gn * D);
    free(E64); free(A64); free(PE64); free(PA64); free(sum); free(hit);
    return 0;
}

/*
 * Gradient propagation (the strawman of Sec. 3.3.1) under either update rule: every update is applied
 * to its entry with the entry's state AND to the stripe's parity entry with the parity's state, in
 * arrival order.  Adagrad's step depends on the state, so the parity drifts away from the sum of its
 * entries.  The momentum rule breaks it too although it is linear: an update decays the parity's
 * whole velocity, i.e. also the share of the stripe's entries that were not updated.  Both are
 * pinned by hand-computed chains in the tests.
 */
int ecrm_oracle_update_gradient_propagation_rule(float *E, float *A, float *PE, float *PA,
                                                 uint64_t R, uint32_t D, uint32_t k, float lr_f, float eps_f,
                                                 float mu_f, uint32_t optimizer,
                                                 const uint64_t *keys, const float *grads, uint64_t n)
{
    if (k == 0 || R % k != 0 || optimizer > 1) return -3;
    for (uint64_t i = 0; i < n; ++i)
        if (keys[i] >= R) return -1;
    const double lr = (double)lr_f, eps = (double)eps_f, mu = (double)mu_f;
    const uint64_t Gn = R / k;
    double *E64 = widen(E, R * D), *A64 = widen(A, R * D);
    double *PE64 = widen(PE, Gn * D), *PA64 = widen(PA, Gn * D);
    if (!E64 || !A64 || !PE64 || !PA64) { free(E64); free(A64); free(PE64); free(PA64); return -2; }
    for (uint64_t i = 0; i < n; ++i) {
        const uint64_t x = keys[i], g = stripe_of(x, k);
        for (uint32_t d = 0; d < D; ++d) {
            const double gd = (double)grads[i * D + d];
            rule_step(&E64[x * D + d], &A64[x * D + d], gd, optimizer, lr, eps, mu);
            rule_step(&PE64[g * D + d], &PA64[g * D + d], gd, optimizer, lr, eps, mu);
        }
    }
    narrow(E, E64, R * D);   narrow(A, A64, R * D);
    narrow(PE, PE64, Gn * D); narrow(PA, PA64, Gn * D);
    free(E64); free(A64); free(PE64); free(PA64);
    return 0;
}

int ecrm_oracle_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
