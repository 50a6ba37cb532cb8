/*
 * CPU oracle for farthest point sampling (FPS) and the FlashFPS variants.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain statement of what
 * the GPU library must compute.  It is used by the tests, by the smoke check
 * and by the benchmark's CPU-baseline leg.  The product path never calls it,
 * and it shares no code, header, table or helper with the HIP sources.
 *
 * Build: gcc -O2 -ffp-contract=off -fno-fast-math -shared -fPIC
 * (contraction must stay off: a fused multiply-add changes low bits of the
 * squared distance and therefore changes picks).
 *
 * Conventions fixed for the whole build (the paper leaves them open):
 *   - coordinates are fp32, array-of-structs [N][3]; indices are int32;
 *   - squared Euclidean distance  ((dx*dx) + (dy*dy)) + (dz*dz), every
 *     operation rounded to fp32 (round-to-nearest-even), no FMA.  Squared
 *     and true distance order points identically, so Eq. 1's norm is never
 *     taken inside the loop;
 *   - running minimum distance starts at +inf;
 *   - the argmax runs over ALL points (Eq. 2's form of the rule): a sampled
 *     point has minimum distance 0 and can only win when every point has 0;
 *   - ties go to the lowest index (lowest position in the array FPS runs on).
 *
 * Every function is pinned by tests that do not use this file's own
 * arithmetic: hand-worked lattice sequences, a from-scratch brute force of
 * Eq. 1 in exact integer arithmetic, the p = 0 and prefix-equivalence
 * identities of Sec. 3.2 / 3.3, and closed-form index sets for the
 * pruning and fill rules.  Nothing here is "parity unpinned".
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORACLE_FLAG_CP 1u /* candidate pruning  (Alg. 1, step "P' <- UniformSample") */
#define ORACLE_FLAG_IP 2u /* iteration pruning  (Alg. 1, step "k <- (1-p) M1")       */
#define ORACLE_FLAG_PERM 4u /* seeded random sub-sample and fill instead of strided ones */

#define ORACLE_MODE_CACHED 0      /* Alg. 1, layers 2..L: prefixes of the cached P1 */
#define ORACLE_MODE_CHAIN 1       /* Sec. 3.3: every layer runs its own FPS          */

static float sqdist(const float *a, const float *b)
{
    float dx = a[0] - b[0];
    float dy = a[1] - b[1];
    float dz = a[2] - b[2];
    float xx = dx * dx;
    float yy = dy * dy;
    float zz = dz * dz;
    float s = xx + yy;
    return s + zz;
}

/*
 * Exact FPS, Eq. 1 (Sec. 3.1), as the loop Sec. 1 describes: after each pick,
 * every point's minimum distance to the sampled set is refreshed with its
 * distance to the newest sample, then the point with the largest minimum
 * distance is the next pick.
 *
 * idx[0] = start; idx[1..M-1] = picks.  maxdist (optional) receives the
 * squared minimum distance each pick had when it was chosen; maxdist[0] = +inf.
 * Returns 0, or -1 on invalid arguments.
 */
int oracle_fps_exact(const float *xyz, int N, int M, int start, int32_t *idx, float *maxdist)
{
    if (!xyz || !idx || N < 1 || M < 1 || M > N || start < 0 || start >= N)
        return -1;
    float *mind = (float *)malloc((size_t)N * sizeof(float));
    if (!mind)
        return -2;
    for (int i = 0; i < N; ++i)
        mind[i] = INFINITY;
    idx[0] = start;
    if (maxdist)
        maxdist[0] = INFINITY;
    int last = start;
    for (int k = 1; k < M; ++k) {
        const float *q = xyz + 3 * (size_t)last;
        int best = -1;
        float bestd = 0.0f;
        for (int i = 0; i < N; ++i) {
            float d = sqdist(xyz + 3 * (size_t)i, q);
            if (d < mind[i])
                mind[i] = d;
            if (best < 0 || mind[i] > bestd) { /* strict >: lowest index keeps a tie */
                best = i;
                bestd = mind[i];
            }
        }
        idx[k] = best;
        if (maxdist)
            maxdist[k] = bestd;
        last = best;
    }
    free(mind);
    return 0;
}

/* ceil(a * num / den) in 64-bit integers */
static int64_t ceil_frac(int64_t a, int64_t num, int64_t den)
{
    return (a * num + den - 1) / den;
}

/*
 * Sizes of FPS-Prune (Alg. 1, layer 1; Sec. 3.2).  keep_num/keep_den = 1 - p.
 *   N' = ceil(N * keep) if candidate pruning is on, else N
 *   k  = ceil(M * keep) if iteration pruning is on, else M
 *   R  = M - k  random-fill picks (= floor(p * M) when IP is on)
 * Returns 0, or -1 when the ratio is outside (0, 1] or k > N'.
 */
int oracle_prune_sizes(int N, int M, int keep_num, int keep_den, unsigned flags,
                       int *Nc, int *k, int *R)
{
    if (N < 1 || M < 1 || M > N || keep_num < 1 || keep_den < 1 || keep_num > keep_den)
        return -1;
    if (flags & ~(ORACLE_FLAG_CP | ORACLE_FLAG_IP | ORACLE_FLAG_PERM))
        return -1;
    int64_t nc = (flags & ORACLE_FLAG_CP) ? ceil_frac(N, keep_num, keep_den) : N;
    int64_t kk = (flags & ORACLE_FLAG_IP) ? ceil_frac(M, keep_num, keep_den) : M;
    if (kk < 1 || kk > nc)
        return -1;
    *Nc = (int)nc;
    *k = (int)kk;
    *R = M - (int)kk;
    return 0;
}

static int cmp_i32(const void *a, const void *b)
{
    int32_t x = *(const int32_t *)a, y = *(const int32_t *)b;
    return (x > y) - (x < y);
}

/*
 * Candidate list of candidate pruning: an index-uniform subsample of N' of the
 * N points, shifted so that it contains `start`, kept in ascending index order.
 *   cand = sort{ (start + floor(j * N / N')) mod N : j = 0..N'-1 }
 * *start_pos receives the position of `start` inside cand.
 */
int oracle_candidates(int N, int Nc, int start, int32_t *cand, int *start_pos)
{
    if (N < 1 || Nc < 1 || Nc > N || start < 0 || start >= N)
        return -1;
    for (int j = 0; j < Nc; ++j)
        cand[j] = (int32_t)(((int64_t)start + ((int64_t)j * N) / Nc) % N);
    qsort(cand, (size_t)Nc, sizeof(int32_t), cmp_i32);
    *start_pos = -1;
    for (int j = 0; j < Nc; ++j)
        if (cand[j] == start)
            *start_pos = j;
    return *start_pos < 0 ? -1 : 0;
}

/*
 * Seeded bijection of [0, N) for the random variants of "UniformSample" and
 * "RandomSample" (Alg. 1, layer 1), which the paper leaves unspecified.
 * A 4-round Feistel network over 2h bits, 2^(2h) >= N, with a 32-bit integer
 * mixer as round function, walked until the value falls below N (a cycle walk
 * of a bijection of a superset is a bijection of the subset).  Stateless:
 * element j is computed on its own, so a parallel implementation needs no
 * sequential random stream.
 */
static uint32_t perm_mix(uint32_t x)
{
    x ^= x >> 16;
    x *= 0x85EBCA6Bu;
    x ^= x >> 13;
    x *= 0xC2B2AE35u;
    x ^= x >> 16;
    return x;
}

int64_t oracle_perm(int64_t N, uint64_t seed, int64_t j)
{
    if (N < 1 || j < 0 || j >= N)
        return -1;
    int h = 1;
    while (((int64_t)1 << (2 * h)) < N)
        ++h;
    const uint32_t mask = ((uint32_t)1 << h) - 1u;
    const uint32_t key[2] = {(uint32_t)seed, (uint32_t)(seed >> 32)};
    uint64_t x = (uint64_t)j;
    do {
        uint32_t l = (uint32_t)(x >> h) & mask, r = (uint32_t)x & mask;
        for (uint32_t round = 0; round < 4; ++round) {
            uint32_t f = perm_mix(r ^ (key[round & 1] + 0x9E3779B9u * (round + 1))) & mask;
            uint32_t t = l ^ f;
            l = r;
            r = t;
        }
        x = ((uint64_t)l << h) | r;
    } while (x >= (uint64_t)N);
    return (int64_t)x;
}

/*
 * Random candidate list: the N' images perm(j), j < N', with perm(N'-1)
 * replaced by `start` when start is not among them; ascending order.
 */
int oracle_candidates_perm(int N, int Nc, int start, uint64_t seed, int32_t *cand, int *start_pos)
{
    if (N < 1 || Nc < 1 || Nc > N || start < 0 || start >= N)
        return -1;
    int has = 0;
    for (int j = 0; j < Nc; ++j) {
        cand[j] = (int32_t)oracle_perm(N, seed, j);
        if (cand[j] == start)
            has = 1;
    }
    if (!has)
        cand[Nc - 1] = start;
    qsort(cand, (size_t)Nc, sizeof(int32_t), cmp_i32);
    *start_pos = -1;
    for (int j = 0; j < Nc; ++j)
        if (cand[j] == start)
            *start_pos = j;
    return *start_pos < 0 ? -1 : 0;
}

/* second, independent permutation for the fill */
#define ORACLE_FILL_SEED_XOR 0xD1B54A32D192ED03ull

/*
 * FPS-Prune (Alg. 1, layer 1).  idx[0..k-1] = FPS order on the candidate
 * cloud mapped back to indices of the full cloud; idx[k..M-1] = fill picks:
 * with free = ascending list of the N - k indices not picked by FPS,
 *   fill[j] = free[ floor(j * (N - k) / R) ],  j = 0..R-1.
 * The fill is drawn from the full cloud, not from the candidate cloud.
 * With ORACLE_FLAG_PERM both the candidate list and the fill are seeded random
 * draws instead (oracle_candidates_perm; fill as described in the body).
 */
int oracle_fps_prune(const float *xyz, int N, int M, int start, int keep_num, int keep_den,
                     unsigned flags, uint64_t seed, int32_t *idx, int *k_out)
{
    int Nc, k, R;
    if (!xyz || !idx || start < 0 || start >= N)
        return -1;
    if (oracle_prune_sizes(N, M, keep_num, keep_den, flags, &Nc, &k, &R))
        return -1;
    int32_t *cand = (int32_t *)malloc((size_t)Nc * sizeof(int32_t));
    float *cxyz = (float *)malloc((size_t)Nc * 3 * sizeof(float));
    int32_t *loc = (int32_t *)malloc((size_t)k * sizeof(int32_t));
    unsigned char *taken = (unsigned char *)calloc((size_t)N, 1);
    int32_t *freelist = (int32_t *)malloc((size_t)N * sizeof(int32_t));
    int rc = -2, spos = 0;
    if (!cand || !cxyz || !loc || !taken || !freelist)
        goto done;
    if ((flags & ORACLE_FLAG_PERM) ? oracle_candidates_perm(N, Nc, start, seed, cand, &spos)
                                   : oracle_candidates(N, Nc, start, cand, &spos)) {
        rc = -1;
        goto done;
    }
    for (int j = 0; j < Nc; ++j)
        memcpy(cxyz + 3 * (size_t)j, xyz + 3 * (size_t)cand[j], 3 * sizeof(float));
    rc = oracle_fps_exact(cxyz, Nc, k, spos, loc, NULL);
    if (rc)
        goto done;
    for (int j = 0; j < k; ++j) {
        idx[j] = cand[loc[j]];
        taken[idx[j]] = 1;
    }
    if (flags & ORACLE_FLAG_PERM) {
        /* random fill: walk a second permutation of [0, N) and keep the first R
         * indices that FPS did not pick, in that order */
        int got = 0;
        for (int64_t j = 0; j < N && got < R; ++j) {
            int32_t t = (int32_t)oracle_perm(N, seed ^ ORACLE_FILL_SEED_XOR, j);
            if (!taken[t])
                idx[k + got++] = t;
        }
    } else {
        int64_t nfree = 0;
        for (int i = 0; i < N; ++i)
            if (!taken[i])
                freelist[nfree++] = i;
        for (int j = 0; j < R; ++j)
            idx[k + j] = freelist[((int64_t)j * nfree) / R];
    }
    if (k_out)
        *k_out = k;
    rc = 0;
done:
    free(cand);
    free(cxyz);
    free(loc);
    free(taken);
    free(freelist);
    return rc;
}

/*
 * Hierarchical stage chain (Alg. 1; Sec. 3.3).  Ms[0] >= Ms[1] >= ... >= Ms[L-1].
 * Layer 1 is oracle_fps_prune with Ms[0] (exact FPS when keep = 1/1).
 *   CACHED: layer l = first Ms[l] entries of layer 1 (Alg. 1, layers 2..L).
 *   CHAIN : layer l = FPS over the points of layer l-1 stored in sample
 *           order, started at position 0, Ms[l] picks, mapped back to indices
 *           of the full cloud (the independent per-layer FPS of Sec. 3.3).
 * out holds the layers back to back: layer l at offset Ms[0] + ... + Ms[l-1].
 */
int oracle_fps_stages(const float *xyz, int N, int L, const int *Ms, int start, int keep_num,
                      int keep_den, unsigned flags, uint64_t seed, int mode, int32_t *out)
{
    if (!xyz || !Ms || !out || L < 1)
        return -1;
    for (int l = 1; l < L; ++l)
        if (Ms[l] > Ms[l - 1] || Ms[l] < 1)
            return -1;
    int rc = oracle_fps_prune(xyz, N, Ms[0], start, keep_num, keep_den, flags, seed, out, NULL);
    if (rc)
        return rc;
    size_t off = (size_t)Ms[0];
    const int32_t *prev = out;
    for (int l = 1; l < L; ++l) {
        int32_t *cur = out + off;
        if (mode == ORACLE_MODE_CACHED) {
            memcpy(cur, out, (size_t)Ms[l] * sizeof(int32_t));
        } else {
            int Np = Ms[l - 1];
            float *pxyz = (float *)malloc((size_t)Np * 3 * sizeof(float));
            int32_t *loc = (int32_t *)malloc((size_t)Ms[l] * sizeof(int32_t));
            if (!pxyz || !loc) {
                free(pxyz);
                free(loc);
                return -2;
            }
            for (int j = 0; j < Np; ++j)
                memcpy(pxyz + 3 * (size_t)j, xyz + 3 * (size_t)prev[j], 3 * sizeof(float));
            rc = oracle_fps_exact(pxyz, Np, Ms[l], 0, loc, NULL);
            for (int j = 0; rc == 0 && j < Ms[l]; ++j)
                cur[j] = prev[loc[j]];
            free(pxyz);
            free(loc);
            if (rc)
                return rc;
        }
        prev = cur;
        off += (size_t)Ms[l];
    }
    return 0;
}

/*
 * Coverage radius of a sampled set over the full cloud:
 *   R_P(S) = sqrt( max_{p in P} min_{q in S} d2(p, q) ),
 * d2 in fp32 as above, the square root in double.  Used to state how far a
 * pruned or cached sample set is from exact FPS.
 */
double oracle_coverage_radius(const float *xyz, int N, const int32_t *sel, int S)
{
    if (!xyz || !sel || N < 1 || S < 1)
        return -1.0;
    float worst = 0.0f;
    for (int i = 0; i < N; ++i) {
        float m = INFINITY;
        for (int s = 0; s < S; ++s) {
            float d = sqdist(xyz + 3 * (size_t)i, xyz + 3 * (size_t)sel[s]);
            if (d < m)
                m = d;
        }
        if (m > worst)
            worst = m;
    }
    return sqrt((double)worst);
}

/*
 * Exact FPS on several host threads: the same loop as oracle_fps_exact with the
 * points of each iteration divided into `nthreads` contiguous chunks.  Every
 * thread refreshes the minimum distances of its chunk and finds the chunk's
 * best point (largest value, lowest index: strict > in ascending order);
 * after a barrier every thread merges the chunk results in ascending chunk
 * order with the same strict >, which again keeps the lowest index among equal
 * values.  Per-point arithmetic is that of the single-thread loop, so the
 * result is identical to it for any number of threads (asserted by the tests).
 * Exists for the all-cores CPU baseline of the benchmark; the single-thread
 * function above stays the reference statement of the method.
 */
#include <pthread.h>
#include <sched.h>
#include <stdatomic.h>

typedef struct {
    atomic_int count;
    atomic_int sense;
    int n;
} spin_barrier;

static void spin_barrier_wait(spin_barrier *b, int *local_sense)
{
    *local_sense = !*local_sense;
    if (atomic_fetch_add(&b->count, 1) == b->n - 1) {
        atomic_store(&b->count, 0);
        atomic_store(&b->sense, *local_sense);
    } else {
        int spins = 0;
        while (atomic_load(&b->sense) != *local_sense)
            if (++spins > 2000) /* more threads than free cores: let the others run */
                sched_yield();
    }
}

typedef struct {
    float d;
    int i;
    char pad[56]; /* one cache line per slot */
} chunk_best;

typedef struct {
    const float *xyz;
    float *mind;
    int N, M, start;
    int32_t *idx;
    float *maxdist;
    int nthreads;
    chunk_best *slots; /* [2][nthreads], alternating by iteration parity */
    spin_barrier bar;
} mt_shared;

typedef struct {
    mt_shared *sh;
    int t;
} mt_arg;

static void *mt_worker(void *p)
{
    mt_arg *a = (mt_arg *)p;
    mt_shared *sh = a->sh;
    const int T = sh->nthreads, t = a->t;
    const int lo = (int)((int64_t)sh->N * t / T), hi = (int)((int64_t)sh->N * (t + 1) / T);
    const float *xyz = sh->xyz;
    float *mind = sh->mind;
    int sense = 0;
    for (int i = lo; i < hi; ++i)
        mind[i] = INFINITY;
    int last = sh->start;
    for (int k = 1; k < sh->M; ++k) {
        const float *q = xyz + 3 * (size_t)last;
        int best = -1;
        float bestd = 0.0f;
        for (int i = lo; i < hi; ++i) {
            float d = sqdist(xyz + 3 * (size_t)i, q);
            if (d < mind[i])
                mind[i] = d;
            if (best < 0 || mind[i] > bestd) {
                best = i;
                bestd = mind[i];
            }
        }
        chunk_best *slot = sh->slots + (size_t)(k & 1) * T;
        slot[t].d = bestd;
        slot[t].i = best; /* -1: empty chunk */
        spin_barrier_wait(&sh->bar, &sense);
        best = -1;
        bestd = 0.0f;
        for (int c = 0; c < T; ++c)
            if (slot[c].i >= 0 && (best < 0 || slot[c].d > bestd)) {
                best = slot[c].i;
                bestd = slot[c].d;
            }
        if (t == 0) {
            sh->idx[k] = best;
            if (sh->maxdist)
                sh->maxdist[k] = bestd;
        }
        last = best;
    }
    return NULL;
}

int oracle_fps_exact_mt(const float *xyz, int N, int M, int start, int32_t *idx, float *maxdist,
                        int nthreads)
{
    if (!xyz || !idx || N < 1 || M < 1 || M > N || start < 0 || start >= N || nthreads < 1 ||
        nthreads > 1024)
        return -1;
    mt_shared sh;
    sh.xyz = xyz;
    sh.N = N;
    sh.M = M;
    sh.start = start;
    sh.idx = idx;
    sh.maxdist = maxdist;
    sh.nthreads = nthreads;
    atomic_init(&sh.bar.count, 0);
    atomic_init(&sh.bar.sense, 0);
    sh.bar.n = nthreads;
    sh.mind = (float *)malloc((size_t)N * sizeof(float));
    sh.slots = (chunk_best *)malloc((size_t)2 * nthreads * sizeof(chunk_best));
    pthread_t *th = (pthread_t *)malloc((size_t)nthreads * sizeof(pthread_t));
    mt_arg *args = (mt_arg *)malloc((size_t)nthreads * sizeof(mt_arg));
    int rc = -2;
    if (sh.mind && sh.slots && th && args) {
        idx[0] = start;
        if (maxdist)
            maxdist[0] = INFINITY;
        int made = 0;
        for (; made < nthreads; ++made) {
            args[made].sh = &sh;
            args[made].t = made;
            if (pthread_create(&th[made], NULL, mt_worker, &args[made]))
                break;
        }
        if (made == nthreads) {
            rc = 0;
        } else {
            /* the barrier would wait for the missing threads for ever: this cannot
             * be recovered without them, so treat it as fatal for the process */
            abort();
        }
        for (int t = 0; t < made; ++t)
            pthread_join(th[t], NULL);
    }
    free(sh.mind);
    free(sh.slots);
    free(th);
    free(args);
    return rc;
}
