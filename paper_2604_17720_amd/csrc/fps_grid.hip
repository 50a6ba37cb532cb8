// k_fps_grid: exact FPS (Sec. 3.1, Eq. 1) of ONE cloud spread over all CUs.
//
// Each of G co-resident workgroups keeps a contiguous slice of the cloud and
// its running minimum distances in registers for the whole call.  Workgroups
// meet once per ROUND, and a round can deliver several picks:
//
//   1. every workgroup applies the picks of the previous round to its points
//      and finds its best point (value, lowest index) and an upper bound on
//      all its OTHER points (its second-best value);
//   2. it publishes {best value, index, bound} and {x, y, z} as two 16-byte
//      chunks, each closed by a checksum that also encodes the round; one wave
//      per workgroup gathers all G records with coalesced device-scope loads
//      (this all-gather is the only cross-workgroup step: no counters, no
//      fences, no separate barrier);
//   3. that wave replays the greedy rule on the G published candidates only:
//      the best candidate is the next pick of Eq. 1 as long as its value is
//      strictly above B = max of all bounds, because no unpublished point can
//      then reach it; picking it lowers the other candidates' values by the
//      same distance rule, and the replay continues until the test fails.
//      The first pick of a round never needs the test (a workgroup's best
//      dominates its own other points, ties included, since it is the lowest
//      index among equals and slices are in index order).
//
// Every workgroup replays the same deterministic arithmetic on the same
// records, so all agree on the picks without further communication.  The
// picks are exactly those of the one-pick-per-pass loop: a pick is accepted
// only when it is provably the global (value, lowest index) maximum.
//
// Exit: every spin loop is bounded; a workgroup that gives up sets the status
// word and leaves, and the others then run into their own bound.
#include "fps_device.h"
#include "fps_launch.h"

namespace ffps {

namespace {

constexpr int kRPL = kMaxGridWG / kWave;  // records per lane of the gathering wave
constexpr int kSpinLimit = 1 << 19;

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// Exchange area: two buffers (round parity); each holds chunk array A
// {value, index, bound, check} and chunk array B {x, y, z, check}, 256 slots
// of 16 bytes each.  Workgroup w uses slot (w & 3) * 64 + (w >> 2), so that a
// wave reading slot q*64 + lane with one 16-byte load per lane touches one
// contiguous KiB, while lane L still ends up with workgroups 4L .. 4L+3.
constexpr size_t kChunkBytes = (size_t)kMaxGridWG * 16;
constexpr size_t kBufBytes = 2 * kChunkBytes;
__device__ __forceinline__ int slot_of(int w) { return (w & 3) * kWave + (w >> 2); }

// A chunk is valid for a round when its last word equals this value.  Memory
// cleared to zero never validates (the round term is non-zero for round >= 1),
// a chunk of round-2 in the same buffer does not validate, and a read that
// mixed old and new words fails the test and is simply polled again.
__device__ __forceinline__ uint32_t chunk_check(uint32_t a, uint32_t b, uint32_t c, uint32_t round,
                                                uint32_t which) {
    uint32_t m = a ^ ((b << 11) | (b >> 21)) ^ ((c << 22) | (c >> 10));
    return m ^ (round * 0x9E3779B1u + which * 0x85EBCA6Bu);
}

// Device-scope (all XCDs) 16-byte store and loads.  The compiler offers atomics
// up to 8 bytes only, so these are spelled out; sc1 is the device-scope cache
// policy the compiler itself uses for agent-scope atomics on this target.
__device__ __forceinline__ void store_chunk(void *p, u32x4 v) {
    asm volatile("global_store_dwordx4 %0, %1, off sc1" : : "v"(p), "v"(v) : "memory");
}
// r[q] = 16 bytes at p + q * 1024, q < 4: one batch of four loads, then one wait.
__device__ __forceinline__ void load_chunks(const void *p, u32x4 (&r)[kMaxGridWG / kWave]) {
    static_assert(kMaxGridWG / kWave == 4, "four slots per lane");
    asm volatile(
        "global_load_dwordx4 %0, %4, off sc1\n\t"
        "global_load_dwordx4 %1, %4, off offset:1024 sc1\n\t"
        "global_load_dwordx4 %2, %4, off offset:2048 sc1\n\t"
        "global_load_dwordx4 %3, %4, off offset:3072 sc1\n\t"
        "s_waitcnt vmcnt(0)"
        : "=&v"(r[0]), "=&v"(r[1]), "=&v"(r[2]), "=&v"(r[3])
        : "v"(p)
        : "memory");
}

struct WaveTop {
    uint32_t m1;  // best value (bits)
    int idx;
    float x, y, z;
    uint32_t m2;  // upper bound on the wave's other points (bits)
    uint32_t pad[2];
};

struct GridArgs {
    const float *xyz;
    int N, M, start;
    int chunk;  // points per workgroup
    int32_t *idx_out;
    float *md_out;
    char *exchange;      // two buffers of kBufBytes
    int *status;
    int max_picks;
};

// Phase timing of workgroup 0 (100 MHz wall clock), compiled in only for
// profiling builds: status[8 + i] accumulates phase i, status[15] the polls.
#ifdef FFPS_PROFILE
#define FFPS_STAMP(i)                                        \
    do {                                                     \
        if (w == 0 && tid == 0) {                            \
            uint64_t now_ = wall_clock64();                  \
            prof_acc[i] += (uint32_t)(now_ - prof_last);     \
            prof_last = now_;                                \
        }                                                    \
    } while (0)
#else
#define FFPS_STAMP(i) do { } while (0)
#endif

template <int NT, int P>
__global__ __launch_bounds__(NT) void k_fps_grid(GridArgs a) {
    constexpr int NW = NT / kWave;
    __shared__ WaveTop wtop[NW];
    __shared__ float pkx[kMaxPicksPerRound], pky[kMaxPicksPerRound], pkz[kMaxPicksPerRound];
    __shared__ int s_cnt, s_abort;
    __shared__ uint32_t cmp_v[kWave];
    __shared__ int cmp_i[kWave];
    __shared__ float cmp_x[kWave], cmp_y[kWave], cmp_z[kWave];

    const int G = gridDim.x;
    const int w = blockIdx.x;
    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1);
    const int wave = tid / kWave;
    const int lo = w * a.chunk;
    const int hi = min(a.N, lo + a.chunk);
    const int base = lo + tid * P;

    float x[P], y[P], z[P], m[P];
#pragma unroll
    for (int j = 0; j < P; ++j) {
        int i = base + j;
        bool ok = i < hi;
        x[j] = ok ? a.xyz[3 * (size_t)i + 0] : 0.f;
        y[j] = ok ? a.xyz[3 * (size_t)i + 1] : 0.f;
        z[j] = ok ? a.xyz[3 * (size_t)i + 2] : 0.f;
        m[j] = ok ? __builtin_inff() : 0.f;  // padding: value 0, never preferred
    }

    if (tid == 0) {
        pkx[0] = a.xyz[3 * (size_t)a.start + 0];
        pky[0] = a.xyz[3 * (size_t)a.start + 1];
        pkz[0] = a.xyz[3 * (size_t)a.start + 2];
        s_cnt = 1;
        s_abort = 0;
        if (w == 0) {
            a.idx_out[0] = a.start;
            if (a.md_out) a.md_out[0] = __builtin_inff();
        }
    }
    __syncthreads();

    int npicked = 1;
    uint32_t round = 0;
#ifdef FFPS_PROFILE
    uint32_t prof_acc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    uint64_t prof_last = wall_clock64();
#endif
    while (npicked < a.M) {
        ++round;
        FFPS_STAMP(5);
        // ---- 1. apply last round's picks, then per-lane best and bound ----
        const int cnt_prev = s_cnt;
        for (int q = 0; q < cnt_prev; ++q) {
            float lx = pkx[q], ly = pky[q], lz = pkz[q];
#pragma unroll
            for (int j = 0; j < P; ++j) m[j] = fminf(m[j], sqdist(x[j], y[j], z[j], lx, ly, lz));
        }
        float m1 = m[0], m2 = 0.f;
        int j1 = 0;
#pragma unroll
        for (int j = 1; j < P; ++j) {
            bool gt = m[j] > m1;  // strict: the lowest j keeps a tie
            m2 = fmaxf(m2, gt ? m1 : m[j]);
            j1 = gt ? j : j1;
            m1 = gt ? m[j] : m1;
        }
        uint32_t W1 = wave_max_u32(f2u(m1));
        int wl = first_lane(f2u(m1) == W1);
        uint32_t W2 = wave_max_u32(lane == wl ? f2u(m2) : f2u(m1));
        int wj = readlane_i(j1, wl);
        float wx = pick_elem<P>(x, wj, wl);
        float wy = pick_elem<P>(y, wj, wl);
        float wz = pick_elem<P>(z, wj, wl);
        if (lane == 0) {
            wtop[wave].m1 = W1;
            wtop[wave].idx = lo + (wave * kWave + wl) * P + wj;
            wtop[wave].x = wx;
            wtop[wave].y = wy;
            wtop[wave].z = wz;
            wtop[wave].m2 = W2;
        }
        FFPS_STAMP(0);
        __syncthreads();  // wave tops visible; everyone is done with pk*/s_cnt
        FFPS_STAMP(1);

        if (wave == 0) {
            // ---- 2a. workgroup best and bound ----
            uint32_t s1 = lane < NW ? wtop[lane].m1 : 0u;
            uint32_t G1 = (uint32_t)readlane_i((int)row16_max_u32(s1), 15);
            int ww = first_lane(lane < NW && s1 == G1);
            uint32_t s2 = lane < NW ? (lane == ww ? wtop[lane].m2 : s1) : 0u;
            uint32_t Bw = (uint32_t)readlane_i((int)row16_max_u32(s2), 15);
            // ---- 2b. publish: two 16-byte chunks, each closed by a checksum ----
            char *buf = a.exchange + (size_t)(round & 1) * kBufBytes;
            if (lane == 0) {
                u32x4 ca, cb4;
                ca.x = G1; ca.y = (uint32_t)wtop[ww].idx; ca.z = Bw;
                ca.w = chunk_check(ca.x, ca.y, ca.z, round, 0);
                cb4.x = f2u(wtop[ww].x); cb4.y = f2u(wtop[ww].y); cb4.z = f2u(wtop[ww].z);
                cb4.w = chunk_check(cb4.x, cb4.y, cb4.z, round, 1);
                const int slot = slot_of(w);
                store_chunk(buf + (size_t)slot * 16, ca);
                store_chunk(buf + kChunkBytes + (size_t)slot * 16, cb4);
            }
            FFPS_STAMP(2);
            // ---- 2c. gather: lane L reads slots q*64+L = workgroups 4L+q ----
            u32x4 ra[kRPL], rb4[kRPL];
            bool gave_up = false;
            for (int spin = 0;; ++spin) {
                load_chunks(buf + (size_t)lane * 16, ra);
                load_chunks(buf + kChunkBytes + (size_t)lane * 16, rb4);
                bool all = true;
#pragma unroll
                for (int q = 0; q < kRPL; ++q) {
                    bool ok = ra[q].w == chunk_check(ra[q].x, ra[q].y, ra[q].z, round, 0) &&
                              rb4[q].w == chunk_check(rb4[q].x, rb4[q].y, rb4[q].z, round, 1);
                    all = all && (ok || lane * kRPL + q >= G);
                }
#ifdef FFPS_PROFILE
                if (w == 0 && tid == 0) ++prof_acc[7];
#endif
                if (__builtin_amdgcn_ballot_w64(!all) == 0) break;
                if (spin >= kSpinLimit) {
                    gave_up = true;
                    break;
                }
            }
            FFPS_STAMP(3);
            if (gave_up) {
                if (lane == 0) {
                    __hip_atomic_store(a.status, -5, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    s_abort = 1;
                    s_cnt = 0;
                }
            } else {
                uint32_t cv[kRPL], lb = 0u;
                int ci[kRPL];
                float cx[kRPL], cy[kRPL], cz[kRPL];
#pragma unroll
                for (int q = 0; q < kRPL; ++q) {
                    bool present = lane * kRPL + q < G;  // absent records: value 0, bound 0
                    cv[q] = present ? ra[q].x : 0u;
                    ci[q] = present ? (int)ra[q].y : 0x7fffffff;
                    lb = umax(lb, present ? ra[q].z : 0u);
                    cx[q] = present ? u2f(rb4[q].x) : 0.f;
                    cy[q] = present ? u2f(rb4[q].y) : 0.f;
                    cz[q] = present ? u2f(rb4[q].z) : 0.f;
                }
                // ---- 3. replay the greedy rule on the published candidates ----
                const uint32_t Bound = wave_max_u32(lb);
                const int cap = min(a.max_picks, a.M - npicked);
                int cnt = 0;
                // first pick of the round: best candidate, no test needed
                uint32_t bv = cv[0];
                int bq = 0;
#pragma unroll
                for (int q = 1; q < kRPL; ++q)
                    if (cv[q] > bv) {
                        bv = cv[q];
                        bq = q;
                    }
                uint32_t V = wave_max_u32(bv);
                int pl = first_lane(bv == V);
                int pq = readlane_i(bq, pl);
                float px = pick_elem<kRPL>(cx, pq, pl);
                float py = pick_elem<kRPL>(cy, pq, pl);
                float pz = pick_elem<kRPL>(cz, pq, pl);
                int pidx = 0;
#pragma unroll
                for (int q = 0; q < kRPL; ++q)
                    if (pq == q) pidx = readlane_i(ci[q], pl);
                auto emit = [&](int c, int idx, uint32_t vbits, float ex, float ey, float ez) {
                    if (lane == 0) {
                        pkx[c] = ex;
                        pky[c] = ey;
                        pkz[c] = ez;
                        if (w == 0) {
                            a.idx_out[npicked + c] = idx;
                            if (a.md_out) a.md_out[npicked + c] = u2f(vbits);
                        }
                    }
                };
                emit(0, pidx, V, px, py, pz);
                cnt = 1;
                if (V > Bound && cnt < cap) {
                    // Only candidates above the bound can be picked later in this
                    // round.  Compact them, one per lane, in workgroup order.
                    uint64_t mk[kRPL];
                    int total = 0, before = 0;
                    const uint64_t lt = ((uint64_t)1 << lane) - 1;
#pragma unroll
                    for (int q = 0; q < kRPL; ++q) {
                        mk[q] = __builtin_amdgcn_ballot_w64(cv[q] > Bound);
                        total += __builtin_popcountll(mk[q]);
                        before += __builtin_popcountll(mk[q] & lt);
                    }
                    if (total <= kWave) {
                        int pos = before;
#pragma unroll
                        for (int q = 0; q < kRPL; ++q) {
                            if (cv[q] > Bound) {
                                cmp_v[pos] = cv[q];
                                cmp_i[pos] = ci[q];
                                cmp_x[pos] = cx[q];
                                cmp_y[pos] = cy[q];
                                cmp_z[pos] = cz[q];
                                ++pos;
                            }
                        }
                        // same wave wrote and reads: LDS keeps program order
                        bool live = lane < total;
                        uint32_t v1 = live ? cmp_v[lane] : 0u;
                        int i1 = live ? cmp_i[lane] : 0x7fffffff;
                        float x1 = live ? cmp_x[lane] : 0.f;
                        float y1 = live ? cmp_y[lane] : 0.f;
                        float z1 = live ? cmp_z[lane] : 0.f;
                        while (true) {
                            v1 = f2u(fminf(u2f(v1), sqdist(x1, y1, z1, px, py, pz)));
                            V = wave_max_u32(v1);
                            if (!(V > Bound)) break;
                            pl = first_lane(v1 == V);  // lowest lane = lowest workgroup
                            px = readlane_f(x1, pl);
                            py = readlane_f(y1, pl);
                            pz = readlane_f(z1, pl);
                            emit(cnt, readlane_i(i1, pl), V, px, py, pz);
                            if (++cnt >= cap) break;
                        }
                    } else {
                        while (true) {  // more than 64 live candidates: keep all four per lane
#pragma unroll
                            for (int q = 0; q < kRPL; ++q)
                                cv[q] = f2u(fminf(u2f(cv[q]), sqdist(cx[q], cy[q], cz[q], px, py, pz)));
                            bv = cv[0];
                            bq = 0;
#pragma unroll
                            for (int q = 1; q < kRPL; ++q)
                                if (cv[q] > bv) {
                                    bv = cv[q];
                                    bq = q;
                                }
                            V = wave_max_u32(bv);
                            if (!(V > Bound)) break;
                            pl = first_lane(bv == V);
                            pq = readlane_i(bq, pl);
                            px = pick_elem<kRPL>(cx, pq, pl);
                            py = pick_elem<kRPL>(cy, pq, pl);
                            pz = pick_elem<kRPL>(cz, pq, pl);
                            pidx = 0;
#pragma unroll
                            for (int q = 0; q < kRPL; ++q)
                                if (pq == q) pidx = readlane_i(ci[q], pl);
                            emit(cnt, pidx, V, px, py, pz);
                            if (++cnt >= cap) break;
                        }
                    }
                }
                if (lane == 0) s_cnt = cnt;
            }
            FFPS_STAMP(4);
        }
        __syncthreads();  // picks of this round visible to all waves
        if (s_abort) return;
        npicked += s_cnt;
    }
    if (w == 0 && tid == 0) a.status[1] = (int)round;  // exchange rounds this launch took
#ifdef FFPS_PROFILE
    if (w == 0 && tid == 0)
        for (int i = 0; i < 8; ++i) a.status[8 + i] = (int)prof_acc[i];
#endif
}

template <int NT, int P>
hipError_t launch_t(GridArgs &a, int G, hipStream_t s) {
    void *params[] = {&a};
    return hipLaunchCooperativeKernel((const void *)k_fps_grid<NT, P>, dim3(G), dim3(NT), params,
                                      0, s);
}

}  // namespace

size_t grid_exchange_bytes() { return 2 * kBufBytes; }

long grid_capacity(int num_cu) {
    int G = num_cu < kMaxGridWG ? num_cu : kMaxGridWG;
    return (long)G * 1024 * 16;
}

hipError_t launch_fps_grid(const float *xyz, int N, int M, int start, int32_t *idx, float *md,
                           void *exchange, int *status, int num_cu, int max_picks,
                           hipStream_t s) {
    int maxG = num_cu < kMaxGridWG ? num_cu : kMaxGridWG;
    // at least 128 points per workgroup before another CU is worth a record
    int G = (N + 127) / 128;
    if (G > maxG) G = maxG;
    if (G < 1) G = 1;
    GridArgs a;
    a.xyz = xyz; a.N = N; a.M = M; a.start = start;
    a.chunk = (N + G - 1) / G;
    a.idx_out = idx; a.md_out = md;
    a.exchange = (char *)exchange; a.status = status;
    a.max_picks = max_picks < 1 ? 1 : (max_picks > kMaxPicksPerRound ? kMaxPicksPerRound : max_picks);
#define FFPS_GRID_CASE(NT, P) \
    if (a.chunk <= (NT) * (P)) return launch_t<NT, P>(a, G, s);
    FFPS_GRID_CASE(256, 1)
    FFPS_GRID_CASE(256, 2)
    FFPS_GRID_CASE(256, 3)
    FFPS_GRID_CASE(256, 4)
    FFPS_GRID_CASE(256, 5)
    FFPS_GRID_CASE(256, 6)
    FFPS_GRID_CASE(256, 8)
    FFPS_GRID_CASE(512, 6)
    FFPS_GRID_CASE(512, 8)
    FFPS_GRID_CASE(1024, 6)
    FFPS_GRID_CASE(1024, 8)
    FFPS_GRID_CASE(1024, 12)
    FFPS_GRID_CASE(1024, 16)
#undef FFPS_GRID_CASE
    return hipErrorInvalidValue;
}

}  // namespace ffps
