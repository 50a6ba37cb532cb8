// k_fps_grid: exact FPS (Sec. 3.1, Eq. 1) of ONE cloud spread over all CUs.
//
// Each of G co-resident workgroups keeps a contiguous slice of the cloud and
// its running minimum distances in registers for the whole call.  Workgroups
// meet once per ROUND, and a round can deliver several picks:
//
//   1. every workgroup applies the picks of the previous round to its points
//      and finds its best point (value, lowest index) and an upper bound on
//      all its OTHER points (its second-best value);
//   2. it publishes {best value, index, x, y, z, bound} as six self-tagged
//      64-bit words; one wave per workgroup gathers all G records (this
//      all-gather is the only cross-workgroup step: no counters, no fences,
//      no separate barrier);
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
    uint64_t *exchange;  // [2][G][kRecWords]
    int *status;
    int max_picks;
};

template <int NT, int P>
__global__ __launch_bounds__(NT) void k_fps_grid(GridArgs a) {
    constexpr int NW = NT / kWave;
    __shared__ WaveTop wtop[NW];
    __shared__ float pkx[kMaxPicksPerRound], pky[kMaxPicksPerRound], pkz[kMaxPicksPerRound];
    __shared__ int s_cnt, s_abort;

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
    while (npicked < a.M) {
        ++round;
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
        __syncthreads();  // wave tops visible; everyone is done with pk*/s_cnt

        if (wave == 0) {
            // ---- 2a. workgroup best and bound ----
            uint32_t s1 = lane < NW ? wtop[lane].m1 : 0u;
            uint32_t G1 = (uint32_t)readlane_i((int)row16_max_u32(s1), 15);
            int ww = first_lane(lane < NW && s1 == G1);
            uint32_t s2 = lane < NW ? (lane == ww ? wtop[lane].m2 : s1) : 0u;
            uint32_t Bw = (uint32_t)readlane_i((int)row16_max_u32(s2), 15);
            // ---- 2b. publish ----
            uint64_t *mine = a.exchange + ((size_t)(round & 1) * G + w) * kRecWords;
            if (lane == 0) {
                store_word(mine + 0, G1, round);
                store_word(mine + 1, (uint32_t)wtop[ww].idx, round);
                store_word(mine + 2, f2u(wtop[ww].x), round);
                store_word(mine + 3, f2u(wtop[ww].y), round);
                store_word(mine + 4, f2u(wtop[ww].z), round);
                store_word(mine + 5, Bw, round);
            }
            // ---- 2c. gather all G records (lane L owns records L*kRPL .. +kRPL) ----
            uint32_t cv[kRPL], cb[kRPL];
            int ci[kRPL];
            float cx[kRPL], cy[kRPL], cz[kRPL];
            bool have[kRPL];
#pragma unroll
            for (int q = 0; q < kRPL; ++q) {
                int r = lane * kRPL + q;
                have[q] = r >= G;  // absent records: value 0, bound 0
                cv[q] = 0u; cb[q] = 0u; ci[q] = 0x7fffffff;
                cx[q] = cy[q] = cz[q] = 0.f;
            }
            const uint64_t *rb = a.exchange + (size_t)(round & 1) * G * kRecWords;
            bool gave_up = false;
            for (int spin = 0;; ++spin) {
                // all loads of a poll are issued before any is examined; lanes
                // past the last record re-read record G-1 and ignore it
                uint64_t wd[kRPL][6];
#pragma unroll
                for (int q = 0; q < kRPL; ++q) {
                    const uint64_t *rp = rb + (size_t)min(lane * kRPL + q, G - 1) * kRecWords;
#pragma unroll
                    for (int t = 0; t < 6; ++t) wd[q][t] = load_word(rp + t);
                }
                bool all = true;
#pragma unroll
                for (int q = 0; q < kRPL; ++q) {
                    bool ok = true;
#pragma unroll
                    for (int t = 0; t < 6; ++t) ok = ok && (uint32_t)(wd[q][t] >> 32) == round;
                    if (!have[q] && ok) {
                        cv[q] = (uint32_t)wd[q][0];
                        ci[q] = (int)(uint32_t)wd[q][1];
                        cx[q] = u2f((uint32_t)wd[q][2]);
                        cy[q] = u2f((uint32_t)wd[q][3]);
                        cz[q] = u2f((uint32_t)wd[q][4]);
                        cb[q] = (uint32_t)wd[q][5];
                        have[q] = true;
                    }
                    all = all && have[q];
                }
                if (__builtin_amdgcn_ballot_w64(!all) == 0) break;
                if (spin >= kSpinLimit) {
                    gave_up = true;
                    break;
                }
                __builtin_amdgcn_s_sleep(1);
            }
            if (gave_up) {
                if (lane == 0) {
                    __hip_atomic_store(a.status, -5, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    s_abort = 1;
                    s_cnt = 0;
                }
            } else {
                // ---- 3. replay the greedy rule on the published candidates ----
                uint32_t lb = cb[0];
#pragma unroll
                for (int q = 1; q < kRPL; ++q) lb = umax(lb, cb[q]);
                const uint32_t Bound = wave_max_u32(lb);
                int cnt = 0;
                while (true) {
                    uint32_t bv = cv[0];
                    int bq = 0;
#pragma unroll
                    for (int q = 1; q < kRPL; ++q)
                        if (cv[q] > bv) {
                            bv = cv[q];
                            bq = q;
                        }
                    uint32_t V = wave_max_u32(bv);
                    if (cnt > 0 && !(V > Bound)) break;
                    int pl = first_lane(bv == V);
                    int pq = readlane_i(bq, pl);
                    float px = pick_elem<kRPL>(cx, pq, pl);
                    float py = pick_elem<kRPL>(cy, pq, pl);
                    float pz = pick_elem<kRPL>(cz, pq, pl);
                    int pidx = 0;
#pragma unroll
                    for (int q = 0; q < kRPL; ++q)
                        if (pq == q) pidx = readlane_i(ci[q], pl);
                    if (lane == 0) {
                        pkx[cnt] = px;
                        pky[cnt] = py;
                        pkz[cnt] = pz;
                        if (w == 0) {
                            a.idx_out[npicked + cnt] = pidx;
                            if (a.md_out) a.md_out[npicked + cnt] = u2f(V);
                        }
                    }
                    ++cnt;
                    if (npicked + cnt >= a.M || cnt >= a.max_picks) break;
#pragma unroll
                    for (int q = 0; q < kRPL; ++q)
                        cv[q] = f2u(fminf(u2f(cv[q]), sqdist(cx[q], cy[q], cz[q], px, py, pz)));
                }
                if (lane == 0) s_cnt = cnt;
            }
        }
        __syncthreads();  // picks of this round visible to all waves
        if (s_abort) return;
        npicked += s_cnt;
    }
}

template <int NT, int P>
hipError_t launch_t(GridArgs &a, int G, hipStream_t s) {
    void *params[] = {&a};
    return hipLaunchCooperativeKernel((const void *)k_fps_grid<NT, P>, dim3(G), dim3(NT), params,
                                      0, s);
}

}  // namespace

size_t grid_exchange_bytes() { return (size_t)2 * kMaxGridWG * kRecWords * sizeof(uint64_t); }

long grid_capacity(int num_cu) {
    int G = num_cu < kMaxGridWG ? num_cu : kMaxGridWG;
    return (long)G * 1024 * 16;
}

hipError_t launch_fps_grid(const float *xyz, int N, int M, int start, int32_t *idx, float *md,
                           uint64_t *exchange, int *status, int num_cu, int max_picks,
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
    a.exchange = exchange; a.status = status;
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
