// k_fps_grid: exact FPS (Sec. 3.1, Eq. 1) of ONE cloud spread over all CUs.
//
// Each of G co-resident workgroups keeps a contiguous slice of the cloud and
// its running minimum distances in registers for the whole call.  A workgroup
// is one COMMUNICATION wave (wave 0) plus NWK WORKER waves that own the points.
// Waves i and i+4 of a workgroup share a SIMD, so waves 4, 8 and 12 exit at
// once: the communication wave, whose dependent chain sets the pace, then has
// its SIMD to itself and the workers fill the other three.
// Workgroups meet once per ROUND, and a round can deliver many picks:
//
//   1. the workers apply the picks of the previous round to their points (they
//      take them from LDS one by one while the communication wave is still
//      producing them), then reduce their slice to its two best points and an
//      upper bound on every other point (the third-best value);
//   2. the communication wave publishes {v_a, v_b, bound | xyz_a | xyz_b} as
//      three 16-byte chunks, each closed by a checksum that also encodes the
//      round, and gathers the chunks of all G workgroups with coalesced
//      device-scope loads.  This all-gather is the only cross-workgroup step:
//      no counters, no fences, no separate barrier;
//   3. it then replays the greedy rule on the 2G published candidates only:
//      the best candidate is the next pick of Eq. 1 as long as its value is
//      strictly above B = max of all bounds, because no unpublished point can
//      then reach it; picking it lowers the other candidates' values by the
//      same distance rule, and the replay continues until the test fails.
//      The first pick of a round never needs the test: the global best point
//      is the best of its own slice, hence published.
//
// Ties.  Slices are in index order and a workgroup lists its two candidates in
// index order, so "lowest position among equal values" is "lowest index".
//
// Every workgroup replays the same deterministic arithmetic on the same
// records, so all agree on the picks without further communication, and the
// picks are exactly those of the one-pick-per-pass loop.  The workgroup that
// owns a pick writes its index to the output.
//
// Exit: every wait is bounded or ends when the communication wave says so; a
// workgroup that gives up sets the status word and leaves, and the others then
// run into their own bound.
#include "fps_device.h"
#include "fps_launch.h"

namespace ffps {

namespace {

constexpr int kRPL = kMaxGridWG / kWave;  // workgroup records per lane of the gathering wave
constexpr int kCPL = 2 * kRPL;            // candidates per lane before compaction
constexpr int kSpinLimit = 1 << 19;

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// Exchange area: two buffers (round parity); each holds three chunk arrays
// (A: {v_a, v_b, bound, check}, B: {x_a, y_a, z_a, check}, C: {x_b, y_b, z_b,
// check}) of 256 slots x 16 bytes.  Workgroup w uses slot (w & 3) * 64 + (w >> 2),
// so that a wave reading slot q*64 + lane with one 16-byte load per lane touches
// one contiguous KiB, while lane L still ends up with workgroups 4L .. 4L+3.
constexpr size_t kChunkBytes = (size_t)kMaxGridWG * 16;
constexpr size_t kBufBytes = 3 * kChunkBytes;
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
// ra/rb/rc[q] = 16 bytes at pa/pb/pc + q * 1024, q < 4: all twelve loads are
// issued before the single wait, so a poll costs one round trip.
__device__ __forceinline__ void load_chunks3(const void *pa, const void *pb, const void *pc,
                                             u32x4 (&ra)[kRPL], u32x4 (&rb)[kRPL],
                                             u32x4 (&rc)[kRPL]) {
    static_assert(kRPL == 4, "four slots per lane");
    asm volatile(
        "global_load_dwordx4 %0, %12, off sc1\n\t"
        "global_load_dwordx4 %1, %12, off offset:1024 sc1\n\t"
        "global_load_dwordx4 %2, %12, off offset:2048 sc1\n\t"
        "global_load_dwordx4 %3, %12, off offset:3072 sc1\n\t"
        "global_load_dwordx4 %4, %13, off sc1\n\t"
        "global_load_dwordx4 %5, %13, off offset:1024 sc1\n\t"
        "global_load_dwordx4 %6, %13, off offset:2048 sc1\n\t"
        "global_load_dwordx4 %7, %13, off offset:3072 sc1\n\t"
        "global_load_dwordx4 %8, %14, off sc1\n\t"
        "global_load_dwordx4 %9, %14, off offset:1024 sc1\n\t"
        "global_load_dwordx4 %10, %14, off offset:2048 sc1\n\t"
        "global_load_dwordx4 %11, %14, off offset:3072 sc1\n\t"
        "s_waitcnt vmcnt(0)"
        : "=&v"(ra[0]), "=&v"(ra[1]), "=&v"(ra[2]), "=&v"(ra[3]), "=&v"(rb[0]), "=&v"(rb[1]),
          "=&v"(rb[2]), "=&v"(rb[3]), "=&v"(rc[0]), "=&v"(rc[1]), "=&v"(rc[2]), "=&v"(rc[3])
        : "v"(pa), "v"(pb), "v"(pc)
        : "memory");
}

// 16-byte LDS accesses as single instructions (a compiler-generated access of
// a 16-byte vector may be split, which would let a reader see half of a slot).
__device__ __forceinline__ uint32_t lds_offset(const void *p) { return (uint32_t)(uintptr_t)p; }
__device__ __forceinline__ void lds_write16(uint32_t off, u32x4 v) {
    asm volatile("ds_write_b128 %0, %1" : : "v"(off), "v"(v) : "memory");
}
__device__ __forceinline__ u32x4 lds_read16(uint32_t off) {
    u32x4 r;
    asm volatile("ds_read_b128 %0, %1\n\ts_waitcnt lgkmcnt(0)" : "=v"(r) : "v"(off) : "memory");
    return r;
}

// Coordinates of element `sel` of lane `lane` (both wave-uniform) of three
// register arrays: a scalar jump picks the element, then three lane reads.
template <int P>
__device__ __forceinline__ void pick_xyz(const float (&x)[P], const float (&y)[P],
                                         const float (&z)[P], int sel, int lane, float &ox,
                                         float &oy, float &oz) {
    ox = oy = oz = 0.f;
#pragma unroll
    for (int j = 0; j < P; ++j) {
        if (sel == j) {
            ox = readlane_f(x[j], lane);
            oy = readlane_f(y[j], lane);
            oz = readlane_f(z[j], lane);
        }
    }
}

struct WaveTop {  // a worker wave's two best points and the bound on its others
    uint32_t v1, v2, v3;
    int i1, i2;
    float x1, y1, z1, x2, y2, z2;
    uint32_t pad;
};

// One pick handed from the communication wave to the workers is a single
// 16-byte LDS word {x, y, z, seq}: written and read by one instruction each, so
// a reader that sees the expected seq also sees its coordinates.

struct GridArgs {
    const float *xyz;
    int N, M, start;
    int chunk;  // points per workgroup
    int32_t *idx_out;
    float *md_out;
    char *exchange;  // two buffers of kBufBytes
    int *status;
    int max_picks;
};

// Phase timing of workgroup 0's communication wave (100 MHz wall clock),
// compiled in only for profiling builds: status[8 + i] accumulates phase i,
// status[15] the polls.
#ifdef FFPS_PROFILE
#define FFPS_STAMP(i)                                    \
    do {                                                 \
        if (w == 0 && tid == 0) {                        \
            uint64_t now_ = wall_clock64();              \
            prof_acc[i] += (uint32_t)(now_ - prof_last); \
            prof_last = now_;                            \
        }                                                \
    } while (0)
#else
#define FFPS_STAMP(i) \
    do {              \
    } while (0)
#endif

// Largest of up to 16 values held by lanes 0..15 (other lanes pass 0), wave-uniform.
__device__ __forceinline__ uint32_t row_max_uniform(uint32_t v) {
    return (uint32_t)readlane_i((int)row16_max_u32(v), 15);
}

// Number of waves a workgroup with NWK worker waves launches: wave 0
// communicates, waves 4, 8, 12 exit at once, the rest work.
__host__ __device__ constexpr int grid_waves(int nwk) { return nwk + nwk / 3; }

template <int NWK, int P>
__global__ __launch_bounds__(kWave *grid_waves(NWK)) void k_fps_grid(GridArgs a) {
    static_assert(NWK % 3 == 0 && NWK >= 3 && NWK <= 12, "worker waves come in threes");
    __shared__ WaveTop wtop[NWK];
    __shared__ __attribute__((aligned(16))) u32x4 pk[kMaxPicksPerRound];
    __shared__ int pk_id[kMaxPicksPerRound];        // candidate number of each pick of the round
    __shared__ uint32_t pk_val[kMaxPicksPerRound];  // and the value it was picked with
    __shared__ int fin[2];  // {batch id, picks emitted in total once that batch is complete}
    __shared__ int s_abort;
    __shared__ uint32_t cmp_v[2 * kWave];
    __shared__ int cmp_id[2 * kWave];
    __shared__ float cmp_x[2 * kWave], cmp_y[2 * kWave], cmp_z[2 * kWave];

    const int G = gridDim.x;
    const int w = blockIdx.x;
    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1);
    const int wave = tid / kWave;
    if (wave != 0 && (wave & 3) == 0) return;  // leaves the communication wave's SIMD to it

    const int lo = w * a.chunk;
    const int hi = min(a.N, lo + a.chunk);
    const uint32_t pk_off = lds_offset(pk);
    volatile int *vfin = fin;

    if (wave == 0) {
        // batch 0 is the seed point alone; other slots start with an impossible seq
        u32x4 s;
        s.x = f2u(a.xyz[3 * (size_t)a.start + 0]);
        s.y = f2u(a.xyz[3 * (size_t)a.start + 1]);
        s.z = f2u(a.xyz[3 * (size_t)a.start + 2]);
        s.w = lane == 0 ? 0u : 0xffffffffu;
        lds_write16(pk_off + lane * 16, s);
        if (lane == 0) {
            vfin[1] = 1;
            vfin[0] = 0;
            s_abort = 0;
            if (w == 0) {
                a.idx_out[0] = a.start;
                if (a.md_out) a.md_out[0] = __builtin_inff();
            }
        }
    }
    __syncthreads();

    if (wave != 0) {
        // =============================== worker ===============================
        const int wk = wave - 1 - wave / 4;  // 0 .. NWK-1
        const int first = lo + (wk * kWave + lane) * P;
        float x[P], y[P], z[P], m[P];
#pragma unroll
        for (int j = 0; j < P; ++j) {
            int i = first + j;
            bool ok = i < hi;
            x[j] = ok ? a.xyz[3 * (size_t)i + 0] : 0.f;
            y[j] = ok ? a.xyz[3 * (size_t)i + 1] : 0.f;
            z[j] = ok ? a.xyz[3 * (size_t)i + 2] : 0.f;
            m[j] = ok ? __builtin_inff() : 0.f;  // padding: value 0, never preferred
        }
        int applied = 0;  // picks applied so far = sequence number of the next pick
        for (int batch = 0;; ++batch) {
            // ---- 1a. take this batch's picks from LDS as they appear ----
            const int batch_base = applied;
            while (true) {
                const int pos = min(applied - batch_base, kMaxPicksPerRound - 1);
                const u32x4 slot = lds_read16(pk_off + pos * 16);
                if ((int)slot.w == applied) {
                    const float lx = u2f(slot.x), ly = u2f(slot.y), lz = u2f(slot.z);
                    ++applied;
#pragma unroll
                    for (int j = 0; j < P; ++j)
                        m[j] = fminf(m[j], sqdist(x[j], y[j], z[j], lx, ly, lz));
                } else {
                    int fb = vfin[0];  // batch id first, then the total it vouches for
                    int ft = vfin[1];
                    if (fb == batch && applied >= ft) break;
                    __builtin_amdgcn_s_sleep(1);
                }
            }
            if (s_abort || applied >= a.M) break;
            // ---- 1b. per-lane top three values (element numbers for the first two) ----
            float a1 = m[0], a2 = 0.f, a3 = 0.f;
            int j1 = 0, j2 = 0;
#pragma unroll
            for (int j = 1; j < P; ++j) {
                float v = m[j];
                bool g1 = v > a1, g2 = v > a2;  // strict: the earlier (lower) j keeps a tie
                a3 = fmaxf(a3, fminf(v, a2));
                j2 = g1 ? j1 : (g2 ? j : j2);
                a2 = fmaxf(a2, fminf(v, a1));
                j1 = g1 ? j : j1;
                a1 = fmaxf(a1, v);
            }
            // ---- 1c. wave top two + bound ----
            uint32_t W1 = wave_max_u32(f2u(a1));
            int l1 = first_lane(f2u(a1) == W1);
            uint32_t b = lane == l1 ? f2u(a2) : f2u(a1);
            uint32_t W2 = wave_max_u32(b);
            int l2 = first_lane(b == W2);
            uint32_t c = lane == l1 ? (l1 == l2 ? f2u(a3) : f2u(a2)) : (lane == l2 ? f2u(a2) : f2u(a1));
            uint32_t W3 = wave_max_u32(c);
            int e1 = readlane_i(j1, l1);
            int e2 = readlane_i(l1 == l2 ? j2 : j1, l2);
            float x1, y1, z1, x2, y2, z2;
            pick_xyz<P>(x, y, z, e1, l1, x1, y1, z1);
            pick_xyz<P>(x, y, z, e2, l2, x2, y2, z2);
            if (lane == 0) {
                WaveTop &t = wtop[wk];
                t.v1 = W1; t.v2 = W2; t.v3 = W3;
                t.i1 = lo + (wk * kWave + l1) * P + e1;
                t.i2 = lo + (wk * kWave + l2) * P + e2;
                t.x1 = x1; t.y1 = y1; t.z1 = z1;
                t.x2 = x2; t.y2 = y2; t.z2 = z2;
            }
            __syncthreads();  // wave tops ready for the communication wave
        }
        return;
    }

    // ========================== communication wave ==========================
    int npicked = 1;
    uint32_t round = 0;
#ifdef FFPS_PROFILE
    uint32_t prof_acc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    uint32_t prof_loop[4] = {0, 0, 0, 0};  // cycles/16 and picks inside the packed loops
    uint64_t prof_last = wall_clock64();
    const uint64_t prof_w0 = prof_last, prof_c0 = clock64();
#endif
    while (npicked < a.M) {
        ++round;
        FFPS_STAMP(0);
        __syncthreads();  // workers have applied every pick so far and filled wtop
        FFPS_STAMP(1);
        // ---- 2a. workgroup top two + bound from the worker waves' triples ----
        const bool act = lane < NWK;
        const int wl = act ? lane : 0;
        uint32_t t1 = act ? wtop[wl].v1 : 0u;
        uint32_t t2 = act ? wtop[wl].v2 : 0u;
        uint32_t t3 = act ? wtop[wl].v3 : 0u;
        uint32_t G1 = row_max_uniform(t1);
        int w1 = first_lane(act && t1 == G1);
        uint32_t bb = act ? (lane == w1 ? t2 : t1) : 0u;
        uint32_t G2 = row_max_uniform(bb);
        int w2 = first_lane(act && bb == G2);
        uint32_t cc = act ? (lane == w1 ? (w1 == w2 ? t3 : t2) : (lane == w2 ? t2 : t1)) : 0u;
        uint32_t G3 = row_max_uniform(cc);
        // candidate 1 = wave w1's first; candidate 2 = wave w2's first, or w1's second
        int gi1 = wtop[w1].i1;
        float gx1 = wtop[w1].x1, gy1 = wtop[w1].y1, gz1 = wtop[w1].z1;
        const bool same = w1 == w2;
        int gi2 = same ? wtop[w1].i2 : wtop[w2].i1;
        float gx2 = same ? wtop[w1].x2 : wtop[w2].x1;
        float gy2 = same ? wtop[w1].y2 : wtop[w2].y1;
        float gz2 = same ? wtop[w1].z2 : wtop[w2].z1;
        // list the two candidates in index order (see "Ties" above)
        uint32_t va = G1, vb = G2;
        int ia = gi1, ib = gi2;
        float xa = gx1, ya = gy1, za = gz1, xb = gx2, yb = gy2, zb = gz2;
        if (gi2 < gi1) {
            va = G2; vb = G1; ia = gi2; ib = gi1;
            xa = gx2; ya = gy2; za = gz2; xb = gx1; yb = gy1; zb = gz1;
        }
        // ---- 2b. publish ----
        char *buf = a.exchange + (size_t)(round & 1) * kBufBytes;
        if (lane == 0) {
            u32x4 ca, cb4, cc4;
            ca.x = va; ca.y = vb; ca.z = G3;
            ca.w = chunk_check(ca.x, ca.y, ca.z, round, 0);
            cb4.x = f2u(xa); cb4.y = f2u(ya); cb4.z = f2u(za);
            cb4.w = chunk_check(cb4.x, cb4.y, cb4.z, round, 1);
            cc4.x = f2u(xb); cc4.y = f2u(yb); cc4.z = f2u(zb);
            cc4.w = chunk_check(cc4.x, cc4.y, cc4.z, round, 2);
            const size_t so = (size_t)slot_of(w) * 16;
            store_chunk(buf + so, ca);
            store_chunk(buf + kChunkBytes + so, cb4);
            store_chunk(buf + 2 * kChunkBytes + so, cc4);
        }
        FFPS_STAMP(2);
        // ---- 2c. gather: lane L reads slots q*64+L = workgroups 4L+q ----
        u32x4 ra[kRPL], rb[kRPL], rc[kRPL];
        bool gave_up = false;
        for (int spin = 0;; ++spin) {
            load_chunks3(buf + (size_t)lane * 16, buf + kChunkBytes + (size_t)lane * 16,
                         buf + 2 * kChunkBytes + (size_t)lane * 16, ra, rb, rc);
            bool all = true;
#pragma unroll
            for (int q = 0; q < kRPL; ++q) {
                bool ok = ra[q].w == chunk_check(ra[q].x, ra[q].y, ra[q].z, round, 0) &&
                          rb[q].w == chunk_check(rb[q].x, rb[q].y, rb[q].z, round, 1) &&
                          rc[q].w == chunk_check(rc[q].x, rc[q].y, rc[q].z, round, 2);
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
                vfin[1] = 0;
                vfin[0] = (int)round;  // releases the workers, which then see s_abort
            }
            return;
        }
        // candidate c = 2q + r of this lane: workgroup 4*lane + q, its r-th in index order
        uint32_t cv[kCPL], lb = 0u;
        float cx[kCPL], cy[kCPL], cz[kCPL];
#pragma unroll
        for (int q = 0; q < kRPL; ++q) {
            bool present = lane * kRPL + q < G;  // absent records: value 0, bound 0
            cv[2 * q] = present ? ra[q].x : 0u;
            cv[2 * q + 1] = present ? ra[q].y : 0u;
            lb = umax(lb, present ? ra[q].z : 0u);
            cx[2 * q] = u2f(rb[q].x); cy[2 * q] = u2f(rb[q].y); cz[2 * q] = u2f(rb[q].z);
            cx[2 * q + 1] = u2f(rc[q].x); cy[2 * q + 1] = u2f(rc[q].y); cz[2 * q + 1] = u2f(rc[q].z);
        }
        // ---- 3. replay the greedy rule on the published candidates ----
        const uint32_t Bound = wave_max_u32(lb);
        const int cap = __builtin_amdgcn_readfirstlane(min(a.max_picks, a.M - npicked));
        // Hand pick number c of this round to the workers (one 16-byte LDS write) and
        // note which candidate it was; `mine` holds in exactly one lane.
        auto emit = [&](bool mine, int c, int cid, uint32_t vbits, float ex, float ey, float ez) {
            if (mine) {
                u32x4 s;
                s.x = f2u(ex); s.y = f2u(ey); s.z = f2u(ez); s.w = (uint32_t)(npicked + c);
                lds_write16(pk_off + c * 16, s);
                pk_id[c] = cid;
                pk_val[c] = vbits;
            }
        };
        uint32_t bv = cv[0];
        int bq = 0;
#pragma unroll
        for (int q = 1; q < kCPL; ++q)
            if (cv[q] > bv) {
                bv = cv[q];
                bq = q;
            }
        uint32_t V = wave_max_u32(bv);
        int cnt = 0;
        int pl;
        float px, py, pz;
        // Only candidates above the bound can be picked after the first pick, and
        // when the best candidate is above it the first pick is one of them too:
        // compact them, in candidate (= index) order.
        int total = 0, before = 0;
        if (V > Bound && cap > 1) {
            const uint64_t lt = ((uint64_t)1 << lane) - 1;
#pragma unroll
            for (int q = 0; q < kCPL; ++q) {
                uint64_t mk = __builtin_amdgcn_ballot_w64(cv[q] > Bound);
                total += __builtin_popcountll(mk);
                before += __builtin_popcountll(mk & lt);
            }
        }
        // With at most 128 live candidates whose values lie within 2^24 ulps above
        // the bound, value and position fit one 32-bit key
        //   key = (value_bits - bound_bits) << 7 | (127 - position),
        // so a single wave-wide max yields the best value AND, among equal values,
        // the lowest position (= lowest index).  Values at or below the bound
        // saturate to 0 and end the round.
        const bool packed = total >= 1 && total <= 2 * kWave && V - Bound < (1u << 24);
#ifdef FFPS_PROFILE
        if (w == 0 && tid == 0) {
            if (packed) prof_acc[total <= kWave ? 5 : 6] += 1;
        }
#endif
        if (packed) {
            int pos = before;
#pragma unroll
            for (int q = 0; q < kCPL; ++q) {
                if (cv[q] > Bound) {
                    cmp_v[pos] = cv[q];
                    cmp_id[pos] = lane * kCPL + q;
                    cmp_x[pos] = cx[q];
                    cmp_y[pos] = cy[q];
                    cmp_z[pos] = cz[q];
                    ++pos;
                }
            }
            // the same wave wrote and now reads: LDS keeps its accesses in order
            if (total <= kWave) {
                // one candidate per lane: lane L takes position L
                const bool h = lane < total;
                uint32_t v0 = h ? cmp_v[lane] : 0u;
                int id0 = h ? cmp_id[lane] : 0;
                float x0 = h ? cmp_x[lane] : 0.f, y0 = h ? cmp_y[lane] : 0.f,
                      z0 = h ? cmp_z[lane] : 0.f;
                const uint32_t inv = 127u - (uint32_t)lane;
#ifdef FFPS_PROFILE
                const uint64_t lc0 = clock64();
#endif
                while (true) {
                    const uint32_t K = wave_max_u32((__builtin_elementwise_sub_sat(v0, Bound) << 7) | inv);
                    if ((K >> 7) == 0) break;  // cannot happen for the first pick
                    pl = 127 - (int)(K & 127u);
                    px = readlane_f(x0, pl);
                    py = readlane_f(y0, pl);
                    pz = readlane_f(z0, pl);
                    emit(lane == pl, cnt, id0, v0, x0, y0, z0);  // the winning lane hands over its own
                    if (++cnt >= cap) break;
                    v0 = f2u(fminf(u2f(v0), sqdist(x0, y0, z0, px, py, pz)));
                }
#ifdef FFPS_PROFILE
                prof_loop[0] += (uint32_t)(clock64() - lc0);
                prof_loop[1] += cnt;
#endif
            } else {
                // two candidates per lane: lane L takes positions 2L and 2L+1
                const int p0 = 2 * lane, p1 = 2 * lane + 1;
                const bool h0 = p0 < total, h1 = p1 < total;
                uint32_t v0 = h0 ? cmp_v[p0] : 0u, v1 = h1 ? cmp_v[p1] : 0u;
                int id0 = h0 ? cmp_id[p0] : 0, id1 = h1 ? cmp_id[p1] : 0;
                float x0 = h0 ? cmp_x[p0] : 0.f, y0 = h0 ? cmp_y[p0] : 0.f,
                      z0 = h0 ? cmp_z[p0] : 0.f;
                float x1 = h1 ? cmp_x[p1] : 0.f, y1 = h1 ? cmp_y[p1] : 0.f,
                      z1 = h1 ? cmp_z[p1] : 0.f;
                const uint32_t inv0 = 127u - (uint32_t)p0, inv1 = 127u - (uint32_t)p1;
#ifdef FFPS_PROFILE
                const uint64_t lc0 = clock64();
#endif
                while (true) {
                    const uint32_t k0 = (__builtin_elementwise_sub_sat(v0, Bound) << 7) | inv0;
                    const uint32_t k1 = (__builtin_elementwise_sub_sat(v1, Bound) << 7) | inv1;
                    // each lane puts forward the better of its two (keys are distinct)
                    const bool sec = k1 > k0;
                    const float bx = sec ? x1 : x0, by = sec ? y1 : y0, bz = sec ? z1 : z0;
                    const uint32_t K = wave_max_u32(sec ? k1 : k0);
                    if ((K >> 7) == 0) break;
                    pl = (127 - (int)(K & 127u)) >> 1;
                    px = readlane_f(bx, pl);
                    py = readlane_f(by, pl);
                    pz = readlane_f(bz, pl);
                    emit(lane == pl, cnt, sec ? id1 : id0, sec ? v1 : v0, bx, by, bz);
                    if (++cnt >= cap) break;
                    v0 = f2u(fminf(u2f(v0), sqdist(x0, y0, z0, px, py, pz)));
                    v1 = f2u(fminf(u2f(v1), sqdist(x1, y1, z1, px, py, pz)));
                }
#ifdef FFPS_PROFILE
                prof_loop[2] += (uint32_t)(clock64() - lc0);
                prof_loop[3] += cnt;
#endif
            }
        } else {
            // a single pick (best candidate not above the bound, or cap 1), more than
            // 128 live candidates, or values spread too far above the bound for the
            // packed key: work on all eight candidates per lane
            while (true) {
                if (cnt > 0) {
                    bv = cv[0];
                    bq = 0;
#pragma unroll
                    for (int q = 1; q < kCPL; ++q)
                        if (cv[q] > bv) {
                            bv = cv[q];
                            bq = q;
                        }
                    V = wave_max_u32(bv);
                    if (!(V > Bound)) break;
                }
                pl = first_lane(bv == V);
                int pq = readlane_i(bq, pl);
                pick_xyz<kCPL>(cx, cy, cz, pq, pl, px, py, pz);
                emit(lane == 0, cnt, pl * kCPL + pq, V, px, py, pz);
                if (++cnt >= cap) break;
#pragma unroll
                for (int q = 0; q < kCPL; ++q)
                    cv[q] = f2u(fminf(u2f(cv[q]), sqdist(cx[q], cy[q], cz[q], px, py, pz)));
            }
        }
        // the workgroup that owns a pick records it (same wave wrote pk_id / pk_val)
        if (lane < cnt) {
            const int cid = pk_id[lane];
            if ((cid >> 1) == w) {
                a.idx_out[npicked + lane] = (cid & 1) ? ib : ia;
                if (a.md_out) a.md_out[npicked + lane] = u2f(pk_val[lane]);
            }
        }
        npicked += cnt;
        if (lane == 0) {
            vfin[1] = npicked;  // total first, then the batch id that vouches for it
            vfin[0] = (int)round;
        }
        FFPS_STAMP(4);
    }
    if (w == 0 && lane == 0) {
        a.status[1] = (int)round;  // exchange rounds this launch took
#ifdef FFPS_PROFILE
        for (int i = 0; i < 8; ++i) a.status[8 + i] = (int)prof_acc[i];
        for (int i = 0; i < 4; ++i) a.status[20 + i] = (int)prof_loop[i];
        a.status[16] = (int)(wall_clock64() - prof_w0);       // 10 ns units
        a.status[17] = (int)((clock64() - prof_c0) >> 4);     // shader cycles / 16
#endif
    }
}

template <int NWK, int P>
hipError_t launch_t(GridArgs &a, int G, hipStream_t s) {
    void *params[] = {&a};
    return hipLaunchCooperativeKernel((const void *)k_fps_grid<NWK, P>, dim3(G),
                                      dim3(kWave * grid_waves(NWK)), params, 0, s);
}

}  // namespace

size_t grid_exchange_bytes() { return 2 * kBufBytes; }

long grid_capacity(int num_cu) {
    int G = num_cu < kMaxGridWG ? num_cu : kMaxGridWG;
    return (long)G * 12 * kWave * 16;
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
#define FFPS_GRID_CASE(NWK, P) \
    if (a.chunk <= (NWK) * kWave * (P)) return launch_t<NWK, P>(a, G, s);
    FFPS_GRID_CASE(3, 1)
    FFPS_GRID_CASE(3, 2)
    FFPS_GRID_CASE(3, 3)
    FFPS_GRID_CASE(3, 4)
    FFPS_GRID_CASE(3, 5)
    FFPS_GRID_CASE(3, 6)
    FFPS_GRID_CASE(3, 7)
    FFPS_GRID_CASE(3, 8)
    FFPS_GRID_CASE(6, 6)
    FFPS_GRID_CASE(6, 8)
    FFPS_GRID_CASE(12, 6)
    FFPS_GRID_CASE(12, 8)
    FFPS_GRID_CASE(12, 12)
    FFPS_GRID_CASE(12, 16)
#undef FFPS_GRID_CASE
    return hipErrorInvalidValue;
}

}  // namespace ffps
