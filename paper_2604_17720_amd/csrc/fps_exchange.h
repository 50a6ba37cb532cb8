// Cross-workgroup exchange and candidate replay shared by the multi-workgroup
// FPS kernels (register-resident and HBM-streaming).
//
// Once per ROUND every workgroup contributes its two best points (listed in
// index order) and an upper bound on all its other points.  One wave per
// workgroup publishes them as three 16-byte chunks, each closed by a checksum
// that also encodes the round, gathers the chunks of all G workgroups with
// coalesced device-scope loads (the only cross-workgroup step: no counters, no
// fences, no separate barrier), and replays the greedy rule of Eq. 1 on the 2G
// published candidates: the best candidate is the next pick as long as its
// value is strictly above B = max of all bounds, because no unpublished point
// can then reach it; picking it lowers the other candidates' values by the same
// distance rule, and the replay continues until the test fails.  The first pick
// of a round never needs the test: the global best point is the best of its own
// slice, hence published.  Every workgroup replays the same arithmetic on the
// same records, so all agree on the picks without further communication.
//
// Ties.  Slices are in index order and a workgroup lists its two candidates in
// index order, so "lowest position among equal values" is "lowest index".
#pragma once
#include "fps_device.h"
#include "fps_launch.h"

namespace ffps {

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


// What a workgroup contributes to a round: candidates a, b in index order
// (ia < ib) with their current values, and the bound on its other points.
struct RoundInput {
    uint32_t va, vb, bound;
    float xa, ya, za, xb, yb, zb;
    int ia, ib;
};

// LDS used by the wave that runs exchange_round.
struct RoundLds {
    __attribute__((aligned(16))) u32x4 pk[kMaxPicksPerRound];  // picks of the round: {x, y, z, seq}
    int pk_id[kMaxPicksPerRound];        // candidate number of each pick of the round
    uint32_t pk_val[kMaxPicksPerRound];  // and the value it was picked with
    uint32_t cmp_v[2 * kWave];           // compacted live candidates
    int cmp_id[2 * kWave];
    float cmp_x[2 * kWave], cmp_y[2 * kWave], cmp_z[2 * kWave];
};

// Counters of a profiling build (workgroup 0 only).
struct RoundProf {
    uint32_t acc[8];   // 100 MHz ticks per phase; [5], [6]: rounds on the packed paths; [7]: polls
    uint32_t loop[4];  // shader cycles and picks inside the two packed loops
    uint64_t last;
};
#ifdef FFPS_PROFILE
#define FFPS_STAMP(P, i)                                        \
    do {                                                        \
        if ((P) != nullptr) {                                   \
            uint64_t now_ = wall_clock64();                     \
            (P)->acc[i] += (uint32_t)(now_ - (P)->last);        \
            (P)->last = now_;                                   \
        }                                                       \
    } while (0)
#else
#define FFPS_STAMP(P, i) \
    do {                 \
    } while (0)
#endif

// One round, run by ONE full wave of workgroup w.  Publishes `in`, gathers all
// G records, replays, writes each pick as {x, y, z, npicked + c} to L.pk[c]
// (16-byte LDS writes, in pick order, so other waves may consume them while
// the replay is still running) and records the picks this workgroup owns in
// idx_out / md_out.  Returns the number of picks of the round (1 .. cap), or -1
// after setting *status when another workgroup's record never arrived.
__device__ __forceinline__ int exchange_round(RoundLds &L, char *exchange, int G, int w, int lane,
                                              uint32_t round, const RoundInput &in, int npicked,
                                              int cap, int32_t *idx_out, float *md_out, int *status,
                                              RoundProf *prof) {
    const uint32_t pk_off = lds_offset(L.pk);
    uint32_t *cmp_v = L.cmp_v;
    int *cmp_id = L.cmp_id;
    float *cmp_x = L.cmp_x, *cmp_y = L.cmp_y, *cmp_z = L.cmp_z;
    int *pk_id = L.pk_id;
    uint32_t *pk_val = L.pk_val;
    const uint32_t va = in.va, vb = in.vb, G3 = in.bound;
    const float xa = in.xa, ya = in.ya, za = in.za, xb = in.xb, yb = in.yb, zb = in.zb;
    const int ia = in.ia, ib = in.ib;
    // ---- 2b. publish ----
    char *buf = exchange + (size_t)(round & 1) * kBufBytes;
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
    FFPS_STAMP(prof, 2);
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
        if (prof) ++prof->acc[7];
#endif
        if (__builtin_amdgcn_ballot_w64(!all) == 0) break;
        if (spin >= kSpinLimit) {
            gave_up = true;
            break;
        }
    }
    FFPS_STAMP(prof, 3);
    if (gave_up) {
        if (lane == 0) __hip_atomic_store(status, -5, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        return -1;
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
    if (prof && packed) prof->acc[total <= kWave ? 5 : 6] += 1;
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
            if (prof) {
                prof->loop[0] += (uint32_t)(clock64() - lc0);
                prof->loop[1] += cnt;
            }
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
            if (prof) {
                prof->loop[2] += (uint32_t)(clock64() - lc0);
                prof->loop[3] += cnt;
            }
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
            idx_out[npicked + lane] = (cid & 1) ? ib : ia;
            if (md_out) md_out[npicked + lane] = u2f(pk_val[lane]);
        }
    }
    return cnt;
}

}  // namespace ffps
