// Cross-workgroup exchange and candidate replay shared by the multi-workgroup
// FPS kernels (register-resident and HBM-streaming).
//
// The points of a cloud are divided among U <= 256 reporting UNITS (a whole
// workgroup, or each worker wave of a workgroup).  Once per ROUND every unit
// contributes its two best points and an upper bound on all its other points
// (its third-best value).  One wave per workgroup publishes the records of its
// units as four 16-byte chunks each, every chunk closed by a checksum that also
// encodes the round, gathers the chunks of all U units with coalesced
// device-scope loads (the only cross-workgroup step: no counters, no fences, no
// separate barrier), and replays the greedy rule of Eq. 1 on the 2U published
// candidates: the best candidate is the next pick as long as its value is
// strictly above B = max of all bounds, because no unpublished point can then
// reach it; picking it lowers the other candidates' values by the same distance
// rule, and the replay continues until the test fails.  The first pick of a
// round never needs the test: the global best point (largest value, lowest
// index among equals) is the best of its own unit, hence published.
// Every workgroup replays the same arithmetic on the same records, so all agree
// on the picks without further communication.
//
// "Best" always means largest value, then lowest point index.  Points may be
// assigned to units in any way; candidates carry their indices, and equal
// values are detected and resolved on the index wherever they can occur.
#pragma once
#include "fps_device.h"
#include "fps_launch.h"

namespace ffps {

constexpr int kMaxUnits = kMaxGridWG;     // reporting units of a cloud
constexpr int kRPL = kMaxUnits / kWave;   // unit records per lane of the gathering wave
constexpr int kSpinLimit = 1 << 19;
constexpr uint32_t kNoIndex = 0x7fffffffu;  // index of a candidate that does not exist

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

// Exchange area: two buffers (round parity); each holds one array of 256 slots
// x 16 bytes per chunk of a record.  A record of T candidates is, in chunks of
// three words plus a check word,
//   T = 2: {v0, v1, bound} {x0, y0, z0} {x1, y1, z1} {i0, i1, 0}
//   T = 3: {v0, v1, v2} {x0, y0, z0} {x1, y1, z1} {x2, y2, z2} {i0, i1, i2} {bound, 0, 0}.
// Unit u uses slot u, and lane L of a gathering wave reads slots L, L + 64,
// L + 128, L + 192: each 16-byte load per lane touches one contiguous KiB, and
// units with consecutive numbers, which hold consecutive point indices, land in
// different lanes.
__host__ __device__ constexpr int chunks_of(int T) { return T == 2 ? 4 : 6; }
constexpr size_t kChunkBytes = (size_t)kMaxUnits * 16;
__host__ __device__ constexpr size_t buf_bytes(int T) { return chunks_of(T) * kChunkBytes; }

// A chunk is valid for a round when its last word equals this value.  Memory
// cleared to zero never validates (the round term is non-zero for round >= 1),
// a chunk of round-2 in the same buffer does not validate, and a read that
// mixed old and new words fails the test and is simply polled again.
__device__ __forceinline__ uint32_t chunk_check(uint32_t a, uint32_t b, uint32_t c, uint32_t round,
                                                uint32_t which) {
    uint32_t m = a ^ ((b << 11) | (b >> 21)) ^ ((c << 22) | (c >> 10));
    return m ^ (round * 0x9E3779B1u + which * 0x85EBCA6Bu);
}
__device__ __forceinline__ bool chunk_ok(const u32x4 &c, uint32_t round, uint32_t which) {
    return c.w == chunk_check(c.x, c.y, c.z, round, which);
}

// Device-scope (all XCDs) 16-byte store and loads.  The compiler offers atomics
// up to 8 bytes only, so these are spelled out; sc1 is the device-scope cache
// policy the compiler itself uses for agent-scope atomics on this target.
// A vector-memory store of more than 8 bytes reads its data registers a few
// cycles after it issues, and a vector instruction that overwrites them right
// behind it changes what is stored.  The compiler keeps the distance for its
// own stores but cannot see into this text, hence the two idle cycles.
__device__ __forceinline__ void store_chunk(void *p, u32x4 v) {
    asm volatile("global_store_dwordx4 %0, %1, off sc1\n\ts_nop 1" : : "v"(p), "v"(v) : "memory");
}
// r[c][q] = 16 bytes at p + c * kChunkBytes + q * 1024, q < 4: all loads are
// issued before the single wait, so a poll costs one round trip.
__device__ __forceinline__ void load_chunks(const char *p, u32x4 (&r)[4][kRPL]) {
    static_assert(kRPL == 4, "four slots per lane");
    const char *pa = p, *pb = p + kChunkBytes, *pc = p + 2 * kChunkBytes, *pd = p + 3 * kChunkBytes;
    asm volatile(
        "global_load_dwordx4 %0, %16, off sc1\n\t"
        "global_load_dwordx4 %1, %16, off offset:1024 sc1\n\t"
        "global_load_dwordx4 %2, %16, off offset:2048 sc1\n\t"
        "global_load_dwordx4 %3, %16, off offset:3072 sc1\n\t"
        "global_load_dwordx4 %4, %17, off sc1\n\t"
        "global_load_dwordx4 %5, %17, off offset:1024 sc1\n\t"
        "global_load_dwordx4 %6, %17, off offset:2048 sc1\n\t"
        "global_load_dwordx4 %7, %17, off offset:3072 sc1\n\t"
        "global_load_dwordx4 %8, %18, off sc1\n\t"
        "global_load_dwordx4 %9, %18, off offset:1024 sc1\n\t"
        "global_load_dwordx4 %10, %18, off offset:2048 sc1\n\t"
        "global_load_dwordx4 %11, %18, off offset:3072 sc1\n\t"
        "global_load_dwordx4 %12, %19, off sc1\n\t"
        "global_load_dwordx4 %13, %19, off offset:1024 sc1\n\t"
        "global_load_dwordx4 %14, %19, off offset:2048 sc1\n\t"
        "global_load_dwordx4 %15, %19, off offset:3072 sc1\n\t"
        "s_waitcnt vmcnt(0)"
        : "=&v"(r[0][0]), "=&v"(r[0][1]), "=&v"(r[0][2]), "=&v"(r[0][3]), "=&v"(r[1][0]),
          "=&v"(r[1][1]), "=&v"(r[1][2]), "=&v"(r[1][3]), "=&v"(r[2][0]), "=&v"(r[2][1]),
          "=&v"(r[2][2]), "=&v"(r[2][3]), "=&v"(r[3][0]), "=&v"(r[3][1]), "=&v"(r[3][2]),
          "=&v"(r[3][3])
        : "v"(pa), "v"(pb), "v"(pc), "v"(pd)
        : "memory");
}
__device__ __forceinline__ void load_chunks(const char *p, u32x4 (&r)[6][kRPL]) {
    static_assert(kRPL == 4, "four slots per lane");
    const char *pa = p, *pb = p + kChunkBytes, *pc = p + 2 * kChunkBytes, *pd = p + 3 * kChunkBytes,
               *pe = p + 4 * kChunkBytes, *pf = p + 5 * kChunkBytes;
    asm volatile(
        "global_load_dwordx4 %0, %24, off sc1\n\t"
        "global_load_dwordx4 %1, %24, off offset:1024 sc1\n\t"
        "global_load_dwordx4 %2, %24, off offset:2048 sc1\n\t"
        "global_load_dwordx4 %3, %24, off offset:3072 sc1\n\t"
        "global_load_dwordx4 %4, %25, off sc1\n\t"
        "global_load_dwordx4 %5, %25, off offset:1024 sc1\n\t"
        "global_load_dwordx4 %6, %25, off offset:2048 sc1\n\t"
        "global_load_dwordx4 %7, %25, off offset:3072 sc1\n\t"
        "global_load_dwordx4 %8, %26, off sc1\n\t"
        "global_load_dwordx4 %9, %26, off offset:1024 sc1\n\t"
        "global_load_dwordx4 %10, %26, off offset:2048 sc1\n\t"
        "global_load_dwordx4 %11, %26, off offset:3072 sc1\n\t"
        "global_load_dwordx4 %12, %27, off sc1\n\t"
        "global_load_dwordx4 %13, %27, off offset:1024 sc1\n\t"
        "global_load_dwordx4 %14, %27, off offset:2048 sc1\n\t"
        "global_load_dwordx4 %15, %27, off offset:3072 sc1\n\t"
        "global_load_dwordx4 %16, %28, off sc1\n\t"
        "global_load_dwordx4 %17, %28, off offset:1024 sc1\n\t"
        "global_load_dwordx4 %18, %28, off offset:2048 sc1\n\t"
        "global_load_dwordx4 %19, %28, off offset:3072 sc1\n\t"
        "global_load_dwordx4 %20, %29, off sc1\n\t"
        "global_load_dwordx4 %21, %29, off offset:1024 sc1\n\t"
        "global_load_dwordx4 %22, %29, off offset:2048 sc1\n\t"
        "global_load_dwordx4 %23, %29, off offset:3072 sc1\n\t"
        "s_waitcnt vmcnt(0)"
        : "=&v"(r[0][0]), "=&v"(r[0][1]), "=&v"(r[0][2]), "=&v"(r[0][3]), "=&v"(r[1][0]),
          "=&v"(r[1][1]), "=&v"(r[1][2]), "=&v"(r[1][3]), "=&v"(r[2][0]), "=&v"(r[2][1]),
          "=&v"(r[2][2]), "=&v"(r[2][3]), "=&v"(r[3][0]), "=&v"(r[3][1]), "=&v"(r[3][2]),
          "=&v"(r[3][3]), "=&v"(r[4][0]), "=&v"(r[4][1]), "=&v"(r[4][2]), "=&v"(r[4][3]),
          "=&v"(r[5][0]), "=&v"(r[5][1]), "=&v"(r[5][2]), "=&v"(r[5][3])
        : "v"(pa), "v"(pb), "v"(pc), "v"(pd), "v"(pe), "v"(pf)
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

// Two dwords, `d0` and `d1` dwords behind `off` (both below 256), complete on return.
template <int D0, int D1>
__device__ __forceinline__ u32x2 lds_read2(uint32_t off) {
    u32x2 r;
    asm volatile("ds_read2_b32 %0, %1 offset0:%2 offset1:%3\n\ts_waitcnt lgkmcnt(0)"
                 : "=v"(r) : "v"(off), "n"(D0), "n"(D1) : "memory");
    return r;
}
// Two 16-byte reads in flight together, complete on return.
__device__ __forceinline__ void lds_read16x2(u32x4 &a, u32x4 &b, uint32_t off_a, uint32_t off_b) {
    asm volatile("ds_read_b128 %0, %2\n\tds_read_b128 %1, %3\n\ts_waitcnt lgkmcnt(0)"
                 : "=&v"(a), "=&v"(b) : "v"(off_a), "v"(off_b) : "memory");
}
// Four consecutive 16-byte words (64 bytes from `off`), complete on return.
__device__ __forceinline__ void lds_read64(u32x4 &a, u32x4 &b, u32x4 &c, u32x4 &d, uint32_t off) {
    asm volatile("ds_read_b128 %0, %4\n\tds_read_b128 %1, %4 offset:16\n\t"
                 "ds_read_b128 %2, %4 offset:32\n\tds_read_b128 %3, %4 offset:48\n\t"
                 "s_waitcnt lgkmcnt(0)"
                 : "=&v"(a), "=&v"(b), "=&v"(c), "=&v"(d) : "v"(off) : "memory");
}
// Eight consecutive 16-byte words (128 bytes from `off`), complete on return.
__device__ __forceinline__ void lds_read128(u32x4 (&r)[8], uint32_t off) {
    asm volatile("ds_read_b128 %0, %8\n\tds_read_b128 %1, %8 offset:16\n\t"
                 "ds_read_b128 %2, %8 offset:32\n\tds_read_b128 %3, %8 offset:48\n\t"
                 "ds_read_b128 %4, %8 offset:64\n\tds_read_b128 %5, %8 offset:80\n\t"
                 "ds_read_b128 %6, %8 offset:96\n\tds_read_b128 %7, %8 offset:112\n\t"
                 "s_waitcnt lgkmcnt(0)"
                 : "=&v"(r[0]), "=&v"(r[1]), "=&v"(r[2]), "=&v"(r[3]), "=&v"(r[4]), "=&v"(r[5]),
                   "=&v"(r[6]), "=&v"(r[7])
                 : "v"(off) : "memory");
}
// The records of two candidates, their values (each with the value that follows
// it in the array) and their indices, with all reads in flight together.
__device__ __forceinline__ void lds_read_pair(u32x4 &c0, u32x4 &c1, u32x2 &v0, u32x2 &v1, uint32_t &i0,
                                              uint32_t &i1, uint32_t a_c0, uint32_t a_c1, uint32_t a_v0,
                                              uint32_t a_v1, uint32_t a_i0, uint32_t a_i1) {
    asm volatile("ds_read_b128 %0, %6\n\tds_read_b128 %1, %7\n\t"
                 "ds_read2_b32 %2, %8 offset1:1\n\tds_read2_b32 %3, %9 offset1:1\n\t"
                 "ds_read_b32 %4, %10\n\tds_read_b32 %5, %11\n\t"
                 "s_waitcnt lgkmcnt(0)"
                 : "=&v"(c0), "=&v"(c1), "=&v"(v0), "=&v"(v1), "=&v"(i0), "=&v"(i1)
                 : "v"(a_c0), "v"(a_c1), "v"(a_v0), "v"(a_v1), "v"(a_i0), "v"(a_i1)
                 : "memory");
}
__device__ __forceinline__ void lds_write4(uint32_t off, uint32_t v) {
    asm volatile("ds_write_b32 %0, %1" : : "v"(off), "v"(v) : "memory");
}
__device__ __forceinline__ uint32_t lds_read4(uint32_t off) {
    uint32_t r;
    asm volatile("ds_read_b32 %0, %1\n\ts_waitcnt lgkmcnt(0)" : "=v"(r) : "v"(off) : "memory");
    return r;
}
// 8-byte LDS word written and read by one instruction each.
__device__ __forceinline__ void lds_write8(uint32_t off, u32x2 v) {
    asm volatile("ds_write_b64 %0, %1" : : "v"(off), "v"(v) : "memory");
}
__device__ __forceinline__ u32x2 lds_read8(uint32_t off) {
    u32x2 r;
    asm volatile("ds_read_b64 %0, %1\n\ts_waitcnt lgkmcnt(0)" : "=v"(r) : "v"(off) : "memory");
    return r;
}

__device__ __forceinline__ uint32_t wave_min_u32(uint32_t v) { return ~wave_max_u32(~v); }
// Reductions over lanes 0..15 only (other lanes must pass the identity), wave-uniform.
__device__ __forceinline__ uint32_t row_max_uniform(uint32_t v) {
    return (uint32_t)readlane_i((int)row16_max_u32(v), 15);
}
__device__ __forceinline__ uint32_t row_min_uniform(uint32_t v) { return ~row_max_uniform(~v); }

// Lane that holds the best of the pairs (value v, index i): largest value, then
// lowest index.  `vmax` is the (uniform) largest value; the index reduction is
// only paid when several lanes hold it.
template <typename MINF>
__device__ __forceinline__ int best_lane(uint32_t v, uint32_t i, uint32_t vmax, MINF minf) {
    const uint64_t tied = __builtin_amdgcn_ballot_w64(v == vmax);
    if (__builtin_popcountll(tied) == 1) return (int)__builtin_ctzll(tied);
    const uint32_t imin = minf(v == vmax ? i : 0xffffffffu);
    return first_lane(v == vmax && i == imin);
}

// The K best (value, index) pairs of a set and the value that follows them,
// in (value descending, index ascending) order.
template <int K>
struct TopK {
    uint32_t v[K + 1];
    uint32_t i[K];
};

// Merge the TopK of the participating lanes (`act`) into one.  src[r] receives
// the lane that supplied entry r and ent[r] which of that lane's entries it
// was.  MAXF / MINF reduce over the participating lanes and return wave-uniform
// values.
template <int K, typename MAXF, typename MINF>
__device__ __forceinline__ TopK<K> merge_topk(const TopK<K> &t, bool act, int lane, MAXF maxf,
                                              MINF minf, int (&src)[K], int (&ent)[K]) {
    TopK<K> r;
    int cur = 0;  // entries of this lane already taken
    uint32_t hv = act ? t.v[0] : 0u, hi = act ? t.i[0] : 0xffffffffu;  // this lane's next entry
#pragma unroll
    for (int k = 0; k < K; ++k) {
        r.v[k] = maxf(hv);
        const int l = best_lane(hv, hi, r.v[k], minf);
        r.i[k] = (uint32_t)readlane_i((int)hi, l);
        src[k] = l;
        ent[k] = readlane_i(cur, l);
        if (lane == l) {
            ++cur;
            hv = t.v[K];
            hi = 0xffffffffu;
#pragma unroll
            for (int e = 1; e < K; ++e) {
                hv = cur == e ? t.v[e] : hv;
                hi = cur == e ? t.i[e] : hi;
            }
        }
    }
    r.v[K] = maxf(hv);
    return r;
}

// What a reporting unit contributes to a round: its T best points (any order)
// with their current values and indices, and the bound on its other points.
// A candidate that does not exist has value 0 and index kNoIndex.
template <int T>
struct RoundInput {
    uint32_t v[T], bound;
    float x[T], y[T], z[T];
    uint32_t i[T];
};

// LDS used by the wave that runs exchange_round.
struct RoundLds {
    // picks of the round: {x, y, z, seq}; spare slots that are never picks (they
    // keep the seed point), so that readers may read a few slots past the last pick
    __attribute__((aligned(16))) u32x4 pk[kMaxPicksPerRound + 8];
    uint32_t pk_idx[kMaxPicksPerRound];  // index of each pick of the round (general replay loop)
    uint32_t pk_val[kMaxPicksPerRound];  // and the value it was picked with
    // live candidates, first in compaction order, then in the order of the replay:
    __attribute__((aligned(16))) u32x4 cand[2 * kWave + 3];  // {x, y, z, value; later sequence number}; spare entries for reads ahead
    __attribute__((aligned(16))) uint32_t keyw[2 * kWave + 32];  // 32-bit sort keys, zero-padded; later the values in order
    // (entries cand[130], keyw[130], idxw[130] take what the compaction discards)
    uint32_t idxw[2 * kWave + 3];                                // point indices
};

// Counters of a profiling build (workgroup 0 only).
struct RoundProf {
    uint32_t acc[8];   // 100 MHz ticks per phase; [5], [6]: rounds of the ordered replay with up to 64 / more candidates; [7]: polls
    uint32_t loop[4];  // shader cycles and picks inside the ordered replay's pick loop, by the same split
    uint32_t sub[4];   // shader cycles of the replay set-up: bounds, counting, compaction, ordering
    uint32_t ev[4];    // live candidates, candidates passed over, rounds ended by a lowered candidate, exact re-orderings
    uint64_t last;
};
#ifdef FFPS_PROFILE
#define FFPS_STAMP(P, i)                                 \
    do {                                                 \
        if ((P) != nullptr) {                            \
            uint64_t now_ = wall_clock64();              \
            (P)->acc[i] += (uint32_t)(now_ - (P)->last); \
            (P)->last = now_;                            \
        }                                                \
    } while (0)
#else
#define FFPS_STAMP(P, i) \
    do {                 \
    } while (0)
#endif

// The inner loop of the ordered replay, for one set of candidates (lane L holds
// candidate L of the set: current value v, coordinates x, y, z; `o` is the value
// it had at the start of the round, or 0xffffffff for the lanes from `lim` on,
// where the set ends; `seq` is the sequence number the candidate has as a pick
// and `a_pk` the address of the LDS slot it goes to, both per lane).  Starting
// at candidate i, with `bit` = 1 << i:
//   - candidate i's value is unchanged (v == o in lane i): lane i alone writes
//     its record {x, y, z, seq} to its slot for the worker waves, its
//     coordinates are read out of the lane, every lane's value is lowered by
//     the squared distance to it, and i steps on (21 instructions, nothing to
//     wait for: LDS is only written).  The distances are worked out before the
//     branch on the comparison, whose way from the vector to the scalar unit is
//     long; a candidate that turns out lowered has cost eight wasted operations;
//   - it has been lowered to the threshold T or below: it is out of this round;
//     its bit is noted in `gone`, the sequence numbers and slots of all lanes
//     move down by one, and i steps on.  With `soft` set the block returns here
//     instead (the caller then moves the end of the set, which depends on the
//     number of candidates passed over when the picks left to do are few);
//   - it has been lowered but is still above T, or i has reached `lim`: return.
// The registers named in the text are scratch of this block; distances are the
// individually rounded operations of sqdist; a lane read into a scalar register
// needs two instructions before a vector instruction may use it, which the
// order of the reads provides.
__device__ __forceinline__ void ordered_run(uint32_t &v, uint32_t o, float x, float y, float z,
                                            uint32_t seq, uint32_t a_pk, uint64_t &bit, int &i,
                                            uint64_t &gone, uint32_t T, int lim, int soft) {
    uint32_t sx, sy, sz;
#define FFPS_STEP                                          \
    "v_readlane_b32 %[sx], %[x], %[i]\n\t"                 \
    "v_readlane_b32 %[sy], %[y], %[i]\n\t"                 \
    "v_readlane_b32 %[sz], %[z], %[i]\n\t"                 \
    "v_cmp_eq_u32 vcc, %[v], %[o]\n\t"                     \
    "v_subrev_f32 v112, %[sx], %[x]\n\t"                   \
    "v_subrev_f32 v113, %[sy], %[y]\n\t"                   \
    "v_subrev_f32 v114, %[sz], %[z]\n\t"                   \
    "v_mul_f32 v112, v112, v112\n\t"                       \
    "v_mul_f32 v113, v113, v113\n\t"                       \
    "v_mul_f32 v114, v114, v114\n\t"                       \
    "v_add_f32 v112, v112, v113\n\t"                       \
    "v_add_f32 v112, v112, v114\n\t"                       \
    "s_and_b64 vcc, vcc, %[bit]\n\t"                       \
    "s_cbranch_scc0 7f\n\t"                                \
    "s_mov_b64 exec, vcc\n\t"                              \
    "ds_write_b128 %[ap], v[108:111]\n\t"                  \
    "s_mov_b64 exec, -1\n\t"                               \
    "v_min_f32 %[v], %[v], v112\n\t"                       \
    "s_lshl_b64 %[bit], %[bit], 1\n\t"                     \
    "s_add_i32 %[i], %[i], 1\n\t"
    asm volatile(
        "v_mov_b32 v108, %[x]\n\t"
        "v_mov_b32 v109, %[y]\n\t"
        "v_mov_b32 v110, %[z]\n\t"
        "v_mov_b32 v111, %[seq]\n\t"
        "1:\n\t"
        FFPS_STEP
        FFPS_STEP
        "s_branch 1b\n\t"
        "7:\n\t"
        "s_cmp_ge_i32 %[i], %[lim]\n\t"
        "s_cbranch_scc1 9f\n\t"
        "s_cmp_lg_u32 %[soft], 0\n\t"
        "s_cbranch_scc1 9f\n\t"
        "v_readlane_b32 %[sx], %[v], %[i]\n\t"
        "s_nop 1\n\t"
        "s_cmp_gt_u32 %[sx], %[T]\n\t"
        "s_cbranch_scc1 9f\n\t"
        "s_or_b64 %[gone], %[gone], %[bit]\n\t"
        "v_subrev_u32 v111, 1, v111\n\t"
        "v_subrev_u32 %[ap], 16, %[ap]\n\t"
        "s_lshl_b64 %[bit], %[bit], 1\n\t"
        "s_add_i32 %[i], %[i], 1\n\t"
        "s_branch 1b\n\t"
        "9:\n\t"
        : [v] "+v"(v), [bit] "+s"(bit), [i] "+s"(i), [gone] "+s"(gone), [ap] "+v"(a_pk), [sx] "=&s"(sx),
          [sy] "=&s"(sy), [sz] "=&s"(sz)
        : [o] "v"(o), [x] "v"(x), [y] "v"(y), [z] "v"(z), [seq] "v"(seq), [T] "s"(T), [lim] "s"(lim),
          [soft] "s"(soft)
        : "memory", "vcc", "scc", "v108", "v109", "v110", "v111", "v112", "v113", "v114");
#undef FFPS_STEP
}

// Replay of the greedy rule of Eq. 1 on KC candidates per lane of ONE full wave
// (value bits cv, point index ci, coordinates cx/cy/cz; a candidate that does
// not exist has value 0 and index kNoIndex), given lb = the lane's share of the
// bounds on all points that are not candidates.  Pick number c of the round is
// written as {x, y, z, npicked + c} to L.pk[c] (16-byte LDS writes, in pick
// order, so other waves may consume them while the replay is still running),
// and what record_picks needs to name its index and value is left in L.
// Returns the number of picks (1 .. cap) and how they were noted.  The
// candidate arrays are used up.
struct RoundResult {
    int cnt;        // picks of the round, or -1 when the round failed
    bool by_lane;   // picks noted in the lanes (below) rather than in L.pk_idx / L.pk_val
    // by_lane: what this lane's two candidates of the ordered replay became: pick
    // number within the round (-1: not picked), point index, value when picked
    int pc[2];
    uint32_t pi[2], pv[2];
};

// Writes index (and value) of the picks of a round to the outputs; run by the
// wave that ran the round, in one workgroup of the cloud.
__device__ __forceinline__ void record_picks(const RoundLds &L, int lane, const RoundResult &r,
                                             int npicked, int32_t *idx_out, float *md_out);

template <int KC>
__device__ __forceinline__ RoundResult replay_round(RoundLds &L, int lane, uint32_t (&cv)[KC],
                                            uint32_t (&ci)[KC], float (&cx)[KC], float (&cy)[KC],
                                            float (&cz)[KC], uint32_t lb, int npicked, int cap,
                                            RoundProf *prof) {
    const uint32_t pk_off = lds_offset(L.pk);
#ifdef FFPS_PROFILE
    uint64_t sc = clock64();
#define FFPS_SUB(i)                              \
    do {                                         \
        if (prof) {                              \
            uint64_t n_ = clock64();             \
            prof->sub[i] += (uint32_t)(n_ - sc); \
            sc = n_;                             \
        }                                        \
    } while (0)
#else
#define FFPS_SUB(i) \
    do {            \
    } while (0)
#endif
    const uint32_t Bound = wave_max_u32(lb);
    // Hand pick number c of this round to the other waves (one 16-byte LDS write)
    // and note its index and value; `mine` holds in exactly one lane.
    auto emit = [&](bool mine, int c, uint32_t idx, uint32_t vbits, float ex, float ey, float ez) {
        if (mine) {
            u32x4 s;
            s.x = f2u(ex); s.y = f2u(ey); s.z = f2u(ez); s.w = (uint32_t)(npicked + c);
            lds_write16(pk_off + c * 16, s);
            L.pk_idx[c] = idx;
            L.pk_val[c] = vbits;
        }
    };
    auto lane_best = [&](uint32_t &bv, uint32_t &bi, int &bq) {
        bv = cv[0]; bi = ci[0]; bq = 0;
#pragma unroll
        for (int q = 1; q < KC; ++q) {
            const bool better = cv[q] > bv || (cv[q] == bv && ci[q] < bi);
            bv = better ? cv[q] : bv;
            bi = better ? ci[q] : bi;
            bq = better ? q : bq;
        }
    };
    auto wmin = [](uint32_t v) { return wave_min_u32(v); };
    uint32_t lv = cv[0];
#pragma unroll
    for (int q = 1; q < KC; ++q) lv = umax(lv, cv[q]);
    uint32_t V = wave_max_u32(lv);  // best candidate value
    int cnt = 0;
    int pl;
    float px, py, pz;
    // Only candidates above the bound can be picked after the first pick, and
    // when the best candidate is above it the first pick is one of them too:
    // compact them (in any order).  Any threshold T >= Bound serves as well (the
    // round then ends when the best candidate is no longer above T), so when more
    // than 128 candidates are above the bound T is raised to the largest
    // third-best candidate value of any lane, which leaves at most two per lane.
    uint32_t T = Bound;
    int total = 0, before = 0;
    FFPS_SUB(0);
    if (V > Bound && cap > 1) {
        // total = live candidates of the wave, before = those of lower lanes: the
        // per-lane count goes through one ballot per bit of it
        auto count_live = [&]() {
            uint32_t c = 0u;
#pragma unroll
            for (int q = 0; q < KC; ++q) c += cv[q] > T ? 1u : 0u;
            total = 0;
            before = 0;
#pragma unroll
            for (int bit = 0; (1 << bit) <= KC; ++bit) {
                const uint64_t mk = __builtin_amdgcn_ballot_w64((c >> bit) & 1u);
                total += __builtin_popcountll(mk) << bit;
                before += (int)__builtin_amdgcn_mbcnt_hi(
                              (uint32_t)(mk >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)mk, 0u))
                          << bit;
            }
        };
        count_live();
        if (total > 2 * kWave) {
            uint32_t t1 = 0u, t2 = 0u, t3 = 0u;
#pragma unroll
            for (int q = 0; q < KC; ++q) {
                const uint32_t v = cv[q];
                t3 = umax(t3, v < t2 ? v : t2);
                t2 = umax(t2, v < t1 ? v : t1);
                t1 = umax(t1, v);
            }
            T = umax(Bound, wave_max_u32(t3));
            count_live();
        }
    }
    // With at most 128 live candidates the replay needs no argmax per pick.  Put
    // the candidates in the order (value descending, index ascending).  The first
    // one is the next pick.  Picking a point can only lower other values, so the
    // next candidate in that order is the following pick as long as its own value
    // has not been lowered by a pick of this round: everything behind it started
    // no higher and has not grown, candidates ahead of it are picked or gone, and
    // unreported points are at or below the threshold.  A candidate whose value
    // has been lowered to the threshold or below is out of this round and is
    // passed over; one that has been lowered but is still above the threshold
    // may now belong further back in the order, and the round ends before it
    // (the next round sees it with its new value).  Per pick this costs the
    // distance update of the candidates and one comparison.
    const bool ordered = total >= 1 && total <= 2 * kWave;
    FFPS_SUB(1);
#ifdef FFPS_PROFILE
    if (prof && ordered) prof->acc[total <= kWave ? 5 : 6] += 1;
#endif
    RoundResult res;
    res.pc[0] = res.pc[1] = -1;
    res.pi[0] = res.pi[1] = kNoIndex;
    res.pv[0] = res.pv[1] = 0u;
    if (ordered) {
        const uint32_t cand_off = lds_offset(L.cand), key_off = lds_offset(L.keyw),
                       idx_off = lds_offset(L.idxw);
        // 32-bit sort key of a live candidate: its value above the threshold and its
        // compaction position, (value - T) << 7 | position, which orders by value
        // and is unique.  Candidates of equal value come out in position order
        // rather than index order; that is detected below and then put right.
        const bool narrow = V - T < (1u << 24);
        // compaction without branches: a candidate that is not live goes to a slot
        // behind the live ones, which nobody reads
        {
            const uint32_t dump = (uint32_t)(2 * kWave + 2);
            uint32_t pos = (uint32_t)before;
#pragma unroll
            for (int q = 0; q < KC; ++q) {
                const bool live = cv[q] > T;
                const uint32_t at = live ? pos : dump;
                u32x4 r;
                r.x = f2u(cx[q]); r.y = f2u(cy[q]); r.z = f2u(cz[q]); r.w = cv[q];
                lds_write16(cand_off + at * 16, r);
                lds_write4(key_off + at * 4, ((cv[q] - T) << 7) | pos);
                lds_write4(idx_off + at * 4, ci[q]);
                pos += live ? 1u : 0u;
            }
        }
        if (lane < 32) lds_write4(key_off + (total + lane) * 4, 0u);  // padding: below every key
        // the same wave wrote and now reads: LDS keeps its accesses in order
        FFPS_SUB(2);
        // ---- order: every lane ranks its candidates (positions `lane` and
        //      `lane + 64`) by counting the candidates that precede them ----
        const int p1 = lane + kWave;
        const bool h0 = lane < total, h1 = p1 < total;
        const uint32_t q0 = h0 ? (uint32_t)lane : 0u, q1 = h1 ? (uint32_t)p1 : 0u;  // safe positions
        u32x4 c0, c1;
        u32x2 w0, w1;
        uint32_t i0, i1;
        lds_read_pair(c0, c1, w0, w1, i0, i1, cand_off + q0 * 16, cand_off + q1 * 16, key_off + q0 * 4,
                      key_off + q1 * 4, idx_off + q0 * 4, idx_off + q1 * 4);
        uint32_t o0 = h0 ? c0.w : 0u, o1 = h1 ? c1.w : 0u;  // values at the start of the round
        bool ties = false;
        // Candidates go to their places in the order: records {x, y, z, sequence
        // number as a pick if no candidate ahead is passed over} (what the workers
        // take), values and indices.  Every lane then takes candidates number `lane`
        // (set 0) and `lane + 64` (set 1) of the order, and sees whether the
        // candidate behind each of them has the same value.
        auto place = [&](int r0, int r1) {
            if (h0) {
                c0.w = (uint32_t)(npicked + r0);
                lds_write16(cand_off + r0 * 16, c0);
                lds_write4(key_off + r0 * 4, o0);
                lds_write4(idx_off + r0 * 4, i0);
            }
            if (h1) {
                c1.w = (uint32_t)(npicked + r1);
                lds_write16(cand_off + r1 * 16, c1);
                lds_write4(key_off + r1 * 4, o1);
                lds_write4(idx_off + r1 * 4, i1);
            }
            if (lane == 0) lds_write4(key_off + total * 4, 0u);  // behind the last value
            lds_read_pair(c0, c1, w0, w1, i0, i1, cand_off + q0 * 16, cand_off + q1 * 16,
                          key_off + q0 * 4, key_off + q1 * 4, idx_off + q0 * 4, idx_off + q1 * 4);
            o0 = h0 ? w0.x : 0u;
            o1 = h1 ? w1.x : 0u;
            ties = __builtin_amdgcn_ballot_w64((h0 && w0.y == w0.x) || (h1 && w1.y == w1.x)) != 0;
        };
        // by (value descending, index ascending) on the full values: always right
        auto order_exact = [&]() {
            const uint64_t key0 = ((uint64_t)o0 << 32) | ~i0, key1 = ((uint64_t)o1 << 32) | ~i1;
            int r0 = 0, r1 = 0;
            for (int j = 0; j < total; ++j) {
                const uint64_t kj = ((uint64_t)lds_read4(key_off + j * 4) << 32) | ~lds_read4(idx_off + j * 4);
                r0 += kj > key0 ? 1 : 0;
                r1 += kj > key1 ? 1 : 0;
            }
            place(r0, r1);
        };
        if (narrow) {
            const uint32_t key0 = ((o0 - T) << 7) | (uint32_t)lane, key1 = ((o1 - T) << 7) | (uint32_t)p1;
            int r0 = 0, r1 = 0;
            for (int j = 0; j < total; j += 32) {
                // thirty-two keys per step, read by all lanes from the same addresses (a broadcast)
                u32x4 k[8];
                lds_read128(k, key_off + j * 4);
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    r0 += k[e].x > key0 ? 1 : 0; r0 += k[e].y > key0 ? 1 : 0;
                    r0 += k[e].z > key0 ? 1 : 0; r0 += k[e].w > key0 ? 1 : 0;
                }
                if (total > kWave) {
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        r1 += k[e].x > key1 ? 1 : 0; r1 += k[e].y > key1 ? 1 : 0;
                        r1 += k[e].z > key1 ? 1 : 0; r1 += k[e].w > key1 ? 1 : 0;
                    }
                }
            }
            place(r0, r1);
            if (ties) order_exact();  // the values are in LDS in order now: equal neighbours are ties
        } else {
            lds_write4(key_off + q0 * 4, c0.w);  // order_exact reads the values there
            if (h1) lds_write4(key_off + p1 * 4, c1.w);
            order_exact();
        }
        const float x0 = u2f(c0.x), y0 = u2f(c0.y), z0 = u2f(c0.z);
        const float x1 = u2f(c1.x), y1 = u2f(c1.y), z1 = u2f(c1.z);
        uint32_t v0 = o0, v1 = o1;  // current values
        FFPS_SUB(3);
#ifdef FFPS_PROFILE
        const uint64_t lc0 = clock64();
#endif
        // ---- replay, one set after the other ----
        uint64_t gone0 = 0ull, gone1 = 0ull;  // candidates passed over
        int ngone = 0;
        bool stop = false;
        // Candidates [base, base + n) of the order are lanes 0 .. n-1 of a set.
        // Candidate base + li is pick number base + li - ngone of the round, so with
        // `cap` picks allowed the set ends at lane cap + ngone - base.  Returns the
        // number of candidates of the set that were dealt with.
        auto run_set = [&](uint32_t &v, uint32_t o, float x, float y, float z, int base, int n,
                           uint64_t &gone) {
            int li = 0;
            while (true) {
                // the end of the set moves with the candidates passed over only when
                // fewer picks are left to do than the set has candidates
                const bool soft = cap - base < n;
                const int lend = soft ? (n < cap + ngone - base ? n : cap + ngone - base) : n;
                if (li >= lend) break;
                const int c = base + lane - ngone;  // this lane's candidate as a pick of the round
                uint64_t bit = 1ull << li;
                const uint64_t gone_before = gone;
                ordered_run(v, lane < lend ? o : 0xffffffffu, x, y, z, (uint32_t)(npicked + c),
                            pk_off + (uint32_t)c * 16, bit, li, gone,
                            (uint32_t)__builtin_amdgcn_readfirstlane((int)T),
                            __builtin_amdgcn_readfirstlane(lend),
                            __builtin_amdgcn_readfirstlane(soft ? 1 : 0));
                ngone += __builtin_popcountll(gone ^ gone_before);
                if (li >= lend) break;
                // candidate li has been lowered by a pick of this round
                if ((uint32_t)readlane_i((int)v, li) > T) {
                    stop = true;  // still a candidate, but maybe no longer the next one
                    break;
                }
                // out of this round: the candidates behind it become picks one number earlier
                gone |= 1ull << li;
                ++ngone;
                ++li;
            }
            return li;
        };
        const int nA = total < kWave ? total : kWave;
        const int iA = run_set(v0, o0, x0, y0, z0, 0, nA, gone0);
        int iB = 0;
        if (!stop && iA == kWave && total > kWave && cap + ngone > kWave) {
            // set 1 has not seen the picks of set 0 yet: apply them (the workers are
            // busy with the same picks meanwhile)
            // Eight slots per LDS read.  Slots behind the picks of this round hold
            // picks of earlier rounds (or the seed point), which every value already
            // reflects, so applying those again changes nothing.
            const int done = kWave - ngone;
            for (int c = 0; c < done; c += 8) {
                u32x4 r[8];
                lds_read128(r, pk_off + c * 16);
#pragma unroll
                for (int e = 0; e < 8; ++e)
                    v1 = f2u(min_dist(u2f(v1), sqdist(x1, y1, z1, u2f(r[e].x), u2f(r[e].y), u2f(r[e].z))));
            }
            iB = run_set(v1, o1, x1, y1, z1, kWave, total - kWave, gone1);
        }
        cnt = iA + iB - ngone;
#ifdef FFPS_PROFILE
        if (prof) {
            prof->ev[0] += (uint32_t)total;
            prof->ev[1] += (uint32_t)ngone;
            prof->ev[2] += stop ? 1u : 0u;
        }
#endif
        // the candidates dealt with were picked unless passed over; the pick number
        // of one of them is its place minus the candidates passed over before it
        const int g0 = (int)__builtin_amdgcn_mbcnt_hi((uint32_t)(gone0 >> 32),
                                                      __builtin_amdgcn_mbcnt_lo((uint32_t)gone0, 0u));
        const int g1 = (int)__builtin_amdgcn_mbcnt_hi((uint32_t)(gone1 >> 32),
                                                      __builtin_amdgcn_mbcnt_lo((uint32_t)gone1, 0u));
        if (lane < iA && !((gone0 >> lane) & 1ull)) res.pc[0] = lane - g0;
        if (lane < iB && !((gone1 >> lane) & 1ull)) res.pc[1] = p1 - __builtin_popcountll(gone0) - g1;
        res.pi[0] = i0; res.pi[1] = i1;
        res.pv[0] = o0; res.pv[1] = o1;
#ifdef FFPS_PROFILE
        if (prof) {
            prof->loop[total <= kWave ? 0 : 2] += (uint32_t)(clock64() - lc0);
            prof->loop[total <= kWave ? 1 : 3] += cnt;
        }
#endif
    } else {
        // a single pick (best candidate not above the bound, or cap 1), or more
        // than 128 candidates above every threshold tried: work on all candidates
        // of every lane
        while (true) {
            uint32_t bv, bi;
            int bq;
            lane_best(bv, bi, bq);
            V = wave_max_u32(bv);
            if (cnt > 0 && !(V > Bound)) break;
            pl = best_lane(bv, bi, V, wmin);
            const int pq = readlane_i(bq, pl);
            pick_xyz<KC>(cx, cy, cz, pq, pl, px, py, pz);
            emit(lane == pl, cnt, bi, V, px, py, pz);
            if (++cnt >= cap) break;
#pragma unroll
            for (int q = 0; q < KC; ++q)
                cv[q] = f2u(fminf(u2f(cv[q]), sqdist(cx[q], cy[q], cz[q], px, py, pz)));
        }
    }
    res.cnt = cnt;
    res.by_lane = ordered;
    return res;
}

__device__ __forceinline__ void record_picks(const RoundLds &L, int lane, const RoundResult &r,
                                             int npicked, int32_t *idx_out, float *md_out) {
    if (r.by_lane) {
#pragma unroll
        for (int e = 0; e < 2; ++e) {
            if (r.pc[e] >= 0) {
                idx_out[npicked + r.pc[e]] = (int32_t)r.pi[e];
                if (md_out) md_out[npicked + r.pc[e]] = u2f(r.pv[e]);
            }
        }
        return;
    }
    for (int c = lane; c < r.cnt; c += kWave) {
        idx_out[npicked + c] = (int32_t)L.pk_idx[c];
        if (md_out) md_out[npicked + c] = u2f(L.pk_val[c]);
    }
}

// One round, run by ONE full wave of a workgroup.  The cloud has U reporting
// units (a whole workgroup, or each of its worker waves); lanes 0 .. nsub-1 of
// this wave publish `in` as unit unit0 + lane.  The wave then gathers all U
// records, replays, writes each pick as {x, y, z, npicked + c} to L.pk[c]
// (16-byte LDS writes, in pick order, so other waves may consume them while
// the replay is still running).  Returns the picks of the round (1 .. cap; see
// record_picks), or a count of -1 after setting *status when another unit's
// record never arrived.
template <int T>
__device__ __forceinline__ RoundResult exchange_round(RoundLds &L, char *exchange, int U, int unit0,
                                                      int nsub, int lane, uint32_t round,
                                                      const RoundInput<T> &in, int npicked, int cap,
                                                      int *status, RoundProf *prof) {
    static_assert(T == 2 || T == 3, "two or three candidates per unit");
    constexpr int NCH = chunks_of(T);
    constexpr int KC = T * kRPL;  // candidates per lane before compaction
    // ---- publish ----
    char *buf = exchange + (size_t)(round & 1) * buf_bytes(T);
    if (lane < nsub) {
        uint32_t d[NCH][3] = {};
#pragma unroll
        for (int t = 0; t < T; ++t) {
            d[0][t] = in.v[t];
            d[1 + t][0] = f2u(in.x[t]); d[1 + t][1] = f2u(in.y[t]); d[1 + t][2] = f2u(in.z[t]);
            d[T + 1][t] = in.i[t];
        }
        if (T == 2) d[0][2] = in.bound; else d[NCH - 1][0] = in.bound;
        const size_t so = (size_t)(unit0 + lane) * 16;
#pragma unroll
        for (int c = 0; c < NCH; ++c) {
            u32x4 ch;
            ch.x = d[c][0]; ch.y = d[c][1]; ch.z = d[c][2];
            ch.w = chunk_check(ch.x, ch.y, ch.z, round, (uint32_t)c);
            store_chunk(buf + c * kChunkBytes + so, ch);
        }
    }
    FFPS_STAMP(prof, 2);
    // ---- gather: lane L reads slots (= units) q*64+L ----
    u32x4 r[NCH][kRPL];
    bool gave_up = false;
    for (int spin = 0;; ++spin) {
        load_chunks(buf + (size_t)lane * 16, r);
        bool all = true;
#pragma unroll
        for (int q = 0; q < kRPL; ++q) {
            bool ok = true;
#pragma unroll
            for (int c = 0; c < NCH; ++c) ok = ok && chunk_ok(r[c][q], round, (uint32_t)c);
            all = all && (ok || q * kWave + lane >= U);
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
        // the first workgroup to give up notes what it was waiting for: status[2] =
        // round, status[3] = lowest unit whose record had not arrived, status[4] = its own unit
        int missing = 0x7fffffff;
#pragma unroll
        for (int q = kRPL - 1; q >= 0; --q) {
            bool ok = true;
#pragma unroll
            for (int c = 0; c < NCH; ++c) ok = ok && chunk_ok(r[c][q], round, (uint32_t)c);
            if (!ok && q * kWave + lane < U) missing = q * kWave + lane;
        }
        missing = (int)wave_min_u32((uint32_t)missing);
        if (lane == 0) {
            int expected = 0;
            if (__hip_atomic_compare_exchange_strong(status, &expected, -5, __ATOMIC_RELAXED,
                                                     __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) {
                status[2] = (int)round;
                status[3] = missing;
                status[4] = unit0;
            }
        }
        RoundResult failed = {};
        failed.cnt = -1;
        return failed;
    }
    // candidate c = T q + t of this lane: unit q*64 + lane, its t-th entry
    uint32_t cv[KC], ci[KC], lb = 0u;
    float cx[KC], cy[KC], cz[KC];
#pragma unroll
    for (int q = 0; q < kRPL; ++q) {
        const bool present = q * kWave + lane < U;  // absent records: value 0, bound 0
        const uint32_t vals[3] = {r[0][q].x, r[0][q].y, r[0][q].z};
        const uint32_t idxs[3] = {r[T + 1][q].x, r[T + 1][q].y, r[T + 1][q].z};
#pragma unroll
        for (int t = 0; t < T; ++t) {
            cv[T * q + t] = present ? vals[t] : 0u;
            ci[T * q + t] = present ? idxs[t] : kNoIndex;
            cx[T * q + t] = u2f(r[1 + t][q].x);
            cy[T * q + t] = u2f(r[1 + t][q].y);
            cz[T * q + t] = u2f(r[1 + t][q].z);
        }
        const uint32_t bnd = T == 2 ? r[0][q].z : r[NCH - 1][q].x;
        lb = umax(lb, present ? bnd : 0u);
    }
    return replay_round<KC>(L, lane, cv, ci, cx, cy, cz, lb, npicked, cap, prof);
}

}  // namespace ffps
